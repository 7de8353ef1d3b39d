"""Host-only checks of the C ABI: the library loads, exports every declared symbol, and
validates arguments before touching a GPU."""
import ctypes as C
import os
import re

import pytest

import paper_2511_18191_amd as tsd
import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _cfg(**over):
    c = synth.get_config("cfg2")
    cfg = tsd.make_config(c.target, c.draft, c.patch, c.K, c.batch, c.max_tokens, c.dtype, 1.0)
    for k, v in over.items():
        setattr(cfg, k, v)
    return cfg


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "tsd.h")).read()
    declared = set(re.findall(r"\b(tsd_[a-z_]+)\s*\(", header))
    assert declared and declared == set(tsd.binding.SYMBOLS)
    L = tsd.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert L.tsd_abi_version() == 1


def test_struct_layout_matches_header():
    assert C.sizeof(tsd.TsdModelCfg) == 24
    assert C.sizeof(tsd.TsdConfig) == 2 * 24 + 6 * 4 + 3 * 4 + 4 + 8
    assert tsd.TsdConfig.seed.offset % 8 == 0
    assert C.sizeof(tsd.TsdStats) == 40


def test_workspace_and_weight_counts():
    L = tsd.lib()
    n = C.c_size_t()
    cfg = _cfg()
    assert L.tsd_workspace_bytes(C.byref(cfg), C.byref(n)) == 0
    c = synth.get_config("cfg2")
    kv = 2 * c.batch * 48 * 2 * (c.target.n_layers * c.target.d_model + c.draft.n_layers * c.draft.d_model)
    assert n.value > kv and n.value % 256 == 0
    for which, m in ((tsd.TSD_TARGET, c.target), (tsd.TSD_DRAFT, c.draft)):
        assert L.tsd_weights_count(C.byref(cfg), which, C.byref(n)) == 0
        assert n.value == sum(int(__import__("numpy").prod(s)) for _, s in synth.weight_spec(m, c.patch))
    assert L.tsd_weights_count(C.byref(cfg), 2, C.byref(n)) == -1


@pytest.mark.parametrize("field,value,fragment", [
    ("K", 0, "K must"), ("K", 17, "K must"), ("patch", 50, "patch"), ("dtype", 3, "dtype"),
    ("page_tokens", 12, "page_tokens"), ("sigma_p", 0.0, "sigma"), ("sigma_q", float("nan"), "sigma"),
    ("fallback_r", -0.1, "fallback_r"), ("fallback_r", 1e3, "fallback_r"), ("fallback_r", float("nan"), "fallback_r"), ("max_tokens", 5, "max_tokens"), ("max_batch", 0, "max_batch"),
    ("flags", 8192, "flag"),
    ("flags", 1024 | 2048, "exclude"),
])
def test_config_validation(field, value, fragment):
    L = tsd.lib()
    n = C.c_size_t()
    cfg = _cfg(**{field: value})
    assert L.tsd_workspace_bytes(C.byref(cfg), C.byref(n)) == -1
    assert fragment in L.tsd_last_error(None).decode()


def test_model_validation():
    L = tsd.lib()
    n = C.c_size_t()
    cfg = _cfg()
    cfg.target.n_heads = 7
    assert L.tsd_workspace_bytes(C.byref(cfg), C.byref(n)) == -1 and b"target" in L.tsd_last_error(None)
    cfg = _cfg()
    cfg.draft.d_model = 1024          # head_dim 256 is not supported
    assert L.tsd_workspace_bytes(C.byref(cfg), C.byref(n)) == -1 and b"draft" in L.tsd_last_error(None)


def test_null_and_misuse_are_errors_not_crashes():
    L = tsd.lib()
    n = C.c_size_t()
    h = C.c_void_p()
    cfg = _cfg()
    assert L.tsd_workspace_bytes(None, C.byref(n)) == -1
    assert L.tsd_workspace_bytes(C.byref(cfg), None) == -1
    assert L.tsd_create(C.byref(cfg), None, 1 << 30, C.byref(h)) == -1 and not h.value
    assert L.tsd_create(C.byref(cfg), 0x1001, 1 << 40, C.byref(h)) == -1      # misaligned arena
    assert L.tsd_create(C.byref(cfg), 0x1000, 1024, C.byref(h)) == -1         # arena too small
    assert L.tsd_create(C.byref(cfg), 0x1000, 1 << 40, None) == -1
    for fn in (L.tsd_round, L.tsd_draft_propose, L.tsd_target_verify, L.tsd_target_step, L.tsd_reset_decode):
        assert fn(None, None) == -1
    assert L.tsd_accept_commit(None, None, None) == -1
    assert L.tsd_destroy(None) == -1
    assert L.tsd_set_sigma(None, 1.0, 1.0) == -1
    assert b"NULL" in L.tsd_last_error(None)


def test_measurement_taps_validate_before_any_launch():
    # argument checks come first, so they can be exercised without a GPU
    L = tsd.lib()
    assert L.tsd_bench_mfma(8, 100, None, None) == -1 and b"sink_dev" in L.tsd_last_error(None)
    assert L.tsd_bench_mfma(0, 100, 0x1000, None) == -1
    assert L.tsd_bench_mfma(8, 0, 0x1000, None) == -1
    assert L.tsd_bench_mfma(1 << 20, 1, 0x1000, None) == -1
    assert L.tsd_bench_copy(None, 0x1000, 1024, None) == -1
    assert L.tsd_bench_copy(0x1000, 0x2000, 1000, None) == -1                 # not a multiple of 16
    assert L.tsd_bench_gemm(tsd.TSD_BF16, 4, 64, 64, 64, 0x1000, 0x2000, 0x3000, None) == -1   # unknown variant
    assert L.tsd_bench_gemm(tsd.TSD_F32, 3, 64, 64, 64, 0x1000, 0x2000, 0x3000, None) == -1    # the FFN-up variant is bf16 only
    assert L.tsd_bench_gemm(tsd.TSD_BF16, 0, 64, 64, 60, 0x1000, 0x2000, 0x3000, None) == -1   # K not a multiple of 8
    assert L.tsd_trace_draft(None, None, 8, None, None) != 0                 # no handle


def test_static_accept_validates_before_touching_the_gpu():
    # tsd_accept_commit_static checks sizes against its fixed device array and its flags on the host first;
    # the pointers below are never dereferenced
    L = tsd.lib()
    dummy = C.c_void_p(4096)
    call = lambda B, K, P, flags=0, X=dummy: L.tsd_accept_commit_static(X, dummy, dummy, None, B, K, P, 1.0, 1.0, 0.0, 0, flags,
                                                                       dummy, dummy, None, None, None)
    assert call(4097, 4, 16) == -3 and b"4096" in L.tsd_last_error(None)
    assert call(8, 17, 16) == -3
    assert call(4096, 4, 96) == -3
    assert call(0, 4, 16) == -1 and call(8, 0, 16) == -1
    assert call(8, 4, 16, flags=tsd.TSD_FLAG_NO_GRAPH) == -1 and b"flags" in L.tsd_last_error(None)
    assert call(8, 4, 16, X=None) == -1
    assert L.tsd_accept_commit_static(dummy, dummy, dummy, None, 8, 4, 16, 0.0, 1.0, 0.0, 0, 0, dummy, dummy, None, None, None) == -1
    assert L.tsd_accept_commit_static(dummy, dummy, dummy, None, 8, 4, 16, 1.0, 1.0, 2.0, 0, 0, dummy, dummy, None, None, None) == -1
