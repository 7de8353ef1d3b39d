"""GPU tests of the one-launch draft phase (Algorithm "One speculative round", first loop) against the
kernel-by-kernel draft phase and against the oracle."""
import numpy as np
import pytest
import torch

import paper_2511_18191_amd as tsd
from harness import TOL, Case, lockstep, rel_err

pytestmark = pytest.mark.gpu

FUSED, UNFUSED = tsd.TSD_FLAG_FUSED_DRAFT, tsd.TSD_FLAG_NO_FUSED_DRAFT


def _proposals(case, flags, rounds, **kw):
    """X of `rounds` consecutive rounds (every round fully accepted through the forced-length hook, so
    both handles walk the same states as long as their proposals agree)."""
    c = case.cfg
    sess = case.session(flags=flags, **kw)
    sess.prefill(case.context, c.n_ctx, c.horizon)
    out = []
    for _ in range(rounds):
        sess.draft_propose()
        X = sess.get_round_io()["X"].cpu().numpy().copy()
        out.append(X)
        sess.target_verify()
        sess.accept_commit(torch.zeros(c.batch, dtype=torch.int32, device="cuda"))   # reject at once: commit the target's patch
    return out


# mini2: 1 layer, 1 head, 5 series (one ragged group); mini3: 2 layers, 2 heads, 7 series, K=6;
# mini5: P=32 (one k-step of patch, two column blocks of head), K=8
@pytest.mark.parametrize("name", ["mini2", "mini3", "mini5"])
def test_fused_draft_matches_the_kernel_by_kernel_draft(name):
    case = Case(name)
    c = case.cfg
    a = _proposals(case, FUSED, 3)
    b = _proposals(case, UNFUSED, 3)
    for r, (xa, xb) in enumerate(zip(a, b)):
        e = rel_err(xa, xb).max()
        print(f"\n{name} round {r}: fused vs unfused proposals rel err {e:.2e}")
        # same operands, same roundings, another summation order inside the products
        assert e <= 1e-2
        assert np.isfinite(xa).all()


@pytest.mark.parametrize("max_batch", [1100, 600])
def test_fused_draft_with_eight_and_four_series_per_workgroup(max_batch):
    """A handle sized for a large batch packs 8 (4) series into a workgroup: mini3's 7 series then fill one
    workgroup with a dead slot (two workgroups, the second with a dead slot)."""
    case = Case("mini3")
    a = _proposals(case, FUSED, 2, max_batch=max_batch)
    b = _proposals(case, UNFUSED, 2, max_batch=max_batch)
    for xa, xb in zip(a, b):
        assert np.isfinite(xa).all()
        assert rel_err(xa, xb).max() <= 1e-2


@pytest.mark.parametrize("name", ["mini2", "mini3", "mini5"])
@pytest.mark.parametrize("flags", [FUSED, UNFUSED])
def test_both_bf16_draft_paths_follow_the_oracle(name, flags):
    case = Case(name)
    c = case.cfg
    sess = case.session(flags=flags)
    rep = lockstep(case, sess)
    assert rep["max_rel_X"] <= TOL[c.dtype] and rep["max_rel_mu_p"] <= TOL[c.dtype]
    assert sess.get_stats()["committed"] == c.batch * c.T


def test_fused_draft_with_compaction_and_graphs_is_deterministic():
    """Whole decodes (round graphs, compacted active lists whose device-side count shrinks): two runs give
    the same bits, and the forecast is the kernel-by-kernel draft's within the bf16 tolerance wherever the
    two decodes took the same decisions."""
    case = Case("mini3")
    c = case.cfg
    outs = []
    for flags in (FUSED, FUSED, UNFUSED):
        sess = case.session(flags=flags)
        sess.prefill(case.context, c.n_ctx, c.horizon)
        sess.run_rounds()
        outs.append((sess.get_forecast().cpu().numpy().copy(), sess.get_series_stats().cpu().numpy().copy()))
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])
    same = (outs[0][1] == outs[2][1]).all(axis=1)
    print(f"\nseries with identical decisions fused/unfused: {int(same.sum())} of {c.batch}")
    assert same.any()
    for b in np.nonzero(same)[0]:
        assert rel_err(outs[0][0][b], outs[2][0][b]) <= 6e-2


def test_single_series_handle_runs_the_fused_draft():
    """max_batch = 1: one series per workgroup, one workgroup."""
    import synth
    case = Case("mini3")
    c = case.cfg
    outs = []
    for flags in (FUSED, UNFUSED):
        sess = case.session(flags=flags, max_batch=1)
        sess.prefill(case.context[:1], c.n_ctx, c.horizon)
        sess.draft_propose()
        outs.append(sess.get_round_io()["X"].cpu().numpy().copy())
    assert np.isfinite(outs[0]).all()
    assert rel_err(outs[0], outs[1]).max() <= 1e-2


def test_fused_draft_full_size_cfg2_in_step_with_the_unfused_path():
    """Benchmark size (B = 256: 128 workgroups of 2 series, K = 4), where the one-launch draft is the default."""
    case = Case("cfg2")
    a = _proposals(case, 0, 2)
    b = _proposals(case, UNFUSED, 2)
    for xa, xb in zip(a, b):
        assert np.isfinite(xa).all()
        assert rel_err(xa, xb).max() <= 1e-2
