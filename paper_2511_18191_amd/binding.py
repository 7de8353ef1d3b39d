"""ctypes binding of libtsd.so.  Every function of include/tsd.h is reachable as `lib().tsd_*`
with plain pointers; `Session` bundles the calls with torch-owned device memory (torch is used
for allocation and streams only; every step of the method runs inside the library's kernels)."""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))

TSD_F32, TSD_BF16 = 0, 1
TSD_TARGET, TSD_DRAFT = 0, 1
TSD_FLAG_SCRAMBLE_PAGES, TSD_FLAG_NO_TEMPERING, TSD_FLAG_NO_GRAPH, TSD_FLAG_NO_COMPACT, TSD_FLAG_NO_SKINNY, TSD_FLAG_SAMPLE_PROPOSALS, TSD_FLAG_NAIVE_VERIFY = 1, 2, 4, 8, 16, 32, 64
TSD_FLAG_THRESHOLD_RULE, TSD_FLAG_BATCH_SYNC, TSD_FLAG_NO_PINNED_COUNTS, TSD_FLAG_NO_FUSED_DRAFT, TSD_FLAG_FUSED_DRAFT = 128, 256, 512, 1024, 2048
TSD_FLAG_NO_WIDE_GEMM = 4096
KERNEL_CLASSES = ["embed", "qkv", "attn", "resid", "gelu", "head", "accept", "route", "draft"]   # TSD_K_* order


class TsdModelCfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_ff", C.c_int32),
                ("n_experts", C.c_int32), ("top_k", C.c_int32)]


class TsdConfig(C.Structure):
    _fields_ = [("target", TsdModelCfg), ("draft", TsdModelCfg), ("patch", C.c_int32), ("K", C.c_int32),
                ("max_batch", C.c_int32), ("max_tokens", C.c_int32), ("dtype", C.c_int32), ("page_tokens", C.c_int32),
                ("sigma_p", C.c_float), ("sigma_q", C.c_float), ("fallback_r", C.c_float), ("flags", C.c_uint32),
                ("seed", C.c_uint64)]


class TsdStats(C.Structure):
    _fields_ = [("rounds", C.c_int64), ("tested", C.c_int64), ("accepted", C.c_int64), ("committed", C.c_int64),
                ("near_ties", C.c_int64)]


class TsdLaunchRec(C.Structure):
    _fields_ = [("kernel_class", C.c_int32), ("model", C.c_int32), ("tile", C.c_int32), ("M", C.c_int32), ("N", C.c_int32),
                ("K", C.c_int32), ("ms", C.c_float), ("work", C.c_double)]


class TsdError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libtsd error {code}: {msg}")
        self.code = code


SYMBOLS = {
    "tsd_abi_version": ([], C.c_int),
    "tsd_last_error": ([C.c_void_p], C.c_char_p),
    "tsd_workspace_bytes": ([C.POINTER(TsdConfig), C.POINTER(C.c_size_t)], C.c_int),
    "tsd_weights_count": ([C.POINTER(TsdConfig), C.c_int, C.POINTER(C.c_size_t)], C.c_int),
    "tsd_create": ([C.POINTER(TsdConfig), C.c_void_p, C.c_size_t, C.POINTER(C.c_void_p)], C.c_int),
    "tsd_destroy": ([C.c_void_p], C.c_int),
    "tsd_load_weights": ([C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p], C.c_int),
    "tsd_prefill": ([C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p], C.c_int),
    "tsd_refill": ([C.c_void_p, C.POINTER(C.c_int32), C.c_int32, C.c_void_p, C.c_void_p], C.c_int),
    "tsd_reset_decode": ([C.c_void_p, C.c_void_p], C.c_int),
    "tsd_draft_propose": ([C.c_void_p, C.c_void_p], C.c_int),
    "tsd_target_verify": ([C.c_void_p, C.c_void_p], C.c_int),
    "tsd_accept_commit": ([C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
    "tsd_accept_commit_static": ([C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                  C.c_float, C.c_float, C.c_uint64, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                  C.c_void_p], C.c_int),
    "tsd_round": ([C.c_void_p, C.c_void_p], C.c_int),
    "tsd_run_rounds": ([C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
    "tsd_target_step": ([C.c_void_p, C.c_void_p], C.c_int),
    "tsd_num_active": ([C.c_void_p, C.POINTER(C.c_int32), C.c_void_p], C.c_int),
    "tsd_get_forecast": ([C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
    "tsd_get_round_io": ([C.c_void_p] + [C.c_void_p] * 6 + [C.c_void_p], C.c_int),
    "tsd_set_round_io": ([C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
    "tsd_get_state": ([C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
    "tsd_get_stats": ([C.c_void_p, C.POINTER(TsdStats), C.c_void_p], C.c_int),
    "tsd_profile_begin": ([C.c_void_p, C.c_int], C.c_int),
    "tsd_profile_end": ([C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_void_p], C.c_int),
    "tsd_set_route_tap": ([C.c_void_p, C.c_int, C.c_void_p, C.c_size_t], C.c_int),
    "tsd_profile_launches": ([C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(C.c_int32)], C.c_int),
    "tsd_bench_gemm": ([C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
    "tsd_bench_copy": ([C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p], C.c_int),
    "tsd_bench_mfma": ([C.c_int32, C.c_int32, C.c_void_p, C.c_void_p], C.c_int),
    "tsd_trace_draft": ([C.c_void_p, C.POINTER(C.c_int64), C.c_int32, C.POINTER(C.c_int32), C.c_void_p], C.c_int),
    "tsd_set_accept_override": ([C.c_void_p, C.c_float], C.c_int),
    "tsd_get_series_stats": ([C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
    "tsd_set_block_size": ([C.c_void_p, C.c_int32], C.c_int),
    "tsd_set_sigma_diag": ([C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p], C.c_int),
    "tsd_set_sigma": ([C.c_void_p, C.c_float, C.c_float], C.c_int),
}

_lib = None


def library_path():
    return os.path.join(HERE, "libtsd.so")


def lib():
    """Load libtsd.so (building it first only if it does not exist).  Raises if unavailable:
    there is no fallback implementation."""
    global _lib
    if _lib is None:
        # torch ships its own HIP runtime; load it first so that libtsd binds to the same one
        # (two runtimes in one process do not share device pointers or streams)
        import torch  # noqa: F401
        path = library_path()
        if not os.path.exists(path):
            from . import build as _build
            _build.build(verbose=False)
        handle = C.CDLL(path)
        for name, (argtypes, restype) in SYMBOLS.items():
            fn = getattr(handle, name)
            fn.argtypes, fn.restype = argtypes, restype
        _lib = handle
    return _lib


def make_config(target, draft, patch, K, max_batch, max_tokens, dtype, sigma_p, sigma_q=None, seed=0,
                page_tokens=16, flags=0, fallback_r=0.0):
    """target/draft: objects with n_layers, d_model, n_heads, d_ff, n_experts, top_k."""
    mk = lambda m: TsdModelCfg(m.n_layers, m.d_model, m.n_heads, m.d_ff, getattr(m, "n_experts", 0), getattr(m, "top_k", 0))
    dt = {"fp32": TSD_F32, "bf16": TSD_BF16}.get(dtype, dtype)
    return TsdConfig(mk(target), mk(draft), patch, K, max_batch, max_tokens, dt, page_tokens, sigma_p,
                     sigma_p if sigma_q is None else sigma_q, fallback_r, flags, seed)


def _check(rc, ctx=None):
    if rc != 0:
        msg = lib().tsd_last_error(ctx)
        raise TsdError(rc, msg.decode() if msg else "")


def bench_gemm(A, Wt, out=None, variant=0):
    """C = A @ Wt.T through libtsd's tiled GEMM on torch's current stream.  A: [M,K], Wt: [N,K]
    (both bf16 or both fp32, on the GPU); returns fp32 [M,N].  variant 1 fuses the RMSNorm row
    scale, variant 2 accumulates into `out`, variant 3 (bf16) is the FFN-up product with GELU and a bf16 result."""
    import torch
    M, K = A.shape
    N = Wt.shape[0]
    dt = TSD_BF16 if A.dtype == torch.bfloat16 else TSD_F32
    if out is None:
        out = torch.empty(M, N, dtype=torch.bfloat16 if (variant & 7) == 3 else torch.float32, device=A.device)
    _check(lib().tsd_bench_gemm(dt, variant, M, N, K, A.data_ptr(), Wt.data_ptr(), out.data_ptr(),
                                torch.cuda.current_stream(A.device).cuda_stream))
    return out


def accept_commit_static(X, mu_q, mu_p, sigma_p, sigma_q=None, rounds=None, fallback_r=0.0, seed=0, flags=0, want_taps=True):
    """tsd_accept_commit_static on torch's current stream.  X, mu_q: [B,K,P], mu_p: [B,K+1,P] float32 GPU tensors;
    rounds: int32 [B] or None.  Returns dict(n_acc, commit, ell, logu); the output tensors are allocated HERE, by
    the caller's side, before the call: the library call itself allocates nothing."""
    import torch
    B, K, P = X.shape
    dev = X.device
    n_acc = torch.full((B,), -7, dtype=torch.int32, device=dev)
    commit = torch.zeros(B, K + 1, P, dtype=torch.float32, device=dev)
    ell = torch.zeros(B, K, dtype=torch.float32, device=dev) if want_taps else None
    logu = torch.zeros(B, K, dtype=torch.float32, device=dev) if want_taps else None
    ptr = lambda t: None if t is None else t.data_ptr()
    _check(lib().tsd_accept_commit_static(X.data_ptr(), mu_q.data_ptr(), mu_p.data_ptr(), ptr(rounds), B, K, P, sigma_p,
                                          sigma_p if sigma_q is None else sigma_q, fallback_r, seed, flags, n_acc.data_ptr(),
                                          commit.data_ptr(), ptr(ell), ptr(logu), torch.cuda.current_stream(dev).cuda_stream))
    return dict(n_acc=n_acc, commit=commit, ell=ell, logu=logu)


def bench_copy(dst, src):
    """dst <- src with libtsd's plain copy kernel on torch's current stream (same-size GPU tensors)."""
    import torch
    n = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == n
    _check(lib().tsd_bench_copy(dst.data_ptr(), src.data_ptr(), n, torch.cuda.current_stream(src.device).cuda_stream))


def bench_mfma(blocks, iters, sink):
    """Matrix-core tap (see tsd_bench_mfma) on torch's current stream; sink: float32 GPU tensor [blocks * 256]."""
    import torch
    assert sink.dtype == torch.float32 and sink.numel() >= blocks * 256
    _check(lib().tsd_bench_mfma(blocks, iters, sink.data_ptr(), torch.cuda.current_stream(sink.device).cuda_stream))


class Session:
    """One libtsd handle plus the torch-owned device memory behind it."""

    def __init__(self, cfg, device="cuda:0"):
        import torch
        self.torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        L = lib()
        n = C.c_size_t()
        _check(L.tsd_workspace_bytes(C.byref(cfg), C.byref(n)))
        self.arena_bytes = n.value
        self.arena = torch.empty(n.value + 256, dtype=torch.uint8, device=self.device)
        base = (self.arena.data_ptr() + 255) & ~255
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(L.tsd_create(C.byref(cfg), base, n.value, C.byref(h)))
        self.h = h
        self.B = 0
        self.H = 0
        # a stream of its own (default priority): HIP graphs cannot be captured on the NULL stream
        self.stream = torch.cuda.Stream(self.device)

    def _stream(self):
        return self.stream.cuda_stream

    def sync(self):
        self.stream.synchronize()

    def _to_dev(self, t, dtype):
        """Copy to the device on torch's current stream and wait, so the library's stream sees it."""
        torch = self.torch
        if not isinstance(t, torch.Tensor):
            t = torch.from_numpy(t)
        t = t.to(self.device, dtype).contiguous()
        torch.cuda.current_stream(self.device).synchronize()
        return t

    def _new(self, *shape, dtype=None):
        """Output buffer for the library to fill; allocated after the library's stream is idle."""
        self.sync()
        return self.torch.empty(*shape, dtype=dtype or self.torch.float32, device=self.device)

    def close(self):
        if self.h:
            _check(lib().tsd_destroy(self.h))
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def weights_count(self, which):
        n = C.c_size_t()
        _check(lib().tsd_weights_count(C.byref(self.cfg), which, C.byref(n)))
        return n.value

    def load_weights(self, which, blob):
        """blob: float32 torch tensor on the device (or numpy array, copied over)."""
        blob = self._to_dev(blob, self.torch.float32)
        _check(lib().tsd_load_weights(self.h, which, blob.data_ptr(), blob.numel(), self._stream()), self.h)
        self.sync()  # blob may be freed after this

    def prefill(self, series, n_ctx_patches, horizon_steps):
        self.series = self._to_dev(series, self.torch.float32)
        self.B, self.H = self.series.shape[0], horizon_steps
        _check(lib().tsd_prefill(self.h, self.series.data_ptr(), self.B, n_ctx_patches, horizon_steps, self._stream()), self.h)

    def refill(self, slots, series):
        """New series (array [n, context steps]) into the listed slots of the running forecast."""
        slots = [int(x) for x in slots]
        arr = (C.c_int32 * len(slots))(*slots)
        self._refill_series = self._to_dev(series, self.torch.float32)     # kept alive until the stream has used it
        assert self._refill_series.shape[0] == len(slots)
        _check(lib().tsd_refill(self.h, arr, len(slots), self._refill_series.data_ptr(), self._stream()), self.h)

    def reset_decode(self):
        _check(lib().tsd_reset_decode(self.h, self._stream()), self.h)

    def draft_propose(self):
        _check(lib().tsd_draft_propose(self.h, self._stream()), self.h)

    def trace_draft(self, max_ticks=512):
        """Stage stamps (units of 10 ns) of one traced draft phase: see tsd_trace_draft."""
        buf = (C.c_int64 * max_ticks)()
        n = C.c_int32(0)
        _check(lib().tsd_trace_draft(self.h, buf, max_ticks, C.byref(n), self._stream()), self.h)
        return list(buf[: min(n.value, max_ticks)])

    def target_verify(self):
        _check(lib().tsd_target_verify(self.h, self._stream()), self.h)

    def accept_commit(self, forced_len=None):
        ptr = None
        if forced_len is not None:
            self._forced = self._to_dev(forced_len, self.torch.int32)
            ptr = self._forced.data_ptr()
        _check(lib().tsd_accept_commit(self.h, ptr, self._stream()), self.h)

    def round(self):
        _check(lib().tsd_round(self.h, self._stream()), self.h)

    def run_rounds(self, max_rounds=1 << 20):
        """Rounds until every series has its horizon (or max_rounds): returns (rounds run, series still active)."""
        r, n = C.c_int32(), C.c_int32()
        _check(lib().tsd_run_rounds(self.h, max_rounds, C.byref(r), C.byref(n), self._stream()), self.h)
        return r.value, n.value

    def target_step(self):
        _check(lib().tsd_target_step(self.h, self._stream()), self.h)

    def num_active(self):
        n = C.c_int32()
        _check(lib().tsd_num_active(self.h, C.byref(n), self._stream()), self.h)
        return n.value

    def get_forecast(self):
        out = self._new(self.B, self.H)
        _check(lib().tsd_get_forecast(self.h, out.data_ptr(), self._stream()), self.h)
        self.sync()
        return out

    def get_round_io(self):
        torch, B, K, P = self.torch, self.B, self.cfg.K, self.cfg.patch
        f = self._new
        X, mu_q, mu_p, ell, logu = f(B, K, P), f(B, K, P), f(B, K + 1, P), f(B, K), f(B, K)
        n_acc = f(B, dtype=torch.int32)
        _check(lib().tsd_get_round_io(self.h, X.data_ptr(), mu_q.data_ptr(), mu_p.data_ptr(), n_acc.data_ptr(),
                                      ell.data_ptr(), logu.data_ptr(), self._stream()), self.h)
        self.sync()
        return dict(X=X, mu_q=mu_q, mu_p=mu_p, n_acc=n_acc, ell=ell, logu=logu)

    def set_round_io(self, X, mu_q, mu_p):
        torch = self.torch
        self._inj = [self._to_dev(t, torch.float32) for t in (X, mu_q, mu_p)]
        _check(lib().tsd_set_round_io(self.h, *[t.data_ptr() for t in self._inj], self._stream()), self.h)

    def set_block_size(self, K):
        _check(lib().tsd_set_block_size(self.h, K), self.h)
        self.cfg.K = K

    def get_state(self):
        torch, B, P = self.torch, self.B, self.cfg.patch
        ln, cm, pend = self._new(B, dtype=torch.int32), self._new(B, dtype=torch.int32), self._new(B, P)
        _check(lib().tsd_get_state(self.h, ln.data_ptr(), cm.data_ptr(), pend.data_ptr(), self._stream()), self.h)
        self.sync()
        return dict(len=ln, committed=cm, pending=pend)

    def get_stats(self):
        s = TsdStats()
        _check(lib().tsd_get_stats(self.h, C.byref(s), self._stream()), self.h)
        return {k: getattr(s, k) for k, _ in TsdStats._fields_}

    def get_series_stats(self):
        """int64 [B, 5]: rounds, tested, accepted, committed, near_ties of every series."""
        out = self._new(self.B, 5, dtype=self.torch.int64)
        _check(lib().tsd_get_series_stats(self.h, out.data_ptr(), self._stream()), self.h)
        self.sync()
        return out

    def profile_begin(self, kernel_class):
        _check(lib().tsd_profile_begin(self.h, kernel_class), self.h)

    def profile_end(self):
        n, ms, work = C.c_int64(), C.c_double(), C.c_double()
        _check(lib().tsd_profile_end(self.h, C.byref(n), C.byref(ms), C.byref(work), self._stream()), self.h)
        return n.value, ms.value, work.value

    def route_tap(self, which=TSD_TARGET):
        """Install (and return) an int32 tensor [layers, max_batch, max_tokens, top_k], filled with -1, in which
        the passes through model `which` file the experts their router chose (see tsd_set_route_tap)."""
        m = self.cfg.target if which == TSD_TARGET else self.cfg.draft
        self.sync()
        tap = self.torch.full((m.n_layers, self.cfg.max_batch, self.cfg.max_tokens, m.top_k), -1, dtype=self.torch.int32,
                              device=self.device)
        self.torch.cuda.current_stream(self.device).synchronize()
        _check(lib().tsd_set_route_tap(self.h, which, tap.data_ptr(), tap.numel()), self.h)
        self._route_tap = tap
        return tap

    def profile_launches(self):
        """Per-launch records of the measurement the last profile_end closed: list of dicts."""
        n = C.c_int32()
        _check(lib().tsd_profile_launches(self.h, None, 0, C.byref(n)), self.h)
        buf = (TsdLaunchRec * max(1, n.value))()
        _check(lib().tsd_profile_launches(self.h, buf, n.value, C.byref(n)), self.h)
        return [{k: getattr(r, k) for k, _ in TsdLaunchRec._fields_} for r in buf[: n.value]]

    def set_accept_override(self, alpha):
        _check(lib().tsd_set_accept_override(self.h, alpha), self.h)

    def set_sigma(self, sigma_p, sigma_q=None):
        _check(lib().tsd_set_sigma(self.h, sigma_p, sigma_p if sigma_q is None else sigma_q), self.h)

    def set_sigma_diag(self, sigma_p_vec, sigma_q_vec):
        """Per-dimension scales [P] of the diagonal-covariance surrogate (arrays or tensors)."""
        sp, sq = self._to_dev(sigma_p_vec, self.torch.float32), self._to_dev(sigma_q_vec, self.torch.float32)
        assert sp.numel() == self.cfg.patch and sq.numel() == self.cfg.patch
        _check(lib().tsd_set_sigma_diag(self.h, sp.data_ptr(), sq.data_ptr(), self._stream()), self.h)


def session_for(inputs, flags=0, page_tokens=16, max_batch=None, sigma_q=None, fallback_r=0.0):
    """A Session sized for `inputs` (an object with cfg, wt, wd, seed as synth.Inputs has) with both
    models' weights loaded."""
    import synth
    c = inputs.cfg
    tc = make_config(c.target, c.draft, c.patch, c.K, max_batch or c.batch, c.max_tokens, c.dtype, c.sigma, sigma_q,
                     seed=inputs.seed, page_tokens=page_tokens, flags=flags, fallback_r=fallback_r)
    s = Session(tc)
    s.load_weights(TSD_TARGET, synth.flatten_weights(c.target, c.patch, inputs.wt))
    s.load_weights(TSD_DRAFT, synth.flatten_weights(c.draft, c.patch, inputs.wd))
    return s
