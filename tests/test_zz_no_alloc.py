"""tsd_accept_commit_static (the entry point for callers that cannot allocate: its kernel state lives in a
fixed device array inside the library) against tsd_accept_commit on a handle, through the C ABI: same kernel,
so every output must agree to the bit.  Two calls in a row, the second with a smaller input, so that state the
first call left in the shared array would show."""
import ctypes as C

import numpy as np
import pytest
import torch

from harness import Case

pytestmark = pytest.mark.gpu


def _inputs(B, K, P, seed, sq):
    rng = np.random.default_rng(seed)
    mu_p = rng.standard_normal((B, K + 1, P)).astype(np.float32)
    gap = rng.uniform(0.0, 1.2, size=(B, K, 1)).astype(np.float32)
    mu_q = (mu_p[:, :K] + gap * rng.standard_normal((B, K, P))).astype(np.float32)
    X = (mu_q + sq * 0.3 * rng.standard_normal((B, K, P))).astype(np.float32)
    return X, mu_q, mu_p


def _through_handle(case, sess, X, mu_q, mu_p, n_rounds_before):
    """The existing entry point: a handle whose forecast has room for a whole round (T >= K + 1); `n_rounds_before`
    earlier rounds advance every series' round counter first."""
    c = case.cfg
    sess.prefill(case.context, c.n_ctx, c.horizon)
    for _ in range(n_rounds_before):
        sess.set_round_io(torch.from_numpy(X), torch.from_numpy(mu_q), torch.from_numpy(mu_p))
        sess.accept_commit(np.zeros(c.batch, np.int32))      # forced to keep nothing: one patch committed per round
    before = sess.get_state()["committed"].cpu().numpy()
    sess.set_round_io(torch.from_numpy(X), torch.from_numpy(mu_q), torch.from_numpy(mu_p))
    sess.accept_commit()
    io = {k: v.cpu().numpy() for k, v in sess.get_round_io().items()}
    st = sess.get_state()
    return io, st["pending"].cpu().numpy(), st["committed"].cpu().numpy() - before


@pytest.mark.parametrize("flags_name", ["none", "threshold", "sync"])
def test_static_entry_point_equals_handle_entry_point(flags_name):
    import paper_2511_18191_amd as tsd
    flags = {"none": 0, "threshold": tsd.TSD_FLAG_THRESHOLD_RULE, "sync": tsd.TSD_FLAG_BATCH_SYNC}[flags_name]
    sq, sp, K, P = 0.35, 0.5 if flags_name != "threshold" else 1.1, 6, 96
    for B, seed, rounds_before in ((1024, 7, 0), (37, 8, 2)):          # the second call is smaller and at a later round
        case = Case("mini3", B=B, sigma=sp, horizon=96 * 12)          # T = 12 >= 2 + K + 1
        sess = case.session(sigma_q=sq, flags=flags)
        X, mu_q, mu_p = _inputs(B, K, P, seed, sq)
        io, pending, dcommit = _through_handle(case, sess, X, mu_q, mu_p, rounds_before)
        dX, dq, dp = (torch.from_numpy(a).cuda() for a in (X, mu_q, mu_p))
        rounds = torch.full((B,), rounds_before, dtype=torch.int32, device="cuda")
        out = tsd.accept_commit_static(dX, dq, dp, sp, sq, rounds=rounds, seed=case.seed, flags=flags)
        torch.cuda.synchronize()
        n_acc = out["n_acc"].cpu().numpy()
        np.testing.assert_array_equal(n_acc, io["n_acc"])
        np.testing.assert_array_equal(out["ell"].cpu().numpy(), io["ell"])           # NaN pattern included
        np.testing.assert_array_equal(out["logu"].cpu().numpy(), io["logu"])
        n_keep = np.full(B, n_acc.min()) if flags_name == "sync" else n_acc
        np.testing.assert_array_equal(dcommit, n_keep + 1)
        commit = out["commit"].cpu().numpy()
        for b in range(B):
            n = n_keep[b]
            np.testing.assert_array_equal(commit[b, :n], X[b, :n])
            np.testing.assert_array_equal(commit[b, n], pending[b])                  # corrected / bonus patch
            assert not commit[b, n + 1:].any()                                       # later rows untouched
        assert 0 < n_acc.mean() < K or flags_name == "threshold"
        sess.close()
    # without the taps, and with no round counters given (= round 0): same counts as the first call of a handle
    case = Case("mini3", B=5, sigma=sp, horizon=96 * 12)
    sess = case.session(sigma_q=sq, flags=flags)
    X, mu_q, mu_p = _inputs(5, K, P, 9, sq)
    io, pending, _ = _through_handle(case, sess, X, mu_q, mu_p, 0)
    out = tsd.accept_commit_static(*(torch.from_numpy(a).cuda() for a in (X, mu_q, mu_p)), sp, sq, seed=case.seed, flags=flags,
                                   want_taps=False)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out["n_acc"].cpu().numpy(), io["n_acc"])


def test_static_entry_point_rejects_sizes_beyond_its_array():
    import paper_2511_18191_amd as tsd
    L = tsd.lib()
    buf = torch.zeros(16, device="cuda")
    p = buf.data_ptr()
    call = lambda B, K, P: L.tsd_accept_commit_static(p, p, p, None, B, K, P, 1.0, 1.0, 0.0, 0, 0, p, p, None, None, None)
    assert call(4097, 4, 16) == -3 and b"4096" in L.tsd_last_error(None)
    assert call(8, 17, 16) == -3
    assert call(4096, 4, 96) == -3          # B * P beyond 262144
    assert call(0, 4, 16) == -1
    assert L.tsd_accept_commit_static(p, p, p, None, 8, 4, 16, 1.0, 1.0, 0.0, 0, 4, p, p, None, None, None) == -1   # a flag that does not apply
