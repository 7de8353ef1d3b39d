"""GPU tests of the standalone variant's acceptance (Table "TiRex configuration"): the deterministic
threshold rule ||x - mu_p||_d^2 <= sigma^2 and the batch-synchronised commit, against the oracle."""
import numpy as np
import pytest

import paper_2511_18191_amd as tsd
from harness import TOL, Case, lockstep
from oracle import tsd_oracle as orc

pytestmark = pytest.mark.gpu

THR, SYNC = tsd.TSD_FLAG_THRESHOLD_RULE, tsd.TSD_FLAG_BATCH_SYNC


def splitting_sigma(name):
    """A scale at which about half of the first round's proposals lie inside the threshold ball
    (median scaled distance between proposal and target mean over a few series, from the oracle)."""
    case = Case(name)
    c = case.cfg
    d = []
    for b in range(min(4, c.batch)):
        rec = orc.spec_round(case.Wt, c.target, case.Wd, c.draft, case.oracle_hist(b)[0], c.K, 1.0, 1.0, lambda i: 0.5)
        d.extend(np.sqrt(np.mean((rec["X"] - rec["mu_p"][: c.K]) ** 2, axis=1)))
    return float(np.median(d))


@pytest.mark.parametrize("name", ["cfg1", "mini2_fp32", "mini2", "mini5_fp32"])
@pytest.mark.parametrize("flags,rule,sync", [(THR, "threshold", False), (SYNC, "ratio", True),
                                              (THR | SYNC, "threshold", True)])
def test_lockstep_with_oracle(name, flags, rule, sync):
    sigma = splitting_sigma(name)
    case = Case(name, sigma=sigma)
    c = case.cfg
    sess = case.session(flags=flags)
    rep = lockstep(case, sess, rule=rule, sync=sync)
    print(f"\n{name} {rule} sync={sync} sigma={sigma:.4f}: rounds {rep['rounds']} accepted {rep['accepted']}/{rep['tested']} "
          f"near ties {rep['near_ties']} mismatched {rep['mismatched']} X {rep['max_rel_X']:.2e} mu_p {rep['max_rel_mu_p']:.2e}")
    assert rep["max_rel_X"] <= TOL[c.dtype] and rep["max_rel_mu_p"] <= TOL[c.dtype]
    assert 0 < rep["accepted"] < rep["tested"]            # both outcomes occurred
    if c.dtype == "fp32":
        assert rep["mismatched"] <= rep["near_ties"]
    st = sess.get_stats()
    assert st["committed"] == c.batch * c.T
    # the statistics keep every series' own test (the oracle's counts were forced in, ties included)
    assert (st["tested"], st["accepted"]) == (rep["tested"], rep["accepted"]) or rep["mismatched"] > 0
    if sync:
        # every round kept one length for all series: the committed forecast of each series is the oracle's
        f = sess.get_forecast().cpu().numpy()
        for b in range(c.batch):
            _, m, s = case.oracle_hist(b)
            ref = (rep["Y"][b].reshape(-1) * s + m)[: c.horizon]
            tol = (2e-4 if c.dtype == "fp32" else 6e-2) * max(1.0, np.abs(ref).max())
            np.testing.assert_allclose(f[b], ref, rtol=0, atol=tol)


@pytest.mark.parametrize("name", ["cfg1", "mini2_fp32"])
def test_free_running_matches_the_synchronised_oracle(name):
    sigma = splitting_sigma(name)
    case = Case(name, sigma=sigma)
    c = case.cfg
    s = case.session(flags=THR | SYNC)
    s.prefill(case.context, c.n_ctx, c.horizon)
    rounds = 0
    while s.num_active() > 0:
        s.round()
        rounds += 1
        st = s.get_state()
        assert len(set(st["committed"].cpu().tolist())) == 1          # the batch stays in step
    f = s.get_forecast().cpu().numpy()
    stats = s.get_stats()
    per = s.get_series_stats().cpu().numpy()
    ref, rst = orc.forecast_spec_sync(case.Wt, c.target, case.Wd, c.draft, case.context.astype(np.float64), c.patch,
                                      c.horizon, c.K, sigma, sigma, case.seed, rule="threshold")
    print(f"\n{name}: rounds {rounds} (oracle {rst[0]['rounds']}), near ties {stats['near_ties']}")
    if stats["near_ties"] == 0:
        assert rounds == rst[0]["rounds"]
        for b in range(c.batch):
            assert (per[b][1], per[b][2], per[b][3]) == (rst[b]["tested"], rst[b]["accepted"], rst[b]["committed"])
        np.testing.assert_allclose(f, ref, rtol=0, atol=2e-4 * max(1.0, np.abs(ref).max()))


def test_threshold_taps_and_graph_replay_bitwise():
    sigma = splitting_sigma("mini3")
    case = Case("mini3", sigma=sigma)
    c = case.cfg
    out = []
    for flags in (THR | SYNC, THR | SYNC | tsd.TSD_FLAG_NO_GRAPH):
        s = case.session(flags=flags)
        s.prefill(case.context, c.n_ctx, c.horizon)
        first = None
        while s.num_active() > 0:
            s.round()
            if first is None:
                first = {k: v.cpu().numpy() for k, v in s.get_round_io().items()}
        out.append((s.get_forecast().cpu().numpy(), s.get_stats(), first))
    (f0, s0, io), (f1, s1, _) = out
    assert np.array_equal(f0, f1) and s0 == s1
    # first round: no uniform is drawn, log u is the constant -1/2 wherever a position was tested, and the
    # recorded count is the number of leading positions whose recorded ell is at least -1/2
    K = c.K
    for b in range(c.batch):
        n = int(io["n_acc"][b])
        t = n + (n < K)
        assert np.all(io["logu"][b][:t] == -0.5) and np.all(np.isnan(io["logu"][b][t:]))
        assert np.all(io["ell"][b][:n] >= -0.5) and (n == K or io["ell"][b][n] < -0.5)
        # ell itself: the scaled squared distance recomputed from the tapped tensors
        e = np.mean((io["X"][b][:t].astype(np.float64) - io["mu_p"][b][:t]) ** 2, axis=1) / (2 * sigma * sigma)
        np.testing.assert_allclose(-io["ell"][b][:t], e, rtol=1e-4)


def test_full_size_cfg2_batch_stays_in_step():
    # benchmark shape, in the launch configuration bench.py times (graph replay, device-side counts)
    case = Case("cfg2", sigma=0.5)
    c = case.cfg
    res = {}
    for name, flags in (("free", 0), ("sync", SYNC), ("thr_sync", THR | SYNC)):
        s = case.session(flags=flags)
        s.prefill(case.context, c.n_ctx, c.horizon)
        rounds, prev = 0, 0
        while s.num_active() > 0:
            s.round()
            rounds += 1
            if flags & SYNC:
                com = s.get_state()["committed"].cpu().numpy()
                assert com.min() == com.max() and com[0] > prev
                io = s.get_round_io()
                n_own = io["n_acc"].cpu().numpy()
                assert com[0] - prev == min(n_own.min() + 1, c.T - prev)   # the round kept the smallest own count
                prev = int(com[0])
        st = s.get_stats()
        assert st["committed"] == c.batch * c.T
        assert np.isfinite(s.get_forecast().cpu().numpy()).all()
        res[name] = (rounds, st)
    print("\ncfg2 rounds:", {k: v[0] for k, v in res.items()},
          "acceptance:", {k: round(v[1]["accepted"] / max(1, v[1]["tested"]), 3) for k, v in res.items()})
    assert res["sync"][0] >= res["free"][0]               # waiting for the slowest series never saves rounds
