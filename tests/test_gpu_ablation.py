"""GPU tests of the ablation switches: the naive per-prefix verifier (the component ablation's
"w/o single-pass verification") against single-pass verification and against the oracle."""
import numpy as np
import pytest

import paper_2511_18191_amd as tsd
from harness import TOL, Case, lockstep, rel_err

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,tol", [("mini2_fp32", 1e-5), ("cfg1", 1e-5), ("mini3", 6e-3)])
def test_naive_verifier_gives_the_single_pass_means(name, tol):
    # invariant 1 on the GPU: K+1 separate prefix passes read the same K+1 boundaries as one causal pass
    case = Case(name, sigma=0.5)
    c = case.cfg
    out = []
    for flags in (0, tsd.TSD_FLAG_NAIVE_VERIFY):
        s = case.session(flags=flags)
        s.prefill(case.context, c.n_ctx, c.horizon)
        s.draft_propose()
        s.target_verify()
        out.append(s.get_round_io()["mu_p"].cpu().numpy())
    err = rel_err(out[1], out[0]).max()
    print(f"\n{name}: naive vs single-pass mu_p rel {err:.2e}")
    assert err <= tol


@pytest.mark.parametrize("name", ["mini2_fp32", "mini2"])
def test_naive_verifier_lockstep_with_oracle(name):
    case = Case(name, sigma=0.5)
    c = case.cfg
    sess = case.session(flags=tsd.TSD_FLAG_NAIVE_VERIFY)
    rep = lockstep(case, sess)
    assert rep["max_rel_X"] <= TOL[c.dtype] and rep["max_rel_mu_p"] <= TOL[c.dtype]
    if c.dtype == "fp32":
        assert rep["mismatched"] <= rep["near_ties"]
    assert sess.get_stats()["committed"] == c.batch * c.T


def test_naive_verifier_free_running_matches_single_pass_fp32():
    case = Case("mini2_fp32", sigma=0.5)
    c = case.cfg
    fcs = []
    for flags in (0, tsd.TSD_FLAG_NAIVE_VERIFY):
        s = case.session(flags=flags)
        s.prefill(case.context, c.n_ctx, c.horizon)
        while s.num_active() > 0:
            s.round()
        fcs.append((s.get_forecast().cpu().numpy(), s.get_stats()))
    (f0, s0), (f1, s1) = fcs
    if s0["near_ties"] == 0 and s1["near_ties"] == 0:
        assert (s0["accepted"], s0["tested"], s0["rounds"]) == (s1["accepted"], s1["tested"], s1["rounds"])
        np.testing.assert_allclose(f1, f0, rtol=0, atol=1e-4 * np.abs(f0).max())


def test_ablation_module_runs():
    from paper_2511_18191_amd import ablate
    import synth
    inputs = synth.Inputs("mini2", sigma=0.5)
    full = ablate.run(inputs, 0, 0.0, reps=1)
    raw = ablate.run(inputs, tsd.TSD_FLAG_NO_TEMPERING, 0.0, reps=1)
    noisy = ablate.run(inputs, 0, 0.5, reps=1)
    assert raw["accept"] < full["accept"]                 # the 0/1 gate
    assert raw["dev"] <= full["dev"] + 1e-12              # rejecting everything reproduces the target-only forecast
    assert noisy["dev"] > full["dev"]                     # fallback noise only hurts
    # deterministic fidelity (Eq. 9): the full rule's mean deviation stays under 2 sigma^2 / e per patch
    # (a bound on the per-patch expectation given equal histories; with drifted histories it is a sanity scale)
    assert full["dev"] < 10 * 2 * 0.5 ** 2 / np.e
