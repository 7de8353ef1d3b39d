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


def _decode(sess):
    sess.run_rounds()
    return sess.get_forecast().cpu().numpy().copy(), sess.get_stats()


def test_fused_draft_page_scramble_batch_independence_and_small_pages():
    """The one-launch draft walks the same page tables: physical page placement is invisible, a series alone
    decodes as it does in the batch (whatever the other slots of its workgroup hold), 8-token pages work."""
    case = Case("mini3", sigma=0.5)
    c = case.cfg

    def run(ctx, **kw):
        sess = case.session(**kw)
        sess.prefill(ctx, c.n_ctx, c.horizon)
        return _decode(sess)[0]

    full = run(case.context, flags=FUSED)
    scr = run(case.context, flags=FUSED | tsd.TSD_FLAG_SCRAMBLE_PAGES, page_tokens=8)
    np.testing.assert_array_equal(full, scr)
    alone = run(case.context[:1], flags=FUSED)
    np.testing.assert_array_equal(alone[0], full[0])
    three = run(case.context[:3], flags=FUSED)       # an odd count: the last workgroup has a dead slot
    np.testing.assert_array_equal(three, full[:3])


@pytest.mark.parametrize("name,K,horizon,n_ctx", [("mini2", 1, 96, 2), ("mini2", 16, 96 * 20, 3), ("mini2", 3, 50, 6)])
def test_fused_draft_edge_shapes(name, K, horizon, n_ctx):
    """K = 1, K = 16 (maximum), a two-patch context, a horizon shorter than one patch."""
    import dataclasses
    case = Case(name, K=K, horizon=horizon, sigma=0.7)
    case.cfg = dataclasses.replace(case.cfg, context=n_ctx * 96)
    case.context = np.ascontiguousarray(case.series[:, : n_ctx * 96])
    c = case.cfg
    sess = case.session(flags=FUSED)
    rep = lockstep(case, sess, tol=0.06 if K == 16 else None)
    assert all(1 <= L <= K + 1 for L in rep["lengths"])
    assert sess.num_active() == 0 and sess.get_stats()["committed"] == c.batch * c.T


def test_fused_draft_block_size_change_equals_a_fresh_handle_bitwise():
    big = Case("mini3", K=6, sigma=0.5)
    small = Case("mini3", K=3, sigma=0.5)
    c = small.cfg
    flags = FUSED | tsd.TSD_FLAG_NO_SKINNY
    s_big = big.session(flags=flags)
    s_big.prefill(big.context, c.n_ctx, c.horizon)
    s_big.set_block_size(3)
    f1, st1 = _decode(s_big)
    s_small = small.session(flags=flags)
    s_small.prefill(small.context, c.n_ctx, c.horizon)
    f2, st2 = _decode(s_small)
    np.testing.assert_array_equal(f1, f2)
    assert st1 == st2


def test_fused_draft_stream_through_refilled_slots():
    """Continuous batching: finished slots are refilled mid-decode and the one-launch draft picks the new
    series up from the slot's state; draft = target accepts everything, so stream and batches agree exactly."""
    from paper_2511_18191_amd import serve
    case = Case("mini2", B=10, sigma=0.5, draft_is_target=True)
    c = case.cfg
    sess = case.session(max_batch=5, flags=FUSED)
    out, _ = serve.run_stream(sess, case.context, c.n_ctx, c.horizon)
    ref = serve.run_batches(sess, case.context, c.n_ctx, c.horizon)
    np.testing.assert_array_equal(out.cpu().numpy(), ref.cpu().numpy())
    # and against the kernel-by-kernel draft within the bf16 tolerance (identical decisions: all accepted)
    sess2 = case.session(max_batch=5, flags=UNFUSED)
    ref2 = serve.run_batches(sess2, case.context, c.n_ctx, c.horizon)
    assert rel_err(out.cpu().numpy(), ref2.cpu().numpy()).max() <= 6e-2


def test_fused_draft_with_threshold_rule_and_batch_sync():
    case = Case("mini3", sigma=0.6)
    c = case.cfg
    sess = case.session(flags=FUSED | tsd.TSD_FLAG_THRESHOLD_RULE | tsd.TSD_FLAG_BATCH_SYNC)
    rep = lockstep(case, sess, rule="threshold", sync=True)
    assert rep["max_rel_X"] <= TOL[c.dtype] and rep["max_rel_mu_p"] <= TOL[c.dtype]
    assert sess.get_stats()["committed"] == c.batch * c.T


@pytest.mark.parametrize("draft", [(2, 384, 6, 1536), (1, 256, 4, 1024), (3, 192, 3, 768)])
def test_fused_draft_other_widths_follow_the_oracle(draft):
    """Draft shapes of the benchmark configurations on the scaled-down target: 6 heads with 12 k-steps in
    4-step chunks (configuration 3's draft), 4 heads in 8-step chunks (configurations 2, 4, 5), and an odd
    width (6 k-steps: the fragment copy pads every block to 8) with three layers."""
    from synth.configs import ModelCfg
    case = Case("mini3", sigma=0.6, draft=ModelCfg(*draft))
    c = case.cfg
    sess = case.session(flags=FUSED)
    rep = lockstep(case, sess)
    assert rep["max_rel_X"] <= TOL[c.dtype] and rep["max_rel_mu_p"] <= TOL[c.dtype]
    assert sess.get_stats()["committed"] == c.batch * c.T
    # and the kernel-by-kernel path on the same shapes
    a = _proposals(case, FUSED, 1)[0]
    b = _proposals(case, UNFUSED, 1)[0]
    assert np.isfinite(a).all() and rel_err(a, b).max() <= 1e-2


@pytest.mark.parametrize("name,sigma,r", [("mini2", 0.5, 0.25), ("mini3", 0.6, 0.3)])
def test_fused_draft_with_sampled_proposals(name, sigma, r):
    """Sec. "Fallback Correction and Sampled Variants": x_i = mu_q^(i) + sigma_q eps drawn inside the one-launch
    draft (the next step consumes the draw): rounds in step with the oracle, and X - mu_q is sigma_q times the
    oracle generator's normals, element by element."""
    from oracle import tsd_oracle as orc
    flags = FUSED | tsd.TSD_FLAG_SAMPLE_PROPOSALS
    case = Case(name, sigma=sigma)
    c = case.cfg
    sess = case.session(flags=flags, fallback_r=r)
    rep = lockstep(case, sess, sample_proposals=True, fallback_r=r)
    assert rep["max_rel_X"] <= TOL[c.dtype] and rep["max_rel_mu_p"] <= TOL[c.dtype]
    assert sess.get_stats()["committed"] == c.batch * c.T
    sess = case.session(flags=flags, fallback_r=r)
    sess.prefill(case.context, c.n_ctx, c.horizon)
    for rnd in range(2):
        sess.draft_propose()
        sess.target_verify()
        sess.accept_commit()
        io = {k: v.cpu().numpy() for k, v in sess.get_round_io().items()}
        for b in range(c.batch):
            for i in range(c.K):
                z = (io["X"][b, i].astype(np.float64) - io["mu_q"][b, i]) / c.sigma
                np.testing.assert_allclose(z, orc.normal(case.seed, b, rnd, i + 1, orc.STREAM_PROPOSAL, c.patch), atol=2e-4)


def test_stage_tap_of_the_one_launch_draft():
    """tsd_trace_draft: 2 + steps * (3 + 5 * layers) increasing stamps, proposals unchanged by tracing, and a
    clean error on a handle that runs the draft kernel by kernel."""
    case = Case("mini3")
    c = case.cfg
    sess = case.session(flags=FUSED)
    sess.prefill(case.context, c.n_ctx, c.horizon)
    sess.draft_propose()
    x0 = sess.get_round_io()["X"].cpu().numpy().copy()
    t = sess.trace_draft()
    assert len(t) == 2 + c.K * (3 + 5 * c.draft.n_layers)
    assert all(b > a for a, b in zip(t, t[1:]))
    assert (t[-1] - t[0]) * 0.01 < 5000.0          # the whole phase takes well under 5 ms
    np.testing.assert_array_equal(sess.get_round_io()["X"].cpu().numpy(), x0)
    assert len(sess.trace_draft(max_ticks=5)) == 5
    plain = case.session(flags=UNFUSED)
    plain.prefill(case.context, c.n_ctx, c.horizon)
    with pytest.raises(tsd.TsdError):
        plain.trace_draft()
