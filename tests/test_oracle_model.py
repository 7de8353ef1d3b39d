"""Pins for the oracle's transformer pieces: library routines for the sub-steps that have one,
textbook properties for the rest, and structural special cases of the whole forward."""
import math

import numpy as np
import torch
import torch.nn.functional as F

import synth
from oracle import tsd_oracle as orc

T64 = torch.float64


def _tiny(n_experts=0, seed=3, gains=True):
    m = synth.ModelCfg(2, 32, 2, 64, n_experts, 2 if n_experts else 0)
    W = orc.as_f64(synth.make_weights(m, 8, np.random.default_rng(seed), random_gains=gains, std=0.3))
    return m, W


def test_rmsnorm_matches_torch():
    rng = np.random.default_rng(0)
    x, g = rng.standard_normal((5, 32)), rng.standard_normal(32)
    ref = F.rms_norm(torch.tensor(x, dtype=T64), (32,), torch.tensor(g, dtype=T64), eps=1e-6).numpy()
    np.testing.assert_allclose(orc.rmsnorm(x, g), ref, rtol=1e-12)


def test_gelu_matches_torch_tanh_form():
    z = np.linspace(-6, 6, 101)
    ref = F.gelu(torch.tensor(z, dtype=T64), approximate="tanh").numpy()
    np.testing.assert_allclose(orc.gelu_tanh(z), ref, rtol=1e-12, atol=1e-15)


def test_attention_matches_torch_sdpa_causal():
    rng = np.random.default_rng(1)
    n, H, hd = 7, 3, 16
    q, k, v = rng.standard_normal((3, n, H, hd))
    tq, tk, tv = (torch.tensor(a, dtype=T64).permute(1, 0, 2)[None] for a in (q, k, v))
    ref = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).reshape(n, H * hd).numpy()
    np.testing.assert_allclose(orc.attention(q, k, v), ref, rtol=1e-10, atol=1e-12)
    # one key: the output is that key's value
    np.testing.assert_allclose(orc.attention(q[:1], k[:1], v[:1]), v[:1].reshape(1, -1), rtol=1e-14)


def test_rope_properties():
    rng = np.random.default_rng(2)
    hd = 16
    x = rng.standard_normal((4, 2, hd))
    # position 0 is the identity; rotations preserve each pair's norm
    np.testing.assert_array_equal(orc.rope(x, np.zeros(4)), x)
    y = orc.rope(x, np.array([3, 11, 0, 40]))
    np.testing.assert_allclose((y ** 2).sum(-1), (x ** 2).sum(-1), rtol=1e-12)
    # pair (i, i + hd/2) turns by pos * base^(-2i/hd): check one coordinate pair by hand
    pos, i = 5, 3
    th = pos * 10000.0 ** (-2 * i / hd)
    e = np.zeros((1, 1, hd)); e[0, 0, i] = 1.0
    r = orc.rope(e, np.array([pos]))[0, 0]
    assert math.isclose(r[i], math.cos(th), rel_tol=1e-12) and math.isclose(r[i + hd // 2], math.sin(th), rel_tol=1e-12)
    assert np.count_nonzero(r) == 2
    # relative-position property: <R_m q, R_n k> depends on m - n only
    q, k = rng.standard_normal((2, 1, 1, hd))
    d1 = np.sum(orc.rope(q, np.array([9])) * orc.rope(k, np.array([4])))
    d2 = np.sum(orc.rope(q, np.array([25])) * orc.rope(k, np.array([20])))
    d3 = np.sum(orc.rope(q, np.array([4])) * orc.rope(k, np.array([9])))
    assert math.isclose(d1, d2, rel_tol=1e-10) and not math.isclose(d1, d3, rel_tol=1e-3)


def test_forward_collapses_to_two_matmuls_without_mixing():
    # with W_o = W_2 = 0 every block adds nothing: mu = RMSNorm(tokens W_e; g_f) W_h
    m, W = _tiny()
    for l in range(m.n_layers):
        W[f"l{l}.W_o"][:] = 0
        W[f"l{l}.W_2"][:] = 0
    tok = np.random.default_rng(4).standard_normal((6, 8))
    x = tok @ W["W_e"]
    ref = (x / np.sqrt((x * x).mean(-1, keepdims=True) + 1e-6) * W["g_f"]) @ W["W_h"]
    np.testing.assert_allclose(orc.forward(W, m, tok), ref, rtol=1e-12)


def test_forward_single_token_closed_form():
    # one token: attention returns v, RoPE at position 0 is the identity
    m = synth.ModelCfg(1, 32, 2, 64)
    W = orc.as_f64(synth.make_weights(m, 8, np.random.default_rng(8), random_gains=True, std=0.3))
    tok = np.random.default_rng(9).standard_normal((1, 8))
    rn = lambda x, g: (F.rms_norm(torch.tensor(x, dtype=T64), (32,), torch.tensor(g, dtype=T64), eps=1e-6)).numpy()
    x = tok @ W["W_e"]
    x = x + (rn(x, W["l0.g1"]) @ W["l0.W_v"]) @ W["l0.W_o"]
    h = F.gelu(torch.tensor(rn(x, W["l0.g2"]) @ W["l0.W_1"], dtype=T64), approximate="tanh").numpy()
    x = x + h @ W["l0.W_2"]
    np.testing.assert_allclose(orc.forward(W, m, tok), rn(x, W["g_f"]) @ W["W_h"], rtol=1e-11)


def test_forward_is_causal_and_position_dependent():
    m, W = _tiny()
    tok = np.random.default_rng(5).standard_normal((9, 8))
    base = orc.forward(W, m, tok)
    pert = tok.copy(); pert[5] += 1.0
    out = orc.forward(W, m, pert)
    np.testing.assert_array_equal(out[:5], base[:5])          # earlier outputs cannot see token 5
    assert np.all(np.abs(out[5:] - base[5:]).max(axis=1) > 1e-6)
    # a prefix forward equals the first rows of the longer forward
    np.testing.assert_allclose(orc.forward(W, m, tok[:4]), base[:4], rtol=1e-12, atol=1e-14)
    # swapping two earlier tokens changes later outputs (positions matter, through RoPE)
    sw = tok.copy(); sw[[1, 2]] = sw[[2, 1]]
    assert np.abs(orc.forward(W, m, sw)[-1] - base[-1]).max() > 1e-6


def test_routed_ffn_special_cases():
    m, W = _tiny(n_experts=4)
    b = np.random.default_rng(6).standard_normal((5, 32))
    # identical experts: gates sum to one, so routing is invisible
    for e in range(1, 4):
        W[f"l0.e{e}.W_1"] = W["l0.e0.W_1"]; W[f"l0.e{e}.W_2"] = W["l0.e0.W_2"]
    dense = orc.gelu_tanh(b @ W["l0.e0.W_1"]) @ W["l0.e0.W_2"]
    np.testing.assert_allclose(orc.ffn_routed(b, W, 0, m), dense, rtol=1e-12)
    # zero router: all probabilities tie, the lowest two indices win with gate 1/2 each
    m2, W2 = _tiny(n_experts=4, seed=11)
    W2["l1.W_r"][:] = 0
    ex = lambda e: orc.gelu_tanh(b @ W2[f"l1.e{e}.W_1"]) @ W2[f"l1.e{e}.W_2"]
    np.testing.assert_allclose(orc.ffn_routed(b, W2, 1, m2), 0.5 * ex(0) + 0.5 * ex(1), rtol=1e-12)
    # a router that strongly prefers experts 3 then 1 for every token
    W2["l1.W_r"][:] = 0
    bias_dir = b.mean(0) / np.dot(b.mean(0), b.mean(0))
    bpos = b * 0 + b.mean(0)                      # identical tokens so the preference is uniform
    W2["l1.W_r"][:, 3] = 5 * bias_dir; W2["l1.W_r"][:, 1] = 3 * bias_dir
    p3, p1 = math.exp(5), math.exp(3)
    exb = lambda e: orc.gelu_tanh(bpos @ W2[f"l1.e{e}.W_1"]) @ W2[f"l1.e{e}.W_2"]
    ref = (p3 * exb(3) + p1 * exb(1)) / (p3 + p1)
    np.testing.assert_allclose(orc.ffn_routed(bpos, W2, 1, m2), ref, rtol=1e-10)
    # top_k = all experts: the full softmax mixture
    m3 = synth.ModelCfg(2, 32, 2, 64, 4, 4)
    m4, W4 = _tiny(n_experts=4, seed=12)
    pr = orc.softmax(b @ W4["l0.W_r"])
    ex4 = lambda e: orc.gelu_tanh(b @ W4[f"l0.e{e}.W_1"]) @ W4[f"l0.e{e}.W_2"]
    np.testing.assert_allclose(orc.ffn_routed(b, W4, 0, m3), sum(pr[:, [e]] * ex4(e) for e in range(4)), rtol=1e-12)


def test_context_stats_frozen_on_context():
    x = np.random.default_rng(7).standard_normal(64) * 3 + 5
    m, s = orc.context_stats(x)
    assert math.isclose(m, x.mean()) and math.isclose(s, math.sqrt(x.var() + 1e-5))
    # the same through the standard library's population statistics and torch's biased variance
    import statistics
    assert math.isclose(m, statistics.fmean(x.tolist()), rel_tol=1e-12)
    assert math.isclose(s * s - 1e-5, statistics.pvariance(x.tolist()), rel_tol=1e-10)
    assert math.isclose(s * s - 1e-5, float(torch.var(torch.tensor(x, dtype=T64), unbiased=False)), rel_tol=1e-10)
    # a constant context: zero variance, the scale is the floor sqrt(1e-5); a shifted and scaled one follows
    m0, s0 = orc.context_stats(np.full(32, 4.0))
    assert m0 == 4.0 and math.isclose(s0, math.sqrt(1e-5))
    m2, s2 = orc.context_stats(3.0 * x - 7.0)
    assert math.isclose(m2, 3.0 * m - 7.0, rel_tol=1e-12) and math.isclose(s2 ** 2 - 1e-5, 9.0 * (s ** 2 - 1e-5), rel_tol=1e-10)


def _rope_complex(x, pos, base=10000.0):
    """Rotary embedding written a second way: the pair (x_i, x_{i + hd/2}) is the complex number
    x_i + j x_{i + hd/2}, multiplied by exp(j pos base^(-2i/hd)).  x: torch [n, heads, hd]."""
    hd = x.shape[-1]
    half = hd // 2
    z = torch.complex(x[..., :half], x[..., half:])
    theta = torch.tensor(pos, dtype=T64)[:, None] * base ** (-2.0 * torch.arange(half, dtype=T64) / hd)[None, :]
    z = z * torch.polar(torch.ones_like(theta), theta)[:, None, :]
    return torch.cat([z.real, z.imag], dim=-1)


def test_rope_complex_form_is_the_hand_rotation():
    # the helper the composition pin below relies on, against rotation matrices written out by hand
    rng = np.random.default_rng(21)
    hd, pos = 8, [0, 3, 17]
    x = rng.standard_normal((3, 2, hd))
    got = _rope_complex(torch.tensor(x, dtype=T64), pos).numpy()
    for t, p in enumerate(pos):
        for h in range(2):
            for i in range(hd // 2):
                th = p * 10000.0 ** (-2.0 * i / hd)
                a, b = x[t, h, i], x[t, h, i + hd // 2]
                assert math.isclose(got[t, h, i], a * math.cos(th) - b * math.sin(th), rel_tol=1e-12, abs_tol=1e-14)
                assert math.isclose(got[t, h, i + hd // 2], a * math.sin(th) + b * math.cos(th), rel_tol=1e-12, abs_tol=1e-14)


def _forward_from_library_pieces(W, m, tokens):
    """The documented model composed from torch float64 library routines (rms_norm, scaled_dot_product_attention
    with its own causal mask, tanh gelu) and the complex-form rotary embedding; heads are split by
    view(n, heads, hd) of the projection's columns, positions are 0..n-1."""
    t = lambda a: torch.tensor(np.asarray(a), dtype=T64)
    n, D, H = tokens.shape[0], m.d_model, m.n_heads
    hd = D // H
    pos = list(range(n))
    x = t(tokens) @ t(W["W_e"])
    for l in range(m.n_layers):
        a = F.rms_norm(x, (D,), t(W[f"l{l}.g1"]), eps=1e-6)
        q = _rope_complex((a @ t(W[f"l{l}.W_q"])).view(n, H, hd), pos)
        k = _rope_complex((a @ t(W[f"l{l}.W_k"])).view(n, H, hd), pos)
        v = (a @ t(W[f"l{l}.W_v"])).view(n, H, hd)
        o = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], k.permute(1, 0, 2)[None], v.permute(1, 0, 2)[None],
                                           is_causal=True)[0]                      # [H, n, hd], scale 1/sqrt(hd)
        x = x + o.permute(1, 0, 2).reshape(n, D) @ t(W[f"l{l}.W_o"])
        b = F.rms_norm(x, (D,), t(W[f"l{l}.g2"]), eps=1e-6)
        x = x + F.gelu(b @ t(W[f"l{l}.W_1"]), approximate="tanh") @ t(W[f"l{l}.W_2"])
    return (F.rms_norm(x, (D,), t(W["g_f"]), eps=1e-6) @ t(W["W_h"])).numpy()


def test_forward_multi_token_multi_head_matches_library_composition():
    # The whole forward (several layers, heads and tokens at positions > 0) against a composition of library
    # routines: a wrong head split, RoPE on the wrong tensor or with the wrong position, a missing residual, a
    # transposed projection or a mask off by one all fail this.
    for (L, D, H, Fd, P, n, seed) in ((2, 32, 2, 64, 8, 9, 31), (3, 48, 3, 80, 16, 13, 32), (2, 64, 1, 96, 8, 5, 33)):
        m = synth.ModelCfg(L, D, H, Fd)
        W = orc.as_f64(synth.make_weights(m, P, np.random.default_rng(seed), random_gains=True, std=0.3))
        tok = np.random.default_rng(seed + 100).standard_normal((n, P))
        ref = _forward_from_library_pieces(W, m, tok)
        got = orc.forward(W, m, tok)
        assert np.abs(ref).max() > 0.1                       # not a degenerate comparison
        np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-12)
        # (and the comparison can fail: the composition on the reversed token order is far away)
        assert np.abs(got - _forward_from_library_pieces(W, m, tok[::-1].copy())[::-1]).max() > 1e-3


def test_forced_expert_choice_is_the_same_mixture_with_other_experts():
    # the comparison aid of the routed FFN: imposing a token's own choice changes nothing; imposing another set
    # gives that set's mixture with the router's probabilities renormalised over it; rows of -1 stay free;
    # the reported gap is the log ratio between the last expert taken and the first one left out
    m, W = _tiny(n_experts=4)
    b = np.random.default_rng(41).standard_normal((6, 32))
    info = []
    free = orc.ffn_routed(b, W, 0, m, info=info)
    own = np.array([list(i[0]) for i in info])
    np.testing.assert_array_equal(orc.ffn_routed(b, W, 0, m, forced=own), free)
    pr = orc.softmax(b @ W["l0.W_r"])
    ex = lambda e: orc.gelu_tanh(b @ W[f"l0.e{e}.W_1"]) @ W[f"l0.e{e}.W_2"]
    forced = np.full((6, 2), -1)
    forced[2] = (3, 0); forced[4] = (1, 2)
    got = orc.ffn_routed(b, W, 0, m, forced=forced)
    np.testing.assert_array_equal(got[[0, 1, 3, 5]], free[[0, 1, 3, 5]])
    for t, (e0, e1) in ((2, (3, 0)), (4, (1, 2))):
        ref = (pr[t, e0] * ex(e0)[t] + pr[t, e1] * ex(e1)[t]) / (pr[t, e0] + pr[t, e1])
        np.testing.assert_allclose(got[t], ref, rtol=1e-12)
    for t, (order, gap) in enumerate(info):
        srt = np.sort(pr[t])[::-1]
        assert set(order) == set(np.argsort(-pr[t], kind="stable")[:2]) and math.isclose(gap, math.log(srt[1] / srt[2]), rel_tol=1e-12)
    # through the whole forward: the model's own choices imposed = the free forward, and the info has one list per layer
    tok = np.random.default_rng(42).standard_normal((5, 8))
    ri = []
    base = orc.forward(W, m, tok, route_info=ri)
    assert len(ri) == m.n_layers and all(len(x) == 5 for x in ri)
    ids = np.array([[list(i[0]) for i in layer] for layer in ri])
    np.testing.assert_array_equal(orc.forward(W, m, tok, forced_experts=ids), base)
    ids2 = ids.copy(); ids2[1, 3] = [e for e in range(4) if e not in ids[1, 3]][:2]
    out2 = orc.forward(W, m, tok, forced_experts=ids2)
    np.testing.assert_array_equal(out2[:3], base[:3])                 # causal: only tokens from 3 on can move
    assert np.abs(out2[3:] - base[3:]).max() > 1e-6
