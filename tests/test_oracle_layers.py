"""Pins for the oracle's layer arithmetic: closed forms, brute force, invariants
and independent library routines (scipy, torch CPU).  CPU only."""
import numpy as np
import pytest
import scipy.special
import torch

import oracle as O

RNG = np.random.default_rng(123)


@pytest.mark.parametrize("dt", [np.float32, np.float64])
def test_rmsnorm_closed_form(dt):
    v = np.array([[3.0, 4.0, 0.0, 0.0]], dtype=dt)          # mean square = 25/4
    g = np.array([1.0, 2.0, 3.0, 4.0], dtype=dt)
    out = O.rmsnorm(v, g, 0.0)
    np.testing.assert_allclose(out, [[3 / 2.5 * 1, 4 / 2.5 * 2, 0, 0]], rtol=1e-6)
    # eps enters under the root, added to the mean square
    out = O.rmsnorm(v, g, 2.75)                              # 6.25 + 2.75 = 9
    np.testing.assert_allclose(out, [[1.0, 8 / 3, 0, 0]], rtol=1e-6)


def test_rmsnorm_invariants():
    v = RNG.standard_normal((5, 64))
    g = np.ones(64)
    out = O.rmsnorm(v, g, 0.0)
    np.testing.assert_allclose(np.sqrt((out ** 2).mean(-1)), 1.0, rtol=1e-12)
    np.testing.assert_allclose(O.rmsnorm(7.5 * v, g, 0.0), out, rtol=1e-12)
    g2 = RNG.standard_normal(64)
    np.testing.assert_allclose(O.rmsnorm(v, g2, 1e-6), out * g2, rtol=1e-5)


def test_rope_identity_norm_and_relative_position():
    hd = 32
    q = RNG.standard_normal((1, 1, hd))
    k = RNG.standard_normal((1, 1, hd))
    np.testing.assert_array_equal(O.rope(q, np.array([0]), 1e6), q)            # p = 0 is identity
    for m in (1, 17, 4000):
        np.testing.assert_allclose(np.linalg.norm(O.rope(q, np.array([m]), 1e6)), np.linalg.norm(q), rtol=1e-12)
    def dot(m, n):
        return float((O.rope(q, np.array([m]), 1e6) * O.rope(k, np.array([n]), 1e6)).sum())
    np.testing.assert_allclose(dot(10, 3), dot(107, 100), rtol=1e-9)
    np.testing.assert_allclose(dot(5, 5), float((q * k).sum()), rtol=1e-9)
    assert abs(dot(10, 3) - dot(3, 10)) > 1e-6                                  # sign of rotation matters


def test_rope_matches_complex_multiplication():
    hd, theta = 16, 1e6
    u = RNG.standard_normal((3, 2, hd))
    pos = np.array([2, 9, 1234])
    half = hd // 2
    z = u[..., :half] + 1j * u[..., half:]                                     # pair (i, i + hd/2)
    ang = pos[:, None] * theta ** (-2.0 * np.arange(half) / hd)
    zr = z * np.exp(1j * ang)[:, None, :]
    want = np.concatenate([zr.real, zr.imag], -1)
    np.testing.assert_allclose(O.rope(u, pos, theta), want, rtol=1e-10, atol=1e-12)
    # first pair rotates by exactly pos radians, last pair by pos * theta**(-(hd-2)/hd)
    e = np.zeros((1, 1, hd)); e[0, 0, 0] = 1.0
    r = O.rope(e, np.array([1]), theta)
    np.testing.assert_allclose([r[0, 0, 0], r[0, 0, half]], [np.cos(1.0), np.sin(1.0)], rtol=1e-12)


@pytest.mark.parametrize("hq,hkv", [(4, 2), (8, 1), (2, 2)])
def test_attention_vs_bruteforce_and_sdpa(hq, hkv):
    nk, nq, hd = 7, 3, 8
    q = RNG.standard_normal((nq, hq, hd))
    k = RNG.standard_normal((nk, hkv, hd))
    v = RNG.standard_normal((nk, hkv, hd))
    a = O.attention(q, k, v)
    np.testing.assert_allclose(a, O.attention_bruteforce(q, k, v), rtol=1e-10, atol=1e-12)
    # independent routine: torch CPU scaled_dot_product_attention with an explicit mask,
    # GQA written as MHA with repeated KV heads
    grp = hq // hkv
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, grp, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, grp, axis=1)).permute(1, 0, 2)[None]
    mask = torch.from_numpy(np.arange(nk)[None, :] <= (np.arange(nq) + nk - nq)[:, None])
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(a, ref, rtol=1e-9, atol=1e-12)


def test_attention_special_cases():
    hd = 8
    q = RNG.standard_normal((1, 2, hd)); k = RNG.standard_normal((1, 1, hd)); v = RNG.standard_normal((1, 1, hd))
    np.testing.assert_allclose(O.attention(q, k, v), np.repeat(v, 2, axis=1), rtol=1e-12)   # one key: o = v
    # causality: changing a later key/value leaves earlier rows unchanged
    n = 6
    q = RNG.standard_normal((n, 2, hd)); k = RNG.standard_normal((n, 2, hd)); v = RNG.standard_normal((n, 2, hd))
    a = O.attention(q, k, v)
    k2, v2 = k.copy(), v.copy(); k2[4:] += 3.0; v2[4:] -= 2.0
    b = O.attention(q, k2, v2)
    np.testing.assert_array_equal(a[:4], b[:4])
    assert np.abs(a[4:] - b[4:]).max() > 1e-3
    # zero queries: uniform average of the visible values
    a0 = O.attention(np.zeros_like(q), k, v)
    np.testing.assert_allclose(a0[3, 0], v[:4, 0].mean(0), rtol=1e-12)
    # 1/sqrt(hd) scale: with one-hot q and two keys the weights are a closed-form logistic
    q1 = np.zeros((1, 1, hd)); q1[0, 0, 0] = 2.0
    kk = np.zeros((2, 1, hd)); kk[1, 0, 0] = 3.0
    vv = np.zeros((2, 1, hd)); vv[1, 0, 1] = 1.0
    p = 1 / (1 + np.exp(-6.0 / np.sqrt(hd)))
    np.testing.assert_allclose(O.attention(q1, kk, vv)[0, 0, 1], p, rtol=1e-12)


def test_silu_swiglu():
    assert O.silu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(O.silu(np.array([40.0])), [40.0], rtol=1e-12)
    np.testing.assert_allclose(O.silu(np.array([1.0])), [1 / (1 + np.exp(-1.0))], rtol=1e-12)
    np.testing.assert_allclose(O.silu(np.array([-2.0])), [-2 / (1 + np.exp(2.0))], rtol=1e-12)
    x = np.array([[1.0, 2.0]])
    wg = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]])     # [out=3, in=2]
    wu = np.array([[2.0, 0.0], [0.0, -1.0], [0.5, 0.5]])
    wd = np.array([[1.0, 1.0, 1.0], [1.0, -1.0, 0.0]])       # [out=2, in=3]
    s = lambda z: z / (1 + np.exp(-z))
    hid = np.array([s(1.0) * 2.0, s(2.0) * -2.0, s(3.0) * 1.5])
    np.testing.assert_allclose(O.swiglu_ffn(x, wg, wu, wd), [[hid.sum(), hid[0] - hid[1]]], rtol=1e-12)


def test_moe_gate_topk_bruteforce_and_ties():
    for _ in range(20):
        r = RNG.standard_normal(32)
        idx, w, gap = O.moe_gate(r, 8)
        full = sorted(range(32), key=lambda e: (-r[e], e))[:8]
        assert list(idx) == full
        np.testing.assert_allclose(w.sum(), 1.0, rtol=1e-12)
        # softmax -> top-k -> renormalise == softmax over the selected logits
        np.testing.assert_allclose(w, scipy.special.softmax(r[idx]), rtol=1e-10)
        srt = np.sort(r)[::-1]
        np.testing.assert_allclose(gap, srt[7] - srt[8], rtol=1e-12)
    r = np.zeros(16); r[[3, 9, 12]] = 1.0                     # 3 large, 13 tied
    idx, w, gap = O.moe_gate(r, 8)
    assert list(idx) == [3, 9, 12, 0, 1, 2, 4, 5] and gap == 0.0
    idx, w, gap = O.moe_gate(RNG.standard_normal(8), 8)
    assert sorted(idx) == list(range(8)) and gap == float("inf")


def _experts(e, d, f, scale=0.3):
    return (RNG.standard_normal((e, d)), RNG.standard_normal((e, f, d)) * scale,
            RNG.standard_normal((e, f, d)) * scale, RNG.standard_normal((e, d, f)) * scale)


def test_moe_ffn_grouped_equals_bruteforce_and_dense_special_case():
    e, d, f, k, n = 16, 12, 10, 4, 9
    wr, wg, wu, wd = _experts(e, d, f)
    x = RNG.standard_normal((n, d))
    y, idx, gap, own, ogap = O.moe_ffn(x, wr, wg, wu, wd, k)
    yb, idxb, gapb, ownb, ogapb = O.moe_ffn_bruteforce(x, wr, wg, wu, wd, k)
    np.testing.assert_array_equal(own, idx)
    np.testing.assert_array_equal(ownb, idx)
    np.testing.assert_array_equal(idx, idxb)
    np.testing.assert_allclose(y, yb, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(gap, gapb)
    # margin of the emitted order: the smallest step of the chosen logits, by hand from a full sort
    r_all = x @ wr.T
    for t in range(n):
        srt = np.sort(r_all[t])[::-1][:k]
        np.testing.assert_allclose(ogap[t], np.diff(srt).__neg__().min(), rtol=1e-12)
    np.testing.assert_allclose(ogap, ogapb)
    assert O.moe_order_gap(np.array([0.5, 3.0, 1.0]), np.array([1, 2, 0])) == 0.5
    assert O.moe_order_gap(np.array([2.0]), np.array([0])) == float("inf")
    # identical experts: mixture weights sum to one, so the layer equals one dense FFN
    wg1, wu1, wd1 = (np.repeat(a[:1], e, axis=0) for a in (wg, wu, wd))
    y1 = O.moe_ffn(x, wr, wg1, wu1, wd1, k)[0]
    np.testing.assert_allclose(y1, O.swiglu_ffn(x, wg[0], wu[0], wd[0]), rtol=1e-9, atol=1e-12)
    # K = E: the full softmax mixture
    yf = O.moe_ffn(x, wr, wg, wu, wd, e)[0]
    p = scipy.special.softmax(x @ wr.T, axis=-1)
    want = sum(p[:, j:j + 1] * O.swiglu_ffn(x, wg[j], wu[j], wd[j]) for j in range(e))
    np.testing.assert_allclose(yf, want, rtol=1e-9, atol=1e-12)


def test_moe_replay():
    e, d, f, k, n = 16, 12, 10, 4, 6
    wr, wg, wu, wd = _experts(e, d, f)
    x = RNG.standard_normal((n, d))
    y, idx, _, _, _ = O.moe_ffn(x, wr, wg, wu, wd, k)
    y2, idx2, _, _, _ = O.moe_ffn(x, wr, wg, wu, wd, k, forced_idx=idx)       # own indices: idempotent
    np.testing.assert_array_equal(idx, idx2)
    np.testing.assert_allclose(y, y2, rtol=1e-12)
    other = (idx + 1) % e
    y3, idx3, _, own3, _ = O.moe_ffn(x, wr, wg, wu, wd, k, forced_idx=other)
    np.testing.assert_array_equal(idx3, other)
    np.testing.assert_array_equal(own3, idx)                  # the router's own choice is still reported
    assert np.abs(y3 - y).max() > 1e-3
    # replay weights: own probabilities renormalised over the forced set
    p = scipy.special.softmax(x[0] @ wr.T)
    w = p[other[0]] / p[other[0]].sum()
    want = sum(w[j] * O.swiglu_ffn(x[:1], wg[other[0, j]], wu[other[0, j]], wd[other[0, j]])[0] for j in range(k))
    np.testing.assert_allclose(y3[0], want, rtol=1e-9)


def test_log_softmax():
    z = RNG.standard_normal((4, 100)) * 5
    lp = O.log_softmax(z)
    np.testing.assert_allclose(np.exp(lp).sum(-1), 1.0, rtol=1e-12)
    np.testing.assert_allclose(lp, scipy.special.log_softmax(z, axis=-1), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(O.log_softmax(z + 1000.0), lp, atol=1e-9)          # shift invariance, no overflow
    np.testing.assert_allclose(lp[:, 7], z[:, 7] - scipy.special.logsumexp(z, axis=-1), rtol=1e-10)
    z32 = z.astype(np.float32)
    assert abs(np.exp(O.log_softmax(z32).astype(np.float64)).sum(-1) - 1).max() < 1e-5
