"""Layer arithmetic of the oracle (test infrastructure; see package docstring).

The paper (Sec. 3.1, Sec. 5.5) fixes only what the rollout stage must emit; the
layer definitions below are the textbook ones the workload shapes name.  Each
function works in the dtype of its inputs.
"""
from __future__ import annotations

import numpy as np


def rmsnorm(v: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """v / sqrt(mean(v^2) + eps) * g over the last axis."""
    ms = np.mean(v * v, axis=-1, keepdims=True)
    return v / np.sqrt(ms + v.dtype.type(eps)) * g


def rope(u: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary position embedding, half-split pairing.

    u: [..., n_pos, n_heads, hd]; pos: [n_pos] absolute positions.  Pair (i, i+hd/2)
    is rotated by angle pos * theta**(-2i/hd).
    """
    hd = u.shape[-1]
    half = hd // 2
    inv = np.float64(theta) ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv[None, :]          # [n_pos, half]
    c = np.cos(ang).astype(u.dtype)[:, None, :]
    s = np.sin(ang).astype(u.dtype)[:, None, :]
    a, b = u[..., :half], u[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def attention_bruteforce(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """Causal GQA attention by explicit loops (tiny inputs only).

    q: [nq, Hq, hd] for the LAST nq positions of a sequence whose keys/values
    k, v: [nk, Hkv, hd] cover positions 0..nk-1.  Query row r sits at position
    nk - nq + r and sees keys 0..that position.
    """
    nq, hq, hd = q.shape
    nk, hkv, _ = k.shape
    grp = hq // hkv
    out = np.zeros_like(q)
    scale = 1.0 / np.sqrt(hd)
    for r in range(nq):
        p = nk - nq + r
        for h in range(hq):
            kh = h // grp
            s = np.empty(p + 1, dtype=q.dtype)
            for j in range(p + 1):
                acc = q.dtype.type(0)
                for d in range(hd):
                    acc += q[r, h, d] * k[j, kh, d]
                s[j] = acc * q.dtype.type(scale)
            m = s.max()
            e = np.exp(s - m)
            a = e / e.sum()
            for j in range(p + 1):
                out[r, h] += a[j] * v[j, kh]
    return out


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """Causal GQA attention, vectorised per head; same contract as the brute force."""
    nq, hq, hd = q.shape
    nk, hkv, _ = k.shape
    grp = hq // hkv
    scale = q.dtype.type(1.0 / np.sqrt(hd))
    qpos = np.arange(nk - nq, nk)[:, None]
    mask = np.arange(nk)[None, :] > qpos                     # True where key is in the future
    out = np.empty_like(q)
    for h in range(hq):
        kh = h // grp
        s = (q[:, h, :] @ k[:, kh, :].T) * scale             # [nq, nk]
        s = np.where(mask, q.dtype.type(-np.inf), s)
        s = s - s.max(axis=-1, keepdims=True)
        e = np.exp(s)
        a = e / e.sum(axis=-1, keepdims=True)
        out[:, h, :] = a @ v[:, kh, :]
    return out


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1 + np.exp(-z))


def swiglu_ffn(x: np.ndarray, wg: np.ndarray, wu: np.ndarray, wd: np.ndarray) -> np.ndarray:
    """(silu(x Wg^T) * (x Wu^T)) Wd^T with W stored [out, in]."""
    return (silu(x @ wg.T) * (x @ wu.T)) @ wd.T


def moe_gate(r: np.ndarray, top_k: int):
    """Top-k softmax gating of one token's router logits r [E].

    Returns (idx [k] int32 in descending probability, ties to the smaller expert id;
    w [k] = P[idx] / sum(P[idx]) with P = softmax(r); gap = r[k-th] - r[(k+1)-th],
    inf when k == E).  moe_order_gap(r, idx) gives the margin of the ORDER of the chosen ids.
    """
    e = r.shape[0]
    p = np.exp(r - r.max())
    p = p / p.sum()
    # stable sort of -p keeps the smaller index first among equals
    order = np.argsort(-p, kind="stable")
    idx = order[:top_k].astype(np.int32)
    w = p[idx] / p[idx].sum()
    rs = np.sort(r)[::-1]
    gap = float(rs[top_k - 1] - rs[top_k]) if top_k < e else float("inf")
    return idx, w, gap


def moe_order_gap(r: np.ndarray, idx: np.ndarray) -> float:
    """Smallest difference between the logits of consecutive chosen experts (idx in descending order): how far
    the emitted ORDER of the ids is from a swap.  inf for a single id."""
    v = np.asarray(r, dtype=np.float64)[np.asarray(idx)]
    return float(np.min(v[:-1] - v[1:])) if len(v) > 1 else float("inf")


def moe_ffn_bruteforce(x: np.ndarray, w_router: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray,
                       w_down: np.ndarray, top_k: int, forced_idx: np.ndarray = None):
    """Sparse MoE FFN for tokens x [n, d], one token and one expert at a time.

    Returns (y [n, d], idx [n, k] int32 experts used, gap [n], own [n, k] int32 the
    router's own choice, order_gap [n] = moe_order_gap of the router's own choice).  With forced_idx [n, k] the given experts are used (routing
    replay, paper Sec. 5.5) while the mixing weights still come from this model's
    own router probabilities, renormalised over them.
    """
    n = x.shape[0]
    y = np.zeros_like(x)
    idx_out = np.empty((n, top_k), dtype=np.int32)
    own_out = np.empty((n, top_k), dtype=np.int32)
    gaps = np.empty(n, dtype=np.float64)
    ogaps = np.empty(n, dtype=np.float64)
    r_all = x @ w_router.T
    for t in range(n):
        r = r_all[t]
        idx, w, gap = moe_gate(r, top_k)
        own_out[t] = idx
        ogaps[t] = moe_order_gap(r, idx)
        if forced_idx is not None:
            idx = np.asarray(forced_idx[t], dtype=np.int32)
            p = np.exp(r - r.max())
            p = p / p.sum()
            w = p[idx] / p[idx].sum()
        for j in range(top_k):
            e = int(idx[j])
            y[t] += w[j] * swiglu_ffn(x[t:t + 1], w_gate[e], w_up[e], w_down[e])[0]
        idx_out[t] = idx
        gaps[t] = gap
    return y, idx_out, gaps, own_out, ogaps


def moe_ffn(x: np.ndarray, w_router: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray, w_down: np.ndarray,
            top_k: int, forced_idx: np.ndarray = None):
    """Same result as moe_ffn_bruteforce; the expert FFN is evaluated once per
    (slot j, expert) on all tokens that chose it, and every token still adds its
    K expert outputs in slot order j = 0..K-1.
    """
    n = x.shape[0]
    r_all = x @ w_router.T
    idx_out = np.empty((n, top_k), dtype=np.int32)
    own_out = np.empty((n, top_k), dtype=np.int32)
    w_out = np.empty((n, top_k), dtype=x.dtype)
    gaps = np.empty(n, dtype=np.float64)
    ogaps = np.empty(n, dtype=np.float64)
    for t in range(n):
        r = r_all[t]
        idx, w, gaps[t] = moe_gate(r, top_k)
        own_out[t] = idx
        ogaps[t] = moe_order_gap(r, idx)
        if forced_idx is not None:
            idx = np.asarray(forced_idx[t], dtype=np.int32)
            p = np.exp(r - r.max())
            p = p / p.sum()
            w = p[idx] / p[idx].sum()
        idx_out[t], w_out[t] = idx, w
    y = np.zeros_like(x)
    for j in range(top_k):
        for e in np.unique(idx_out[:, j]):
            rows = np.nonzero(idx_out[:, j] == e)[0]
            y[rows] += w_out[rows, j:j + 1] * swiglu_ffn(x[rows], w_gate[e], w_up[e], w_down[e])
    return y, idx_out, gaps, own_out, ogaps


def log_softmax(z: np.ndarray) -> np.ndarray:
    """z - logsumexp(z) over the last axis."""
    m = z.max(axis=-1, keepdims=True)
    return z - (m + np.log(np.exp(z - m).sum(axis=-1, keepdims=True)))
