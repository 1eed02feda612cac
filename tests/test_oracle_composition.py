"""Pin of the oracle's layer composition (the order in which the pinned primitives are chained).

`forward_full` and `OracleRollout` share the helpers that chain the primitives, so their agreement says nothing
about the chain itself.  Here one decoder stack is written out a second time, position by position, with torch's
CPU routines in float64 (rms_norm, scaled_dot_product_attention, silu, softmax, topk) and a rotary embedding done
as a complex multiplication, in the order the workload shapes name for a Qwen3-style decoder:

    attn-norm -> q/k/v -> per-head q/k norm -> rotary -> causal GQA attention -> Wo + residual
              -> ffn-norm -> SwiGLU FFN (dense) or top-8 softmax-gated experts (MoE) + residual
    final norm -> LM head

and compared with `forward_full` (KV kept in the working dtype, so the algebra is exact up to rounding order).
The mutants at the end plant the plausible mistakes in a copy of the oracle's helper (on the CPU) and check that
this pin would catch each of them.  CPU only.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle as O
import oracle.model as OM
import rollout_inputs as RI

DENSE_QKN = RI.TINY_DENSE.replace(name="tiny_dense_qkn", n_layers=2, vocab=512, qk_norm=True)
DENSE = RI.TINY_DENSE.replace(n_layers=2, vocab=512)
MOE = RI.TINY_MOE.replace(n_layers=2, vocab=512, d_model=128, n_experts=16, d_ff_expert=48)


def _w(model, layer):
    return {n: torch.from_numpy(np.asarray(v, np.float64)) for n, v in model.layer(layer).items()}


def _rotate(u, pos, theta):
    """[n, H, hd] rotated pairwise (i, i + hd/2) by pos * theta^(-2i/hd), as a complex product."""
    hd = u.shape[-1]
    inv = theta ** (-2.0 * torch.arange(hd // 2, dtype=torch.float64) / hd)
    z = torch.complex(u[..., : hd // 2], u[..., hd // 2:]) * torch.polar(torch.ones_like(inv), pos[:, None] * inv)[:, None, :]
    return torch.cat([z.real, z.imag], -1)


def reference_stack(model, tokens):
    """Logits [n, V] and routing [n, L, K] of one sequence, every step written out with torch CPU routines."""
    s = model.shape
    g = _w(model, RI.GLOBAL_LAYER)
    h = g["embed"][torch.from_numpy(np.asarray(tokens, np.int64))]
    n = h.shape[0]
    pos = torch.arange(n, dtype=torch.float64)
    routing = np.zeros((n, s.n_layers, max(s.top_k, 1)), np.int32)
    for l in range(s.n_layers):
        w = _w(model, l)
        x = F.rms_norm(h, (s.d_model,), w["attn_norm"], s.rms_eps)
        q = (x @ w["wq"].T).view(n, s.n_q_heads, s.head_dim)
        k = (x @ w["wk"].T).view(n, s.n_kv_heads, s.head_dim)
        v = (x @ w["wv"].T).view(n, s.n_kv_heads, s.head_dim)
        if s.qk_norm:                      # per head, over head_dim, BEFORE the rotation
            q = F.rms_norm(q, (s.head_dim,), w["q_norm"], s.rms_eps)
            k = F.rms_norm(k, (s.head_dim,), w["k_norm"], s.rms_eps)
        q, k = _rotate(q, pos, s.rope_theta), _rotate(k, pos, s.rope_theta)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None], v.transpose(0, 1)[None],
                                           is_causal=True, enable_gqa=True)[0].transpose(0, 1).reshape(n, s.q_dim)
        h = h + o @ w["wo"].T
        x = F.rms_norm(h, (s.d_model,), w["ffn_norm"], s.rms_eps)
        if not s.is_moe:
            h = h + (F.silu(x @ w["w_gate"].T) * (x @ w["w_up"].T)) @ w["w_down"].T
            continue
        p = torch.softmax(x @ w["w_router"].T, -1)
        top_p, top_i = torch.topk(p, s.top_k, dim=-1)          # descending probability
        routing[:, l, :] = top_i.numpy()
        wgt = top_p / top_p.sum(-1, keepdim=True)
        y = torch.zeros_like(h)
        for t in range(n):
            for j in range(s.top_k):
                e = int(top_i[t, j])
                y[t] += wgt[t, j] * ((F.silu(x[t] @ w["w_gate"][e].T) * (x[t] @ w["w_up"][e].T)) @ w["w_down"][e].T)
        h = h + y
    x = F.rms_norm(h, (s.d_model,), g["final_norm"], s.rms_eps)
    return (x @ g["lm_head"].T).numpy(), routing


def _oracle_logits(shape, tokens, seed=11):
    model = O.OracleModel(shape, seed, dtype=np.float64, kv_bf16=False)
    return model, O.forward_full(model, [tokens])[0]


@pytest.mark.parametrize("shape", [DENSE_QKN, DENSE, MOE], ids=lambda s: s.name)
def test_forward_full_equals_the_stack_written_out_with_library_routines(shape):
    tokens = RI.workload_tiny(shape, lens=(19,), prompt_seed=3).prompt_tokens[0]
    model, got = _oracle_logits(shape, tokens)
    want, routing = reference_stack(model, tokens)
    assert np.abs(want).max() > 0.5                                 # the logits are not degenerate
    np.testing.assert_allclose(got["logits"], want, atol=1e-9, rtol=0)
    if shape.is_moe:
        np.testing.assert_array_equal(got["routing"], routing)


def test_float32_oracle_with_the_bf16_store_stays_near_the_written_out_stack():
    # the configuration the GPU parity tests compare against (fp32, KV rounded at the store) is the same
    # composition: it differs from the exact stack only by the store's rounding, far below the parity bars
    tokens = RI.workload_tiny(DENSE_QKN, lens=(19,), prompt_seed=3).prompt_tokens[0]
    model64, _ = _oracle_logits(DENSE_QKN, tokens)
    want, _ = reference_stack(model64, tokens)
    got = O.forward_full(O.OracleModel(DENSE_QKN, 11), [tokens])[0]["logits"]
    assert np.abs(got - want).max() < 0.02


# ---- mutants: each plants one plausible composition mistake in a copy of the helper that chains the primitives ----

def _qkv_rope_before_norm(shape, w, h, pos, kv_round):
    x = O.rmsnorm(h, w["attn_norm"], shape.rms_eps)
    n = h.shape[0]
    q = O.rope((x @ w["wq"].T).reshape(n, shape.n_q_heads, shape.head_dim), pos, shape.rope_theta)
    k = O.rope((x @ w["wk"].T).reshape(n, shape.n_kv_heads, shape.head_dim), pos, shape.rope_theta)
    v = (x @ w["wv"].T).reshape(n, shape.n_kv_heads, shape.head_dim)
    return O.rmsnorm(q, w["q_norm"], shape.rms_eps), O.rmsnorm(k, w["k_norm"], shape.rms_eps), v


def _qkv_k_not_normalised(shape, w, h, pos, kv_round):
    x = O.rmsnorm(h, w["attn_norm"], shape.rms_eps)
    n = h.shape[0]
    q = O.rmsnorm((x @ w["wq"].T).reshape(n, shape.n_q_heads, shape.head_dim), w["q_norm"], shape.rms_eps)
    k = (x @ w["wk"].T).reshape(n, shape.n_kv_heads, shape.head_dim)
    v = (x @ w["wv"].T).reshape(n, shape.n_kv_heads, shape.head_dim)
    return O.rope(q, pos, shape.rope_theta), O.rope(k, pos, shape.rope_theta), v


def _qkv_wrong_gain(shape, w, h, pos, kv_round):
    return OM_QKV(shape, dict(w, attn_norm=w["ffn_norm"]), h, pos, kv_round)


def _qkv_no_input_norm(shape, w, h, pos, kv_round):
    n = h.shape[0]
    q = O.rmsnorm((h @ w["wq"].T).reshape(n, shape.n_q_heads, shape.head_dim), w["q_norm"], shape.rms_eps)
    k = O.rmsnorm((h @ w["wk"].T).reshape(n, shape.n_kv_heads, shape.head_dim), w["k_norm"], shape.rms_eps)
    v = (h @ w["wv"].T).reshape(n, shape.n_kv_heads, shape.head_dim)
    return O.rope(q, pos, shape.rope_theta), O.rope(k, pos, shape.rope_theta), v


def _ffn_dropped_residual(shape, w, h, forced_idx):
    out = OM_FFN(shape, w, h, forced_idx)
    return (out[0] - h,) + out[1:]


def _ffn_norm_skipped(shape, w, h, forced_idx):
    return OM_FFN(shape, dict(w, ffn_norm=w["attn_norm"]), h, forced_idx)


def _logits_without_final_norm(model, h):
    return h @ model.globals["lm_head"].T


OM_QKV, OM_FFN, OM_LOGITS = OM._qkv, OM._ffn, OM._logits


@pytest.mark.parametrize("attr,mutant", [("_qkv", _qkv_rope_before_norm), ("_qkv", _qkv_k_not_normalised),
                                         ("_qkv", _qkv_wrong_gain), ("_qkv", _qkv_no_input_norm),
                                         ("_ffn", _ffn_dropped_residual), ("_ffn", _ffn_norm_skipped),
                                         ("_logits", _logits_without_final_norm)],
                         ids=lambda m: getattr(m, "__name__", m))
def test_the_pin_catches_planted_composition_mistakes(monkeypatch, attr, mutant):
    tokens = RI.workload_tiny(DENSE_QKN, lens=(19,), prompt_seed=3).prompt_tokens[0]
    model, good = _oracle_logits(DENSE_QKN, tokens)
    want, _ = reference_stack(model, tokens)
    monkeypatch.setattr(OM, attr, mutant)
    bad = O.forward_full(model, [tokens])[0]["logits"]
    assert np.abs(good["logits"] - want).max() < 1e-9
    assert np.abs(bad - want).max() > 1e-3, "the pin does not see this mistake"
