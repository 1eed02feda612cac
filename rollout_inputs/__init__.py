"""Seeded synthetic inputs for the rollout-decode path: model shapes, 16-bit weight
tensors (bf16, or fp16 for the FP16 precision option) and prompt/length workloads.

This module is shared by the CPU oracle's tests and by the HIP path's tests and
benchmark.  It holds *no* arithmetic of the method itself: it only draws random
numbers, rounds them to 16-bit patterns and lays out integer bookkeeping
(lengths, seeds, group structure).  Both sides consume exactly the same bit
patterns (uint16 arrays), so neither depends on the other's conversion code.

Everything is keyed: a tensor is a pure function of (model_seed, layer, name),
so any tensor can be materialised alone and a large model can be streamed one
layer at a time.

The workloads stand in for the datasets the paper trains on (math prompts with
long chain-of-thought responses, Sec. 5.3; multimodal clips, Sec. 5.2; multi-turn
tool use, Sec. 4.2): only their length mix and structure are mirrored; token ids
are uniform random.
"""
from __future__ import annotations

import dataclasses
import zlib
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

# --------------------------------------------------------------------------
# model shapes
# --------------------------------------------------------------------------


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int            # dense SwiGLU width; 0 for MoE
    n_experts: int       # 0 for dense
    top_k: int           # 0 for dense
    d_ff_expert: int     # 0 for dense
    vocab: int
    qk_norm: bool
    kv_block_size: int = 16
    rms_eps: float = 1e-6
    rope_theta: float = 1e6

    @property
    def is_moe(self) -> bool:
        return self.n_experts > 0

    @property
    def eos_token_id(self) -> int:
        return self.vocab - 1

    @property
    def pad_token_id(self) -> int:
        return self.vocab - 2

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def replace(self, **kw) -> "ModelShape":
        return dataclasses.replace(self, **kw)


TINY_DENSE = ModelShape("tiny_dense", n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64,
                        d_ff=688, n_experts=0, top_k=0, d_ff_expert=0, vocab=2048, qk_norm=False)
# A small MoE model with the structure of the large one (qk-norm, 8-of-E routing,
# GQA group 8); used where the CPU oracle must finish in seconds.
TINY_MOE = ModelShape("tiny_moe", n_layers=3, d_model=256, n_q_heads=8, n_kv_heads=1, head_dim=64,
                      d_ff=0, n_experts=32, top_k=8, d_ff_expert=96, vocab=2048, qk_norm=True)
QWEN3_4B = ModelShape("qwen3_4b_shape", n_layers=36, d_model=2560, n_q_heads=32, n_kv_heads=8, head_dim=128,
                      d_ff=9728, n_experts=0, top_k=0, d_ff_expert=0, vocab=151936, qk_norm=True)
QWEN3_30B_A3B = ModelShape("qwen3_30b_a3b_shape", n_layers=48, d_model=2048, n_q_heads=32, n_kv_heads=4,
                           head_dim=128, d_ff=0, n_experts=128, top_k=8, d_ff_expert=768, vocab=151936,
                           qk_norm=True)

SHAPES: Dict[str, ModelShape] = {s.name: s for s in (TINY_DENSE, TINY_MOE, QWEN3_4B, QWEN3_30B_A3B)}

# --------------------------------------------------------------------------
# bf16 bit patterns
# --------------------------------------------------------------------------


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even); returns uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (b >> np.uint32(16)) & np.uint32(1)
    return ((b + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact upcast of bf16 bit patterns (uint16) to float32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to IEEE fp16 (NumPy's conversion: round-to-nearest-even); uint16 bit patterns."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact upcast of fp16 bit patterns (uint16) to float32."""
    return np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16).astype(np.float32)


FORMATS = {"bf16": (f32_to_bf16_bits, bf16_bits_to_f32), "f16": (f32_to_f16_bits, f16_bits_to_f32)}


def bits_to_f32(bits: np.ndarray, fmt: str) -> np.ndarray:
    return FORMATS[fmt][1](bits)


# --------------------------------------------------------------------------
# weight tensors
# --------------------------------------------------------------------------

GLOBAL_LAYER = -1  # "layer" key of tensors that belong to no layer


def _rng(seed: int, layer: int, name: str) -> np.random.Generator:
    key = [int(seed) & 0xFFFFFFFF, (int(layer) + 1) & 0xFFFFFFFF, zlib.crc32(name.encode())]
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(key)))


def tensor_names(shape: ModelShape, layer: int) -> Dict[str, Tuple[Tuple[int, ...], str]]:
    """name -> (tensor shape, kind) for one layer (or the global tensors).

    All matrices are stored row-major as [out_features, in_features] (y = x @ W.T);
    MoE expert matrices are stacked along a leading expert axis.
    kind: "matrix" ~ N(0, 0.02); "gain" ~ 1 + N(0, 0.02); "router" ~ N(0, 1/d_model).
    """
    s = shape
    if layer == GLOBAL_LAYER:
        return {"embed": ((s.vocab, s.d_model), "matrix"),
                "lm_head": ((s.vocab, s.d_model), "matrix"),
                "final_norm": ((s.d_model,), "gain")}
    t = {"attn_norm": ((s.d_model,), "gain"),
         "wq": ((s.q_dim, s.d_model), "matrix"),
         "wk": ((s.kv_dim, s.d_model), "matrix"),
         "wv": ((s.kv_dim, s.d_model), "matrix"),
         "wo": ((s.d_model, s.q_dim), "matrix"),
         "ffn_norm": ((s.d_model,), "gain")}
    if s.qk_norm:
        t["q_norm"] = ((s.head_dim,), "gain")
        t["k_norm"] = ((s.head_dim,), "gain")
    if s.is_moe:
        t["w_router"] = ((s.n_experts, s.d_model), "router")
        t["w_gate"] = ((s.n_experts, s.d_ff_expert, s.d_model), "matrix")
        t["w_up"] = ((s.n_experts, s.d_ff_expert, s.d_model), "matrix")
        t["w_down"] = ((s.n_experts, s.d_model, s.d_ff_expert), "matrix")
    else:
        t["w_gate"] = ((s.d_ff, s.d_model), "matrix")
        t["w_up"] = ((s.d_ff, s.d_model), "matrix")
        t["w_down"] = ((s.d_model, s.d_ff), "matrix")
    return t


def tensor_bits(shape: ModelShape, model_seed: int, layer: int, name: str, fmt: str = "bf16") -> np.ndarray:
    """Bit patterns (uint16) of one weight tensor: the same float32 draws rounded to `fmt`."""
    to_bits = FORMATS[fmt][0]
    dims, kind = tensor_names(shape, layer)[name]
    g = _rng(model_seed, layer, name)
    n = int(np.prod(dims))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24  # bounded temporaries for the multi-GB tensors
    for a in range(0, n, step):
        z = g.standard_normal(min(step, n - a), dtype=np.float32)
        if kind == "matrix":
            z *= np.float32(0.02)
        elif kind == "gain":
            z *= np.float32(0.02)
            z += np.float32(1.0)
        elif kind == "router":
            z *= np.float32(1.0 / np.sqrt(shape.d_model))
        else:  # pragma: no cover
            raise ValueError(kind)
        out[a:a + z.size] = to_bits(z)
    return out.reshape(dims)


def tensor_bf16(shape: ModelShape, model_seed: int, layer: int, name: str) -> np.ndarray:
    return tensor_bits(shape, model_seed, layer, name, "bf16")


def layer_tensors(shape: ModelShape, model_seed: int, layer: int, fmt: str = "bf16") -> Dict[str, np.ndarray]:
    return {n: tensor_bits(shape, model_seed, layer, n, fmt) for n in tensor_names(shape, layer)}


def layer_tensors_bf16(shape: ModelShape, model_seed: int, layer: int) -> Dict[str, np.ndarray]:
    return layer_tensors(shape, model_seed, layer, "bf16")


# --------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------


@dataclass
class Turn:
    """One later turn of a multi-turn sequence: tool-output ids, then sampled tokens."""
    tool_tokens: np.ndarray   # int32 [n]
    n_decode: int


@dataclass
class Workload:
    """Sequences for one rollout batch.

    prompt_tokens[i] is int32 with -1 where an injected embedding is used instead
    (then prompt_embeds[i][row] is the bf16 bit pattern row for that position, rows
    counted over the -1 positions in order).  group_of[i] is the index of the
    prompt sequence i shares its prompt with (itself if none).
    """
    name: str
    shape: ModelShape
    model_seed: int
    prompt_tokens: List[np.ndarray]
    prompt_embeds: List[Optional[np.ndarray]]
    n_decode: np.ndarray          # int32 [B] tokens to emit in the first turn (incl. the one prefill samples)
    seeds: np.ndarray             # uint64 [B]
    temperature: np.ndarray       # float32 [B]
    group_of: np.ndarray          # int32 [B]
    turns: List[List[Turn]] = field(default_factory=list)

    @property
    def batch(self) -> int:
        return len(self.prompt_tokens)

    @property
    def prompt_lens(self) -> np.ndarray:
        return np.array([len(p) for p in self.prompt_tokens], dtype=np.int32)


def _uniform_ids(g: np.random.Generator, n: int, shape: ModelShape) -> np.ndarray:
    # uniform over the vocabulary without the two reserved ids (pad = V-2, eos = V-1)
    return g.integers(0, shape.vocab - 2, size=n, dtype=np.int64).astype(np.int32)


def workload_tiny(shape: ModelShape = TINY_DENSE, n_decode: int = 32,
                  lens=(16, 32, 48, 64), model_seed: int = 0, prompt_seed: int = 1,
                  seed_base: int = 1000) -> Workload:
    """Four prompts of 16/32/48/64 uniform ids, 32 decoded tokens, temperature 1."""
    g = _rng(prompt_seed, GLOBAL_LAYER, "prompts")
    toks = [_uniform_ids(g, n, shape) for n in lens]
    b = len(lens)
    return Workload("tiny", shape, model_seed, toks, [None] * b, np.full(b, n_decode, np.int32),
                    np.arange(seed_base, seed_base + b, dtype=np.uint64), np.ones(b, np.float32),
                    np.arange(b, dtype=np.int32))


def workload_dense_batch(shape: ModelShape = QWEN3_4B, batch: int = 64, lo: int = 256, hi: int = 1024,
                         n_decode: int = 1024, model_seed: int = 0, prompt_seed: int = 2,
                         seed_base: int = 2000) -> Workload:
    """Batch of independent prompts with lengths uniform on [lo, hi]."""
    g = _rng(prompt_seed, GLOBAL_LAYER, "prompts")
    lens = g.integers(lo, hi + 1, size=batch)
    toks = [_uniform_ids(g, int(n), shape) for n in lens]
    return Workload("dense_batch", shape, model_seed, toks, [None] * batch, np.full(batch, n_decode, np.int32),
                    np.arange(seed_base, seed_base + batch, dtype=np.uint64), np.ones(batch, np.float32),
                    np.arange(batch, dtype=np.int32))


def workload_grouped(shape: ModelShape = QWEN3_4B, n_prompts: int = 32, group: int = 8, lo: int = 512,
                     hi: int = 2048, mean_len: int = 2048, cap: int = 8192, model_seed: int = 0,
                     prompt_seed: int = 3, seed_base: int = 3000, length_seed: int = 30) -> Workload:
    """n_prompts prompts, each shared by `group` sequences; response lengths are
    geometric (support 1,2,...; mean `mean_len`) capped at `cap`."""
    g = _rng(prompt_seed, GLOBAL_LAYER, "prompts")
    lens = g.integers(lo, hi + 1, size=n_prompts)
    base = [_uniform_ids(g, int(n), shape) for n in lens]
    gl = _rng(length_seed, GLOBAL_LAYER, "lengths")
    b = n_prompts * group
    resp = np.minimum(cap, gl.geometric(1.0 / mean_len, size=b)).astype(np.int32)
    toks = [base[i // group] for i in range(b)]
    group_of = np.array([(i // group) * group for i in range(b)], dtype=np.int32)
    return Workload("grouped", shape, model_seed, toks, [None] * b, resp,
                    np.arange(seed_base, seed_base + b, dtype=np.uint64), np.ones(b, np.float32), group_of)


def workload_moe_batch(shape: ModelShape = QWEN3_30B_A3B, batch: int = 128, prompt_len: int = 512,
                       n_decode: int = 2048, model_seed: int = 0, prompt_seed: int = 4,
                       seed_base: int = 4000) -> Workload:
    g = _rng(prompt_seed, GLOBAL_LAYER, "prompts")
    toks = [_uniform_ids(g, prompt_len, shape) for _ in range(batch)]
    return Workload("moe_batch", shape, model_seed, toks, [None] * batch, np.full(batch, n_decode, np.int32),
                    np.arange(seed_base, seed_base + batch, dtype=np.uint64), np.ones(batch, np.float32),
                    np.arange(batch, dtype=np.int32))


def workload_omni_agentic(shape: ModelShape = QWEN3_30B_A3B, batch: int = 64, mm_lo: int = 1024,
                          mm_hi: int = 4096, n_text: int = 256, n_turns: int = 4, tool_len: int = 128,
                          turn_decode: int = 512, model_seed: int = 0, prompt_seed: int = 5,
                          seed_base: int = 5000, embed_seed: int = 50, fmt: str = "bf16") -> Workload:
    """Each sequence: n_mm injected N(0,1) bf16 embedding positions, then n_text ids;
    then n_turns turns of (tool_len prefilled ids -> turn_decode sampled tokens)."""
    g = _rng(prompt_seed, GLOBAL_LAYER, "prompts")
    n_mm = g.integers(mm_lo, mm_hi + 1, size=batch)
    toks, embeds, turns = [], [], []
    for i in range(batch):
        t = np.concatenate([np.full(int(n_mm[i]), -1, np.int32), _uniform_ids(g, n_text, shape)])
        toks.append(t)
        ge = _rng(embed_seed, i, "mm_embeds")
        embeds.append(FORMATS[fmt][0](ge.standard_normal((int(n_mm[i]), shape.d_model), dtype=np.float32)))
        turns.append([Turn(_uniform_ids(g, tool_len, shape), turn_decode) for _ in range(n_turns)])
    # the first response phase belongs to turn 0: prompt -> (tool, decode) x n_turns
    return Workload("omni_agentic", shape, model_seed, toks, embeds, np.zeros(batch, np.int32),
                    np.arange(seed_base, seed_base + batch, dtype=np.uint64), np.ones(batch, np.float32),
                    np.arange(batch, dtype=np.int32), turns)
