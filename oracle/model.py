"""Whole-model oracle: teacher-forced full-sequence forward and incremental
paged-KV rollout (test infrastructure; see package docstring).

Two independent formulations of the same function are kept on purpose:
`forward_full` recomputes every position of a sequence with full causal attention;
`OracleRollout` carries a paged key/value store across prefill chunks, decode
steps and turns (per-session state that persists across turns, paper Sec. 4.2).
Their agreement is one of the pins.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np

from rollout_inputs import GLOBAL_LAYER, ModelShape, bits_to_f32, layer_tensors

from . import layers as L
from .philox import sample_gumbel_max


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even to the bf16 grid (8 significand bits), result kept in x's dtype.
    The workloads fix the KV cache as bf16: keys (after the rotary embedding) and values are
    rounded once, when they are stored, and attention consumes the stored values."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32)
    u = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return u.view(np.float32).astype(x.dtype)


def round_to_f16(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even to the IEEE fp16 grid (11 significand bits, subnormals below 2^-14,
    infinities past 65504), result kept in x's dtype: the KV store of the FP16 precision option
    (paper App. "FP16 vs. BF16 precision ablation").  NumPy's float16 conversion is the rounding."""
    with np.errstate(over="ignore"):
        return np.asarray(x).astype(np.float16).astype(np.asarray(x).dtype)


KV_ROUNDING = {"bf16": round_to_bf16, "f16": round_to_f16}


class OracleModel:
    """Weights of one synthetic policy, upcast exactly from 16-bit patterns of format `fmt`
    ("bf16", or "f16" for the FP16 precision option: weights and the KV store are fp16).

    kv_bf16: keys/values are rounded to the model's 16-bit format when stored (what the workloads
    specify); False keeps them in the working dtype (used by pins that need exact algebra).

    Layers are materialised on demand; with cache_layers=False only one layer is
    resident at a time (needed for the 30B-shape model on a small host).
    `tensors` may supply the bit patterns directly: {(layer, name): uint16 array}, or a function
    layer -> {name: uint16 array} that is called when a layer is needed (weights that live elsewhere).
    """

    def __init__(self, shape: ModelShape, model_seed: int = 0, cache_layers: bool = True,
                 dtype=np.float32, tensors: Optional[Dict] = None, kv_bf16: bool = True, fmt: str = "bf16"):
        self.shape = shape
        self.fmt = fmt
        self.kv_round = KV_ROUNDING[fmt] if kv_bf16 else None
        self.model_seed = model_seed
        self.dtype = np.dtype(dtype)
        self.cache_layers = cache_layers
        self._tensors = tensors
        self._cache: Dict[int, Dict[str, np.ndarray]] = {}

    def _load(self, layer: int) -> Dict[str, np.ndarray]:
        if callable(self._tensors):             # tensors(layer) -> {name: bit patterns}: one layer at a time
            bits = self._tensors(layer)
        elif self._tensors is not None:
            bits = {n: b for (l, n), b in self._tensors.items() if l == layer}
        else:
            bits = layer_tensors(self.shape, self.model_seed, layer, self.fmt)
        return {n: bits_to_f32(b, self.fmt).astype(self.dtype, copy=False) for n, b in bits.items()}

    def layer(self, layer: int) -> Dict[str, np.ndarray]:
        if layer in self._cache:
            return self._cache[layer]
        w = self._load(layer)
        if self.cache_layers or layer == GLOBAL_LAYER:
            self._cache[layer] = w
        return w

    @property
    def globals(self) -> Dict[str, np.ndarray]:
        return self.layer(GLOBAL_LAYER)


# --------------------------------------------------------------------------
# pieces shared by the two formulations (pure layer algebra, no caching logic)
# --------------------------------------------------------------------------


def _embed(model: OracleModel, tokens: np.ndarray, embeds: Optional[np.ndarray]) -> np.ndarray:
    """h[p] = embed[token p], or the injected embedding row where token == -1
    (rows of `embeds`, bit patterns of the model's format, are consumed in order)."""
    g = model.globals
    tokens = np.asarray(tokens)
    h = np.empty((len(tokens), model.shape.d_model), dtype=model.dtype)
    inj = tokens < 0
    h[~inj] = g["embed"][tokens[~inj]]
    if inj.any():
        e = bits_to_f32(np.asarray(embeds), model.fmt).astype(model.dtype)
        assert e.shape[0] == int(inj.sum()), "one embedding row per injected position"
        h[inj] = e
    return h


def _qkv(shape: ModelShape, w: Dict[str, np.ndarray], h: np.ndarray, pos: np.ndarray, kv_round):
    x = L.rmsnorm(h, w["attn_norm"], shape.rms_eps)
    n = h.shape[0]
    q = (x @ w["wq"].T).reshape(n, shape.n_q_heads, shape.head_dim)
    k = (x @ w["wk"].T).reshape(n, shape.n_kv_heads, shape.head_dim)
    v = (x @ w["wv"].T).reshape(n, shape.n_kv_heads, shape.head_dim)
    if shape.qk_norm:
        q = L.rmsnorm(q, w["q_norm"], shape.rms_eps)
        k = L.rmsnorm(k, w["k_norm"], shape.rms_eps)
    q = L.rope(q, pos, shape.rope_theta)
    k = L.rope(k, pos, shape.rope_theta)
    if kv_round is not None:
        k, v = kv_round(k), kv_round(v)
    return q, k, v


def _ffn(shape: ModelShape, w: Dict[str, np.ndarray], h: np.ndarray, forced_idx: Optional[np.ndarray]):
    x = L.rmsnorm(h, w["ffn_norm"], shape.rms_eps)
    if shape.is_moe:
        y, idx, gap, own, ogap = L.moe_ffn(x, w["w_router"], w["w_gate"], w["w_up"], w["w_down"], shape.top_k,
                                           forced_idx)
        return h + y, idx, (gap, ogap), own
    return h + L.swiglu_ffn(x, w["w_gate"], w["w_up"], w["w_down"]), None, None, None


def _logits(model: OracleModel, h: np.ndarray) -> np.ndarray:
    g = model.globals
    x = L.rmsnorm(h, g["final_norm"], model.shape.rms_eps)
    return x @ g["lm_head"].T


# --------------------------------------------------------------------------
# formulation 1: full-sequence teacher-forced forward
# --------------------------------------------------------------------------


def forward_full(model: OracleModel, tokens: Sequence[np.ndarray], embeds: Sequence[Optional[np.ndarray]] = None,
                 forced_routing: Sequence[Optional[np.ndarray]] = None,
                 logits_at: Sequence[Optional[np.ndarray]] = None, progress=None) -> List[dict]:
    """Teacher-forced forward of several sequences, layer by layer.

    tokens[i]: int32 [n_i] (-1 = injected embedding).  forced_routing[i]: None or
    int32 [n_i, L, K] expert indices to replay.  logits_at[i]: positions whose
    logits are wanted (None = all).  Returns per sequence a dict with
      logits  [len(logits_at[i]), V]   logits predicting the token AFTER each listed position
      routing [n_i, L, K] int32 (experts used), own_routing (the router's own choice, which
      differs from routing only under replay), gate_gap [n_i, L] (K-th minus (K+1)-th gate logit) and
      order_gap [n_i, L] (smallest gap between consecutive chosen logits)   (MoE only)
    """
    s = model.shape
    nseq = len(tokens)
    embeds = embeds or [None] * nseq
    forced_routing = forced_routing or [None] * nseq
    hs = [_embed(model, tokens[i], embeds[i]) for i in range(nseq)]
    routing = [np.zeros((len(tokens[i]), s.n_layers, max(s.top_k, 1)), np.int32) for i in range(nseq)]
    own = [np.zeros((len(tokens[i]), s.n_layers, max(s.top_k, 1)), np.int32) for i in range(nseq)]
    gaps = [np.full((len(tokens[i]), s.n_layers), np.inf) for i in range(nseq)]
    ogaps = [np.full((len(tokens[i]), s.n_layers), np.inf) for i in range(nseq)]
    for l in range(s.n_layers):
        w = model.layer(l)
        for i in range(nseq):
            h = hs[i]
            n = h.shape[0]
            q, k, v = _qkv(s, w, h, np.arange(n), model.kv_round)
            o = L.attention(q, k, v).reshape(n, s.q_dim)
            h = h + o @ w["wo"].T
            fr = None if forced_routing[i] is None else forced_routing[i][:, l, :]
            h, idx, gap, own_idx = _ffn(s, w, h, fr)
            if idx is not None:
                routing[i][:, l, :] = idx
                own[i][:, l, :] = own_idx
                gaps[i][:, l], ogaps[i][:, l] = gap
            hs[i] = h
        if progress:
            progress(l)
    out = []
    for i in range(nseq):
        at = np.arange(len(tokens[i])) if logits_at is None or logits_at[i] is None else np.asarray(logits_at[i])
        res = {"logits": _logits(model, hs[i][at]), "positions": at}
        if s.is_moe:
            res["routing"], res["gate_gap"], res["own_routing"] = routing[i], gaps[i], own[i]
            res["order_gap"] = ogaps[i]
        out.append(res)
    return out


# --------------------------------------------------------------------------
# formulation 2: incremental rollout over a paged KV store
# --------------------------------------------------------------------------


class OracleRollout:
    """Sequences with a paged key/value store of the oracle's own.

    Keys/values live in per-layer pools [n_blocks, block, Hkv, hd] (working dtype);
    each sequence owns a list of physical block ids.  `fork` lets a sequence share
    another's full blocks (shared prompt prefix) and copies the partial tail block.
    Blocks are handed out by `alloc_order` so tests can permute physical placement.
    """

    def __init__(self, model: OracleModel, n_blocks: int, block_size: Optional[int] = None,
                 alloc_order: Optional[Sequence[int]] = None):
        self.model = model
        s = model.shape
        self.bs = block_size or s.kv_block_size
        self.n_blocks = n_blocks
        shp = (s.n_layers, n_blocks, self.bs, s.n_kv_heads, s.head_dim)
        self.kpool = np.zeros(shp, model.dtype)
        self.vpool = np.zeros(shp, model.dtype)
        self.free = list(alloc_order) if alloc_order is not None else list(range(n_blocks))
        self.blocks: List[List[int]] = []
        self.ctx: List[int] = []
        self.seeds: List[int] = []
        self.temperature: List[float] = []
        self.max_ctx: List[int] = []
        self.finished: List[bool] = []
        self.last_token: List[int] = []
        self.weight_version = 0

    def set_model(self, model: OracleModel, version: int) -> None:
        """Weight refresh between steps (paper Sec. 3.2, weight synchronisation to the inference engines;
        Sec. 3.3, the rollout-side weight version v_r): later calls use `model`; the stored keys and values
        of sequences in flight are kept, so such a sequence attends to entries of the previous weights."""
        a, b = self.model.shape, model.shape
        assert (a.n_layers, a.n_kv_heads, a.head_dim, a.vocab) == (b.n_layers, b.n_kv_heads, b.head_dim, b.vocab)
        assert model.dtype == self.model.dtype
        self.model = model
        self.weight_version = int(version)

    # ---- sequence bookkeeping -------------------------------------------
    def add_sequence(self, seed: int, temperature: float = 1.0, max_ctx: int = 1 << 30) -> int:
        self.blocks.append([])
        self.ctx.append(0)
        self.seeds.append(int(seed))
        self.temperature.append(float(temperature))
        self.max_ctx.append(int(max_ctx))
        self.finished.append(False)
        self.last_token.append(-1)
        return len(self.ctx) - 1

    def fork(self, src: int, seed: int, temperature: float = 1.0, max_ctx: int = 1 << 30) -> int:
        i = self.add_sequence(seed, temperature, max_ctx)
        n_full = self.ctx[src] // self.bs
        self.blocks[i] = list(self.blocks[src][:n_full])
        if self.ctx[src] % self.bs:
            nb = self.free.pop(0)
            ob = self.blocks[src][n_full]
            self.kpool[:, nb] = self.kpool[:, ob]
            self.vpool[:, nb] = self.vpool[:, ob]
            self.blocks[i].append(nb)
        self.ctx[i] = self.ctx[src]
        self.last_token[i] = self.last_token[src]
        return i

    def set_cache(self, i: int, keys: np.ndarray, values: np.ndarray, last_token: int) -> None:
        """Give sequence i a cache of given contents instead of computing it: keys, values [L, n, Hkv, hd] (stored
        through the model's KV rounding) become its positions 0..n-1 and `last_token` the token its next decode
        step consumes.  For timing the decode step at a chosen context length without paying the prefill."""
        n = keys.shape[1]
        assert self.ctx[i] == 0 and keys.shape == values.shape
        blk, slot = self._slots(i, 0, n)
        rnd = self.model.kv_round or (lambda a: a)
        self.kpool[:, blk, slot] = rnd(np.asarray(keys, self.model.dtype))
        self.vpool[:, blk, slot] = rnd(np.asarray(values, self.model.dtype))
        self.ctx[i] = n
        self.last_token[i] = int(last_token)

    def _slots(self, i: int, p0: int, n: int):
        """(block id, slot) for positions p0..p0+n-1 of sequence i, allocating blocks."""
        need = (p0 + n + self.bs - 1) // self.bs
        while len(self.blocks[i]) < need:
            self.blocks[i].append(self.free.pop(0))
        pos = np.arange(p0, p0 + n)
        return np.asarray(self.blocks[i])[pos // self.bs], pos % self.bs

    def _gather(self, l: int, i: int, n: int):
        pos = np.arange(n)
        b = np.asarray(self.blocks[i])[pos // self.bs]
        return self.kpool[l, b, pos % self.bs], self.vpool[l, b, pos % self.bs]

    # ---- the forward over new positions ----------------------------------
    def _advance(self, seq_ids: Sequence[int], toks: Sequence[np.ndarray], embeds: Sequence[Optional[np.ndarray]],
                 forced_routing: Sequence[Optional[np.ndarray]] = None):
        """Append the given new tokens of each listed sequence; returns the final hidden
        state of every new position and the routing taken."""
        m, s = self.model, self.model.shape
        forced_routing = forced_routing or [None] * len(seq_ids)
        hs = [_embed(m, toks[j], embeds[j]) for j in range(len(seq_ids))]
        routing = [np.zeros((len(toks[j]), s.n_layers, max(s.top_k, 1)), np.int32) for j in range(len(seq_ids))]
        own = [np.zeros((len(toks[j]), s.n_layers, max(s.top_k, 1)), np.int32) for j in range(len(seq_ids))]
        gaps = [np.full((len(toks[j]), s.n_layers), np.inf) for j in range(len(seq_ids))]
        ogaps = [np.full((len(toks[j]), s.n_layers), np.inf) for j in range(len(seq_ids))]
        for l in range(s.n_layers):
            w = m.layer(l)
            for j, i in enumerate(seq_ids):
                h = hs[j]
                n, p0 = h.shape[0], self.ctx[i]
                q, k, v = _qkv(s, w, h, np.arange(p0, p0 + n), m.kv_round)
                blk, slot = self._slots(i, p0, n)
                self.kpool[l, blk, slot] = k
                self.vpool[l, blk, slot] = v
                kk, vv = self._gather(l, i, p0 + n)
                o = L.attention(q, kk, vv).reshape(n, s.q_dim)
                h = h + o @ w["wo"].T
                fr = None if forced_routing[j] is None else forced_routing[j][:, l, :]
                h, idx, gap, own_idx = _ffn(s, w, h, fr)
                if idx is not None:
                    routing[j][:, l, :] = idx
                    own[j][:, l, :] = own_idx
                    gaps[j][:, l], ogaps[j][:, l] = gap
                hs[j] = h
        for j, i in enumerate(seq_ids):
            self.ctx[i] += hs[j].shape[0]
        self._order_gaps = ogaps          # of the call just made, read by the two public steps
        return hs, routing, gaps, own

    def _emit(self, i: int, z: np.ndarray, forced: Optional[int]):
        """Sample the token for position ctx[i] from logits z; apply forcing, the
        length cap (forced EOS) and the finish rule.  Returns (token, logprob, sampled)."""
        s = self.model.shape
        t = self.temperature[i]
        pos = self.ctx[i]                       # position the new token will occupy
        sampled = sample_gumbel_max(z, t, self.seeds[i], pos)
        tok = sampled if forced is None or forced < 0 else int(forced)
        if pos >= self.max_ctx[i] - 1:          # last position this sequence may fill
            tok = s.eos_token_id
        logp = L.log_softmax(z / z.dtype.type(t if t > 0 else 1.0))
        if tok == s.eos_token_id:
            self.finished[i] = True
        self.last_token[i] = tok
        return tok, float(logp[tok]), sampled

    # ---- public steps -----------------------------------------------------
    def prefill_chunk(self, seq_ids: Sequence[int], toks: Sequence[np.ndarray],
                      embeds: Sequence[Optional[np.ndarray]] = None, sample_last: Sequence[bool] = None,
                      forced_tokens: Sequence[Optional[int]] = None, forced_routing=None,
                      want_logits: bool = False) -> dict:
        """Append a chunk of known tokens per sequence; where sample_last is set, emit the
        next token from the chunk's last position."""
        n = len(seq_ids)
        embeds = embeds or [None] * n
        sample_last = sample_last if sample_last is not None else [True] * n
        forced_tokens = forced_tokens if forced_tokens is not None else [None] * n
        hs, routing, gaps, own = self._advance(seq_ids, toks, embeds, forced_routing)
        out = {"tokens": [], "logprobs": [], "sampled": [], "routing": routing, "gate_gap": gaps,
               "own_routing": own, "order_gap": self._order_gaps, "logits": []}
        for j, i in enumerate(seq_ids):
            if sample_last[j]:
                z = _logits(self.model, hs[j][-1:])[0]
                tok, lp, smp = self._emit(i, z, forced_tokens[j])
                out["tokens"].append(tok)
                out["logprobs"].append(lp)
                out["sampled"].append(smp)
                out["logits"].append(z if want_logits else None)
            else:
                out["tokens"].append(self.model.shape.pad_token_id)
                out["logprobs"].append(0.0)
                out["sampled"].append(-1)
                out["logits"].append(None)
        return out

    def decode_step(self, seq_ids: Sequence[int], forced_tokens: Sequence[Optional[int]] = None,
                    forced_routing=None, want_logits: bool = False) -> dict:
        """One decode step for the listed sequences: each live one consumes its last
        emitted token and emits the next; finished ones are inert (pad, 0.0)."""
        s = self.model.shape
        n = len(seq_ids)
        forced_tokens = forced_tokens if forced_tokens is not None else [None] * n
        live = [j for j, i in enumerate(seq_ids) if not self.finished[i]]
        ids = [seq_ids[j] for j in live]
        toks = [np.array([self.last_token[i]], np.int32) for i in ids]
        fr = None if forced_routing is None else [forced_routing[j] for j in live]
        hs, routing, gaps, own = self._advance(ids, toks, [None] * len(ids), fr)
        out = {"tokens": [s.pad_token_id] * n, "logprobs": [0.0] * n, "sampled": [-1] * n,
               "routing": [None] * n, "gate_gap": [None] * n, "own_routing": [None] * n, "order_gap": [None] * n,
               "logits": [None] * n}
        for jj, j in enumerate(live):
            i = seq_ids[j]
            z = _logits(self.model, hs[jj][-1:])[0]
            tok, lp, smp = self._emit(i, z, forced_tokens[j])
            out["tokens"][j], out["logprobs"][j], out["sampled"][j] = tok, lp, smp
            out["routing"][j], out["gate_gap"][j], out["own_routing"][j] = routing[jj], gaps[jj], own[jj]
            out["order_gap"][j] = self._order_gaps[jj]
            out["logits"][j] = z if want_logits else None
        return out
