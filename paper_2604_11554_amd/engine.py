"""Host-side rollout engine over the C ABI: device-resident weights, paged KV pool
with a block allocator, per-sequence state rows, chunked prefill, the decode loop,
prompt-prefix sharing and batch compaction.

Everything numerical happens inside librelax_rollout.so; this module only owns
memory (torch tensors) and integer bookkeeping.  The rollout stage it implements
is the one described in paper Sec. 3.1/3.3 (generation producing responses and
log-probabilities as per-sample fields), Sec. 4.2 (multi-turn sessions whose state
persists across turns) and Sec. 5.5 (expert indices recorded per MoE layer per
token for routing replay).
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as B

PACKED = ("lm_head", "wq", "wk", "wv", "wo", "w_down", "w_router")   # streamed by the skinny GEMM
PER_LAYER = ("attn_norm", "wq", "wk", "wv", "wo", "q_norm", "k_norm", "ffn_norm", "w_gate_up", "w_down",
             "w_router")


def _to_h16_cuda(a, device, dtype) -> torch.Tensor:
    """uint16 bit patterns (numpy) or a tensor -> contiguous CUDA tensor of the model's 16-bit dtype."""
    if isinstance(a, torch.Tensor):
        return a.to(device=device, dtype=dtype).contiguous()
    t = torch.from_numpy(np.ascontiguousarray(a).view(np.int16))
    return t.to(device).view(dtype)


class RolloutModel:
    """Weights on the device plus the library handle.

    cfg: mapping with the fields of rlx_model_config (without struct_size).
    cfg["dtype"] (default bf16) names the 16-bit format of every tensor: binding.RLX_DTYPE_BF16 / RLX_DTYPE_F16.
    tensor(layer, name) returns the row-major tensor (uint16 numpy bits or a torch tensor) under the
    usual names (wq, wk, wv, wo, w_gate, w_up, w_down, ...); layer -1 holds embed / lm_head /
    final_norm.  The streamed matrices are converted to the library's packed layout here.
    """

    def __init__(self, cfg: Dict, tensor: Callable[[int, str], object], device="cuda:0", progress=None):
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.cfg = dict(cfg)
        c = B.ModelConfig()
        c.struct_size = C.sizeof(B.ModelConfig)
        for k, v in self.cfg.items():
            setattr(c, k, v)
        self._c = c
        self.torch_dtype = torch.float16 if c.dtype == B.RLX_DTYPE_F16 else torch.bfloat16
        self._version = 0
        self.tensors, self._tables, self._w = self._upload(tensor, progress)
        self.handle = B.rlx_model_create(c, self._w)

    def _upload(self, tensor: Callable[[int, str], object], progress=None):
        """Device tensors (streamed matrices packed), the per-layer pointer tables and the rlx_weights struct."""
        c, td = self._c, self.torch_dtype
        moe = c.n_experts > 0
        names = [n for n in PER_LAYER if (n not in ("q_norm", "k_norm") or c.qk_norm) and (n != "w_router" or moe)]
        tensors: Dict = {}

        def put(layer, n):
            if n == "w_gate_up":
                t = B.pack_gate_up(_to_h16_cuda(tensor(layer, "w_gate"), self.device, td),
                                   _to_h16_cuda(tensor(layer, "w_up"), self.device, td))
            else:
                t = _to_h16_cuda(tensor(layer, n), self.device, td)
                if n in PACKED:          # row-major copy is dropped once the packed one exists
                    t = B.pack_matrix(t)
            tensors[(layer, n)] = t

        for n in ("embed", "lm_head", "final_norm"):
            put(-1, n)
        for l in range(c.n_layers):
            for n in names:
                put(l, n)
            if progress:
                progress(l)
        torch.cuda.synchronize()
        w = B.Weights()
        w.struct_size = C.sizeof(B.Weights)
        w.embed = tensors[(-1, "embed")].data_ptr()
        w.lm_head = tensors[(-1, "lm_head")].data_ptr()
        w.final_norm = tensors[(-1, "final_norm")].data_ptr()
        tables = {}
        for n in PER_LAYER:
            if n in names:
                tab = B.make_pointer_table([tensors[(l, n)] for l in range(c.n_layers)])
                tables[n] = tab
                setattr(w, n, C.cast(tab, C.POINTER(C.c_void_p)))
        return tensors, tables, w

    @property
    def weight_version(self) -> int:
        """Version tag of the installed weights: the v_r of every token emitted from now on."""
        return self._version

    def update_weights(self, tensor: Callable[[int, str], object], version: int, progress=None) -> None:
        """Weight refresh (paper Sec. 3.2, weight synchronisation to the inference engines): upload and pack a
        new set of tensors beside the current one, wait for every call enqueued so far, then swap the model's
        pointers and drop the old set.  Sequences in flight keep their KV pages (partial rollout)."""
        tensors, tables, w = self._upload(tensor, progress)       # ends with a device synchronisation
        B.rlx_model_set_weights(self.handle, w, version)
        self._version = B.rlx_model_weight_version(self.handle)
        self.tensors, self._tables, self._w = tensors, tables, w   # the old set is released here

    def weight_bytes(self) -> int:
        return sum(t.numel() * 2 for t in self.tensors.values())

    def set_attention_grid(self, n_workgroups: int) -> None:
        """Workgroups of the decode attention kernel (default: two per compute unit)."""
        B.rlx_model_set_attention_grid(self.handle, n_workgroups)

    def close(self):
        if getattr(self, "handle", None):
            B.rlx_model_destroy(self.handle)
            self.handle = None

    def __del__(self):  # pragma: no cover
        try:
            self.close()
        except Exception:
            pass


@dataclass
class StepOutput:
    tokens: torch.Tensor                 # int32 [n]
    logprobs: torch.Tensor               # float32 [n]
    sampled: Optional[torch.Tensor]      # int32 [n] draw before forcing / capping
    routing: Optional[torch.Tensor]      # int32 [tokens, L, K]
    logits: Optional[torch.Tensor]       # float32 [n, V]
    weight_version: int = 0              # v_r: version of the weights that produced these tokens


class RolloutEngine:
    """Rows 0..n-1 of the state tensors are the live batch; a row is one sequence."""

    def may_generate(self, trainer_version: int, max_staleness: int) -> bool:
        """The producer-side staleness rule (paper Sec. 3.3): with v_t the trainer's weight version and v_r the
        version installed here, generation continues only while s = v_t - v_r < max_staleness."""
        return trainer_version - self.m.weight_version < max_staleness

    def __init__(self, model: RolloutModel, n_blocks: int, max_seqs: int, max_chunk_tokens: int,
                 max_blocks_per_seq: int):
        self.m = model
        dev = model.device
        self.n_blocks = int(n_blocks)
        self.max_seqs = max_seqs
        self.max_blocks = max_blocks_per_seq
        self.max_chunk_tokens = max(max_chunk_tokens, max_seqs)
        self.kv_pool = torch.zeros(B.rlx_kv_pool_bytes(model.handle, n_blocks), dtype=torch.uint8, device=dev)
        wb = B.rlx_workspace_bytes(model.handle, max_seqs, self.max_chunk_tokens, max_blocks_per_seq)
        self.workspace = torch.empty(wb, dtype=torch.uint8, device=dev)
        self.free_blocks: List[int] = list(range(n_blocks))
        self.refcount = np.zeros(n_blocks, np.int32)      # sequences listing each page
        self.block_lists: List[List[int]] = []
        i32 = dict(dtype=torch.int32, device=dev)
        self.tokens = torch.zeros(max_seqs, **i32)
        self.ctx_lens = torch.zeros(max_seqs, **i32)
        self.max_ctx = torch.zeros(max_seqs, **i32)
        self.finished = torch.zeros(max_seqs, dtype=torch.uint8, device=dev)
        self.seeds = torch.zeros(max_seqs, dtype=torch.int64, device=dev)
        self.temperature = torch.ones(max_seqs, dtype=torch.float32, device=dev)
        self.block_table = torch.zeros((max_seqs, max_blocks_per_seq), **i32)
        self.n = 0
        self.is_moe = model.cfg["n_experts"] > 0
        # sampling groups: rows that list the same pages for their prompt (fork); decode steps attend to those
        # pages once per subgroup (rollout_decode_step_shared) while share_prefix_attention is set
        self.share_prefix_attention = True
        self.leader: List[int] = []                       # first row of each row's group
        self.shared_pages: List[int] = []                 # leading pages a row shares with its group
        self._sp_desc: Optional[torch.Tensor] = None
        self._sp_dirty = True

    # ---- sequences and pages -------------------------------------------------
    def _set_row(self, i, blocks, seed, temperature, max_ctx, ctx=0, token=0):
        row = torch.zeros(self.max_blocks, dtype=torch.int32)
        row[:len(blocks)] = torch.tensor(blocks, dtype=torch.int32)
        self.block_table[i].copy_(row.to(self.m.device))
        self.seeds[i] = int(np.uint64(seed).astype(np.int64))
        self.temperature[i] = float(temperature)
        self.max_ctx[i] = int(max_ctx)
        self.ctx_lens[i] = int(ctx)
        self.tokens[i] = int(token)
        self.finished[i] = 0

    def _alloc(self, n):
        if n > len(self.free_blocks):
            raise MemoryError("KV pool exhausted: need %d pages, %d free" % (n, len(self.free_blocks)))
        out, self.free_blocks = self.free_blocks[:n], self.free_blocks[n:]
        self.refcount[out] += 1
        return out

    def _release(self, blocks):
        for b in blocks:
            self.refcount[b] -= 1
            if self.refcount[b] == 0:
                self.free_blocks.append(b)

    def add_sequence(self, seed: int, temperature: float = 1.0, max_ctx: int = 1 << 30,
                     reserve_tokens: Optional[int] = None) -> int:
        """New empty sequence; pages for min(max_ctx, reserve_tokens) positions are reserved now
        so the decode loop never has to touch the block table."""
        if self.n >= self.max_seqs:
            raise ValueError("engine is full")
        cap = min(max_ctx, reserve_tokens if reserve_tokens is not None else max_ctx)
        nb = (cap + 15) // 16
        if nb > self.max_blocks:
            raise ValueError("sequence needs %d pages > max_blocks_per_seq %d" % (nb, self.max_blocks))
        i = self.n
        blocks = self._alloc(nb)
        self.block_lists.append(blocks)
        self._set_row(i, blocks, seed, temperature, max_ctx)
        self.leader.append(i)
        self.shared_pages.append(0)
        self._sp_dirty = True
        self.n += 1
        return i

    def fork(self, src: int, seed: int, temperature: float = 1.0, max_ctx: int = 1 << 30,
             reserve_tokens: Optional[int] = None) -> int:
        """New sequence sharing src's full pages (read-only prompt prefix); the partial
        tail page is copied.  Must be called while no work on src is pending elsewhere."""
        if self.n >= self.max_seqs:
            raise ValueError("engine is full")
        ctx = int(self.ctx_lens[src].item())
        cap = min(max_ctx, reserve_tokens if reserve_tokens is not None else max_ctx)
        nb = (cap + 15) // 16
        n_full = ctx // 16
        if nb > self.max_blocks:
            raise ValueError("sequence needs %d pages > max_blocks_per_seq %d" % (nb, self.max_blocks))
        if nb * 16 <= ctx:
            raise ValueError("fork of a %d-token prefix needs room for at least one more position" % ctx)
        own = self._alloc(nb - n_full)
        blocks = self.block_lists[src][:n_full] + own
        self.refcount[self.block_lists[src][:n_full]] += 1
        i = self.n
        self.block_lists.append(blocks)
        self._set_row(i, blocks, seed, temperature, max_ctx, ctx=ctx, token=int(self.tokens[src].item()))
        # the new row joins src's group if that group ends at the previous row (groups are runs of rows)
        root = self.leader[src]
        if n_full > 0 and all(self.leader[r] == root for r in range(root, i)):
            alone = all(self.leader[r] != root for r in range(root + 1, i))
            self.shared_pages[root] = n_full if alone else min(self.shared_pages[root], n_full)
            self.leader.append(root)
            self.shared_pages.append(n_full)
        else:
            self.leader.append(i)
            self.shared_pages.append(0)
        self._sp_dirty = True
        if ctx % 16:
            s = torch.tensor([self.block_lists[src][n_full]], dtype=torch.int32, device=self.m.device)
            d = torch.tensor([own[0]], dtype=torch.int32, device=self.m.device)
            B.rlx_kv_copy_blocks(self.m.handle, self.kv_pool, self.n_blocks, s, d, 1)
        self.n += 1
        return i

    # ---- slots: rows that are refilled in place (continuous refill) --------------
    def open_slots(self, n: int) -> None:
        """Make rows 0..n-1 empty slots: inert rows (finished, no pages) that decode steps skip."""
        if self.n:
            raise ValueError("open_slots needs an empty engine")
        if n > self.max_seqs:
            raise ValueError("more slots than max_seqs")
        self.block_lists = [[] for _ in range(n)]
        self.leader = list(range(n))
        self.shared_pages = [0] * n
        self._sp_dirty = True
        self.block_table[:n].zero_()
        self.ctx_lens[:n].zero_()
        self.finished[:n].fill_(1)
        self.n = n

    def pages_free(self) -> int:
        return len(self.free_blocks)

    def refill_slot(self, row: int, seed: int, temperature: float, max_ctx: int) -> bool:
        """Release the row's pages and start a new empty sequence in it, with pages for max_ctx positions.
        Returns False (row left empty and inert) when the pool cannot hold it now."""
        self.release_slot(row)
        nb = (max_ctx + 15) // 16
        if nb > self.max_blocks:
            raise ValueError("sequence needs %d pages > max_blocks_per_seq %d" % (nb, self.max_blocks))
        if nb > len(self.free_blocks):
            return False
        blocks = self._alloc(nb)
        self.block_lists[row] = blocks
        self._set_row(row, blocks, seed, temperature, max_ctx)
        return True

    def release_slot(self, row: int) -> None:
        self._release(self.block_lists[row])
        self.block_lists[row] = []
        self.finished[row] = 1
        self._leave_group(row)

    def _leave_group(self, row: int) -> None:
        """The row stops sharing pages with its sampling group (its pages are released or replaced): it becomes a
        group of its own, and what is left of the group is cut into the runs before and after it, each led by its
        first row (a group is a run of consecutive rows, see rlx_shared_prefix_build)."""
        root = self.leader[row]
        members = [r for r in range(self.n) if self.leader[r] == root]
        if len(members) > 1:
            after = [r for r in members if r > row]
            for r in after:
                self.leader[r] = after[0]
            for part in ([r for r in members if r < row], after):
                if len(part) == 1:
                    self.shared_pages[part[0]] = 0
        self.leader[row] = row
        self.shared_pages[row] = 0
        self._sp_dirty = True

    # ---- steps ---------------------------------------------------------------
    def prefill(self, rows: Sequence[int], toks: Sequence[np.ndarray], embeds: Sequence[Optional[np.ndarray]] = None,
                sample_last: Sequence[bool] = None, forced: Sequence[int] = None, want_logits=False,
                want_routing=False, want_sampled=False) -> StepOutput:
        """Append one chunk per listed row.  embeds[j]: bit patterns of the model dtype [len(toks[j]), d] aligned with the
        chunk's positions (rows read only where the token id is -1), or None."""
        dev = self.m.device
        n = len(rows)
        lens = [len(t) for t in toks]
        total = int(sum(lens))
        if total > self.max_chunk_tokens or n > self.max_seqs:
            raise ValueError("chunk of %d tokens / %d rows exceeds the workspace" % (total, n))
        idx = torch.tensor(list(rows), dtype=torch.long, device=dev)
        tok = torch.from_numpy(np.concatenate([np.asarray(t, np.int32) for t in toks])).to(dev)
        emb = None
        if embeds is not None and any(e is not None for e in embeds):
            d = self.m.cfg["d_model"]
            full = np.zeros((total, d), np.uint16)
            o = 0
            for e, ln in zip(embeds, lens):
                if e is not None:
                    full[o:o + ln] = e
                o += ln
            emb = torch.from_numpy(full.view(np.int16)).to(dev).view(self.m.torch_dtype)
        cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device=dev)
        ctx = self.ctx_lens[idx].contiguous()
        bt = self.block_table[idx].contiguous()
        sl = torch.tensor([1 if s else 0 for s in (sample_last if sample_last is not None else [True] * n)],
                          dtype=torch.uint8, device=dev)
        fr = None if forced is None else torch.tensor([-1 if f is None else int(f) for f in forced],
                                                      dtype=torch.int32, device=dev)
        out_tok = torch.empty(n, dtype=torch.int32, device=dev)
        out_lp = torch.empty(n, dtype=torch.float32, device=dev)
        fin = torch.empty(n, dtype=torch.uint8, device=dev)
        smp = torch.empty(n, dtype=torch.int32, device=dev) if want_sampled else None
        cfg = self.m.cfg
        routing = (torch.zeros((total, cfg["n_layers"], cfg["top_k"]), dtype=torch.int32, device=dev)
                   if (want_routing and self.is_moe) else None)
        logits = torch.empty((n, cfg["vocab"]), dtype=torch.float32, device=dev) if want_logits else None
        B.rollout_prefill_chunk(self.m.handle, self.kv_pool, self.n_blocks, self.workspace, n, total, tok, emb, cu,
                                ctx, bt, self.max_blocks, sl, self.seeds[idx].contiguous(),
                                self.temperature[idx].contiguous(), self.max_ctx[idx].contiguous(), fr, out_tok,
                                out_lp, fin, smp, routing, logits)
        self.ctx_lens[idx] = ctx + torch.tensor(lens, dtype=torch.int32, device=dev)
        on = sl.bool()
        self.tokens[idx] = torch.where(on, out_tok, self.tokens[idx])
        self.finished[idx] = torch.where(on, fin, self.finished[idx])
        return StepOutput(out_tok, out_lp, smp, routing, logits, self.m.weight_version)

    def score(self, rows: Sequence[int], toks: Sequence[np.ndarray], targets: Sequence[np.ndarray],
              replay_routing: Sequence[Optional[np.ndarray]] = None, embeds: Sequence[Optional[np.ndarray]] = None,
              want_routing=False):
        """Teacher-forced scoring of one chunk per listed row (appends the chunk to the row's cache).
        targets[j][p] is the token whose log-probability is wanted after position p of the chunk (-1: none);
        replay_routing[j]: int32 [len, n_layers, top_k] experts to replay (all rows or none).  Returns
        (log-probs float32 [total], routing used or None), packed in row order."""
        dev = self.m.device
        n = len(rows)
        lens = [len(t) for t in toks]
        total = int(sum(lens))
        if total > self.max_chunk_tokens or n > self.max_seqs:
            raise ValueError("chunk of %d tokens / %d rows exceeds the workspace" % (total, n))
        cfg = self.m.cfg
        idx = torch.tensor(list(rows), dtype=torch.long, device=dev)
        tok = torch.from_numpy(np.concatenate([np.asarray(t, np.int32) for t in toks])).to(dev)
        tgt = torch.from_numpy(np.concatenate([np.asarray(t, np.int32) for t in targets])).to(dev)
        if tgt.numel() != total:
            raise ValueError("targets must align with the chunk tokens")
        emb = None
        if embeds is not None and any(e is not None for e in embeds):
            full = np.zeros((total, cfg["d_model"]), np.uint16)
            o = 0
            for e, ln in zip(embeds, lens):
                if e is not None:
                    full[o:o + ln] = e
                o += ln
            emb = torch.from_numpy(full.view(np.int16)).to(dev).view(self.m.torch_dtype)
        rep = None
        if replay_routing is not None and self.is_moe:
            if any(r is None for r in replay_routing):
                raise ValueError("replay_routing must cover every row of the chunk")
            rep = torch.from_numpy(np.concatenate([np.asarray(r, np.int32) for r in replay_routing])).to(dev).contiguous()
            if tuple(rep.shape) != (total, cfg["n_layers"], cfg["top_k"]):
                raise ValueError("replay_routing must be [tokens, n_layers, top_k]")
        cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device=dev)
        ctx = self.ctx_lens[idx].contiguous()
        bt = self.block_table[idx].contiguous()
        lp = torch.empty(total, dtype=torch.float32, device=dev)
        routing = (torch.zeros((total, cfg["n_layers"], cfg["top_k"]), dtype=torch.int32, device=dev)
                   if (want_routing and self.is_moe) else None)
        B.rollout_score_chunk(self.m.handle, self.kv_pool, self.n_blocks, self.workspace, n, total, tok, emb, cu, ctx,
                              bt, self.max_blocks, tgt, self.temperature[idx].contiguous(), rep, lp, routing)
        self.ctx_lens[idx] = ctx + torch.tensor(lens, dtype=torch.int32, device=dev)
        return lp, routing

    def decode_step(self, forced: Optional[torch.Tensor] = None, out_logprobs: Optional[torch.Tensor] = None,
                    want_logits=False, want_routing=False, want_sampled=False,
                    out_routing: Optional[torch.Tensor] = None) -> StepOutput:
        """One decode step over rows 0..n-1 (enqueue only; no host synchronisation)."""
        dev = self.m.device
        n = self.n
        cfg = self.m.cfg
        lp = out_logprobs if out_logprobs is not None else torch.empty(n, dtype=torch.float32, device=dev)
        smp = torch.empty(n, dtype=torch.int32, device=dev) if want_sampled else None
        routing = out_routing
        if routing is None and want_routing and self.is_moe:
            routing = torch.zeros((n, cfg["n_layers"], cfg["top_k"]), dtype=torch.int32, device=dev)
        logits = torch.empty((n, cfg["vocab"]), dtype=torch.float32, device=dev) if want_logits else None
        B.rollout_decode_step_shared(self.m.handle, self.kv_pool, self.n_blocks, self.workspace, n, self.tokens,
                                     self.ctx_lens, self.block_table, self.max_blocks, self.seeds, self.temperature,
                                     self.max_ctx, self.finished, forced, lp, smp, routing, logits,
                                     self._shared_prefix())
        return StepOutput(self.tokens, lp, smp, routing, logits, self.m.weight_version)

    def _shared_prefix(self) -> Optional[torch.Tensor]:
        """Descriptor of the prompt pages that groups of rows share, rebuilt when rows were added, forked or
        compacted; None when nothing is shared (or share_prefix_attention is off)."""
        if not self.share_prefix_attention:
            return None
        if self._sp_dirty:
            self._sp_dirty = False
            self._sp_desc = None
            n = self.n
            grouped = any(self.leader[i] != i and self.shared_pages[i] >= 2 for i in range(n))
            if grouped:
                desc = torch.empty(B.rlx_shared_prefix_bytes(self.m.handle, n), dtype=torch.uint8,
                                   device=self.m.device)
                B.rlx_shared_prefix_build(self.m.handle, self.leader[:n], self.shared_pages[:n], desc)
                self._sp_desc = desc
        return self._sp_desc

    def compact(self) -> np.ndarray:
        """Drop finished rows (synchronises); returns the old row index of every kept row."""
        fin = self.finished[:self.n].cpu().numpy().astype(bool)
        keep = np.nonzero(~fin)[0]
        for i in np.nonzero(fin)[0]:
            self._release(self.block_lists[i])
        idx = torch.from_numpy(keep).to(self.m.device)
        k = len(keep)
        for t in (self.tokens, self.ctx_lens, self.max_ctx, self.finished, self.seeds, self.temperature,
                  self.block_table):
            t[:k] = t[idx].clone()
        self.block_lists = [self.block_lists[j] for j in keep]
        # groups stay runs of rows; a group whose leader left is led by its first remaining member
        new_leader: Dict[int, int] = {}
        leader = []
        for new, old in enumerate(keep):
            leader.append(new_leader.setdefault(self.leader[old], new))
        self.leader = leader
        self.shared_pages = [self.shared_pages[j] for j in keep]
        self._sp_dirty = True
        self.n = k
        return keep


# ---------------------------------------------------------------------------
# streaming rollout: continuous refill and micro-batch completion events
# ---------------------------------------------------------------------------

@dataclass
class Request:
    prompt: np.ndarray                   # int32 token ids
    seed: int
    temperature: float = 1.0
    max_new_tokens: int = 1 << 20        # the response ends with EOS or, at this length, with a forced EOS


@dataclass
class Completion:
    index: int                           # position of the request in the submitted list
    tokens: np.ndarray                   # int32 response, final EOS included
    logprobs: np.ndarray                 # float32, one per response token
    weight_versions: np.ndarray          # int64 v_r per response token
    routing: Optional[np.ndarray] = None  # int32 [prompt + response - 1, n_layers, top_k] (MoE, if asked for)


class StreamingRollout:
    """Streaming micro-batch scheduling on the rollout side (paper Sec. 3.3, "Streaming data flow"): the request
    list is cut into micro-batches of `micro_batch` consecutive requests; a slot whose sequence has ended is
    refilled with the next pending request instead of letting the batch shrink, and as soon as every member of
    a micro-batch has ended `on_partition(partition_index, completions)` is called, completions in request order.

    The device is polled every `poll_every` decode steps (one host synchronisation per poll); a sequence that ends
    between polls idles as an inert row until the next poll.  `may_admit()` (optional) gates the admission of new
    requests, e.g. the producer-side staleness rule `engine.may_generate(v_t, max_staleness)`; sequences already
    running continue.  The callback may refresh the weights (`model.update_weights`): tokens are tagged with the
    version in force when they were produced.

    `engine` needs: slots via open_slots / refill_slot / release_slot, prefill, decode_step, and the state tensors
    tokens, ctx_lens, finished.
    """

    def __init__(self, engine, requests: Sequence[Request], micro_batch: int = 32, poll_every: int = 8,
                 on_partition: Optional[Callable[[int, List[Completion]], None]] = None,
                 may_admit: Optional[Callable[[], bool]] = None, want_routing: bool = False, slots: Optional[int] = None):
        if micro_batch < 1 or poll_every < 1:
            raise ValueError("micro_batch and poll_every must be positive")
        self.eng = engine
        self.requests = list(requests)
        self.micro_batch = micro_batch
        self.poll_every = poll_every
        self.on_partition = on_partition
        self.may_admit = may_admit
        self.want_routing = want_routing and engine.is_moe
        self.slots = slots if slots is not None else engine.max_seqs
        self.decode_steps = 0
        self.partition_order: List[int] = []

    def run(self) -> List[Completion]:
        eng, reqs = self.eng, self.requests
        n_req = len(reqs)
        done: List[Optional[Completion]] = [None] * n_req
        n_parts = (n_req + self.micro_batch - 1) // self.micro_batch
        left = [min(self.micro_batch, n_req - p * self.micro_batch) for p in range(n_parts)]
        eng.open_slots(self.slots)
        owner = [-1] * self.slots                       # request index running in each slot
        acc: Dict[int, Dict[str, list]] = {}            # per running request: lists of per-poll arrays
        seen = np.zeros(self.slots, np.int64)           # cached length of each slot at the last poll
        nxt = 0
        dev = eng.m.device
        hist_tok = torch.zeros((self.poll_every, self.slots), dtype=torch.int32, device=dev)
        hist_lp = torch.zeros((self.poll_every, self.slots), dtype=torch.float32, device=dev)
        cfg = eng.m.cfg
        hist_rt = (torch.zeros((self.poll_every, self.slots, cfg["n_layers"], cfg["top_k"]), dtype=torch.int32,
                               device=dev) if self.want_routing else None)

        def finish(slot: int) -> None:
            r = owner[slot]
            a = acc.pop(r)
            done[r] = Completion(r, np.concatenate(a["tok"]).astype(np.int32), np.concatenate(a["lp"]).astype(np.float32),
                                 np.concatenate(a["ver"]).astype(np.int64),
                                 np.concatenate(a["rt"], 0) if self.want_routing else None)
            owner[slot] = -1
            eng.release_slot(slot)
            p = r // self.micro_batch
            left[p] -= 1
            if left[p] == 0:
                self.partition_order.append(p)
                if self.on_partition:
                    lo = p * self.micro_batch
                    self.on_partition(p, [done[i] for i in range(lo, min(lo + self.micro_batch, n_req))])

        def admit() -> None:
            nonlocal nxt
            rows, toks = [], []
            budget = eng.max_chunk_tokens
            for slot in range(self.slots):
                if nxt >= n_req or (self.may_admit is not None and not self.may_admit()):
                    break
                if owner[slot] >= 0:
                    continue
                rq = reqs[nxt]
                if len(rq.prompt) > budget:
                    if not rows and len(rq.prompt) > eng.max_chunk_tokens:
                        raise ValueError("prompt of %d tokens exceeds max_chunk_tokens" % len(rq.prompt))
                    break
                if not eng.refill_slot(slot, rq.seed, rq.temperature, len(rq.prompt) + rq.max_new_tokens):
                    break                                # pool full: wait for running sequences to end
                owner[slot] = nxt
                acc[nxt] = dict(tok=[], lp=[], ver=[], rt=[])
                rows.append(slot)
                toks.append(np.asarray(rq.prompt, np.int32))
                budget -= len(rq.prompt)
                nxt += 1
            if not rows:
                return
            out = eng.prefill(rows, toks, want_routing=self.want_routing)
            tok, lp = out.tokens.cpu().numpy(), out.logprobs.cpu().numpy()
            rt = out.routing.cpu().numpy() if self.want_routing else None
            offs = np.concatenate([[0], np.cumsum([len(t) for t in toks])])
            for j, slot in enumerate(rows):
                a = acc[owner[slot]]
                a["tok"].append(tok[j:j + 1]); a["lp"].append(lp[j:j + 1])
                a["ver"].append(np.array([out.weight_version]))
                if self.want_routing:
                    a["rt"].append(rt[offs[j]:offs[j + 1]])
                seen[slot] = len(toks[j])

        def fill() -> None:                              # as many prefill calls as the chunk budget needs
            while True:
                before = nxt
                admit()
                if nxt == before:
                    return

        def reap_first_tokens() -> bool:                 # sequences ended by the token their prefill sampled
            fin = eng.finished[:self.slots].cpu().numpy().astype(bool)
            ended = [slot for slot in range(self.slots) if owner[slot] >= 0 and fin[slot]]
            for slot in ended:
                finish(slot)
            return bool(ended)

        while True:
            fill()
            while reap_first_tokens():
                fill()
            if all(o < 0 for o in owner):
                if nxt >= n_req:
                    break
                if self.may_admit is not None and not self.may_admit():
                    raise RuntimeError("admission is closed and nothing is running: the caller must advance v_r")
                raise MemoryError("the KV pool cannot hold the next request")
            k = self.poll_every
            for s in range(k):
                eng.decode_step(out_logprobs=hist_lp[s], out_routing=None if hist_rt is None else hist_rt[s])
                hist_tok[s].copy_(eng.tokens[:self.slots])
            self.decode_steps += k
            version = eng.m.weight_version
            tok, lp = hist_tok.cpu().numpy(), hist_lp.cpu().numpy()          # synchronises
            rt = hist_rt.cpu().numpy() if self.want_routing else None
            ctx = eng.ctx_lens[:self.slots].cpu().numpy()
            fin = eng.finished[:self.slots].cpu().numpy().astype(bool)
            for slot in range(self.slots):
                r = owner[slot]
                if r < 0:
                    continue
                m = int(ctx[slot] - seen[slot])          # steps in which the row was live: its new tokens
                seen[slot] = ctx[slot]
                a = acc[r]
                a["tok"].append(tok[:m, slot].copy()); a["lp"].append(lp[:m, slot].copy())
                a["ver"].append(np.full(m, version))
                if self.want_routing:
                    a["rt"].append(rt[:m, slot].copy())
                if fin[slot]:
                    finish(slot)
        return [c for c in done if c is not None]
