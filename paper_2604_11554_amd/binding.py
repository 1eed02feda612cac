"""ctypes binding of librelax_rollout.so: argument marshalling only.

Function names and argument order are those of include/relax_rollout.h.  Device
arrays are passed as torch CUDA tensors (or None for NULL); every step of the
path runs in the library's kernels.  Loading fails loudly if the library has not
been built -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librelax_rollout.so")

RLX_OK, RLX_EINVAL, RLX_ENOMEM, RLX_EHIP, RLX_EUNSUPPORTED = 0, -1, -2, -3, -4

EXPORTS = ["rlx_packed_weight_bytes", "rlx_pack_weight", "rlx_pack_gate_up", "rlx_model_create", "rlx_model_destroy", "rlx_model_set_attention_grid", "rlx_model_set_weights", "rlx_model_weight_version", "rlx_kv_pool_bytes", "rlx_workspace_bytes",
           "rlx_kv_copy_blocks", "rollout_prefill_chunk", "rollout_score_chunk", "rollout_decode_step", "rollout_decode_step_static", "rollout_decode_step_shared", "rlx_shared_prefix_bytes", "rlx_shared_prefix_build",
           "rlx_op_linear",
           "rlx_profile_kernel", "rlx_last_error"]

KERNEL_CLASSES = dict(norm=1, qkv=2, rope=3, attn=4, attn_merge=5, oproj=6, gateup=7, down=8, router=9, group=10,
                      lmhead=11, attn_prefix=12)


class RlxError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("relax_rollout error %d: %s" % (code, msg))
        self.code = code


class ModelConfig(C.Structure):
    _fields_ = [("struct_size", C.c_uint32),
                ("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ff", C.c_int32),
                ("n_experts", C.c_int32), ("top_k", C.c_int32), ("d_ff_expert", C.c_int32),
                ("vocab", C.c_int32), ("kv_block_size", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("qk_norm", C.c_int32),
                ("eos_token_id", C.c_int32), ("pad_token_id", C.c_int32), ("activation_split", C.c_int32),
                ("dtype", C.c_int32)]


_PP = C.POINTER(C.c_void_p)


class Weights(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("embed", C.c_void_p), ("lm_head", C.c_void_p),
                ("final_norm", C.c_void_p)] + [(n, _PP) for n in (
                    "attn_norm", "wq", "wk", "wv", "wo", "q_norm", "k_norm", "ffn_norm", "w_gate_up", "w_down",
                    "w_router")]


_lib = None


def lib() -> C.CDLL:
    """The loaded shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: run `python -m paper_2604_11554_amd.build` "
                              "(or __graft_entry__.build()) first" % LIB_PATH)
        l = C.CDLL(LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        l.rlx_last_error.restype = C.c_char_p
        l.rlx_last_error.argtypes = []
        l.rlx_packed_weight_bytes.argtypes = [i32, i32, C.POINTER(sz)]
        l.rlx_pack_weight.argtypes = [vp, vp, i32, i32, i32, vp]
        l.rlx_pack_gate_up.argtypes = [vp, vp, vp, i32, i32, i32, vp]
        l.rlx_model_create.argtypes = [C.POINTER(ModelConfig), C.POINTER(Weights), C.POINTER(vp)]
        l.rlx_model_destroy.argtypes = [vp]
        l.rlx_model_set_attention_grid.argtypes = [vp, i32]
        l.rlx_model_set_weights.argtypes = [vp, C.POINTER(Weights), C.c_uint64]
        l.rlx_model_weight_version.argtypes = [vp, C.POINTER(C.c_uint64)]
        l.rlx_kv_pool_bytes.argtypes = [vp, i64, C.POINTER(sz)]
        l.rlx_workspace_bytes.argtypes = [vp, i32, i32, i32, C.POINTER(sz)]
        l.rlx_kv_copy_blocks.argtypes = [vp, vp, i64, vp, vp, i32, vp]
        l.rollout_prefill_chunk.argtypes = [vp, vp, i64, vp, sz, i32, i32] + [vp] * 5 + [i32] + [vp] * 12
        l.rollout_score_chunk.argtypes = [vp, vp, i64, vp, sz, i32, i32] + [vp] * 5 + [i32] + [vp] * 6
        l.rollout_decode_step.argtypes = [vp, vp, i64, vp, sz, i32, vp, vp, vp, i32] + [vp] * 10
        l.rollout_decode_step_static.argtypes = [vp, vp, i64, i32, vp, vp, vp, i32] + [vp] * 10
        l.rollout_decode_step_shared.argtypes = [vp, vp, i64, vp, sz, i32, vp, vp, vp, i32] + [vp] * 11
        l.rlx_shared_prefix_bytes.argtypes = [vp, i32, C.POINTER(sz)]
        l.rlx_shared_prefix_build.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32), vp, sz, vp]
        l.rlx_op_linear.argtypes = [vp, vp, vp, i32, i32, i32, vp, sz, vp]
        l.rlx_profile_kernel.argtypes = [i32, vp, vp, i32, i32]
        for n in EXPORTS:
            if n != "rlx_last_error":
                getattr(l, n).restype = C.c_int
        _lib = l
    return _lib


def _check(rc: int) -> None:
    if rc != 0:
        raise RlxError(rc, lib().rlx_last_error().decode("utf-8", "replace"))


# the library's 16-bit element formats (RLX_DTYPE_BF16 / RLX_DTYPE_F16) as torch dtypes
RLX_DTYPE_BF16, RLX_DTYPE_F16 = 0, 1
H16 = (torch.bfloat16, torch.float16)


def _ptr(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous CUDA tensor")
    if dtype is not None and t.dtype not in (dtype if isinstance(dtype, tuple) else (dtype,)):
        raise ValueError("expected dtype %s, got %s" % (dtype, t.dtype))
    return t.data_ptr()


def _stream(stream) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def rlx_last_error() -> str:
    return lib().rlx_last_error().decode("utf-8", "replace")


def rlx_packed_weight_bytes(n: int, k: int) -> int:
    out = C.c_size_t()
    _check(lib().rlx_packed_weight_bytes(n, k, C.byref(out)))
    return out.value


def rlx_pack_weight(src: torch.Tensor, dst: torch.Tensor, count: int, n: int, k: int, stream=None) -> None:
    _check(lib().rlx_pack_weight(_ptr(src, H16), _ptr(dst, H16), count, n, k, _stream(stream)))


def pack_matrix(w: torch.Tensor) -> torch.Tensor:
    """Row-major 16-bit [.., n, k] (leading dims = stacked matrices) -> packed streaming layout."""
    n, k = w.shape[-2], w.shape[-1]
    count = int(w.numel() // (n * k))
    per = rlx_packed_weight_bytes(n, k) // 2
    dst = torch.empty(count * per, dtype=w.dtype, device=w.device)
    rlx_pack_weight(w.contiguous(), dst, count, n, k)
    return dst


def rlx_pack_gate_up(gate, up, dst, count: int, f: int, k: int, stream=None) -> None:
    _check(lib().rlx_pack_gate_up(_ptr(gate, H16), _ptr(up, H16), _ptr(dst, H16),
                                  count, f, k, _stream(stream)))


def pack_gate_up(gate: torch.Tensor, up: torch.Tensor) -> torch.Tensor:
    """Row-major 16-bit gate/up [.., f, k] -> interleaved packed [2f, k] matrices."""
    f, k = gate.shape[-2], gate.shape[-1]
    if up.shape != gate.shape:
        raise ValueError("gate and up must have the same shape")
    count = int(gate.numel() // (f * k))
    per = rlx_packed_weight_bytes(2 * f, k) // 2
    dst = torch.empty(count * per, dtype=gate.dtype, device=gate.device)
    rlx_pack_gate_up(gate.contiguous(), up.contiguous(), dst, count, f, k)
    return dst


def rlx_model_create(cfg: ModelConfig, weights: Weights) -> int:
    h = C.c_void_p()
    _check(lib().rlx_model_create(C.byref(cfg), C.byref(weights), C.byref(h)))
    return h.value


def rlx_model_destroy(model: int) -> None:
    _check(lib().rlx_model_destroy(model))


def rlx_model_set_attention_grid(model: int, n_workgroups: int) -> None:
    _check(lib().rlx_model_set_attention_grid(model, n_workgroups))


def rlx_model_set_weights(model: int, weights: Weights, version: int) -> None:
    _check(lib().rlx_model_set_weights(model, C.byref(weights), version))


def rlx_model_weight_version(model: int) -> int:
    out = C.c_uint64()
    _check(lib().rlx_model_weight_version(model, C.byref(out)))
    return out.value


def rlx_kv_pool_bytes(model: int, n_blocks: int) -> int:
    out = C.c_size_t()
    _check(lib().rlx_kv_pool_bytes(model, n_blocks, C.byref(out)))
    return out.value


def rlx_workspace_bytes(model: int, max_seqs: int, max_tokens: int, max_blocks_per_seq: int) -> int:
    out = C.c_size_t()
    _check(lib().rlx_workspace_bytes(model, max_seqs, max_tokens, max_blocks_per_seq, C.byref(out)))
    return out.value


def rlx_kv_copy_blocks(model, kv_pool, n_blocks, src, dst, n, stream=None) -> None:
    _check(lib().rlx_kv_copy_blocks(model, _ptr(kv_pool), n_blocks, _ptr(src, torch.int32), _ptr(dst, torch.int32),
                                    n, _stream(stream)))


def rollout_prefill_chunk(model, kv_pool, n_blocks, workspace, n_seqs, total_tokens, token_ids, input_embeds,
                          cu_seqlens, ctx_lens, block_table, max_blocks_per_seq, sample_last, seeds, temperature,
                          max_ctx_len, forced_tokens, out_tokens, out_logprobs, finished_out, out_sampled=None,
                          out_routing=None, out_logits=None, stream=None) -> None:
    _check(lib().rollout_prefill_chunk(
        model, _ptr(kv_pool), n_blocks, _ptr(workspace), workspace.numel() * workspace.element_size(),
        n_seqs, total_tokens, _ptr(token_ids, torch.int32), _ptr(input_embeds, H16),
        _ptr(cu_seqlens, torch.int32), _ptr(ctx_lens, torch.int32), _ptr(block_table, torch.int32),
        max_blocks_per_seq, _ptr(sample_last, torch.uint8), _ptr(seeds, torch.int64),
        _ptr(temperature, torch.float32), _ptr(max_ctx_len, torch.int32), _ptr(forced_tokens, torch.int32),
        _ptr(out_tokens, torch.int32), _ptr(out_logprobs, torch.float32), _ptr(finished_out, torch.uint8),
        _ptr(out_sampled, torch.int32), _ptr(out_routing, torch.int32), _ptr(out_logits, torch.float32),
        _stream(stream)))


def rollout_score_chunk(model, kv_pool, n_blocks, workspace, n_seqs, total_tokens, token_ids, input_embeds, cu_seqlens,
                        ctx_lens, block_table, max_blocks_per_seq, target_ids, temperature, replay_routing,
                        out_logprobs, out_routing=None, stream=None) -> None:
    _check(lib().rollout_score_chunk(
        model, _ptr(kv_pool), n_blocks, _ptr(workspace), workspace.numel() * workspace.element_size(),
        n_seqs, total_tokens, _ptr(token_ids, torch.int32), _ptr(input_embeds, H16),
        _ptr(cu_seqlens, torch.int32), _ptr(ctx_lens, torch.int32), _ptr(block_table, torch.int32),
        max_blocks_per_seq, _ptr(target_ids, torch.int32), _ptr(temperature, torch.float32),
        _ptr(replay_routing, torch.int32), _ptr(out_logprobs, torch.float32), _ptr(out_routing, torch.int32),
        _stream(stream)))


def rollout_decode_step(model, kv_pool, n_blocks, workspace, n_seqs, tokens_inout, ctx_lens_inout, block_table,
                        max_blocks_per_seq, seeds, temperature, max_ctx_len, finished_inout, forced_tokens,
                        out_logprobs, out_sampled=None, out_routing=None, out_logits=None, stream=None) -> None:
    _check(lib().rollout_decode_step(
        model, _ptr(kv_pool), n_blocks, _ptr(workspace), workspace.numel() * workspace.element_size(), n_seqs,
        _ptr(tokens_inout, torch.int32), _ptr(ctx_lens_inout, torch.int32), _ptr(block_table, torch.int32),
        max_blocks_per_seq, _ptr(seeds, torch.int64), _ptr(temperature, torch.float32),
        _ptr(max_ctx_len, torch.int32), _ptr(finished_inout, torch.uint8), _ptr(forced_tokens, torch.int32),
        _ptr(out_logprobs, torch.float32), _ptr(out_sampled, torch.int32), _ptr(out_routing, torch.int32),
        _ptr(out_logits, torch.float32), _stream(stream)))


RLX_STATIC_WORKSPACE_BYTES = 128 << 20


def rollout_decode_step_static(model, kv_pool, n_blocks, n_seqs, tokens_inout, ctx_lens_inout, block_table,
                               max_blocks_per_seq, seeds, temperature, max_ctx_len, finished_inout, forced_tokens,
                               out_logprobs, out_sampled=None, out_routing=None, out_logits=None, stream=None) -> None:
    """rollout_decode_step on the library's fixed scratch array (no workspace argument, nothing allocated)."""
    _check(lib().rollout_decode_step_static(
        model, _ptr(kv_pool), n_blocks, n_seqs,
        _ptr(tokens_inout, torch.int32), _ptr(ctx_lens_inout, torch.int32), _ptr(block_table, torch.int32),
        max_blocks_per_seq, _ptr(seeds, torch.int64), _ptr(temperature, torch.float32),
        _ptr(max_ctx_len, torch.int32), _ptr(finished_inout, torch.uint8), _ptr(forced_tokens, torch.int32),
        _ptr(out_logprobs, torch.float32), _ptr(out_sampled, torch.int32), _ptr(out_routing, torch.int32),
        _ptr(out_logits, torch.float32), _stream(stream)))


def rollout_decode_step_shared(model, kv_pool, n_blocks, workspace, n_seqs, tokens_inout, ctx_lens_inout, block_table,
                               max_blocks_per_seq, seeds, temperature, max_ctx_len, finished_inout, forced_tokens,
                               out_logprobs, out_sampled=None, out_routing=None, out_logits=None, shared_prefix=None,
                               stream=None) -> None:
    _check(lib().rollout_decode_step_shared(
        model, _ptr(kv_pool), n_blocks, _ptr(workspace), workspace.numel() * workspace.element_size(), n_seqs,
        _ptr(tokens_inout, torch.int32), _ptr(ctx_lens_inout, torch.int32), _ptr(block_table, torch.int32),
        max_blocks_per_seq, _ptr(seeds, torch.int64), _ptr(temperature, torch.float32),
        _ptr(max_ctx_len, torch.int32), _ptr(finished_inout, torch.uint8), _ptr(forced_tokens, torch.int32),
        _ptr(out_logprobs, torch.float32), _ptr(out_sampled, torch.int32), _ptr(out_routing, torch.int32),
        _ptr(out_logits, torch.float32), _ptr(shared_prefix, torch.uint8), _stream(stream)))


def rlx_shared_prefix_bytes(model: int, n_seqs: int) -> int:
    out = C.c_size_t()
    _check(lib().rlx_shared_prefix_bytes(model, n_seqs, C.byref(out)))
    return out.value


def rlx_shared_prefix_build(model: int, leader: Sequence[int], shared_pages: Sequence[int], desc: torch.Tensor,
                            stream=None) -> None:
    """leader / shared_pages: host integers per row; desc: uint8 device tensor of rlx_shared_prefix_bytes."""
    n = len(leader)
    if len(shared_pages) != n:
        raise ValueError("leader and shared_pages must have one entry per row")
    la = (C.c_int32 * n)(*[int(v) for v in leader])
    pa = (C.c_int32 * n)(*[int(v) for v in shared_pages])
    _check(lib().rlx_shared_prefix_build(model, n, la, pa, _ptr(desc, torch.uint8),
                                         desc.numel() * desc.element_size(), _stream(stream)))


def rlx_op_linear(x, w, y, workspace=None, stream=None) -> None:
    """x [n_tokens, k] row-major, w PACKED [n, k] (from pack_matrix), y [n_tokens, n] float32."""
    n_tokens, k = x.shape
    n = y.shape[1]
    # the library cannot see buffer sizes: check them here so a wrong shape can never reach a kernel
    if y.shape[0] != n_tokens or w.numel() * 2 != rlx_packed_weight_bytes(n, k):
        raise ValueError("rlx_op_linear: y must be [n_tokens, n] and w the packed [n, k] matrix")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    need = 2 * 32 * ((n_tokens + 31) // 32) * k + 16 * 4 * n_tokens * n + 1024
    if ws_bytes < need:
        raise ValueError("rlx_op_linear: workspace of %d bytes needed" % need)
    _check(lib().rlx_op_linear(_ptr(x, torch.bfloat16), _ptr(w, torch.bfloat16), _ptr(y, torch.float32), n_tokens, n,
                               k, _ptr(workspace), ws_bytes, _stream(stream)))


class KernelTimer:
    """Brackets every stride-th launch of one kernel class with HIP events (rlx_profile_kernel)."""

    def __init__(self, kernel_class: str, n_events: int, stride: int = 1):
        self.events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                       for _ in range(n_events)]
        # an event gets its handle when first recorded; record once so that cuda_event is valid
        for a, b in self.events:
            a.record()
            b.record()
        torch.cuda.synchronize()
        self._start = (C.c_void_p * n_events)(*[e[0].cuda_event for e in self.events])
        self._stop = (C.c_void_p * n_events)(*[e[1].cuda_event for e in self.events])
        rlx_profile_kernel(KERNEL_CLASSES[kernel_class], self._start, self._stop, n_events, stride)

    def finish(self):
        """Switch the facility off; returns the per-launch durations in milliseconds."""
        n = rlx_profile_kernel(0, None, None, 0, 1)
        torch.cuda.synchronize()
        return [self.events[i][0].elapsed_time(self.events[i][1]) for i in range(n)]


def rlx_profile_kernel(kernel_class: int, start_events, stop_events, n_events: int, stride: int) -> int:
    rc = lib().rlx_profile_kernel(kernel_class, start_events, stop_events, n_events, stride)
    if rc < 0:
        _check(rc)
    return rc


def make_pointer_table(tensors: Sequence[Optional[torch.Tensor]]):
    """Host array of device pointers for one per-layer member of rlx_weights."""
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = _ptr(t, H16)
    return arr
