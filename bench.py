#!/usr/bin/env python3
"""Rollout-decode benchmark on one MI355X.

A "step" is one rollout_decode_step over the whole batch (all layers, LM head,
sampling, state update).  Workloads (synthetic, seeded):
  dense_b64  Qwen3-4B-shaped dense policy, 64 sequences, prompts uniform 256..1024,
             1024 decoded tokens each (default)
  moe_b128   Qwen3-30B-A3B-shaped MoE policy, 128 sequences, 512-token prompts,
             2048 decoded tokens, routing indices captured
  grouped_b256  the 4B shape with 32 prompts (uniform 512..2048) x 8 group members that share
             their prompt's pages; the first 256 decode steps are timed (not the metric's
             configuration: it measures decode attention over shared prefixes,
             --no-shared-prefix for the per-sequence path)
Prints ONE JSON line: decode tokens/s, ms/step, the roofline record of the dominant
kernel (timed in situ with HIP events) and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def gpu_random_model(pkg, synthetic, shape, split, seed=0, fmt="bf16"):
    """Random-init weights of the named shape generated on the device (same distributions as
    rollout_inputs: matrices N(0, 0.02), gains 1 + N(0, 0.02), router N(0, 1/d))."""
    import torch
    import rollout_inputs as RI
    gen = torch.Generator(device="cuda:0")

    def tensor(layer, name):
        dims, kind = RI.tensor_names(shape, layer)[name]
        gen.manual_seed((seed * 1000003 + (layer + 1) * 101 + sum(map(ord, name))) & 0x7FFFFFFF)
        t = torch.randn(dims, generator=gen, device="cuda:0", dtype=torch.float32)
        if kind == "matrix":
            t.mul_(0.02)
        elif kind == "gain":
            t.mul_(0.02).add_(1.0)
        else:
            t.mul_(1.0 / np.sqrt(shape.d_model))
        return t.to(torch.float16 if fmt == "f16" else torch.bfloat16)

    return pkg.RolloutModel(synthetic.config_from_shape(shape, split, fmt), tensor)


def kernel_bytes(shape, cls, ctx_sum_plus_b, touched=None):
    """Algorithmic HBM bytes of one launch of a kernel class (bf16 operands read once)."""
    s = shape
    if cls == "attn":
        return ctx_sum_plus_b * s.n_kv_heads * s.head_dim * 2 * 2
    if cls == "qkv":
        return (s.q_dim + 2 * s.kv_dim) * s.d_model * 2
    if cls == "oproj":
        return s.d_model * s.q_dim * 2
    if cls == "gateup":
        return 2 * s.d_ff * s.d_model * 2 if not s.is_moe else 2 * s.d_ff_expert * s.d_model * 2 * touched
    if cls == "down":
        return s.d_ff * s.d_model * 2 if not s.is_moe else s.d_ff_expert * s.d_model * 2 * touched
    if cls == "lmhead":
        return s.vocab * s.d_model * 2
    raise KeyError(cls)


def step_bytes(shape, ctx_sum_plus_b, batch, touched=None):
    """Algorithmic bytes of one decode step: weights streamed once + KV read once + KV appended."""
    s = shape
    w = sum(kernel_bytes(s, c, 0, touched) for c in ("qkv", "oproj", "gateup", "down")) * s.n_layers
    if s.is_moe:
        w += s.n_experts * s.d_model * 2 * s.n_layers
    w += kernel_bytes(s, "lmhead", 0)
    kv_tok = s.n_layers * s.n_kv_heads * s.head_dim * 2 * 2
    return w + kv_tok * ctx_sum_plus_b + kv_tok * batch


def prefill_flops(shape, plen):
    """Useful floating-point operations of prefilling prompts of the given lengths (2 per multiply-add; the
    two-term activations double the MFMA work actually issued, which is not counted)."""
    s = shape
    qdim, kvdim = s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
    per_tok = s.d_model * (qdim + 2 * kvdim) + qdim * s.d_model
    if s.is_moe:
        per_tok += s.d_model * s.n_experts + s.top_k * 3 * s.d_model * s.d_ff_expert
    else:
        per_tok += 3 * s.d_model * s.d_ff
    lin = 2.0 * per_tok * s.n_layers * float(np.sum(plen))
    attn = sum(2.0 * 2 * qdim * (n * (n + 1) / 2.0) for n in plen) * s.n_layers      # causal q.k and p.v
    head = 2.0 * s.vocab * s.d_model * len(plen)                                     # only the sampled rows
    return lin + attn + head


def traffic_record(workload, kernel_class):
    """Measured-over-algorithmic HBM byte ratio of the dominant kernel from the committed counter summary, or
    None when there is none for this workload/kernel or the kernel's sources have changed since it was taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "%s_decode_%s_traffic.txt" % (kernel_class, workload))
    if not os.path.exists(path):
        return None
    rec = {}
    for line in open(path):
        if "=" in line and not line.startswith("#"):
            k, v = line.split("=", 1)
            rec[k.strip()] = v.strip()
    srcs = [os.path.join(ROOT, "paper_2604_11554_amd", "csrc", f.strip()) for f in rec.get("sources", "").split(",") if f.strip()]
    if not srcs or not all(os.path.exists(f) for f in srcs):
        return None
    if rec.get("source_sha256") != hashlib.sha256(b"".join(open(f, "rb").read() for f in srcs)).hexdigest():
        return None
    return float(rec["ratio_measured_over_algorithmic"])


def cpu_baseline(shape, wl, budget_s=25.0, fmt="bf16"):
    """The oracle's decode step timed on the host: 1- and 3-layer slices of the same shape with the
    full batch and start-of-decode context lengths (synthetic KV contents), scaled to all layers."""
    import oracle as O
    import rollout_inputs as RI
    cores = len(os.sched_getaffinity(0))
    nl = 3
    sub = shape.replace(n_layers=nl)
    log("cpu baseline: generating %d-layer slice of %s" % (nl, shape.name))
    tensors = {}
    for l in [RI.GLOBAL_LAYER] + list(range(nl)):
        for n in RI.tensor_names(sub, l):
            tensors[(l, n)] = RI.tensor_bits(sub, 0, l, n, fmt)
    rng = np.random.default_rng(0)
    times = {}
    bs = min(wl.batch, 16)          # bounded sample: the first 16 sequences of the batch
    for k in (1, nl):
        shp = shape.replace(n_layers=k)
        model = O.OracleModel(shp, 0, tensors={key: v for key, v in tensors.items() if key[0] < k}, fmt=fmt)
        model.globals
        for l in range(k):
            model.layer(l)
        nb = int(sum((int(n) + 32) // 16 + 1 for n in wl.prompt_lens[:bs]))
        ro = O.OracleRollout(model, n_blocks=nb)
        for i in range(bs):
            j = ro.add_sequence(int(wl.seeds[i]))
            n = int(wl.prompt_lens[i])
            ro._slots(j, 0, n + 8)
            ro.ctx[j] = n
            ro.last_token[j] = int(wl.prompt_tokens[i][-1])
        ro.kpool[:] = rng.standard_normal(ro.kpool.shape, dtype=np.float32)
        ro.vpool[:] = rng.standard_normal(ro.vpool.shape, dtype=np.float32)
        ids = list(range(bs))
        ro.decode_step(ids)                      # warm the BLAS threads
        t0 = time.perf_counter()
        n_steps = 0
        while n_steps < 2 or (time.perf_counter() - t0 < budget_s / 4 and n_steps < 8):
            ro.decode_step(ids)
            n_steps += 1
        times[k] = (time.perf_counter() - t0) / n_steps
    per_layer = (times[nl] - times[1]) / (nl - 1)
    full = times[1] + per_layer * (shape.n_layers - 1)
    return {"value": bs / full, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": "%d of %d sequences, start-of-decode contexts, synthetic KV contents; 1- and %d-layer "
                      "slices + LM head timed and scaled to %d layers (%.2f s/step)" % (
                          bs, wl.batch, nl, shape.n_layers, full)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="decode steps to time (0 = the whole decode phase)")
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="dense_b64", choices=["dense_b64", "moe_b128", "grouped_b256"])
    ap.add_argument("--no-shared-prefix", action="store_true",
                    help="grouped_b256: read the shared prompt pages once per sequence instead of once per subgroup")
    ap.add_argument("--split", type=int, default=-1,
                    help="activation_split (default: 1 for bf16, two terms per activation; 0 for f16, one term)")
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f16"],
                    help="16-bit format of weights, KV pages and activation terms (f16: the FP16 precision option)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel", default="auto", help="kernel class for the roofline record")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 256 MiB device copy (reference of known size for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2604_11554_amd as pkg
    import rollout_inputs as RI
    from paper_2604_11554_amd import binding as B
    from paper_2604_11554_amd import synthetic

    B.lib()
    dev = "cuda:0"
    grouped = args.workload == "grouped_b256"
    if args.workload == "dense_b64":
        shape, wl = RI.QWEN3_4B, RI.workload_dense_batch()
    elif grouped:
        shape, wl = RI.QWEN3_4B, RI.workload_grouped()
        wl.n_decode[:] = 512                      # the bench times the first steps of the responses, uncapped
        if args.steps <= 0:
            args.steps = 256
    else:
        shape, wl = RI.QWEN3_30B_A3B, RI.workload_moe_batch()
    # the settings the parity tests at this shape pass with
    split = args.split if args.split >= 0 else (1 if args.dtype == "bf16" else 0)
    n_decode = int(wl.n_decode[0])
    bsz = wl.batch
    plen = wl.prompt_lens
    log("workload %s: %s, batch %d, prompts %d..%d, decode %d, %s, activation_split %d" % (
        args.workload, shape.name, bsz, plen.min(), plen.max(), n_decode, args.dtype, split))

    t0 = time.perf_counter()
    model = gpu_random_model(pkg, synthetic, shape, split, fmt=args.dtype)
    torch.cuda.synchronize()
    log("weights on device: %.2f GB in %.1f s" % (model.weight_bytes() / 1e9, time.perf_counter() - t0))

    max_blocks = (int(plen.max()) + n_decode + 15) // 16 + 1
    n_blocks = int(sum((int(n) + n_decode + 15) // 16 for n in plen)) + 8
    chunk_budget = 32768
    leaders = sorted(set(int(g) for g in wl.group_of)) if grouped else []
    if grouped:                                  # prompts are stored once per group
        n_blocks = int(sum((int(plen[g]) + 15) // 16 for g in leaders)) + bsz * ((n_decode + 15) // 16 + 2) + 8
    eng = pkg.RolloutEngine(model, n_blocks=n_blocks, max_seqs=bsz + len(leaders), max_chunk_tokens=chunk_budget,
                            max_blocks_per_seq=max_blocks)
    eng.share_prefix_attention = not args.no_shared_prefix
    if not grouped:
        for i in range(bsz):
            eng.add_sequence(int(wl.seeds[i]), float(wl.temperature[i]), max_ctx=int(plen[i]) + n_decode)

    if args.copy_probe:
        src = torch.ones(64 << 20, dtype=torch.float32, device=dev)      # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- prefill (untimed for the metric; reported) ----
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    shared_tok = np.zeros(bsz, np.int64)         # cached positions of each sequence that prefix tiles serve
    shared_pages_tok = np.zeros(bsz, np.int64)   # cached positions of each sequence that lie in pages its group shares
    pf_lens = plen                               # lengths of the sequences the prefill calls processed
    if grouped:
        # one donor row per prompt takes all but the last prompt token; the members fork from it (sharing its full
        # pages) and prefill the last token themselves; the donors then leave the batch
        donors, rows = {}, []
        for g in leaders:                        # a group is a run of rows: donor, then its members
            donors[g] = eng.add_sequence(0, reserve_tokens=int(plen[g]))
            eng.prefill([donors[g]], [wl.prompt_tokens[g][:-1]], sample_last=[False])
            for m in [k for k in range(bsz) if int(wl.group_of[k]) == g]:
                rows.append((m, eng.fork(donors[g], int(wl.seeds[m]), float(wl.temperature[m]),
                                         max_ctx=int(plen[m]) + n_decode)))
        eng.prefill([r for _, r in rows], [wl.prompt_tokens[m][-1:] for m, _ in rows])
        for g in leaders:
            eng.finished[donors[g]] = 1
        keep = eng.compact()
        assert len(keep) == bsz and eng.n == bsz
        # rows are now in group order; reorder the host-side lengths to match
        pf_lens = np.array([int(plen[g]) - 1 for g in leaders])      # the members' single tokens are not counted
        plen = np.array([plen[m] for m, _ in rows], dtype=plen.dtype)
        shared_pages_tok[:] = [16 * ((int(n) - 1) // 16) for n in plen]
        if eng.share_prefix_attention:
            shared_tok[:] = [32 * ((int(n) - 1) // 32) for n in plen]
    else:
        chunks, i = [], 0
        while i < bsz:
            j, tot = i, 0
            while j < bsz and tot + int(plen[j]) <= chunk_budget:
                tot += int(plen[j])
                j += 1
            chunks.append((i, j))
            i = j
        # untimed warm-up: the first chunk once (first launches load the kernels), then its rows start again
        i, j = chunks[0]
        eng.prefill(list(range(i, j)), wl.prompt_tokens[i:j])
        eng.ctx_lens[i:j] = 0
        eng.finished[i:j] = 0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i, j in chunks:
            eng.prefill(list(range(i, j)), wl.prompt_tokens[i:j])
    torch.cuda.synchronize()
    t_prefill = time.perf_counter() - t0
    log("prefill: %d tokens in %.2f s (%.0f tok/s, %.0f TFLOP/s useful = %.1f%% of the bf16 MFMA peak)" % (
        pf_lens.sum(), t_prefill, pf_lens.sum() / t_prefill, prefill_flops(shape, pf_lens) / t_prefill / 1e12,
        100 * prefill_flops(shape, pf_lens) / t_prefill / 1e12 / 2500.0))

    total_steps = n_decode - 1
    K = args.steps if args.steps > 0 else total_steps - 0
    K = min(K, total_steps)
    W = args.warmup
    lp_buf = torch.zeros((K + W + 64, bsz), dtype=torch.float32, device=dev)
    routing = (torch.zeros((bsz, shape.n_layers, shape.top_k), dtype=torch.int32, device=dev)
               if shape.is_moe else None)

    def save():
        return [t.clone() for t in (eng.tokens, eng.ctx_lens, eng.finished)]

    def restore(st):
        for t, s in zip((eng.tokens, eng.ctx_lens, eng.finished), st):
            t.copy_(s)

    # ---- warmup on a saved state (the KV written here is overwritten by the timed steps) ----
    st = save()
    for s in range(W):
        eng.decode_step(out_logprobs=lp_buf[s], out_routing=routing)
    torch.cuda.synchronize()

    # ---- pick the dominant kernel class: time each class over two steps ----
    classes = ["qkv", "attn", "oproj", "gateup", "down", "lmhead", "norm", "rope", "attn_merge"]
    if shape.is_moe:
        classes += ["router", "group"]
    if shared_tok.any():
        classes += ["attn_prefix"]
    per_class = {}
    for cls in classes:
        kt = B.KernelTimer(cls, 4 * shape.n_layers, 1)
        for s in range(2):
            eng.decode_step(out_logprobs=lp_buf[s], out_routing=routing)
        d = kt.finish()
        per_class[cls] = float(np.sum(d)) / 2.0
    restore(st)
    dom = args.kernel if args.kernel != "auto" else max(per_class, key=per_class.get)
    log("per-step kernel time by class (ms): " + ", ".join("%s %.3f" % kv for kv in sorted(
        per_class.items(), key=lambda kv: -kv[1])) + " -> roofline kernel: " + dom)

    # ---- timed region ----
    stride = 16                                  # every 16th launch of the dominant class is bracketed
    launches_per_step = 1 if dom == "lmhead" else shape.n_layers
    n_ev = K * launches_per_step // stride + 1
    kt = B.KernelTimer(dom, n_ev, stride)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for s in range(K):
        eng.decode_step(out_logprobs=lp_buf[s], out_routing=routing)
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    durs = kt.finish()
    ms_total = ev0.elapsed_time(ev1)
    ms_step = ms_total / K
    toks_per_s = bsz * K / (ms_total / 1e3)

    # ---- byte model ----
    touched = None
    if shape.is_moe:
        e = shape.n_experts
        touched = e * (1.0 - (1.0 - shape.top_k / e) ** bsz)   # expected distinct experts per layer
    ctx0 = plen.astype(np.int64)
    # launch i of the sampled class happened at step (i * stride) // launches_per_step
    ach_bytes = []
    for i in range(len(durs)):
        step = (i * stride) // launches_per_step
        # the per-sequence attention kernel reads what the prefix tiles do not serve
        ach_bytes.append(kernel_bytes(shape, dom, int((ctx0 + step + 1 - shared_tok).sum()), touched)
                         if dom in ("attn", "qkv", "oproj", "gateup", "down", "lmhead") else 0)
    # cost of an empty event pair on this stream (the brackets themselves), subtracted from every sample
    null_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(64)]
    for a_, b_ in null_ev:
        a_.record(); b_.record()
    torch.cuda.synchronize()
    ev_overhead = float(np.median([a_.elapsed_time(b_) for a_, b_ in null_ev]))
    durs = [max(d - ev_overhead, 1e-4) for d in durs]
    kern_ms = float(np.mean(durs)) if durs else float("nan")
    achieved = float(np.sum(ach_bytes)) / (float(np.sum(durs)) * 1e-3) / 1e9 if durs else float("nan")
    ratio = traffic_record(args.workload, dom)
    traffic = None if ratio is None or not durs else ratio * float(np.mean(ach_bytes))
    # a page shared by the eight members of a group counts once (the strict algorithmic minimum; the prefix tiles
    # read it once per subgroup of 16 / (n_q_heads / n_kv_heads) members); with no groups the two figures coincide
    uniq = (ctx0 - shared_pages_tok).sum() + (shared_pages_tok.sum() // 8 if grouped else 0)
    step_b = np.mean([step_bytes(shape, int(uniq + (s + 1) * bsz), bsz, touched) for s in range(K)])
    step_b_logical = np.mean([step_bytes(shape, int((ctx0 + s + 1).sum()), bsz, touched) for s in range(K)])
    step_gbs = step_b / (ms_step * 1e-3) / 1e9
    fin = int(eng.finished[:bsz].sum().item())
    # every decode step this process ran (warmup, per-class timing, timed region) and the cached positions it
    # attended: what per-dispatch hardware counters of a profiled run average over
    offs = list(range(W)) + [W + i for i in range(2 * len(classes))] + list(range(K))
    log("all decode steps run: %d, mean positions attended per step (sum over sequences, new token included) %.2f" % (
        len(offs), float(np.mean([(ctx0 + o + 1).sum() for o in offs]))))
    log("decode: %d steps, %.3f ms/step, %.0f tok/s; step bytes %.2f GB -> %.0f GB/s (%.1f%% of 8 TB/s); "
        "host wall %.2f s; finished rows %d" % (K, ms_step, toks_per_s, step_b / 1e9, step_gbs,
                                                 100 * step_gbs / HBM_PEAK_GBS, wall, fin))

    rec = {
        "metric": "rollout decode tokens/sec on 1 MI355X; % of HBM roofline per step",
        "value": toks_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": "%s: %s, batch %d, prompts uniform %d..%d, %d decoded tokens, paged %s KV block 16, "
                               "temperature 1 Gumbel-max" % (args.workload, shape.name, bsz, plen.min(), plen.max(),
                                                              n_decode, args.dtype),
                   "activation_split": split, "prefill_tokens_per_s": float(pf_lens.sum() / t_prefill)},
        # the prefill chunks that filled the cache before the timed decode steps (MFMA-bound part of the path)
        "prefill": {"tokens": int(pf_lens.sum()), "seconds": t_prefill, "tokens_per_s": float(pf_lens.sum() / t_prefill),
                    "bound": "mfma", "achieved": prefill_flops(shape, pf_lens) / t_prefill / 1e12, "peak": 2500.0,
                    "unit": "TFLOP/s", "frac": prefill_flops(shape, pf_lens) / t_prefill / 1e12 / 2500.0},
        "step_roofline": {"bound": "hbm", "achieved": step_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": step_gbs / HBM_PEAK_GBS, "bytes_per_step": float(step_b),
                          "bytes_per_step_per_sequence_kv": float(step_b_logical),
                          "frac_per_sequence_kv": step_b_logical / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "avg_launch_ms": kern_ms,
                     "bytes_per_launch": float(np.mean(ach_bytes)) if durs else None,
                     "event_pair_overhead_ms": ev_overhead, "launches_timed": len(durs),
                     "per_step_ms_by_class": per_class},
    }
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(shape, wl, fmt=args.dtype)
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
