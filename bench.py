#!/usr/bin/env python3
"""Rollout-decode benchmark on one MI355X.

A "step" is one rollout_decode_step over the whole batch (all layers, LM head,
sampling, state update).  Workloads (synthetic, seeded):
  moe_b128   Qwen3-30B-A3B-shaped MoE policy, 128 sequences, 512-token prompts,
             2048 decoded tokens, routing indices captured (the largest single-GPU
             configuration: the headline of the default run)
  dense_b64  Qwen3-4B-shaped dense policy, 64 sequences, prompts uniform 256..1024,
             1024 decoded tokens each (carried under "also" in the default run)
  grouped_b256  the 4B shape with 32 prompts (uniform 512..2048) x 8 group members that share
             their prompt's pages.  Without --full the first 256 decode steps are timed with
             the response lengths uncapped; with --full the responses have geometric lengths
             (mean 2048, capped at 8192 by a forced EOS) and the batch is compacted as rows
             finish, to completion (--no-shared-prefix for the per-sequence attention path)
  omni_b64   the 30B-A3B shape, 64 sequences of 1024..4096 injected embedding positions plus
             256 ids, then 4 turns of a 128-token tool chunk followed by 512 sampled tokens,
             KV carried across turns
  stream_b256  the 4B shape, 768 requests of the grouped recipe (own prompt pages) through 256 slots:
             one batch run to completion, then all requests with every freed slot refilled
             (wall time incl. prefill; completion event per micro-batch of 32)
--replay-report (moe_b128 or dense_b64) times nothing: it generates, then scores the responses with
the teacher-forced entry point with and without routing replay and reports |dlogprob|.
Prints ONE JSON line: decode tokens/s, ms/step, the roofline record of the dominant
kernel (timed in situ with HIP events) and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
METRIC = "rollout decode tokens/sec on 1 MI355X; % of HBM roofline per step"


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def gpu_random_model(pkg, synthetic, shape, split, seed=0, fmt="bf16"):
    """Random-init weights of the named shape generated on the device (same distributions as
    rollout_inputs: matrices N(0, 0.02), gains 1 + N(0, 0.02), router N(0, 1/d))."""
    return synthetic.device_random_model(shape, seed, split, fmt)


def kernel_bytes(shape, cls, ctx_sum_plus_b, touched=None):
    """Algorithmic HBM bytes of one launch of a kernel class (16-bit operands read once; touched: distinct
    experts the launch streams, MoE only)."""
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
    """Algorithmic bytes of one decode step: weights streamed once + KV read once + KV appended
    (touched: distinct experts per layer, averaged over the layers)."""
    s = shape
    w = sum(kernel_bytes(s, c, 0, touched) for c in ("qkv", "oproj", "gateup", "down")) * s.n_layers
    if s.is_moe:
        w += s.n_experts * s.d_model * 2 * s.n_layers
    w += kernel_bytes(s, "lmhead", 0)
    kv_tok = s.n_layers * s.n_kv_heads * s.head_dim * 2 * 2
    return w + kv_tok * ctx_sum_plus_b + kv_tok * batch


def prefill_flops(shape, plen, ctx0=None):
    """Useful floating-point operations of prefilling chunks of the given lengths behind ctx0 cached positions
    (2 per multiply-add; the two-term activations double the MFMA work actually issued, which is not counted)."""
    s = shape
    qdim, kvdim = s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
    per_tok = s.d_model * (qdim + 2 * kvdim) + qdim * s.d_model
    if s.is_moe:
        per_tok += s.d_model * s.n_experts + s.top_k * 3 * s.d_model * s.d_ff_expert
    else:
        per_tok += 3 * s.d_model * s.d_ff
    lin = 2.0 * per_tok * s.n_layers * float(np.sum(plen))
    ctx0 = np.zeros(len(plen)) if ctx0 is None else ctx0
    attn = sum(2.0 * 2 * qdim * (n * (n + 1) / 2.0 + c * n) for n, c in zip(plen, ctx0)) * s.n_layers   # causal q.k and p.v
    head = 2.0 * s.vocab * s.d_model * len(plen)                                     # only the sampled rows
    return lin + attn + head


def traffic_record(workload, kernel_class):
    """(ratio, file): measured-over-algorithmic HBM bytes of the dominant kernel from the committed counter summary
    (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script), or (None, None) when there is none for this
    workload/kernel or the kernel's sources have changed since it was taken."""
    import hashlib
    rel = os.path.join("profiles", "%s_decode_%s_traffic.txt" % (kernel_class, workload))
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    rec = {}
    for line in open(path):
        if "=" in line and not line.startswith("#"):
            k, v = line.split("=", 1)
            rec[k.strip()] = v.strip()
    srcs = [os.path.join(ROOT, "paper_2604_11554_amd", "csrc", f.strip()) for f in rec.get("sources", "").split(",") if f.strip()]
    if not srcs or not all(os.path.exists(f) for f in srcs):
        return None, None
    if rec.get("source_sha256") != hashlib.sha256(b"".join(open(f, "rb").read() for f in srcs)).hexdigest():
        return None, None
    return float(rec["ratio_measured_over_algorithmic"]), rel


def cpu_baseline(shape, wl, n_decode, fmt="bf16", sample=128):
    """The oracle's decode step timed on the host.  Bounded sample: the first `sample` sequences of the batch (all
    of them at the benchmark's batch sizes), one step at the start-of-decode context lengths and one at the
    end-of-decode ones, on 1- and 3-layer slices of the same shape (all layers of these shapes do not fit the host as fp32) scaled to the full depth; the caches hold
    synthetic N(0, 1) keys and values handed to the oracle through its set_cache call."""
    import oracle as O
    import rollout_inputs as RI
    from paper_2604_11554_amd import synthetic
    cores = len(os.sched_getaffinity(0))
    nl = 3
    sub = shape.replace(n_layers=nl)
    log("cpu baseline: generating a %d-layer slice of %s on the host" % (nl, shape.name))
    tensors = synthetic.generate_tensors(sub, 0, threads=min(16, cores), fmt=fmt)
    rng = np.random.default_rng(0)
    bs = min(wl.batch, sample)
    t_begin = time.perf_counter()
    times = {}
    for k in (1, nl):
        shp = shape.replace(n_layers=k)
        model = O.OracleModel(shp, 0, tensors={key: v for key, v in tensors.items() if key[0] < k}, fmt=fmt)
        model.globals
        for l in range(k):
            model.layer(l)
        for phase, extra in (("start", 0), ("end", n_decode - 2)):
            lens = [int(n) + extra for n in wl.prompt_lens[:bs]]
            ro = O.OracleRollout(model, n_blocks=int(sum((n + 17) // 16 + 1 for n in lens)))
            for i in range(bs):
                j = ro.add_sequence(int(wl.seeds[i]))
                kv = rng.standard_normal((2, k, lens[i], shp.n_kv_heads, shp.head_dim), dtype=np.float32)
                ro.set_cache(j, kv[0], kv[1], int(wl.prompt_tokens[i][-1]))
            ids = list(range(bs))
            if phase == "start" and k == 1:
                ro.decode_step(ids[:2])                  # warm the BLAS threads (two rows move on by one position)
            t0 = time.perf_counter()
            ro.decode_step(ids)
            times[(k, phase)] = time.perf_counter() - t0
            log("cpu baseline: %d layer(s), %s-of-decode contexts: %.2f s per step of %d sequences" % (
                k, phase, times[(k, phase)], bs))
    full = {}
    for phase in ("start", "end"):
        per_layer = (times[(nl, phase)] - times[(1, phase)]) / (nl - 1)
        full[phase] = times[(1, phase)] + per_layer * (shape.n_layers - 1)
    step_s = 0.5 * (full["start"] + full["end"])
    return {"value": bs / step_s, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": "first %d of %d sequences, one decode step at start-of-decode and one at end-of-decode context "
                      "lengths (synthetic cache contents), on 1- and %d-layer slices + LM head scaled to %d layers: "
                      "%.2f s and %.2f s per step, mean %.2f s; %.0f s of oracle time in all" % (
                          bs, wl.batch, nl, shape.n_layers, full["start"], full["end"], step_s,
                          time.perf_counter() - t_begin)}


def touched_experts(routing_steps, shape, live=None):
    """Distinct experts per layer (mean over layers) of each captured step: routing_steps int32 [K, B, L, top_k]."""
    import torch
    k, b, l, tk = routing_steps.shape
    idx = routing_steps.permute(0, 2, 1, 3).reshape(k, l, b * tk).long().clamp_(0, shape.n_experts - 1)
    hit = torch.zeros((k, l, shape.n_experts), dtype=torch.bool, device=routing_steps.device)
    hit.scatter_(2, idx, True)
    return hit.sum(2).float().mean(1).cpu().numpy()


def prefill_batch(eng, wl, bsz, plen, chunk_budget, embeds=None):
    """Chunked prefill of rows 0..bsz-1 (several sequences per call up to the budget); returns the seconds of the
    timed pass (an untimed pass over the first chunk loads the kernels first)."""
    import torch
    chunks, i = [], 0
    while i < bsz:
        j, tot = i, 0
        while j < bsz and tot + int(plen[j]) <= chunk_budget:
            tot += int(plen[j])
            j += 1
        chunks.append((i, j))
        i = j

    def emb(i, j):
        return None if embeds is None else embeds(i, j)

    i, j = chunks[0]
    eng.prefill(list(range(i, j)), wl.prompt_tokens[i:j], emb(i, j))
    eng.ctx_lens[i:j] = 0
    eng.finished[i:j] = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i, j in chunks:
        eng.prefill(list(range(i, j)), wl.prompt_tokens[i:j], emb(i, j))
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def class_times(B, eng, shape, extra, step_fn, n_steps=2):
    """Per-step kernel time by class: every class bracketed over n_steps steps (rlx_profile_kernel)."""
    classes = ["qkv", "attn", "oproj", "gateup", "down", "lmhead", "norm", "rope", "attn_merge"]
    if shape.is_moe:
        classes += ["router", "group"]
    classes += extra
    per_class = {}
    for cls in classes:
        kt = B.KernelTimer(cls, 4 * shape.n_layers, 1)
        for s in range(n_steps):
            step_fn(s)
        d = kt.finish()
        per_class[cls] = float(np.sum(d)) / n_steps
    return per_class, len(classes) * n_steps


def event_pair_overhead():
    import torch
    null_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(64)]
    for a_, b_ in null_ev:
        a_.record(); b_.record()
    torch.cuda.synchronize()
    return float(np.median([a_.elapsed_time(b_) for a_, b_ in null_ev]))


# ---------------------------------------------------------------------------------------------------------------
# fixed-batch workloads: dense_b64, moe_b128, grouped_b256 (first steps)
# ---------------------------------------------------------------------------------------------------------------

def run_batch(args, workload, with_cpu_baseline):
    import torch
    import paper_2604_11554_amd as pkg
    import rollout_inputs as RI
    from paper_2604_11554_amd import binding as B
    from paper_2604_11554_amd import synthetic

    dev = "cuda:0"
    grouped = workload == "grouped_b256"
    if workload == "dense_b64":
        shape, wl = RI.QWEN3_4B, RI.workload_dense_batch()
    elif grouped:
        shape, wl = RI.QWEN3_4B, RI.workload_grouped()
        wl.n_decode[:] = 512                      # the first steps of the responses are timed, uncapped
    else:
        shape, wl = RI.QWEN3_30B_A3B, RI.workload_moe_batch()
    steps = args.steps
    if grouped and steps <= 0:
        steps = 256
    # the settings the parity tests at this shape pass with
    split = args.split if args.split >= 0 else (1 if args.dtype == "bf16" else 0)
    n_decode = int(wl.n_decode[0])
    bsz = wl.batch
    plen = wl.prompt_lens
    log("workload %s: %s, batch %d, prompts %d..%d, decode %d, %s, activation_split %d" % (
        workload, shape.name, bsz, plen.min(), plen.max(), n_decode, args.dtype, split))

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
    shared_tok = np.zeros(bsz, np.int64)         # cached positions of each sequence that prefix tiles serve
    shared_pages_tok = np.zeros(bsz, np.int64)   # cached positions of each sequence that lie in pages its group shares
    pf_lens = plen                               # lengths of the sequences the prefill calls processed
    if grouped:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        plen, pf_lens = prefill_groups(eng, wl, leaders, bsz, plen, n_decode)
        shared_pages_tok[:] = [16 * ((int(n) - 1) // 16) for n in plen]
        if eng.share_prefix_attention:
            shared_tok[:] = [32 * ((int(n) - 1) // 32) for n in plen]
        torch.cuda.synchronize()
        t_prefill = time.perf_counter() - t0
    else:
        t_prefill = prefill_batch(eng, wl, bsz, plen, chunk_budget)
    log("prefill: %d tokens in %.2f s (%.0f tok/s, %.0f TFLOP/s useful = %.1f%% of the bf16 MFMA peak)" % (
        pf_lens.sum(), t_prefill, pf_lens.sum() / t_prefill, prefill_flops(shape, pf_lens) / t_prefill / 1e12,
        100 * prefill_flops(shape, pf_lens) / t_prefill / 1e12 / 2500.0))

    total_steps = n_decode - 1
    K = min(steps if steps > 0 else total_steps, total_steps)
    W = args.warmup
    # Fewer timed steps than the decode phase has: they are taken around the middle of the phase, not at its start.
    # A step's cost is linear in the cached positions, so the mean step of the whole phase is the step at the mean
    # context; the first steps of the phase, with the shortest contexts, understate it.  The response tokens before
    # the window are random ids appended by an untimed prefill pass in place of sampled ones (same cache contents
    # as far as cost goes); the token that the prompt prefill sampled is dropped.
    skip = 0
    if not grouped and not args.from_start and K + 2 < total_steps:
        skip = (total_steps - K) // 2            # warm-up and class-timing steps run on a saved state and are undone
    if skip > 0:
        g = np.random.default_rng(12345)
        filler = [g.integers(0, shape.vocab - 2, size=skip).astype(np.int32) for _ in range(bsz)]
        t0 = time.perf_counter()
        i = 0
        while i < bsz:
            j = min(bsz, i + max(1, chunk_budget // skip))
            eng.prefill(list(range(i, j)), filler[i:j])
            i = j
        torch.cuda.synchronize()
        log("response tokens 1..%d of every sequence appended as random ids (%.2f s, untimed): the timed steps emit "
            "tokens %d..%d of %d" % (skip, time.perf_counter() - t0, skip + 2, skip + 1 + K, n_decode))
        plen = plen + skip                       # cached positions at the start of the decode steps that follow
    lp_buf = torch.zeros((K + W + 64, bsz), dtype=torch.float32, device=dev)
    # MoE: the routing every timed step captures is kept (what Rollout Routing Replay would consume); the experts a
    # step streams are counted from it afterwards
    routing = (torch.zeros((K + 2, bsz, shape.n_layers, shape.top_k), dtype=torch.int32, device=dev)
               if shape.is_moe else None)

    def step(s, slot=None):
        eng.decode_step(out_logprobs=lp_buf[s], out_routing=None if routing is None else routing[K + 1 if slot is None else slot])

    def save():
        return [t.clone() for t in (eng.tokens, eng.ctx_lens, eng.finished)]

    def restore(st):
        for t, s in zip((eng.tokens, eng.ctx_lens, eng.finished), st):
            t.copy_(s)

    # ---- warmup on a saved state (the KV written here is overwritten by the timed steps) ----
    st = save()
    for s in range(W):
        step(s)
    torch.cuda.synchronize()

    # ---- pick the dominant kernel class: time each class over two steps ----
    per_class, n_class_steps = class_times(B, eng, shape, ["attn_prefix"] if shared_tok.any() else [], step)
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
        step(s, s)
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    durs = kt.finish()
    ms_total = ev0.elapsed_time(ev1)
    ms_step = ms_total / K
    toks_per_s = bsz * K / (ms_total / 1e3)

    # ---- byte model ----
    touched = None                               # per timed step: distinct experts per layer, from the captured routing
    if shape.is_moe:
        touched = touched_experts(routing[:K], shape)
        e = shape.n_experts
        log("experts streamed per layer and step (counted from the captured routing): mean %.2f, min %.2f (expected "
            "%.2f)" % (touched.mean(), touched.min(), e * (1.0 - (1.0 - shape.top_k / e) ** bsz)))
    ctx0 = plen.astype(np.int64)
    # launch i of the sampled class happened at step (i * stride) // launches_per_step
    ach_bytes = []
    for i in range(len(durs)):
        s = (i * stride) // launches_per_step
        # the per-sequence attention kernel reads what the prefix tiles do not serve
        ach_bytes.append(kernel_bytes(shape, dom, int((ctx0 + s + 1 - shared_tok).sum()),
                                      None if touched is None else float(touched[s]))
                         if dom in ("attn", "qkv", "oproj", "gateup", "down", "lmhead") else 0)
    ev_overhead = event_pair_overhead()          # cost of an empty event pair on this stream, subtracted from every sample
    durs = [max(d - ev_overhead, 1e-4) for d in durs]
    kern_ms = float(np.mean(durs)) if durs else float("nan")
    achieved = float(np.sum(ach_bytes)) / (float(np.sum(durs)) * 1e-3) / 1e9 if durs else float("nan")
    ratio, ratio_src = traffic_record(workload, dom)
    traffic = None if ratio is None or not durs else ratio * float(np.mean(ach_bytes))
    # a page shared by the eight members of a group counts once (the strict algorithmic minimum; the prefix tiles
    # read it once per subgroup of 32 / (n_q_heads / n_kv_heads) members); with no groups the two figures coincide
    uniq = (ctx0 - shared_pages_tok).sum() + (shared_pages_tok.sum() // 8 if grouped else 0)
    tch = (lambda s: None) if touched is None else (lambda s: float(touched[s]))
    step_b = np.mean([step_bytes(shape, int(uniq + (s + 1) * bsz), bsz, tch(s)) for s in range(K)])
    step_b_logical = np.mean([step_bytes(shape, int((ctx0 + s + 1).sum()), bsz, tch(s)) for s in range(K)])
    step_gbs = step_b / (ms_step * 1e-3) / 1e9
    fin = int(eng.finished[:bsz].sum().item())
    # every decode step this process ran (warmup, per-class timing, timed region) and the cached positions it
    # attended: what per-dispatch hardware counters of a profiled run average over
    offs = list(range(W)) + [W + i for i in range(n_class_steps)] + list(range(K))
    log("all decode steps run: %d, mean positions attended per step (sum over sequences, new token included) %.2f" % (
        len(offs), float(np.mean([(ctx0 + o + 1).sum() for o in offs]))))
    log("decode: %d steps, %.3f ms/step, %.0f tok/s; step bytes %.2f GB -> %.0f GB/s (%.1f%% of 8 TB/s); "
        "host wall %.2f s; finished rows %d" % (K, ms_step, toks_per_s, step_b / 1e9, step_gbs,
                                                 100 * step_gbs / HBM_PEAK_GBS, wall, fin))

    rec = {
        "metric": METRIC,
        "value": toks_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": "%s: %s, batch %d, prompts uniform %d..%d, %d decoded tokens, paged %s KV block 16, "
                               "temperature 1 Gumbel-max" % (workload, shape.name, bsz, wl.prompt_lens.min(), wl.prompt_lens.max(),
                                                              n_decode, args.dtype),
                   "activation_split": split, "prefill_tokens_per_s": float(pf_lens.sum() / t_prefill),
                   "timed_steps": ("the whole decode phase" if K == total_steps else
                                   "%d steps from the start of the decode phase" % K if skip == 0 else
                                   "%d steps around the middle of the decode phase, after %d response tokens per "
                                   "sequence (random ids appended by an untimed prefill pass)" % (K, skip))},
        # the prefill chunks that filled the cache before the timed decode steps (MFMA-bound part of the path)
        "prefill": {"tokens": int(pf_lens.sum()), "seconds": t_prefill, "tokens_per_s": float(pf_lens.sum() / t_prefill),
                    "bound": "mfma", "achieved": prefill_flops(shape, pf_lens) / t_prefill / 1e12, "peak": 2500.0,
                    "unit": "TFLOP/s", "frac": prefill_flops(shape, pf_lens) / t_prefill / 1e12 / 2500.0},
        "step_roofline": {"bound": "hbm", "achieved": step_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": step_gbs / HBM_PEAK_GBS, "bytes_per_step": float(step_b),
                          "bytes_per_step_per_sequence_kv": float(step_b_logical),
                          "frac_per_sequence_kv": step_b_logical / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                          "experts_streamed_per_layer": None if touched is None else float(touched.mean())},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": ratio_src,
                     "avg_launch_ms": kern_ms,
                     "bytes_per_launch": float(np.mean(ach_bytes)) if durs else None,
                     "event_pair_overhead_ms": ev_overhead, "launches_timed": len(durs),
                     "per_step_ms_by_class": per_class},
    }
    if with_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(shape, wl, n_decode, fmt=args.dtype)
    model.close()
    del eng, model, lp_buf, routing
    torch.cuda.empty_cache()
    return rec


def prefill_groups(eng, wl, leaders, bsz, plen, n_decode, max_ctx_of=None):
    """One donor row per prompt takes all but the last prompt token; the members fork from it (sharing its full
    pages) and prefill the last token themselves; the donors then leave the batch.  Returns (prompt length of each
    row in the engine's row order, lengths the prefill calls processed)."""
    donors, rows = {}, []
    for g in leaders:                        # a group is a run of rows: donor, then its members
        donors[g] = eng.add_sequence(0, reserve_tokens=int(plen[g]))
        eng.prefill([donors[g]], [wl.prompt_tokens[g][:-1]], sample_last=[False])
        for m in [k for k in range(bsz) if int(wl.group_of[k]) == g]:
            mc = int(plen[m]) + (n_decode if max_ctx_of is None else int(max_ctx_of[m]))
            rows.append((m, eng.fork(donors[g], int(wl.seeds[m]), float(wl.temperature[m]), max_ctx=mc)))
    eng.prefill([r for _, r in rows], [wl.prompt_tokens[m][-1:] for m, _ in rows])
    for g in leaders:
        eng.finished[donors[g]] = 1
    keep = eng.compact()
    assert len(keep) == bsz and eng.n == bsz
    # rows are now in group order; the host-side lengths follow
    pf_lens = np.array([int(plen[g]) - 1 for g in leaders])      # the members' single tokens are not counted
    return np.array([plen[m] for m, _ in rows], dtype=plen.dtype), pf_lens


# ---------------------------------------------------------------------------------------------------------------
# grouped_b256 --full: geometric response lengths with forced EOS, batch shrinkage, to completion
# ---------------------------------------------------------------------------------------------------------------

def run_grouped_full(args):
    import torch
    import paper_2604_11554_amd as pkg
    import rollout_inputs as RI
    from paper_2604_11554_amd import synthetic

    shape, wl = RI.QWEN3_4B, RI.workload_grouped()
    split = args.split if args.split >= 0 else (1 if args.dtype == "bf16" else 0)
    bsz, plen0, resp = wl.batch, wl.prompt_lens, wl.n_decode.astype(np.int64)
    log("workload grouped_b256 --full: %s, %d prompts x 8 members, prompts %d..%d, response lengths geometric mean "
        "2048 capped at 8192 (drawn: min %d, mean %.0f, max %d, %d tokens in all), %s" % (
            shape.name, bsz // 8, plen0.min(), plen0.max(), resp.min(), resp.mean(), resp.max(), resp.sum(), args.dtype))
    model = gpu_random_model(pkg, synthetic, shape, split, fmt=args.dtype)
    leaders = sorted(set(int(g) for g in wl.group_of))
    n_blocks = int(sum((int(plen0[g]) + 15) // 16 for g in leaders)) + int(sum((int(r) + 15) // 16 + 2 for r in resp)) + 8
    max_blocks = (int(plen0.max()) + int(resp.max()) + 15) // 16 + 1
    eng = pkg.RolloutEngine(model, n_blocks=n_blocks, max_seqs=bsz + len(leaders), max_chunk_tokens=32768,
                            max_blocks_per_seq=max_blocks)
    eng.share_prefix_attention = not args.no_shared_prefix
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plen, pf_lens = prefill_groups(eng, wl, leaders, bsz, plen0, 0, max_ctx_of=resp)
    torch.cuda.synchronize()
    t_prefill = time.perf_counter() - t0
    # host mirror of the rows: cached length, group, shared positions; the device is read every POLL steps
    POLL = 16
    order = [m for g in leaders for m in range(bsz) if int(wl.group_of[m]) == g]     # engine row -> workload index
    group = np.array([int(wl.group_of[m]) for m in order])
    shared_pos = np.array([16 * ((int(n) - 1) // 16) for n in plen], np.int64)
    ctx = eng.ctx_lens[:bsz].cpu().numpy().astype(np.int64)
    fin = eng.finished[:bsz].cpu().numpy().astype(bool)
    emitted = int(bsz)                           # the members' prefill emitted response token 1 of every row
    kv_tok = shape.n_layers * shape.n_kv_heads * shape.head_dim * 2 * 2
    w_bytes = step_bytes(shape, 0, 0)
    bytes_unique = bytes_logical = 0.0
    steps = compactions = 0
    since_compact = 0
    lp = torch.zeros((POLL, bsz), dtype=torch.float32, device="cuda:0")
    live_hist = []
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_wall = time.perf_counter()
    ev0.record()
    while not fin.all():
        n = eng.n
        for s in range(POLL):
            eng.decode_step(out_logprobs=lp[s, :n])
        steps += POLL
        since_compact += POLL
        new_ctx = eng.ctx_lens[:n].cpu().numpy().astype(np.int64)        # synchronises
        new_fin = eng.finished[:n].cpu().numpy().astype(bool)
        grew = new_ctx - ctx                     # steps of the window in which the row was live = tokens it emitted
        emitted += int(grew.sum())
        # KV bytes of the window: a row live for m steps attends ctx+1 .. ctx+m positions
        own = (ctx - shared_pos)[:, None] + np.arange(1, POLL + 1)[None, :]
        live_steps = np.arange(POLL)[None, :] < grew[:, None]
        bytes_logical += kv_tok * float(((own + shared_pos[:, None]) * live_steps).sum()) + kv_tok * float(grew.sum())
        # unique pages: a group's shared prompt positions count once per step while any member is live
        uniq = float((own * live_steps).sum())
        for g in np.unique(group):
            mem = group == g
            uniq += float(shared_pos[mem][0]) * float(live_steps[mem].any(0).sum())
        bytes_unique += kv_tok * uniq + kv_tok * float(grew.sum())
        any_live_steps = int(live_steps.any(0).sum())
        bytes_unique += w_bytes * any_live_steps
        bytes_logical += w_bytes * any_live_steps
        live_hist.append(int((~new_fin).sum()))
        ctx, fin = new_ctx, new_fin
        if steps % 512 == 0:
            log("  step %d: %d rows live of %d in the batch, %d tokens so far" % (steps, live_hist[-1], n, emitted - bsz))
        # compaction rule: at least a quarter of the rows finished, or 64 steps since the last one with any finished
        if (fin.mean() >= 0.25 or (since_compact >= 64 and fin.any())) and not fin.all():
            keep = eng.compact()
            ctx, fin, group, shared_pos = ctx[keep], fin[keep], group[keep], shared_pos[keep]
            compactions += 1
            since_compact = 0
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_wall
    ms_total = ev0.elapsed_time(ev1)
    decoded = emitted - bsz                      # tokens the decode steps emitted (the first came from the prefill)
    assert emitted == int(resp.sum()) or True    # natural EOS draws can end a response early
    toks_per_s = decoded / (ms_total / 1e3)
    log("decode to completion: %d steps, %d tokens in %.2f s (%.0f tok/s, %.3f ms/step), %d compactions; live rows "
        "per poll: first %d, median %d, last %d" % (steps, decoded, ms_total / 1e3, toks_per_s, ms_total / steps,
                                                     compactions, live_hist[0], int(np.median(live_hist)), live_hist[-1]))
    fu = bytes_unique / (ms_total * 1e-3) / 1e9
    fl = bytes_logical / (ms_total * 1e-3) / 1e9
    log("bytes: unique-page model %.1f TB -> %.0f GB/s (%.1f%% of 8 TB/s); per-sequence model %.1f TB -> %.0f GB/s (%.1f%%)" % (
        bytes_unique / 1e12, fu, 100 * fu / HBM_PEAK_GBS, bytes_logical / 1e12, fl, 100 * fl / HBM_PEAK_GBS))
    rec = {
        "metric": METRIC, "value": toks_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": 0,
        "ms_per_step": ms_total / steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": "grouped_b256 to completion: %s, 32 prompts uniform %d..%d x 8 members sharing prompt pages, "
                               "response lengths geometric (mean 2048) capped at 8192 by forced EOS, compaction when a "
                               "quarter of the rows have finished or every 64 steps, shared-prefix attention %s" % (
                                   shape.name, plen0.min(), plen0.max(), "on" if eng.share_prefix_attention else "off"),
                   "activation_split": split, "decoded_tokens": int(decoded), "compactions": compactions,
                   "decode_seconds": ms_total / 1e3, "host_wall_seconds": wall,
                   "prefill_tokens_per_s": float(pf_lens.sum() / t_prefill)},
        "step_roofline": {"bound": "hbm", "achieved": fu, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": fu / HBM_PEAK_GBS,
                          "bytes_total": bytes_unique, "bytes_total_per_sequence_kv": bytes_logical,
                          "frac_per_sequence_kv": fl / HBM_PEAK_GBS,
                          "note": "frac counts a page shared by a group's live members once per step (unique pages); "
                                  "frac_per_sequence_kv counts it once per member"},
        "roofline": None,
    }
    model.close()
    return rec


# ---------------------------------------------------------------------------------------------------------------
# omni_b64: injected multimodal positions, then turns of (tool chunk prefill -> sampled tokens)
# ---------------------------------------------------------------------------------------------------------------

def run_omni(args):
    import torch
    import paper_2604_11554_amd as pkg
    import rollout_inputs as RI
    from paper_2604_11554_amd import binding as B
    from paper_2604_11554_amd import synthetic

    shape = RI.QWEN3_30B_A3B
    wl = RI.workload_omni_agentic(shape, fmt=args.dtype)
    split = args.split if args.split >= 0 else (1 if args.dtype == "bf16" else 0)
    bsz = wl.batch
    plen = wl.prompt_lens
    n_turns, tool_len, turn_decode = len(wl.turns[0]), len(wl.turns[0][0].tool_tokens), wl.turns[0][0].n_decode
    log("workload omni_b64: %s, %d sequences of %d..%d injected positions + 256 ids, %d turns of %d tool ids + %d "
        "sampled tokens, %s" % (shape.name, bsz, plen.min() - 256, plen.max() - 256, n_turns, tool_len, turn_decode,
                                args.dtype))
    model = gpu_random_model(pkg, synthetic, shape, split, fmt=args.dtype)
    total = [int(p) + n_turns * (tool_len + turn_decode) + 8 for p in plen]
    eng = pkg.RolloutEngine(model, n_blocks=sum((t + 31) // 16 for t in total) + 8, max_seqs=bsz,
                            max_chunk_tokens=32768, max_blocks_per_seq=(max(total) + 31) // 16 + 1)
    for i in range(bsz):
        eng.add_sequence(int(wl.seeds[i]), 1.0, reserve_tokens=total[i])

    def embeds(i, j):
        out = []
        for r in range(i, j):
            full = np.zeros((int(plen[r]), shape.d_model), np.uint16)
            full[wl.prompt_tokens[r] < 0] = wl.prompt_embeds[r]
            out.append(full)
        return out

    # the prompts: nothing is sampled from them (the first turn's tool chunk follows)
    t_prompt = prefill_batch_nosample(eng, wl, bsz, plen, 32768, embeds)
    log("prompt prefill: %d positions in %.2f s (%.0f positions/s incl. the host-side staging of the embeddings)" % (
        plen.sum(), t_prompt, plen.sum() / t_prompt))
    K = turn_decode - 1                           # decode steps per turn: the tool chunk's prefill emits token 1
    routing = torch.zeros((K, bsz, shape.n_layers, shape.top_k), dtype=torch.int32, device="cuda:0")
    lp = torch.zeros((K, bsz), dtype=torch.float32, device="cuda:0")
    rows = list(range(bsz))
    dec_ms = pre_s = 0.0
    step_b = []
    per_class = None
    ctx = plen.astype(np.int64).copy()
    for turn in range(n_turns):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        eng.prefill(rows, [wl.turns[r][turn].tool_tokens for r in range(bsz)])
        torch.cuda.synchronize()
        pre_s += time.perf_counter() - t0
        ctx += tool_len
        if turn == 0:
            st = [t.clone() for t in (eng.tokens, eng.ctx_lens, eng.finished)]
            per_class, _ = class_times(B, eng, shape, [], lambda s: eng.decode_step(out_logprobs=lp[s], out_routing=routing[s]))
            for t, s_ in zip((eng.tokens, eng.ctx_lens, eng.finished), st):
                t.copy_(s_)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for s in range(K):
            eng.decode_step(out_logprobs=lp[s], out_routing=routing[s])
        ev1.record()
        torch.cuda.synchronize()
        dec_ms += ev0.elapsed_time(ev1)
        touched = touched_experts(routing, shape)
        step_b += [step_bytes(shape, int((ctx + s + 1).sum()), bsz, float(touched[s])) for s in range(K)]
        ctx += K
        log("turn %d: tool chunk + %d decode steps done (decode so far %.2f s)" % (turn, K, dec_ms / 1e3))
    n_steps = n_turns * K
    ms_step = dec_ms / n_steps
    toks_per_s = bsz * n_steps / (dec_ms / 1e3)
    sb = float(np.mean(step_b))
    gbs = sb / (ms_step * 1e-3) / 1e9
    log("decode: %d steps, %.3f ms/step, %.0f tok/s; step bytes %.2f GB -> %.0f GB/s (%.1f%% of 8 TB/s); tool-chunk "
        "prefills: %d tokens in %.2f s" % (n_steps, ms_step, toks_per_s, sb / 1e9, gbs, 100 * gbs / HBM_PEAK_GBS,
                                            n_turns * bsz * tool_len, pre_s))
    assert not eng.finished[:bsz].any().item() or True
    rec = {
        "metric": METRIC, "value": toks_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": n_steps, "warmup": 0,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": "omni_b64: %s, batch %d, %d..%d injected N(0,1) embedding positions + 256 ids, %d turns of "
                               "(%d tool ids prefilled, %d tokens sampled), KV carried across turns" % (
                                   shape.name, bsz, plen.min() - 256, plen.max() - 256, n_turns, tool_len, turn_decode),
                   "activation_split": split, "prompt_prefill_positions_per_s": float(plen.sum() / t_prompt),
                   "tool_prefill_tokens_per_s": float(n_turns * bsz * tool_len / pre_s)},
        "step_roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                          "bytes_per_step": sb},
        "roofline": {"per_step_ms_by_class": per_class},
    }
    model.close()
    return rec


def prefill_batch_nosample(eng, wl, bsz, plen, chunk_budget, embeds):
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    i = 0
    while i < bsz:
        j, tot = i, 0
        while j < bsz and tot + int(plen[j]) <= chunk_budget:
            tot += int(plen[j])
            j += 1
        eng.prefill(list(range(i, j)), wl.prompt_tokens[i:j], embeds(i, j), sample_last=[False] * (j - i))
        i = j
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def run_stream(args):
    """Continuous refill against a batch that runs to completion (paper Sec. 3.3, streaming micro-batches): the same
    long-tailed requests (the grouped workload's recipe, every request with its own prompt pages) pass through 256
    slots, first 256 of them as one batch with no request behind them, then all of them with every freed slot
    refilled by the next request and a completion event per micro-batch of 32.  Wall time includes the prefill calls."""
    import torch
    import paper_2604_11554_amd as pkg
    import rollout_inputs as RI
    from paper_2604_11554_amd import synthetic
    from paper_2604_11554_amd.engine import Request, StreamingRollout

    shape = RI.QWEN3_4B
    slots = 256
    n_req = max(slots, args.requests)
    wl = RI.workload_grouped(n_prompts=(n_req + 7) // 8)
    split = args.split if args.split >= 0 else (1 if args.dtype == "bf16" else 0)
    resp = wl.n_decode.astype(np.int64)[:n_req]
    reqs = [Request(wl.prompt_tokens[i], int(wl.seeds[i]), 1.0, int(resp[i])) for i in range(n_req)]
    plen = np.array([len(r.prompt) for r in reqs])
    log("workload stream_b256: %s, %d requests through %d slots, prompts %d..%d, response lengths geometric mean 2048 "
        "capped at 8192 (drawn: mean %.0f, max %d, %d tokens in all), %s" % (
            shape.name, n_req, slots, plen.min(), plen.max(), resp.mean(), resp.max(), resp.sum(), args.dtype))
    model = gpu_random_model(pkg, synthetic, shape, split, fmt=args.dtype)
    kv_tok = shape.n_layers * shape.n_kv_heads * shape.head_dim * 2 * 2
    need = sorted(((int(p) + int(r) + 15) // 16 + 1 for p, r in zip(plen, resp)), reverse=True)
    n_blocks = min(sum(need), int(200e9) // (16 * kv_tok)) + 8

    def run(requests, label):
        eng = pkg.RolloutEngine(model, n_blocks=n_blocks, max_seqs=slots, max_chunk_tokens=32768,
                                max_blocks_per_seq=max(need) + 1)
        events = []
        step_fn, n_calls = eng.decode_step, [0]

        def counted_step(*a, **k):               # a progress line every 1024 decode steps
            n_calls[0] += 1
            if n_calls[0] % 1024 == 0:
                log("  %s: decode step %d, %.1f s" % (label, n_calls[0], time.perf_counter() - t0))
            return step_fn(*a, **k)
        eng.decode_step = counted_step
        t0 = time.perf_counter()
        sr = StreamingRollout(eng, requests, micro_batch=32, poll_every=16, slots=slots,
                              on_partition=lambda p, c: events.append(time.perf_counter() - t0))
        done = sr.run()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        toks = int(sum(len(c.tokens) for c in done))
        sr_steps = sr.decode_steps
        log("%s: %d requests, %d response tokens in %.1f s (%.0f tok/s), %d decode steps, %.1f rows live per step on "
            "average, first micro-batch complete after %.1f s, last after %.1f s" % (
                label, len(requests), toks, wall, toks / wall, sr.decode_steps, toks / max(1, sr.decode_steps),
                events[0], events[-1]))
        del eng.decode_step                      # the counting wrapper refers to the engine
        del sr, eng, done
        gc.collect()
        torch.cuda.empty_cache()                 # the next run allocates its own page pool
        return {"requests": len(requests), "tokens": toks, "seconds": wall, "tokens_per_s": toks / wall,
                "decode_steps": sr_steps, "mean_live_rows": toks / max(1, sr_steps),
                "first_micro_batch_s": events[0], "last_micro_batch_s": events[-1]}

    one = run(reqs[:slots], "one batch to completion")
    allr = run(reqs, "continuous refill")
    rec = {"metric": METRIC, "value": allr["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": allr["decode_steps"],
           "warmup": 0, "ms_per_step": 1e3 * allr["seconds"] / allr["decode_steps"], "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
           "config": {"workload": "stream_b256: %s, %d requests through %d slots with continuous refill, prompts %d..%d, "
                                  "geometric response lengths (mean 2048, cap 8192), wall time incl. prefill" % (
                                      shape.name, n_req, slots, plen.min(), plen.max()), "activation_split": split},
           "continuous_refill": allr, "one_batch_to_completion": one,
           "refill_over_batch": allr["tokens_per_s"] / one["tokens_per_s"]}
    model.close()
    return rec


def run_replay_report(args):
    """Rollout Routing Replay on the library's own two paths (paper Sec. 5.5): sequences are generated by decode steps
    with the routing captured, then prompt + response are scored by the teacher-forced entry point twice, once with
    its own routing and once replaying the captured one.  Reported: |log-prob of the rollout - log-prob of the
    scoring pass| over the response tokens, and how many routed (position, layer) pairs the scoring pass chose
    differently on its own.  Weights are random, so the figures show the mechanism, not the paper's values."""
    import torch
    import paper_2604_11554_amd as pkg
    import rollout_inputs as RI
    from paper_2604_11554_amd import synthetic

    dev = "cuda:0"
    if args.workload == "dense_b64":
        shape, wl = RI.QWEN3_4B, RI.workload_dense_batch()
    else:
        shape, wl = RI.QWEN3_30B_A3B, RI.workload_moe_batch()
    n_gen = args.steps if args.steps > 0 else 256
    split = args.split if args.split >= 0 else (1 if args.dtype == "bf16" else 0)
    bsz, plen = wl.batch, wl.prompt_lens
    log("replay report: %s, batch %d, prompts %d..%d, %d generated tokens per sequence, %s" % (
        shape.name, bsz, plen.min(), plen.max(), n_gen, args.dtype))
    model = gpu_random_model(pkg, synthetic, shape, split, fmt=args.dtype)
    passes = 3 if shape.is_moe else 2            # the rollout and one row set per scoring pass
    max_blocks = (int(plen.max()) + n_gen + 15) // 16 + 1
    n_blocks = passes * int(sum((int(n) + n_gen + 15) // 16 + 1 for n in plen)) + 8
    chunk_budget = 32768
    eng = pkg.RolloutEngine(model, n_blocks=n_blocks, max_seqs=passes * bsz, max_chunk_tokens=chunk_budget,
                            max_blocks_per_seq=max_blocks)
    for i in range(bsz):
        eng.add_sequence(int(wl.seeds[i]), float(wl.temperature[i]), max_ctx=int(plen[i]) + n_gen + 8)

    def chunks_of(lens):
        out, i = [], 0
        while i < len(lens):
            j, tot = i, 0
            while j < len(lens) and tot + int(lens[j]) <= chunk_budget:
                tot += int(lens[j])
                j += 1
            out.append((i, j))
            i = j
        return out

    # ---- rollout: prefill, then n_gen - 1 decode steps, tokens / log-probs / routing kept ----
    gen = torch.zeros((n_gen, bsz), dtype=torch.int32, device=dev)
    lps = torch.zeros((n_gen, bsz), dtype=torch.float32, device=dev)
    rout_prompt = []
    for i, j in chunks_of(plen):
        out = eng.prefill(list(range(i, j)), wl.prompt_tokens[i:j], want_routing=shape.is_moe)
        gen[0, i:j] = out.tokens
        lps[0, i:j] = out.logprobs
        if shape.is_moe:
            r = out.routing.cpu().numpy()
            o = np.concatenate([[0], np.cumsum(plen[i:j])])
            rout_prompt += [r[o[k]:o[k + 1]] for k in range(j - i)]
    rout_dec = (torch.zeros((n_gen - 1, bsz, shape.n_layers, shape.top_k), dtype=torch.int32, device=dev)
                if shape.is_moe else None)
    for s in range(1, n_gen):
        eng.decode_step(out_logprobs=lps[s], out_routing=None if rout_dec is None else rout_dec[s - 1])
        gen[s] = eng.tokens[:bsz]
    torch.cuda.synchronize()
    alive = (eng.finished[:bsz] == 0).cpu().numpy()      # a sequence that sampled an end token stops being recorded
    gen_h, lps_h = gen.cpu().numpy(), lps.cpu().numpy()
    rout_h = None if rout_dec is None else rout_dec.cpu().numpy()
    keep = [i for i in range(bsz) if alive[i]]
    log("rollout done: %d of %d sequences ran all %d steps" % (len(keep), bsz, n_gen - 1))

    toks = [np.concatenate([wl.prompt_tokens[i], gen_h[:-1, i]]).astype(np.int32) for i in keep]
    tg = []
    for i, t in zip(keep, toks):
        x = np.full(len(t), -1, np.int32)
        x[int(plen[i]) - 1:] = gen_h[:, i]
        tg.append(x)
    recorded = ([np.concatenate([rout_prompt[i], rout_h[:, i]]) for i in keep] if shape.is_moe else None)

    def score_pass(replay):
        rows = [eng.add_sequence(0, float(wl.temperature[i]), reserve_tokens=len(t) + 16) for i, t in zip(keep, toks)]
        got, used = [], []
        for a, b in chunks_of([len(t) for t in toks]):
            lp, rt = eng.score(rows[a:b], toks[a:b], tg[a:b], replay_routing=None if not replay else recorded[a:b],
                               want_routing=shape.is_moe)
            lp = lp.cpu().numpy()
            rt = None if rt is None else rt.cpu().numpy()
            o = np.concatenate([[0], np.cumsum([len(t) for t in toks[a:b]])])
            for k in range(b - a):
                got.append(lp[o[k]:o[k + 1]])
                if rt is not None:
                    used.append(rt[o[k]:o[k + 1]])
        return got, used

    def stats(got):
        d = np.concatenate([np.abs(g[int(plen[i]) - 1:].astype(np.float64) - lps_h[:, i]) for i, g in zip(keep, got)])
        return {"tokens": int(d.size), "mean": float(d.mean()), "p99": float(np.quantile(d, 0.99)),
                "max": float(d.max()), "share_above_1e-3": float((d > 1e-3).mean())}

    rec = {"metric": "|log-prob of the rollout - log-prob of teacher-forced scoring| over the response tokens",
           "unit": "nats", "n_gpus": 1, "steps": n_gen - 1, "warmup": 0, "higher_is_better": False,
           "dtype": args.dtype, "data": "synthetic",
           "config": {"workload": "replay report: %s, batch %d, prompts %d..%d, %d generated tokens per sequence" % (
               shape.name, bsz, plen.min(), plen.max(), n_gen), "activation_split": split}}
    own, used = score_pass(False)
    rec["scoring_with_its_own_routing" if shape.is_moe else "scoring"] = st_own = stats(own)
    log("scoring with its own %s: mean |dlogprob| %.2e, p99 %.2e, max %.2e, %.2f %% of %d tokens above 1e-3" % (
        "routing" if shape.is_moe else "kernels", st_own["mean"], st_own["p99"], st_own["max"],
        100 * st_own["share_above_1e-3"], st_own["tokens"]))
    rec["value"] = st_own["mean"]
    if shape.is_moe:
        differ = sum(int((np.sort(u, axis=-1) != np.sort(r, axis=-1)).any(axis=-1).sum()) for u, r in zip(used, recorded))
        pairs = sum(u.shape[0] * u.shape[1] for u in used)
        rec["routed_pairs_chosen_differently"] = {"pairs": pairs, "differ": differ, "share": differ / pairs}
        log("the scoring pass chose another expert set than the rollout at %d of %d (position, layer) pairs (%.3f %%)" % (
            differ, pairs, 100.0 * differ / pairs))
        rep, used = score_pass(True)
        echoed = all((u == r).all() for u, r in zip(used, recorded))
        rec["scoring_with_replayed_routing"] = st_rep = stats(rep)
        rec["replayed_routing_echoed"] = bool(echoed)
        rec["value"] = st_rep["mean"]
        log("scoring with the rollout's routing replayed: mean |dlogprob| %.2e, p99 %.2e, max %.2e, %.2f %% above 1e-3 "
            "(mean %.0f %% lower); replayed ids echoed: %s" % (st_rep["mean"], st_rep["p99"], st_rep["max"],
                                                            100 * st_rep["share_above_1e-3"],
                                                            100 * (1 - st_rep["mean"] / st_own["mean"]), echoed))
    model.close()
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="decode steps to time (0 = the whole decode phase); fewer than "
                    "the phase has are taken around its middle")
    ap.add_argument("--from-start", action="store_true", help="with --steps: time the first steps of the decode phase instead")
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="default",
                    choices=["default", "dense_b64", "moe_b128", "grouped_b256", "omni_b64", "stream_b256"],
                    help="default: moe_b128 as the headline and dense_b64 under \"also\" in the same JSON line")
    ap.add_argument("--full", action="store_true",
                    help="grouped_b256: geometric response lengths with forced EOS and batch compaction, to completion")
    ap.add_argument("--requests", type=int, default=768, help="stream_b256: requests to pass through the 256 slots")
    ap.add_argument("--no-shared-prefix", action="store_true",
                    help="grouped_b256: read the shared prompt pages once per sequence instead of once per subgroup")
    ap.add_argument("--split", type=int, default=-1,
                    help="activation_split (default: 1 for bf16, two terms per activation; 0 for f16, one term)")
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f16"],
                    help="16-bit format of weights, KV pages and activation terms (f16: the FP16 precision option)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--replay-report", action="store_true",
                    help="moe_b128 / dense_b64: generate --steps tokens per sequence (default 256), score them with the "
                         "teacher-forced entry point with and without routing replay, report |dlogprob| (no timing)")
    ap.add_argument("--kernel", default="auto", help="kernel class for the roofline record")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 256 MiB device copy (reference of known size for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    from paper_2604_11554_amd import binding as B
    B.lib()
    if args.replay_report:
        if args.workload not in ("default", "moe_b128", "dense_b64"):
            ap.error("--replay-report runs on moe_b128 (the default) or dense_b64")
        rec = run_replay_report(args)
    elif args.workload == "grouped_b256" and args.full:
        rec = run_grouped_full(args)
    elif args.workload == "omni_b64":
        rec = run_omni(args)
    elif args.workload == "stream_b256":
        rec = run_stream(args)
    elif args.workload == "default":
        rec = run_batch(args, "moe_b128", not args.no_cpu_baseline)
        rec["also"] = {"dense_b64": run_batch(args, "dense_b64", False)}
    else:
        rec = run_batch(args, args.workload, not args.no_cpu_baseline)
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
