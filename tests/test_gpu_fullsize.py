"""Parity at the benchmark's full shapes, in the launch configuration bench.py times (same batch, same
kernels), on sampled sequences the oracle can recompute one by one.  The dense 4B shape runs with all 36
layers; the 30B-A3B MoE shape runs as a 2-layer slice of the same per-layer shape (all 128 experts, top-8,
batch 128), because generating and holding its 61 GB of synthetic weights on the host takes too long for a test."""
import sys
import time

import numpy as np
import pytest
import torch

import oracle as O
import rollout_inputs as RI

pytestmark = pytest.mark.gpu

LOGIT_BAR, LOGPROB_BAR, TIE_GAP = 0.05, 0.02, 1e-3


def say(msg):
    print("[gpu-case %s] %s" % (time.strftime("%H:%M:%S"), msg), flush=True)
    sys.stdout.flush()


def _prefill_all(eng, wl, budget, rows_of_interest):
    """Chunked prefill of the whole batch; returns {row: (token, logprob, logits, routing rows)}."""
    got = {}
    plen = wl.prompt_lens
    i = 0
    while i < wl.batch:
        j, tot = i, 0
        while j < wl.batch and tot + int(plen[j]) <= budget:
            tot += int(plen[j]); j += 1
        rows = list(range(i, j))
        o = eng.prefill(rows, wl.prompt_tokens[i:j], want_logits=True, want_routing=True)
        torch.cuda.synchronize()
        offs = np.concatenate([[0], np.cumsum(plen[i:j])])
        for k, r in enumerate(rows):
            if r in rows_of_interest:
                rt = None if o.routing is None else o.routing[offs[k]:offs[k + 1]].cpu().numpy()
                got[r] = (int(o.tokens[k]), float(o.logprobs[k]), o.logits[k].cpu().numpy(), rt)
        say("prefilled rows %d..%d (%d tokens)" % (i, j - 1, tot))
        i = j
    return got


def _run_case(shape, wl, split, n_steps, sample_rows, budget=32768, fmt="bf16", also_fp32_kv=False):   # bench.py's chunk budget
    import paper_2604_11554_amd as pkg
    from paper_2604_11554_amd import synthetic
    pkg.binding.lib()
    say("generating %s weights on the host" % shape.name)
    tensors = synthetic.generate_tensors(shape, 0, threads=12, progress=lambda i, n: say("  tensor %d/%d" % (i, n)),
                                        fmt=fmt)
    say("uploading")
    model = synthetic.model_from_tensors(shape, tensors, activation_split=split, fmt=fmt)
    plen = wl.prompt_lens
    mb = (int(plen.max()) + n_steps + 16) // 16 + 1
    eng = pkg.RolloutEngine(model, n_blocks=int(sum((int(n) + n_steps + 31) // 16 for n in plen)) + 8,
                            max_seqs=wl.batch, max_chunk_tokens=budget, max_blocks_per_seq=mb)
    for i in range(wl.batch):
        eng.add_sequence(int(wl.seeds[i]), 1.0, reserve_tokens=int(plen[i]) + n_steps + 8)
    got = _prefill_all(eng, wl, budget, set(sample_rows))
    steps = []                                    # per decode step: tokens, logprobs, logits, routing of sampled rows
    idx = torch.tensor(sample_rows, device="cuda:0")
    for s in range(n_steps):
        o = eng.decode_step(want_logits=True, want_routing=True)
        torch.cuda.synchronize()
        steps.append((o.tokens[idx].cpu().numpy().copy(), o.logprobs[idx].cpu().numpy().copy(),
                      o.logits[idx].cpu().numpy().copy(),
                      None if o.routing is None else o.routing[idx].cpu().numpy().copy()))
        say("decode step %d done" % s)
    # ---- oracle: teacher-forced on the GPU's own tokens, replaying the GPU's routing (routing replay) so
    # that a tolerated near-tie does not hide everything after it; its own router choice is still reported
    seqs, replay = [], []
    for k, r in enumerate(sample_rows):
        toks = list(wl.prompt_tokens[r]) + [got[r][0]] + [int(st[0][k]) for st in steps[:-1]]
        seqs.append(np.array(toks, np.int32))
        if shape.is_moe:
            replay.append(np.concatenate([got[r][3]] + [st[3][k][None] for st in steps], axis=0))
    at = [np.arange(int(plen[r]) - 1, int(plen[r]) + n_steps) for r in sample_rows]
    all_stats = {}
    # first the oracle that rounds K/V at the store like the library (all bars asserted), then the one that keeps
    # K/V in fp32 (logit and log-probability bars asserted; routing differences reported with their gaps)
    for kv_bf16 in ((True, False) if also_fp32_kv else (True,)):
        om = O.OracleModel(shape, 0, cache_layers=False, tensors=tensors, fmt=fmt, kv_bf16=kv_bf16)
        name = "rounded-KV oracle" if kv_bf16 else "fp32-KV oracle"
        say("%s: forward of %d sampled sequences (%s tokens)" % (name, len(seqs), [len(s) for s in seqs]))
        res = O.forward_full(om, seqs, forced_routing=replay if shape.is_moe else None, logits_at=at,
                             progress=lambda l: say("  oracle layer %d" % l))
        stats = dict(dlogit=0.0, dlogprob=0.0, tie_flips=0, routes=0, max_flip_gap=0.0)
        for k, r in enumerate(sample_rows):
            z_o = res[k]["logits"]
            lp_o = O.log_softmax(z_o)
            emitted = [got[r][0]] + [int(st[0][k]) for st in steps]
            z_g = [got[r][2]] + [st[2][k] for st in steps]
            lp_g = [got[r][1]] + [float(st[1][k]) for st in steps]
            for p in range(n_steps + 1):
                stats["dlogit"] = max(stats["dlogit"], float(np.abs(z_g[p] - z_o[p]).max()))
                stats["dlogprob"] = max(stats["dlogprob"], abs(lp_g[p] - float(lp_o[p, emitted[p]])))
                # the GPU's draw must be (nearly) the oracle's best perturbed score
                g = O.gumbel_noise(int(wl.seeds[r]), int(plen[r]) + p, shape.vocab)
                sc = z_o[p].astype(np.float64) + g
                assert sc[emitted[p]] >= sc.max() - 2 * LOGIT_BAR, "row %d step %d: bad draw" % (r, p)
            if shape.is_moe:
                own, gaps = res[k]["own_routing"], res[k]["gate_gap"]
                bad = (np.sort(replay[k], -1) != np.sort(own, -1)).any(-1)
                stats["routes"] += bad.size
                stats["tie_flips"] += int(bad.sum())
                if bad.any():
                    stats["max_flip_gap"] = max(stats["max_flip_gap"], float(gaps[bad].max()))
                if kv_bf16:
                    assert (gaps[bad] < TIE_GAP).all(), "routing differs at gate gap %.2e" % float(gaps[bad].max())
        say("%s %s sampled-row stats vs the %s: %s" % (shape.name, fmt, name, stats))
        if kv_bf16:
            assert stats["dlogit"] <= LOGIT_BAR and stats["dlogprob"] <= LOGPROB_BAR
            z_rounded = [r_["logits"] for r_ in res]
        else:
            # What separates the two oracles is the rounding of K and V at the store, which the workloads specify
            # ("paged KV bf16") and which no implementation of them can avoid.  The distance of the library to the
            # fp32-KV oracle is reported next to the distance between the two oracles themselves (logits, and the
            # log-probabilities of the emitted tokens) and must be explained by it.
            between = max(float(np.abs(a - r_["logits"]).max()) for a, r_ in zip(z_rounded, res))
            between_lp = 0.0
            for k, r in enumerate(sample_rows):
                emitted = [got[r][0]] + [int(st[0][k]) for st in steps]
                la, lb = O.log_softmax(z_rounded[k]), O.log_softmax(res[k]["logits"])
                between_lp = max(between_lp, max(abs(float(la[p, emitted[p]] - lb[p, emitted[p]])) for p in range(n_steps + 1)))
            say("DISTANCE to the fp32-KV oracle, %s %s, contexts %s: max |dlogit| %.5f, max |dlogprob| %.5f, routing "
                "differences %d of %d (largest oracle gap among them %.2e); the two oracles differ by max |dlogit| %.5f, "
                "max |dlogprob| %.5f" % (shape.name, fmt, [int(plen[r]) for r in sample_rows], stats["dlogit"],
                                         stats["dlogprob"], stats["tie_flips"], stats["routes"], stats["max_flip_gap"],
                                         between, between_lp))
            own = all_stats["rounded-KV oracle"]
            assert stats["dlogit"] <= between + own["dlogit"] + 1e-6
            assert stats["dlogprob"] <= between_lp + own["dlogprob"] + 1e-6
        all_stats[name] = stats
    model.close()
    return all_stats


def test_dense_4b_shape_batch64_sampled_rows():
    shape = RI.QWEN3_4B
    wl = RI.workload_dense_batch(shape)                       # 64 sequences, prompts uniform 256..1024
    plen = wl.prompt_lens
    rows = [int(np.argmin(plen)), int(np.argsort(plen)[len(plen) // 2])]   # shortest and median prompt
    # two more rows jump to the context lengths at which the benchmark's decode phase ends (prompt + 1024
    # decoded tokens, about 1650 positions): their prompts are replaced by 1600 and 1664 uniform ids
    g = np.random.default_rng(77)
    late = [r for r in range(wl.batch) if r not in rows][:2]
    for r, n in zip(late, (1600, 1664)):
        wl.prompt_tokens[r] = g.integers(0, shape.vocab - 2, size=n).astype(np.int32)
    _run_case(shape, wl, split=1, n_steps=3, sample_rows=rows + late, also_fp32_kv=True)


def test_dense_4b_layer_slice_batch200_decode_forms():
    """Decode steps of 200 tokens at the 4B per-layer shape (a 3-layer slice): the batch of the grouped workload
    before it shrinks takes the forms of 129..256-token calls (128-token tiles twice over in every GEMM, eleven
    split-K planes, the norm in quarters), which the 64-sequence batch does not reach."""
    shape = RI.QWEN3_4B.replace(name="qwen3_4b_shape_3layers", n_layers=3)
    wl = RI.workload_dense_batch(shape, batch=200, lo=20, hi=90, prompt_seed=12, seed_base=12000)
    _run_case(shape, wl, split=1, n_steps=3, sample_rows=[0, 101, 199])


def test_dense_4b_shape_batch64_sampled_rows_fp16():
    """The FP16 precision option (paper App. "FP16 vs. BF16 precision ablation") at the benchmark's shape:
    fp16 weights and KV pages, one fp16 term per activation, against the oracle with the same fp16 roundings."""
    shape = RI.QWEN3_4B
    wl = RI.workload_dense_batch(shape)
    plen = wl.prompt_lens
    rows = [int(np.argmin(plen)), int(np.argsort(plen)[len(plen) // 2])]
    _run_case(shape, wl, split=0, n_steps=3, sample_rows=rows, fmt="f16")


def test_dense_4b_shape_sampling_groups_shared_prefix_sampled_rows():
    """Decode over shared prompt pages at the 4B shape (head_dim 128, four members per prefix tile, several chunks
    per prefix): two prompts x 8 group members, the tokens the GPU emits checked by the oracle's full forward of two
    members (no sharing on the oracle's side)."""
    import paper_2604_11554_amd as pkg
    from paper_2604_11554_amd import synthetic
    pkg.binding.lib()
    shape = RI.QWEN3_4B
    n_steps, lens, members = 3, (700, 333), 8
    g = np.random.default_rng(21)
    prompts = [g.integers(0, shape.vocab - 2, size=n).astype(np.int32) for n in lens]
    say("generating %s weights on the host" % shape.name)
    tensors = synthetic.generate_tensors(shape, 0, threads=12, progress=lambda i, n: say("  tensor %d/%d" % (i, n)))
    model = synthetic.model_from_tensors(shape, tensors, activation_split=1)
    mb = (max(lens) + n_steps + 16) // 16 + 1
    n_rows = len(lens) * (members + 1)
    eng = pkg.RolloutEngine(model, n_blocks=n_rows * mb, max_seqs=n_rows, max_chunk_tokens=1024, max_blocks_per_seq=mb)
    rows, seeds = [], []
    for gi, p in enumerate(prompts):
        d = eng.add_sequence(0, reserve_tokens=len(p))
        eng.prefill([d], [p[:-1]], sample_last=[False])
        for k in range(members):
            seeds.append(7000 + 10 * gi + k)
            rows.append(eng.fork(d, seeds[-1], reserve_tokens=len(p) + n_steps + 8))
        eng.finished[d] = 1
    o = eng.prefill(rows, [prompts[i // members][-1:] for i in range(len(rows))], want_logits=True)
    torch.cuda.synchronize()
    keep = eng.compact()                                      # the donors leave; groups are runs of 8 rows
    assert eng.n == len(rows)
    desc = eng._shared_prefix()
    n_tiles = int(desc[:8].view(torch.int32)[1].item())
    # 21 and 10 shared units: 3 and 2 chunks x one subgroup of the eight members x 8 KV heads
    assert n_tiles == (3 + 2) * shape.n_kv_heads, n_tiles
    sample = [3, members + 6]                                 # a member of each group
    got = {r: [(int(o.tokens[r]), float(o.logprobs[r]), o.logits[r].cpu().numpy())] for r in sample}
    for s in range(n_steps):
        o = eng.decode_step(want_logits=True)
        torch.cuda.synchronize()
        for r in sample:
            got[r].append((int(o.tokens[r]), float(o.logprobs[r]), o.logits[r].cpu().numpy()))
        say("decode step %d done" % s)
    om = O.OracleModel(shape, 0, cache_layers=False, tensors=tensors)
    seqs = [np.concatenate([prompts[r // members], [t for t, _, _ in got[r][:-1]]]).astype(np.int32) for r in sample]
    at = [np.arange(lens[r // members] - 1, lens[r // members] + n_steps) for r in sample]
    say("oracle forward of the two sampled members (%s tokens)" % [len(q) for q in seqs])
    res = O.forward_full(om, seqs, logits_at=at, progress=lambda l: say("  oracle layer %d" % l))
    dl = dp = 0.0
    for k, r in enumerate(sample):
        z_o = res[k]["logits"]
        lp_o = O.log_softmax(z_o)
        for p, (tok, lp, z) in enumerate(got[r]):
            dl = max(dl, float(np.abs(z - z_o[p]).max()))
            dp = max(dp, abs(lp - float(lp_o[p, tok])))
            sc = z_o[p].astype(np.float64) + O.gumbel_noise(seeds[r], lens[r // members] + p, shape.vocab)
            assert sc[tok] >= sc.max() - 2 * LOGIT_BAR, "row %d step %d: bad draw" % (r, p)
    say("%s shared prefixes: max |dlogit| %.5f, max |dlogprob| %.5f" % (shape.name, dl, dp))
    assert dl <= LOGIT_BAR and dp <= LOGPROB_BAR
    model.close()


def test_moe_30b_a3b_layer_slice_batch128_sampled_rows():
    shape = RI.QWEN3_30B_A3B.replace(name="qwen3_30b_a3b_shape_2layers", n_layers=2)
    wl = RI.workload_moe_batch(shape, prompt_len=128)         # 128 sequences, all experts touched every step
    _run_case(shape, wl, split=1, n_steps=3, sample_rows=[0, 77], also_fp32_kv=True)


def test_moe_30b_a3b_layer_slice_batch200_short_prompts():
    """Decode steps of 200 tokens at the 30B-A3B per-layer shape: the forms that calls of 129..256 tokens take (two
    128-token tiles in the store GEMMs, the gate/up kernel grouping 1600 (token, slot) pairs, a pair count that no
    workgroup size divides, about 12 rows per expert) are not reached by the benchmark batches of 64 and 128."""
    shape = RI.QWEN3_30B_A3B.replace(name="qwen3_30b_a3b_shape_2layers", n_layers=2)
    wl = RI.workload_moe_batch(shape, batch=200, prompt_len=24, prompt_seed=14, seed_base=14000)
    _run_case(shape, wl, split=1, n_steps=3, sample_rows=[3, 150, 199])


def test_moe_30b_a3b_full_depth_batch128_sampled_rows():
    """All 48 layers of the 30B-A3B shape with the benchmark's batch (128 sequences, 512-token prompts): the 61 GB of
    weights are drawn on the device, as the benchmark does; the oracle receives them one layer at a time (the same
    draws copied to the host) and recomputes two sampled rows teacher-forced on the tokens the GPU emitted,
    replaying the GPU's routing; its own routing choice at every (token, layer) is compared with the GPU's."""
    import paper_2604_11554_amd as pkg
    from paper_2604_11554_amd import synthetic
    pkg.binding.lib()
    shape = RI.QWEN3_30B_A3B
    wl = RI.workload_moe_batch(shape)                          # 128 sequences of 512 prompt tokens
    n_steps, sample_rows, budget = 3, [5, 101], 32768
    draw = synthetic.device_random_tensor(shape, 0)
    say("drawing and packing %s on the device" % shape.name)
    model = pkg.RolloutModel(synthetic.config_from_shape(shape, 1), draw)
    plen = wl.prompt_lens
    mb = (int(plen.max()) + n_steps + 16) // 16 + 1
    eng = pkg.RolloutEngine(model, n_blocks=wl.batch * mb, max_seqs=wl.batch, max_chunk_tokens=budget,
                            max_blocks_per_seq=mb)
    for i in range(wl.batch):
        eng.add_sequence(int(wl.seeds[i]), 1.0, reserve_tokens=int(plen[i]) + n_steps + 8)
    got = _prefill_all(eng, wl, budget, set(sample_rows))
    idx = torch.tensor(sample_rows, device="cuda:0")
    steps = []
    for s in range(n_steps):
        o = eng.decode_step(want_logits=True, want_routing=True)
        torch.cuda.synchronize()
        steps.append((o.tokens[idx].cpu().numpy().copy(), o.logprobs[idx].cpu().numpy().copy(),
                      o.logits[idx].cpu().numpy().copy(), o.routing[idx].cpu().numpy().copy()))
    say("decode steps done; oracle forward of rows %s, one layer of weights at a time" % sample_rows)

    def layer_bits(layer):                                     # the same draws, copied to the host as bit patterns
        return {n: draw(layer, n).cpu().view(torch.int16).numpy().view(np.uint16)
                for n in RI.tensor_names(shape, layer)}

    om = O.OracleModel(shape, 0, cache_layers=False, tensors=layer_bits)
    seqs, replay = [], []
    for k, r in enumerate(sample_rows):
        seqs.append(np.array(list(wl.prompt_tokens[r]) + [got[r][0]] + [int(st[0][k]) for st in steps[:-1]], np.int32))
        replay.append(np.concatenate([got[r][3]] + [st[3][k][None] for st in steps], axis=0))
    at = [np.arange(int(plen[r]) - 1, int(plen[r]) + n_steps) for r in sample_rows]
    res = O.forward_full(om, seqs, forced_routing=replay, logits_at=at,
                         progress=lambda l: say("  oracle layer %d" % l) if l % 8 == 7 else None)
    stats = dict(dlogit=0.0, dlogprob=0.0, tie_flips=0, routes=0, max_flip_gap=0.0)
    flips = []
    for k, r in enumerate(sample_rows):
        z_o = res[k]["logits"]
        lp_o = O.log_softmax(z_o)
        emitted = [got[r][0]] + [int(st[0][k]) for st in steps]
        z_g = [got[r][2]] + [st[2][k] for st in steps]
        lp_g = [got[r][1]] + [float(st[1][k]) for st in steps]
        for p in range(n_steps + 1):
            stats["dlogit"] = max(stats["dlogit"], float(np.abs(z_g[p] - z_o[p]).max()))
            stats["dlogprob"] = max(stats["dlogprob"], abs(lp_g[p] - float(lp_o[p, emitted[p]])))
            sc = z_o[p].astype(np.float64) + O.gumbel_noise(int(wl.seeds[r]), int(plen[r]) + p, shape.vocab)
            assert sc[emitted[p]] >= sc.max() - 2 * LOGIT_BAR, "row %d step %d: bad draw" % (r, p)
        own, gaps = res[k]["own_routing"], res[k]["gate_gap"]
        bad = (np.sort(replay[k], -1) != np.sort(own, -1)).any(-1)
        stats["routes"] += bad.size
        stats["tie_flips"] += int(bad.sum())
        if bad.any():
            stats["max_flip_gap"] = max(stats["max_flip_gap"], float(gaps[bad].max()))
            tok, lay = np.nonzero(bad)
            say("row %d: expert sets differ at (position, layer, oracle gap): %s" % (
                r, sorted([(int(t), int(l), float("%.2e" % gaps[t, l])) for t, l in zip(tok, lay)], key=lambda x: -x[2])[:40]))
        flips.append((gaps[bad], np.nonzero(bad)[1]))
        # full ordered lists wherever no two chosen logits are closer than the tie gap
        ordered = ~bad & (res[k]["order_gap"] >= TIE_GAP)
        n_order = int((replay[k][ordered] != own[ordered]).any(-1).sum())
        say("row %d: ordered lists compared at %d (position, layer) pairs, %d differ" % (r, int(ordered.sum()), n_order))
    say("FULL DEPTH %s, 48 layers, batch 128: sampled-row stats %s" % (shape.name, stats))
    allgaps = np.concatenate([g for g, _ in flips])
    say("gap quantiles of the differing sets: %s; by layer: %s" % (
        np.round(np.quantile(allgaps, [0.5, 0.9, 0.99, 1.0]), 5).tolist() if allgaps.size else [],
        np.bincount(np.concatenate([l for _, l in flips]), minlength=shape.n_layers).tolist()))
    # The 1e-3 tie rule is asserted where the oracle can resolve it: in the first two layers (as on the 2-layer
    # slice).  Deeper, the bf16 KV store turns differences of 1e-6 into differences of 1e-3 and more (the oracle in
    # float32 against itself in float64 shows the same: tests/test_oracle_kv_store_sensitivity.py), so over all 48
    # layers the expert sets may differ on at most 1 % of the (position, layer) pairs, nowhere at a gap of 1e-2 or
    # more; the logit and log-probability bars are asserted in full.
    alllay = np.concatenate([l for _, l in flips])
    assert (allgaps[alllay < 2] < TIE_GAP).all(), "routing differs in the first layers at gate gap %.2e" % float(
        allgaps[alllay < 2].max())
    assert (allgaps < 10 * TIE_GAP).all(), "routing differs at gate gap %.2e" % float(allgaps.max())
    assert stats["tie_flips"] <= 0.01 * stats["routes"]
    assert stats["dlogit"] <= LOGIT_BAR and stats["dlogprob"] <= LOGPROB_BAR
    model.close()


def test_moe_30b_a3b_layer_slice_omni_agentic_turns():
    """The omni/agentic workload at the 30B-A3B per-layer shape (2-layer slice): sequences that start with
    1024..4096 injected embedding positions plus 256 ids, then turns of a 128-token tool chunk followed by sampled
    tokens, with the KV carried across turns.  The GPU samples freely; the sampled rows are then recomputed by the
    oracle's teacher-forced full forward over everything that entered the cache (replaying the GPU's routing), and
    every emitted token, log-probability and logit row is compared."""
    import paper_2604_11554_amd as pkg
    from paper_2604_11554_amd import synthetic
    pkg.binding.lib()
    shape = RI.QWEN3_30B_A3B.replace(name="qwen3_30b_a3b_shape_2layers", n_layers=2)
    n_turns, n_decode, batch, budget = 2, 3, 6, 8192
    wl = RI.workload_omni_agentic(shape, batch=batch, n_turns=n_turns, turn_decode=n_decode)
    plen = [len(t) for t in wl.prompt_tokens]
    sample_rows = [int(r) for r in np.argsort(plen)[:2]]     # the oracle's attention cost grows with length squared
    say("omni/agentic: prompts of %s positions, sampled rows %s" % (plen, sample_rows))
    tensors = synthetic.generate_tensors(shape, 0, threads=12, progress=lambda i, n: say("  tensor %d/%d" % (i, n)))
    model = synthetic.model_from_tensors(shape, tensors, activation_split=1)
    total = [p + n_turns * (128 + n_decode) + 8 for p in plen]
    eng = pkg.RolloutEngine(model, n_blocks=sum((t + 31) // 16 for t in total) + 8, max_seqs=batch,
                            max_chunk_tokens=budget, max_blocks_per_seq=(max(total) + 31) // 16 + 1)
    rows = [eng.add_sequence(int(wl.seeds[i]), 1.0, reserve_tokens=total[i]) for i in range(batch)]
    fed = {r: [] for r in sample_rows}           # what entered the cache: (token ids, routing rows)
    checks = {r: [] for r in sample_rows}        # (position whose logits predict it, emitted token, logprob, logits)

    def prefill(rows_, toks, embeds=None, sample=True):
        o = eng.prefill(rows_, toks, embeds, sample_last=[sample] * len(rows_), want_logits=sample, want_routing=True)
        torch.cuda.synchronize()
        offs = np.concatenate([[0], np.cumsum([len(t) for t in toks])])
        for k, r in enumerate(rows_):
            if r in fed:
                fed[r].append((np.asarray(toks[k], np.int32), o.routing[offs[k]:offs[k + 1]].cpu().numpy()))
                if sample:
                    n_in = sum(len(t) for t, _ in fed[r])
                    checks[r].append((n_in - 1, int(o.tokens[k]), float(o.logprobs[k]), o.logits[k].cpu().numpy()))
        return o

    i = 0
    while i < batch:                             # prompts, several sequences per chunk, nothing sampled
        j, tot = i, 0
        while j < batch and tot + plen[j] <= budget:
            tot += plen[j]; j += 1
        embeds = []
        for r in range(i, j):
            full = np.zeros((plen[r], shape.d_model), np.uint16)
            full[wl.prompt_tokens[r] < 0] = wl.prompt_embeds[r]
            embeds.append(full)
        prefill(list(range(i, j)), wl.prompt_tokens[i:j], embeds, sample=False)
        say("prompt chunk: rows %d..%d (%d positions)" % (i, j - 1, tot))
        i = j
    for turn in range(n_turns):
        prefill(rows, [wl.turns[r][turn].tool_tokens for r in range(batch)])
        for s in range(n_decode):                # feeds the previous token, emits the next
            prev = eng.tokens[:batch].cpu().numpy().copy()
            o = eng.decode_step(want_logits=True, want_routing=True)
            torch.cuda.synchronize()
            for r in sample_rows:
                fed[r].append((prev[r:r + 1].astype(np.int32), o.routing[r:r + 1].cpu().numpy()))
                n_in = sum(len(t) for t, _ in fed[r])
                checks[r].append((n_in - 1, int(o.tokens[r]), float(o.logprobs[r]), o.logits[r].cpu().numpy()))
        say("turn %d done" % turn)
    assert not eng.finished[:batch].any()
    assert eng.ctx_lens[:batch].cpu().tolist() == [p + n_turns * (128 + n_decode) for p in plen]

    om = O.OracleModel(shape, 0, cache_layers=False, tensors=tensors)
    seqs = [np.concatenate([t for t, _ in fed[r]]) for r in sample_rows]
    replay = [np.concatenate([rt for _, rt in fed[r]], axis=0) for r in sample_rows]
    at = [np.array([c[0] for c in checks[r]]) for r in sample_rows]
    say("oracle forward of the sampled sequences (%s positions)" % [len(s) for s in seqs])
    res = O.forward_full(om, seqs, embeds=[wl.prompt_embeds[r] for r in sample_rows], forced_routing=replay,
                         logits_at=at, progress=lambda l: say("  oracle layer %d" % l))
    stats = dict(dlogit=0.0, dlogprob=0.0, tie_flips=0, routes=0)
    for k, r in enumerate(sample_rows):
        z_o = res[k]["logits"]
        lp_o = O.log_softmax(z_o)
        for p, (pos, tok, lp, z_g) in enumerate(checks[r]):
            stats["dlogit"] = max(stats["dlogit"], float(np.abs(z_g - z_o[p]).max()))
            stats["dlogprob"] = max(stats["dlogprob"], abs(lp - float(lp_o[p, tok])))
            sc = z_o[p].astype(np.float64) + O.gumbel_noise(int(wl.seeds[r]), pos + 1, shape.vocab)
            assert sc[tok] >= sc.max() - 2 * LOGIT_BAR, "row %d check %d: bad draw" % (r, p)
        bad = (np.sort(replay[k], -1) != np.sort(res[k]["own_routing"], -1)).any(-1)
        stats["routes"] += bad.size
        stats["tie_flips"] += int(bad.sum())
        assert (res[k]["gate_gap"][bad] < TIE_GAP).all(), "routing differs at gate gap %.2e" % float(
            res[k]["gate_gap"][bad].max())
    say("omni/agentic sampled-row stats %s" % stats)
    assert stats["dlogit"] <= LOGIT_BAR and stats["dlogprob"] <= LOGPROB_BAR
    model.close()
