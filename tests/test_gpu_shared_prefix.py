"""GPU parity of decode attention over shared prompt prefixes (rollout_decode_step_shared): sampling groups whose
members list the same pages for their prompt (the G responses per prompt of the group-relative algorithms, paper
Sec. 2.1) against the oracle, which attends to every sequence on its own.  The prefix tiles, the per-sequence
kernel starting after the shared units and the merge must reproduce plain attention: bars as for the rollout, and
the shared and unshared GPU paths must agree to merge-order rounding."""
import sys

import numpy as np
import pytest
import torch

import oracle as O
import rollout_inputs as RI

pytestmark = pytest.mark.gpu

LOGIT_BAR, LOGPROB_BAR, TIE_GAP = 0.05, 0.02, 1e-3
COMPACT_AT = 9
# (prompt length, members): 4 and 8 shared pages, 2 shared pages (one unit), 1 shared page (nothing to share),
# then two sequences on their own; 40 steps
SHORT = ([(75, 5), (130, 3), (33, 2), (20, 2), (50, 1), (9, 1)], 40)
# prefixes of 19 and 9 units: several chunks per subgroup (a chunk is at least eight units); 12 steps.  (More than
# one subgroup per group: the five members plus donor of SHORT at the MoE shape's four members per tile.)
LONG = ([(620, 3), (300, 2), (40, 1)], 12)


def say(msg):
    print("[gpu-case] " + msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def amd():
    import paper_2604_11554_amd as pkg
    from paper_2604_11554_amd import synthetic
    pkg.binding.lib()            # fail loudly if the library is not built
    return pkg, synthetic


def _prompts(shape, GROUPS):
    g = np.random.default_rng(5)
    return [g.integers(0, shape.vocab - 2, size=n).astype(np.int32) for n, _ in GROUPS]


def _oracle(shape, prompts, forced, replay, GROUPS, N_STEPS):
    """One oracle sequence per group member (no sharing); returns per step the result dict."""
    om = O.OracleModel(shape, 0)
    n = sum(m for _, m in GROUPS)
    ro = O.OracleRollout(om, n_blocks=n * ((max(p for p, _ in GROUPS) + N_STEPS) // 16 + 2))
    ids, toks = [], []
    for gi, (_, mem) in enumerate(GROUPS):
        for k in range(mem):
            ids.append(ro.add_sequence(900 + 10 * gi + k))
            toks.append(prompts[gi])
    f = (lambda s: None) if forced is None else (lambda s: forced[s])
    r = (lambda s: None) if replay is None else (lambda s: replay[s])
    steps = [ro.prefill_chunk(ids, toks, forced_tokens=f(0), forced_routing=r(0), want_logits=True)]
    for s in range(1, N_STEPS):
        steps.append(ro.decode_step(ids, forced_tokens=f(s), forced_routing=r(s), want_logits=True))
    return steps


def _gpu(pkg, synthetic, shape, prompts, forced, share, GROUPS, N_STEPS):
    """Donor row per group (prompt minus its last token, never sampled), members forked from it; donors are dropped
    by a compaction after COMPACT_AT steps.  Returns per step (logits, logprobs, routing) in member order."""
    model = synthetic.model_from_shape(shape, 0, activation_split=1)
    n_rows = sum(m + (1 if m > 1 else 0) for _, m in GROUPS)
    mb = (max(p for p, _ in GROUPS) + N_STEPS) // 16 + 2
    eng = pkg.RolloutEngine(model, n_blocks=n_rows * mb, max_seqs=n_rows, max_chunk_tokens=1024, max_blocks_per_seq=mb)
    eng.share_prefix_attention = share
    member_rows, donors, donor_rt = [], [], []
    for gi, (plen, mem) in enumerate(GROUPS):
        if mem == 1:
            member_rows.append(eng.add_sequence(900 + 10 * gi, reserve_tokens=plen + N_STEPS))
            donor_rt.append(None)
            continue
        d = eng.add_sequence(0, reserve_tokens=plen)
        o = eng.prefill([d], [prompts[gi][:-1]], sample_last=[False], want_routing=True)
        donors.append(d)
        for k in range(mem):
            member_rows.append(eng.fork(d, 900 + 10 * gi + k, reserve_tokens=plen + N_STEPS))
            donor_rt.append(None if o.routing is None else o.routing.cpu().numpy())
    for d in donors:
        eng.tokens[d] = shape.pad_token_id
        eng.finished[d] = 1                                    # a donor takes no part in decoding
    toks = [prompts[gi] if mem == 1 else prompts[gi][-1:] for gi, (_, mem) in enumerate(GROUPS) for _ in range(mem)]
    out = eng.prefill(member_rows, toks, forced=forced[0], want_logits=True, want_routing=True)
    torch.cuda.synchronize()
    offs = np.concatenate([[0], np.cumsum([len(t) for t in toks])])
    rt = None if out.routing is None else out.routing.cpu().numpy()
    # a member's prompt routing = the donor's rows for all but the last prompt position, then its own row
    steps = [(out.logits.cpu().numpy(), out.logprobs.cpu().numpy(),
              None if rt is None else [rt[offs[j]:offs[j + 1]] if donor_rt[j] is None else
                                       np.concatenate([donor_rt[j], rt[offs[j]:offs[j + 1]]], 0) for j in range(len(toks))])]
    idx = torch.tensor(member_rows, device="cuda:0")
    n_tiles = []
    for s in range(1, N_STEPS):
        if s == COMPACT_AT:
            keep = eng.compact()                               # drops the donors; groups are led by their first member
            pos = {int(old): new for new, old in enumerate(keep)}
            member_rows = [pos[r] for r in member_rows]
            idx = torch.tensor(member_rows, device="cuda:0")
        ft = torch.full((eng.n,), -1, dtype=torch.int32, device="cuda:0")
        ft[idx] = torch.tensor(forced[s], dtype=torch.int32, device="cuda:0")
        out = eng.decode_step(forced=ft, want_logits=True, want_routing=True)
        torch.cuda.synchronize()
        desc = eng._shared_prefix()
        n_tiles.append(0 if desc is None else int(desc[:8].view(torch.int32)[1].item()))
        rt = None if out.routing is None else out.routing[idx].cpu().numpy()
        steps.append((out.logits[idx].cpu().numpy(), out.logprobs[idx].cpu().numpy(),
                      None if rt is None else [rt[j][None] for j in range(len(member_rows))]))
    model.close()
    return steps, n_tiles


@pytest.mark.parametrize("shape_name,case", [("tiny_dense", "short"), ("tiny_moe", "short"), ("tiny_dense", "long"),
                                             ("tiny_moe", "long")])
def test_group_decode_over_shared_prefix_matches_oracle(amd, shape_name, case):
    pkg, synthetic = amd
    shape = {"tiny_dense": RI.TINY_DENSE, "tiny_moe": RI.TINY_MOE}[shape_name]
    GROUPS, N_STEPS = SHORT if case == "short" else LONG
    prompts = _prompts(shape, GROUPS)
    say("%s %s: oracle free run, one sequence per member" % (shape.name, case))
    osteps = _oracle(shape, prompts, None, None, GROUPS, N_STEPS)
    forced = [st["tokens"] for st in osteps]
    say("%s: gpu with prefix tiles" % shape.name)
    gs, tiles = _gpu(pkg, synthetic, shape, prompts, forced, True, GROUPS, N_STEPS)
    say("%s: gpu without" % shape.name)
    gu, tiles_u = _gpu(pkg, synthetic, shape, prompts, forced, False, GROUPS, N_STEPS)
    ms = min(16, 32 // (shape.n_q_heads // shape.n_kv_heads))
    # tiles = subgroups x chunks x KV heads over the groups that share at least one unit (donor included until the
    # compaction); a chunk holds at least eight units and a subgroup has at most ms members
    def n_tiles(extra):
        n = 0
        for p, m in GROUPS:
            units = ((p - 1) // 16) // 2
            if m > 1 and units > 0:
                n += ((m + extra + ms - 1) // ms) * min(4, (units + 7) // 8) * shape.n_kv_heads
        return n
    assert tiles[0] == n_tiles(1) and tiles[-1] == n_tiles(0), (tiles[0], tiles[-1], n_tiles(1), n_tiles(0))
    assert set(tiles_u) == {0}
    d_paths = max(float(np.abs(a[0] - b[0]).max()) for a, b in zip(gs, gu))
    say("%s: prefix tiles per step %d -> %d; shared vs unshared max |dlogit| %.2e" % (shape.name, tiles[0], tiles[-1], d_paths))
    assert d_paths <= 2e-3                                      # the order of the softmax merges is all that differs
    if shape.is_moe:   # replay the GPU's routing so that a tolerated near-tie does not hide what follows
        osteps = _oracle(shape, prompts, forced, [g[2] for g in gs], GROUPS, N_STEPS)
        flips = routes = 0
        for g, o in zip(gs, osteps):
            for j in range(len(g[2])):
                bad = (np.sort(g[2][j], -1) != np.sort(o["own_routing"][j], -1)).any(-1)
                flips += int(bad.sum())
                routes += bad.size
                assert (o["gate_gap"][j][bad] < TIE_GAP).all()
        say("%s: %d near-tie routing differences in %d routed (token, layer) pairs" % (shape.name, flips, routes))
    dl = dp = 0.0
    for s, (g, o) in enumerate(zip(gs, osteps)):
        for j in range(len(o["tokens"])):
            dl = max(dl, float(np.abs(g[0][j] - o["logits"][j]).max()))
            dp = max(dp, abs(float(g[1][j]) - o["logprobs"][j]))
    say("%s: against the oracle max |dlogit| %.5f, max |dlogprob| %.5f over %d steps" % (shape.name, dl, dp, N_STEPS))
    assert dl <= LOGIT_BAR and dp <= LOGPROB_BAR


def test_descriptor_of_another_batch_size_is_ignored(amd):
    """A descriptor built for a different number of rows must not be applied: the step then equals the plain one."""
    pkg, synthetic = amd
    B = pkg.binding
    shape = RI.TINY_DENSE
    prompt = _prompts(shape, SHORT[0])[0]
    outs = []
    for stale in (False, True):
        model = synthetic.model_from_shape(shape, 0, activation_split=1)
        eng = pkg.RolloutEngine(model, n_blocks=64, max_seqs=8, max_chunk_tokens=256, max_blocks_per_seq=12)
        d = eng.add_sequence(0, reserve_tokens=len(prompt))
        eng.prefill([d], [prompt[:-1]], sample_last=[False])
        kids = [eng.fork(d, 40 + k, reserve_tokens=len(prompt) + 8) for k in range(3)]
        eng.finished[d] = 1
        eng.prefill(kids, [prompt[-1:]] * 3)
        eng.share_prefix_attention = False
        if stale:   # a descriptor for 6 rows that claims four shared pages for everyone, passed to a 4-row step
            desc = torch.empty(B.rlx_shared_prefix_bytes(model.handle, 6), dtype=torch.uint8, device="cuda:0")
            B.rlx_shared_prefix_build(model.handle, [0] * 6, [4] * 6, desc)
            eng._shared_prefix = lambda: desc
        z = []
        for _ in range(3):
            z.append(eng.decode_step(want_logits=True).logits.cpu().numpy().copy())
        outs.append(np.stack(z))
        model.close()
    np.testing.assert_array_equal(outs[0], outs[1])


def test_slot_refilled_inside_a_group_leaves_the_group(amd):
    """release_slot / refill_slot on a row that shares prompt pages with its sampling group: the row gets pages of
    its own, so it must stop claiming the group's pages (the descriptor of the next step is rebuilt without it and
    the rows after it form a group of their own).  The refilled row then decodes a different prompt; every row is
    compared with an engine that never shared anything."""
    pkg, synthetic = amd
    shape = RI.TINY_DENSE
    g = np.random.default_rng(5)
    prompt = g.integers(0, shape.vocab - 2, size=70).astype(np.int32)
    other = g.integers(0, shape.vocab - 2, size=45).astype(np.int32)

    def run(shared):
        model = synthetic.model_from_shape(shape, 0, activation_split=1)
        eng = pkg.RolloutEngine(model, n_blocks=96, max_seqs=8, max_chunk_tokens=512, max_blocks_per_seq=12)
        if shared:
            d = eng.add_sequence(0, reserve_tokens=len(prompt))
            eng.prefill([d], [prompt[:-1]], sample_last=[False])
            kids = [eng.fork(d, 60 + k, reserve_tokens=len(prompt) + 12) for k in range(4)]
            eng.finished[d] = 1
            eng.prefill(kids, [prompt[-1:]] * 4)
        else:
            d = eng.add_sequence(0, reserve_tokens=8)
            eng.finished[d] = 1
            kids = [eng.add_sequence(60 + k, reserve_tokens=len(prompt) + 12) for k in range(4)]
            eng.prefill(kids, [prompt] * 4)
        z = []
        for _ in range(2):
            z.append(eng.decode_step(want_logits=True).logits.cpu().numpy()[1:5].copy())
        assert (eng._shared_prefix() is not None) == shared
        # the second member ends; its row is refilled with another request
        row = kids[1]
        assert eng.refill_slot(row, 99, 1.0, len(other) + 12)
        if shared:
            assert eng.leader[row] == row and eng.shared_pages[row] == 0
            assert eng.leader[kids[0]] == d and eng.leader[kids[2]] == kids[2] and eng.leader[kids[3]] == kids[2]
        eng.prefill([row], [other])
        for _ in range(3):
            z.append(eng.decode_step(want_logits=True).logits.cpu().numpy()[1:5].copy())
        model.close()
        return np.stack(z)

    a, b = run(True), run(False)
    assert np.abs(a - b).max() <= 2e-3, float(np.abs(a - b).max())     # summation order of the softmax merges only


def test_shared_prefix_descriptor_validation(amd):
    pkg, synthetic = amd
    B = pkg.binding
    model = synthetic.model_from_shape(RI.TINY_DENSE, 0, activation_split=1)
    desc = torch.empty(B.rlx_shared_prefix_bytes(model.handle, 4), dtype=torch.uint8, device="cuda:0")
    B.rlx_shared_prefix_build(model.handle, [0, 0, 0, 3], [4, 4, 5, 0], desc)
    hdr = desc[:32].view(torch.int32).cpu().numpy()
    assert hdr[0] == 4 and hdr[2] == 16 and hdr[1] == 2          # one subgroup, one chunk of two units, two KV heads
    start = desc[32:48].view(torch.int32).cpu().numpy()
    assert list(start) == [2, 2, 2, 0]
    for leader, pages in (([0, 2, 0, 3], [4, 4, 4, 0]), ([0, 0, 0, 3], [4, -1, 4, 0]), ([1, 0, 0, 3], [4, 4, 4, 0])):
        with pytest.raises(B.RlxError) as e:
            B.rlx_shared_prefix_build(model.handle, leader, pages, desc)
        assert e.value.code == B.RLX_EINVAL
    with pytest.raises(B.RlxError) as e:
        B.rlx_shared_prefix_build(model.handle, [0, 0, 0, 3], [4, 4, 5, 0], desc[:64])
    assert e.value.code == B.RLX_ENOMEM
    model.close()
