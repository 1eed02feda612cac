"""GPU parity of the teacher-forced scoring entry point (rollout_score_chunk) against the oracle's full
forward: per-position log-probabilities of given targets, with and without routing replay (paper Sec. 3.3,
5.5).  Bars as for the rollout: max |dlogprob| <= 0.02; replayed routing is echoed bit-exactly."""
import sys

import numpy as np
import pytest
import torch
from scipy.special import log_softmax

import oracle as O
import rollout_inputs as RI

pytestmark = pytest.mark.gpu

LOGPROB_BAR = 0.02
TIE_GAP = 1e-3
LENS = (5, 33, 70, 300, 17)                 # 300 tokens: more than one 256-row LM-head block per call
TEMPS = (1.0, 0.7, 1.0, 1.3, 1.0)


def say(msg):
    print("[gpu-case] " + msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def amd():
    import paper_2604_11554_amd as pkg
    from paper_2604_11554_amd import synthetic
    pkg.binding.lib()            # fail loudly if the library is not built
    return pkg, synthetic


def _sequences(shape, seed):
    g = np.random.default_rng(seed)
    return [g.integers(0, shape.vocab - 2, size=n).astype(np.int32) for n in LENS]


def _targets(toks):
    return [np.concatenate([t[1:], [-1]]).astype(np.int32) for t in toks]


def _oracle_logprobs(res, toks):
    out = []
    for r, t, temp in zip(res, toks, TEMPS):
        lp = log_softmax(r["logits"].astype(np.float64) / temp, axis=-1)
        out.append(np.concatenate([lp[np.arange(len(t) - 1), t[1:]], [0.0]]))
    return out


def _engine(pkg, synthetic, shape):
    model = synthetic.model_from_shape(shape, 0, activation_split=1)
    eng = pkg.RolloutEngine(model, n_blocks=len(LENS) * 24, max_seqs=8, max_chunk_tokens=sum(LENS),
                            max_blocks_per_seq=24)
    for i, temp in enumerate(TEMPS):
        eng.add_sequence(100 + i, temperature=temp, reserve_tokens=max(LENS) + 16)
    return model, eng


def _split(lp, lens):
    o = np.concatenate([[0], np.cumsum(lens)])
    lp = lp.cpu().numpy()
    return [lp[o[i]:o[i + 1]] for i in range(len(lens))]


@pytest.mark.parametrize("shape_name", ["tiny_dense_qkn", "tiny_moe"])
def test_score_matches_oracle_forward(amd, shape_name):
    pkg, synthetic = amd
    shape = RI.TINY_MOE if shape_name == "tiny_moe" else RI.TINY_DENSE.replace(qk_norm=True, name="tiny_dense_qkn")
    toks = _sequences(shape, 11)
    tg = _targets(toks)
    omodel = O.OracleModel(shape, 0)
    say("%s: oracle forward" % shape.name)
    ores = O.forward_full(omodel, toks)
    olp = _oracle_logprobs(ores, toks)

    model, eng = _engine(pkg, synthetic, shape)
    rows = list(range(len(toks)))
    # replaying the oracle's own expert choice removes the near-tie freedom of the router
    replay = [r["routing"] for r in ores] if shape.is_moe else None
    lp, routing = eng.score(rows, toks, tg, replay_routing=replay, want_routing=True)
    torch.cuda.synchronize()
    glp = _split(lp, LENS)
    worst = max(float(np.abs(a - b).max()) for a, b in zip(glp, olp))
    say("%s: max |dlogprob| over %d positions = %.4f" % (shape.name, sum(LENS), worst))
    assert worst <= LOGPROB_BAR
    for a in glp:
        assert a[-1] == 0.0                       # target -1: not scored
    if shape.is_moe:
        np.testing.assert_array_equal(routing.cpu().numpy(), np.concatenate(replay))
    assert list(eng.ctx_lens[:len(LENS)].cpu().numpy()) == list(LENS)
    model.close()

    # chunked scoring (two calls per row, the second over the cached prefix) gives the same numbers
    model, eng = _engine(pkg, synthetic, shape)
    cut = [max(1, n // 2) for n in LENS]
    lp1, _ = eng.score(rows, [t[:c] for t, c in zip(toks, cut)], [x[:c] for x, c in zip(tg, cut)],
                       replay_routing=None if replay is None else [r[:c] for r, c in zip(replay, cut)])
    keep = [i for i in rows if cut[i] < LENS[i]]
    lp2, _ = eng.score(keep, [toks[i][cut[i]:] for i in keep], [tg[i][cut[i]:] for i in keep],
                       replay_routing=None if replay is None else [replay[i][cut[i]:] for i in keep])
    torch.cuda.synchronize()
    a1 = _split(lp1, cut)
    a2 = dict(zip(keep, _split(lp2, [LENS[i] - cut[i] for i in keep])))
    for i in rows:
        whole = np.concatenate([a1[i], a2[i]]) if i in a2 else a1[i]
        assert np.abs(whole - glp[i]).max() <= 2e-3      # chunking changes summation order only
    model.close()


def test_score_with_foreign_routing_replay(amd):
    """Replay of a routing record that is NOT the router's own choice: experts are taken from the record, mixing
    weights from the layer's own gate probabilities renormalised over the record (the oracle's replay mode)."""
    pkg, synthetic = amd
    shape = RI.TINY_MOE
    toks = _sequences(shape, 12)
    tg = _targets(toks)
    omodel = O.OracleModel(shape, 0)
    own = O.forward_full(omodel, toks)
    # every chosen expert is replaced by another one (a fixed shift keeps the ids of a token distinct)
    foreign = [((r["routing"] + 5) % shape.n_experts).astype(np.int32) for r in own]
    say("oracle forward replaying a foreign routing record")
    ores = O.forward_full(omodel, toks, forced_routing=foreign)
    olp = _oracle_logprobs(ores, toks)
    own_lp = _oracle_logprobs(own, toks)
    assert max(float(np.abs(a - b).max()) for a, b in zip(olp, own_lp)) > 3 * LOGPROB_BAR    # the record matters

    model, eng = _engine(pkg, synthetic, shape)
    lp, routing = eng.score(list(range(len(toks))), toks, tg, replay_routing=foreign, want_routing=True)
    torch.cuda.synchronize()
    glp = _split(lp, LENS)
    worst = max(float(np.abs(a - b).max()) for a, b in zip(glp, olp))
    say("foreign replay: max |dlogprob| = %.4f" % worst)
    assert worst <= LOGPROB_BAR
    np.testing.assert_array_equal(routing.cpu().numpy(), np.concatenate(foreign))
    model.close()


def test_replay_that_sends_every_token_to_the_same_experts(amd):
    """A short call (64 tokens: the expert GEMMs take their decode form and the gate/up kernel groups the pairs
    itself) whose routing record names the same eight experts for every token: each of them receives 64 rows, two
    32-row tiles, and the other experts none.  Compared with the oracle replaying the same record; the record is
    echoed bit for bit."""
    pkg, synthetic = amd
    shape = RI.TINY_MOE
    lens = (40, 24)
    g = np.random.default_rng(21)
    toks = [g.integers(0, shape.vocab - 2, size=n).astype(np.int32) for n in lens]
    tg = _targets(toks)
    omodel = O.OracleModel(shape, 0)
    fixed = (np.arange(shape.top_k) * 3 + 1) % shape.n_experts        # eight distinct experts
    rec = [np.broadcast_to(fixed.astype(np.int32), (n, shape.n_layers, shape.top_k)).copy() for n in lens]
    rec[1][:, 1] = (fixed[::-1] + 1) % shape.n_experts                # another set, in another order, for one layer
    ores = O.forward_full(omodel, toks, forced_routing=rec)
    olp = []
    for r, t in zip(ores, toks):
        lp = log_softmax(r["logits"].astype(np.float64), axis=-1)
        olp.append(np.concatenate([lp[np.arange(len(t) - 1), t[1:]], [0.0]]))
    model = synthetic.model_from_shape(shape, 0, activation_split=1)
    eng = pkg.RolloutEngine(model, n_blocks=16, max_seqs=4, max_chunk_tokens=sum(lens), max_blocks_per_seq=8)
    for i in range(len(lens)):
        eng.add_sequence(300 + i, temperature=1.0, reserve_tokens=max(lens) + 16)
    lp, routing = eng.score([0, 1], toks, tg, replay_routing=rec, want_routing=True)
    torch.cuda.synchronize()
    glp = _split(lp, lens)
    worst = max(float(np.abs(a - b).max()) for a, b in zip(glp, olp))
    say("one expert set for all %d tokens: max |dlogprob| = %.4f" % (sum(lens), worst))
    assert worst <= LOGPROB_BAR
    np.testing.assert_array_equal(routing.cpu().numpy(), np.concatenate(rec))
    model.close()


def test_replay_table_with_repeated_and_invalid_ids(amd):
    """A defective routing record (an expert listed twice for a token, ids outside the experts): every such slot
    falls back to the layer's own best expert not yet in the token's list, so that no expert receives a token twice
    (the grouped GEMMs hold at most one row per token and expert).  Checked: the experts used are distinct and equal
    the record wherever the record was usable; each replaced slot holds the best expert, by the oracle's own router
    order, among those the token had not taken by then; the log-probabilities equal the oracle's when it replays
    the experts actually used."""
    pkg, synthetic = amd
    shape = RI.TINY_MOE
    toks = _sequences(shape, 12)
    tg = _targets(toks)
    omodel = O.OracleModel(shape, 0)
    own = O.forward_full(omodel, toks)
    rec = [((r["routing"] + 5) % shape.n_experts).astype(np.int32) for r in own]
    g = np.random.default_rng(3)
    planted = 0
    for r in rec:                                   # plant defects in a tenth of the (position, layer) lists
        for t, l in zip(*np.nonzero(g.random(r.shape[:2]) < 0.1)):
            kind = g.integers(0, 3)
            if kind == 0:
                r[t, l, g.integers(1, shape.top_k)] = r[t, l, 0]             # a repeat of the first id
            elif kind == 1:
                r[t, l, g.integers(0, shape.top_k)] = shape.n_experts + 3    # past the last expert
            else:
                r[t, l, 2] = -1; r[t, l, 5] = r[t, l, 4]                     # a negative id and a repeat
            planted += 1
    model, eng = _engine(pkg, synthetic, shape)
    lp, routing = eng.score(list(range(len(toks))), toks, tg, replay_routing=rec, want_routing=True)
    torch.cuda.synchronize()
    used = np.split(routing.cpu().numpy(), np.cumsum(LENS)[:-1])
    ores = O.forward_full(omodel, toks, forced_routing=used)
    n_fallback = 0
    for u, r, o in zip(used, rec, ores):
        assert ((u >= 0) & (u < shape.n_experts)).all()
        assert (np.sort(u, -1)[..., 1:] != np.sort(u, -1)[..., :-1]).all()      # distinct experts per token
        for t in range(u.shape[0]):
            for l in range(u.shape[1]):
                taken = []
                for k in range(shape.top_k):
                    want = int(r[t, l, k])
                    if 0 <= want < shape.n_experts and want not in taken:
                        assert u[t, l, k] == want
                    else:                           # the oracle's own order, first expert not yet taken ...
                        best = [e for e in o["own_routing"][t, l] if e not in taken]
                        n_fallback += 1
                        # ... unless the token's list already holds all of its own eight, or a near-tie decides
                        if best and o["order_gap"][t, l] >= TIE_GAP and o["gate_gap"][t, l] >= TIE_GAP:
                            assert u[t, l, k] == best[0], (t, l, k, u[t, l], r[t, l], o["own_routing"][t, l])
                    taken.append(int(u[t, l, k]))
    glp, olp = _split(lp, LENS), _oracle_logprobs(ores, toks)
    worst = max(float(np.abs(a - b).max()) for a, b in zip(glp, olp))
    say("defective replay table: %d lists with planted defects, %d slots fell back, max |dlogprob| = %.4f" % (
        planted, n_fallback, worst))
    assert n_fallback >= planted and worst <= LOGPROB_BAR
    model.close()


def test_rollout_then_score_reproduces_rollout_logprobs(amd):
    """The paper's consistency loop on our own path: generate with routing capture, then score the generated
    tokens replaying the captured routing; the scored log-probabilities equal the ones the rollout reported."""
    pkg, synthetic = amd
    shape = RI.TINY_MOE
    wl = RI.workload_tiny(shape, n_decode=12, seed_base=7000)
    model = synthetic.model_from_shape(shape, 0, activation_split=1)
    B = wl.batch
    eng = pkg.RolloutEngine(model, n_blocks=2 * B * 8, max_seqs=2 * B, max_chunk_tokens=int(wl.prompt_lens.sum()) + 64,
                            max_blocks_per_seq=8)
    for i in range(B):
        eng.add_sequence(int(wl.seeds[i]), reserve_tokens=int(wl.prompt_lens[i]) + 16)
    out = eng.prefill(list(range(B)), wl.prompt_tokens, want_routing=True)
    gen = [[int(t)] for t in out.tokens.cpu().numpy()]
    lps = [[float(x)] for x in out.logprobs.cpu().numpy()]
    o = np.concatenate([[0], np.cumsum(wl.prompt_lens)])
    r0 = out.routing.cpu().numpy()
    rout = [[r0[o[i]:o[i + 1]]] for i in range(B)]
    for s in range(1, 12):
        out = eng.decode_step(want_routing=True)
        tk, lp, rr = out.tokens.cpu().numpy(), out.logprobs.cpu().numpy(), out.routing.cpu().numpy()
        for i in range(B):
            gen[i].append(int(tk[i])); lps[i].append(float(lp[i])); rout[i].append(rr[i][None])
    # score prompt + generated tokens (the last generated token is a target only) on fresh rows of the same engine
    rows = []
    for i in range(B):
        rows.append(eng.add_sequence(0, reserve_tokens=int(wl.prompt_lens[i]) + 16))
    toks = [np.concatenate([wl.prompt_tokens[i], gen[i][:-1]]).astype(np.int32) for i in range(B)]
    tg = []
    for i in range(B):
        t = np.full(len(toks[i]), -1, np.int32)
        t[len(wl.prompt_tokens[i]) - 1:] = gen[i]
        tg.append(t)
    replay = [np.concatenate(rout[i])[:len(toks[i])] for i in range(B)]
    lp, _ = eng.score(rows, toks, tg, replay_routing=replay)
    torch.cuda.synchronize()
    got = _split(lp, [len(t) for t in toks])
    worst = 0.0
    for i in range(B):
        worst = max(worst, float(np.abs(got[i][len(wl.prompt_tokens[i]) - 1:] - np.array(lps[i])).max()))
    say("rollout vs replayed scoring: max |dlogprob| = %.5f over %d tokens" % (worst, 12 * B))
    assert worst <= 5e-3          # same kernels, different batching and summation order
    model.close()


def test_workspace_size_covers_every_smaller_call(amd):
    """Calls of at most 256 tokens keep split-K planes per token, longer ones do not: the size reported for a
    large call must still cover every smaller call."""
    pkg, synthetic = amd
    B = pkg.binding
    model = synthetic.model_from_shape(RI.TINY_DENSE, 0, activation_split=1)
    big = B.rlx_workspace_bytes(model.handle, 8, 4096, 24)
    for t in (8, 100, 211, 256, 257, 1000, 4096):
        assert B.rlx_workspace_bytes(model.handle, min(8, t), t, 24) <= big
    model.close()
