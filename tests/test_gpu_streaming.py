"""GPU: streaming rollout with continuous refill (paper Sec. 3.3, "Streaming data flow") against the oracle.
Sequences enter and leave slots at different steps, so every decode step sees a different mix of live, inert and
freshly prefilled rows; each completed response is then checked by the oracle's teacher-forced full forward of
that sequence alone: per-token log-probabilities within the rollout bar, every emitted token the oracle's own
Gumbel-max draw (or within twice the logit bar of its best perturbed score), routing rows equal to the oracle's
own top-k except at near-ties."""
import sys

import numpy as np
import pytest

import oracle as O
import rollout_inputs as RI

pytestmark = pytest.mark.gpu

LOGIT_BAR, LOGPROB_BAR, TIE_GAP = 0.05, 0.02, 1e-3


def say(msg):
    print("[gpu-case] " + msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def amd():
    import paper_2604_11554_amd as pkg
    from paper_2604_11554_amd import synthetic
    pkg.binding.lib()            # fail loudly if the library is not built
    return pkg, synthetic


@pytest.mark.parametrize("shape_name", ["tiny_dense", "tiny_moe"])
def test_streaming_rollout_with_refill_matches_oracle(amd, shape_name):
    pkg, synthetic = amd
    shape = {"tiny_dense": RI.TINY_DENSE, "tiny_moe": RI.TINY_MOE}[shape_name]
    g = np.random.default_rng(11)
    n_req, slots = 14, 4
    reqs = [pkg.Request(g.integers(0, shape.vocab - 2, size=int(g.integers(5, 60))).astype(np.int32),
                        seed=7000 + i, temperature=float(g.choice([1.0, 0.8])), max_new_tokens=int(g.integers(1, 24)))
            for i in range(n_req)]
    model = synthetic.model_from_shape(shape, 0, activation_split=1)
    eng = pkg.RolloutEngine(model, n_blocks=slots * 8, max_seqs=slots, max_chunk_tokens=96, max_blocks_per_seq=8)
    events = []
    sr = pkg.StreamingRollout(eng, reqs, micro_batch=4, poll_every=3, want_routing=True,
                              on_partition=lambda p, cs: events.append((p, [c.index for c in cs])))
    done = sr.run()
    say("%s: %d requests through %d slots in %d decode steps, partitions reported in order %s" % (
        shape.name, n_req, slots, sr.decode_steps, sr.partition_order))
    assert [c.index for c in done] == list(range(n_req))
    assert sorted(p for p, _ in events) == [0, 1, 2, 3]
    for p, idx in events:
        assert idx == list(range(4 * p, min(4 * p + 4, n_req)))
    assert len(eng.free_blocks) == slots * 8                     # every page came back
    # fewer steps than running the requests one batch of `slots` after the other
    lens = [len(c.tokens) for c in done]
    serial = sum(max(lens[i:i + slots]) for i in range(0, n_req, slots))
    assert sr.decode_steps <= serial + 3 * len(range(0, n_req, slots))

    om = O.OracleModel(shape, 0)
    eos = shape.eos_token_id
    dlp = 0.0
    flips = routes = 0
    for c, rq in zip(done, reqs):
        n, p = len(c.tokens), len(rq.prompt)
        assert 1 <= n <= rq.max_new_tokens and (c.tokens[:-1] != eos).all()
        assert c.tokens[-1] == eos or n == rq.max_new_tokens
        if n == rq.max_new_tokens:
            assert c.tokens[-1] == eos                           # the token at the cap is a forced EOS
        seq = np.concatenate([rq.prompt, c.tokens[:-1]]).astype(np.int32)
        replay = [c.routing] if shape.is_moe else None
        res = O.forward_full(om, [seq], forced_routing=replay, logits_at=[np.arange(p - 1, p - 1 + n)])[0]
        z = res["logits"].astype(np.float64)
        lp = O.log_softmax(z / rq.temperature)
        for k in range(n):
            tok = int(c.tokens[k])
            forced = (k == rq.max_new_tokens - 1)
            dlp = max(dlp, abs(float(c.logprobs[k]) - float(lp[k, tok])))
            if not forced:
                sc = z[k] / rq.temperature + O.gumbel_noise(rq.seed, p + k, shape.vocab)
                assert sc[tok] >= sc.max() - 2 * LOGIT_BAR, "request %d token %d: not the oracle's draw" % (c.index, k)
        if shape.is_moe:
            assert c.routing.shape == (p + n - 1, shape.n_layers, shape.top_k)
            bad = (np.sort(c.routing, -1) != np.sort(res["own_routing"], -1)).any(-1)
            routes += bad.size
            flips += int(bad.sum())
            assert (res["gate_gap"][bad] < TIE_GAP).all()
    say("%s: max |dlogprob| %.5f over %d tokens; routing near-tie differences %d of %d" % (
        shape.name, dlp, sum(lens), flips, routes))
    assert dlp <= LOGPROB_BAR
    model.close()
