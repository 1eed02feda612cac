"""GPU parity of the weight refresh between steps (rlx_model_set_weights): a teacher-forced rollout whose weights
are replaced after a few decode steps, against the oracle doing the same (paper Sec. 3.2, weight synchronisation
to the inference engines; Sec. 3.3, the rollout-side weight version v_r and the staleness rule).  Sequences in
flight keep their KV pages across the refresh.  Bars as for the rollout."""
import sys

import numpy as np
import pytest
import torch

import oracle as O
import rollout_inputs as RI

pytestmark = pytest.mark.gpu

LOGIT_BAR, LOGPROB_BAR, TIE_GAP = 0.05, 0.02, 1e-3
N_DECODE, SWAP_AT = 12, 5


def say(msg):
    print("[gpu-case] " + msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def amd():
    import paper_2604_11554_amd as pkg
    from paper_2604_11554_amd import synthetic
    pkg.binding.lib()            # fail loudly if the library is not built
    return pkg, synthetic


def _oracle_steps(shape, wl, forced, replay):
    """Oracle rollout with weights of seed 0 for steps < SWAP_AT and of seed 1 afterwards."""
    a, b = O.OracleModel(shape, 0), O.OracleModel(shape, 1)
    ro = O.OracleRollout(a, n_blocks=sum((len(p) + N_DECODE + 16) // 16 + 1 for p in wl.prompt_tokens))
    ids = [ro.add_sequence(int(wl.seeds[i]), float(wl.temperature[i])) for i in range(wl.batch)]
    steps = []
    for s in range(N_DECODE):
        if s == SWAP_AT:
            ro.set_model(b, 3)
        f = None if forced is None else forced[s]
        r = None if replay is None else replay[s]
        if s == 0:
            st = ro.prefill_chunk(ids, wl.prompt_tokens, wl.prompt_embeds, forced_tokens=f, forced_routing=r,
                                  want_logits=True)
        else:
            st = ro.decode_step(ids, forced_tokens=f, forced_routing=r, want_logits=True)
        st["weight_version"] = ro.weight_version
        steps.append(st)
    return steps


@pytest.mark.parametrize("shape_name", ["tiny_dense", "tiny_moe"])
def test_weight_refresh_mid_rollout_matches_oracle(amd, shape_name):
    pkg, synthetic = amd
    shape = {"tiny_dense": RI.TINY_DENSE, "tiny_moe": RI.TINY_MOE}[shape_name]
    wl = RI.workload_tiny(shape, n_decode=N_DECODE)
    say("%s: oracle rollout with a refresh before step %d" % (shape.name, SWAP_AT))
    osteps = _oracle_steps(shape, wl, None, None)
    forced = [st["tokens"] for st in osteps]

    model = synthetic.model_from_shape(shape, 0, activation_split=1)
    mb = (int(wl.prompt_lens.max()) + N_DECODE + 15) // 16 + 1
    eng = pkg.RolloutEngine(model, n_blocks=wl.batch * mb, max_seqs=8, max_chunk_tokens=int(wl.prompt_lens.sum()),
                            max_blocks_per_seq=mb)
    rows = [eng.add_sequence(int(wl.seeds[i]), float(wl.temperature[i]),
                             reserve_tokens=len(wl.prompt_tokens[i]) + N_DECODE) for i in range(wl.batch)]
    assert model.weight_version == 0 and pkg.binding.rlx_model_weight_version(model.handle) == 0
    gsteps = []
    for s in range(N_DECODE):
        if s == SWAP_AT:
            # the staleness rule on the producer side: trainer at version 3, this engine still at 0
            assert eng.may_generate(trainer_version=3, max_staleness=4)
            assert not eng.may_generate(trainer_version=3, max_staleness=3)
            say("%s: refresh to the weights of seed 1 as version 3" % shape.name)
            model.update_weights(lambda l, n: RI.tensor_bf16(shape, 1, l, n), version=3)
            assert pkg.binding.rlx_model_weight_version(model.handle) == 3
            assert eng.may_generate(trainer_version=3, max_staleness=1)
        if s == 0:
            out = eng.prefill(rows, wl.prompt_tokens, None, forced=forced[0], want_logits=True, want_routing=True,
                              want_sampled=True)
            per_seq = wl.prompt_lens
        else:
            out = eng.decode_step(forced=torch.tensor(forced[s], dtype=torch.int32, device="cuda:0"),
                                  want_logits=True, want_routing=True, want_sampled=True)
            per_seq = np.ones(wl.batch, int)
        torch.cuda.synchronize()
        d = dict(logits=out.logits.cpu().numpy(), logprobs=out.logprobs.cpu().numpy(),
                 tokens=out.tokens.cpu().numpy()[:wl.batch].copy(), weight_version=out.weight_version)
        if out.routing is not None:
            r = out.routing.cpu().numpy()
            offs = np.concatenate([[0], np.cumsum(per_seq)])
            d["routing"] = [r[offs[j]:offs[j + 1]] for j in range(wl.batch)]
        gsteps.append(d)

    if shape.is_moe:   # a tolerated near-tie would hide everything after it: replay the GPU's routing in the oracle
        osteps = _oracle_steps(shape, wl, forced, [g["routing"] for g in gsteps])
    dl = dp = 0.0
    for s, (g, o) in enumerate(zip(gsteps, osteps)):
        assert g["weight_version"] == o["weight_version"] == (0 if s < SWAP_AT else 3)
        for j in range(wl.batch):
            dl = max(dl, float(np.abs(g["logits"][j] - o["logits"][j]).max()))
            dp = max(dp, abs(float(g["logprobs"][j]) - o["logprobs"][j]))
            assert int(g["tokens"][j]) == o["tokens"][j]
            if shape.is_moe:
                bad = (np.sort(g["routing"][j], -1) != np.sort(o["own_routing"][j], -1)).any(-1)
                assert (o["gate_gap"][j][bad] < TIE_GAP).all(), "step %d row %d: routing differs off a near-tie" % (s, j)
    say("%s: max |dlogit| %.5f, max |dlogprob| %.5f over %d steps" % (shape.name, dl, dp, N_DECODE))
    assert dl <= LOGIT_BAR and dp <= LOGPROB_BAR
    # the refresh did change the function: the old weights' logits at the first refreshed step are far off
    stale = O.OracleRollout(O.OracleModel(shape, 0), n_blocks=wl.batch * mb)
    ids = [stale.add_sequence(int(wl.seeds[i])) for i in range(wl.batch)]
    z = None
    for s in range(SWAP_AT + 1):
        st = stale.prefill_chunk(ids, wl.prompt_tokens, forced_tokens=forced[0], want_logits=True) if s == 0 else \
            stale.decode_step(ids, forced_tokens=forced[s], want_logits=True)
        z = st["logits"]
    assert max(float(np.abs(gsteps[SWAP_AT]["logits"][j] - z[j]).max()) for j in range(wl.batch)) > 10 * LOGIT_BAR
    model.close()


def test_set_weights_rejects_bad_tables_and_keeps_the_old_ones(amd):
    pkg, synthetic = amd
    B = pkg.binding
    model = synthetic.model_from_shape(RI.TINY_DENSE, 0, activation_split=1)
    import ctypes as C
    bad = B.Weights()
    C.memmove(C.byref(bad), C.byref(model._w), C.sizeof(B.Weights))
    bad.lm_head = None
    with pytest.raises(B.RlxError) as e:
        B.rlx_model_set_weights(model.handle, bad, 9)
    assert e.value.code == B.RLX_EINVAL
    assert B.rlx_model_weight_version(model.handle) == 0
    B.rlx_model_set_weights(model.handle, model._w, 9)      # the same tensors under a new tag
    assert B.rlx_model_weight_version(model.handle) == 9
    model.close()
