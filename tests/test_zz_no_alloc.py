"""rollout_decode_step_static (the decode step on the library's fixed scratch array, for callers that cannot
allocate) against rollout_decode_step with a caller workspace: same inputs, same state, every output compared, on
two calls in a row, the second with fewer sequences (the array then still holds the larger call's contents)."""
import sys

import numpy as np
import pytest
import torch

import rollout_inputs as RI

pytestmark = pytest.mark.gpu


def say(msg):
    print("[gpu-case] " + msg, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("shape_name", ["tiny_dense", "tiny_moe"])
def test_static_scratch_decode_step_equals_the_workspace_one(shape_name):
    import paper_2604_11554_amd as pkg
    from paper_2604_11554_amd import binding as B
    from paper_2604_11554_amd import synthetic
    B.lib()
    shape = {"tiny_dense": RI.TINY_DENSE, "tiny_moe": RI.TINY_MOE}[shape_name]
    say("static scratch decode step, %s" % shape.name)
    wl = RI.workload_tiny(shape, n_decode=8, lens=(16, 33, 48, 64, 5, 21))
    model = synthetic.model_from_shape(shape, 0)
    eng = pkg.RolloutEngine(model, n_blocks=64, max_seqs=8, max_chunk_tokens=256, max_blocks_per_seq=8)
    rows = [eng.add_sequence(int(s), reserve_tokens=len(p) + 8) for s, p in zip(wl.seeds, wl.prompt_tokens)]
    eng.prefill(rows, wl.prompt_tokens)
    eng.decode_step()                                    # one step through the usual path first
    torch.cuda.synchronize()
    dev = eng.m.device
    cfg = eng.m.cfg

    def snapshot():
        return [t.clone() for t in (eng.tokens, eng.ctx_lens, eng.finished, eng.kv_pool)]

    def restore(st):
        for t, s in zip((eng.tokens, eng.ctx_lens, eng.finished, eng.kv_pool), st):
            t.copy_(s)

    def outputs(n):
        o = dict(lp=torch.full((n,), 7.0, dtype=torch.float32, device=dev),
                 smp=torch.full((n,), -7, dtype=torch.int32, device=dev),
                 logits=torch.full((n, cfg["vocab"]), 7.0, dtype=torch.float32, device=dev))
        o["routing"] = (torch.full((n, cfg["n_layers"], cfg["top_k"]), -7, dtype=torch.int32, device=dev)
                        if eng.is_moe else None)
        return o

    def step(n, static):
        o = outputs(n)
        common = (n, eng.tokens, eng.ctx_lens, eng.block_table, eng.max_blocks, eng.seeds, eng.temperature,
                  eng.max_ctx, eng.finished, None, o["lp"], o["smp"], o["routing"], o["logits"])
        if static:
            B.rollout_decode_step_static(eng.m.handle, eng.kv_pool, eng.n_blocks, *common)
        else:
            B.rollout_decode_step(eng.m.handle, eng.kv_pool, eng.n_blocks, eng.workspace, *common)
        torch.cuda.synchronize()
        state = [t.clone() for t in (eng.tokens, eng.ctx_lens, eng.finished, eng.kv_pool)]
        return o, state

    for n in (6, 2):                                     # the second call is the smaller one
        st = snapshot()
        want, want_state = step(n, static=False)
        restore(st)
        got, got_state = step(n, static=True)
        for name, a, b in zip(("tokens", "ctx_lens", "finished", "kv_pool"), got_state, want_state):
            assert torch.equal(a, b), "%s differs after a step of %d sequences" % (name, n)
        assert torch.equal(got["smp"], want["smp"])
        if eng.is_moe:
            assert torch.equal(got["routing"], want["routing"])
        # the same kernels on the same inputs: the floating-point outputs are equal to the bit, far inside the
        # 0.05 / 0.02 bars of the parity tests
        assert torch.equal(got["logits"], want["logits"]) and torch.equal(got["lp"], want["lp"])
        assert int(eng.ctx_lens[0]) == len(wl.prompt_tokens[0]) + 1 + (1 if n == 6 else 2)
        say("n_seqs %d: tokens, cache, routing, logits and log-probabilities identical" % n)
    # a step that does not fit the fixed array is refused before anything is enqueued
    with pytest.raises(B.RlxError) as e:
        B.rollout_decode_step_static(eng.m.handle, eng.kv_pool, eng.n_blocks, 1 << 16, eng.tokens, eng.ctx_lens,
                                     eng.block_table, eng.max_blocks, eng.seeds, eng.temperature, eng.max_ctx,
                                     eng.finished, None, outputs(1)["lp"])
    assert e.value.code == B.RLX_ENOMEM and "fixed array" in str(e.value)
    model.close()
