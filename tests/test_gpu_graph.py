"""GPU: a decode step is made of kernel launches on the caller's stream only (no allocation, no host
synchronisation, no memset nodes), so a serving loop can capture it in a HIP graph once and replay it; the state
tensors advance in place, so every replay is the next step.  Each replay is checked against the eager run of the
same rollout, with eager work and synchronisations between replays."""
import numpy as np
import pytest
import torch

import rollout_inputs as RI

pytestmark = pytest.mark.gpu

N_STEPS = 7


@pytest.fixture(scope="module")
def amd():
    import paper_2604_11554_amd as pkg
    from paper_2604_11554_amd import synthetic
    pkg.binding.lib()            # fail loudly if the library is not built
    return pkg, synthetic


def _start(pkg, synthetic, shape, wl, grouped):
    model = synthetic.model_from_shape(shape, 0, activation_split=1)
    eng = pkg.RolloutEngine(model, n_blocks=96, max_seqs=8, max_chunk_tokens=512, max_blocks_per_seq=12)
    if grouped:                  # a sampling group of three members on the first prompt, then the others
        d = eng.add_sequence(0, reserve_tokens=len(wl.prompt_tokens[3]))
        eng.prefill([d], [wl.prompt_tokens[3][:-1]], sample_last=[False])
        kids = [eng.fork(d, 70 + k, reserve_tokens=len(wl.prompt_tokens[3]) + N_STEPS + 2) for k in range(3)]
        eng.finished[d] = 1
        eng.prefill(kids, [wl.prompt_tokens[3][-1:]] * 3)
    rows = [eng.add_sequence(int(wl.seeds[i]), reserve_tokens=len(wl.prompt_tokens[i]) + N_STEPS + 2) for i in range(3)]
    eng.prefill(rows, wl.prompt_tokens[:3])
    torch.cuda.synchronize()
    return model, eng


@pytest.mark.parametrize("shape_name,grouped", [("tiny_dense", False), ("tiny_moe", False), ("tiny_dense", True)])
def test_decode_step_replayed_from_a_graph_equals_eager(amd, shape_name, grouped):
    pkg, synthetic = amd
    shape = {"tiny_dense": RI.TINY_DENSE, "tiny_moe": RI.TINY_MOE}[shape_name]
    wl = RI.workload_tiny(shape)
    # eager reference
    model, eng = _start(pkg, synthetic, shape, wl, grouped)
    n = eng.n
    want = []
    for _ in range(N_STEPS):
        o = eng.decode_step(want_routing=True)
        torch.cuda.synchronize()
        want.append((o.tokens[:n].cpu().numpy().copy(), o.logprobs.cpu().numpy().copy(),
                     None if o.routing is None else o.routing.cpu().numpy().copy(), eng.ctx_lens[:n].cpu().numpy().copy()))
    model.close()
    # the same rollout with the step captured once
    model, eng = _start(pkg, synthetic, shape, wl, grouped)
    lp = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    rt = (torch.zeros((n, shape.n_layers, shape.top_k), dtype=torch.int32, device="cuda:0") if shape.is_moe else None)
    eng._shared_prefix()                                      # built (and its stream synchronised) outside the capture
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    got = []
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            eng.decode_step(out_logprobs=lp, out_routing=rt)
    torch.cuda.synchronize()
    scratch = torch.zeros(1 << 16, device="cuda:0")
    for s in range(N_STEPS):
        g.replay()
        torch.cuda.synchronize()
        got.append((eng.tokens[:n].cpu().numpy().copy(), lp.cpu().numpy().copy(),
                    None if rt is None else rt.cpu().numpy().copy(), eng.ctx_lens[:n].cpu().numpy().copy()))
        scratch.add_(1.0)                                      # eager work of the program between replays
        assert float(scratch.sum().item()) == (s + 1) * (1 << 16)
    for s, (w, h) in enumerate(zip(want, got)):
        np.testing.assert_array_equal(w[0], h[0], err_msg="tokens of step %d" % s)
        np.testing.assert_array_equal(w[1], h[1], err_msg="log-probabilities of step %d" % s)
        np.testing.assert_array_equal(w[3], h[3], err_msg="cached lengths of step %d" % s)
        if w[2] is not None:
            np.testing.assert_array_equal(w[2], h[2], err_msg="routing of step %d" % s)
    model.close()
