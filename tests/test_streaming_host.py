"""Host logic of the streaming rollout scheduler (continuous refill, micro-batch completion events, admission
gate; paper Sec. 3.3 "Streaming data flow" and "staleness control") against a stand-in engine that emits a known
token function on the CPU.  No GPU, no library call: only the scheduling is under test."""
import types

import numpy as np
import pytest
import torch

from paper_2604_11554_amd.engine import Request, StreamingRollout

V, EOS, PAD = 1000, 999, 998


def fake_token(seed, pos):
    return EOS if (seed + pos) % 11 == 0 else (seed * 31 + pos * 17) % (V - 2)


def expected(rq):
    """Response of one request under the engine's rules: EOS ends it; the token at position prompt + max_new - 1
    is a forced EOS."""
    p, out = len(rq.prompt), []
    for pos in range(p, p + rq.max_new_tokens):
        t = EOS if pos >= p + rq.max_new_tokens - 1 else fake_token(rq.seed, pos)
        out.append(t)
        if t == EOS:
            break
    return out


class FakeEngine:
    def __init__(self, max_seqs, n_pages, max_chunk_tokens):
        self.max_seqs, self.max_chunk_tokens = max_seqs, max_chunk_tokens
        self.m = types.SimpleNamespace(device=torch.device("cpu"), cfg=dict(n_layers=1, top_k=0), weight_version=0)
        self.is_moe = False
        self.free = n_pages
        self.pages = [0] * max_seqs
        self.tokens = torch.zeros(max_seqs, dtype=torch.int32)
        self.ctx_lens = torch.zeros(max_seqs, dtype=torch.int32)
        self.finished = torch.ones(max_seqs, dtype=torch.uint8)
        self.seed = [0] * max_seqs
        self.max_ctx = [0] * max_seqs
        self.n = 0
        self.prefill_calls, self.live_row_steps, self.row_steps = [], 0, 0

    def open_slots(self, n):
        self.n = n

    def pages_free(self):
        return self.free

    def release_slot(self, row):
        self.free += self.pages[row]
        self.pages[row] = 0
        self.finished[row] = 1

    def refill_slot(self, row, seed, temperature, max_ctx):
        self.release_slot(row)
        nb = (max_ctx + 15) // 16
        if nb > self.free:
            return False
        self.free -= nb
        self.pages[row], self.seed[row], self.max_ctx[row] = nb, seed, max_ctx
        self.ctx_lens[row] = 0
        self.finished[row] = 0
        return True

    def _emit(self, row, pos):
        t = EOS if pos >= self.max_ctx[row] - 1 else fake_token(self.seed[row], pos)
        self.tokens[row] = t
        self.finished[row] = 1 if t == EOS else 0
        return t

    def prefill(self, rows, toks, want_routing=False):
        assert sum(len(t) for t in toks) <= self.max_chunk_tokens
        self.prefill_calls.append(list(rows))
        out = []
        for r, t in zip(rows, toks):
            assert not self.finished[r] and self.ctx_lens[r] == 0
            self.ctx_lens[r] = len(t)
            out.append(self._emit(r, len(t)))
        return types.SimpleNamespace(tokens=torch.tensor(out, dtype=torch.int32),
                                     logprobs=-torch.tensor(out, dtype=torch.float32) / 1000, routing=None,
                                     weight_version=self.m.weight_version)

    def decode_step(self, out_logprobs=None, out_routing=None):
        for r in range(self.n):
            self.row_steps += 1
            if self.finished[r]:
                self.tokens[r] = PAD
                out_logprobs[r] = 0.0
                continue
            self.live_row_steps += 1
            self.ctx_lens[r] += 1
            t = self._emit(r, int(self.ctx_lens[r]))
            out_logprobs[r] = -t / 1000.0


def make_requests(n, seed=0):
    g = np.random.default_rng(seed)
    return [Request(g.integers(0, V - 2, size=int(g.integers(3, 40))).astype(np.int32), int(g.integers(1, 10 ** 6)),
                    1.0, int(g.integers(1, 30))) for _ in range(n)]


@pytest.mark.parametrize("slots,micro_batch,poll_every", [(4, 3, 4), (8, 32, 1), (1, 1, 5), (5, 4, 16)])
def test_streaming_outputs_partitions_and_refill(slots, micro_batch, poll_every):
    reqs = make_requests(23)
    eng = FakeEngine(slots, n_pages=1000, max_chunk_tokens=64)
    events = []
    sr = StreamingRollout(eng, reqs, micro_batch=micro_batch, poll_every=poll_every,
                          on_partition=lambda p, cs: events.append((p, [c.index for c in cs], [len(c.tokens) for c in cs])))
    done = sr.run()
    assert [c.index for c in done] == list(range(len(reqs)))
    for c, rq in zip(done, reqs):
        want = expected(rq)
        assert list(c.tokens) == want
        np.testing.assert_allclose(c.logprobs, -np.array(want, np.float32) / 1000)
        assert len(c.weight_versions) == len(want) and (c.weight_versions == 0).all()
    # every micro-batch reported exactly once, members in request order, complete when reported
    n_parts = (len(reqs) + micro_batch - 1) // micro_batch
    assert sorted(p for p, _, _ in events) == list(range(n_parts)) and sr.partition_order == [p for p, _, _ in events]
    for p, idx, lens in events:
        assert idx == list(range(p * micro_batch, min((p + 1) * micro_batch, len(reqs))))
        assert lens == [len(expected(reqs[i])) for i in idx]
    # refill: slots are reused (more prefill calls than one batch), all pages come back, no slot ran two requests at once
    assert eng.free == 1000 and len(eng.prefill_calls) > 1
    # a row idles only between its end and the next poll: with a poll every step, live row-steps are all but the
    # steps of the final drain
    if poll_every == 1 and slots < len(reqs):
        assert eng.live_row_steps >= 0.7 * eng.row_steps


def test_admission_waits_for_pages_and_for_the_gate():
    reqs = make_requests(9, seed=1)
    need = max((len(r.prompt) + r.max_new_tokens + 15) // 16 for r in reqs)
    eng = FakeEngine(4, n_pages=need + 1, max_chunk_tokens=64)       # room for about one sequence at a time
    done = StreamingRollout(eng, reqs, micro_batch=2, poll_every=2).run()
    assert [list(c.tokens) for c in done] == [expected(r) for r in reqs] and eng.free == need + 1
    assert max(len(rows) for rows in eng.prefill_calls) <= 2
    # a pool that cannot hold the next request at all is an error, not a hang
    with pytest.raises(MemoryError):
        StreamingRollout(FakeEngine(4, n_pages=need - 1, max_chunk_tokens=64),
                         sorted(reqs, key=lambda r: -(len(r.prompt) + r.max_new_tokens)), micro_batch=2).run()
    # the gate: closed after the second partition event until the "trainer" catches up inside the callback
    state = dict(v_t=0, v_r=0, events=0)
    eng = FakeEngine(2, n_pages=1000, max_chunk_tokens=64)

    def on_partition(p, cs):
        state["events"] += 1
        state["v_t"] += 1                       # the trainer consumed a partition and published new weights ...
        if state["events"] % 2 == 0:
            state["v_r"] = state["v_t"]         # ... and every second time the rollout side installs them
            eng.m.weight_version = state["v_r"]

    sr = StreamingRollout(eng, reqs, micro_batch=1, poll_every=1, on_partition=on_partition,
                          may_admit=lambda: state["v_t"] - state["v_r"] < 2)
    done = sr.run()
    assert len(done) == len(reqs) and state["events"] == len(reqs)
    vers = np.concatenate([c.weight_versions for c in done])
    assert vers.min() == 0 and vers.max() > 0 and (np.diff([c.weight_versions[0] for c in done]) >= 0).all()
    # a gate that never opens while nothing runs is reported
    with pytest.raises(RuntimeError):
        StreamingRollout(FakeEngine(2, 1000, 64), reqs, may_admit=lambda: False).run()
