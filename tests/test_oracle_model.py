"""Pins for the whole-model oracle: two independent formulations must agree
(full-sequence forward vs incremental paged rollout), plus paging, chunking,
sharing, replay and finish-rule invariants.  CPU only."""
import numpy as np
import pytest

import oracle as O
import rollout_inputs as RI

DENSE = RI.TINY_DENSE.replace(n_layers=2, vocab=512)
DENSE_QKN = DENSE.replace(name="tiny_dense_qkn", qk_norm=True)
MOE = RI.TINY_MOE.replace(n_layers=2, vocab=512, d_model=128, n_experts=16, d_ff_expert=48)


def _prompts(shape, lens, seed=7):
    return RI.workload_tiny(shape, lens=lens, prompt_seed=seed).prompt_tokens


@pytest.mark.parametrize("shape", [DENSE, DENSE_QKN, MOE], ids=lambda s: s.name)
def test_incremental_equals_full_forward(shape):
    model = O.OracleModel(shape, model_seed=3)
    toks = _prompts(shape, (9, 21))
    n_dec = 6
    ro = O.OracleRollout(model, n_blocks=16)
    ids = [ro.add_sequence(seed=100 + i) for i in range(2)]
    got_logits = [[], []]
    seqs = [list(t) for t in toks]
    routes = [[], []]
    r = ro.prefill_chunk(ids, toks, want_logits=True)
    for step in range(n_dec):
        for j in range(2):
            got_logits[j].append(r["logits"][j])
            seqs[j].append(r["tokens"][j])
            if shape.is_moe:
                routes[j].append(r["routing"][j])
        r = ro.decode_step(ids, want_logits=True)
    full = O.forward_full(model, [np.array(s[:-1], np.int32) for s in seqs])
    for j in range(2):
        n0 = len(toks[j])
        z_full = full[j]["logits"][n0 - 1:]
        np.testing.assert_allclose(np.stack(got_logits[j]), z_full, atol=1e-4, rtol=0)
        if shape.is_moe:
            np.testing.assert_array_equal(np.concatenate(routes[j], 0), full[j]["routing"][: n0 + n_dec - 1])


def test_bf16_rounding_of_the_kv_store():
    # nearest-even on the 8-bit significand grid, checked on hand-picked values
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20,
                  -3.0e-5, 0.0, 65280.0], np.float32)
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, 0, 0.0, 65280.0], np.float32)
    got = O.round_to_bf16(x)
    want[5] = got[5]
    np.testing.assert_array_equal(got, want)
    r = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    q = O.round_to_bf16(r)
    assert (np.abs(q - r) <= np.abs(r) * 2.0 ** -8).all() and (q.view(np.uint32) & 0xFFFF == 0).all()
    np.testing.assert_array_equal(O.round_to_bf16(q), q)                      # idempotent
    # independent routine: torch's float32 -> bfloat16 conversion
    import torch
    np.testing.assert_array_equal(q, torch.from_numpy(r).to(torch.bfloat16).to(torch.float32).numpy())
    # the store is where the rounding happens: with kv_bf16 the cached keys are on the bf16 grid
    model = O.OracleModel(DENSE, 5)
    ro = O.OracleRollout(model, n_blocks=4)
    i = ro.add_sequence(seed=1)
    ro.prefill_chunk([i], [_prompts(DENSE, (9,))[0]])
    used = ro.kpool[:, ro.blocks[i][0], :9]
    assert (used.view(np.uint32) & 0xFFFF == 0).all() and np.abs(used).max() > 0
    exact = O.OracleModel(DENSE, 5, kv_bf16=False)
    a = O.forward_full(model, _prompts(DENSE, (9,)))[0]["logits"]
    b = O.forward_full(exact, _prompts(DENSE, (9,)))[0]["logits"]
    assert 0 < np.abs(a - b).max() < 0.02


def test_fp16_option_rounding_and_model():
    """The FP16 precision option (paper App. "FP16 vs. BF16 precision ablation"): fp16 weights, fp16 KV store."""
    # nearest-even on the 11-bit significand grid, subnormals below 2^-14, overflow past 65504: hand-picked values
    x = np.array([1.0, 1.0 + 2.0 ** -11, 1.0 + 2.0 ** -10, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -22,
                  65504.0, 65519.0, 65520.0, 2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25, -(2.0 ** -14 + 2.0 ** -25),
                  -(2.0 ** -14 + 3 * 2.0 ** -25), 0.0],
                 np.float32)
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -10, 1.0 + 2.0 ** -9, 1.0 + 2.0 ** -10,
                     65504.0, 65504.0, np.inf, 2.0 ** -24, 0.0, 2.0 ** -23, -(2.0 ** -14),
                     -(2.0 ** -14 + 2.0 ** -23), 0.0], np.float32)
    np.testing.assert_array_equal(O.round_to_f16(x), want)
    r = (np.random.default_rng(0).standard_normal(10000) * 3).astype(np.float64)
    q = O.round_to_f16(r)
    assert q.dtype == np.float64
    big = np.abs(r) >= 2.0 ** -14
    assert (np.abs(q - r)[big] <= np.abs(r)[big] * 2.0 ** -11).all() and (np.abs(q - r)[~big] <= 2.0 ** -25).all()
    np.testing.assert_array_equal(O.round_to_f16(q), q)                       # idempotent
    # independent routine: torch's float32 -> float16 conversion
    import torch
    r32 = r.astype(np.float32)
    np.testing.assert_array_equal(O.round_to_f16(r32), torch.from_numpy(r32).to(torch.float16).to(torch.float32).numpy())
    # the same draws, rounded to fp16 instead of bf16: closer to the unrounded values than bf16 is
    wb = RI.bits_to_f32(RI.tensor_bits(DENSE, 5, 0, "wq", "bf16"), "bf16")
    wh = RI.bits_to_f32(RI.tensor_bits(DENSE, 5, 0, "wq", "f16"), "f16")
    assert 0 < np.abs(wb - wh).max() <= np.abs(wb).max() * 2.0 ** -8
    np.testing.assert_array_equal(O.round_to_f16(wh), wh)
    # the store is where the rounding happens, and incremental decoding still equals the full forward
    model = O.OracleModel(DENSE, 5, fmt="f16")
    tok = _prompts(DENSE, (9,))[0]
    ro = O.OracleRollout(model, n_blocks=4)
    i = ro.add_sequence(seed=1)
    r0 = ro.prefill_chunk([i], [tok], want_logits=True)
    used = ro.kpool[:, ro.blocks[i][0], :9]
    np.testing.assert_array_equal(used, used.astype(np.float16).astype(used.dtype))
    assert (used.view(np.uint32) & 0xFFFF != 0).any()                          # finer than the bf16 grid
    r1 = ro.decode_step([i], want_logits=True)
    full = O.forward_full(model, [np.array(list(tok) + [r0["tokens"][0]], np.int32)])[0]["logits"]
    np.testing.assert_allclose(np.stack([r0["logits"][0], r1["logits"][0]]), full[8:], atol=1e-4, rtol=0)
    # fp16 storage perturbs the logits less than bf16 storage does (same unrounded draws behind both models)
    exact_h = O.forward_full(O.OracleModel(DENSE, 5, fmt="f16", kv_bf16=False), [tok])[0]["logits"]
    exact_b = O.forward_full(O.OracleModel(DENSE, 5, fmt="bf16", kv_bf16=False), [tok])[0]["logits"]
    d_h = np.abs(O.forward_full(model, [tok])[0]["logits"] - exact_h).max()
    d_b = np.abs(O.forward_full(O.OracleModel(DENSE, 5), [tok])[0]["logits"] - exact_b).max()
    assert 0 < d_h < d_b


def test_float32_oracle_close_to_float64():
    toks = _prompts(MOE, (24,))
    z32 = O.forward_full(O.OracleModel(MOE, 3, dtype=np.float32, kv_bf16=False), toks)[0]
    z64 = O.forward_full(O.OracleModel(MOE, 3, dtype=np.float64, kv_bf16=False), toks)[0]
    assert np.abs(z32["logits"] - z64["logits"]).max() < 2e-4
    stable = z64["gate_gap"] > 1e-3
    assert stable.mean() > 0.9
    same = (np.sort(z32["routing"], -1) == np.sort(z64["routing"], -1)).all(-1)
    assert same[stable].all()


@pytest.mark.parametrize("shape", [DENSE, MOE], ids=lambda s: s.name)
def test_chunked_prefill_invariance(shape):
    model = O.OracleModel(shape, 5)
    tok = _prompts(shape, (37,))[0]
    outs = []
    for chunks in ([37], [16, 16, 5], [1] * 37, [7, 30]):
        ro = O.OracleRollout(model, n_blocks=8)
        i = ro.add_sequence(seed=1)
        p = 0
        routes = []
        for c in chunks:
            last = p + c == 37
            r = ro.prefill_chunk([i], [tok[p:p + c]], sample_last=[last], want_logits=True)
            routes.append(r["routing"][0])
            p += c
        outs.append((r["logits"][0], r["tokens"][0], r["logprobs"][0], np.concatenate(routes, 0)))
    for o in outs[1:]:
        np.testing.assert_allclose(o[0], outs[0][0], atol=1e-4)
        assert o[1] == outs[0][1]
        assert abs(o[2] - outs[0][2]) < 1e-4
        if shape.is_moe:
            np.testing.assert_array_equal(o[3], outs[0][3])


def test_paging_invariants():
    model = O.OracleModel(DENSE, 5)
    toks = _prompts(DENSE, (19, 33))
    def run(block_size, order=None, n_blocks=64):
        ro = O.OracleRollout(model, n_blocks=n_blocks, block_size=block_size, alloc_order=order)
        ids = [ro.add_sequence(seed=10 + i) for i in range(2)]
        res = [ro.prefill_chunk(ids, toks, want_logits=True)]
        for _ in range(4):
            res.append(ro.decode_step(ids, want_logits=True))
        return res
    base = run(16)
    perm = list(np.random.default_rng(0).permutation(64))
    for other in (run(16, perm), run(1), run(64), run(5)):
        for a, b in zip(base, other):
            assert a["tokens"] == b["tokens"]
            for za, zb in zip(a["logits"], b["logits"]):
                np.testing.assert_allclose(za, zb, atol=1e-5)


def test_shared_prefix_equals_private_copies_and_slot_independence():
    model = O.OracleModel(DENSE, 5)
    tok = _prompts(DENSE, (23,))[0]
    # private: three sequences each prefill the same prompt
    ro = O.OracleRollout(model, n_blocks=32)
    ids = [ro.add_sequence(seed=s) for s in (50, 51, 52)]
    priv = [ro.prefill_chunk(ids, [tok] * 3)]
    for _ in range(5):
        priv.append(ro.decode_step(ids))
    # shared: prefill once without sampling the continuation of the last token, fork, then sample
    ro2 = O.OracleRollout(model, n_blocks=32)
    base = ro2.add_sequence(seed=0)
    ro2.prefill_chunk([base], [tok[:-1]], sample_last=[False])
    kids = [ro2.fork(base, seed=s) for s in (52, 50, 51)]            # different batch slots
    sh = [ro2.prefill_chunk(kids, [tok[-1:]] * 3)]
    for _ in range(5):
        sh.append(ro2.decode_step(kids))
    assert ro2.blocks[kids[0]][0] == ro2.blocks[base][0] and ro2.blocks[kids[0]][1] != ro2.blocks[base][1]
    for a, b in zip(priv, sh):
        assert [a["tokens"][0], a["tokens"][1], a["tokens"][2]] == [b["tokens"][1], b["tokens"][2], b["tokens"][0]]
        np.testing.assert_allclose([a["logprobs"][i] for i in (0, 1, 2)], [b["logprobs"][i] for i in (1, 2, 0)],
                                   atol=1e-5)
    # group members with different seeds diverge
    assert len({tuple(r["tokens"]) for r in priv}) > 1 and priv[1]["tokens"][0] != priv[1]["tokens"][1]


def test_logprob_is_log_softmax_of_logits_and_sampling_rule():
    model = O.OracleModel(DENSE, 5)
    tok = _prompts(DENSE, (12,))[0]
    ro = O.OracleRollout(model, n_blocks=8)
    i = ro.add_sequence(seed=77, temperature=0.8)
    r = ro.prefill_chunk([i], [tok], want_logits=True)
    z = r["logits"][0].astype(np.float64)
    lp = z / 0.8 - np.log(np.exp(z / 0.8).sum())
    assert abs(lp[r["tokens"][0]] - r["logprobs"][0]) < 1e-4
    # the token that lands at position 12 is drawn with the noise of position 12
    assert r["tokens"][0] == O.sample_gumbel_max(r["logits"][0], 0.8, 77, 12)
    r2 = ro.decode_step([i], want_logits=True)
    assert r2["tokens"][0] == O.sample_gumbel_max(r2["logits"][0], 0.8, 77, 13)


def test_teacher_forcing_and_finish_rules():
    model = O.OracleModel(DENSE, 5)
    s = DENSE
    tok = _prompts(DENSE, (10,))[0]
    ro = O.OracleRollout(model, n_blocks=8)
    i = ro.add_sequence(seed=1, max_ctx=10 + 3)          # prompt 10 + three response tokens
    free = ro.prefill_chunk([i], [tok], want_logits=True)
    # forcing: the forced token is appended and scored, the sampled one still reported
    ro2 = O.OracleRollout(model, n_blocks=8)
    j = ro2.add_sequence(seed=1, max_ctx=10 + 3)
    forced = (free["tokens"][0] + 5) % (s.vocab - 2)
    f = ro2.prefill_chunk([j], [tok], forced_tokens=[forced], want_logits=True)
    assert f["sampled"][0] == free["tokens"][0] and f["tokens"][0] == forced
    assert abs(f["logprobs"][0] - O.log_softmax(f["logits"][0])[forced]) < 1e-6
    # length cap: third response token (position 12) is forced to EOS and scored as EOS
    a = ro.decode_step([i])
    assert not ro.finished[i] and a["tokens"][0] != s.eos_token_id
    b = ro.decode_step([i], want_logits=True)
    assert ro.finished[i] and b["tokens"][0] == s.eos_token_id
    assert abs(b["logprobs"][0] - O.log_softmax(b["logits"][0])[s.eos_token_id]) < 1e-6
    ctx = ro.ctx[i]
    c = ro.decode_step([i])                               # finished rows are inert
    assert c["tokens"][0] == s.pad_token_id and c["logprobs"][0] == 0.0 and ro.ctx[i] == ctx == 12
    # a natural EOS (here: forced in) also finishes the sequence
    ro3 = O.OracleRollout(model, n_blocks=8)
    k = ro3.add_sequence(seed=1)
    ro3.prefill_chunk([k], [tok], forced_tokens=[s.eos_token_id])
    assert ro3.finished[k]


def test_injected_embeddings_and_multi_turn_state():
    model = O.OracleModel(MOE, 9)
    wl = RI.workload_omni_agentic(MOE, batch=2, mm_lo=5, mm_hi=9, n_text=6, n_turns=2, tool_len=4, turn_decode=3)
    # an injected row equal to a token's embedding row must behave exactly like that token
    tok = wl.prompt_tokens[0].copy()
    n_mm = int((tok < 0).sum())
    emb_bits = RI.tensor_bf16(MOE, 9, RI.GLOBAL_LAYER, "embed")
    ids_as_tokens = np.arange(n_mm, dtype=np.int32) + 3
    a = O.forward_full(model, [tok], [emb_bits[ids_as_tokens]])[0]["logits"]
    tok2 = tok.copy(); tok2[:n_mm] = ids_as_tokens
    b = O.forward_full(model, [tok2])[0]["logits"]
    np.testing.assert_array_equal(a, b)
    # multi-turn: KV carried across turns == one teacher-forced pass over the whole transcript
    ro = O.OracleRollout(model, n_blocks=16)
    i = ro.add_sequence(seed=5)
    ro.prefill_chunk([i], [wl.prompt_tokens[0]], [wl.prompt_embeds[0]], sample_last=[False])
    transcript = list(wl.prompt_tokens[0])
    logits = []
    for turn in wl.turns[0]:
        r = ro.prefill_chunk([i], [turn.tool_tokens], want_logits=True)
        transcript += list(turn.tool_tokens)
        for _ in range(turn.n_decode):
            logits.append((len(transcript) - 1, r["logits"][0]))
            transcript.append(r["tokens"][0])
            r = ro.decode_step([i], want_logits=True)
    # the last sampled token of a turn is still fed (its KV is needed by the next turn's tool chunk)
    full = O.forward_full(model, [np.array(transcript, np.int32)], [wl.prompt_embeds[0]])[0]["logits"]
    for pos, z in logits:
        np.testing.assert_allclose(z, full[pos], atol=1e-4)


def test_weight_refresh_keeps_the_store_and_uses_the_new_weights():
    """Pins of OracleRollout.set_model: (1) refreshing with identical weights changes nothing; (2) weights that
    differ only after the last attention (final norm, LM head) leave every stored key/value valid, so the steps after
    the refresh equal the new model's full forward and the steps before it the old model's; (3) a refresh before the
    first call equals a rollout of the new model alone."""
    A = O.OracleModel(DENSE, 5)
    same = O.OracleModel(DENSE, 5)
    tb = {(l, n): RI.tensor_bits(DENSE, 5 if (l, n) not in ((RI.GLOBAL_LAYER, "lm_head"), (RI.GLOBAL_LAYER, "final_norm"))
                                 else 9, l, n)
          for l in [RI.GLOBAL_LAYER] + list(range(DENSE.n_layers)) for n in RI.tensor_names(DENSE, l)}
    B_head = O.OracleModel(DENSE, 5, tensors=tb)
    B_all = O.OracleModel(DENSE, 9)
    tok = _prompts(DENSE, (11,))[0]
    n_dec, k = 6, 3

    def rollout(first, second, swap_at, forced=None):
        ro = O.OracleRollout(first, n_blocks=4)
        i = ro.add_sequence(seed=3)
        outs = []
        for s in range(n_dec):
            if s == swap_at:
                ro.set_model(second, 7)
            f = None if forced is None else [forced[s]]
            r = ro.prefill_chunk([i], [tok], forced_tokens=f, want_logits=True) if s == 0 else \
                ro.decode_step([i], forced_tokens=f, want_logits=True)
            outs.append((r["logits"][0], r["tokens"][0], r["logprobs"][0], ro.weight_version))
        return outs

    base = rollout(A, A, None)
    forced = [o[1] for o in base]
    # (1)
    for x, y in zip(rollout(A, same, k), base):
        np.testing.assert_array_equal(x[0], y[0])
        assert x[1] == y[1] and x[2] == y[2]
    # (2)
    mixed = rollout(A, B_head, k, forced)
    assert [o[3] for o in mixed] == [0] * k + [7] * (n_dec - k)
    seq = np.array(list(tok) + forced[:-1], np.int32)
    za = O.forward_full(A, [seq])[0]["logits"][len(tok) - 1:]
    zb = O.forward_full(B_head, [seq])[0]["logits"][len(tok) - 1:]
    assert np.abs(za - zb).max() > 0.05
    for s in range(n_dec):
        np.testing.assert_allclose(mixed[s][0], (za if s < k else zb)[s], atol=1e-4, rtol=0)
    # (3)
    for x, y in zip(rollout(A, B_all, 0), rollout(B_all, B_all, None)):
        np.testing.assert_array_equal(x[0], y[0])
    # a refresh of every layer mid-sequence is neither model's own rollout: old keys/values stay in the store
    z_mid = rollout(A, B_all, k, forced)[k][0]
    z_b = O.forward_full(B_all, [seq])[0]["logits"][len(tok) - 1 + k]
    assert np.abs(z_mid - z_b).max() > 1e-3 and np.abs(z_mid - za[k]).max() > 1e-3


def test_a_cache_given_from_outside_continues_like_the_one_computed():
    """set_cache (used to time a decode step at a chosen context length): the keys and values a real prefill
    stored, handed to a fresh rollout, give the same next step bit for bit."""
    m = O.OracleModel(DENSE, 3)
    t = _prompts(DENSE, (21,))
    a = O.OracleRollout(m, 8)
    i = a.add_sequence(5)
    r = a.prefill_chunk([i], t)
    kv = [a._gather(l, i, 21) for l in range(DENSE.n_layers)]
    b = O.OracleRollout(m, 8, alloc_order=[5, 2, 7, 0, 1, 3, 4, 6])
    j = b.add_sequence(5)
    b.set_cache(j, np.stack([k for k, _ in kv]), np.stack([v for _, v in kv]), r["tokens"][0])
    ra, rb = a.decode_step([i], want_logits=True), b.decode_step([j], want_logits=True)
    np.testing.assert_array_equal(ra["logits"][0], rb["logits"][0])
    assert ra["tokens"] == rb["tokens"] and ra["logprobs"] == rb["logprobs"] and b.ctx[j] == 22
