"""Host logic of bench.py: the algorithmic byte and flop counts that the roofline figures are quoted against are
checked with numbers worked out by hand from the two benchmark shapes (dimensions written out here, not read from
the shape objects), the counted experts against a table built by hand, and the argument handling that needs no GPU."""
import os
import subprocess
import sys

import numpy as np
import pytest
import torch

import rollout_inputs as RI

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_shapes_are_the_ones_the_hand_numbers_assume():
    s = RI.QWEN3_4B
    assert (s.n_layers, s.d_model, s.n_q_heads, s.n_kv_heads, s.head_dim, s.d_ff, s.vocab) == (36, 2560, 32, 8, 128, 9728, 151936)
    m = RI.QWEN3_30B_A3B
    assert (m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.d_ff_expert, m.n_experts, m.top_k, m.vocab) == (
        48, 2048, 32, 4, 128, 768, 128, 8, 151936)


def test_dense_step_bytes_by_hand():
    # per layer, parameters: q|k|v 2560 x (32 + 2 x 8) x 128 = 15 728 640; output 4096 x 2560 = 10 485 760;
    # gate, up, down 3 x 2560 x 9728 = 74 711 040; 36 layers: 3 633 315 840; LM head 151 936 x 2560 = 388 956 160
    weights = 2 * (36 * (15_728_640 + 10_485_760 + 74_711_040) + 388_956_160)
    assert weights == 8_044_544_000
    kv_tok = 2 * 2 * 36 * 8 * 128                    # K and V, two bytes, every layer and KV head
    assert kv_tok == 147_456
    ctx_plus_b, batch = 72_391, 64
    assert bench.step_bytes(RI.QWEN3_4B, ctx_plus_b, batch) == weights + kv_tok * ctx_plus_b + kv_tok * batch
    assert bench.step_bytes(RI.QWEN3_4B, 0, 0) == weights


def test_dense_kernel_bytes_by_hand():
    s = RI.QWEN3_4B
    assert bench.kernel_bytes(s, "attn", 72_391) == 72_391 * 8 * 128 * 4        # K and V of every attended position
    assert bench.kernel_bytes(s, "qkv", 0) == 2 * 15_728_640
    assert bench.kernel_bytes(s, "oproj", 0) == 2 * 10_485_760
    assert bench.kernel_bytes(s, "gateup", 0) == 2 * 2 * 2560 * 9728
    assert bench.kernel_bytes(s, "down", 0) == 2 * 2560 * 9728
    assert bench.kernel_bytes(s, "lmhead", 0) == 2 * 388_956_160
    with pytest.raises(KeyError):
        bench.kernel_bytes(s, "norm", 0)


def test_moe_step_bytes_by_hand():
    # per layer: q|k|v 2048 x (32 + 8) x 128 = 10 485 760; output 4096 x 2048 = 8 388 608; router 128 x 2048 = 262 144;
    # an expert: 3 x 2048 x 768 = 4 718 592 parameters, streamed once per step if any token of the batch chose it
    touched = 127.5
    per_layer = 10_485_760 + 8_388_608 + 262_144 + touched * 4_718_592
    weights = 2 * (48 * per_layer + 151_936 * 2048)
    kv_tok = 2 * 2 * 48 * 4 * 128
    assert kv_tok == 98_304
    got = bench.step_bytes(RI.QWEN3_30B_A3B, 196_801, 128, touched)
    assert got == pytest.approx(weights + kv_tok * (196_801 + 128), rel=1e-12)
    assert bench.kernel_bytes(RI.QWEN3_30B_A3B, "gateup", 0, 128.0) == 128 * 2 * 2048 * 768 * 2
    assert bench.kernel_bytes(RI.QWEN3_30B_A3B, "down", 0, 128.0) == 128 * 2048 * 768 * 2


def test_prefill_flops_by_hand():
    # one 3-token sequence on the 4B shape: linear layers 2 x parameters per token, attention q.k and p.v over the
    # causal triangle (1 + 2 + 3 = 6 query-key pairs), the LM head on the sampled row only
    lin = 2.0 * (15_728_640 + 10_485_760 + 74_711_040) * 36 * 3
    attn = 2.0 * 2 * 4096 * 6 * 36
    head = 2.0 * 388_956_160
    assert bench.prefill_flops(RI.QWEN3_4B, np.array([3])) == pytest.approx(lin + attn + head, rel=1e-12)
    # behind 5 cached positions every query also sees those: 3 x 5 more pairs
    more = 2.0 * 2 * 4096 * 15 * 36
    assert bench.prefill_flops(RI.QWEN3_4B, np.array([3]), np.array([5])) == pytest.approx(lin + attn + more + head, rel=1e-12)
    # MoE: router + top-8 experts per token instead of the dense FFN
    per_tok = 10_485_760 + 8_388_608 + 262_144 + 8 * 4_718_592
    assert bench.prefill_flops(RI.QWEN3_30B_A3B, np.array([1])) == pytest.approx(
        2.0 * per_tok * 48 + 2.0 * 2 * 4096 * 1 * 48 + 2.0 * 151_936 * 2048, rel=1e-12)


def test_touched_experts_counts_distinct_ids_per_layer():
    shape = RI.TINY_MOE
    e, k, layers = shape.n_experts, shape.top_k, shape.n_layers
    steps, batch = 2, 3
    r = torch.zeros((steps, batch, layers, k), dtype=torch.int32)
    # step 0: every token picks experts 0 .. k-1 in every layer -> k distinct per layer
    r[0] = torch.arange(k, dtype=torch.int32)
    # step 1, layer 0: token b picks b, b+1, ... (wrapping) -> k + batch - 1 distinct (if it fits); other layers as step 0
    r[1] = torch.arange(k, dtype=torch.int32)
    for b in range(batch):
        r[1, b, 0] = (torch.arange(k) + b) % e
    want0 = float(k)
    want1 = (min(e, k + batch - 1) + (layers - 1) * k) / layers
    got = bench.touched_experts(r, shape)
    assert got.shape == (steps,)
    assert float(got[0]) == pytest.approx(want0)
    assert float(got[1]) == pytest.approx(want1)


def test_traffic_record_is_dropped_when_the_sources_change(tmp_path, monkeypatch):
    ratio, src = bench.traffic_record("dense_b64", "attn")
    if ratio is not None:                            # the committed record matches the committed sources
        assert src == os.path.join("profiles", "attn_decode_dense_b64_traffic.txt")
        assert 0.9 < ratio < 1.5
    assert bench.traffic_record("dense_b64", "no_such_class") == (None, None)
    # the same record next to sources with another content: no ratio
    fake = tmp_path / "repo"
    (fake / "profiles").mkdir(parents=True)
    (fake / "paper_2604_11554_amd" / "csrc").mkdir(parents=True)
    rec = open(os.path.join(ROOT, "profiles", "attn_decode_dense_b64_traffic.txt")).read()
    (fake / "profiles" / "attn_decode_dense_b64_traffic.txt").write_text(rec)
    for f in ("attention_decode.hip", "attn_core.h", "common.h"):
        (fake / "paper_2604_11554_amd" / "csrc" / f).write_text("// changed\n")
    monkeypatch.setattr(bench, "ROOT", str(fake))
    assert bench.traffic_record("dense_b64", "attn") == (None, None)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""
