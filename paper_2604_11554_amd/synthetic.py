"""Adapters from the seeded synthetic inputs (rollout_inputs) to the engine."""
from __future__ import annotations

import rollout_inputs as RI

from .engine import RolloutModel


FORMAT_IDS = {"bf16": 0, "f16": 1}   # rlx_model_config.dtype


def config_from_shape(s: RI.ModelShape, activation_split: int = 1, fmt: str = "bf16") -> dict:
    """fmt "f16": the FP16 precision option (one fp16 term per activation: activation_split is forced to 0)."""
    if fmt == "f16":
        activation_split = 0
    return dict(dtype=FORMAT_IDS[fmt], activation_split=activation_split, n_layers=s.n_layers, d_model=s.d_model, n_q_heads=s.n_q_heads, n_kv_heads=s.n_kv_heads,
                head_dim=s.head_dim, d_ff=s.d_ff, n_experts=s.n_experts, top_k=s.top_k,
                d_ff_expert=s.d_ff_expert, vocab=s.vocab, kv_block_size=s.kv_block_size, rms_eps=s.rms_eps,
                rope_theta=s.rope_theta, qk_norm=int(s.qk_norm), eos_token_id=s.eos_token_id,
                pad_token_id=s.pad_token_id)


def model_from_shape(s: RI.ModelShape, model_seed: int = 0, device="cuda:0", progress=None,
                     activation_split: int = 1, fmt: str = "bf16") -> RolloutModel:
    """Upload the keyed synthetic weights of `s` (same bit patterns the oracle upcasts)."""
    return RolloutModel(config_from_shape(s, activation_split, fmt),
                        lambda l, n: RI.tensor_bits(s, model_seed, l, n, fmt), device, progress)


def device_random_tensor(s: RI.ModelShape, model_seed: int = 0, fmt: str = "bf16", device="cuda:0"):
    """tensor(layer, name) -> random-init weights of shape `s` drawn on the device, a pure function of
    (model_seed, layer, name), with the distributions of rollout_inputs (matrices N(0, 0.02), gains
    1 + N(0, 0.02), router rows N(0, 1/d_model)) but torch's generator: for models too large to draw on the host."""
    import numpy as np
    import torch
    gen = torch.Generator(device=device)

    def tensor(layer, name):
        dims, kind = RI.tensor_names(s, layer)[name]
        gen.manual_seed((model_seed * 1000003 + (layer + 1) * 101 + sum(map(ord, name))) & 0x7FFFFFFF)
        t = torch.randn(dims, generator=gen, device=device, dtype=torch.float32)
        if kind == "matrix":
            t.mul_(0.02)
        elif kind == "gain":
            t.mul_(0.02).add_(1.0)
        else:
            t.mul_(1.0 / np.sqrt(s.d_model))
        return t.to(torch.float16 if fmt == "f16" else torch.bfloat16)

    return tensor


def device_random_model(s: RI.ModelShape, model_seed: int = 0, activation_split: int = 1, fmt: str = "bf16",
                        device="cuda:0") -> RolloutModel:
    return RolloutModel(config_from_shape(s, activation_split, fmt), device_random_tensor(s, model_seed, fmt, device),
                        device)


def generate_tensors(s: RI.ModelShape, model_seed: int = 0, threads: int = 8, progress=None,
                     fmt: str = "bf16") -> dict:
    """All bit patterns of a synthetic model, {(layer, name): uint16 array}, generated on several
    host threads (NumPy's generators release the GIL)."""
    from concurrent.futures import ThreadPoolExecutor
    keys = [(l, n) for l in [RI.GLOBAL_LAYER] + list(range(s.n_layers)) for n in RI.tensor_names(s, l)]
    out = {}

    def make(key):
        return key, RI.tensor_bits(s, model_seed, key[0], key[1], fmt)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        for i, (key, bits) in enumerate(ex.map(make, keys)):
            out[key] = bits
            if progress and i % 32 == 0:
                progress(i, len(keys))
    return out


def model_from_tensors(s: RI.ModelShape, tensors: dict, device="cuda:0", activation_split: int = 1,
                       progress=None, fmt: str = "bf16") -> RolloutModel:
    return RolloutModel(config_from_shape(s, activation_split, fmt), lambda l, n: tensors[(l, n)], device, progress)
