"""Seeded synthetic inputs and layer shapes for the FCDP hot path.

This module holds none of the method's arithmetic: it only names transformer
layer shapes and draws random values.  Both the HIP path and the CPU oracle
are fed from here (the same bytes go to both), and neither imports the other.

The paper trains GPT-2-XL-derived models on SQuAD (Sec. 5.1); neither the
weights nor the dataset are used here.  The path never touches token data, so
the stand-in is: transformer-layer *shapes* (GPT-2-small, Llama-2 7B/13B/70B)
with init-like value distributions -- parameters N(0, sigma=0.02) rounded to
bf16, gradient partials N(0, sigma=1e-3) in fp32, LoRA A uniform on
[-1/64, 1/64), LoRA B zero ("init") or N(0, sigma=1e-3) ("after a step").

Generators: ``numpy.random.Philox`` keyed by (SEED, stream id) on the host; a
seeded ``torch.Generator`` when buffers are drawn directly on the device for
full-size runs.  The two draw different values; every consumer of one buffer
sees the same bytes.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Sequence, Tuple

import numpy as np

SEED = 20260227

KIND_PARAM = 1
KIND_GRAD = 2
KIND_LORA_A = 3
KIND_LORA_B = 4
KIND_MISC = 5


@dataclasses.dataclass(frozen=True)
class LayerConfig:
    """Shape of one transformer layer as a list of flat tensors."""
    name: str
    config_id: int
    tensor_names: Tuple[str, ...]
    numel: Tuple[int, ...]
    trainable: Tuple[int, ...]      # 1 = trainable (W_t), 0 = frozen (W_f)
    kinds: Tuple[int, ...]          # KIND_* per tensor (value distribution)
    G: int                          # data-parallel ranks = shards per layer
    layers: int                     # layers in the stack
    pad_quantum: int = 64

    @property
    def N(self) -> int:
        return int(sum(self.numel))


def _gpt2_layer(hidden: int, ffn: int):
    names = ("ln_1.weight", "ln_1.bias", "attn.c_attn.weight",
             "attn.c_attn.bias", "attn.c_proj.weight", "attn.c_proj.bias",
             "ln_2.weight", "ln_2.bias", "mlp.c_fc.weight", "mlp.c_fc.bias",
             "mlp.c_proj.weight", "mlp.c_proj.bias")
    numel = (hidden, hidden, hidden * 3 * hidden, 3 * hidden,
             hidden * hidden, hidden, hidden, hidden, hidden * ffn, ffn,
             ffn * hidden, hidden)
    return names, numel


def _llama_layer(hidden: int, ffn: int, q_heads: int, kv_heads: int,
                 lora_rank: int = 0, lora_on: Sequence[str] = ()):
    head_dim = hidden // q_heads
    kv = kv_heads * head_dim
    base = [("q_proj", hidden * hidden), ("k_proj", kv * hidden),
            ("v_proj", kv * hidden), ("o_proj", hidden * hidden),
            ("gate_proj", ffn * hidden), ("up_proj", ffn * hidden),
            ("down_proj", hidden * ffn), ("input_layernorm", hidden),
            ("post_attention_layernorm", hidden)]
    out_dim = {"q_proj": hidden, "k_proj": kv, "v_proj": kv,
               "o_proj": hidden}
    names: List[str] = []
    numel: List[int] = []
    trainable: List[int] = []
    kinds: List[int] = []
    for nm, k in base:
        names.append(nm + ".weight")
        numel.append(k)
        trainable.append(0 if lora_rank else 1)
        kinds.append(KIND_PARAM)
        if lora_rank and nm in lora_on:
            names.append(nm + ".lora_A")
            numel.append(lora_rank * hidden)
            trainable.append(1)
            kinds.append(KIND_LORA_A)
            names.append(nm + ".lora_B")
            numel.append(out_dim[nm] * lora_rank)
            trainable.append(1)
            kinds.append(KIND_LORA_B)
    return tuple(names), tuple(numel), tuple(trainable), tuple(kinds)


def _mk_gpt2(name, cid, hidden, ffn, G, layers):
    names, numel = _gpt2_layer(hidden, ffn)
    return LayerConfig(name, cid, names, numel, (1,) * len(numel),
                       (KIND_PARAM,) * len(numel), G, layers)


def _mk_llama(name, cid, hidden, ffn, qh, kvh, G, layers, lora_rank=0,
              lora_on=()):
    names, numel, tr, kinds = _llama_layer(hidden, ffn, qh, kvh, lora_rank,
                                           lora_on)
    return LayerConfig(name, cid, names, numel, tr, kinds, G, layers)


CONFIGS: Dict[str, LayerConfig] = {
    # GPT-2-small layer: hidden 768, FFN 3072, all four linears with bias.
    "gpt2_small_g4": _mk_gpt2("gpt2_small_g4", 1, 768, 3072, 4, 1),
    # Llama-2-7B-shaped stack, 32 layers.
    "llama7b_g8": _mk_llama("llama7b_g8", 2, 4096, 11008, 32, 32, 8, 32),
    # PEFT on the 7B shape: LoRA rank 16 on q_proj and v_proj.
    "llama7b_lora_g8": _mk_llama("llama7b_lora_g8", 3, 4096, 11008, 32, 32,
                                 8, 32, 16, ("q_proj", "v_proj")),
    # 13B shape: 40 layers, every matrix straddles shard boundaries at G = 16.
    "llama13b_g16": _mk_llama("llama13b_g16", 4, 5120, 13824, 40, 40, 16, 40),
    # 70B shape with grouped-query attention: 64 query heads, 8 KV heads.
    "llama70b_g32": _mk_llama("llama70b_g32", 5, 8192, 28672, 64, 8, 32, 80),
}


def _stream_id(config_id: int, layer: int, kind: int, rank: int,
               tensor: int) -> int:
    return ((config_id & 0xFF) << 56) | ((kind & 0xFF) << 48) | \
        ((rank & 0xFFFF) << 32) | ((layer & 0xFFFF) << 16) | (tensor & 0xFFFF)


def rng(config_id: int, layer: int, kind: int, rank: int = 0,
        tensor: int = 0) -> np.random.Generator:
    """Counter-based generator keyed by (SEED, stream id)."""
    key = np.array([SEED, _stream_id(config_id, layer, kind, rank, tensor)],
                   dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round an fp32 array to bf16 with PyTorch's CPU cast; uint16 bits."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def layer_params_bf16(cfg: LayerConfig, layer: int,
                      lora_b: str = "zero") -> List[np.ndarray]:
    """Per-tensor bf16 parameters (uint16 bits) of one layer."""
    out = []
    for t, (k, kind) in enumerate(zip(cfg.numel, cfg.kinds)):
        g = rng(cfg.config_id, layer, kind, 0, t)
        if kind == KIND_LORA_A:
            x = g.random(k, dtype=np.float32) * np.float32(1 / 32) \
                - np.float32(1 / 64)
        elif kind == KIND_LORA_B:
            if lora_b == "zero":
                x = np.zeros(k, dtype=np.float32)
            else:
                x = g.standard_normal(k, dtype=np.float32) * np.float32(1e-3)
        else:
            x = g.standard_normal(k, dtype=np.float32) * np.float32(0.02)
        out.append(to_bf16_bits(x))
    return out


def grad_partial_f32(cfg: LayerConfig, layer: int, rank: int, count: int,
                     sigma: float = 1e-3) -> np.ndarray:
    """Rank `rank`'s fp32 partial gradient, `count` elements."""
    g = rng(cfg.config_id, layer, KIND_GRAD, rank, 0)
    return g.standard_normal(count, dtype=np.float32) * np.float32(sigma)


def random_layer(seed: int, T: int, max_numel: int, odd: bool = True
                 ) -> List[int]:
    """Random tensor sizes for property tests (odd sizes, zeros, ones)."""
    g = rng(0, seed, KIND_MISC)
    sizes = []
    for _ in range(T):
        c = int(g.integers(0, 10))
        if c == 0:
            sizes.append(0)
        elif c == 1:
            sizes.append(1)
        else:
            k = int(g.integers(1, max_numel + 1))
            if not odd:
                k = (k + 7) // 8 * 8
            sizes.append(k)
    return sizes


def torch_device_generator(device, config_id: int, layer: int, kind: int,
                           rank: int = 0):
    """Seeded torch generator on `device` for full-size on-device draws."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed((SEED * 1000003 + _stream_id(config_id, layer, kind, rank,
                                               0)) % (2 ** 63 - 1))
    return g
