"""Seeded synthetic inputs for the fused decoder-block forward.

This module only *draws numbers and changes their storage type*.  It holds none
of the arithmetic of the method (no norm, no matmul, no softmax): the CPU oracle
and the HIP library both receive the arrays produced here, and neither imports
the other.

The paper evaluates on pretrained models (Sec. "Models and Architectural
Diversity", the model table) and 128-token text windows (Sec. "Datasets").
Neither the weights nor the text exist here, so random tensors with the same
shapes stand in: weights ~ N(0, 0.02), activations ~ N(0, 1), token ids uniform
over the vocabulary.

Every tensor has its own stream: ``PCG64(SeedSequence([16498, config, layer,
slot]))`` so a single tensor can be regenerated without generating the rest.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

BASE_SEED = 16498

# ----------------------------------------------------------------------------
# storage-type conversion (bf16 <-> fp32), round-to-nearest-even
# ----------------------------------------------------------------------------


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 array holding the bf16 bit patterns (RNE, NaN kept quiet)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    out = rounded.astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> fp32 array (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """fp32 array -> fp32 array whose values are all exactly representable in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


# ----------------------------------------------------------------------------
# streams
# ----------------------------------------------------------------------------

# slot numbers: the order of the weight pointers in the block descriptor, then
# the model-level tensors and the activations
_SLOTS = {
    "norm1_g": 0, "norm1_b": 1, "w_qkv": 2, "b_qkv": 3, "w_o": 4, "b_o": 5,
    "norm2_g": 6, "norm2_b": 7, "w_up": 8, "b_up": 9, "w_down": 10, "b_down": 11,
    "x": 20, "k_cache": 21, "v_cache": 22, "ids": 23,
    "wte": 30, "wpe": 31, "normf_g": 32, "normf_b": 33,
    "q": 40, "k": 41, "v": 42, "delta": 43, "residual": 44, "misc": 45,
}


def rng_for(config: int, layer: int, slot: str | int) -> np.random.Generator:
    s = _SLOTS[slot] if isinstance(slot, str) else int(slot)
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([BASE_SEED, config, layer, s])))


def normal(config: int, layer: int, slot: str | int, shape, std: float = 1.0,
           mean: float = 0.0, bf16: bool = False) -> np.ndarray:
    """fp32 N(mean, std) tensor; with bf16=True the values are bf16-representable."""
    g = rng_for(config, layer, slot)
    a = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if mean != 0.0:
        a += np.float32(mean)
    return bf16_round(a) if bf16 else a


def token_ids(config: int, batch: int, seq: int, vocab: int) -> np.ndarray:
    g = rng_for(config, 0, "ids")
    return g.integers(0, vocab, size=(batch, seq), dtype=np.int64).astype(np.int32)


# ----------------------------------------------------------------------------
# shapes
# ----------------------------------------------------------------------------


@dataclass(frozen=True)
class BlockShape:
    """One decoder layer's shape and flavour (plain data)."""
    d_model: int
    q_heads: int
    kv_heads: int
    head_dim: int
    d_ff: int
    norm: str = "layernorm"        # "layernorm" | "rmsnorm"
    eps: float = 1e-5
    mlp_act: str = "gelu_tanh"     # "gelu_tanh" | "swiglu"
    use_rope: bool = False
    rope_base: float = 10000.0
    has_bias: bool = True

    @property
    def qkv_out(self) -> int:
        return (self.q_heads + 2 * self.kv_heads) * self.head_dim

    @property
    def up_out(self) -> int:
        return 2 * self.d_ff if self.mlp_act == "swiglu" else self.d_ff


@dataclass(frozen=True)
class Workload:
    """One of the five evaluation configurations."""
    cid: int
    name: str
    block: BlockShape
    layers: int
    batch: int
    seq: int                # new tokens per sequence in one forward
    pos0: int = 0           # cache positions already filled (decode: 2048)
    bf16: bool = True
    vocab: int = 0          # 0: hidden-state input, no embedding / LM head
    n_pos: int = 0          # learned position rows
    bias_std: float = 0.02  # std of the linear biases (0 -> zeros)


GPT2_SMALL = BlockShape(768, 12, 12, 64, 3072)
OPT_1P3B = BlockShape(2048, 16, 16, 128, 8192)
LLAMA_8B = BlockShape(4096, 32, 8, 128, 14336, norm="rmsnorm", mlp_act="swiglu",
                      use_rope=True, rope_base=500000.0, has_bias=False)

WORKLOADS: Dict[int, Workload] = {
    1: Workload(1, "gpt2s_layer_fp32_b1_s128", GPT2_SMALL, 1, 1, 128, bf16=False, bias_std=0.0),
    2: Workload(2, "gpt2s_12L_bf16_b8_s1024", GPT2_SMALL, 12, 8, 1024, vocab=50257, n_pos=1024),
    3: Workload(3, "1p3b_24L_bf16_b4_s2048", OPT_1P3B, 24, 4, 2048, vocab=50272, n_pos=2048),
    4: Workload(4, "llama8b_32L_bf16_b1_s4096_prefill", LLAMA_8B, 32, 1, 4096),
    5: Workload(5, "llama8b_32L_bf16_b64_decode_kv2048", LLAMA_8B, 32, 64, 1, pos0=2048),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (smaller batch, fewer layers...)."""
    return replace(w, **kw)


# ----------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------


def block_weights(shape: BlockShape, config: int, layer: int, bf16: bool,
                  bias_std: float = 0.02, random_affine: bool = False,
                  weight_std: float = 0.02) -> Dict[str, Optional[np.ndarray]]:
    """Weights of one layer as fp32 arrays (bf16-representable when bf16=True).

    Linear weights are [out_features, in_features].  ``w_up`` of a SwiGLU block
    is [2*d_ff, d]: the gate rows first, the up rows after them.
    Norm gains are 1 and shifts 0 unless random_affine (used by parity tests so
    that the affine step is exercised).
    """
    d = shape.d_model

    def lin(slot, rows, cols):
        return normal(config, layer, slot, (rows, cols), weight_std, bf16=bf16)

    def bias(slot, n):
        if not shape.has_bias:
            return None
        if bias_std == 0.0:
            return np.zeros(n, np.float32)
        return normal(config, layer, slot, (n,), bias_std, bf16=bf16)

    def gain(slot):
        if random_affine:
            return normal(config, layer, slot, (d,), 0.1, mean=1.0, bf16=bf16)
        return np.ones(d, np.float32)

    def shift(slot):
        if shape.norm == "rmsnorm":
            return None
        if random_affine:
            return normal(config, layer, slot, (d,), 0.1, bf16=bf16)
        return np.zeros(d, np.float32)

    return {
        "norm1_g": gain("norm1_g"), "norm1_b": shift("norm1_b"),
        "w_qkv": lin("w_qkv", shape.qkv_out, d), "b_qkv": bias("b_qkv", shape.qkv_out),
        "w_o": lin("w_o", d, shape.q_heads * shape.head_dim), "b_o": bias("b_o", d),
        "norm2_g": gain("norm2_g"), "norm2_b": shift("norm2_b"),
        "w_up": lin("w_up", shape.up_out, d), "b_up": bias("b_up", shape.up_out),
        "w_down": lin("w_down", d, shape.d_ff), "b_down": bias("b_down", d),
    }


def model_weights(w: Workload, random_affine: bool = False) -> Dict[str, Optional[np.ndarray]]:
    """Model-level tensors: token table (also the LM head: tied), positions, final norm."""
    d = w.block.d_model
    out: Dict[str, Optional[np.ndarray]] = {}
    if w.vocab:
        out["wte"] = normal(w.cid, 0, "wte", (w.vocab, d), 0.02, bf16=w.bf16)
        out["wpe"] = normal(w.cid, 0, "wpe", (w.n_pos, d), 0.02, bf16=w.bf16)
    if random_affine:
        out["normf_g"] = normal(w.cid, 0, "normf_g", (d,), 0.1, mean=1.0, bf16=w.bf16)
        out["normf_b"] = (None if w.block.norm == "rmsnorm"
                          else normal(w.cid, 0, "normf_b", (d,), 0.1, bf16=w.bf16))
    else:
        out["normf_g"] = np.ones(d, np.float32)
        out["normf_b"] = None if w.block.norm == "rmsnorm" else np.zeros(d, np.float32)
    return out


def hidden_states(w: Workload, batch: Optional[int] = None, seq: Optional[int] = None) -> np.ndarray:
    b = w.batch if batch is None else batch
    s = w.seq if seq is None else seq
    return normal(w.cid, 0, "x", (b, s, w.block.d_model), 1.0, bf16=w.bf16)


def kv_cache(w: Workload, layer: int, which: str, batch: int, cap: int, filled: int) -> np.ndarray:
    """[B, Hkv, cap, dh] cache; the first ``filled`` positions ~ N(0,1), the rest zero."""
    sh = w.block
    a = np.zeros((batch, sh.kv_heads, cap, sh.head_dim), np.float32)
    if filled:
        a[:, :, :filled, :] = normal(w.cid, layer, which, (batch, sh.kv_heads, filled, sh.head_dim),
                                     1.0, bf16=w.bf16)
    return a
