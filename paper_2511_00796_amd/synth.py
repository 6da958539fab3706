"""Seeded synthetic workloads for the rollout decode step.

The paper evaluates rollout generation with distilled Qwen-2.5 checkpoints of 1.5B / 7B / 14B
parameters on a math-reasoning task whose response lengths follow a skewed, profiled
distribution (Section 5.2; Section 4.2.2).  Neither the checkpoints nor the task data are
available, so everything here is a stand-in: decoder shapes of those model sizes with random
weights, uniform / log-uniform ("long-tail") context lengths, random token ids and a randomly
permuted block table.

This module is the single producer of inputs for both the HIP path and the CPU checker.  It
holds none of the decode arithmetic: it only draws numbers (through torch / numpy generators),
casts them to bf16 with the library cast, and lays out index tables.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np
import torch

BASE_SEED = 2511007960


@dataclass(frozen=True)
class ModelShape:
    """Dimensions of a Qwen2-style decoder (GQA, rotate-half RoPE, SwiGLU, RMSNorm)."""

    name: str
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    intermediate: int
    vocab: int
    rms_eps: float = 1e-6
    rope_theta: float = 1e6
    block_size: int = 16
    qkv_bias: bool = True

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def qkv_dim(self) -> int:
        return self.q_dim + 2 * self.kv_dim

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def weight_elements(self) -> int:
        """Elements streamed once per step: every per-layer matrix, bias and gain, the final
        gain and the LM head (the embedding table is gathered, not streamed)."""
        per_layer = (self.hidden * self.qkv_dim + self.q_dim * self.hidden
                     + 3 * self.hidden * self.intermediate
                     + (self.qkv_dim if self.qkv_bias else 0) + 2 * self.hidden)
        return self.n_layers * per_layer + self.hidden * self.vocab + self.hidden

    def kv_bytes_per_token(self) -> int:
        """bf16 K and V of one token over all layers."""
        return 2 * self.kv_dim * 2 * self.n_layers


@dataclass(frozen=True)
class Workload:
    """One benchmark / parity configuration: a model shape plus a batch of ragged contexts."""

    name: str
    shape: ModelShape
    batch: int
    length_law: str          # "uniform", "loguniform" or "prompt"
    lo: int
    hi: int
    seed: int
    decode_steps: int = 1
    kv_fill: str = "normal"  # "normal": cache pre-filled with N(0,1); "model": produced by decoding


TINY = ModelShape("tiny", 2, 256, 4, 2, 64, 688, 1024)
QWEN_1P5B = ModelShape("qwen2-1.5b", 28, 1536, 12, 2, 128, 8960, 151936)
QWEN_7B = ModelShape("qwen2-7b", 28, 3584, 28, 4, 128, 18944, 152064)
QWEN_14B = ModelShape("qwen2-14b", 48, 5120, 40, 8, 128, 13824, 152064)

WORKLOADS: Dict[str, Workload] = {
    "tiny-b4": Workload("tiny-b4", TINY, 4, "prompt", 32, 128, BASE_SEED + 0, 16, "model"),
    "1.5b-b64": Workload("1.5b-b64", QWEN_1P5B, 64, "uniform", 512, 8192, BASE_SEED + 1),
    "1.5b-b256-longtail": Workload("1.5b-b256-longtail", QWEN_1P5B, 256, "loguniform", 256, 16384,
                                   BASE_SEED + 2),
    "7b-b128": Workload("7b-b128", QWEN_7B, 128, "uniform", 1024, 16384, BASE_SEED + 3),
    "14b-b64": Workload("14b-b64", QWEN_14B, 64, "uniform", 1024, 16384, BASE_SEED + 4),
}

# tensor kinds (also the sub-stream ids of the seeded generators)
T_EMBED, T_G1, T_WQKV, T_BQKV, T_WO, T_G2, T_WG, T_WU, T_WD, T_GF, T_WLM = range(11)
T_KFILL, T_VFILL, T_LENGTHS, T_TOKENS, T_TABLE = range(11, 16)


def stream_seed(seed: int, kind: int, layer: int = 0) -> int:
    """Seed of the sub-stream of one tensor: a fixed injective mix of (seed, kind, layer)."""
    return (int(seed) * 1_000_003 + kind * 10_007 + layer * 101 + 17) % (2 ** 62)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _normal_bf16(shape: Tuple[int, ...], mean: float, std: float, seed: int, device) -> torch.Tensor:
    """bf16 cast of N(mean, std^2) drawn in fp32 (chunked so that a 1e9-element tensor never
    holds a full fp32 copy)."""
    n = int(np.prod(shape))
    out = torch.empty(n, dtype=torch.bfloat16, device=device)
    g = _gen(device, seed)
    step = 1 << 26
    for s in range(0, n, step):
        e = min(n, s + step)
        out[s:e] = torch.randn(e - s, generator=g, device=device, dtype=torch.float32).mul_(std).add_(mean)
    return out.view(*shape)


def layer_weights(shape: ModelShape, layer: int, seed: int, device="cpu") -> Dict[str, torch.Tensor]:
    """bf16 tensors of one decoder layer, logical row-major ``[in, out]``.

    Projections ~ N(0, 0.02^2); q/k/v biases ~ N(0, 0.02^2); gains = 1 + N(0, 0.02^2) (a
    zero-mean gain would null the normalised activations).
    """
    H, I = shape.hidden, shape.intermediate
    w = {
        "g1": _normal_bf16((H,), 1.0, 0.02, stream_seed(seed, T_G1, layer), device),
        "wqkv": _normal_bf16((H, shape.qkv_dim), 0.0, 0.02, stream_seed(seed, T_WQKV, layer), device),
        "bqkv": _normal_bf16((shape.qkv_dim,), 0.0, 0.02, stream_seed(seed, T_BQKV, layer), device),
        "wo": _normal_bf16((shape.q_dim, H), 0.0, 0.02, stream_seed(seed, T_WO, layer), device),
        "g2": _normal_bf16((H,), 1.0, 0.02, stream_seed(seed, T_G2, layer), device),
        "wg": _normal_bf16((H, I), 0.0, 0.02, stream_seed(seed, T_WG, layer), device),
        "wu": _normal_bf16((H, I), 0.0, 0.02, stream_seed(seed, T_WU, layer), device),
        "wd": _normal_bf16((I, H), 0.0, 0.02, stream_seed(seed, T_WD, layer), device),
    }
    if not shape.qkv_bias:
        w["bqkv"].zero_()
    return w


def global_weights(shape: ModelShape, seed: int, device="cpu") -> Dict[str, torch.Tensor]:
    """Embedding table ``[V, H]``, final gain ``[H]`` and the (untied) LM head ``[H, V]``."""
    return {
        "embed": _normal_bf16((shape.vocab, shape.hidden), 0.0, 0.02, stream_seed(seed, T_EMBED), device),
        "gf": _normal_bf16((shape.hidden,), 1.0, 0.02, stream_seed(seed, T_GF), device),
        "wlm": _normal_bf16((shape.hidden, shape.vocab), 0.0, 0.02, stream_seed(seed, T_WLM), device),
    }


def context_lengths(wl: Workload) -> np.ndarray:
    """Tokens already cached per sequence before the decode step (int32 ``[batch]``).

    "uniform": integers uniform on [lo, hi]; "loguniform": round(exp(U(ln lo, ln hi))) clipped
    to [lo, hi] (the long-tail stand-in for the skewed response-length law of Section 4.2.2);
    "prompt": uniform prompt lengths on [lo, hi].
    """
    rng = np.random.Generator(np.random.PCG64(stream_seed(wl.seed, T_LENGTHS)))
    if wl.length_law in ("uniform", "prompt"):
        v = rng.integers(wl.lo, wl.hi + 1, size=wl.batch)
    elif wl.length_law == "loguniform":
        v = np.rint(np.exp(rng.uniform(math.log(wl.lo), math.log(wl.hi), size=wl.batch)))
        v = np.clip(v, wl.lo, wl.hi)
    else:
        raise ValueError(wl.length_law)
    return v.astype(np.int32)


def token_ids(wl: Workload, count: int, salt: int = 0) -> np.ndarray:
    """``count`` token ids uniform over the vocabulary (int32)."""
    rng = np.random.Generator(np.random.PCG64(stream_seed(wl.seed, T_TOKENS, salt)))
    return rng.integers(0, wl.shape.vocab, size=count).astype(np.int32)


def blocks_needed(seq_lens: np.ndarray, block_size: int) -> np.ndarray:
    return (np.asarray(seq_lens, dtype=np.int64) + block_size - 1) // block_size


def block_table(seq_lens: np.ndarray, block_size: int, seed: int, spare_blocks: int = 8,
                shuffle: bool = True, max_blocks_per_seq: int | None = None) -> Tuple[np.ndarray, int]:
    """Block table ``[batch, max_blocks_per_seq]`` (int32, -1 padded) over a pool of
    ``sum(ceil(T_b / block_size)) + spare_blocks`` physical blocks whose ids are one random
    permutation of the pool (identity when ``shuffle`` is false).  Returns (table, num_blocks).
    """
    need = blocks_needed(seq_lens, block_size)
    total = int(need.sum())
    num_blocks = total + spare_blocks
    ids = np.arange(num_blocks, dtype=np.int32)
    if shuffle:
        rng = np.random.Generator(np.random.PCG64(stream_seed(seed, T_TABLE)))
        ids = rng.permutation(num_blocks).astype(np.int32)
    width = int(need.max()) if max_blocks_per_seq is None else int(max_blocks_per_seq)
    if width < int(need.max()):
        raise ValueError("max_blocks_per_seq too small")
    table = np.full((len(need), width), -1, dtype=np.int32)
    at = 0
    for b, n in enumerate(need):
        table[b, :n] = ids[at:at + n]
        at += int(n)
    return table, num_blocks


def kv_fill(shape: ModelShape, layer: int, total_tokens: int, seed: int, device="cpu"
            ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Pre-filled cache content of one layer: K and V ``[total_tokens, n_kv_heads, head_dim]``
    bf16 ~ N(0, 1), sequences concatenated in batch order."""
    shp = (total_tokens, shape.n_kv_heads, shape.head_dim)
    k = _normal_bf16(shp, 0.0, 1.0, stream_seed(seed, T_KFILL, layer), device)
    v = _normal_bf16(shp, 0.0, 1.0, stream_seed(seed, T_VFILL, layer), device)
    return k, v


def algorithmic_bytes(shape: ModelShape, seq_lens: np.ndarray, kv_elem_bytes: int = 2) -> Dict[str, int]:
    """Bytes a decode step must move: every streamed weight once plus the K and V of every
    attended position (``seq_lens`` = keys attended per sequence, new token included).
    ``kv_elem_bytes``: 2 for the bf16 cache, 1 for the 8-bit variant."""
    w = 2 * shape.weight_elements()
    kv = int(np.asarray(seq_lens, dtype=np.int64).sum()) * shape.kv_bytes_per_token() * kv_elem_bytes // 2
    return {"weights": w, "kv": kv, "total": w + kv}


def as_u16(t: torch.Tensor) -> np.ndarray:
    """Bit pattern of a bf16 tensor as a contiguous uint16 numpy array on the host."""
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)
