"""CPU oracle of the decode step -- TEST INFRASTRUCTURE, not product code.

``decode_oracle.c`` states what the step computes; this file only compiles it with gcc, loads
it with ctypes and marshals numpy arrays into it.  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import this package; the HIP path never does.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "decode_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_LIB_DESC = os.path.join(_HERE, "liboracle_desc.so")

# plain IEEE arithmetic: no fast-math, no fused multiply-add contraction
_CFLAGS = ["-O2", "-ftree-vectorize", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-std=c11"]


def build(force: bool = True, descending: bool = False) -> str:
    """Compile the oracle with gcc.  AVX2 is used when this CPU has it (it only widens the
    loops that run over independent outputs; every sum keeps its order).  ``descending`` builds the
    sensitivity variant whose matrix products add their terms in descending k."""
    out = _LIB_DESC if descending else _LIB
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
        return out
    flags = list(_CFLAGS)
    if descending:
        flags.append("-DORC_SUM_DESCENDING")
    try:
        with open("/proc/cpuinfo") as f:
            if " avx2 " in f.read():
                flags.append("-mavx2")
    except OSError:
        pass
    tmp = out + ".tmp.%d" % os.getpid()
    subprocess.run(["gcc", *flags, _SRC, "-o", tmp, "-lm"], check=True)
    os.replace(tmp, out)
    return out


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim",
                                         "intermediate", "vocab", "block_size", "qkv_bias", "round_act", "kv_fp8")]
    _fields_ += [("rms_eps", C.c_float), ("rope_theta", C.c_float)]


class _Layer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("g1", "wqkv", "bqkv", "wo", "g2", "wg", "wu", "wd")]


class _Trace(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("u1", "qkv", "q", "k_new", "v_new", "o", "y_o", "x_mid", "u2", "m", "y_d")]


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("gf", C.c_void_p), ("wlm", C.c_void_p), ("layers", C.POINTER(_Layer))]


_lib = None
_lib_desc = None
_use_desc = False


class descending_sums:
    """Context manager: inside it every oracle call runs the variant built with
    -DORC_SUM_DESCENDING (same arithmetic, matrix-product terms added in the opposite order)."""

    def __enter__(self):
        global _use_desc
        self._prev = _use_desc
        _use_desc = True
        return self

    def __exit__(self, *exc):
        global _use_desc
        _use_desc = self._prev
        return False


def _load(path):
    L = C.CDLL(path)
    L.orc_bf16_to_f32.restype = C.c_float
    L.orc_bf16_to_f32.argtypes = [C.c_uint16]
    L.orc_f32_to_bf16.restype = C.c_uint16
    L.orc_f32_to_bf16.argtypes = [C.c_float]
    L.orc_silu.restype = C.c_float
    L.orc_silu.argtypes = [C.c_float]
    L.orc_argmax.restype = C.c_int32
    L.orc_head.restype = C.c_int32
    L.orc_decode_step.restype = C.c_int
    L.orc_num_threads.restype = C.c_int
    L.orc_e4m3_round.restype = C.c_float
    L.orc_e4m3_round.argtypes = [C.c_float]
    L.orc_uniform_open.restype = C.c_float
    L.orc_uniform_open.argtypes = [C.c_uint32]
    L.orc_sample.restype = None
    L.orc_sample.argtypes = [C.c_void_p, C.c_int, C.c_float, C.c_uint64, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p]
    L.orc_sample_top_p.restype = None
    L.orc_sample_top_p.argtypes = [C.c_void_p, C.c_int, C.c_float, C.c_float, C.c_uint64, C.c_uint32, C.c_uint32,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.orc_philox4x32_10.restype = None
    return L


def lib():
    """The loaded shared object (built on first use when absent or older than its source)."""
    global _lib, _lib_desc
    if _use_desc:
        if _lib_desc is None:
            _lib_desc = _load(build(force=False, descending=True))
        return _lib_desc
    if _lib is None:
        _lib = _load(build(force=False))
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def make_config(shape, round_act: bool = True, block_size: Optional[int] = None, kv_fp8: bool = False) -> _Config:
    """orc_config from any object with the ModelShape field names.  kv_fp8: the 8-bit (E4M3) cache variant."""
    return _Config(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                   shape.intermediate, shape.vocab, block_size or shape.block_size,
                   1 if shape.qkv_bias else 0, 1 if round_act else 0, 1 if kv_fp8 else 0, shape.rms_eps,
                   shape.rope_theta)


# ---- elementary operations (used by the pins) ------------------------------------------------

def e4m3_round(x) -> np.ndarray:
    """Nearest E4M3 value (ties to even, saturating at 448) of every fp32 element."""
    a = _f32(x)
    out = np.empty(a.shape, dtype=np.float32)
    f = lib().orc_e4m3_round
    flat_in, flat_out = a.reshape(-1), out.reshape(-1)
    for i in range(flat_in.size):
        flat_out[i] = f(C.c_float(float(flat_in[i])))
    return out


def bf16_round_bits(x) -> np.ndarray:
    """uint16 bf16 patterns of fp32 values, through the oracle's own rounding."""
    x = _f32(x)
    out = np.empty(x.shape, dtype=np.uint16)
    f = lib().orc_f32_to_bf16
    flat, o = x.reshape(-1), out.reshape(-1)
    for i in range(flat.size):
        o[i] = f(float(flat[i]))
    return out


def rmsnorm(x, g_bits, eps: float) -> np.ndarray:
    x = _f32(x)
    y = np.empty_like(x)
    lib().orc_rmsnorm(_p(x), _p(_u16(g_bits)), C.c_int(x.size), C.c_float(eps), _p(y))
    return y


def linear(x, w_bits, bias_bits=None) -> np.ndarray:
    x = _f32(x)
    w_bits = _u16(w_bits)
    K, N = w_bits.shape
    assert x.shape == (K,)
    y = np.empty(N, dtype=np.float32)
    lib().orc_linear(_p(x), _p(w_bits), _p(None if bias_bits is None else _u16(bias_bits)),
                     C.c_int(K), C.c_int(N), _p(y))
    return y


def rope(v, pos: int, theta: float) -> np.ndarray:
    v = _f32(v).copy()
    lib().orc_rope(_p(v), C.c_int(v.size), C.c_int(pos), C.c_float(theta))
    return v


def softmax(s) -> np.ndarray:
    s = _f32(s)
    p = np.empty_like(s)
    lib().orc_softmax(_p(s), C.c_int(s.size), _p(p))
    return p


def silu(x: float) -> float:
    return float(lib().orc_silu(C.c_float(x)))


def argmax(x) -> int:
    x = _f32(x)
    return int(lib().orc_argmax(_p(x), C.c_int(x.size)))


def philox4x32_10(ctr, key) -> np.ndarray:
    """One block of the counter-based generator: 4 counter words, 2 key words -> 4 output words."""
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    assert c.size == 4 and k.size == 2
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def uniform_open(word: int) -> float:
    return float(lib().orc_uniform_open(C.c_uint32(word)))


def sample(logits, temperature: float, seed: int, rows, positions):
    """Temperature sample (Gumbel-max over the counter-based generator) of every row of ``logits`` [B, V].
    Returns (tokens int32 [B], logprobs float32 [B], gaps float32 [B]); gap = best minus runner-up of the
    perturbed scores."""
    x = _f32(logits)
    if x.ndim == 1:
        x = x[None]
    B, V = x.shape
    rows = np.asarray(rows, dtype=np.uint32)
    positions = np.asarray(positions, dtype=np.uint32)
    tok = np.zeros(B, dtype=np.int32)
    lp = np.zeros(B, dtype=np.float32)
    gap = np.zeros(B, dtype=np.float32)
    for b in range(B):
        xb = np.ascontiguousarray(x[b])
        lib().orc_sample(_p(xb), V, C.c_float(temperature), C.c_uint64(seed), C.c_uint32(int(rows[b])),
                         C.c_uint32(int(positions[b])), tok[b:].ctypes.data, lp[b:].ctypes.data, gap[b:].ctypes.data)
    return tok, lp, gap


def sample_top_p(logits, temperature: float, top_p: float, seed: int, rows, positions):
    """Nucleus (top-p) sample of every row of ``logits`` [B, V] after temperature scaling.
    Returns (tokens int32 [B], logprobs float32 [B] under the renormalised kept set, sizes int32 [B] of the kept
    set, margins float64 [B]: distance of top_p from the running masses that decide the size, gaps float32 [B]:
    best minus runner-up perturbed score among the kept entries)."""
    x = _f32(logits)
    if x.ndim == 1:
        x = x[None]
    B, V = x.shape
    rows = np.asarray(rows, dtype=np.uint32)
    positions = np.asarray(positions, dtype=np.uint32)
    tok = np.zeros(B, dtype=np.int32)
    lp = np.zeros(B, dtype=np.float32)
    size = np.zeros(B, dtype=np.int32)
    margin = np.zeros(B, dtype=np.float64)
    gap = np.zeros(B, dtype=np.float32)
    for b in range(B):
        xb = np.ascontiguousarray(x[b])
        lib().orc_sample_top_p(_p(xb), V, C.c_float(temperature), C.c_float(top_p), C.c_uint64(seed),
                               C.c_uint32(int(rows[b])), C.c_uint32(int(positions[b])), tok[b:].ctypes.data,
                               lp[b:].ctypes.data, size[b:].ctypes.data, margin[b:].ctypes.data, gap[b:].ctypes.data)
    return tok, lp, size, margin, gap


# ---- model-level objects -----------------------------------------------------------------------

class Weights:
    """Host bf16 bit patterns (uint16 numpy arrays) of a whole model, in the oracle's structs."""

    def __init__(self, global_w: Dict[str, np.ndarray], layers: Sequence[Dict[str, np.ndarray]]):
        self._keep: List[np.ndarray] = []
        arr = (_Layer * len(layers))()
        for i, lw in enumerate(layers):
            for name in ("g1", "wqkv", "bqkv", "wo", "g2", "wg", "wu", "wd"):
                a = _u16(lw[name])
                self._keep.append(a)
                setattr(arr[i], name, a.ctypes.data)
        self._layers = arr
        g = {k: _u16(global_w[k]) for k in ("embed", "gf", "wlm")}
        self._keep.extend(g.values())
        self.struct = _Weights(g["embed"].ctypes.data, g["gf"].ctypes.data, g["wlm"].ctypes.data, arr)
        self.n_layers = len(layers)

    def layer(self, i: int) -> _Layer:
        return self._layers[i]


class PagedKV:
    """The oracle's own paged cache: per layer, K and V pools [num_blocks, block_size, n_kv_heads,
    head_dim] of bf16 bit patterns."""

    def __init__(self, cfg: _Config, num_blocks: int, n_layers: Optional[int] = None):
        L = cfg.n_layers if n_layers is None else n_layers
        shp = (num_blocks, cfg.block_size, cfg.n_kv_heads, cfg.head_dim)
        self.k = [np.zeros(shp, dtype=np.uint16) for _ in range(L)]
        self.v = [np.zeros(shp, dtype=np.uint16) for _ in range(L)]
        self.cfg = cfg
        self.kptr = (C.c_void_p * L)(*[a.ctypes.data for a in self.k])
        self.vptr = (C.c_void_p * L)(*[a.ctypes.data for a in self.v])

    def fill(self, layer: int, k_bits, v_bits, seq_start, block_table) -> None:
        """Scatter concatenated K/V rows [tokens, n_kv_heads, head_dim] of one layer."""
        bt = _i32(block_table)
        ss = _i32(seq_start)
        lib().orc_kv_fill(C.byref(self.cfg), _p(self.k[layer]), _p(self.v[layer]), _p(_u16(k_bits)),
                          _p(_u16(v_bits)), _p(ss), _p(bt), C.c_int(bt.shape[1]), C.c_int(ss.size - 1))


def attention(cfg: _Config, q, kpool, vpool, table_row, T: int) -> np.ndarray:
    """One sequence, one layer: q [n_q_heads*head_dim] fp32 -> o [n_q_heads*head_dim]."""
    q = _f32(q).reshape(-1)
    o = np.empty_like(q)
    lib().orc_attention(C.byref(cfg), _p(q), _p(_u16(kpool)), _p(_u16(vpool)), _p(_i32(table_row)),
                        C.c_int(T), _p(o))
    return o


def layer_step(cfg: _Config, layer: _Layer, x, pos: int, kpool, vpool, table_row,
               want_attn: bool = False, trace: Optional[dict] = None):
    """One decoder layer for one sequence; x (fp32 [hidden]) is updated in place.  trace: a dict that receives the
    layer's intermediate results (u1, qkv, q, k_new, v_new, o, y_o, x_mid, u2, m, y_d: see orc_trace)."""
    assert x.dtype == np.float32 and x.flags.c_contiguous
    attn = np.empty(cfg.n_q_heads * cfg.head_dim, dtype=np.float32) if want_attn else None
    if trace is None:
        lib().orc_layer_step(C.byref(cfg), C.byref(layer), _p(x), C.c_int(pos), _p(kpool), _p(vpool),
                             _p(_i32(table_row)), _p(attn))
        return attn
    H, QD, KD = cfg.hidden, cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    sizes = {"u1": H, "qkv": QD + 2 * KD, "q": QD, "k_new": KD, "v_new": KD, "o": QD, "y_o": H, "x_mid": H, "u2": H,
             "m": cfg.intermediate, "y_d": H}
    for name, n in sizes.items():
        trace[name] = np.empty(n, dtype=np.float32)
    tr = _Trace(*[trace[name].ctypes.data for name, _ in _Trace._fields_])
    lib().orc_layer_step_trace(C.byref(cfg), C.byref(layer), _p(x), C.c_int(pos), _p(kpool), _p(vpool),
                               _p(_i32(table_row)), _p(attn), C.byref(tr))
    return attn


def embed(cfg: _Config, w: Weights, token: int) -> np.ndarray:
    x = np.empty(cfg.hidden, dtype=np.float32)
    lib().orc_embed(C.byref(cfg), C.byref(w.struct), C.c_int32(token), _p(x))
    return x


def head(cfg: _Config, w: Weights, x):
    """Final norm + LM head + greedy token for one residual row."""
    logits = np.empty(cfg.vocab, dtype=np.float32)
    tok = lib().orc_head(C.byref(cfg), C.byref(w.struct), _p(_f32(x)), _p(logits))
    return logits, int(tok)


def decode_step(cfg: _Config, w: Weights, kv: PagedKV, tokens, positions, seq_lens, block_table,
                want_attn: bool = False):
    """One decode step for a batch.  Returns (logits [B, vocab], next_tokens [B], attn or None)
    where attn is [n_layers, B, n_q_heads*head_dim] before its bf16 rounding."""
    tokens, positions, seq_lens = _i32(tokens), _i32(positions), _i32(seq_lens)
    bt = _i32(block_table)
    B = tokens.size
    logits = np.empty((B, cfg.vocab), dtype=np.float32)
    nxt = np.empty(B, dtype=np.int32)
    attn = np.empty((cfg.n_layers, B, cfg.n_q_heads * cfg.head_dim), dtype=np.float32) if want_attn else None
    rc = lib().orc_decode_step(C.byref(cfg), C.byref(w.struct), C.c_int(B), _p(tokens), _p(positions),
                               _p(seq_lens), _p(bt), C.c_int(bt.shape[1]), kv.kptr, kv.vptr,
                               _p(logits), _p(nxt), _p(attn))
    if rc != 0:
        raise ValueError("seq_lens must equal positions + 1")
    return logits, nxt, attn


def full_causal(cfg: _Config, w: Weights, tokens, want_attn: bool = False):
    """Dense causal recomputation of all positions of one sequence (no cache, no paging)."""
    tokens = _i32(tokens)
    n = tokens.size
    logits = np.empty((n, cfg.vocab), dtype=np.float32)
    attn = np.empty((cfg.n_layers, n, cfg.n_q_heads * cfg.head_dim), dtype=np.float32) if want_attn else None
    lib().orc_full_causal(C.byref(cfg), C.byref(w.struct), _p(tokens), C.c_int(n), _p(logits), _p(attn))
    return logits, attn


def num_threads() -> int:
    return int(lib().orc_num_threads())
