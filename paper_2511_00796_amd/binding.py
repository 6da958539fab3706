"""ctypes binding of libhexdecode.so: the same names as include/hexdecode.h, argument marshalling
only.  PyTorch is used for device memory (``torch.empty``) and the current stream handle; every
step of the decode path runs in the library's HIP kernels.  There is no fallback: if the library
has not been built, ``load()`` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# HEXDECODE_LIB points at another build of the same library (e.g. one compiled with different tuning macros)
LIB_PATH = os.environ.get("HEXDECODE_LIB") or os.path.join(_HERE, "libhexdecode.so")

HX_OK, HX_E_NULL, HX_E_CONFIG, HX_E_SHAPE, HX_E_ALIGN, HX_E_TOO_SMALL, HX_E_RANGE, HX_E_HIP = 0, -1, -2, -3, -4, -5, -6, -7
(HX_T_EMBED, HX_T_G1, HX_T_WQKV, HX_T_BQKV, HX_T_WO, HX_T_G2, HX_T_WG, HX_T_WU, HX_T_WD, HX_T_GF,
 HX_T_WLM) = range(11)

EXPORTS = ["hx_last_error", "hx_weights_bytes", "hx_workspace_bytes", "hx_kv_bytes", "hx_engine_create",
           "hx_engine_destroy", "hx_weights_pack", "kv_alloc", "kv_free", "prefill_fill", "hx_kv_gather",
           "decode_step", "decode_step_sample", "decode_step_top_p", "prefill_chunk", "prefill_rows", "hx_prefill_workspace_bytes",
           "hx_validate_step_inputs", "hx_set_attn_capture", "hx_stage_schedule", "hx_attention_waves", "hx_plan_product",
           "hx_stage_rope_append", "hx_stage_attention", "hx_stage_attention_static", "hx_stage_rmsnorm", "hx_stage_linear", "hx_stage_linear_rows", "hx_stage_lm_head_top_p",
           "hx_profile_enable", "hx_profile_sample_every", "hx_profile_read"]

KERNEL_CLASSES = ["attention", "combine", "gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down", "gemm_lm", "norm",
                  "rope_append", "setup"]


class ModelConfig(C.Structure):
    _fields_ = [("struct_size", C.c_uint32)]
    _fields_ += [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim",
                                          "intermediate", "vocab", "block_size", "qkv_bias")]
    _fields_ += [("rms_eps", C.c_float), ("rope_theta", C.c_float), ("max_batch", C.c_int32),
                 ("max_seq_len", C.c_int32), ("kv_dtype", C.c_int32)]


HX_KV_BF16, HX_KV_FP8_E4M3 = 0, 1


class HexError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("hexdecode error %d: %s" % (code, text))
        self.code = code


_lib = None


def load():
    """Load libhexdecode.so (must have been built with ``paper_2511_00796_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libhexdecode.so is not built: run `python -m paper_2511_00796_amd.build` "
                           "(or __graft_entry__.build()); there is no CPU fallback")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    cfgp = C.POINTER(ModelConfig)
    L.hx_last_error.restype = C.c_char_p
    L.hx_last_error.argtypes = []
    sig = {
        "hx_weights_bytes": [cfgp, C.POINTER(sz)],
        "hx_workspace_bytes": [cfgp, C.POINTER(sz)],
        "hx_kv_bytes": [cfgp, i64, C.POINTER(sz)],
        "hx_engine_create": [cfgp, vp, sz, vp, sz, C.POINTER(vp)],
        "hx_engine_destroy": [vp],
        "hx_weights_pack": [vp, C.c_int, C.c_int, vp, i64, i64, vp],
        "kv_alloc": [vp, vp, sz, i64, C.POINTER(vp)],
        "kv_free": [vp],
        "prefill_fill": [vp, C.c_int, vp, vp, vp, vp, i32, i32, i64, vp],
        "hx_kv_gather": [vp, C.c_int, vp, vp, vp, vp, i32, i32, i64, vp],
        "decode_step": [vp, vp, i32, vp, vp, vp, vp, i32, vp, vp, vp],
        "prefill_chunk": [vp, vp, i32, vp, vp, vp, vp, i32, vp],
        "prefill_rows": [vp, vp, i32, vp, vp, vp, vp, i32, vp, sz, vp],
        "hx_prefill_workspace_bytes": [cfgp, i32, C.POINTER(sz)],
        "hx_validate_step_inputs": [vp, vp, i32, vp, vp, vp, vp, i32, vp],
        "decode_step_sample": [vp, vp, i32, vp, vp, vp, vp, i32, C.c_float, C.c_uint64, vp, vp, vp, vp, vp],
        "decode_step_top_p": [vp, vp, i32, vp, vp, vp, vp, i32, C.c_float, C.c_float, C.c_uint64, vp, vp, vp, vp, vp, vp],
        "hx_set_attn_capture": [vp, vp],
        "hx_stage_schedule": [vp, i32, vp, vp, vp, vp],
        "hx_attention_waves": [vp],
        "hx_plan_product": [i32, i32, i32, i32, vp, vp, vp],
        "hx_stage_rope_append": [vp, vp, C.c_int, i32, vp, vp, vp, i32, vp, vp],
        "hx_stage_attention": [vp, vp, C.c_int, i32, vp, vp, vp, i32, vp, vp],
        "hx_stage_attention_static": [vp, vp, C.c_int, i32, vp, vp, vp, i32, vp, vp],
        "hx_stage_rmsnorm": [vp, C.c_int, C.c_int, i32, vp, vp, vp],
        "hx_stage_linear": [vp, C.c_int, C.c_int, i32, vp, vp, vp, vp],
        "hx_stage_linear_rows": [vp, C.c_int, C.c_int, i32, vp, vp, vp, sz, vp],
        "hx_stage_lm_head_top_p": [vp, i32, vp, vp, vp, C.c_float, C.c_float, C.c_uint64, vp, vp, vp, vp, vp],
        "hx_profile_enable": [vp, C.c_uint32],
        "hx_profile_sample_every": [vp, C.c_int32],
        "hx_profile_read": [vp, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)],
    }
    for name, args in sig.items():
        f = getattr(L, name)
        f.restype = C.c_int
        f.argtypes = args
    _lib = L
    return L


def _check(rc: int) -> None:
    if rc != 0:
        raise HexError(rc, load().hx_last_error().decode())


def last_error() -> str:
    return load().hx_last_error().decode()


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_config(shape, max_batch: int, max_seq_len: int, kv_dtype: int = HX_KV_BF16) -> ModelConfig:
    """hx_model_config from any object with the ModelShape field names."""
    return ModelConfig(C.sizeof(ModelConfig), shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads,
                       shape.head_dim, shape.intermediate, shape.vocab, shape.block_size,
                       1 if shape.qkv_bias else 0, shape.rms_eps, shape.rope_theta, max_batch, max_seq_len, kv_dtype)


def weights_bytes(cfg: ModelConfig) -> int:
    out = C.c_size_t()
    _check(load().hx_weights_bytes(C.byref(cfg), C.byref(out)))
    return out.value


def prefill_workspace_bytes(cfg: ModelConfig, max_rows: int) -> int:
    out = C.c_size_t()
    _check(load().hx_prefill_workspace_bytes(C.byref(cfg), max_rows, C.byref(out)))
    return out.value


def workspace_bytes(cfg: ModelConfig) -> int:
    out = C.c_size_t()
    _check(load().hx_workspace_bytes(C.byref(cfg), C.byref(out)))
    return out.value


def kv_bytes(cfg: ModelConfig, num_blocks: int) -> int:
    out = C.c_size_t()
    _check(load().hx_kv_bytes(C.byref(cfg), num_blocks, C.byref(out)))
    return out.value


class Engine:
    """hx_engine plus the torch-owned device buffers it wraps."""

    def __init__(self, shape, max_batch: int, max_seq_len: int, device="cuda:0", kv_dtype: int = HX_KV_BF16,
                 weights: Optional[torch.Tensor] = None):
        """weights: the packed-weight buffer of another engine of the same shape, to share it (each engine has its
        own workspace, so two engines may run on two streams over one copy of the weights); None allocates one."""
        self.shape = shape
        self.cfg = make_config(shape, max_batch, max_seq_len, kv_dtype)
        self.device = torch.device(device)
        if weights is None:
            weights = torch.empty(weights_bytes(self.cfg), dtype=torch.uint8, device=self.device)
        assert weights.dtype == torch.uint8 and weights.is_cuda and weights.is_contiguous()
        self.weights = weights
        self.workspace = torch.empty(workspace_bytes(self.cfg), dtype=torch.uint8, device=self.device)
        h = C.c_void_p()
        _check(load().hx_engine_create(C.byref(self.cfg), _ptr(self.weights), self.weights.numel(),
                                       _ptr(self.workspace), self.workspace.numel(), C.byref(h)))
        self.handle = h
        self._capture = None

    def close(self) -> None:
        if self.handle:
            load().hx_engine_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- weights
    def weights_pack(self, kind: int, layer: int, src: torch.Tensor) -> None:
        assert src.dtype == torch.bfloat16 and src.is_cuda and src.is_contiguous()
        rows, cols = (src.shape[0], 1) if src.dim() == 1 else src.shape
        _check(load().hx_weights_pack(self.handle, kind, layer, _ptr(src), rows, cols, _stream()))

    def pack_layer(self, layer: int, w: Dict[str, torch.Tensor]) -> None:
        for name, kind in (("g1", HX_T_G1), ("wqkv", HX_T_WQKV), ("bqkv", HX_T_BQKV), ("wo", HX_T_WO),
                           ("g2", HX_T_G2), ("wg", HX_T_WG), ("wu", HX_T_WU), ("wd", HX_T_WD)):
            self.weights_pack(kind, layer, w[name].to(self.device))

    def pack_globals(self, w: Dict[str, torch.Tensor]) -> None:
        for name, kind in (("embed", HX_T_EMBED), ("gf", HX_T_GF), ("wlm", HX_T_WLM)):
            self.weights_pack(kind, 0, w[name].to(self.device))

    # -- decode
    def decode_step(self, kv: "KVCache", tokens, positions, seq_lens, block_table, logits: Optional[torch.Tensor],
                    next_tokens: torch.Tensor) -> None:
        B = tokens.numel()
        _check(load().decode_step(self.handle, kv.handle, B, _ptr(tokens), _ptr(positions), _ptr(seq_lens),
                                  _ptr(block_table), block_table.shape[1], _ptr(logits), _ptr(next_tokens), _stream()))

    def validate_step_inputs(self, kv: "KVCache", tokens, positions, seq_lens, block_table) -> None:
        """Raises HexError naming the first row whose device-side inputs are out of range (synchronises)."""
        _check(load().hx_validate_step_inputs(self.handle, kv.handle, tokens.numel(), _ptr(tokens), _ptr(positions),
                                              _ptr(seq_lens), _ptr(block_table), block_table.shape[1], _stream()))

    def prefill_chunk(self, kv: "KVCache", tokens, positions, seq_lens, block_table) -> None:
        """Rows = prompt tokens (<= max_batch); block_table holds one table row per ROW."""
        _check(load().prefill_chunk(self.handle, kv.handle, tokens.numel(), _ptr(tokens), _ptr(positions), _ptr(seq_lens),
                                    _ptr(block_table), block_table.shape[1], _stream()))

    def prefill_rows(self, kv: "KVCache", tokens, positions, seq_lens, block_table, workspace: torch.Tensor) -> None:
        """prefill_chunk for a multiple of 256 rows with the products over all rows at once; `workspace` is a device
        byte tensor of at least prefill_workspace_bytes(cfg, rows) bytes."""
        _check(load().prefill_rows(self.handle, kv.handle, tokens.numel(), _ptr(tokens), _ptr(positions), _ptr(seq_lens),
                                   _ptr(block_table), block_table.shape[1], _ptr(workspace), workspace.numel() * workspace.element_size(),
                                   _stream()))

    def decode_step_sample(self, kv: "KVCache", tokens, positions, seq_lens, block_table, temperature: float, seed: int,
                           logits: Optional[torch.Tensor], out_tokens: torch.Tensor, out_logprobs: torch.Tensor,
                           row_ids: Optional[torch.Tensor] = None) -> None:
        B = tokens.numel()
        _check(load().decode_step_sample(self.handle, kv.handle, B, _ptr(tokens), _ptr(positions), _ptr(seq_lens),
                                         _ptr(block_table), block_table.shape[1], C.c_float(temperature),
                                         C.c_uint64(seed), _ptr(row_ids), _ptr(logits), _ptr(out_tokens),
                                         _ptr(out_logprobs), _stream()))

    def decode_step_top_p(self, kv: "KVCache", tokens, positions, seq_lens, block_table, temperature: float, top_p: float,
                          seed: int, logits: Optional[torch.Tensor], out_tokens: torch.Tensor, out_logprobs: torch.Tensor,
                          row_ids: Optional[torch.Tensor] = None, out_sizes: Optional[torch.Tensor] = None) -> None:
        B = tokens.numel()
        _check(load().decode_step_top_p(self.handle, kv.handle, B, _ptr(tokens), _ptr(positions), _ptr(seq_lens),
                                        _ptr(block_table), block_table.shape[1], C.c_float(temperature), C.c_float(top_p),
                                        C.c_uint64(seed), _ptr(row_ids), _ptr(logits), _ptr(out_tokens),
                                        _ptr(out_logprobs), _ptr(out_sizes), _stream()))

    def set_attn_capture(self, buf: Optional[torch.Tensor]) -> None:
        self._capture = buf
        _check(load().hx_set_attn_capture(self.handle, _ptr(buf)))

    # -- per-kernel timing
    def profile_enable(self, classes, every: int = 1) -> None:
        """every: bracket only every n-th launch of the selected classes."""
        _check(load().hx_profile_sample_every(self.handle, every))
        mask = 0
        for c in classes:
            mask |= 1 << (KERNEL_CLASSES.index(c) if isinstance(c, str) else int(c))
        _check(load().hx_profile_enable(self.handle, mask))

    def profile_read(self, klass):
        k = KERNEL_CLASSES.index(klass) if isinstance(klass, str) else int(klass)
        ms, n = C.c_double(), C.c_int64()
        _check(load().hx_profile_read(self.handle, k, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    # -- single stages
    def attention_waves(self) -> int:
        return load().hx_attention_waves(self.handle)

    def stage_schedule(self, seq_lens: torch.Tensor):
        B = seq_lens.numel()
        prefix = torch.zeros(B + 1, dtype=torch.int32, device=self.device)
        sched = torch.zeros(2, dtype=torch.int32, device=self.device)
        _check(load().hx_stage_schedule(self.handle, B, _ptr(seq_lens), _ptr(prefix), _ptr(sched), _stream()))
        return prefix, sched

    def stage_rope_append(self, kv: "KVCache", layer: int, qkv: torch.Tensor, positions, block_table) -> torch.Tensor:
        B = qkv.shape[0]
        q = torch.empty(B, self.shape.n_q_heads * self.shape.head_dim, dtype=torch.float32, device=self.device)
        _check(load().hx_stage_rope_append(self.handle, kv.handle, layer, B, _ptr(qkv), _ptr(positions),
                                           _ptr(block_table), block_table.shape[1], _ptr(q), _stream()))
        return q

    def stage_attention(self, kv: "KVCache", layer: int, q: torch.Tensor, seq_lens, block_table) -> torch.Tensor:
        B = q.shape[0]
        out = torch.empty_like(q)
        _check(load().hx_stage_attention(self.handle, kv.handle, layer, B, _ptr(q), _ptr(seq_lens),
                                         _ptr(block_table), block_table.shape[1], _ptr(out), _stream()))
        return out

    def stage_attention_static(self, kv: "KVCache", layer: int, q: torch.Tensor, seq_lens, block_table, out: torch.Tensor) -> None:
        """hx_stage_attention_static: scratch in the library's static device array; `out` is provided by the caller."""
        _check(load().hx_stage_attention_static(self.handle, kv.handle, layer, q.shape[0], _ptr(q), _ptr(seq_lens),
                                                _ptr(block_table), block_table.shape[1], _ptr(out), _stream()))

    def stage_rmsnorm(self, gain_kind: int, layer: int, x: torch.Tensor) -> torch.Tensor:
        y = torch.empty_like(x)
        _check(load().hx_stage_rmsnorm(self.handle, gain_kind, layer, x.shape[0], _ptr(x), _ptr(y), _stream()))
        return y

    def stage_linear(self, kind: int, layer: int, x: torch.Tensor, want_argmax: bool = False):
        s = self.shape
        n_out = {HX_T_WQKV: s.qkv_dim, HX_T_WO: s.hidden, HX_T_WG: s.intermediate, HX_T_WD: s.hidden,
                 HX_T_WLM: s.vocab}[kind]
        B = x.shape[0]
        y = torch.empty(B, n_out, dtype=torch.float32, device=self.device)
        am = torch.empty(B, dtype=torch.int32, device=self.device) if want_argmax else None
        _check(load().hx_stage_linear(self.handle, kind, layer, B, _ptr(x), _ptr(y), _ptr(am), _stream()))
        return (y, am) if want_argmax else y

    def stage_linear_rows(self, kind: int, layer: int, x: torch.Tensor, workspace: torch.Tensor) -> torch.Tensor:
        """The product as prefill_rows runs it: x fp32 [rows (multiple of 256), in] -> y fp32 [rows, out]."""
        s = self.shape
        n_out = {HX_T_WQKV: s.qkv_dim, HX_T_WO: s.hidden, HX_T_WG: s.intermediate, HX_T_WD: s.hidden}[kind]
        y = torch.empty(x.shape[0], n_out, dtype=torch.float32, device=self.device)
        _check(load().hx_stage_linear_rows(self.handle, kind, layer, x.shape[0], _ptr(x), _ptr(y), _ptr(workspace),
                                           workspace.numel() * workspace.element_size(), _stream()))
        return y

    def stage_lm_head_top_p(self, x: torch.Tensor, positions: torch.Tensor, temperature: float, top_p: float, seed: int,
                            row_ids: Optional[torch.Tensor] = None):
        """-> (logits fp32 [B, vocab], tokens int32 [B], logprobs fp32 [B], kept-set sizes int32 [B])"""
        B = x.shape[0]
        y = torch.empty(B, self.shape.vocab, dtype=torch.float32, device=self.device)
        tok = torch.empty(B, dtype=torch.int32, device=self.device)
        lp = torch.empty(B, dtype=torch.float32, device=self.device)
        n = torch.empty(B, dtype=torch.int32, device=self.device)
        _check(load().hx_stage_lm_head_top_p(self.handle, B, _ptr(x), _ptr(positions), _ptr(row_ids), C.c_float(temperature),
                                             C.c_float(top_p), C.c_uint64(seed), _ptr(y), _ptr(tok), _ptr(lp), _ptr(n),
                                             _stream()))
        return y, tok, lp, n


class KVCache:
    """hx_kv plus the torch-owned pool it wraps."""

    def __init__(self, engine: Engine, num_blocks: int):
        self.engine = engine
        self.num_blocks = num_blocks
        self.pool = torch.empty(kv_bytes(engine.cfg, num_blocks), dtype=torch.uint8, device=engine.device)
        h = C.c_void_p()
        _check(load().kv_alloc(engine.handle, _ptr(self.pool), self.pool.numel(), num_blocks, C.byref(h)))
        self.handle = h

    def close(self) -> None:
        if self.handle:
            load().kv_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def prefill_fill(self, layer: int, k: torch.Tensor, v: torch.Tensor, seq_start: torch.Tensor,
                     block_table: torch.Tensor) -> None:
        assert k.dtype == torch.bfloat16 and k.is_contiguous() and v.is_contiguous()
        _check(load().prefill_fill(self.handle, layer, _ptr(k), _ptr(v), _ptr(seq_start), _ptr(block_table),
                                   block_table.shape[1], seq_start.numel() - 1, k.shape[0], _stream()))

    def gather(self, layer: int, total_tokens: int, seq_start: torch.Tensor, block_table: torch.Tensor):
        s = self.engine.shape
        k = torch.empty(total_tokens, s.n_kv_heads, s.head_dim, dtype=torch.bfloat16, device=self.engine.device)
        v = torch.empty_like(k)
        _check(load().hx_kv_gather(self.handle, layer, _ptr(k), _ptr(v), _ptr(seq_start), _ptr(block_table),
                                   block_table.shape[1], seq_start.numel() - 1, total_tokens, _stream()))
        return k, v
