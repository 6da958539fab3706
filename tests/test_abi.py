"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header
declares, its pure-host entry points (size queries, argument validation) behave as documented."""
import ctypes as C
import os
import re

import pytest

from paper_2511_00796_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hexdecode.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(?:int|const char \*)\s*\*?\s*([a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS), sorted(set(names) ^ set(binding.EXPORTS))
    for n in names:
        assert hasattr(lib, n), n


def test_size_queries_are_consistent_with_the_shapes():
    for wl in synth.WORKLOADS.values():
        s = wl.shape
        cfg = binding.make_config(s, wl.batch, 16400)
        wb = binding.weights_bytes(cfg)
        # packed weights = streamed weights + embedding table, plus padding only
        logical = 2 * (s.weight_elements() + s.vocab * s.hidden)
        assert logical <= wb <= logical * 1.01 + (1 << 20)
        assert binding.kv_bytes(cfg, 1000) == s.n_layers * 1000 * s.n_kv_heads * 2 * 16 * s.head_dim * 2
        assert binding.workspace_bytes(cfg) > 0


def test_bad_configurations_are_rejected_with_codes_not_crashes():
    s = synth.TINY
    good = binding.make_config(s, 4, 256)
    assert binding.weights_bytes(good) > 0

    def expect(code, **kw):
        cfg = binding.make_config(s, 4, 256)
        for k, v in kw.items():
            setattr(cfg, k, v)
        out = C.c_size_t()
        rc = binding.load().hx_weights_bytes(C.byref(cfg), C.byref(out))
        assert rc == code, (kw, rc, binding.last_error())
        assert binding.last_error()

    expect(binding.HX_E_CONFIG, struct_size=8)
    expect(binding.HX_E_CONFIG, head_dim=96)
    expect(binding.HX_E_CONFIG, n_q_heads=5)
    expect(binding.HX_E_CONFIG, n_q_heads=34)          # 17 query heads per KV head
    expect(binding.HX_E_CONFIG, hidden=250)
    expect(binding.HX_E_CONFIG, intermediate=100)
    expect(binding.HX_E_CONFIG, block_size=32)
    expect(binding.HX_E_CONFIG, max_batch=0)
    expect(binding.HX_E_CONFIG, max_batch=257)
    expect(binding.HX_E_CONFIG, vocab=1023)
    lib = binding.load()
    assert lib.hx_weights_bytes(None, C.byref(C.c_size_t())) == binding.HX_E_NULL
    assert lib.hx_weights_bytes(C.byref(good), None) == binding.HX_E_NULL
    out = C.c_size_t()
    assert lib.hx_kv_bytes(C.byref(good), 0, C.byref(out)) == binding.HX_E_RANGE


def test_engine_create_validates_buffers_on_the_host():
    lib = binding.load()
    cfg = binding.make_config(synth.TINY, 4, 256)
    wb, sb = binding.weights_bytes(cfg), binding.workspace_bytes(cfg)
    h = C.c_void_p()
    fake = 0x10000000   # never dereferenced: creation only records addresses
    assert lib.hx_engine_create(C.byref(cfg), None, wb, fake, sb, C.byref(h)) == binding.HX_E_NULL
    assert lib.hx_engine_create(C.byref(cfg), fake + 8, wb, fake, sb, C.byref(h)) == binding.HX_E_ALIGN
    assert lib.hx_engine_create(C.byref(cfg), fake, wb - 1, fake, sb, C.byref(h)) == binding.HX_E_TOO_SMALL
    assert lib.hx_engine_create(C.byref(cfg), fake, wb, fake, sb - 1, C.byref(h)) == binding.HX_E_TOO_SMALL
    assert lib.hx_engine_create(C.byref(cfg), fake, wb, fake, sb, C.byref(h)) == binding.HX_OK
    eng = h
    kvh = C.c_void_p()
    kb = binding.kv_bytes(cfg, 10)
    assert lib.kv_alloc(eng, fake, kb - 1, 10, C.byref(kvh)) == binding.HX_E_TOO_SMALL
    assert lib.kv_alloc(eng, fake, kb, 10, C.byref(kvh)) == binding.HX_OK
    # scalar validation of the step happens before anything is enqueued
    p = C.c_void_p(fake)
    assert lib.decode_step(eng, kvh, 0, p, p, p, p, 4, None, p, None) == binding.HX_E_RANGE
    assert lib.decode_step(eng, kvh, 5, p, p, p, p, 4, None, p, None) == binding.HX_E_RANGE
    assert lib.decode_step(eng, kvh, 4, p, p, p, p, 0, None, p, None) == binding.HX_E_RANGE
    assert lib.decode_step(eng, kvh, 4, None, p, p, p, 4, None, p, None) == binding.HX_E_NULL
    assert lib.decode_step(None, kvh, 4, p, p, p, p, 4, None, p, None) == binding.HX_E_NULL
    f32 = C.c_float
    assert lib.decode_step_sample(eng, kvh, 4, p, p, p, p, 4, f32(0.0), 1, None, None, p, p, None) == binding.HX_E_RANGE
    assert lib.decode_step_sample(eng, kvh, 4, p, p, p, p, 4, f32(-2.0), 1, None, None, p, p, None) == binding.HX_E_RANGE
    assert lib.decode_step_sample(eng, kvh, 4, p, p, p, p, 4, f32(float("nan")), 1, None, None, p, p, None) == binding.HX_E_RANGE
    assert lib.decode_step_sample(eng, kvh, 4, p, p, p, p, 4, f32(1.0), 1, None, None, p, None, None) == binding.HX_E_NULL
    assert lib.decode_step_sample(eng, kvh, 9, p, p, p, p, 4, f32(1.0), 1, None, None, p, p, None) == binding.HX_E_RANGE
    assert lib.hx_weights_pack(eng, binding.HX_T_WO, 0, p, 3, 3, None) == binding.HX_E_SHAPE
    assert lib.hx_weights_pack(eng, binding.HX_T_WO, 9, p, 256, 256, None) == binding.HX_E_SHAPE
    assert lib.hx_weights_pack(eng, 99, 0, p, 256, 256, None) == binding.HX_E_SHAPE
    assert lib.kv_free(kvh) == binding.HX_OK
    assert lib.hx_engine_destroy(eng) == binding.HX_OK
    assert lib.hx_engine_destroy(None) == binding.HX_E_NULL


def test_product_plans_fill_the_chip_and_respect_their_limits():
    """Host-side launch planner: every plan keeps at least 16 k-steps per split, never splits a product whose epilogue
    needs the whole sum, stays within 9 splits and 4..6 tiles per workgroup (10 only for unsplit products of up to 128 rows),
    and for the 7B shapes picks the plans the design rests on (gate|up: 237 workgroups of 5 = one round on 256 compute
    units; O and QKV: 7 splits of exactly two ring revolutions; down: 9 splits; LM head: two rounds of 10 tiles)."""
    lib = binding.load()

    def plan(n_tiles, k_steps, batch, partial):
        wn, wk, sp = C.c_int32(), C.c_int32(), C.c_int32()
        assert lib.hx_plan_product(n_tiles, k_steps, batch, int(partial), C.byref(wn), C.byref(wk), C.byref(sp)) == binding.HX_OK
        return wn.value, wk.value, sp.value

    for s in (synth.TINY, synth.QWEN_1P5B, synth.QWEN_7B, synth.QWEN_14B):
        for K, N, partial in ((s.hidden, s.qkv_dim, True), (s.q_dim, s.hidden, True), (s.hidden, 2 * s.intermediate, False),
                              (s.intermediate, s.hidden, True), (s.hidden, s.vocab, False)):
            for batch in (1, 4, 64, 128, 256):
                wn, wk, sp = plan((N + 31) // 32, K // 16, batch, partial)
                assert (4 <= wn <= 6 or (wn == 10 and not partial and batch <= 128)) and wk == 1 and 1 <= sp <= 9
                assert sp == 1 or (K // 16) // sp >= 16
                assert partial or sp == 1
    s = synth.QWEN_7B
    assert plan(2 * s.intermediate // 32, s.hidden // 16, 128, False) == (5, 1, 1)
    assert plan(s.hidden // 32, s.q_dim // 16, 128, True) == (4, 1, 7)
    assert plan(s.qkv_dim // 32, s.hidden // 16, 128, True) == (4, 1, 7)
    assert plan(s.hidden // 32, s.intermediate // 16, 128, True) == (4, 1, 9)
    assert plan(s.vocab // 32, s.hidden // 16, 128, False) == (10, 1, 1)
    assert plan(s.vocab // 32, s.hidden // 16, 256, False) == (4, 1, 1)
    none = C.c_int32()
    assert lib.hx_plan_product(0, 10, 4, 1, C.byref(none), C.byref(none), C.byref(none)) == binding.HX_E_RANGE
    assert lib.hx_plan_product(10, 10, 300, 1, C.byref(none), C.byref(none), C.byref(none)) == binding.HX_E_RANGE
    assert lib.hx_plan_product(10, 10, 4, 1, None, C.byref(none), C.byref(none)) == binding.HX_E_NULL
