"""Pins of the oracle's elementary operations against things other than itself: closed forms,
invariants, numpy float64 / torch CPU library routines, integer arithmetic.  Each test is chosen
so that a plausible slip (dropped term, wrong sign or index, transposed operand) fails it.
CPU only."""
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import make_config
from paper_2511_00796_amd import synth
from util import bits_to_f32, f32_to_bf16_bits_ref

RNG = np.random.default_rng(7)


def bf16_bits(x):
    return synth.as_u16(torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.bfloat16))


# ---- bf16 rounding ------------------------------------------------------------------------------

def test_bf16_round_matches_integer_rne_on_all_upper_halves():
    # every 16-bit upper half (finite) x lower halves around the tie point
    lows = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF], dtype=np.uint32)
    ups = np.arange(0, 1 << 16, 37, dtype=np.uint32)  # stride keeps the python loop short
    ups = np.concatenate([ups, np.array([0x0000, 0x0001, 0x007F, 0x0080, 0x3F7F, 0x3F80, 0x7F7E, 0x7F7F,
                                         0x8000, 0xBF80, 0xFF7F], dtype=np.uint32)])
    u = ((ups[:, None] << 16) | lows[None, :]).reshape(-1).astype(np.uint32)
    x = u.view(np.float32)
    finite = np.isfinite(x)
    x = x[finite]
    got = oracle.bf16_round_bits(x)
    ref = f32_to_bf16_bits_ref(x)
    assert np.array_equal(got, ref)
    # and against the library cast
    lib_bits = bf16_bits(x)
    assert np.array_equal(got, lib_bits)


def test_bf16_ties_go_to_even():
    one_plus_half_ulp = np.array([0x3F808000], dtype=np.uint32).view(np.float32)   # 1 + 2^-8: tie, even below
    three_halves_ulp = np.array([0x3F818000], dtype=np.uint32).view(np.float32)    # tie, even above
    assert oracle.bf16_round_bits(one_plus_half_ulp)[0] == 0x3F80
    assert oracle.bf16_round_bits(three_halves_ulp)[0] == 0x3F82


# ---- softmax --------------------------------------------------------------------------------------

def test_softmax_rows_sum_to_one_and_shift_invariant():
    for n in (1, 2, 17, 300, 5000):
        s = RNG.normal(0, 3, size=n).astype(np.float32)
        p = oracle.softmax(s)
        assert abs(p.astype(np.float64).sum() - 1.0) <= 1e-6
        assert np.all(p >= 0)
        p2 = oracle.softmax(s + np.float32(11.5))
        assert np.allclose(p, p2, rtol=2e-6, atol=1e-9)


def test_softmax_two_keys_is_logistic():
    for a, b in ((0.3, -1.2), (5.0, 5.0), (-40.0, 2.0)):
        p = oracle.softmax(np.array([a, b], dtype=np.float32))
        assert p[0] == pytest.approx(1.0 / (1.0 + math.exp(b - a)), rel=1e-6, abs=1e-12)


def test_softmax_vs_float64():
    s = RNG.normal(0, 2, size=777).astype(np.float32)
    e = np.exp(s.astype(np.float64) - s.max())
    assert np.allclose(oracle.softmax(s), e / e.sum(), rtol=1e-5, atol=1e-10)


def test_softmax_large_scores_do_not_overflow():
    p = oracle.softmax(np.array([1000.0, 999.0, -1000.0], dtype=np.float32))
    assert np.all(np.isfinite(p)) and p[0] == pytest.approx(1 / (1 + math.exp(-1)), rel=1e-6)


# ---- RMSNorm --------------------------------------------------------------------------------------

def test_rmsnorm_constant_vector_closed_form():
    n, c, eps = 256, 0.75, 1e-6
    g = RNG.normal(1, 0.1, size=n).astype(np.float32)
    gb = bf16_bits(g)
    y = oracle.rmsnorm(np.full(n, c, dtype=np.float32), gb, eps)
    assert np.allclose(y, bits_to_f32(gb) * c / math.sqrt(c * c + eps), rtol=1e-6)


def test_rmsnorm_vs_float64_and_eps_matters():
    n = 1536
    x = RNG.normal(0, 2.0, size=n).astype(np.float32)
    gb = bf16_bits(RNG.normal(1, 0.02, size=n))
    ref = x.astype(np.float64) / np.sqrt((x.astype(np.float64) ** 2).mean() + 1e-6) * bits_to_f32(gb)
    assert np.allclose(oracle.rmsnorm(x, gb, 1e-6), ref, rtol=1e-5, atol=1e-7)
    # eps is inside the square root, added to the MEAN (not the sum): tiny inputs expose it
    xt = np.full(n, 1e-4, dtype=np.float32)
    y = oracle.rmsnorm(xt, bf16_bits(np.ones(n)), 1e-6)
    assert np.allclose(y, 1e-4 / math.sqrt(1e-8 + 1e-6), rtol=1e-5)


def test_rmsnorm_unit_gain_has_unit_rms():
    x = RNG.normal(0, 5, size=512).astype(np.float32)
    y = oracle.rmsnorm(x, bf16_bits(np.ones(512)), 1e-6)
    assert math.sqrt(float((y.astype(np.float64) ** 2).mean())) == pytest.approx(1.0, rel=1e-5)


# ---- linear ---------------------------------------------------------------------------------------

def test_linear_vs_numpy_float64_nonsquare():
    K, N = 96, 40   # non-square: a transposed operand cannot pass
    x = bits_to_f32(bf16_bits(RNG.normal(0, 1, size=K)))
    wb = bf16_bits(RNG.normal(0, 0.05, size=(K, N)))
    bb = bf16_bits(RNG.normal(0, 0.05, size=N))
    ref = x.astype(np.float64) @ bits_to_f32(wb).astype(np.float64)
    assert np.allclose(oracle.linear(x, wb), ref, rtol=1e-5, atol=1e-6)
    assert np.allclose(oracle.linear(x, wb, bb), ref + bits_to_f32(bb), rtol=1e-5, atol=1e-6)


def test_linear_one_hot_reads_back_exact_row_and_ones_sum():
    K, N = 33, 21
    wb = bf16_bits(RNG.normal(0, 1, size=(K, N)))
    for k in (0, 7, K - 1):
        x = np.zeros(K, dtype=np.float32)
        x[k] = 1.0
        assert np.array_equal(oracle.linear(x, wb), bits_to_f32(wb)[k])
    ones = bf16_bits(np.ones((K, N)))
    assert np.array_equal(oracle.linear(np.full(K, 0.5, dtype=np.float32), ones), np.full(N, K * 0.5, np.float32))


# ---- RoPE -----------------------------------------------------------------------------------------

def test_rope_position_zero_is_identity_and_norm_is_kept():
    v = RNG.normal(0, 1, size=128).astype(np.float32)
    assert np.array_equal(oracle.rope(v, 0, 1e6), v)
    for pos in (1, 77, 16384):
        r = oracle.rope(v, pos, 1e6)
        assert np.linalg.norm(r.astype(np.float64)) == pytest.approx(np.linalg.norm(v.astype(np.float64)), rel=1e-6)
        # pairwise norms too: the pair is (i, i + d/2), not (2i, 2i+1)
        assert np.allclose(r[:64] ** 2 + r[64:] ** 2, v[:64] ** 2 + v[64:] ** 2, rtol=1e-5, atol=1e-7)


def test_rope_is_complex_rotation_of_half_pairs_in_float64():
    d, theta = 64, 1e6
    v = RNG.normal(0, 1, size=d).astype(np.float32)
    for pos in (3, 1000, 16384):
        z = v[: d // 2].astype(np.float64) + 1j * v[d // 2:].astype(np.float64)
        ang = pos * theta ** (-2.0 * np.arange(d // 2) / d)
        zr = z * np.exp(1j * ang)
        r = oracle.rope(v, pos, theta)
        assert np.allclose(r[: d // 2], zr.real, atol=2e-6) and np.allclose(r[d // 2:], zr.imag, atol=2e-6)


def test_rope_dot_depends_only_on_position_difference():
    d = 128
    q = RNG.normal(0, 1, size=d).astype(np.float32)
    k = RNG.normal(0, 1, size=d).astype(np.float32)
    base = float(oracle.rope(q, 500, 1e6).astype(np.float64) @ oracle.rope(k, 100, 1e6).astype(np.float64))
    for shift in (1, 4000, 15884):
        moved = float(oracle.rope(q, 500 + shift, 1e6).astype(np.float64)
                      @ oracle.rope(k, 100 + shift, 1e6).astype(np.float64))
        assert moved == pytest.approx(base, abs=2e-4)


# ---- SiLU, argmax -----------------------------------------------------------------------------------

def test_silu_special_values_and_library():
    assert oracle.silu(0.0) == 0.0
    assert oracle.silu(30.0) == pytest.approx(30.0, rel=1e-6)
    assert oracle.silu(-30.0) == pytest.approx(0.0, abs=1e-10)
    for x in (-3.0, -0.5, 0.25, 2.0):
        assert oracle.silu(x) == pytest.approx(float(torch.nn.functional.silu(torch.tensor(x, dtype=torch.float64))), rel=1e-6)


def test_argmax_planted_maximum_and_lowest_index_on_ties():
    x = RNG.normal(0, 1, size=1000).astype(np.float32)
    x[613] = 50.0
    assert oracle.argmax(x) == 613
    x[100] = 50.0
    assert oracle.argmax(x) == 100      # exact tie: the smaller index
    x[999] = 51.0
    assert oracle.argmax(x) == 999


# ---- attention over the paged cache -------------------------------------------------------------------

class Shape:
    n_layers, hidden, n_q_heads, n_kv_heads, head_dim, intermediate, vocab = 1, 64, 6, 2, 32, 64, 64
    block_size, qkv_bias, rms_eps, rope_theta = 16, True, 1e-6, 1e6


def make_cache(T, block_size=16, shape=Shape, perm_seed=None, k=None, v=None):
    cfg = make_config(shape, block_size=block_size)
    nblk = (T + block_size - 1) // block_size
    ids = np.arange(nblk + 3, dtype=np.int32)
    if perm_seed is not None:
        ids = np.random.default_rng(perm_seed).permutation(nblk + 3).astype(np.int32)
    table = ids[:nblk][None, :].copy()
    kv = oracle.PagedKV(cfg, nblk + 3, n_layers=1)
    if k is None:
        k = bf16_bits(RNG.normal(0, 1, size=(T, shape.n_kv_heads, shape.head_dim)))
        v = bf16_bits(RNG.normal(0, 1, size=(T, shape.n_kv_heads, shape.head_dim)))
    kv.fill(0, k, v, np.array([0, T], dtype=np.int32), table)
    return cfg, kv, table, k, v


def test_attention_single_key_returns_its_value_exactly():
    cfg, kv, table, k, v = make_cache(1)
    q = RNG.normal(0, 1, size=Shape.n_q_heads * Shape.head_dim).astype(np.float32)
    o = oracle.attention(cfg, q, kv.k[0], kv.v[0], table[0], 1).reshape(Shape.n_q_heads, -1)
    G = Shape.n_q_heads // Shape.n_kv_heads
    for h in range(Shape.n_q_heads):
        assert np.array_equal(o[h], bits_to_f32(v[0, h // G]))   # also pins head h -> KV head h // G


def test_attention_equal_scores_give_mean_of_values():
    T = 37
    cfg, kv, table, k, v = make_cache(T)
    o = oracle.attention(cfg, np.zeros(Shape.n_q_heads * Shape.head_dim, np.float32), kv.k[0], kv.v[0], table[0], T)
    o = o.reshape(Shape.n_q_heads, -1)
    G = Shape.n_q_heads // Shape.n_kv_heads
    for h in range(Shape.n_q_heads):
        assert np.allclose(o[h], bits_to_f32(v[:, h // G]).astype(np.float64).mean(0), atol=2e-6)


def test_attention_dominant_key_selects_its_value():
    T, d = 50, Shape.head_dim
    k = np.zeros((T, Shape.n_kv_heads, d), dtype=np.float32)
    k[23, :, 0] = 64.0
    v = RNG.normal(0, 1, size=(T, Shape.n_kv_heads, d))
    cfg, kv, table, kb, vb = make_cache(T, k=bf16_bits(k), v=bf16_bits(v))
    q = np.zeros((Shape.n_q_heads, d), dtype=np.float32)
    q[:, 0] = 8.0                                  # score 8*64/sqrt(32) = 90.5 at key 23, 0 elsewhere
    o = oracle.attention(cfg, q, kv.k[0], kv.v[0], table[0], T).reshape(Shape.n_q_heads, -1)
    G = Shape.n_q_heads // Shape.n_kv_heads
    for h in range(Shape.n_q_heads):
        assert np.allclose(o[h], bits_to_f32(vb[23, h // G]), atol=1e-6)


def test_attention_vs_torch_sdpa_and_float64():
    T, d, nq, nkv = 83, Shape.head_dim, Shape.n_q_heads, Shape.n_kv_heads
    cfg, kv, table, kb, vb = make_cache(T, perm_seed=5)
    q = bits_to_f32(bf16_bits(RNG.normal(0, 1, size=(nq, d))))
    o = oracle.attention(cfg, q, kv.k[0], kv.v[0], table[0], T).reshape(nq, d)
    K = torch.from_numpy(bits_to_f32(kb)).permute(1, 0, 2).repeat_interleave(nq // nkv, dim=0)   # [nq, T, d]
    V = torch.from_numpy(bits_to_f32(vb)).permute(1, 0, 2).repeat_interleave(nq // nkv, dim=0)
    ref = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q)[:, None, :], K, V)[:, 0, :]
    assert np.allclose(o, ref.numpy(), atol=2e-6)
    ref64 = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q).double()[:, None, :], K.double(), V.double())
    assert np.allclose(o, ref64[:, 0, :].numpy(), atol=2e-6)


def test_attention_attends_exactly_T_keys():
    # keys beyond T must not contribute, key T-1 must
    T = 40
    cfg, kv, table, kb, vb = make_cache(T)
    q = RNG.normal(0, 1, size=Shape.n_q_heads * Shape.head_dim).astype(np.float32)
    full = oracle.attention(cfg, q, kv.k[0], kv.v[0], table[0], T)
    short = oracle.attention(cfg, q, kv.k[0], kv.v[0], table[0], T - 1)
    assert not np.array_equal(full, short)
    K = torch.from_numpy(bits_to_f32(kb[:T - 1])).permute(1, 0, 2).repeat_interleave(3, dim=0)
    V = torch.from_numpy(bits_to_f32(vb[:T - 1])).permute(1, 0, 2).repeat_interleave(3, dim=0)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).view(Shape.n_q_heads, 1, -1), K, V)[:, 0, :]
    assert np.allclose(short.reshape(Shape.n_q_heads, -1), ref.numpy(), atol=2e-6)


def test_attention_gqa_equals_mha_with_duplicated_kv_heads():
    T, d, nq, nkv = 45, Shape.head_dim, Shape.n_q_heads, Shape.n_kv_heads
    cfg, kv, table, kb, vb = make_cache(T)
    q = RNG.normal(0, 1, size=nq * d).astype(np.float32)
    grouped = oracle.attention(cfg, q, kv.k[0], kv.v[0], table[0], T)

    class Mha(Shape):
        n_kv_heads = Shape.n_q_heads
    kd = np.repeat(kb, nq // nkv, axis=1)
    vd = np.repeat(vb, nq // nkv, axis=1)
    cfg2, kv2, table2, _, _ = make_cache(T, shape=Mha, k=kd, v=vd)
    assert np.array_equal(grouped, oracle.attention(cfg2, q, kv2.k[0], kv2.v[0], table2[0], T))


def test_attention_invariant_to_block_permutation_and_block_size():
    T = 100
    k = bf16_bits(RNG.normal(0, 1, size=(T, Shape.n_kv_heads, Shape.head_dim)))
    v = bf16_bits(RNG.normal(0, 1, size=(T, Shape.n_kv_heads, Shape.head_dim)))
    q = RNG.normal(0, 1, size=Shape.n_q_heads * Shape.head_dim).astype(np.float32)
    outs = []
    for bs, perm in ((16, None), (16, 1), (16, 2), (1, 3), (7, 4), (128, None)):
        cfg, kv, table, _, _ = make_cache(T, block_size=bs, perm_seed=perm, k=k, v=v)
        outs.append(oracle.attention(cfg, q, kv.k[0], kv.v[0], table[0], T))
    for o in outs[1:]:
        assert np.array_equal(outs[0], o)          # bit-identical
