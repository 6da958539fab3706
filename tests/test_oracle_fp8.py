"""Pins of the oracle's 8-bit cache variant: its E4M3 rounding against the format's code table and a library cast
(torch.float8_e4m3fn on the CPU), ties and saturation by closed form, and the model-level invariant that stepwise
decoding through the 8-bit paged cache equals the dense causal recomputation with the same rounding."""
import numpy as np
import torch

import oracle
from paper_2511_00796_amd import synth
from util import host_model


def code_table():
    """The 256 codes decoded by the library; NaN for S.1111.111."""
    return torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy()


def test_code_table_matches_the_published_format():
    """Value of code S.EEEE.MMM from the format's definition: (-1)^S 2^(E-7) (1 + M/8), E = 0: 2^-6 (M/8);
    S.1111.111 is NaN; the largest finite value is 448.  Checks the library table the other pins lean on."""
    t = code_table()
    for code in range(256):
        s, e, m = code >> 7, (code >> 3) & 15, code & 7
        if e == 15 and m == 7:
            assert np.isnan(t[code])
            continue
        v = (2.0 ** -6) * (m / 8.0) if e == 0 else (2.0 ** (e - 7)) * (1 + m / 8.0)
        assert t[code] == (-v if s else v), code
    assert np.nanmax(t) == 448.0


def test_every_format_value_is_a_fixed_point_and_a_bf16_value():
    t = code_table()
    finite = t[~np.isnan(t)]
    assert np.array_equal(oracle.e4m3_round(finite), finite)
    bits = oracle.bf16_round_bits(finite)
    assert np.array_equal((bits.astype(np.uint32) << 16).view(np.float32), finite)


def test_rounding_matches_the_library_cast_inside_the_finite_range():
    """200 000 values, dense near zero (subnormals), around 1 and up to +-448, against torch's cast."""
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(0, 1, 80000), rng.uniform(-448, 448, 40000), rng.normal(0, 0.01, 40000),
                        rng.uniform(-2 ** -5, 2 ** -5, 40000)]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).to(torch.float32).numpy()
    got = oracle.e4m3_round(x)
    assert np.array_equal(got, ref)
    assert np.array_equal(np.signbit(got), np.signbit(ref))


def test_ties_go_to_the_even_mantissa_and_large_values_saturate():
    t = np.sort(code_table()[:127])                       # the non-negative finite values, ascending (code order)
    for i in range(len(t) - 1):
        mid = np.float32((np.float64(t[i]) + np.float64(t[i + 1])) / 2)   # exact in fp32
        even = t[i] if i % 2 == 0 else t[i + 1]           # codes ascend with the values: even code = even mantissa
        assert oracle.e4m3_round([mid])[0] == even, (t[i], t[i + 1])
        assert oracle.e4m3_round([-mid])[0] == -even
        assert oracle.e4m3_round([np.nextafter(mid, np.float32(np.inf))])[0] == t[i + 1]
        assert oracle.e4m3_round([np.nextafter(mid, np.float32(-np.inf))])[0] == t[i]
    assert np.array_equal(oracle.e4m3_round([449.0, 464.0, 465.0, 1e6, 3e38, -1e6]), [448, 448, 448, 448, 448, -448])
    assert np.isnan(oracle.e4m3_round([np.nan])[0])


def test_stepwise_decode_through_the_8_bit_cache_equals_dense_causal_recomputation():
    """The brute-force invariant in the 8-bit variant (bit for bit inside the oracle), and the variant is not a
    no-op: its logits differ from the bf16 cache's, by a moderate amount."""
    s = synth.ModelShape("fp8-tiny", 2, 128, 4, 2, 32, 256, 512)
    ow, g, layers = host_model(s, 5)
    cfg8 = oracle.make_config(s, kv_fp8=True)
    cfg16 = oracle.make_config(s)
    n = 40
    toks = np.random.default_rng(2).integers(0, s.vocab, size=n).astype(np.int32)
    dense8 = oracle.full_causal(cfg8, ow, toks)[0]
    dense16 = oracle.full_causal(cfg16, ow, toks)[0]
    table, nb = synth.block_table(np.array([n]), s.block_size, 3)
    kv = oracle.PagedKV(cfg8, nb)
    for p in range(n):
        logits = oracle.decode_step(cfg8, ow, kv, toks[p:p + 1], np.array([p]), np.array([p + 1]), table)[0]
        assert np.array_equal(logits[0], dense8[p]), p
    # what the cache holds is 8-bit data: every stored value survives the rounding unchanged
    held = (kv.k[0].astype(np.uint32) << 16).view(np.float32)
    used = held[np.isfinite(held)]
    assert np.array_equal(oracle.e4m3_round(used), used)
    drift = np.abs(dense8 - dense16).max() / np.abs(dense16).max()
    assert 1e-4 < drift < 0.3, drift
