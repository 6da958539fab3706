"""hx_stage_attention_static -- the attention stage with its scratch in the library's static device array, for callers
that cannot allocate -- against hx_stage_attention (scratch in the engine's workspace): the same kernels on the same
schedule, so the outputs must be equal bit for bit; and both against the oracle's attention.  Two calls in a row, the
second with a smaller input (fewer and shorter sequences), which finds the first call's contents in the array."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_00796_amd import synth
from util import bits_to_f32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hx():
    from paper_2511_00796_amd import binding
    binding.load()
    assert torch.cuda.is_available()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("cache", ["bf16", "fp8"])
def test_static_scratch_attention_equals_the_workspace_one_on_two_calls_in_a_row(hx, cache):
    shape = synth.ModelShape("no-alloc", 1, 512, 14, 2, 128, 1376, 2048)
    kvd = hx.HX_KV_FP8_E4M3 if cache == "fp8" else hx.HX_KV_BF16
    eng = hx.Engine(shape, 24, 4100, kv_dtype=kvd)
    cfg = oracle.make_config(shape, kv_fp8=cache == "fp8")
    rng = np.random.default_rng(3)
    calls = [np.array([4096, 1, 17, 700, 2500, 16, 333, 1029, 48, 3000, 512, 95, 2048, 15, 640, 1200, 31, 257, 4000, 64],
                      dtype=np.int32),
             np.array([300, 1, 1500, 33, 16], dtype=np.int32)]         # second call: smaller batch, shorter sequences
    for n, lens in enumerate(calls):
        table, nb = synth.block_table(lens, 16, 50 + n)
        k, v = synth.kv_fill(shape, 0, int(lens.sum()), 60 + n)
        start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        kv = hx.KVCache(eng, nb)
        kv.pool.fill_(0xFF)
        kv.prefill_fill(0, k.cuda(), v.cuda(), dev(start), dev(table))
        q = dev(rng.normal(0, 1.2, size=(len(lens), shape.q_dim)).astype(np.float32))
        lens_d, table_d = dev(lens), dev(table)
        want = eng.stage_attention(kv, 0, q, lens_d, table_d)
        out = torch.full_like(want, float("nan"))                     # provided by the caller, as the entry point requires
        torch.cuda.synchronize()
        eng.stage_attention_static(kv, 0, q, lens_d, table_d, out)
        torch.cuda.synchronize()
        assert torch.isfinite(out).all()
        assert torch.equal(out, want), (n, float((out - want).abs().max()))
        # and both are the oracle's attention to the stage bar
        okv = oracle.PagedKV(cfg, nb)
        okv.fill(0, synth.as_u16(k), synth.as_u16(v), start, table)
        qr = bits_to_f32(synth.as_u16(q.cpu().to(torch.bfloat16)))
        got = out.cpu().numpy()
        for b, T in enumerate(lens):
            ref = oracle.attention(cfg, qr[b], okv.k[0], okv.v[0], table[b], int(T))
            assert float(np.abs(got[b] - ref).max()) <= 1e-3, (n, b)


def test_a_call_beyond_the_static_array_is_refused(hx, monkeypatch):
    """16 384 wavefronts x 7 heads x 128 x 4 bytes of partial results do not fit 16 MiB: HX_E_RANGE, nothing launched."""
    monkeypatch.setenv("HX_ATTN_WAVES", "16384")
    shape = synth.ModelShape("no-alloc-big", 1, 512, 14, 2, 128, 1376, 2048)
    eng = hx.Engine(shape, 8, 256)
    lens = np.array([40, 100], dtype=np.int32)
    table, nb = synth.block_table(lens, 16, 1)
    kv = hx.KVCache(eng, nb)
    q = torch.zeros(2, shape.q_dim, device="cuda")
    out = torch.zeros_like(q)
    with pytest.raises(hx.HexError, match="static array holds") as err:
        eng.stage_attention_static(kv, 0, q, dev(lens), dev(table), out)
    assert err.value.code == hx.HX_E_RANGE
    eng.stage_attention(kv, 0, q, dev(lens), dev(table))              # the workspace variant takes the same call
    torch.cuda.synchronize()
