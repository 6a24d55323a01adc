"""The entry point that allocates nothing (rlhf_decode_attention_static): its
output against rlhf_decode_attention's on two calls in a row, the second with a
smaller input, so that what the first call left in the library's scratch array
and arrival counters cannot go unnoticed."""
import numpy as np
import pytest
import torch

from paper_2410_15651_amd import binding as rb
from paper_2410_15651_amd import workloads as wl

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3


@pytest.fixture(scope="module")
def gu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    return gpu_util


def _both(gu, cfg, lens, out_dtype):
    q, ks, vs = wl.qkv(cfg, lens, device=gu.DEV)
    A = gu.FilledArena(cfg, lens, ks, vs)
    try:
        k, v, table, dl = A.views()
        params = rb.attn_params(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, A.mpps,
                                wl.DTYPE_CODE[cfg.kv_dtype], out_dtype=out_dtype)
        odt = torch.float32 if out_dtype == rb.RLHF_F32 else q.dtype
        ws = torch.full((rb.rlhf_decode_attention_workspace_bytes(params),), 0xFF, dtype=torch.uint8,
                        device=gu.DEV)
        ref = torch.full((cfg.batch, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=odt, device=gu.DEV)
        got = torch.full_like(ref, float("nan"))
        rb.rlhf_decode_attention(params, q, k, v, table, dl, ref, ws)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        rb.rlhf_decode_attention_static(params, q, k, v, table, dl, got)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        return ref, got
    finally:
        A.close()


@pytest.mark.parametrize("heads", [(64, 8), (32, 32)])
def test_static_scratch_entry_point_matches_the_workspace_one_twice_in_a_row(gu, heads):
    hq, hkv = heads
    big = wl.small_variant(wl.config(5), batch=48, n_q_heads=hq, n_kv_heads=hkv, len_lo=0, len_hi=1500)
    small = wl.small_variant(wl.config(5), batch=5, n_q_heads=hq, n_kv_heads=hkv, len_lo=1, len_hi=90)
    for cfg in (big, small):                      # the second call is the smaller one
        lens = wl.seq_lengths(cfg)
        if cfg.len_lo == 0:
            lens[3] = 0
        print(f"static scratch: heads {heads} batch {cfg.batch} lens {lens.tolist()[:8]}...", flush=True)
        for out_dtype in (rb.RLHF_F32, None):
            ref, got = _both(gu, cfg, lens, out_dtype)
            assert torch.isfinite(got).all()
            err = (got.double() - ref.double()).abs().max().item()
            assert err <= ATTN_TOL
            assert int((got.view(torch.uint8) != ref.view(torch.uint8)).sum()) == 0   # same kernels, same arithmetic


def test_static_scratch_entry_point_refuses_what_its_array_cannot_hold(gu):
    params = rb.attn_params(8192, 64, 64, 128, 4, rb.RLHF_BF16)
    assert rb.rlhf_decode_attention_workspace_bytes(params) > (16 << 20)
    dummy = torch.zeros(16, dtype=torch.uint8, device=gu.DEV)
    with pytest.raises(rb.RlhfError) as e:
        rb.rlhf_decode_attention_static(params, dummy, dummy, dummy, dummy, dummy, dummy)
    assert e.value.status == rb.RLHF_ERR_UNSUPPORTED
    assert "16777216" in str(e.value)
