"""hero_int8_gemm_static (the entry point that allocates nothing: its split-K scratch is a fixed array inside the
library) against hero_int8_gemm_ws with a caller's workspace, through the C ABI, bit for bit: two calls in a row,
the second with a smaller input (the shared array still holds the first call's planes), then the first shape
again; a shape beyond the built-in scratch is refused."""
import numpy as np
import pytest
import torch

from paper_2310_17723_amd import binding as HB
from paper_2310_17723_amd import synth

pytestmark = pytest.mark.gpu

STATIC_BYTES = 16 << 20


def _case(seed, M, K, N):
    c = synth.gemm_case(seed, M, K, N)
    return {k: torch.from_numpy(v).cuda() for k, v in c.items()}


def _both(hero, c, epi, dt, residual=None):
    M, K = c["A"].shape
    N = c["Bt"].shape[0]
    need = hero.hero_int8_gemm_workspace_bytes(M, N, K)
    assert 0 < need <= STATIC_BYTES, need                     # the case does split, and fits the built-in scratch
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    kw = dict(a_row_scale=c["a_row_scale"], b_col_scale=c["b_col_scale"], bias=c["bias"], epi=epi, out_dtype=dt)
    ref = hero.hero_int8_gemm(c["A"], c["Bt"], residual=residual, workspace=ws, **kw)
    out = torch.full((M, N), 77, dtype=dt, device="cuda")
    free0 = torch.cuda.memory_allocated()
    hero.hero_int8_gemm(c["A"], c["Bt"], residual=residual, C_out=out, static_scratch=True, **kw)
    assert torch.cuda.memory_allocated() == free0
    torch.cuda.synchronize()
    return out, ref


def test_static_scratch_gemm_matches_workspace_gemm(hero):
    big = _case(901, 64, 16384, 4096)                          # the FC2 of a GPT decode step: 8 planes, 8 MiB
    small = _case(902, 48, 8192, 1024)                         # 16 planes of 48 x 1024
    o1, r1 = _both(hero, big, HB.EPI_REQUANT, torch.int8)
    assert torch.equal(o1, r1)
    o2, r2 = _both(hero, small, HB.EPI_REQUANT, torch.int8)
    assert torch.equal(o2, r2)
    res = (torch.randn((64, 4096), device="cuda") * 2).to(torch.bfloat16)
    o3, r3 = _both(hero, big, HB.EPI_DEQUANT, torch.bfloat16, residual=res)
    assert torch.equal(o3.view(torch.int16), r3.view(torch.int16))
    o4, r4 = _both(hero, small, HB.EPI_RAW_I32, torch.int32)
    assert torch.equal(o4, r4)
    # a shape that does not split runs without scratch
    c = _case(903, 256, 256, 512)
    assert hero.hero_int8_gemm_workspace_bytes(256, 512, 256) == 0
    a = hero.hero_int8_gemm(c["A"], c["Bt"], a_row_scale=c["a_row_scale"], b_col_scale=c["b_col_scale"], bias=c["bias"],
                            epi=HB.EPI_REQUANT, out_dtype=torch.int8, static_scratch=True)
    b = hero.hero_int8_gemm(c["A"], c["Bt"], a_row_scale=c["a_row_scale"], b_col_scale=c["b_col_scale"], bias=c["bias"],
                            epi=HB.EPI_REQUANT, out_dtype=torch.int8)
    assert torch.equal(a, b)


def test_static_scratch_gemm_refuses_what_does_not_fit(hero):
    M, K, N = 128, 16384, 4096
    assert hero.hero_int8_gemm_workspace_bytes(M, N, K) > STATIC_BYTES
    c = _case(904, M, K, N)
    with pytest.raises(HB.HeroError) as e:
        hero.hero_int8_gemm(c["A"], c["Bt"], a_row_scale=c["a_row_scale"], b_col_scale=c["b_col_scale"], bias=c["bias"],
                            epi=HB.EPI_REQUANT, out_dtype=torch.int8, static_scratch=True)
    assert e.value.status == 5
