"""dsk_linear_static, the entry point that allocates nothing (its split-K partial sums live in a fixed array inside
the library), against dsk_linear: same bits, on two calls in a row, the second with a smaller input, and against
the fp64 definition; sizes beyond its limits are refused."""
import numpy as np
import pytest
import torch

from oracle import dsk_oracle as O
from paper_2411_02820_amd import synth

pytestmark = pytest.mark.gpu


def _bf16(a):
    return synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(a))


def test_static_scratch_linear_equals_dsk_linear_on_two_calls_in_a_row():
    from paper_2411_02820_amd import binding as B
    dev = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    # the 8B gate/up projection over 64 suffix rows (64x128 tiles, 3 splits: 22 MB of partial sums), then the
    # smaller 8B QKV projection over 17 rows with a residual (64x64 tiles, 8 splits), which reuses the same array
    for M, N, K, residual in ((64, 28672, 4096, False), (17, 6144, 4096, True)):
        x = _bf16(synth.normal(M * K, 31, 0, 1.0).reshape(M, K))
        w = _bf16(synth.normal(N * K, 31, 1, 0.02).reshape(N, K))
        r = _bf16(synth.normal(M * N, 31, 2, 1.0).reshape(M, N)) if residual else None
        xd, wd, rd = dev(x), dev(w), None if r is None else dev(r)
        y_ref = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.dsk_linear(B.DSK_BF16, xd, wd, y_ref, rd, M, N, K)
        B.dsk_set_option("reset_stats", 0)
        B.dsk_linear_static(B.DSK_BF16, xd, wd, y, rd, M, N, K)
        torch.cuda.synchronize()
        assert B.dsk_get_stat("gemm_mfma_launches") == 1 and B.dsk_get_stat("gemm_generic_launches") == 0
        assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16)), (M, N, K)
        ref = x.astype(np.float64) @ w.astype(np.float64).T + (0 if r is None else r.astype(np.float64))
        assert O.max_rel_err(y.float().cpu().numpy(), ref) <= 2 ** -8


def test_static_scratch_linear_refuses_sizes_beyond_its_limits():
    from paper_2411_02820_amd import binding as B
    t = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    for M, N in ((B.DSK_STATIC_MAX_M + 1, 256), (8, B.DSK_STATIC_MAX_N + 4)):
        with pytest.raises(B.DskError) as e:
            B.dsk_linear_static(B.DSK_BF16, t, t, t, None, M, N, 64)
        assert e.value.status == B.DSK_ELIMIT
    torch.cuda.synchronize()
