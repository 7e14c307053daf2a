"""Parity of single steps (projection GEMM, attention) with the oracle, through the C-ABI component calls."""
import numpy as np
import pytest
import torch

from oracle import dsk_oracle as O
from paper_2411_02820_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2411_02820_amd import binding
    return binding


def _bf16(a):
    return synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(a))


# shapes span: several tiles + ragged M tail, small-M weight-streaming path, N not a multiple of the tile, K tail
@pytest.mark.parametrize("M,N,K,residual", [
    (300, 512, 256, False), (1000, 768, 512, True), (64, 1024, 2048, True), (17, 4096, 1024, False),
    (1, 256, 64, True), (513, 320, 192, False), (130, 6144, 4096, True),
])
def test_linear_bf16(B, M, N, K, residual):
    x = _bf16(synth.normal(M * K, 11, 0, 1.0).reshape(M, K))
    w = _bf16(synth.normal(N * K, 11, 1, 0.05).reshape(N, K))
    r = _bf16(synth.normal(M * N, 11, 2, 1.0).reshape(M, N)) if residual else None
    ref = x.astype(np.float64) @ w.astype(np.float64).T + (0 if r is None else r.astype(np.float64))
    dev = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    B.dsk_linear(B.DSK_BF16, dev(x), dev(w), y, None if r is None else dev(r), M, N, K)
    torch.cuda.synchronize()
    # one bf16 rounding of the result: 2^-9 relative to the element, bounded here by max|ref|
    assert O.max_rel_err(y.float().cpu().numpy(), ref) <= 2 ** -8


# The few-row weight-streaming path at the widths the 8B and 70B suffix passes run it at: the 64x128 tiling it takes
# for a very wide N (gate/up: 2F = 28672 and 57344 columns), the 64x64 tiling for the others, full (64) and ragged
# (17) row counts, the long contraction of the down projection.
@pytest.mark.parametrize("M,N,K,residual", [
    (64, 28672, 4096, False), (17, 57344, 8192, False), (64, 57344, 8192, False), (64, 6144, 4096, False),
    (64, 4096, 14336, True), (33, 8192, 28672, True), (64, 10240, 8192, False),
])
def test_linear_bf16_few_rows_at_model_widths(B, M, N, K, residual):
    x = _bf16(synth.normal(M * K, 16, 0, 1.0).reshape(M, K))
    w = _bf16(synth.normal(N * K, 16, 1, 0.02).reshape(N, K))
    r = _bf16(synth.normal(M * N, 16, 2, 1.0).reshape(M, N)) if residual else None
    ref = x.astype(np.float64) @ w.astype(np.float64).T + (0 if r is None else r.astype(np.float64))
    dev = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    B.dsk_set_option("reset_stats", 0)
    B.dsk_linear(B.DSK_BF16, dev(x), dev(w), y, None if r is None else dev(r), M, N, K)
    torch.cuda.synchronize()
    assert B.dsk_get_stat("gemm_mfma_launches") == 1 and B.dsk_get_stat("gemm_generic_launches") == 0
    assert O.max_rel_err(y.float().cpu().numpy(), ref) <= 2 ** -8


def test_linear_bf16_unsupported_shape_is_an_error_not_a_slower_kernel(B):
    # K = 100 is no whole number of 64-element k-tiles: the tensor-core kernel refuses it, and the call says so;
    # the plain-ALU kernel runs only when the test hook asks for it
    M, N, K = 100, 96, 100
    x = _bf16(synth.normal(M * K, 11, 0, 1.0).reshape(M, K))
    w = _bf16(synth.normal(N * K, 11, 1, 0.05).reshape(N, K))
    dev = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.DskError) as e:
        B.dsk_linear(B.DSK_BF16, dev(x), dev(w), y, None, M, N, K)
    assert e.value.status == B.DSK_ESHAPE
    torch.cuda.synchronize()
    assert torch.isnan(y.float()).all(), "a refused call writes nothing"
    B.dsk_set_option("force_generic", 1)
    try:
        B.dsk_linear(B.DSK_BF16, dev(x), dev(w), y, None, M, N, K)
        torch.cuda.synchronize()
    finally:
        B.dsk_set_option("force_generic", 0)
    assert O.max_rel_err(y.float().cpu().numpy(), x.astype(np.float64) @ w.astype(np.float64).T) <= 2 ** -8


# the two prefill tilings (1: 256x256 on the 16x16x32 MFMA, 2: 128x128 on the 32x32x16 MFMA) forced on shapes with
# 1, 2, 3 and 7 k-tiles (the peeled head and tail of the software pipeline), ragged M and N, with and without residual
@pytest.mark.parametrize("variant", [1, 2])
@pytest.mark.parametrize("M,N,K,residual", [(300, 516, 64, False), (257, 512, 128, True), (513, 260, 192, False),
                                            (700, 1028, 448, True)])
def test_linear_bf16_forced_tiling(B, variant, M, N, K, residual):
    x = _bf16(synth.normal(M * K, 14, 0, 1.0).reshape(M, K))
    w = _bf16(synth.normal(N * K, 14, 1, 0.05).reshape(N, K))
    r = _bf16(synth.normal(M * N, 14, 2, 1.0).reshape(M, N)) if residual else None
    ref = x.astype(np.float64) @ w.astype(np.float64).T + (0 if r is None else r.astype(np.float64))
    dev = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    B.dsk_set_option("gemm_tiling", variant)
    try:
        B.dsk_linear(B.DSK_BF16, dev(x), dev(w), y, None if r is None else dev(r), M, N, K)
        torch.cuda.synchronize()
    finally:
        B.dsk_set_option("gemm_tiling", 0)
    assert O.max_rel_err(y.float().cpu().numpy(), ref) <= 2 ** -8


# the tiling the library picks by itself for a prefill-sized problem (>= 192 tiles of 256x256), short K
@pytest.mark.parametrize("K", [64, 320])
def test_linear_bf16_large_grid_short_k(B, K):
    M, N = 3585, 3332
    x = _bf16(synth.normal(M * K, 15, 0, 1.0).reshape(M, K))
    w = _bf16(synth.normal(N * K, 15, 1, 0.05).reshape(N, K))
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    dev = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    B.dsk_linear(B.DSK_BF16, dev(x), dev(w), y, None, M, N, K)
    torch.cuda.synchronize()
    assert O.max_rel_err(y.float().cpu().numpy(), ref) <= 2 ** -8


@pytest.mark.parametrize("M,N,K", [(70, 96, 40), (128, 64, 256)])
def test_linear_fp32(B, M, N, K):
    x = synth.normal(M * K, 12, 0, 1.0).reshape(M, K)
    w = synth.normal(N * K, 12, 1, 0.05).reshape(N, K)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    y = torch.empty((M, N), dtype=torch.float32, device="cuda")
    B.dsk_linear(B.DSK_F32, torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), y, None, M, N, K)
    torch.cuda.synchronize()
    assert O.max_rel_err(y.cpu().numpy(), ref) <= 1e-5


def test_linear_in_place_residual(B):
    M, N, K = 64, 512, 512
    x = _bf16(synth.normal(M * K, 13, 0, 1.0).reshape(M, K))
    w = _bf16(synth.normal(N * K, 13, 1, 0.05).reshape(N, K))
    r = _bf16(synth.normal(M * N, 13, 2, 1.0).reshape(M, N))
    ref = x.astype(np.float64) @ w.astype(np.float64).T + r
    dev = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    y = dev(r)
    B.dsk_linear(B.DSK_BF16, dev(x), dev(w), y, y, M, N, K)
    torch.cuda.synchronize()
    assert O.max_rel_err(y.float().cpu().numpy(), ref) <= 2 ** -8


def _attention_case(B, lens, plens, Hq, Hkv, dh, dtype, use_scratch, key_gain=None, q_gain=1.0):
    from paper_2411_02820_amd import binding
    cu = synth.cu_seqlens(lens)
    n_q = int(cu[-1])
    pcu = synth.cu_seqlens(plens) if plens else None
    n_pre = int(pcu[-1]) if plens else 0
    own_row0 = n_pre + 3 if plens else 0          # a gap between the two ranges
    rows = own_row0 + n_q
    rnd = (lambda a: _bf16(a)) if dtype == "bf16" else (lambda a: a)
    q = rnd(synth.normal(n_q * Hq * dh, 21, 0, 1.0).reshape(n_q, Hq, dh) * np.float32(q_gain))
    k = synth.normal(rows * Hkv * dh, 21, 1, 1.0).reshape(rows, Hkv, dh)
    if key_gain is not None:   # per-row gain on the keys: shapes how the running maximum moves along the keys
        k = k * key_gain(np.arange(rows)).astype(np.float32)[:, None, None]
    k = rnd(k)
    v = rnd(synth.normal(rows * Hkv * dh, 21, 2, 1.0).reshape(rows, Hkv, dh))
    seq = np.repeat(np.arange(len(lens)), lens)
    ref = np.empty((n_q, Hq, dh))
    for i in range(n_q):
        b = seq[i]
        vis = list(range(pcu[b], pcu[b + 1])) if plens else []
        vis += list(range(own_row0 + cu[b], own_row0 + i + 1))
        ref[i] = O.attend_row(q[i].astype(np.float64), k[vis].astype(np.float64), v[vis].astype(np.float64))
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(tdt).cuda()
    out = torch.empty((n_q, Hq * dh), dtype=tdt, device="cuda")
    qb = binding.Batch(cu)
    pb = binding.Batch(pcu) if plens else None
    scratch = torch.empty(Hkv * dh * ((rows + 63) // 64 * 64), dtype=tdt, device="cuda") if use_scratch else None
    B.dsk_set_option("reset_stats", 0)
    B.dsk_attention(B.DSK_BF16 if dtype == "bf16" else B.DSK_F32, dev(q), dev(k), dev(v), out, qb.desc,
                    None if pb is None else pb.desc, own_row0, Hq, Hkv, dh, scratch)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().reshape(n_q, Hq, dh)
    return O.max_rel_err(got, ref)


@pytest.mark.parametrize("lens,plens", [([300], None), ([129, 1, 64, 200], None), ([40, 7], [200, 130]), ([1], [65])])
def test_attention_bf16_tensor_core_kernel(B, lens, plens):
    err = _attention_case(B, lens, plens, 8, 2, 128, "bf16", True)
    assert B.dsk_get_stat("attn_mfma_launches") == 1, "the MFMA kernel must be the one that ran"
    assert err <= 1e-2


@pytest.mark.parametrize("ramp", ["up", "down", "spikes"])
def test_attention_bf16_peaked_scores(B, ramp):
    # Scores with a standard deviation of tens instead of one, so the softmax is sharply peaked and the running
    # maximum matters: growing along the keys (the maximum keeps jumping by far more than the kernel's lazy
    # threshold, every jump rescales the accumulated output), shrinking (the first tile holds the maximum, later
    # probabilities underflow), and isolated large keys (long stretches where the reference maximum stays put).
    gain = {"up": lambda r: 1.0 + r / 24.0, "down": lambda r: 1.0 + (r.max() - r) / 24.0,
            "spikes": lambda r: np.where(r % 97 == 5, 12.0, 1.0)}[ramp]
    err = _attention_case(B, [333, 90], [70, 150], 8, 2, 128, "bf16", True, key_gain=gain, q_gain=3.0)
    assert B.dsk_get_stat("attn_mfma_launches") == 1
    assert err <= 1e-2


def test_attention_bf16_dh64_and_mha(B):
    assert _attention_case(B, [150, 70], None, 4, 4, 64, "bf16", True) <= 1e-2
    assert B.dsk_get_stat("attn_mfma_launches") == 1


def test_attention_plain_kernel_both_dtypes(B):
    assert _attention_case(B, [90, 33], [50, 20], 4, 2, 64, "f32", False) <= 1e-5
    assert _attention_case(B, [90, 33], [50, 20], 4, 2, 64, "bf16", False) <= 1e-2
    assert B.dsk_get_stat("attn_generic_launches") == 1


def test_attention_bf16_unsupported_shape_is_an_error(B):
    from paper_2411_02820_amd import binding
    n_q, Hq, Hkv, dh = 16, 4, 2, 32     # head_dim 32: not a shape of the tensor-core kernel
    t = lambda *s: torch.zeros(s, dtype=torch.bfloat16, device="cuda")
    qb = binding.Batch(synth.cu_seqlens([n_q]))
    scratch = t(Hkv * dh * 64)
    with pytest.raises(B.DskError) as e:
        B.dsk_attention(B.DSK_BF16, t(n_q, Hq * dh), t(n_q, Hkv * dh), t(n_q, Hkv * dh), t(n_q, Hq * dh), qb.desc, None, 0,
                        Hq, Hkv, dh, scratch)
    assert e.value.status == B.DSK_ESHAPE
    # a prefix range that reaches into the queries' own rows
    pb = binding.Batch(synth.cu_seqlens([8]))
    with pytest.raises(B.DskError) as e:
        B.dsk_attention(B.DSK_BF16, t(n_q, 8 * 128), t(n_q + 4, 2 * 128), t(n_q + 4, 2 * 128), t(n_q, 8 * 128), qb.desc,
                        pb.desc, 4, 8, 2, 128, t(2 * 128 * 64))
    assert e.value.status == B.DSK_EINVAL
    torch.cuda.synchronize()


def test_bf16_model_with_unsupported_shape_is_refused_at_creation(B):
    # hidden 96 is no whole number of k-tiles; head_dim 32 has no tensor-core attention kernel
    for bad in (synth.ModelShape(2, 96, 2, 2, 64, 128, 1e4, 1e-5, "bf16"),
                synth.ModelShape(2, 128, 4, 4, 32, 128, 1e4, 1e-5, "bf16")):
        with pytest.raises(B.DskError) as e:
            B.dsk_model_create(B.config_from_shape(bad), 8, 8)
        assert e.value.status == B.DSK_ESHAPE
    # the same shapes are fine as fp32 models (plain-ALU kernels by design)
    ok = synth.ModelShape(2, 96, 2, 2, 64, 128, 1e4, 1e-5, "f32")
    B.dsk_model_destroy(B.dsk_model_create(B.config_from_shape(ok), 8, 8))


def test_bf16_model_runs_on_tensor_core_kernels(B):
    from tests import gpu_util as G
    shape = synth.ModelShape(2, 512, 8, 2, 128, 1536, 500000.0, 1e-5, "bf16")
    T = 200
    with G.GpuModel(shape, T) as m:
        m.init_random(0)
        B.dsk_set_option("reset_stats", 0)
        m.partial(G.to_dev(synth.hidden_states(shape, T), shape), 0, 2, None, [T])
        torch.cuda.synchronize()
        assert B.dsk_get_stat("gemm_mfma_launches") == 8 and B.dsk_get_stat("gemm_generic_launches") == 0
        assert B.dsk_get_stat("attn_mfma_launches") == 2 and B.dsk_get_stat("attn_generic_launches") == 0
