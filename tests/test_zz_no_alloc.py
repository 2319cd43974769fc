"""tidar_gemm_static: the GEMM entry point that allocates nothing (its scratch is a static device array of the
library image).  Collected last on purpose (file name): it must pass after every other GPU test and alone."""
import pytest
import torch

import tidar_inputs as TI

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def T():
    import paper_2511_08923_amd as T
    assert torch.cuda.is_available()
    return T


def _pair(T, ctx, dtype, M, N, K, seed):
    """The workspace entry point and the static one on the same operands."""
    tdt = torch.bfloat16 if dtype == T.TIDAR_BF16 else torch.float32
    esz = 2 if dtype == T.TIDAR_BF16 else 4
    a = TI.make_normal((M, K), seed=seed, dtype=tdt).cuda()
    w = TI.make_normal((N, K), seed=seed + 1, dtype=tdt, std=0.02).cuda()
    packed = torch.zeros(T.tidar_packed_weight_bytes(dtype, N, K) // esz, dtype=tdt, device="cuda")
    T.tidar_pack_weight(dtype, w, packed, N)
    ws = torch.empty(T.tidar_gemm_workspace_bytes(dtype, M, N, K), dtype=torch.uint8, device="cuda")
    want = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    T.tidar_gemm(ctx, a, packed, want, M, N, K, ws)
    got = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    T.tidar_gemm_static(ctx, a, packed, got, M, N, K)
    torch.cuda.synchronize()
    return got, want, a, w


def test_static_scratch_gemm_equals_workspace_gemm_two_calls_in_a_row(T):
    """Two calls in a row through the C ABI, the second with a smaller input (its scratch then still holds the first
    call's A fragments and partial sums beyond what it overwrites): same kernels, same split plan, so the result
    must equal tidar_gemm's bit for bit; both stay within the GEMM tolerance of the fp64 product."""
    ctx = T.tidar_create(T.make_config(TI.SHAPE_8B.with_layers(1), T.TIDAR_BF16, max_k=16, max_batch=1))
    for M, N, K in [(272, 4096, 4096), (20, 1040, 1056), (272, 4096, 12288), (1, 6144, 4096), (33, 528, 288)]:
        print(f"static gemm M={M} N={N} K={K}", flush=True)
        got, want, a, w = _pair(T, ctx, T.TIDAR_BF16, M, N, K, seed=M + N)
        assert not torch.isnan(got).any()
        assert torch.equal(got, want), float((got - want).abs().max())
        ref = a.double().cpu() @ w.double().cpu().T
        assert float((got.cpu().double() - ref).abs().max()) < 2e-4 * (K / 256) ** 0.5
    T.tidar_destroy(ctx)


def test_static_scratch_gemm_fp32_and_limits(T):
    ctx = T.tidar_create(T.make_config(TI.TINY, T.TIDAR_F32, max_k=4, max_batch=1))
    for M, N, K in [(20, 512, 128), (3, 128, 512)]:
        got, want, a, w = _pair(T, ctx, T.TIDAR_F32, M, N, K, seed=5)
        assert torch.equal(got, want)
    T.tidar_destroy(ctx)
    ctx = T.tidar_create(T.make_config(TI.SHAPE_8B.with_layers(1), T.TIDAR_BF16, max_k=16, max_batch=1))
    M, N, K = 4096, 4096, 12288                       # needs far more than the 32 MiB array: refused on the host
    assert T.tidar_gemm_workspace_bytes(T.TIDAR_BF16, M, N, K) > T.STATIC_SCRATCH_BYTES
    dummy = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(16, dtype=torch.float32, device="cuda")
    with pytest.raises(T.TidarError) as e:
        T.tidar_gemm_static(ctx, dummy, dummy, out, M, N, K)
    assert e.value.status == 2
    T.tidar_destroy(ctx)
