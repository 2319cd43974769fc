"""GPU parity of the two heavy kernels on their own, through the C ABI: skinny GEMM and hybrid-mask attention."""
import math

import pytest
import torch

import tidar_inputs as TI
from oracle import tidar_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def T():
    import paper_2511_08923_amd as T
    assert torch.cuda.is_available()
    return T


@pytest.fixture(scope="module")
def ctx8b(T):
    ctx = T.tidar_create(T.make_config(TI.SHAPE_8B.with_layers(1), T.TIDAR_BF16, max_k=16, max_batch=4))
    yield ctx
    T.tidar_destroy(ctx)


def _gemm(T, ctx, a, w):
    M, K = a.shape
    N = w.shape[0]
    ad, wd = a.cuda(), w.cuda()
    packed = torch.zeros(T.tidar_packed_weight_bytes(T.TIDAR_BF16, N, K) // 2, dtype=torch.bfloat16, device="cuda")
    T.tidar_pack_weight(T.TIDAR_BF16, wd, packed, N)
    out = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(T.tidar_gemm_workspace_bytes(T.TIDAR_BF16, M, N, K), dtype=torch.uint8, device="cuda")
    T.tidar_gemm(ctx, ad, packed, out, M, N, K, ws)
    torch.cuda.synchronize()
    return out.cpu()


# M spans every row-tile class and ragged tails; N covers a non-multiple of the workgroup width; K ragged vs chunk
@pytest.mark.parametrize("M,N,K", [(1, 256, 512), (1, 4096, 4096), (3, 2048, 1536), (16, 1024, 8960), (20, 6144, 4096),
                                   (33, 528, 288), (72, 4096, 4096), (81, 1040, 1056), (144, 2048, 12288),
                                   (145, 784, 608), (272, 6144, 4096), (272, 4096, 12288), (272, 24576, 4096),
                                   (273, 512, 256), (600, 1024, 1024),
                                   # 256-column workgroups with a ragged last block and an odd 32-column tile count
                                   (272, 16400, 512), (161, 16384, 256), (289, 32752, 384),
                                   # row passes: 3 tiles as 2+1, 5 as 3+2, 7 as 4+3, 12 as 6+6; one tile (no row split)
                                   (65, 4096, 2048), (160, 1536, 1536), (200, 4096, 1024), (384, 2048, 4096),
                                   (40, 6144, 1024),
                                   # two row passes with the waves side by side, one column tile each: passes of
                                   # 1 (one real row in the second), 2, 6+5, 7+6 and 8+7 tiles, ragged N and K
                                   (33, 784, 608), (100, 1040, 1056), (350, 528, 288), (416, 784, 608),
                                   (470, 1040, 1056),
                                   # 512 rows and more: 256 x 256 workgroup tiles (eight row tiles per wave, half-size
                                   # staging ring), whole and ragged row passes, split K, ragged column block, an
                                   # odd chunk count (K = 384), and a grid wide enough for the XCD super-tiles
                                   (512, 1024, 1024), (1000, 4096, 4096), (1025, 784, 608), (2176, 1536, 12288),
                                   (600, 16400, 384), (777, 65536 + 48, 256),
                                   # six row tiles per pass (17 tiles as 6+6+5, 18 as 6+6+6)
                                   (544, 2048, 1024), (576, 6144, 512),
                                   # many rows: the split count follows the number of 256-row passes (3, 2 and 1
                                   # splits where up to 1024 rows take 4)
                                   (1280, 4096, 4096), (1536, 4096, 2048), (2176, 4096, 4096)])
def test_gemm_matches_oracle_matmul(T, ctx8b, M, N, K):
    print(f"gemm M={M} N={N} K={K}", flush=True)
    a = TI.make_normal((M, K), seed=M * 7 + K, dtype=torch.bfloat16)
    w = TI.make_normal((N, K), seed=N * 3 + K, dtype=torch.bfloat16, std=0.02)
    got = _gemm(T, ctx8b, a, w)
    want = a.double() @ w.double().T
    err = float((got.double() - want).abs().max())
    assert not torch.isnan(got).any()
    assert err < 2e-4 * math.sqrt(K / 256), err


def test_gemm_lm_head_shape_sampled(T, ctx8b):
    """Full LM-head width at the benchmark's row count; the oracle computes sampled columns."""
    M, N, K = 272, 151936, 4096
    a = TI.make_normal((M, K), seed=1, dtype=torch.bfloat16)
    w = TI.make_normal((N, K), seed=2, dtype=torch.bfloat16, std=0.02)
    got = _gemm(T, ctx8b, a, w)
    cols = torch.cat([torch.arange(0, 64), torch.arange(75000, 75064), torch.arange(N - 64, N),
                      torch.randint(0, N, (256,), generator=torch.Generator().manual_seed(3))])
    want = a.double() @ w[cols].double().T
    assert float((got[:, cols].double() - want).abs().max()) < 1e-3
    assert not torch.isnan(got).any()


def _attention_case(T, shape, B, Ls, nc, nb, bl, cond0, seed, dtype_id):
    """Runs tidar_hybrid_attention on seeded inputs and returns (device output, oracle output) per sequence."""
    tdt = torch.bfloat16 if dtype_id == T.TIDAR_BF16 else torch.float32
    ctx = T.tidar_create(T.make_config(shape.with_layers(1), dtype_id, max_k=16, max_batch=B))
    n_q, n_kv, hd = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    R = nc + nb * bl
    Lmax = max(Ls)
    pps = (Lmax + nc + 15) // 16 + 1
    n_pages = B * pps + 5
    table = TI.shuffled_page_table(B * pps, n_pages, seed).view(B, pps)
    kp = torch.full((1, n_pages, n_kv, 16, hd), float("nan"), dtype=tdt)       # stale slots must never leak
    vp = torch.full((1, n_pages, n_kv, hd, 16), float("nan"), dtype=tdt)
    pk = [TI.make_normal((Ls[b], n_kv, hd), seed + 10 + b, tdt) for b in range(B)]
    pv = [TI.make_normal((Ls[b], n_kv, hd), seed + 20 + b, tdt) for b in range(B)]
    for b in range(B):
        for p in range(Ls[b]):
            kp[0, table[b, p // 16], :, p % 16, :] = pk[b][p]
            vp[0, table[b, p // 16], :, :, p % 16] = pv[b][p]
    q = TI.make_normal((B, R, n_q, hd), seed + 1, tdt)
    kn = TI.make_normal((B, R, n_kv, hd), seed + 2, tdt)
    vn = TI.make_normal((B, R, n_kv, hd), seed + 3, tdt)
    dev = lambda t: t.cuda().contiguous()
    kpd, vpd, tabd = dev(kp), dev(vp), dev(table)
    kv = T.tidar_kv_cache(kpd.data_ptr(), vpd.data_ptr(), tabd.data_ptr(), pps, n_pages)
    plen = torch.tensor(Ls, dtype=torch.int32, device="cuda")
    out = torch.full((B, R, n_q, hd), float("nan"), dtype=tdt, device="cuda")
    ws = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    T.tidar_hybrid_attention(ctx, kv, 0, B, plen, dev(q), dev(kn), dev(vn), nc, nb, bl, cond0, out, Lmax, ws)
    torch.cuda.synchronize()
    T.tidar_destroy(ctx)
    results = []
    for b in range(B):
        L = Ls[b]
        if cond0 == 1 and nc == nb == bl:
            mask = O.decode_mask(nc, L)
        elif nb == 0:
            mask = O.causal_mask(nc, L)
        else:
            assert nb == 1 and cond0 == nc
            mask = O.prefill_mask(L + nc, bl)[L:]
        keys = torch.cat([pk[b], kn[b]]).double()
        vals = torch.cat([pv[b], vn[b]]).double()
        want = O.attention_dense(q[b].double(), keys, vals, mask)
        got = out[b].cpu().double()
        if dtype_id == T.TIDAR_BF16:
            # against the oracle's bf16 rounding points the device differs only where an fp32-level difference
            # flips one rounding (of a numerator or of the output): rare, and of bf16-ulp size (values are O(1))
            faithful = O.round_bf16(O.attention_dense(q[b].double(), keys, vals, mask, round_p=True))
            diff = (got - faithful).abs()
            assert bool((diff <= faithful.abs().clamp(min=0.5) * 2.0 ** -7).all()), float(diff.max())
            assert float((diff > 0).double().mean()) < 0.02
        results.append((got, want))
    # the causal rows' K/V must have landed in the cache at L..L+nc-1
    for b in range(B):
        for i in (0, nc - 1):
            p = Ls[b] + i
            assert torch.equal(kpd[0, table[b, p // 16], :, p % 16, :].cpu(), kn[b, i])
            assert torch.equal(vpd[0, table[b, p // 16], :, :, p % 16].cpu(), vn[b, i])
    return results


@pytest.mark.parametrize("k,L", [(1, 0), (2, 1), (3, 5), (4, 17), (4, 33), (8, 100), (16, 0), (16, 15), (16, 16),
                                 (16, 300), (5, 64)])
def test_hybrid_attention_bf16_small(T, k, L):
    print(f"attn bf16 k={k} L={L}", flush=True)
    for got, want in _attention_case(T, TI.SMALL_GQA, 1, [L], k, k, k, 1, seed=100 * k + L, dtype_id=T.TIDAR_BF16):
        assert not torch.isnan(got).any()
        assert torch.allclose(got, want, atol=1e-2, rtol=2e-2), float((got - want).abs().max())


def test_hybrid_attention_bf16_batch_ragged_prefixes(T):
    res = _attention_case(T, TI.SMALL_GQA, 3, [7, 130, 64], 4, 4, 4, 1, seed=5, dtype_id=T.TIDAR_BF16)
    for got, want in res:
        assert torch.allclose(got, want, atol=1e-2, rtol=2e-2), float((got - want).abs().max())


@pytest.mark.parametrize("nc,nb,bl,cond0,L", [(1, 0, 1, 1, 200), (1, 0, 1, 1, 0), (40, 1, 8, 40, 64),
                                              (256, 1, 16, 256, 256), (256, 0, 16, 256, 0),
                                              # causal passes of many tiles: the rows of the pass before a tile run
                                              # in the loop without predicate, a different count for every wave
                                              (600, 1, 16, 600, 77), (333, 0, 16, 333, 1000)])
def test_hybrid_attention_bf16_ar_and_prefill_shapes(T, nc, nb, bl, cond0, L):
    print(f"attn bf16 nc={nc} nb={nb} bl={bl} L={L}", flush=True)
    for got, want in _attention_case(T, TI.SMALL_GQA, 1, [L], nc, nb, bl, cond0, seed=nc + L, dtype_id=T.TIDAR_BF16):
        assert torch.allclose(got, want, atol=1e-2, rtol=2e-2), float((got - want).abs().max())


def test_hybrid_attention_bf16_microbench_shape(T):
    """The attention micro-benchmark configuration: 32 query / 8 kv heads, head_dim 128, prefix 4096 in shuffled
    16-token pages, k = 16 (272 rows)."""
    print("attn bf16 config-2 shape", flush=True)
    (got, want), = _attention_case(T, TI.SHAPE_8B, 1, [4096], 16, 16, 16, 1, seed=42, dtype_id=T.TIDAR_BF16)
    assert not torch.isnan(got).any()
    assert torch.allclose(got, want, atol=1e-2, rtol=2e-2), float((got - want).abs().max())


@pytest.mark.parametrize("k,L", [(1, 0), (3, 5), (4, 64), (4, 77)])
def test_hybrid_attention_fp32(T, k, L):
    for got, want in _attention_case(T, TI.TINY, 2, [L, max(L - 3, 0)], k, k, k, 1, seed=k + L, dtype_id=T.TIDAR_F32):
        assert torch.allclose(got, want, atol=2e-5), float((got - want).abs().max())


@pytest.mark.parametrize("L1,L2,nc", [(990, 968, 40), (290, 260, 48), (4100, 4070, 272), (2050, 2000, 272)])
def test_attention_row_does_not_depend_on_how_much_of_its_context_is_cached(T, L1, L2, nc):
    """The same query over the same keys in two calls of the same shape (nc new causal rows, one bound on the key
    count), once after L1 cached keys, once after L2 < L1: the rows at positions [L1, L2 + nc) appear in both, with
    the same context, and their outputs must be the same bits.  Between L2 and L1 lie key pages that are plain
    prefix in one call (the kernel's loop without predicate and without a rescale arm) and predicated pages in the
    other; the key splits are the same (same bound, same row count), and the softmax reference of a row moves by a
    rule that looks at its keys alone, so nothing of that difference may show.  8B-shape heads (32 query / 8 kv
    heads); the scores are N(0, 16), so that a row's running maximum keeps moving over thousands of keys."""
    sh = TI.SHAPE_8B.with_layers(1)
    n_q, n_kv, hd = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    tdt = torch.bfloat16
    ctx = T.tidar_create(T.make_config(sh, T.TIDAR_BF16, max_k=16, max_batch=1))
    total = L1 + nc
    pps = (total + 15) // 16 + 1
    table = TI.shuffled_page_table(pps, pps + 3, seed=total).view(1, pps)
    K = TI.make_normal((total, n_kv, hd), total + 1, tdt)
    V = TI.make_normal((total, n_kv, hd), total + 2, tdt)
    Q = TI.make_normal((total, n_q, hd), total + 3, tdt, std=4.0)       # scores ~ N(0, 4^2): the running maximum keeps growing
    ws = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    outs = {}
    for L in (L1, L2):
        print(f"attention rows at {L}..{L + nc - 1}", flush=True)
        kp = torch.zeros((1, pps + 3, n_kv, 16, hd), dtype=tdt)
        vp = torch.zeros((1, pps + 3, n_kv, hd, 16), dtype=tdt)
        for p in range(L):
            kp[0, table[0, p // 16], :, p % 16, :] = K[p]
            vp[0, table[0, p // 16], :, :, p % 16] = V[p]
        kpd, vpd, tabd = kp.cuda(), vp.cuda(), table.cuda().contiguous()
        kv = T.tidar_kv_cache(kpd.data_ptr(), vpd.data_ptr(), tabd.data_ptr(), pps, pps + 3)
        out = torch.empty((1, nc, n_q, hd), dtype=tdt, device="cuda")
        plen = torch.tensor([L], dtype=torch.int32, device="cuda")
        sl = slice(L, L + nc)
        T.tidar_hybrid_attention(ctx, kv, 0, 1, plen, Q[sl].cuda().contiguous()[None], K[sl].cuda().contiguous()[None],
                                 V[sl].cuda().contiguous()[None], nc, 0, 1, 1, out, L1, ws)
        torch.cuda.synchronize()
        outs[L] = out[0].cpu()
    a, b = outs[L1][: L2 + nc - L1], outs[L2][L1 - L2:]
    assert a.shape[0] >= 8 and not torch.isnan(a.float()).any()
    assert torch.equal(a, b), float((a.float() - b.float()).abs().max())
    T.tidar_destroy(ctx)


def test_hybrid_attention_bf16_every_prefix_length_mod_32(T):
    """The tile pipeline's edge cases in one sweep: prefix lengths 0..70 (every offset inside a key pair, an odd and
    an even number of key units, sequences that end in a partly filled page, workgroups with one or two iterations,
    splits that come out empty) for the decode shapes k = 4 and k = 16; cache pages start out as NaN."""
    for k in (4, 16):
        for L in list(range(0, 36)) + list(range(60, 71)):
            for got, want in _attention_case(T, TI.SMALL_GQA, 1, [L], k, k, k, 1, seed=1000 * k + L,
                                             dtype_id=T.TIDAR_BF16):
                assert not torch.isnan(got).any(), (k, L)
                assert torch.allclose(got, want, atol=1e-2, rtol=2e-2), (k, L, float((got - want).abs().max()))
