// Skinny bf16 GEMM for the decode step: out[M][N] (fp32) = A[M][K] (bf16) x W[N][K]^T (bf16, packed).
//
// M is the step's row count (1 .. 272 per pass), N and K are model dimensions, so every weight byte is used
// once per step and the kernel is a weight streamer with MFMA attached:
//   * W lives in HBM as the register image of the MFMA B operand ([16-column tile][32-wide k step][lane][8]),
//     so a wave's load of one fragment is one fully coalesced 1 KiB read that goes straight to VGPRs.  Each
//     wave owns its column tiles exclusively: weights never pass through LDS and are never read twice.
//   * A (small, L2 resident) is staged through LDS once per workgroup and shared by its four waves.
//   * split-K over blockIdx.y fills the 256 CUs when N alone gives too few workgroups; partial sums go to
//     out[split][M][N] and are summed in fixed order by the consumer kernel (deterministic, no atomics).
// MFMA: v_mfma_f32_16x16x32_bf16.  A operand lane l: row l%16, k slots 8*(l/16)..+7;  B operand lane l:
// column l%16, same k slots;  D lane l register i: row 4*(l/16)+i, column l%16.
#include "tidar_internal.h"

namespace {

template <int MT> struct GemmCfg;
template <> struct GemmCfg<1>  { static constexpr int BK = 512; };
template <> struct GemmCfg<2>  { static constexpr int BK = 256; };
template <> struct GemmCfg<5>  { static constexpr int BK = 128; };
template <> struct GemmCfg<9>  { static constexpr int BK = 64; };
template <> struct GemmCfg<17> { static constexpr int BK = 64; };

// PF = weight chunks kept in flight per wave (register ring).
template <int MT, int NT, int PF>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const bf16_t *__restrict__ a, const bf16_t *__restrict__ w,
                                                        float *__restrict__ out, int M, int N, int K, int splits) {
    constexpr int BK = GemmCfg<MT>::BK;
    constexpr int KS = BK / 32;                 // MFMA k steps per chunk
    constexpr int ROWS = MT * 16;
    constexpr int LDS_STRIDE = BK + 8;          // bf16 elements; +16 bytes keeps ds_read_b128 conflict free
    constexpr int PIECES = ROWS * (BK / 8);     // 16-byte pieces per chunk
    constexpr int STAGE = (PIECES + 255) / 256; // pieces per thread
    extern __shared__ __attribute__((aligned(16))) unsigned char gemm_smem[];
    bf16_t (*lds)[ROWS * LDS_STRIDE] = reinterpret_cast<bf16_t (*)[ROWS * LDS_STRIDE]>(gemm_smem);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_tiles = N / 16, ksteps_total = K / 32;
    const int m_base = blockIdx.z * ROWS;
    const int split = blockIdx.y;
    const int n_chunks = (K + BK - 1) / BK;
    const int per = (n_chunks + splits - 1) / splits;
    const int c0 = split * per;
    const int c1 = min(n_chunks, c0 + per);
    const int tile0 = (blockIdx.x * 4 + wave) * NT;          // this wave's first column tile
    const bool wave_active = tile0 < n_tiles;

    f32x4 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // ---- A staging: thread -> (row, 16-byte piece) pairs of the chunk
    bf16x8 stage[STAGE];
    auto load_a = [&](int chunk) {
#pragma unroll
        for (int s = 0; s < STAGE; ++s) {
            int p = tid + s * 256;
            int row = p / (BK / 8), piece = p % (BK / 8);
            int kk = chunk * BK + piece * 8;
            bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (p < PIECES && m_base + row < M && kk < K)
                v = *(const bf16x8 *)(a + (size_t)(m_base + row) * K + kk);
            stage[s] = v;
        }
    };
    auto store_a = [&](int buf) {
#pragma unroll
        for (int s = 0; s < STAGE; ++s) {
            int p = tid + s * 256;
            int row = p / (BK / 8), piece = p % (BK / 8);
            if (p < PIECES) *(bf16x8 *)(&lds[buf][row * LDS_STRIDE + piece * 8]) = stage[s];
        }
    };

    // ---- W ring: wbuf[slot][nt][ks]
    bf16x8 wbuf[PF][NT][KS];
    auto load_w = [&](int slot, int chunk) {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            int tile = tile0 + j;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                int q = chunk * KS + ks;
                bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
                if (tile < n_tiles && q < ksteps_total)
                    v = *(const bf16x8 *)(w + (((size_t)tile * ksteps_total + q) * 64 + lane) * 8);
                wbuf[slot][j][ks] = v;
            }
        }
    };

    if (c0 < c1) {
        load_a(c0);
#pragma unroll
        for (int i = 0; i < PF; ++i)
            if (c0 + i < c1 && wave_active) load_w(i, c0 + i);
        store_a(0);
    }
    __syncthreads();

    const int a_lane_off = (lane & 15) * LDS_STRIDE + (lane >> 4) * 8;
    for (int cb = c0; cb < c1; cb += PF) {
#pragma unroll
        for (int i = 0; i < PF; ++i) {
            const int c = cb + i;
            if (c < c1) {
                const int buf = (c - c0) & 1;
                if (c + 1 < c1) load_a(c + 1);
                if (wave_active) {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) {
                            bf16x8 af = *(const bf16x8 *)(&lds[buf][mt * 16 * LDS_STRIDE + a_lane_off + ks * 32]);
#pragma unroll
                            for (int j = 0; j < NT; ++j)
                                acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, wbuf[i][j][ks], acc[mt][j],
                                                                                     0, 0, 0);
                        }
                    }
                    if (c + PF < c1) load_w(i, c + PF);
                }
                if (c + 1 < c1) store_a(buf ^ 1);
                __syncthreads();
            }
        }
    }

    // ---- epilogue: D lane l reg i -> row 4*(l/16)+i, column l%16
    if (wave_active) {
        float *o = out + (size_t)split * M * N;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                int tile = tile0 + j;
                if (tile >= n_tiles) continue;
                int col = tile * 16 + (lane & 15);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    int row = m_base + mt * 16 + (lane >> 4) * 4 + i;
                    if (row < M) o[(size_t)row * N + col] = acc[mt][j][i];
                }
            }
        }
    }
}

template <int MT, int NT>
void launch_cfg(const bf16_t *a, const bf16_t *w, float *out, int M, int N, int K, const GemmPlan &p, hipStream_t st) {
    int n_tiles = N / 16;
    dim3 grid((n_tiles + 4 * NT - 1) / (4 * NT), p.splits, p.m_chunks);
    constexpr int PF = (NT == 4) ? 2 : ((MT >= 9) ? 4 : 2);
    constexpr int BK = GemmCfg<MT>::BK;
    constexpr size_t SMEM = (size_t)2 * MT * 16 * (BK + 8) * sizeof(bf16_t);
    static bool attr_set = false;          // LDS above 64 KiB has to be granted per kernel
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void *)gemm_bf16_kernel<MT, NT, PF>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)SMEM);
        attr_set = true;
    }
    gemm_bf16_kernel<MT, NT, PF><<<grid, 256, SMEM, st>>>(a, w, out, M, N, K, p.splits);
}

template <int MT>
void launch_mt(const bf16_t *a, const bf16_t *w, float *out, int M, int N, int K, const GemmPlan &p, hipStream_t st) {
    if (p.nt == 1) launch_cfg<MT, 1>(a, w, out, M, N, K, p, st);
    else if (p.nt == 2 || MT < 9) launch_cfg<MT, 2>(a, w, out, M, N, K, p, st);
    else if constexpr (MT >= 9) launch_cfg<MT, 4>(a, w, out, M, N, K, p, st);
}

}  // namespace

GemmPlan plan_gemm_bf16(int M, int N, int K, bool force_single_split) {
    GemmPlan p;
    int m_tiles = (M + 15) / 16;
    if (m_tiles <= 1) p.mt = 1;
    else if (m_tiles <= 2) p.mt = 2;
    else if (m_tiles <= 5) p.mt = 5;
    else if (m_tiles <= 9) p.mt = 9;
    else p.mt = 17;
    p.m_chunks = (m_tiles + p.mt - 1) / p.mt;
    p.bk = p.mt == 1 ? 512 : p.mt == 2 ? 256 : p.mt == 5 ? 128 : 64;
    int n_tiles = N / 16;
    // columns per workgroup: wide enough that A's L2 traffic stays a small multiple of the weight stream,
    // narrow enough that split-K partials stay small
    p.nt = (p.mt >= 9) ? 2 : 1;
    if (n_tiles >= 4 * 4 * 512) p.nt = (p.mt >= 9) ? 4 : 2;     // very wide N (LM head)
    if (p.mt < 9 && p.nt > 2) p.nt = 2;
    int wgs = (n_tiles + 4 * p.nt - 1) / (4 * p.nt);
    int n_chunks = (K + p.bk - 1) / p.bk;
    int splits = 1;
    if (!force_single_split && wgs * p.m_chunks < 224) {
        splits = (256 + wgs * p.m_chunks - 1) / (wgs * p.m_chunks);
        if (splits > n_chunks) splits = n_chunks;
        if (splits > 16) splits = 16;
        // avoid empty trailing splits
        int per = (n_chunks + splits - 1) / splits;
        splits = (n_chunks + per - 1) / per;
    }
    p.splits = splits < 1 ? 1 : splits;
    return p;
}

void launch_gemm_bf16(const bf16_t *a, const bf16_t *w, float *out, int M, int N, int K, const GemmPlan &p,
                      hipStream_t st) {
    switch (p.mt) {
        case 1: launch_mt<1>(a, w, out, M, N, K, p, st); break;
        case 2: launch_mt<2>(a, w, out, M, N, K, p, st); break;
        case 5: launch_mt<5>(a, w, out, M, N, K, p, st); break;
        case 9: launch_mt<9>(a, w, out, M, N, K, p, st); break;
        default: launch_mt<17>(a, w, out, M, N, K, p, st); break;
    }
}
