// bf16 MFMA GEMM for the dense contractions of the verify step (QKV, O,
// gate/up, down, LM head):  C[M][N] = A[M][K] * W[N][K]^T, fp32 accumulation.
//
// Both operands live in HBM in MFMA fragment order (see das_internal.h), so a
// tile is a run of contiguous 4 KiB pieces: it is copied to LDS linearly and
// read back with lane-linear ds_read_b128 -- no swizzle, no bank conflicts.
// v_mfma_f32_32x32x16_bf16; the K loop of every output element runs in the same
// order whatever M is, so a row's result does not depend on the batch around it.
#include "das_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ bf16_t f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// 16-byte-per-lane asynchronous copy HBM -> LDS (no VGPR staging): lane l's 16 bytes land at lds + 16*l.
__device__ __forceinline__ void dma16(const void *g, void *lds_wave_base) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)g,
                                     (__attribute__((address_space(3))) void *)lds_wave_base, 16, 0, 0);
}

// WGM x WGN waves, each owning TM x TN blocks of 32x32.  BK = 64 (4 MFMA k-steps).
// Two k-tile stages live in two separate LDS arrays so that the compiler can tell the stage being
// filled by the DMA from the stage being read, and lets the copy run under the MFMAs.
template <int WGM, int WGN, int TM, int TN, int EPI>
__global__ __launch_bounds__(WGM *WGN * 64) void gemm_kernel(const bf16_t *__restrict__ A, const bf16_t *__restrict__ W,
                                                             void *__restrict__ Cv, int M, int N, int K, int ldc,
                                                             int tiles_m, int tiles_n) {
    constexpr int NT = WGM * WGN * 64;
    constexpr int AB = WGM * TM, BB = WGN * TN;          // 32-row blocks per tile
    constexpr int A_UNITS = AB * 256, B_UNITS = BB * 256; // 16-byte units per k-tile
    constexpr int NLOAD = (A_UNITS + B_UNITS) / NT;
    static_assert((A_UNITS + B_UNITS) % NT == 0, "tile must divide evenly over the threads");
    static_assert(A_UNITS % NT == 0, "A/W split must fall on a whole pass over the threads");
    constexpr int STAGE_BYTES = (AB + BB) * 4096;
    __shared__ __align__(16) unsigned char stage0[STAGE_BYTES];
    __shared__ __align__(16) unsigned char stage1[STAGE_BYTES];

    // XCD-aware tile order: the workgroups of one XCD (id % 8) walk a contiguous
    // run of tiles, M fastest, so tiles sharing a weight tile share an L2.
    const int nt = tiles_m * tiles_n;
    const int per_xcd = (nt + 7) >> 3;
    const int t = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (t >= nt) return;
    const int tile_m = t % tiles_m, tile_n = t / tiles_m;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int KF = K >> 4;                                 // fragments per row block
    const int KT = K >> 6;                                 // k-tiles
    const uint4 *Ag = reinterpret_cast<const uint4 *>(A);
    const uint4 *Wg = reinterpret_cast<const uint4 *>(W);

    // per-thread source of each 16-byte unit u = tid + j*NT: units below A_UNITS come from A, the rest from W
    const uint4 *src[NLOAD];
#pragma unroll
    for (int j = 0; j < NLOAD; ++j) {
        const int u = tid + j * NT;
        if (j * NT < A_UNITS) src[j] = Ag + ((size_t)(tile_m * AB + (u >> 8)) * KF) * 64 + (u & 255);
        else { const int v = u - A_UNITS; src[j] = Wg + ((size_t)(tile_n * BB + (v >> 8)) * KF) * 64 + (v & 255); }
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    auto issue = [&](int kt, unsigned char *stage) {       // 4 fragments = 256 uint4 per k-tile and row block
#pragma unroll
        for (int j = 0; j < NLOAD; ++j) dma16(src[j] + (size_t)kt * 256, stage + j * NT * 16 + wave * 1024);
    };
    auto compute = [&](const unsigned char *cur) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                a[i] = *reinterpret_cast<const bf16x8 *>(cur + ((wm * TM + i) * 4 + ks) * 1024 + lane * 16);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                b[j] = *reinterpret_cast<const bf16x8 *>(cur + AB * 4096 + ((wn * TN + j) * 4 + ks) * 1024 + lane * 16);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if (EPI == EPI_SILU_FRAG)   // transposed block: rows = weight rows, cols = activation rows
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
                    else
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
                }
        }
    };
    auto landed = [&]() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); __syncthreads(); };

    issue(0, stage0);
    landed();
    for (int kt = 0;; kt += 2) {                           // even k-tiles in stage0, odd ones in stage1
        if (kt + 1 < KT) issue(kt + 1, stage1);
        compute(stage0);
        if (kt + 1 >= KT) break;
        landed();
        if (kt + 2 < KT) issue(kt + 2, stage0);
        compute(stage1);
        if (kt + 2 >= KT) break;
        landed();
    }

    const int m0 = tile_m * AB * 32 + wm * TM * 32, n0 = tile_n * BB * 32 + wn * TN * 32;
    const int lr = lane & 31, lh = lane >> 5;
    if (EPI == EPI_SILU_FRAG) {
        // packed weight rows come in groups of 64: 32 gate rows then the 32 up rows of the same features
        bf16_t *out = reinterpret_cast<bf16_t *>(Cv);
        const int Fp = ldc;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = m0 + i * 32 + lr;
            if (row >= M) continue;
#pragma unroll
            for (int j = 0; j < TN; j += 2) {
                const int fbase = ((n0 + j * 32) >> 6) * 32;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    bf16_t o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float g = acc[i][j][q * 4 + e], u = acc[i][j + 1][q * 4 + e];
                        o[e] = f2bf(g / (1.f + __expf(-g)) * u);
                    }
                    const int f0 = fbase + 8 * q + 4 * lh;
                    *reinterpret_cast<uint2 *>(out + frag_off(row, f0, Fp)) = *reinterpret_cast<uint2 *>(o);
                }
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + j * 32 + lr;
                if (col >= N) continue;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = m0 + i * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                    if (row >= M) continue;
                    const size_t idx = (size_t)row * ldc + col;
                    if (EPI == EPI_BF16_ROWMAJOR) reinterpret_cast<bf16_t *>(Cv)[idx] = f2bf(acc[i][j][r]);
                    else if (EPI == EPI_RESID_F32) reinterpret_cast<float *>(Cv)[idx] += acc[i][j][r];
                    else reinterpret_cast<float *>(Cv)[idx] = acc[i][j][r];
                }
            }
    }
}

template <int WGM, int WGN, int TM, int TN>
static void launch_cfg(int epi, const bf16_t *A, const bf16_t *W, void *C, int M, int N, int K, int ldc, hipStream_t st) {
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int nt = tiles_m * tiles_n;
    const int grid = ((nt + 7) / 8) * 8;
    const size_t lds = 0;     // the two k-tile stages are static LDS arrays
    dim3 g(grid), b(WGM * WGN * 64);
    switch (epi) {
    case EPI_BF16_ROWMAJOR:
        gemm_kernel<WGM, WGN, TM, TN, EPI_BF16_ROWMAJOR><<<g, b, lds, st>>>(A, W, C, M, N, K, ldc, tiles_m, tiles_n); break;
    case EPI_RESID_F32:
        gemm_kernel<WGM, WGN, TM, TN, EPI_RESID_F32><<<g, b, lds, st>>>(A, W, C, M, N, K, ldc, tiles_m, tiles_n); break;
    case EPI_SILU_FRAG:
        gemm_kernel<WGM, WGN, TM, TN, EPI_SILU_FRAG><<<g, b, lds, st>>>(A, W, C, M, N, K, ldc, tiles_m, tiles_n); break;
    default:
        gemm_kernel<WGM, WGN, TM, TN, EPI_F32_ROWMAJOR><<<g, b, lds, st>>>(A, W, C, M, N, K, ldc, tiles_m, tiles_n); break;
    }
}

// A must be allocated for M rounded up to 256 rows, W for N rounded up to 256 rows; K % 64 == 0.
// For EPI_SILU_FRAG, N counts packed (gate+up interleaved) rows and ldc is the padded FFN width.
void launch_gemm(int epi, const bf16_t *A, const bf16_t *W, void *C, int M, int N, int K, int ldc, hipStream_t st) {
    if (M <= 0) return;
    launch_cfg<2, 2, 2, 2>(epi, A, W, C, M, N, K, ldc, st);
}
