// Copy-ring probe: the HBM/L2 -> LDS tile ring of the GEMM and attention kernels with nothing else in it.
//
// Every kernel of the verify step that matters is fed by the same mechanism: waves issue asynchronous 16-byte-per-lane
// copies straight into a ring of LDS stages, wait with s_waitcnt vmcnt(n) until the oldest tile has landed, meet at a
// barrier, and refill the stage they left.  This probe runs exactly that loop over synthetic buffers, so that the rate
// a workgroup can pull through it -- as a function of ring depth, of how many workgroups run, of the share of copies
// that find their line in L2, and of the non-temporal hint -- is a measurement of its own, not an inference from the
// kernels' timings.  Test and measurement infrastructure: nothing of the verify step calls it.
#include "das_internal.h"

namespace {

__device__ __forceinline__ void ring_copy(const void *g, uint32_t lds_wave_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_wave_base) : "memory", "m0");
}
__device__ __forceinline__ void ring_copy_nt(const void *g, uint32_t lds_wave_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" ::"v"(g), "s"(lds_wave_base) : "memory", "m0");
}

// 4 waves; a tile is 4 * NL KiB: every wave issues NL copies of 1 KiB per tile.  The first `nls` copies of a wave read a
// region of 64 tiles that all workgroups share (L2 hits after the first touches), the others the workgroup's own stream
// (every line once: misses).  priv: [workgroups][tiles][4][NL - nls] KiB; shared_r: [64][4][nls] KiB.
// (Everything but the tile count is a compile-time constant: at 130 GB/s a CU takes a 16-KiB tile every 250 cycles, and
// address arithmetic or branches per copy at run time halve the rate the loop can issue.)
template <int NS, int NL, int NLS, bool NT>
__global__ __launch_bounds__(256) void copy_ring_kernel(const uint4 *__restrict__ priv, const uint4 *__restrict__ shared_r, int tiles) {
    constexpr int nls = NLS;
    extern __shared__ __align__(16) unsigned char smem[];
    const uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    constexpr int STAGE = 4 * NL * 1024;
    constexpr int npv = NL - nls;      // private copies per wave and tile
    const uint4 *p = priv + (size_t)blockIdx.x * tiles * 4 * npv * 64 + (size_t)wave * npv * 64 + lane;
    const uint4 *s = shared_r + (size_t)wave * nls * 64 + lane;
    auto issue = [&](int t, int stage) {
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const uint32_t dst = base + stage * STAGE + (wave * NL + j) * 1024;
            if (j < nls) ring_copy(s + ((size_t)(t & 63) * 4 * nls + j) * 64, dst);
            else if (NT) ring_copy_nt(p + ((size_t)t * 4 * npv + (j - nls)) * 64, dst);
            else ring_copy(p + ((size_t)t * 4 * npv + (j - nls)) * 64, dst);
        }
    };
    const int last = tiles - 1;
#pragma unroll
    for (int s0 = 0; s0 < NS - 1; ++s0) issue(min(s0, last), s0);
    int stage = 0;
    for (int t = 0; t < tiles; ++t) {
        constexpr int NEWER = (NS - 2) * NL;
        __builtin_amdgcn_s_waitcnt(0xF70 | (NEWER & 15) | ((NEWER >> 4) << 14));      // vmcnt only: tile t has landed
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        issue(min(t + NS - 1, last), stage == 0 ? NS - 1 : stage - 1);
        stage = stage == NS - 1 ? 0 : stage + 1;
    }
    __builtin_amdgcn_s_waitcnt(0xF70);      // no copy may land in LDS after the workgroup is gone
}

template <int NS, int NL, int NLS, bool NT>
hipError_t launch_ring(const uint4 *priv, const uint4 *shared_r, int workgroups, int tiles, hipStream_t st) {
    static_assert((NS - 2) * NL <= 63 && NS * 4 * NL <= 144, "6-bit counter; ring within the LDS of one CU");
    auto k = copy_ring_kernel<NS, NL, NLS, NT>;
    // more than half of the CU's LDS whatever the ring needs: one workgroup per CU, so "workgroups" counts busy CUs
    constexpr int LDS = NS * 4 * NL * 1024 > 96 * 1024 ? NS * 4 * NL * 1024 : 96 * 1024;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (e != hipSuccess) return e;
    k<<<dim3(workgroups), dim3(256), LDS, st>>>(priv, shared_r, tiles);
    return hipGetLastError();
}


// ---------------------------------------------------------------------------------------------------------------------
// Matrix-pipe probe: what a loop of v_mfma_f32_32x32x16_bf16 delivers, and at which shader clock.
//
// 256 workgroups of 4 waves (one per SIMD; more than half of a CU's LDS each, so one workgroup per CU), every wave issuing
// 16 independent MFMAs per k-step, as a wave of the 256x256-tile GEMM does.  MODE 0: operands constant, in registers.
// MODE 1: the 8 operand fragments of every k-step are read from LDS (pseudo-random bf16 bit patterns) one k-step ahead,
// requests dealt out one per MFMA as in the GEMM's pipelined loop.  MODE 2: as 1, plus the GEMM's copy traffic: per
// k-tile of two k-steps every wave copies 8 KiB from an L2-resident region into a four-stage LDS ring, with the
// s_waitcnt + s_barrier per k-tile of the real loop.  Thread 0 of one workgroup brackets the loop with the shader-clock
// counter (s_memtime) and the constant 100 MHz counter (s_memrealtime): their ratio is the clock the loop ran at.
typedef __attribute__((ext_vector_type(8))) __bf16 probe_bf16x8;
typedef __attribute__((ext_vector_type(16))) float probe_f32x16;

template <int MODE>
__global__ __launch_bounds__(256) void mfma_loop_kernel(const uint4 *__restrict__ src, float *__restrict__ sink, int iters,
                                                        long long *__restrict__ clk) {
    extern __shared__ __align__(16) unsigned char smem[];      // 128 KiB: four stages of 32 KiB
    const uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int i = tid; i < 32768; i += 256) {      // bf16 pairs with random sign and mantissa, exponents of 0.5 .. 2
        uint32_t h = (uint32_t)i * 2654435761u; h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        reinterpret_cast<uint32_t *>(smem)[i] = (h & 0x807F807Fu) | 0x3F003F00u;
    }
    __syncthreads();
    probe_bf16x8 fa[2][4], fb[2][4];
    for (int p = 0; p < 2; ++p)
        for (int q = 0; q < 4; ++q)
            for (int i = 0; i < 8; ++i) { fa[p][q][i] = (__bf16)1.0f; fb[p][q][i] = (__bf16)1.0f; }
    probe_f32x16 acc[16];
    for (int i = 0; i < 16; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    const unsigned char *rb = smem + lane * 16 + (wave & 1) * 8192;
    const uint4 *g = src + (size_t)blockIdx.x * 8192 + wave * 512 + lane;      // 128 KiB per workgroup, re-read every other k-tile
    int stage = 0;
    const long long t0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            if (MODE == 2 && ks == 1) {
                __builtin_amdgcn_s_waitcnt(0xF70 | 8);      // all but the newest tile's copies have landed
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int m = 0; m < 16; ++m) {
                acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks][m & 3], fa[ks][m >> 2], acc[m], 0, 0, 0);
                if (MODE >= 1 && m < 4) fb[ks ^ 1][m] = *reinterpret_cast<const probe_bf16x8 *>(rb + stage * 32768 + 16384 + (ks * 4 + m) * 1024);
                else if (MODE >= 1 && m < 8) fa[ks ^ 1][m - 4] = *reinterpret_cast<const probe_bf16x8 *>(rb + stage * 32768 + (ks * 4 + m - 4) * 1024);
                else if (MODE == 2 && m >= 12)
                    ring_copy(g + ((ks * 4 + m - 12) * 4 + (it & 1) * 32) * 64, base + ((stage + 3) & 3) * 32768 + wave * 8192 + (ks * 4 + m - 12) * 1024);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (MODE >= 1) stage = (stage + 1) & 3;
    }
    __builtin_amdgcn_s_waitcnt(0xF70);
    const long long t1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
    if (blockIdx.x == 17 && tid == 0) { clk[0] = t1 - t0; clk[1] = r1 - r0; }
    float s = 0.f;
    for (int i = 0; i < 16; ++i)
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    if (s == 1.2345f) sink[0] = s;      // keeps the accumulators alive
}

}  // namespace

// the ring shapes that are built: stages, copies per wave and tile, of which shared
#define COPY_RING_SHAPES(X) X(4, 4, 0) X(9, 4, 0) X(4, 9, 0) X(4, 4, 4) X(9, 4, 4) X(4, 9, 9) X(4, 9, 6) X(4, 9, 3) X(5, 7, 5) X(3, 7, 5)

bool copy_ring_supported(int stages, int copies, int shared_copies) {
#define RING(ns, nl, nls) if (stages == ns && copies == nl && shared_copies == nls) return true;
    COPY_RING_SHAPES(RING)
#undef RING
    return false;
}

hipError_t launch_copy_ring(const void *priv, const void *shared_r, int workgroups, int stages, int copies, int shared_copies,
                            int tiles, bool non_temporal, hipStream_t st) {
    const uint4 *p = reinterpret_cast<const uint4 *>(priv), *s = reinterpret_cast<const uint4 *>(shared_r);
#define RING(ns, nl, nls) if (stages == ns && copies == nl && shared_copies == nls) \
        return (non_temporal && nls < nl) ? launch_ring<ns, nl, nls, (nls < nl)>(p, s, workgroups, tiles, st) : launch_ring<ns, nl, nls, false>(p, s, workgroups, tiles, st);
    COPY_RING_SHAPES(RING)
#undef RING
    return hipErrorInvalidValue;
}

// src: at least 256 x 128 KiB of initialised device memory; clk: two 64-bit counters (shader cycles, 100 MHz ticks)
hipError_t launch_mfma_loop(int mode, const void *src, float *sink, int iters, long long *clk, hipStream_t st) {
    const uint4 *p = reinterpret_cast<const uint4 *>(src);
    constexpr int LDS = 128 * 1024;
    auto go = [&](auto kern) -> hipError_t {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        kern<<<dim3(256), dim3(256), LDS, st>>>(p, sink, iters, clk);
        return hipGetLastError();
    };
    if (mode == 0) return go(mfma_loop_kernel<0>);
    if (mode == 1) return go(mfma_loop_kernel<1>);
    if (mode == 2) return go(mfma_loop_kernel<2>);
    return hipErrorInvalidValue;
}
