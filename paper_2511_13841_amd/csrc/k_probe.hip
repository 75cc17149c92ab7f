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
