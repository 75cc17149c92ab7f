// bf16 MFMA GEMM for the dense contractions of the verify step (QKV, O,
// gate/up, down, LM head):  C[M][N] = A[M][K] * W[N][K]^T, fp32 accumulation.
//
// Both operands live in HBM in MFMA fragment order (see das_internal.h), so a
// tile is a run of contiguous 4 KiB pieces: it is copied to LDS linearly and
// read back with lane-linear ds_read_b128 -- no swizzle, no bank conflicts.
// v_mfma_f32_32x32x16_bf16; the K loop of every output element runs in the same
// order whatever M is, so a row's result does not depend on the batch around it.
#include "das_internal.h"
#include <cstdlib>
#include <type_traits>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ bf16_t f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// 16-byte-per-lane asynchronous copy HBM -> LDS (no VGPR staging): lane l's 16 bytes land at
// lds_wave_base + 16*l.  Issued as inline assembly so that the copies are ordered only by the explicit
// s_waitcnt/s_barrier below: the compiler's own bookkeeping would drain every copy in flight before
// the first LDS read after a loop header.  M0 carries the LDS address (1 wait state before its use).
__device__ __forceinline__ void dma16(const void *g, uint32_t lds_wave_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_wave_base) : "memory", "m0");
}

// The same copy with the non-temporal hint, for weight tiles that only this workgroup reads (see W_ONCE in gemm_kernel).
__device__ __forceinline__ void dma16_nt(const void *g, uint32_t lds_wave_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" ::"v"(g), "s"(lds_wave_base) : "memory", "m0");
}

// WGM x WGN waves, each owning TM x TN blocks of 32x32.  A k-tile is KS MFMA k-steps (BK = 16*KS: 64 or 32).  NS LDS stages form a
// ring: while k-tile kt is multiplied, k-tiles kt+1 .. kt+NS-2 are already in flight and the stage of
// kt-1 is being refilled with kt+NS-1.
//
// SL selects how K is summed.  0: one pass over K.  Narrow outputs (QKV, O, down) are DEFINED as a sum of K slices
// of `slice_tiles` k-tiles, each slice accumulated from zero and the slices added in ascending order, so that few-row
// launches can spread the slices over workgroups without changing a single bit of the result:
// 1: this workgroup walks all slices and folds each finished slice into a second set of registers;
// 2: this workgroup computes slice blockIdx.y and stores the raw fp32 partial to slab blockIdx.y of Cv ([slices][M][ldc]);
// 3: this workgroup walks the `xslices` slices of group blockIdx.y, folds them like 1 and stores the group's sum to slab
//    blockIdx.y of Cv ([groups][M][ldc]).
// A sum of eight slices (K >= 16384) is DEFINED as two groups of four, (((s0+s1)+s2)+s3) + (((s4+s5)+s6)+s7), so that the
// two halves of a long K can go to two workgroups (mode 3) and meet in one addition; with mode 1 `xslices` = 4 asks for
// that grouping inside one workgroup (only the small-tile kernels have the registers for it).
// PIPE: the k loop is pipelined across k-tiles and its instruction order is pinned (see k_loop_pipe).
template <int WGM, int WGN, int TM, int TN, int NS, int EPI, int KS = 4, bool SPREAD = (NS >= 3), int SL = 0, bool PIPE = false, bool WNT = false>
__global__ __launch_bounds__(WGM *WGN * 64) void gemm_kernel(const bf16_t *__restrict__ A, const bf16_t *__restrict__ W,
                                                             void *__restrict__ Cv, int M, int N, int K, int ldc,
                                                             int tiles_m, int tiles_n, int slice_tiles, int xslices,
                                                             const int *__restrict__ aux_tok, float aux_f, int copies_only, RopeEpi re) {
    constexpr int NT = WGM * WGN * 64;
    constexpr int AB = WGM * TM, BB = WGN * TN;          // 32-row blocks per tile
    constexpr int RBU = KS * 64;                          // 16-byte units of one row block in one k-tile
    constexpr int A_UNITS = AB * RBU, B_UNITS = BB * RBU; // 16-byte units per k-tile
    constexpr int UNITS = A_UNITS + B_UNITS;
    constexpr int NLOAD = (UNITS + NT - 1) / NT;         // every wave issues NLOAD copies per k-tile, so that one
    constexpr bool PADDED = (UNITS % NT) != 0;           // s_waitcnt fits all; surplus copies go to a dump area
    static_assert((NS - 2) * NLOAD <= 63, "vmcnt is a 6-bit counter");
    static_assert(EPI != EPI_SILU_FRAG || TN % 2 == 0, "gate and up blocks must sit in the same wave");
    constexpr bool TRANSPOSED = EPI == EPI_SILU_FRAG || EPI == EPI_ROWMAX || EPI == EPI_ROWSTATS || EPI == EPI_ROPE_KV;      // blocks with rows = weight rows
    constexpr int STAGE_BYTES = (AB + BB) * KS * 1024;
    extern __shared__ __align__(16) unsigned char smem[];

    // XCD-aware tile order: the workgroups of one XCD (id % 8) walk a contiguous
    // run of tiles, M fastest, so tiles sharing a weight tile share an L2.
    const int nt = tiles_m * tiles_n;
    int t, slice = 0;
    if (SL == 2 && xslices > 0) {
        // K slices over workgroups, one-dimensional grid: every XCD works on ONE slice (xslices divides 8), so the part of
        // the activation panel that an XCD reads is 1/xslices of it and stays in that XCD's L2 while the weights of the
        // slice stream past it once
        const int xcd = blockIdx.x & 7, per = 8 / xslices;
        slice = xcd % xslices;
        t = (int)(blockIdx.x >> 3) * per + xcd / xslices;
    } else {
        const int per_xcd = (nt + 7) >> 3;
        t = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
        if (SL >= 2) slice = blockIdx.y;
    }
    if (t >= nt) return;
    const int tile_m = t % tiles_m, tile_n = t / tiles_m;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int KF = K >> 4;                                 // fragments per row block
    const int KT = K / (16 * KS);                          // k-tiles
    const int wg_tiles = SL == 3 ? xslices * slice_tiles : slice_tiles;      // k-tiles of this workgroup (modes 2, 3)
    const int kt_begin = SL >= 2 ? slice * wg_tiles : 0;
    const int kt_end = SL >= 2 ? min(KT, kt_begin + wg_tiles) : KT;
    if (SL >= 2) Cv = reinterpret_cast<float *>(Cv) + (size_t)slice * M * ldc;
    const uint4 *Ag = reinterpret_cast<const uint4 *>(A);
    const uint4 *Wg = reinterpret_cast<const uint4 *>(W);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem + wave * 1024;

    // per-thread source of each 16-byte unit u = tid + j*NT: units below A_UNITS come from A, the rest from W
    const uint4 *src[NLOAD];
#pragma unroll
    for (int j = 0; j < NLOAD; ++j) {
        const int u = min(tid + j * NT, UNITS - 64 + lane);      // surplus waves re-read the last fragment
        if (u < A_UNITS) src[j] = Ag + ((size_t)(tile_m * AB + u / RBU) * KF) * 64 + (u % RBU);
        else {      // (tiles whose width does not divide 256 reach past the padded weight rows: those copies re-read the last block)
            const int v = u - A_UNITS, wb = min(tile_n * BB + v / RBU, ((N + 255) >> 8) * 8 - 1);
            src[j] = Wg + ((size_t)wb * KF) * 64 + (v % RBU);
        }
    }
    // surplus copies of the last pass (whole waves: UNITS is a multiple of 64) land behind the ring
    const bool surplus = PADDED && (wave * 64 + (NLOAD - 1) * NT >= UNITS);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // The 64-row gate/up tiles are launched for passes of up to 64 rows only: one M tile, so every weight byte is read by
    // exactly one workgroup.  Its weight copies carry the non-temporal hint, so that the stream does not push the
    // activation panel, which all workgroups share, out of L2 (decoding a batch of 64: 63.6 -> 61.0 us per layer).  A
    // compile-time choice: decided at run time in every kernel, the branch cost the many-row narrow GEMMs 4 %.
    // The same holds for every launch whose workgroups own ALL rows of the pass (one wave row, three or more row blocks
    // per wave: the few-row shapes): a weight tile is read by exactly one workgroup.
    constexpr bool W_ONCE = (EPI == EPI_SILU_FRAG && AB == 2 && !PIPE && (A_UNITS % NT) == 0) || (WGM == 1 && TM >= 3 && WNT);
    // (whether copy j of this wave is a weight copy is the same for all its lanes: the boundary is a multiple of 64)
    uint32_t wmask = 0;
#pragma unroll
    for (int j = 0; j < NLOAD; ++j) wmask |= (uint32_t)(wave * 64 + j * NT >= A_UNITS) << j;
    wmask = __builtin_amdgcn_readfirstlane(wmask);
    auto copy = [&](int j, int kt, int stage) {
        const uint32_t dst = (j == NLOAD - 1 && surplus) ? lds_base + NS * STAGE_BYTES : lds_base + stage * STAGE_BYTES + j * NT * 16;
        if (W_ONCE && ((wmask >> j) & 1)) dma16_nt(src[j] + (size_t)kt * RBU, dst);
        else dma16(src[j] + (size_t)kt * RBU, dst);
    };
    auto issue = [&](int kt, int stage) {                  // KS fragments = RBU uint4 per k-tile and row block
#pragma unroll
        for (int j = 0; j < NLOAD; ++j) copy(j, kt, stage);
    };
    // the copies of one k-tile, cut into KS slices that are issued between the MFMA k-steps: sixteen copies
    // issued back to back would fill the vector-memory queue and stall the wave that should be multiplying
    auto issue_slice = [&](int kt, int stage, int slice) {
#pragma unroll
        for (int j = 0; j < NLOAD; ++j)
            if (j % KS == slice) copy(j, kt, stage);
    };
    // Row blocks of this wave that hold rows below M.  In the last M tile a wave whose blocks are all (or, with
    // four blocks, half) past M skips their fragment reads and MFMAs: the workgroup still copies and
    // synchronises, but finishes early and frees its CU, which is worth ~10% when M is just past a multiple of
    // the tile height (T = 1088 = 4 x 256 + 64).  Straight-line variants only: per-block branches inside the
    // k loop make the compiler spill accumulators.
    // A short last M tile (at most four of its eight row blocks hold rows) of the 2 x 2 wave layout is split by COLUMNS
    // instead: every wave takes all valid row blocks and two of the eight column blocks, so that the four waves share
    // the work instead of two of them doing all of it (half the time for such a tile).
    constexpr bool CAN_COLSPLIT = PIPE && WGM == 2 && WGN == 2 && TM == 4 && TN == 4;
    const int tile_vb = min(AB, max(0, (M - tile_m * AB * 32 + 31) >> 5));      // row blocks of this tile that hold rows
    const bool colsplit = CAN_COLSPLIT && tile_vb <= 4;
    const int rb0 = colsplit ? 0 : wm * TM;              // first row block and column block of this wave inside the tile
    const int cb0 = colsplit ? wave * 2 : wn * TN;
    const int tnv = colsplit ? 2 : TN;                   // column blocks this wave owns
    // (copies_only: a timing mode of the debug entry point -- every wave takes the path of a wave without rows, so the
    // launch moves exactly the same bytes HBM/L2 -> LDS with the same synchronisation and multiplies nothing)
    const int vb = copies_only ? 0 : min(TM, max(0, (M - (tile_m * AB + rb0) * 32 + 31) >> 5));
    auto compute = [&](auto tm_tag, const unsigned char *cur, int next_kt, int next_stage) {
        constexpr int TMV = decltype(tm_tag)::value;      // row blocks 0 .. TMV-1 are multiplied
        // fragments of k-step ks+1 are requested before the MFMAs of k-step ks are issued
        bf16x8 a[2][TMV], b[2][TN];
        auto fetch = [&](int ks, int buf) {
#pragma unroll
            for (int i = 0; i < TMV; ++i)
                a[buf][i] = *reinterpret_cast<const bf16x8 *>(cur + ((wm * TM + i) * KS + ks) * 1024 + lane * 16);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                b[buf][j] = *reinterpret_cast<const bf16x8 *>(cur + AB * KS * 1024 + ((wn * TN + j) * KS + ks) * 1024 + lane * 16);
        };
        fetch(0, 0);
        if (!SPREAD) issue(next_kt, next_stage);     // two stages and many rows: no slack, request the next tile at once
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (SPREAD) issue_slice(next_kt, next_stage, ks);
            if (ks < KS - 1) fetch(ks + 1, (ks + 1) & 1);
#pragma unroll
            for (int i = 0; i < TMV; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if (TRANSPOSED)   // transposed block: rows = weight rows, cols = activation rows
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[ks & 1][j], a[ks & 1][i], acc[i][j], 0, 0, 0);
                    else
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks & 1][i], b[ks & 1][j], acc[i][j], 0, 0, 0);
                }
        }
    };

    // Copies are issued unconditionally (past the end: the last k-tile again, into a stage nobody will read),
    // so "all but the newest NS-2 tiles have landed" is the same s_waitcnt in every iteration.
    const int last = kt_end - 1;
#pragma unroll
    for (int s0 = 0; s0 < NS - 1; ++s0) issue(min(kt_begin + s0, last), s0);
    constexpr bool FOLD = SL == 1 || SL == 3;            // slices folded in registers
    constexpr bool GROUPS = SL == 1 && TM * TN <= 2;     // ... and two groups of slices kept apart (see above)
    f32x16 tot[FOLD ? TM : 1][FOLD ? TN : 1];            // sum of the finished slices
    f32x16 first[GROUPS ? TM : 1][GROUPS ? TN : 1];      // sum of the first group
    int folds = 0;
    if (FOLD) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) tot[FOLD ? i : 0][FOLD ? j : 0][r] = 0.f;
    }
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    auto fold = [&]() {      // (whole-vector operations: element loops over nine blocks are not unrolled and would put acc in memory)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                tot[FOLD ? i : 0][FOLD ? j : 0] += acc[i][j];
                acc[i][j] = zero16;
            }
        if (GROUPS && xslices > 0 && ++folds == xslices) {      // the first group is complete: the second starts from zero
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    first[GROUPS ? i : 0][GROUPS ? j : 0] = tot[FOLD ? i : 0][FOLD ? j : 0];
                    tot[FOLD ? i : 0][FOLD ? j : 0] = zero16;
                }
        }
    };
    auto total = [&]() {      // after the last fold: the sum of all slices goes back to acc for the epilogue
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                acc[i][j] = tot[FOLD ? i : 0][FOLD ? j : 0];
                if (GROUPS && xslices > 0 && folds >= xslices) acc[i][j] = first[GROUPS ? i : 0][GROUPS ? j : 0] + acc[i][j];
            }
    };
    // one copy of the whole k loop per variant (the choice is made once per wave, outside the loop)
    auto k_loop = [&](auto tm_tag) {
        int stage = 0, in_slice = 0;
        for (int kt = kt_begin; kt < kt_end; ++kt) {
            __builtin_amdgcn_s_waitcnt(0xF70 | ((NS - 2) * NLOAD & 15) | (((NS - 2) * NLOAD >> 4) << 14));   // vmcnt only
            __builtin_amdgcn_s_barrier();      // tile kt visible to all waves; all waves are done with tile kt-1
            asm volatile("" ::: "memory");
            const int refill = stage == 0 ? NS - 1 : stage - 1;
            if (decltype(tm_tag)::value == 0) issue(min(kt + NS - 1, last), refill);
            else compute(tm_tag, smem + stage * STAGE_BYTES, min(kt + NS - 1, last), refill);
            stage = stage == NS - 1 ? 0 : stage + 1;
            if (FOLD && decltype(tm_tag)::value != 0 && ++in_slice == slice_tiles) { fold(); in_slice = 0; }
        }
        if (FOLD && decltype(tm_tag)::value != 0) {      // the last, possibly shorter slice; then the total goes to the epilogue
            if (in_slice) fold();
            total();
        }
    };
    // PIPE: the k loop pipelined across k-tiles.  The barrier that publishes tile kt+1 sits before the LAST k-step of tile
    // kt, and the first fragments of tile kt+1 are requested right after it, so that their LDS latency (and the wait at
    // the barrier of the slower waves) passes under the MFMAs of that last k-step instead of in front of an idle matrix
    // pipe -- which is what a workgroup with one wave per SIMD cannot afford.  Needs NS >= 3 and spread copies: the
    // copy of tile kt+NS-1 starts after that barrier (every wave has left tile kt-1) and its remaining slices follow
    // in the first k-steps of tile kt+1; all of them are issued before the next such barrier, so "tile kt+1 has
    // landed" is again one constant s_waitcnt: at most NS-3 newer tiles outstanding.
    auto k_loop_pipe = [&](auto tm_tag, auto tn_tag) {
        constexpr int TMV = decltype(tm_tag)::value, TNV = decltype(tn_tag)::value;      // row and column blocks multiplied
        static_assert(!PIPE || (NS >= 3 && SPREAD && KS % 2 == 0), "pipelined k loop: three stages, spread copies, even k-steps");
        constexpr int NMF = TMV * TNV, NRD = TMV > 0 ? TMV + TNV : 0;      // MFMAs and fragment reads per k-step
        bf16x8 a[2][TMV > 0 ? TMV : 1], b[2][TNV];
        auto fetch_one = [&](const unsigned char *cur, int ks, int buf, int r) {      // r-th fragment of a k-step
            // weight fragments first: the MFMAs run over them in the inner loop, so both are needed by the second MFMA
            if (r < TNV) b[buf][r] = *reinterpret_cast<const bf16x8 *>(cur + AB * KS * 1024 + ((cb0 + r) * KS + ks) * 1024 + lane * 16);
            else a[buf][r - TNV] = *reinterpret_cast<const bf16x8 *>(cur + ((rb0 + r - TNV) * KS + ks) * 1024 + lane * 16);
        };
        auto copy_one = [&](int kt, int stg, int j) { copy(j, kt, stg); };
        int stage = 0, in_slice = 0;
        __builtin_amdgcn_s_waitcnt(0xF70 | ((NS - 2) * NLOAD & 15) | (((NS - 2) * NLOAD >> 4) << 14));
        __builtin_amdgcn_s_barrier();          // the first tile is there
        asm volatile("" ::: "memory");
#pragma unroll
        for (int r = 0; r < NRD; ++r) fetch_one(smem, 0, 0, r);
        // Tile whose later copy slices are still to be issued.  Before the first barrier of the loop that is the tile
        // of the one free stage: its slices 1.. are then written twice with the same bytes, which keeps the number of
        // copies per k-step, and with it every s_waitcnt below, the same in all iterations.
        int pend_kt = min(kt_begin + NS - 1, last), pend_stage = NS - 1;
        // One k-tile.  The last one is a separate copy of the code (no barrier, no requests for a next tile), so that the
        // steady-state loop body is straight-line: at a join of the two paths the compiler's s_waitcnt for the last
        // k-step's fragments would also wait for the next tile's fragments requested just before it.
        // Within a k-step the requests for the next k-step are dealt out one per MFMA, in this order and pinned by
        // scheduling barriers: after the workgroup barrier all eight waves would otherwise send their fragment reads at
        // once, the LDS queue fills, and the MFMAs behind them in program order start late; left to itself the
        // scheduler also sinks the reads below the MFMAs to shorten register live ranges and exposes their latency.
        auto tile = [&](int kt, auto last_tag) {
            constexpr bool LAST = decltype(last_tag)::value;
            const unsigned char *cur = smem + stage * STAGE_BYTES;
            const int next_stage = stage == NS - 1 ? 0 : stage + 1;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bool tail = ks == KS - 1;
                if (tail && !LAST) {
                    constexpr int NEWER = NS >= 3 ? (NS - 3) * NLOAD : 0;
                    __builtin_amdgcn_s_waitcnt(0xF70 | (NEWER & 15) | ((NEWER >> 4) << 14));
                    __builtin_amdgcn_s_barrier();      // tile kt+1 visible to all waves; all waves have left tile kt-1
                    asm volatile("" ::: "memory");
                    pend_kt = min(kt + NS - 1, last); pend_stage = stage == 0 ? NS - 1 : stage - 1;
                }
                const unsigned char *fsrc = tail ? smem + next_stage * STAGE_BYTES : cur;
                const int fks = tail ? 0 : ks + 1, fbuf = tail ? 0 : (ks + 1) & 1, slice = tail ? 0 : ks + 1;
                const bool requests = !(tail && LAST);
                if (NMF == 0) {
                    if (requests) issue_slice(pend_kt, pend_stage, slice);
                    continue;
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < TMV; ++i)
#pragma unroll
                    for (int j = 0; j < TNV; ++j) {
                        if (TRANSPOSED)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[ks & 1][j], a[ks & 1][i], acc[i][j], 0, 0, 0);
                        else
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks & 1][i], b[ks & 1][j], acc[i][j], 0, 0, 0);
                        const int slot = i * TNV + j;
                        if (requests) {
                            if (slot < NRD) fetch_one(fsrc, fks, fbuf, slot);
                            if (NRD > NMF && slot == NMF - 1) {
#pragma unroll
                                for (int r = NMF; r < NRD; ++r) fetch_one(fsrc, fks, fbuf, r);
                            }
                            // this slice's copies go with the last MFMAs of the k-step
                            constexpr int PER = (NLOAD + KS - 1) / KS;
#pragma unroll
                            for (int q = 0; q < NLOAD; ++q)
                                if (q % KS == slice && slot == min(max(NMF - PER + q / KS, 0), NMF - 1)) copy_one(pend_kt, pend_stage, q);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
            }
            stage = next_stage;
            if (FOLD && TMV != 0 && ++in_slice == slice_tiles) { fold(); in_slice = 0; }
        };
        for (int kt = kt_begin; kt < kt_end - 1; ++kt) tile(kt, std::false_type{});
        tile(kt_end - 1, std::true_type{});
        if (FOLD && TMV != 0) {
            if (in_slice) fold();
            total();
        }
    };
    if (PIPE) {
        using TNfull = std::integral_constant<int, TN>;
        using TNhalf = std::integral_constant<int, (CAN_COLSPLIT ? 2 : TN)>;
        if (vb == 0) k_loop_pipe(std::integral_constant<int, 0>{}, TNfull{});
        else if (colsplit && vb <= 2) k_loop_pipe(std::integral_constant<int, (TM == 4 ? 2 : TM)>{}, TNhalf{});
        else if (colsplit) k_loop_pipe(std::integral_constant<int, TM>{}, TNhalf{});
        else if (TM == 4 && vb <= 2) k_loop_pipe(std::integral_constant<int, (TM == 4 ? 2 : TM)>{}, TNfull{});
        else k_loop_pipe(std::integral_constant<int, TM>{}, TNfull{});
    } else {
        if (vb == 0) k_loop(std::integral_constant<int, 0>{});
        else if (TM == 4 && vb <= 2) k_loop(std::integral_constant<int, (TM == 4 ? 2 : TM)>{});
        else k_loop(std::integral_constant<int, TM>{});
    }
    __builtin_amdgcn_s_waitcnt(0xF70);     // vmcnt(0): no copy may land in LDS after this workgroup is gone

    const int m0 = tile_m * AB * 32 + rb0 * 32, n0 = tile_n * BB * 32 + cb0 * 32;
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
                if (fbase >= Fp || j >= tnv) continue;      // column blocks of the last tile past the (padded) FFN width; blocks of other waves
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    bf16_t o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float g = acc[i][j][q * 4 + e], u = acc[i][j + 1][q * 4 + e];
                        o[e] = f2bf(g * __builtin_amdgcn_rcpf(1.f + __expf(-g)) * u);
                    }
                    const int f0 = fbase + 8 * q + 4 * lh;
                    *reinterpret_cast<uint2 *>(out + frag_off(row, f0, Fp)) = *reinterpret_cast<uint2 *>(o);
                }
            }
        }
    } else if (EPI == EPI_ROWMAX) {
        // transposed blocks: a lane holds 16 output columns of ONE row per block, in ascending column order, so the
        // first strict maximum it meets is the lowest column of its share; lanes, waves and workgroups then meet in
        // an atomic max over (value, ~column), whose result does not depend on the order of arrival
        unsigned long long *keys = reinterpret_cast<unsigned long long *>(Cv);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = m0 + i * 32 + lr;
            float best = -INFINITY;
            int bi = 0x7FFFFFFF;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int col = n0 + j * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                    const float v = acc[i][j][r] + 0.f;      // -0 -> +0: equal values must give equal keys
                    if (col < N && j < tnv && v > best) { best = v; bi = col; }
                }
            uint32_t u = __float_as_uint(best);
            u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
            unsigned long long key = ((unsigned long long)u << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)bi);
            const unsigned long long other = ((unsigned long long)__shfl_xor((int)(key >> 32), 32) << 32) | (uint32_t)__shfl_xor((int)(key & 0xFFFFFFFFu), 32);
            if (other > key) key = other;
            if (lh == 0 && row < M) atomicMax(keys + row, key);
        }
    } else if (EPI == EPI_ROWSTATS) {
        // Sampling passes need, per row, the softmax statistics at temperature 1/aux_f and the logit of the row's draft
        // token -- not the logits.  Per 32-column block: a lane holds half of a row's block (16 columns, ascending, in its
        // registers): m_h, then with the other half's lane m_b = max(m_0, m_1), z_h = sum of exp((l - m_b) * aux_f) in
        // register order, z_b = z_0 + z_1 (the definition in k_head.hip, which the kernels there share).
        // Cv: float2 [blocks][ldc] (m_b, z_b), followed by float [ldc] draft logits; aux_tok[row]: the draft token (or -1).
        float2 *part = reinterpret_cast<float2 *>(Cv);
        const int nblk = (N + 31) >> 5;
        float *draft_logit = reinterpret_cast<float *>(part + (size_t)nblk * ldc);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = m0 + i * 32 + lr;
            const int dt = row < M ? aux_tok[row] : -1;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int c0 = n0 + j * 32;
                if (j >= tnv || c0 >= N) continue;
                float mh = -INFINITY;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int col = c0 + 8 * (r >> 2) + 4 * lh + (r & 3);
                    if (col < N) mh = fmaxf(mh, acc[i][j][r]);
                    if (col == dt) draft_logit[row] = acc[i][j][r];
                }
                const float mb = fmaxf(mh, __shfl_xor(mh, 32));
                float zh = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int col = c0 + 8 * (r >> 2) + 4 * lh + (r & 3);
                    if (col < N) zh += __expf((acc[i][j][r] - mb) * aux_f);
                }
                const float zo = __shfl_xor(zh, 32);
                if (lh == 0 && row < M) part[(size_t)(c0 >> 5) * ldc + row] = make_float2(mb, zh + zo);
                __builtin_amdgcn_sched_barrier(0);      // one block at a time: interleaved, the blocks' temporaries spill
            }
        }
    } else if (EPI == EPI_ROPE_KV) {
        // The tile is exactly one head of the QKV projection (128 columns = head dim): rotate, round and store what
        // rope_kv_kernel would, from the accumulators.  Transposed blocks: a lane holds ONE row and, per block, four runs
        // of four consecutive head dims, so q and k leave in 8-byte stores and the row's tables are looked up once.  The
        // rotate-half partner of a dim (64 further on or back) sits in the same lane and register of another wave of the
        // same wave row: the finished accumulators change hands through the LDS ring, which is free once every wave has
        // left the k loop.
        static_assert(EPI != EPI_ROPE_KV || (BB == 4 && (TN == 1 || TN == 2) && !CAN_COLSPLIT), "one head per tile");
        static_assert(EPI != EPI_ROPE_KV || (size_t)NT * TM * TN * 16 * 4 <= (size_t)NS * STAGE_BYTES, "exchange area within the ring");
        constexpr int PER_WAVE = TM * TN * 16 * 64;
        float *xch = reinterpret_cast<float *>(smem);
        __syncthreads();      // (every copy has landed: vmcnt(0) above)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) xch[wave * PER_WAVE + ((i * TN + j) * 16 + r) * 64 + lane] = acc[i][j][r];
        __syncthreads();
        const int hh = tile_n;                                                  // head: q heads, then k heads, then v heads
        const int pwave = wm * WGN + (TN == 1 ? (wn ^ 2) : (wn ^ 1));
        const bool rotate = hh < re.Hq + re.Hkv;
        constexpr int D = 128, HALF = 64;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = m0 + i * 32 + lr;
            if (row >= M) continue;
            f16_t *dst = nullptr;       // q row, or the (page, head) block of k or v
            int t = 0;
            if (hh < re.Hq) dst = re.q_h + (size_t)row * re.Hq * D + (size_t)hh * D;
            else {
                const int b = re.row_b[row], pos = re.row_pos[row];
                const int page = re.page_table[(size_t)re.b_slot[b] * re.max_pages + (pos >> 4)];
                t = pos & 15;
                dst = hh < re.Hq + re.Hkv ? re.kpool + ((size_t)page * re.Hkv + (hh - re.Hq)) * (size_t)(DAS_PAGE * D)
                                          : re.vpool + ((size_t)page * re.Hkv + (hh - re.Hq - re.Hkv)) * (size_t)(DAS_PAGE * D);
            }
            const float4 *csrow = reinterpret_cast<const float4 *>(re.cs + (size_t)row * HALF);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int c0 = (wn * TN + j) * 32 + 8 * q + 4 * lh;         // four consecutive head dims c0 .. c0 + 3
                    float y[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) y[e] = acc[i][j][4 * q + e];
                    if (rotate) {
                        const float4 cs01 = csrow[(c0 & (HALF - 1)) >> 1], cs23 = csrow[((c0 & (HALF - 1)) >> 1) + 1];
                        const float2 c[4] = {make_float2(cs01.x, cs01.y), make_float2(cs01.z, cs01.w), make_float2(cs23.x, cs23.y), make_float2(cs23.z, cs23.w)};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float other = xch[pwave * PER_WAVE + ((i * TN + j) * 16 + 4 * q + e) * 64 + lane];
                            y[e] = c0 < HALF ? das_rope_first(y[e], other, c[e]) : das_rope_second(other, y[e], c[e]);
                        }
                    }
                    if (hh < re.Hq) {
                        const f16_t o[4] = {das_f2h(y[0]), das_f2h(y[1]), das_f2h(y[2]), das_f2h(y[3])};
                        *reinterpret_cast<uint2 *>(dst + c0) = *reinterpret_cast<const uint2 *>(o);
                    } else if (hh < re.Hq + re.Hkv) {
                        const f16_t o[4] = {das_kv_elem_counted(y[0], re.sat), das_kv_elem_counted(y[1], re.sat), das_kv_elem_counted(y[2], re.sat), das_kv_elem_counted(y[3], re.sat)};
                        *reinterpret_cast<uint2 *>(dst + kpage_off(t, c0)) = *reinterpret_cast<const uint2 *>(o);      // (dims c0 .. c0 + 3 are contiguous in a K page)
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) dst[vpage_off(t, c0 + e)] = das_kv_elem_counted(y[e], re.sat);
                    }
                }
        }
    } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + j * 32 + lr;
                if (col >= N || j >= tnv) continue;
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

// set by the timing entry point around its own launches only (gemm_debug_copies_only)
static bool g_copies_only = false;
void gemm_debug_copies_only(bool on) { g_copies_only = on; }

template <int WGM, int WGN, int TM, int TN, int NS, int EPI, int KS = 4, bool SPREAD = (NS >= 3), int SL = 0, bool PIPE = false, bool WNT = false>
static void launch_one(const bf16_t *A, const bf16_t *W, void *C, int M, int N, int K, int ldc, hipStream_t st,
                       int slice_tiles = 0, int slices = 1, bool slice_per_xcd = false, const int *aux_tok = nullptr, float aux_f = 0.f,
                       int group = 0, const RopeEpi *rope = nullptr) {
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    constexpr int LDS = NS * (WGM * TM + WGN * TN) * KS * 1024 + WGM * WGN * 1024;      // ring + dump area for padded copies
    static_assert(LDS <= 160 * 1024, "LDS of one CU");
    static bool configured = false;
    auto kern = gemm_kernel<WGM, WGN, TM, TN, NS, EPI, KS, SPREAD, SL, PIPE, WNT>;
    if (!configured) {      // dynamic LDS above the default limit has to be granted once per kernel
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        configured = true;
    }
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const RopeEpi re = rope ? *rope : RopeEpi{};
    if (SL == 2 && slice_per_xcd && slices >= 2 && (8 % slices) == 0) {
        const int grid = ((tiles_m * tiles_n * slices + 7) / 8) * 8;
        kern<<<dim3(grid), dim3(WGM * WGN * 64), LDS, st>>>(A, W, C, M, N, K, ldc, tiles_m, tiles_n, slice_tiles, slices, aux_tok, aux_f, (int)g_copies_only, re);
        return;
    }
    const int grid = ((tiles_m * tiles_n + 7) / 8) * 8;
    // mode 2: one workgroup per slice; mode 3: `slices` groups of `group` slices; mode 1: `group` = slices of the first group (0: one run)
    kern<<<dim3(grid, SL >= 2 ? slices : 1), dim3(WGM * WGN * 64), LDS, st>>>(A, W, C, M, N, K, ldc, tiles_m, tiles_n, slice_tiles, group, aux_tok, aux_f, (int)g_copies_only, re);
}

// Sum of the slice partials in ascending order (in two groups when group > 0: slices [0, group) and [group, slices), each
// in ascending order, then the two sums added), then the epilogue.  ws: [slices][MN] fp32; MN % 4 == 0.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_reduce_kernel(const float4 *__restrict__ ws, int slices, int group, size_t mn4, void *__restrict__ Cv) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= mn4) return;
    const int n1 = group > 0 ? group : slices;
    float4 t = ws[i];
    for (int s2 = 1; s2 < n1; ++s2) {
        const float4 v = ws[(size_t)s2 * mn4 + i];
        t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
    }
    if (n1 < slices) {
        float4 u = ws[(size_t)n1 * mn4 + i];
        for (int s2 = n1 + 1; s2 < slices; ++s2) {
            const float4 v = ws[(size_t)s2 * mn4 + i];
            u.x += v.x; u.y += v.y; u.z += v.z; u.w += v.w;
        }
        t.x += u.x; t.y += u.y; t.z += u.z; t.w += u.w;
    }
    if (EPI == EPI_RESID_F32) {
        float4 *c = reinterpret_cast<float4 *>(Cv) + i;
        float4 o = *c;
        o.x += t.x; o.y += t.y; o.z += t.z; o.w += t.w;
        *c = o;
    } else if (EPI == EPI_F32_ROWMAJOR) {
        reinterpret_cast<float4 *>(Cv)[i] = t;
    } else {
        bf16_t o[4] = {f2bf(t.x), f2bf(t.y), f2bf(t.z), f2bf(t.w)};
        reinterpret_cast<uint2 *>(Cv)[i] = *reinterpret_cast<uint2 *>(o);
    }
}

// EPI_ROWSTATS is built for the wide one-pass shapes: small vocabularies write their logits (they are small)
bool gemm_rowstats_supported(int M, int N) { return M >= 1 && N >= 16384; }

// K slices of a narrow GEMM: a function of K alone (never of M), so that every launch shape sums in the same order
int gemm_slices(int K, int *slice_tiles) {
    const int KT = K / 64;
    const int want = KT >= 256 ? 8 : KT >= 48 ? 4 : KT >= 16 ? 2 : 1;
    *slice_tiles = (KT + want - 1) / want;
    return (KT + *slice_tiles - 1) / *slice_tiles;
}
// ... and how they are added: eight slices as two groups of four (0 = one ascending run)
int gemm_slice_group(int slices) { return slices == 8 ? 4 : 0; }
// Workspace (floats) that lets launch_gemm pick its fastest shape for a narrow output of M x N over K
size_t gemm_ws_floats_needed(int M, int N, int K) {
    int slice_tiles = 0;
    const int slices = gemm_slices(K, &slice_tiles);
    if (slices == 1) return 0;
    const size_t few = (size_t)slices * (size_t)(M < 512 ? M : 512) * N;
    const size_t many = (gemm_slice_group(slices) > 0 && M > 512) ? (size_t)2 * M * N : 0;
    return few > many ? few : many;
}

template <int WGM, int WGN, int TM, int TN, int NS>
static void launch_cfg(int epi, const bf16_t *A, const bf16_t *W, void *C, int M, int N, int K, int ldc, hipStream_t st) {
    switch (epi) {
    case EPI_BF16_ROWMAJOR: launch_one<WGM, WGN, TM, TN, NS, EPI_BF16_ROWMAJOR>(A, W, C, M, N, K, ldc, st); break;
    case EPI_RESID_F32: launch_one<WGM, WGN, TM, TN, NS, EPI_RESID_F32>(A, W, C, M, N, K, ldc, st); break;
    case EPI_SILU_FRAG: launch_one<WGM, WGN, TM, TN, NS, EPI_SILU_FRAG>(A, W, C, M, N, K, ldc, st); break;
    case EPI_ROWMAX: launch_one<WGM, WGN, TM, TN, NS, EPI_ROWMAX>(A, W, C, M, N, K, ldc, st); break;
    default: launch_one<WGM, WGN, TM, TN, NS, EPI_F32_ROWMAJOR>(A, W, C, M, N, K, ldc, st); break;
    }
}

// the epilogues that any wave layout supports
template <int WGM, int WGN, int TM, int TN, int NS>
static void launch_cfg3(int epi, const bf16_t *A, const bf16_t *W, void *C, int M, int N, int K, int ldc, hipStream_t st) {
    switch (epi) {
    case EPI_ROWMAX: launch_one<WGM, WGN, TM, TN, NS, EPI_ROWMAX>(A, W, C, M, N, K, ldc, st); break;
    case EPI_BF16_ROWMAJOR: launch_one<WGM, WGN, TM, TN, NS, EPI_BF16_ROWMAJOR>(A, W, C, M, N, K, ldc, st); break;
    case EPI_RESID_F32: launch_one<WGM, WGN, TM, TN, NS, EPI_RESID_F32>(A, W, C, M, N, K, ldc, st); break;
    default: launch_one<WGM, WGN, TM, TN, NS, EPI_F32_ROWMAJOR>(A, W, C, M, N, K, ldc, st); break;
    }
}

// Compute units of the current device (asked once; 256 if the query fails).
static int cu_count() {
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        (void)hipGetLastError();
        n_cu = cus;
    }
    return n_cu;
}


// Height, in 32-row blocks, of the equal M tiles of a wide GEMM (256-column tiles) with M rows: lo .. 8.  The launch takes
// about (rounds of workgroups) x (time of one tile); a tile of h row blocks takes about (h + 4) units (measured at
// K = 3584: 49, 56, 62, 70, 82, 89 us for h = 3 .. 8), and a last round counts in full unless it is nearly empty (measured
// on 148 column tiles: 296 and 444 workgroups on 256 CUs take the same time).  Ties go to the taller tile.
static int pick_tile_height(int M, int N, int lo) {
    const int mb = (M + 31) / 32, tn = (N + 255) / 256, cus = cu_count();
    int hb = 8;
    double best = 1e30;
    for (int h = 8; h >= lo; --h) {
        const double x = (double)((mb + h - 1) / h) * tn / cus, whole = (double)(long)x, frac = x - whole;
        const double rounds = frac <= 0 ? whole : x <= 2.0 ? whole + 1 : whole + (frac > 0.4 ? 1.0 : 0.6 + frac);
        const double cost = rounds * (h + 4);
        if (cost < best * 0.999) { best = cost; hb = h; }
    }
    return hb;
}

// A must be allocated for M rounded up to 256 rows plus another 256 (tiles of 96, 192 or 288 rows read past a multiple
// of 256), W for N rounded up to 256 rows; K % 64 == 0.
// EPI_ROWMAX needs N >= 16384 (the wide, one-pass shapes) and C = one zeroed 64-bit key per row.
// For EPI_SILU_FRAG, N counts packed (gate+up interleaved) rows and ldc is the padded FFN width.
bool launch_gemm(int epi, const bf16_t *A, const bf16_t *W, void *C, int M, int N, int K, int ldc, hipStream_t st,
                 float *ws, size_t ws_floats, const GemmNormTail *tail, int *left_slices, const int *aux_tok, float aux_f, const RopeEpi *rope) {
    if (left_slices) *left_slices = 1;
    if (M <= 0) return false;
    if (epi == EPI_ROWSTATS) {
        // the LM head of a sampling pass (the caller checks gemm_rowstats_supported): the tiles of the greedy head, with
        // the statistics epilogue.  Up to 256 rows one M tile of all rows per 256 columns, above that M tiles of equal
        // height from the cost model (as for the greedy head and for gate/up below).
        const int hb = M <= 256 ? (M + 31) / 32 : pick_tile_height(M, N, 3);
#define ROWSTATS_TILE(tm, ns) launch_one<1, 4, tm, 2, ns, EPI_ROWSTATS, 2, true, 0, true>(A, W, C, M, N, K, ldc, st, 0, 1, false, aux_tok, aux_f)
        if (hb == 1) ROWSTATS_TILE(1, 8);
        else if (hb == 2) ROWSTATS_TILE(2, 7);
        else if (hb == 3) ROWSTATS_TILE(3, 7);
        else if (hb == 4) ROWSTATS_TILE(4, 6);
        else if (hb == 5) ROWSTATS_TILE(5, 5);
        else if (hb == 6) ROWSTATS_TILE(6, 4);
        else if (hb == 7) ROWSTATS_TILE(7, 4);
        else launch_one<2, 2, 4, 4, 4, EPI_ROWSTATS, 2, true, 0, true>(A, W, C, M, N, K, ldc, st, 0, 1, false, aux_tok, aux_f);
#undef ROWSTATS_TILE
        return false;
    }
    // Tile shapes, picked from measurements on MI355X (every shape keeps the same K order per output element):
    //  * wide outputs (gate/up, LM head): 256x256 -- half the bytes per flop of a 128x128 tile through the HBM->LDS
    //    copy path, which is what saturates first -- on 4 waves of 128x128 with the pipelined k loop at many rows,
    //    on 8 waves (2 x 4) of 128x64 or 12 waves of 96x64 (288x256) otherwise;
    //  * narrow outputs (QKV, O, down; N of a few thousand): 128x128 with 8 waves and a 4-stage ring so that the
    //    one workgroup a CU gets covers the copy latency by itself;
    //  * few rows (T <= 512: weight streaming): 128x64 tiles, 5 stages, twice as many workgroups.
    // The SiLU epilogue pairs a gate block with the up block next to it, so its waves own two column blocks.
    if (M <= 320 && epi == EPI_SILU_FRAG && N >= 16384) {
        // Few rows, wide gate/up (at the ridge between weight streaming and MFMA): 96x128 tiles (64x128 up to 64 rows),
        // k-tiles of 32 in a five-stage ring, two workgroups per CU.  The M tiles of one weight tile run side by side on
        // one XCD, so each weight byte leaves HBM once; per weight byte only 0.75 (0.5) bytes of activations come
        // through the copy path.  Measured 10% faster at T = 272 than one 320x64 tile per weight tile.
        if (M <= 64) launch_one<2, 1, 1, 2, 6, EPI_SILU_FRAG, 2, true>(A, W, C, M, N, K, ldc, st);
        // 193..320 rows: 96x256 tiles on 4 waves of 96x64 (6 MFMAs per 5 fragment reads against 2 per 3), pipelined k loop,
        // seven stages of 22 KiB (six tiles in flight per CU): 121 -> 106 us per layer at T = 272
        else if (M > 192 && M <= 288 && (N % 512) == 0 && ((N / 512) * 3 + 7) / 8 * 8 <= cu_count())
            // 193..288 rows and a width that 96x512 tiles cover in ONE round of workgroups (the 7B gate/up: 3 x 74 = 222
            // tiles on 256 CUs): 4 waves of 96x128, 12 MFMAs per 7 fragment reads, and a third less copied per MFMA than with
            // 96x256 tiles; 105 -> 94 us per layer at T = 272
            launch_one<1, 4, 3, 4, 4, EPI_SILU_FRAG, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
        else if (M > 192) {
            // ... or 128x256 tiles (4 waves of 128x64) where those finish in fewer rounds of workgroups times tile height:
            // 320 rows x 17920 packed columns are 280 tiles of 96 rows (a second round for 24 of them on 256 CUs) but 210
            // tiles of 128 rows.  The K order per output element is the same in both.
            const long nt = (N + 255) / 256, cus = cu_count();
            const long cost96 = ((M + 95) / 96 * nt + cus - 1) / cus * 96, cost128 = ((M + 127) / 128 * nt + cus - 1) / cus * 128;
            if (cost128 < cost96) launch_one<1, 4, 4, 2, 6, EPI_SILU_FRAG, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else launch_one<1, 4, 3, 2, 7, EPI_SILU_FRAG, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
        }
        else launch_one<3, 2, 1, 2, 5, EPI_SILU_FRAG, 2, true>(A, W, C, M, N, K, ldc, st);
        return false;
    }
    if (M > 256 && N >= 16384) {
        // 256-row or 288-row tiles (12 waves, 3 x 4), whichever pads M less: T = 1088 is 4 x 288 - 64 but 5 x 256 - 192
        const int pad256 = (M + 255) / 256 * 256, pad288 = (M + 287) / 288 * 288;
        // LM head at many rows: the same 4-wave pipelined kernel (1.10 -> 1.00 ms at T = 1088 against 288x256 tiles of 12 waves)
        // ... and at 257..512 rows on 4 waves of 128x64 or 96x64 (128x256 or 96x256 tiles), whichever pads M less:
        // 221 -> 186 us for the 1.5B head at 320 rows against 256x256 tiles of 8 waves
        const bool rows96 = (M + 95) / 96 * 96 < (M + 127) / 128 * 128;
        if (epi == EPI_ROWMAX) {
            // M tiles of equal height, as for gate/up at many rows below: e.g. 448 rows are two tiles of 224, not five of 96
            const int hb = pick_tile_height(M, N, 3);
            if (hb == 7) launch_one<1, 4, 7, 2, 4, EPI_ROWMAX, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else if (hb == 6) launch_one<1, 4, 6, 2, 4, EPI_ROWMAX, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else if (hb == 5) launch_one<1, 4, 5, 2, 5, EPI_ROWMAX, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else if (hb == 4) launch_one<1, 4, 4, 2, 6, EPI_ROWMAX, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else if (hb == 3) launch_one<1, 4, 3, 2, 7, EPI_ROWMAX, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else launch_one<2, 2, 4, 4, 4, EPI_ROWMAX, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
        }
        else if (M <= 512 && pad288 >= pad256 && epi == EPI_F32_ROWMAJOR) {
            if (rows96) launch_one<1, 4, 3, 2, 7, EPI_F32_ROWMAJOR, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else launch_one<1, 4, 4, 2, 6, EPI_F32_ROWMAJOR, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
        }
        else if (epi == EPI_F32_ROWMAJOR && M > 512) launch_one<2, 2, 4, 4, 4, EPI_F32_ROWMAJOR, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
        else if (pad288 < pad256 && epi != EPI_SILU_FRAG) launch_cfg3<3, 4, 3, 2, 2>(epi, A, W, C, M, N, K, ldc, st);   // (slower with the SiLU epilogue)
        else if (epi == EPI_SILU_FRAG)
            // gate/up at many rows: 4 waves (2 x 2), one per SIMD, each 128x128 of the 256x256 tile (all 256 accumulator
            // registers of the wave): 8 fragment reads per 16 MFMAs, a third less LDS traffic per MFMA than 8 waves of
            // 128x64.  k-tiles of 32 in a four-stage ring, k loop pipelined across k-tiles, requests dealt out one per
            // MFMA (see k_loop_pipe).  283 -> 251 us per layer at T = 1088 against the 8-wave loop the compiler scheduled.
        {
            // M tiles of EQUAL height (3 .. 8 blocks of 32 rows).  A short last tile (T = 1088 = 4 x 256 + 64) ends early, the workgroups that follow it
            // start out of phase with the others that share their weight tile, and the weight tile is streamed into L2 again
            // for them: with five tiles of 224 rows (4 waves side by side, each 224x64) gate/up at 1088 rows fetches 500 MB
            // instead of 760 MB and takes 240 instead of 250 us, although a 1 x 4 wave layout reads 9 fragments per 14 MFMAs.
            // The height comes from pick_tile_height: e.g. 384 rows run as three tiles of 128 (444 workgroups, 112 us)
            // instead of two of 192 (296 workgroups, 139 us), 448 rows as three of 160 (124 against 151 us), 896 rows as
            // five of 192 (218 against 232 us).
            const int hb = pick_tile_height(M, N, 3);
            if (hb == 7) launch_one<1, 4, 7, 2, 4, EPI_SILU_FRAG, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else if (hb == 6) launch_one<1, 4, 6, 2, 4, EPI_SILU_FRAG, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else if (hb == 5) launch_one<1, 4, 5, 2, 5, EPI_SILU_FRAG, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else if (hb == 4) launch_one<1, 4, 4, 2, 6, EPI_SILU_FRAG, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else if (hb == 3) launch_one<1, 4, 3, 2, 7, EPI_SILU_FRAG, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else launch_one<2, 2, 4, 4, 4, EPI_SILU_FRAG, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
        }
        else launch_cfg<2, 4, 4, 2, 2>(epi, A, W, C, M, N, K, ldc, st);
        return false;
    }
    if (epi == EPI_SILU_FRAG) {
        if (M > 512) launch_one<4, 2, 1, 2, 4, EPI_SILU_FRAG>(A, W, C, M, N, K, ldc, st);
        else launch_one<4, 1, 1, 2, 5, EPI_SILU_FRAG>(A, W, C, M, N, K, ldc, st);
        return false;
    }
    if (N >= 16384) {      // wide output, up to 256 rows (LM head of a small batch): one pass over K like every wide GEMM
        if (epi == EPI_ROWMAX) {
            // 129 .. 256 rows: one M tile of 5 .. 8 row blocks per 256 columns (every weight tile is copied into LDS once)
            // instead of two tiles of 128x64
            const int hb = (M + 31) / 32;
            if (hb == 1) launch_one<1, 4, 1, 2, 8, EPI_ROWMAX, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else if (hb == 2) launch_one<1, 4, 2, 2, 7, EPI_ROWMAX, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else if (hb == 3) launch_one<1, 4, 3, 2, 7, EPI_ROWMAX, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else if (hb == 4) launch_one<1, 4, 4, 2, 6, EPI_ROWMAX, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else if (hb == 5) launch_one<1, 4, 5, 2, 5, EPI_ROWMAX, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else if (hb == 6) launch_one<1, 4, 6, 2, 4, EPI_ROWMAX, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else if (hb == 7) launch_one<1, 4, 7, 2, 4, EPI_ROWMAX, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            else launch_one<2, 2, 4, 4, 4, EPI_ROWMAX, 2, true, 0, true>(A, W, C, M, N, K, ldc, st);
            return false;
        }
        launch_cfg3<2, 2, 2, 1, 5>(epi, A, W, C, M, N, K, ldc, st);
        return false;
    }
    // Narrow outputs: K in slices (see gemm_kernel).  With few rows a 128x128 tile grid leaves most CUs idle and
    // every workgroup walks all of K alone (down projection: 296 k-tiles), so the slices go to separate
    // workgroups, 64-column tiles, two or more workgroups per CU, and a small kernel adds the partials in order.
    int slice_tiles = 0;
    const int slices = gemm_slices(K, &slice_tiles);
    if (slices == 1) {
        if (M > 512) launch_cfg3<2, 4, 2, 1, 4>(epi, A, W, C, M, N, K, ldc, st);
        else launch_cfg3<2, 2, 2, 1, 5>(epi, A, W, C, M, N, K, ldc, st);
        return false;
    }
    const size_t mn = (size_t)M * N;
    const int group = gemm_slice_group(slices);
    const bool halves192 = ((M + 191) / 192) * ((N + 191) / 192) * 2 <= cu_count(), halves256 = ((M + 255) / 256) * ((N + 191) / 192) * 2 <= cu_count();
    if (M > 512 && group > 0 && ws && ldc == N && (N % 4) == 0 && ws_floats >= 2 * mn && (halves192 || halves256)) {
        // Many rows, long K (the down projection): 128x128 tiles over all of K move 32 KiB per k-tile of 64 and the launch
        // runs at the speed of that copy stream.  When they fit the chip in one round, the two slice groups of the sum go to
        // two workgroups instead, each with a tile of 192x192 over half of K: a quarter fewer bytes per multiply through
        // L2 -> LDS for the same number of workgroups; 4 waves (2 x 2) of 3x3 blocks (accumulators and the folded slices
        // fill the register file), pipelined k loop, k-tiles of 32; with more rows a tile of 256x192 on 8 waves (4 x 2) of
        // 2x3 blocks.  The kernel that adds the two halves also adds the residual and applies the RMSNorm that follows.
        if (halves192) launch_one<2, 2, 3, 3, 6, EPI_F32_ROWMAJOR, 2, true, 3, true>(A, W, ws, M, N, K, N, st, 2 * slice_tiles, 2, false, nullptr, 0.f, group);
        else launch_one<4, 2, 2, 3, 5, EPI_F32_ROWMAJOR, 2, true, 3, true>(A, W, ws, M, N, K, N, st, 2 * slice_tiles, 2, false, nullptr, 0.f, group);
        if (epi == EPI_RESID_F32 && tail) {
            launch_reduce_resid_rmsnorm(ws, 2, 0, reinterpret_cast<float *>(C), tail->g, tail->y, M, N, tail->eps, st);
            return true;
        }
        const size_t mn4 = mn / 4;
        const dim3 g((unsigned)((mn4 + 255) / 256));
        const float4 *w4 = reinterpret_cast<const float4 *>(ws);
        if (epi == EPI_RESID_F32) gemm_reduce_kernel<EPI_RESID_F32><<<g, 256, 0, st>>>(w4, 2, 0, mn4, C);
        else if (epi == EPI_BF16_ROWMAJOR) gemm_reduce_kernel<EPI_BF16_ROWMAJOR><<<g, 256, 0, st>>>(w4, 2, 0, mn4, C);
        else gemm_reduce_kernel<EPI_F32_ROWMAJOR><<<g, 256, 0, st>>>(w4, 2, 0, mn4, C);
        return false;
    }
    // few rows: slices over workgroups when the tile grid alone would not fill the chip or K is long
    const bool few_tiles = M <= 64 || ((M + 127) / 128) * ((N + 63) / 64) < 200 || K >= 8192;
    if (M <= 512 && few_tiles && ws && ldc == N && (N % 4) == 0 && ws_floats >= mn * slices) {
        const int MB = (M + 31) / 32;
        if (M <= 64) launch_one<1, 2, 2, 1, 4, EPI_F32_ROWMAJOR, 4, true, 2>(A, W, ws, M, N, K, N, st, slice_tiles, slices);
        else if (K >= 8192 && MB >= 5 && MB <= 10 && ((N + 127) / 128) * slices >= 128) {
            // Long K, 129 .. 320 rows, enough (column tile, slice) pairs to fill the chip (the 7B down projection): ONE
            // workgroup owns all rows of the pass for its 128 columns, so a weight byte is copied into LDS once instead of
            // once per M tile (non-temporal: nobody else reads it), k-tiles of 32 in a five-stage ring; every XCD works on
            // one K slice, whose share of the activation panel stays in its L2.  Measured at 272 rows: 84 -> 65 us
            // (160 rows: 61 -> 48); shorter K or fewer columns leave too few workgroups and are slower this way.
            switch (MB) {
#define ROWS_ALL(mb) case mb: launch_one<1, 4, mb, 1, 5, EPI_F32_ROWMAJOR, 2, true, 2, false, true>(A, W, ws, M, N, K, N, st, 2 * slice_tiles, slices, true); break;
            ROWS_ALL(5) ROWS_ALL(6) ROWS_ALL(7) ROWS_ALL(8) ROWS_ALL(9) ROWS_ALL(10)
#undef ROWS_ALL
            }
        }
        // long K (down projection): 128x128 tiles, k-tiles of 32 in an eight-stage ring (measured 13% faster) -- unless 128x64 tiles
        // still fit one round of workgroups (a narrow output: the 1.5B down projection up to 256 rows, 27.5 -> 22.7 us at 100 rows)
        else if (K >= 8192 && ((M + 127) / 128) * ((N + 63) / 64) * slices > cu_count())
            launch_one<2, 4, 2, 1, 8, EPI_F32_ROWMAJOR, 2, true, 2>(A, W, ws, M, N, K, N, st, 2 * slice_tiles, slices);
        else launch_one<2, 2, 2, 1, 3, EPI_F32_ROWMAJOR, 4, true, 2>(A, W, ws, M, N, K, N, st, slice_tiles, slices);
        const size_t mn4 = mn / 4;
        const dim3 g((unsigned)((mn4 + 255) / 256));
        const float4 *w4 = reinterpret_cast<const float4 *>(ws);
        if (epi == EPI_RESID_F32 && tail) {      // the kernel that adds the partials also normalises the finished rows
            launch_reduce_resid_rmsnorm(ws, slices, group, reinterpret_cast<float *>(C), tail->g, tail->y, M, N, tail->eps, st);
            return true;
        }
        if (epi == EPI_F32_ROWMAJOR && left_slices && group == 0) { *left_slices = slices; return false; }      // the caller's next kernel adds them (one ascending run)
        if (epi == EPI_RESID_F32) gemm_reduce_kernel<EPI_RESID_F32><<<g, 256, 0, st>>>(w4, slices, group, mn4, C);
        else if (epi == EPI_BF16_ROWMAJOR) gemm_reduce_kernel<EPI_BF16_ROWMAJOR><<<g, 256, 0, st>>>(w4, slices, group, mn4, C);
        else gemm_reduce_kernel<EPI_F32_ROWMAJOR><<<g, 256, 0, st>>>(w4, slices, group, mn4, C);
        return false;
    }
    if (M <= 512 && ((M + 127) / 128) * ((N + 63) / 64) <= cu_count()) {      // few rows, enough tiles for one round of them (QKV at a few hundred rows): 128x64 tiles, slices folded in registers
        switch (epi) {
        case EPI_BF16_ROWMAJOR: launch_one<2, 2, 2, 1, 5, EPI_BF16_ROWMAJOR, 4, true, 1>(A, W, C, M, N, K, ldc, st, slice_tiles, slices, false, nullptr, 0.f, group); break;
        case EPI_RESID_F32: launch_one<2, 2, 2, 1, 5, EPI_RESID_F32, 4, true, 1>(A, W, C, M, N, K, ldc, st, slice_tiles, slices, false, nullptr, 0.f, group); break;
        default: launch_one<2, 2, 2, 1, 5, EPI_F32_ROWMAJOR, 4, true, 1>(A, W, C, M, N, K, ldc, st, slice_tiles, slices, false, nullptr, 0.f, group); break;
        }
        return false;
    }
    // Many rows: one workgroup per tile folds the slices in registers.  128x128 tiles (8 waves), or 192x128 (12 waves) when
    // that needs fewer rounds of workgroups times tile height: 1560 rows x 3584 columns are 364 tiles of 128 rows (two
    // rounds on 256 CUs) but 252 tiles of 192 rows (one round).
    const int n_cu = cu_count();
    const int tn = (N + 127) / 128;
    const long cost128 = (long)((((M + 127) / 128) * tn + n_cu - 1) / n_cu) * 128;
    const long cost192 = (long)((((M + 191) / 192) * tn + n_cu - 1) / n_cu) * 192;
    // 256x128 tiles (8 waves of 64x64) when they fit one round and both smaller shapes need two: one tile of 256 rows copies
    // a quarter less than two of 128 (QKV at 1475 rows: 216 tiles instead of 432).  Slices in one ascending run only (the
    // grouped sum of a long K needs the third accumulator set, which this shape has no registers for).
    // QKV of a pass with many rows, head dim 128: every tile of these shapes is one head, so the rotation and the KV write
    // are done from the accumulators (EPI_ROPE_KV) and the fp32 projections never go through memory
    const bool fuse_rope = rope && left_slices && epi == EPI_F32_ROWMAJOR && group == 0 && (N % 128) == 0;
    if (fuse_rope) *left_slices = 0;
    if (group == 0 && ((M + 255) / 256) * tn <= n_cu && cost128 > 128 && cost192 > 192) {
        if (fuse_rope) { launch_one<4, 2, 2, 2, 3, EPI_ROPE_KV, 4, true, 1>(A, W, C, M, N, K, ldc, st, slice_tiles, slices, false, nullptr, 0.f, group, rope); return false; }
        switch (epi) {
        case EPI_BF16_ROWMAJOR: launch_one<4, 2, 2, 2, 3, EPI_BF16_ROWMAJOR, 4, true, 1>(A, W, C, M, N, K, ldc, st, slice_tiles, slices, false, nullptr, 0.f, group); break;
        case EPI_RESID_F32: launch_one<4, 2, 2, 2, 3, EPI_RESID_F32, 4, true, 1>(A, W, C, M, N, K, ldc, st, slice_tiles, slices, false, nullptr, 0.f, group); break;
        default: launch_one<4, 2, 2, 2, 3, EPI_F32_ROWMAJOR, 4, true, 1>(A, W, C, M, N, K, ldc, st, slice_tiles, slices, false, nullptr, 0.f, group); break;
        }
        return false;
    }
    if (cost192 < cost128) {
        if (fuse_rope) { launch_one<3, 4, 2, 1, 3, EPI_ROPE_KV, 4, true, 1>(A, W, C, M, N, K, ldc, st, slice_tiles, slices, false, nullptr, 0.f, group, rope); return false; }
        switch (epi) {
        case EPI_BF16_ROWMAJOR: launch_one<3, 4, 2, 1, 3, EPI_BF16_ROWMAJOR, 4, true, 1>(A, W, C, M, N, K, ldc, st, slice_tiles, slices, false, nullptr, 0.f, group); break;
        case EPI_RESID_F32: launch_one<3, 4, 2, 1, 3, EPI_RESID_F32, 4, true, 1>(A, W, C, M, N, K, ldc, st, slice_tiles, slices, false, nullptr, 0.f, group); break;
        default: launch_one<3, 4, 2, 1, 3, EPI_F32_ROWMAJOR, 4, true, 1>(A, W, C, M, N, K, ldc, st, slice_tiles, slices, false, nullptr, 0.f, group); break;
        }
        return false;
    }
    if (fuse_rope) { launch_one<2, 4, 2, 1, 4, EPI_ROPE_KV, 4, true, 1>(A, W, C, M, N, K, ldc, st, slice_tiles, slices, false, nullptr, 0.f, group, rope); return false; }
    switch (epi) {
    case EPI_BF16_ROWMAJOR: launch_one<2, 4, 2, 1, 4, EPI_BF16_ROWMAJOR, 4, true, 1>(A, W, C, M, N, K, ldc, st, slice_tiles, slices, false, nullptr, 0.f, group); break;
    case EPI_RESID_F32: launch_one<2, 4, 2, 1, 4, EPI_RESID_F32, 4, true, 1>(A, W, C, M, N, K, ldc, st, slice_tiles, slices, false, nullptr, 0.f, group); break;
    default: launch_one<2, 4, 2, 1, 4, EPI_F32_ROWMAJOR, 4, true, 1>(A, W, C, M, N, K, ldc, st, slice_tiles, slices, false, nullptr, 0.f, group); break;
    }
    return false;
}
