// Ragged causal GQA attention over the paged KV cache (split-KV).  The cache holds bf16-rounded values in
// binary16 containers (see rope_kv_kernel): the MFMAs here are the f16 ones, whose 11-bit operands let the rotated
// query and the probabilities go in as ONE term each (as bf16 each needed a hi + lo pair to keep the scores and the
// weighted sum at fp32-like accuracy, which doubled the matrix work).
//
// One workgroup = one (sequence, KV head, chunk of pm.chunk tokens: 2048, or 1024 for models with two KV heads).
// All G*(1+k_i) query rows that share the KV head are served by ONE pass over the chunk's KV: arithmetic per KV
// byte is G*(1+k) <= 231 flop/B, below the machine's ridge, so the kernel is built around streaming pages at HBM rate:
//   * pages are stored in MFMA operand order, so a 32-token tile (2 pages of K and of V) is four contiguous runs
//     copied to LDS with coalesced 16-byte loads (asynchronous, non-temporal, a ring of four tiles that never
//     drains) and read back lane-linearly (no bank conflicts);
//   * S^T = K Q^T with v_mfma_f32_16x16x32_f16 puts 8 tokens of one query row in each lane, so the row max needs
//     two cross-lane steps and the probabilities are already laid out as the B operand of O^T += V^T P^T;
//   * chunks start at absolute multiples of the chunk length and each chunk is reduced from scratch, then chunks
//     are merged in ascending order: a row's result does not depend on the batch it is verified in (speculative
//     verification and one-token decoding give bit-identical rows).
// Wave w (of 8, or of 16) owns query-row blocks (16 rows each) w*RBW .. w*RBW+RBW-1.
#include "das_internal.h"
#include <cstdlib>

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// two floats -> packed fp16 pair (round to nearest even), and back
__device__ __forceinline__ uint32_t pack_h2(float a, float b) {
    typedef __attribute__((ext_vector_type(2))) _Float16 h2;
    h2 v = {(_Float16)a, (_Float16)b};
    return *reinterpret_cast<uint32_t *>(&v);
}
__device__ __forceinline__ float2 unpack_h2(uint32_t u) {
    typedef __attribute__((ext_vector_type(2))) _Float16 h2;
    h2 v = *reinterpret_cast<h2 *>(&u);
    return make_float2((float)v[0], (float)v[1]);
}

// 16-byte-per-lane asynchronous copy HBM -> LDS (no VGPR staging): lane l's 16 bytes land at
// lds_wave_base + 16*l.  Inline assembly, so that the copies are ordered only by the explicit
// s_waitcnt/s_barrier of the tile loop (M0 carries the LDS address; 1 wait state before its use).  The KV stream is
// read once per launch: the non-temporal hint keeps it from pushing the split-KV partials, which are written here and
// read back by the merge kernel, out of the caches (measured: attention -10 %, merge -20 %).
__device__ __forceinline__ void dma16(const void *g, uint32_t lds_wave_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" ::"v"(g), "s"(lds_wave_base) : "memory", "m0");
}

// Two waves per SIMD are asked for whenever the row blocks fit 256 registers: besides the occupancy, it
// makes the compiler keep the MFMA accumulators in ordinary VGPRs, where the (rare) rescale can reach them
// without copies out of the accumulation register file on every tile.
// DBG != 0 exists only in development builds (see launch_attn): 1 copies only, 6 arithmetic only (no copies after
// the first two tiles), 7 copies only and no partial stores, 8 copies and LDS fragment reads without arithmetic, 9 everything
// but with the partial results stored to a small region that stays in the caches.
template <int D, int RBW, int NS, int MINW, int NW, int DBG = 0>
__global__ __launch_bounds__(NW * 64, MINW) void attn_partial_kernel(PassMeta pm, const int *__restrict__ items,
                                                           const f16_t *__restrict__ q_h,
                                                           const f16_t *__restrict__ kpool,
                                                           const f16_t *__restrict__ vpool,
                                                           uint16_t *__restrict__ part_o, float *__restrict__ part_ml,
                                                           bf16_t *__restrict__ out,
                                                           int Hkv, int G, int qstride, float scale_log2e) {
    constexpr int KFR = D / 32;            // K fragments (1 KiB) per page
    constexpr int VDB = D / 16;            // V dim blocks (512 B) per page
    constexpr int PAGE_E = DAS_PAGE * D;   // elements of one (page, head) block
    constexpr int PAGE_B = PAGE_E * 2;
    constexpr int TILE_B = 4 * PAGE_B;     // K page0, K page1, V page0, V page1
    constexpr int UNITS_PER_SEG = PAGE_B / 16;
    constexpr int NT = NW * 64;
    constexpr int NLOAD = (TILE_B / 16) / NT;
    static_assert((TILE_B / 16) % NT == 0, "tile must divide over the threads");
    // ring of NS tile stages: one being read, NS-1 being filled
    extern __shared__ __align__(16) unsigned char smem[];      // NS * TILE_B bytes
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;

    // work items arrive sorted longest first: sequence, chunk | KV head << 20
    const int b = items[2 * blockIdx.x], chunk = items[2 * blockIdx.x + 1] & 0xFFFFF;
    const int kvh = items[2 * blockIdx.x + 1] >> 20;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ctx = pm.b_start[b], n = pm.b_n[b], row0 = pm.b_row0[b];
    const int R = G * n;
    const int tok_begin = chunk * pm.chunk;
    const int tok_total = ctx + n;
    const int tok_end = min(tok_begin + pm.chunk, tok_total);
    const int ntiles = (tok_end - tok_begin + DAS_ATTN_TILE - 1) / DAS_ATTN_TILE;
    const int npages = (tok_total + DAS_PAGE - 1) / DAS_PAGE;
    const int *pt = pm.page_table + (size_t)pm.b_slot[b] * pm.max_pages;
    // the chunk's (at most 64) page ids, one per lane, fetched once: the tile loop then takes them with
    // v_readlane and never waits on a vector load of its own (which would also wait for every copy in flight)
    const int first_page = tok_begin >> 4;
    constexpr int NPREG = DAS_ATTN_CHUNK_MAX / DAS_PAGE / 64;      // registers of 64 page ids each
    int my_page[NPREG];
#pragma unroll
    for (int q = 0; q < NPREG; ++q) my_page[q] = pt[min(first_page + q * 64 + lane, npages - 1)];

    // ---- query fragments (B operand: lane l = query row l%16, dims 8*(l/16)..+7 of each 32-dim step)
    f16x8 qf[RBW][KFR];
    int lim[RBW];           // last KV position this lane's query row may see (-1: padding row)
    bool any_active = false;
#pragma unroll
    for (int i = 0; i < RBW; ++i) {
        const int rr = (wave * RBW + i) * 16 + (lane & 15);
        const bool valid = rr < R;
        const int j = valid ? rr / G : 0, g = valid ? rr % G : 0;
        lim[i] = valid ? ctx + j : -1;
        any_active |= ((wave * RBW + i) * 16 < R);
        const size_t qo = (size_t)(row0 + j) * qstride + (size_t)(kvh * G + g) * D + 8 * (lane >> 4);
#pragma unroll
        for (int ks = 0; ks < KFR; ++ks) {
            uint4 v = valid ? *reinterpret_cast<const uint4 *>(q_h + qo + ks * 32) : make_uint4(0, 0, 0, 0);
            qf[i][ks] = *reinterpret_cast<f16x8 *>(&v);
        }
    }

    float m_run[RBW], l_run[RBW];
    f32x4 acc[RBW][VDB];
#pragma unroll
    for (int i = 0; i < RBW; ++i) {
        m_run[i] = -INFINITY; l_run[i] = 0.f;
#pragma unroll
        for (int db = 0; db < VDB; ++db) acc[i][db] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }

    // ---- tile loader: 16-byte unit u of the tile belongs to segment u / UNITS_PER_SEG
    auto issue = [&](int ti, int stage) {
        // pages 2*ti and 2*ti+1 of the chunk (the second one was clamped to the last page at load)
        static_assert(NPREG <= 2, "at most two registers of 64 page ids per chunk");
        const int li = (2 * ti) & 63;
        int pg0 = __builtin_amdgcn_readlane(my_page[0], li), pg1 = __builtin_amdgcn_readlane(my_page[0], li + 1);
        if (NPREG == 2) {
            const int qg0 = __builtin_amdgcn_readlane(my_page[NPREG - 1], li), qg1 = __builtin_amdgcn_readlane(my_page[NPREG - 1], li + 1);
            if (2 * ti >= 64) { pg0 = qg0; pg1 = qg1; }
        }
#pragma unroll
        for (int jn = 0; jn < NLOAD; ++jn) {
            const int u = tid + jn * NT;
            const int seg = u / UNITS_PER_SEG, off = u % UNITS_PER_SEG;
            const int pg = (seg & 1) ? pg1 : pg0;
            const f16_t *base = (seg < 2 ? kpool : vpool) + ((size_t)pg * Hkv + kvh) * PAGE_E;
            dma16(reinterpret_cast<const uint4 *>(base) + off, lds_base + stage * TILE_B + jn * NT * 16 + wave * 1024);
        }
    };

    // ---- the three phases of a tile, kept apart so that two tiles can be interleaved below
    struct Scores { f32x4 v[RBW][2]; };
    struct Probs { f16x8 v[RBW]; };

    // S^T = K Q^T : s[i][pg][r] = score of token 16*pg + 4*(lane/16) + r for query row lane%16
    auto qk = [&](const unsigned char *cur, Scores &s) {
#pragma unroll
        for (int i = 0; i < RBW; ++i) { s.v[i][0] = (f32x4){0.f, 0.f, 0.f, 0.f}; s.v[i][1] = (f32x4){0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
        for (int ks = 0; ks < KFR; ++ks) {
            const f16x8 k0 = *reinterpret_cast<const f16x8 *>(cur + (ks * 64 + lane) * 16);
            const f16x8 k1 = *reinterpret_cast<const f16x8 *>(cur + PAGE_B + (ks * 64 + lane) * 16);
            if (DBG == 8) { asm volatile("" ::"v"(k0), "v"(k1)); continue; }      // fragment reads without arithmetic
#pragma unroll
            for (int i = 0; i < RBW; ++i) {
                s.v[i][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(k0, qf[i][ks], s.v[i][0], 0, 0, 0);
                s.v[i][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(k1, qf[i][ks], s.v[i][1], 0, 0, 0);
            }
        }
    };

    // Softmax with a lazily updated reference: p = exp2(s * scale - m_ref).  m_ref only moves when the row's
    // maximum in this tile exceeds it by more than 8 (a factor 256), which after a row's first tile almost never
    // happens: the common path needs no cross-lane step and no rescaling of the accumulators.  The decision is
    // taken per ROW (from the row's own maximum), so a row's arithmetic never depends on its neighbours;
    // softmax is shift-invariant, the result is exact.
    // row_check: causal mask (only the chunk's last tiles need one), row maximum, and the rare move of m_ref.
    auto row_check = [&](int ti, Scores &s) {
        const int tile_tok0 = tok_begin + ti * DAS_ATTN_TILE;
        const bool need_mask = tile_tok0 + DAS_ATTN_TILE - 1 > ctx;
#pragma unroll
        for (int i = 0; i < RBW; ++i) {
            if (need_mask) {
                const int pbase = tile_tok0 + 4 * (lane >> 4);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (pbase + r > lim[i]) s.v[i][0][r] = -INFINITY;
                    if (pbase + 16 + r > lim[i]) s.v[i][1][r] = -INFINITY;
                }
            }
            float mt = fmaxf(s.v[i][0][0], s.v[i][1][0]);
#pragma unroll
            for (int r = 1; r < 4; ++r) mt = fmaxf(mt, fmaxf(s.v[i][0][r], s.v[i][1][r]));
            mt *= scale_log2e;
            if (__any(mt > m_run[i] + 8.f)) {          // some row of this block may have to move its reference
                mt = fmaxf(mt, __shfl_xor(mt, 16));
                mt = fmaxf(mt, __shfl_xor(mt, 32));    // the row's maximum, same in its four lanes
                const float mn = (mt > m_run[i] + 8.f) ? mt : m_run[i];
                const float alpha = exp2f(m_run[i] - ((mn == -INFINITY) ? 0.f : mn));   // 1 for rows that stay
                const bool had_sum = m_run[i] != -INFINITY && alpha != 1.f;            // a first tile has nothing to rescale
                l_run[i] *= alpha;
                m_run[i] = mn;
                if (__any(had_sum)) {                  // rare: a reference moving after the row's first tile
#pragma unroll
                    for (int db = 0; db < VDB; ++db) acc[i][db] *= alpha;
                }
            }
        }
    };
    // probabilities of a checked tile, rounded to binary16 (at most 256 by the rule above; what falls below the
    // format's 6e-8 is lost against a row sum of at least 1), and the row sums of the unrounded values
    auto probs = [&](const Scores &s, Probs &p) {
#pragma unroll
        for (int i = 0; i < RBW; ++i) {
            const float ms = (m_run[i] == -INFINITY) ? 0.f : m_run[i];
            float ps = 0.f;
            float pv[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                pv[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s.v[i][r >> 2][r & 3], scale_log2e, -ms));
                ps += pv[r];
            }
            l_run[i] += ps;
            typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
            const u32x4 hv = {pack_h2(pv[0], pv[1]), pack_h2(pv[2], pv[3]), pack_h2(pv[4], pv[5]), pack_h2(pv[6], pv[7])};
            p.v[i] = *reinterpret_cast<const f16x8 *>(&hv);
        }
    };

    // O^T += V^T P^T : A = V fragment (dims x 32 token slots), B = probabilities
    auto pv = [&](const unsigned char *cur, const Probs &p) {
#pragma unroll
        for (int db = 0; db < VDB; ++db) {
            // the two halves of a fragment (tokens of the first and of the second page) are read by separate
            // 8-byte loads straight into its registers; left to itself the compiler pairs the loads of
            // neighbouring dim blocks instead and pays for it with register moves
            typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
            typedef const volatile __attribute__((address_space(3))) u32x2 *lds_u32x2_ptr;
            const u32x2 lo = *(lds_u32x2_ptr)(cur + 2 * PAGE_B + (db * 64 + lane) * 8);
            const u32x2 hi = *(lds_u32x2_ptr)(cur + 3 * PAGE_B + (db * 64 + lane) * 8);
            typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
            u32x4 vv = {lo[0], lo[1], hi[0], hi[1]};
            const f16x8 vf = *reinterpret_cast<f16x8 *>(&vv);
            if (DBG == 8) { asm volatile("" ::"v"(vf)); continue; }
#pragma unroll
            for (int i = 0; i < RBW; ++i) acc[i][db] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vf, p.v[i], acc[i][db], 0, 0, 0);
        }
    };

    // (Matrix and vector instructions of one SIMD do not overlap on this chip -- measured: their times add even with
    // four waves per SIMD -- so nothing is gained by interleaving the score MFMAs of one tile with the exponentials of
    // another; what counts is the instruction count per tile.)
    const bool work = any_active && DBG != 1 && DBG != 7;
    {
        // One tile per barrier, ring of NS stages: tile ti in use, tiles ti+1 .. ti+NS-1 in flight.  Copies are issued
        // unconditionally (past the end: the last tile again, into a stage nobody reads any more), so "tile ti has
        // landed" is the same s_waitcnt in every iteration and the copy queue never drains at a barrier.
        const int last = ntiles - 1;
#pragma unroll
        for (int s0 = 0; s0 < NS - 1; ++s0) issue(min(s0, last), s0);
        int stage = 0;
        for (int ti = 0; ti < ntiles; ++ti) {
            constexpr int NEWER = (NS - 2) * NLOAD;
            __builtin_amdgcn_s_waitcnt(0xF70 | (NEWER & 15) | ((NEWER >> 4) << 14));
            __builtin_amdgcn_s_barrier();      // tile ti visible to all waves; all waves are done with tile ti-1
            asm volatile("" ::: "memory");
            if (DBG != 6) issue(min(ti + NS - 1, last), stage == 0 ? NS - 1 : stage - 1);
            if (work) {
                const unsigned char *c0 = smem + stage * TILE_B;
                Scores s0;
                Probs p0;
                qk(c0, s0);
                if (DBG != 8) {
                    row_check(ti, s0);
                    probs(s0, p0);
                }
                pv(c0, p0);
            }
            stage = stage == NS - 1 ? 0 : stage + 1;
        }
    }
    __builtin_amdgcn_s_waitcnt(0xF70);     // vmcnt(0): no copy may land in LDS after this workgroup is gone

    // ---- partial results per 16-row block: (m, l) per row in fp32 and the chunk's normalised output acc / l in
    // fp16 (values bounded by the largest |v|; 11 significant bits, well below the bf16 rounding of the merged
    // result), in the lane order the accumulators are held in: dim blocks 2q and 2q+1 share one 16-byte store, a
    // contiguous KiB per instruction.  HBM writes cost this kernel about three times their bytes in read
    // bandwidth, hence the narrow format.
    const int nrb = (R + 15) >> 4;
    // Partials of a long sequence (many chunks) leave with non-temporal stores: they are many, the merge reads each once,
    // and kept in the caches they cost the KV stream more than the merge gains (contexts of 32k-64k: attention -20 us,
    // merge +7 us per layer); the few partials of short sequences stay cached for the merge.
    const int nchunk_b = pm.b_nchunk[b];
    const bool stream_out = nchunk_b >= 8;
    // A sequence of one chunk needs no merge: its rows are finished here with the arithmetic attn_merge_kernel would
    // apply to that one chunk ((o * l) * (1 / l) on the binary16-rounded o, then bf16), so a row comes out the same
    // whether its sequence had one chunk or more (later chunks that the row cannot see are skipped by the merge).
    const bool single = nchunk_b == 1;
#pragma unroll
    for (int i = 0; i < RBW; ++i) {
        float l = l_run[i];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        const int rb = wave * RBW + i;
        if (rb < nrb && DBG != 7) {
            const size_t id = DBG == 9 ? ((size_t)blockIdx.x & 63) * 64 + rb * Hkv + kvh : ((size_t)pm.b_prow[b] + (size_t)chunk * nrb + rb) * Hkv + kvh;
            const float inv = l > 0.f ? 1.f / l : 0.f;
            if (single) {
                const int rr = rb * 16 + (lane & 15);
                if (rr < R) {
                    const int t = pm.b_row0[b] + rr / G, a = kvh * G + rr % G;
                    const float invden = 1.f / l;
                    auto fin = [&](float x, float y) -> uint32_t {      // two neighbouring dims -> two bf16
                        const float2 o = unpack_h2(pack_h2(x, y));
                        uint32_t u0 = __float_as_uint((o.x * l) * invden), u1 = __float_as_uint((o.y * l) * invden);
                        u0 += 0x7FFFu + ((u0 >> 16) & 1u);
                        u1 += 0x7FFFu + ((u1 >> 16) & 1u);
                        return (u0 >> 16) | (u1 & 0xFFFF0000u);
                    };
#pragma unroll
                    for (int db = 0; db < VDB; ++db) {
                        const f32x4 o = acc[i][db] * inv;
                        *reinterpret_cast<uint2 *>(out + frag_off(t, a * D + 16 * db + 4 * (lane >> 4), qstride)) =
                            make_uint2(fin(o[0], o[1]), fin(o[2], o[3]));
                    }
                }
                continue;
            }
            if ((lane >> 4) == 0) *reinterpret_cast<float2 *>(part_ml + id * 32 + 2 * lane) = make_float2(m_run[i], l);
            uint4 *dst = reinterpret_cast<uint4 *>(part_o + id * (16 * D)) + lane;
#pragma unroll
            for (int q = 0; q < VDB / 2; ++q) {
                const f32x4 lo = acc[i][2 * q] * inv, hi = acc[i][2 * q + 1] * inv;
                typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
                const u32x4 val = {pack_h2(lo[0], lo[1]), pack_h2(lo[2], lo[3]), pack_h2(hi[0], hi[1]), pack_h2(hi[2], hi[3])};
                // (inline assembly: written with the builtin, the two branches are merged into one plain store.  The wait
                // states cover the hazard between a 16-byte store and a later write of its data registers, which the
                // compiler handles for its own stores only.  No load may follow these stores in this kernel: the compiler's
                // s_waitcnt bookkeeping does not count them.)
                if (stream_out) asm volatile("global_store_dwordx4 %0, %1, off nt\n\ts_nop 4" ::"v"(dst + q * 64), "v"(val) : "memory");
                else *reinterpret_cast<u32x4 *>(dst + q * 64) = val;
            }
        }
    }
}

// ring depth: four 16 KiB stages per workgroup (one tile in use, three in flight), two workgroups per CU.  Five stages
// (2 x 80 KiB = all of the CU's LDS) leave room for one workgroup only and are slower (320 against 299 us per layer
// on contexts of 32k-64k tokens).
#define DAS_ATTN_STAGES 4
template <int D, int RBW, int DBG, int NW = 8>
static void launch_attn_cfg(const PassMeta &pm, const int *items, int n_items, const f16_t *q_h, const f16_t *kpool_layer,
                            const f16_t *vpool_layer, uint16_t *part_o, float *part_ml, bf16_t *out_frag, const DasDims &dm, float sc, hipStream_t st) {
    // 8 waves per workgroup: the 8 (or 16) query-row blocks of a KV head are spread one (two) per wave, two
    // workgroups per CU, so that MFMA, exp and LDS work of different waves overlap
    auto kern = attn_partial_kernel<D, RBW, DAS_ATTN_STAGES, (RBW == 1 ? 4 : 2), NW, DBG>;
    constexpr int LDS = DAS_ATTN_STAGES * 4 * DAS_PAGE * D * 2;
    static bool configured = false;
    if (!configured) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        configured = true;
    }
    kern<<<dim3(n_items), dim3(NW * 64), LDS, st>>>(pm, items, q_h, kpool_layer, vpool_layer, part_o, part_ml, out_frag, dm.Hkv, dm.G, dm.Hq * dm.D, sc);
}

void launch_attn(const PassMeta &pm, const int *items, int n_items, int rbw, const f16_t *q_h,
                 const f16_t *kpool_layer, const f16_t *vpool_layer, uint16_t *part_o, float *part_ml, bf16_t *out_frag,
                 const DasDims &dm, hipStream_t st) {
    if (n_items <= 0) return;
    const float sc = 1.4426950408889634f / sqrtf((float)dm.D);
#define ATTN_ARGS pm, items, n_items, q_h, kpool_layer, vpool_layer, part_o, part_ml, out_frag, dm, sc, st
#ifdef DAS_ATTN_DEV
    // Development build only (-DDAS_ATTN_DEV): variants that leave parts of the kernel out, to time copies and
    // arithmetic separately.  Their results are wrong by design.  Selected by the DAS_ATTN_DBG environment variable.
    const int dbg = getenv("DAS_ATTN_DBG") ? atoi(getenv("DAS_ATTN_DBG")) : 0;
    if (dbg && dm.D == 128) {
        switch (dbg * 10 + (rbw <= 2 ? 1 : 2)) {
        case 11: launch_attn_cfg<128, 1, 1>(ATTN_ARGS); return; case 12: launch_attn_cfg<128, 2, 1>(ATTN_ARGS); return;
        case 61: launch_attn_cfg<128, 1, 6>(ATTN_ARGS); return; case 62: launch_attn_cfg<128, 2, 6>(ATTN_ARGS); return;
        case 71: launch_attn_cfg<128, 1, 7>(ATTN_ARGS); return; case 72: launch_attn_cfg<128, 2, 7>(ATTN_ARGS); return;
        case 81: launch_attn_cfg<128, 1, 8>(ATTN_ARGS); return; case 82: launch_attn_cfg<128, 2, 8>(ATTN_ARGS); return;
        case 91: launch_attn_cfg<128, 1, 9>(ATTN_ARGS); return; case 92: launch_attn_cfg<128, 2, 9>(ATTN_ARGS); return;
        }
    }
#endif
    // rbw is the class of the launch: 2 = up to 8 row blocks per KV head, 4 = up to 16
    if (dm.D == 128) {
        // up to 16 row blocks at head dim 128: 16 waves with one block each (one workgroup per CU, the register and
        // arithmetic budget of two 8-wave workgroups) rather than 8 waves with two blocks each
        if (rbw <= 2) launch_attn_cfg<128, 1, 0>(ATTN_ARGS); else launch_attn_cfg<128, 1, 0, 16>(ATTN_ARGS);
    } else {
        if (rbw <= 2) launch_attn_cfg<64, 1, 0>(ATTN_ARGS); else launch_attn_cfg<64, 2, 0>(ATTN_ARGS);
    }
#undef ATTN_ARGS
}

// ---------------------------------------------------------------- merge of the chunk partials
// One workgroup per (sequence, 16-row block, KV head), one wave per pair of dim blocks: lane l holds row l%16 and dims
// 16*db + 4*(l/16) .. +3 of its two dim blocks, as the attention kernel left them.  A chunk contributes its
// normalised output with weight l * 2^(m - M); ascending chunk order, fp32; chunks a row cannot see carry
// m = -inf and are skipped.  Output: bf16, fragment order, K = Hq*D.
template <int D>
__global__ __launch_bounds__(64 * (D / 32)) void attn_merge_kernel(PassMeta pm, const uint16_t *__restrict__ part_o,
                                                        const float *__restrict__ part_ml, bf16_t *__restrict__ out,
                                                        int Hq, int Hkv, int G) {
    const int b = pm.mblk[2 * blockIdx.x], rb = pm.mblk[2 * blockIdx.x + 1];
    const int kvh = blockIdx.y, q = threadIdx.y, lane = threadIdx.x;     // this wave: dim blocks 2q and 2q+1
    const int n = pm.b_n[b];
    const int R = G * n, nrb = (R + 15) >> 4, nchunk = pm.b_nchunk[b];
    const int rr = rb * 16 + (lane & 15);
    float M = -INFINITY, den = 0.f;
    float num[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) num[e] = 0.f;
    const size_t id0 = ((size_t)pm.b_prow[b] + rb) * Hkv + kvh, idstep = (size_t)nrb * Hkv;
    auto load = [&](int c, float2 &ml, uint4 &v) {
        const size_t id = id0 + (size_t)c * idstep;
        ml = *reinterpret_cast<const float2 *>(part_ml + id * 32 + 2 * (lane & 15));
        v = (reinterpret_cast<const uint4 *>(part_o + id * (16 * D)) + q * 64)[lane];
    };
    // Four chunks in flight: the merge of a long sequence is one dependent chain of loads, and its partials come from
    // HBM (they were written past the caches), so the depth of this ring is what its duration follows.
    constexpr int PF = 4;
    float2 ml_q[PF];
    uint4 v_q[PF];
#pragma unroll
    for (int u = 0; u < PF; ++u)
        if (u < nchunk) load(u, ml_q[u], v_q[u]);
    for (int c0 = 0; c0 < nchunk; c0 += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int c = c0 + u;
            if (c >= nchunk) break;
            const float2 ml = ml_q[u];
            const uint4 v = v_q[u];
            if (c + PF < nchunk) load(c + PF, ml_q[u], v_q[u]);
            if (ml.x == -INFINITY) continue;
            const float mn = fmaxf(M, ml.x);
            const float a0 = exp2f(M - mn), a1 = ml.y * exp2f(ml.x - mn);
            den = den * a0 + a1;
            const float2 o0 = unpack_h2(v.x), o1 = unpack_h2(v.y), o2 = unpack_h2(v.z), o3 = unpack_h2(v.w);
            const float o[8] = {o0.x, o0.y, o1.x, o1.y, o2.x, o2.y, o3.x, o3.y};
#pragma unroll
            for (int e = 0; e < 8; ++e) num[e] = num[e] * a0 + o[e] * a1;
            M = mn;
        }
    }
    if (rr >= R) return;
    const int j = rr / G, g = rr % G;
    const int t = pm.b_row0[b] + j, a = kvh * G + g;
    const float inv = 1.f / den;
    const int K = Hq * D;
    auto rne = [](float f) -> uint32_t {
        uint32_t u = __float_as_uint(f);
        u += 0x7FFFu + ((u >> 16) & 1u);
        return u >> 16;
    };
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        // four consecutive dims: they share one 8-element group of the fragment layout
        const uint32_t lo = rne(num[4 * h] * inv) | (rne(num[4 * h + 1] * inv) << 16);
        const uint32_t hi = rne(num[4 * h + 2] * inv) | (rne(num[4 * h + 3] * inv) << 16);
        *reinterpret_cast<uint2 *>(out + frag_off(t, a * D + 16 * (2 * q + h) + 4 * (lane >> 4), K)) = make_uint2(lo, hi);
    }
}

void launch_attn_merge(const PassMeta &pm, const uint16_t *part_o, const float *part_ml, bf16_t *out_frag,
                       const DasDims &dm, hipStream_t st) {
    if (pm.n_mblk <= 0) return;
    dim3 g(pm.n_mblk, dm.Hkv), blk(64, dm.D / 32);      // one wave per pair of dim blocks
    if (dm.D == 128) attn_merge_kernel<128><<<g, blk, 0, st>>>(pm, part_o, part_ml, out_frag, dm.Hq, dm.Hkv, dm.G);
    else attn_merge_kernel<64><<<g, blk, 0, st>>>(pm, part_o, part_ml, out_frag, dm.Hq, dm.Hkv, dm.G);
}
