// Internal declarations shared by the host orchestration and the HIP kernels.
//
// Data layout in HBM (gfx950, wave64, MFMA):
//  * GEMM operands, weights AND activations, are stored in "MFMA fragment
//    order" for v_mfma_f32_32x32x16_bf16: a matrix X[R][K] (K contiguous in the
//    logical view) is cut into fragments of 32 rows x 16 k; fragment
//    (rb, ks) is 1 KiB = 64 lanes x 8 bf16, lane l holding row rb*32 + l%32,
//    k = ks*16 + 8*(l/32) .. +7.  Fragments of one row block are contiguous
//    in ks.  A wave fetches an operand with one fully coalesced 16-byte load
//    per lane and no shuffling; tiles copy to LDS linearly and are read back
//    with conflict-free ds_read_b128.
//  * The KV cache is paged (16 tokens); one layer is [page][H_kv][16*D] (measured faster than head-major:
//    the four heads' workgroups of a chunk then stream one contiguous region together).  A K page of one KV head is stored as
//    the A operand of v_mfma_f32_16x16x32_bf16 (16 tokens x 32 dims per
//    fragment, D/32 fragments); a V page as [D/16 dim blocks][4 token
//    groups][16 dims][4 tokens] so that a lane's 8-byte load from each of two
//    pages forms the A operand of the P*V product over a 32-token tile.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint16_t bf16_t;   // raw bf16 bit pattern in memory
typedef uint16_t f16_t;    // raw IEEE binary16 bit pattern in memory (KV pages, rotated queries)

#define DAS_PAGE 16
#define DAS_ATTN_CHUNK_MAX 2048      // most tokens per split-KV work item (absolute-position aligned); a model uses this or half
// Tokens per split-KV work item of a model: a function of the model's shape alone (never of a batch), so that a row's
// reduction order is the same in every pass.  Long chunks halve the partial results to write and merge; with two KV
// heads a batch has too few (sequence, head, chunk) items to fill the chip at 2048.
static inline int das_attn_chunk(int n_kv_heads) { return n_kv_heads <= 2 ? DAS_ATTN_CHUNK_MAX / 2 : DAS_ATTN_CHUNK_MAX; }
#define DAS_ATTN_TILE 32             // tokens per inner tile = 2 pages

enum DasKernelClass {
    KC_META = 0, KC_EMBED, KC_RMSNORM, KC_GEMM_QKV, KC_ROPE_KV, KC_ATTN, KC_ATTN_MERGE, KC_GEMM_O,
    KC_GEMM_GATEUP, KC_GEMM_DOWN, KC_GEMM_LMHEAD, KC_ARGMAX, KC_ACCEPT, KC_SAMPLE, KC_KVIO, KC_COUNT
};

// element offset of X[row][k] inside a fragment-ordered matrix with K columns (K % 16 == 0)
__host__ __device__ inline size_t frag_off(int row, int k, int K) {
    return ((size_t)(row >> 5) * (size_t)(K >> 4) + (size_t)(k >> 4)) * 512
         + (size_t)((((k >> 3) & 1) << 5) + (row & 31)) * 8 + (size_t)(k & 7);
}

// element offset of (token t in page, dim d) inside one (page, head) K block of head dim D
__host__ __device__ inline int kpage_off(int t, int d) {
    return (((d >> 5) * 64) + (((d & 31) >> 3) * 16 + t)) * 8 + (d & 7);
}
// element offset of (token t in page, dim d) inside one (page, head) V block
__host__ __device__ inline int vpage_off(int t, int d) {
    return ((((d >> 4) * 4 + (t >> 2)) * 16) + (d & 15)) * 4 + (t & 3);
}

struct DasDims {
    int L, d, Hq, Hkv, D, F, V, G;
    int Fp;        // d_ffn padded to a multiple of 64 (zero weights)
    int qkvN;      // (Hq + 2 Hkv) * D
    float rope_theta, rms_eps;
};

// Per-pass metadata, all device pointers into one staging block.
struct PassMeta {
    int T;                 // rows in this pass
    int NB;                // sequences (blocks) in this pass
    const int *tok;        // [T]
    const int *row_pos;    // [T] absolute position
    const int *row_b;      // [T] block index
    const int *b_slot;     // [NB] page-table row
    const int *b_start;    // [NB] first position of the block (= committed length)
    const int *b_n;        // [NB] rows of the block
    const int *b_row0;     // [NB] first row of the block
    const int *b_prow;     // [NB] base 16-row block in the split-KV partial buffers
    const int *b_nchunk;   // [NB] split-KV chunks
    const int *mblk;       // [n_mblk][2] (block, 16-row block) pairs: one merge workgroup each per KV head
    int n_mblk;
    const int *sel;        // [n_sel] rows that get logits
    int n_sel;
    const int *page_table; // [max_seqs][max_pages]
    int max_pages;
    int num_pages;         // pages in the pool
    int chunk;             // tokens per split-KV chunk (das_attn_chunk of the model)
};

// EPI_ROWMAX: no matrix is written; every row's (largest value, lowest column holding it) is folded into a 64-bit key per
// row with atomic max (value in the high word as an order-preserving integer, ~column in the low word)
// EPI_ROWSTATS: no matrix is written either; per row and 32-column block the softmax statistics (block maximum, sum of
// exp((l - max) / T)) and, per row, the logit of one given column (the row's draft token): what a sampling pass needs
// EPI_ROPE_KV: no matrix is written; the QKV projection's rows are rotated, rounded and stored as rope_kv_kernel would
// (q to the binary16 query buffer, k and v into their pages), from the accumulators.  Tiles of exactly one head (128 columns).
enum GemmEpilogue { EPI_BF16_ROWMAJOR = 0, EPI_RESID_F32 = 1, EPI_SILU_FRAG = 2, EPI_F32_ROWMAJOR = 3, EPI_ROWMAX = 4, EPI_ROWSTATS = 5, EPI_ROPE_KV = 6 };

// What the rotation + KV-write step needs besides the projections: the pass's row tables, the angles, the outputs.
struct RopeEpi {
    const int *row_b, *row_pos, *b_slot, *page_table;
    int max_pages;
    const float2 *cs;              // [T][D/2] (cos, sin)
    f16_t *q_h, *kpool, *vpool;    // rotated queries [T][Hq*D]; this layer's K and V pages
    int Hq, Hkv;
    unsigned long long *sat;       // count of K/V elements that did not fit their container
};

#ifdef __HIPCC__
// ---- arithmetic shared by rope_kv_kernel and the GEMM epilogue that replaces it at many rows: one definition, so that a
// row has the same bits whichever of the two wrote it.
__device__ __forceinline__ float das_bf16_round(float f) {      // fp32 -> nearest-even bf16 -> fp32
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return __uint_as_float(u & 0xFFFF0000u);
}
// binary16 bit pattern of x, round to nearest even, saturating at the largest finite value
__device__ __forceinline__ f16_t das_f2h(float x) {
    const _Float16 h = (_Float16)fminf(fmaxf(x, -65504.f), 65504.f);
    return __builtin_bit_cast(f16_t, h);
}
// a K or V element: rounded to bf16 exactly once (the cache precision), then kept in a binary16 container; counted in
// *sat when the bf16 value does not fit the container (NaN counts too)
__device__ __forceinline__ f16_t das_kv_elem_counted(float x, unsigned long long *sat) {
    const float b = das_bf16_round(x);
    if (!(fabsf(b) <= 65504.f)) atomicAdd(sat, 1ull);
    return das_f2h(b);
}
// rotate-half pair (x1 at dim i, x2 at dim i + D/2) by the angle (c.x, c.y) = (cos, sin): one multiply and one fused
// multiply-add each, written out so that every caller compiles to the same two instructions
__device__ __forceinline__ float das_rope_first(float x1, float x2, float2 c) { return __builtin_fmaf(x1, c.x, -(x2 * c.y)); }
__device__ __forceinline__ float das_rope_second(float x1, float x2, float2 c) { return __builtin_fmaf(x2, c.x, x1 * c.y); }
#endif

// ---- launchers (each enqueues on `st`; none synchronises) ----
void launch_pack_weight(const bf16_t *src, bf16_t *dst, int N, int K, int Np, int Kp, hipStream_t st);
void launch_pack_gateup(const bf16_t *wg, const bf16_t *wu, bf16_t *dst, int F, int K, int Fp, hipStream_t st);
void launch_pt_update(int *page_table, const int *upd, int n_upd, hipStream_t st);
void launch_embed(const PassMeta &pm, const bf16_t *E, float *h, int d, hipStream_t st);
// y (fragment order, K = d) = rmsnorm(h[row]) for row = sel ? sel[i] : i, i < n
void launch_rmsnorm(const float *h, const bf16_t *g, bf16_t *y, const int *sel, int n, int d, float eps, hipStream_t st);
void launch_reduce_resid_rmsnorm(const float *ws, int slices, int group, float *h, const bf16_t *g, bf16_t *y, int n, int d, float eps, hipStream_t st);
// RMSNorm that follows a residual GEMM (EPI_RESID_F32): when the GEMM's K slices are summed by a second kernel anyway, that
// kernel also normalises the finished rows (gain g, output y in fragment order) and launch_gemm returns true; otherwise the
// caller runs launch_rmsnorm itself.  Same bits either way.
struct GemmNormTail { const bf16_t *g; bf16_t *y; float eps; };
void launch_rope_table(const PassMeta &pm, const double *inv_freq, float *cs, int D, hipStream_t st);
// qkv: fp32 [T][qkvN] projections; q is rotated and rounded to binary16 ([T][Hq*D]); k is rotated, rounded once to
// bf16 and scattered into its page; v is rounded once to bf16 and scattered.  The pages keep those bf16 values in
// binary16 containers (exact for 2^-17 <= |x| <= 65504; larger magnitudes saturate).
// slices > 1: qkv points at `slices` slabs of [T][qkvN] partial sums (see launch_gemm's left_slices); the kernel adds them
// in ascending order first, which gives the bits the GEMM's own reduce kernel would have written.
// sat: device counter of K/V elements that did not fit the container (never cleared)
void launch_rope_kv(const PassMeta &pm, const float *qkv, int slices, f16_t *q_h, const float *cs,
                    f16_t *kpool_layer, f16_t *vpool_layer, const DasDims &dm, unsigned long long *sat, hipStream_t st);
// C[M][N] = A[M][K] * W[N][K]^T, A and W in fragment order
// ws: fp32 workspace of ws_floats elements for the slice partials of narrow few-row GEMMs (may be null: slower, same result)
// left_slices (EPI_F32_ROWMAJOR only): a caller whose next kernel can add the K-slice partials itself passes a pointer.
// When the launch leaves the partials in ws ([slices][M][N], to be added in ascending order) it stores their count there
// and C stays unwritten; otherwise it stores 1 and C holds the product.
// rope (EPI_F32_ROWMAJOR with left_slices only, head dim 128): when the launch shape allows it the rotation + KV write is
// done from the accumulators (EPI_ROPE_KV); the launch then stores 0 in *left_slices and C stays unwritten.
// EPI_ROWSTATS (only where gemm_rowstats_supported): C = float2 [ceil(N/32)][ldc] block statistics followed by float [ldc]
// draft logits; aux_tok[row] = the column whose logit is wanted (-1: none), aux_f = 1 / temperature.
bool launch_gemm(int epi, const bf16_t *A, const bf16_t *W, void *C, int M, int N, int K, int ldc, hipStream_t st,
                 float *ws, size_t ws_floats, const GemmNormTail *tail = nullptr, int *left_slices = nullptr,
                 const int *aux_tok = nullptr, float aux_f = 0.f, const RopeEpi *rope = nullptr);
bool gemm_rowstats_supported(int M, int N);
// copy-ring probe (k_probe.hip): stages x (4 * copies) KiB ring, 4 waves; the built shapes are listed there
bool copy_ring_supported(int stages, int copies, int shared_copies);
hipError_t launch_copy_ring(const void *priv, const void *shared_r, int workgroups, int stages, int copies, int shared_copies,
                            int tiles, bool non_temporal, hipStream_t st);
// matrix-pipe probe (k_probe.hip): mode 0 register operands, 1 operands from LDS, 2 with the GEMM's copy traffic
hipError_t launch_mfma_loop(int mode, const void *src, float *sink, int iters, long long *clk, hipStream_t st);
void gemm_debug_copies_only(bool on);      // timing mode of das_debug_gemm_time: launches copy their tiles and multiply nothing
int gemm_slices(int K, int *slice_tiles);
int gemm_slice_group(int slices);                       // eight slices are added as two groups of four (0: one ascending run)
size_t gemm_ws_floats_needed(int M, int N, int K);     // workspace that lets launch_gemm pick its fastest shape
// split-KV partial attention for the items of one row-block class, then the merge.  Sequences of one chunk are finished
// by launch_attn itself (their rows go straight to out_frag, bit-equal to what the merge would write), so pm.mblk lists
// only the row blocks of sequences with two or more chunks.
void launch_attn(const PassMeta &pm, const int *items, int n_items, int rbw, const f16_t *q_h,
                 const f16_t *kpool_layer, const f16_t *vpool_layer, uint16_t *part_o, float *part_ml, bf16_t *out_frag,
                 const DasDims &dm, hipStream_t st);
void launch_attn_merge(const PassMeta &pm, const uint16_t *part_o, const float *part_ml, bf16_t *out_frag,
                       const DasDims &dm, hipStream_t st);
void launch_argmax(const float *logits, int n_rows, int V, int *out, hipStream_t st);
void launch_rowmax_keys_clear(unsigned long long *keys, int n_rows, hipStream_t st);
void launch_rowmax_keys_decode(const unsigned long long *keys, int n_rows, int *out, hipStream_t st);
void launch_accept_greedy(const int *g, const int *b_row0, const int *b_n, const int *tok, int NB,
                          int *accept_len, int *next_token, hipStream_t st);
// Stochastic acceptance on per-block softmax statistics (see k_head.hip): part = float2 [ceil(V/32)][ldp], from the LM-head
// GEMM (EPI_ROWSTATS) or from written logits (launch_block_stats); stats = float2 [rows] (M, Z).
void launch_block_stats(const float *logits, int n_rows, int V, float inv_temp, const int *dtok, float2 *part, int ldp,
                        float *draft_logit, hipStream_t st);
void launch_row_stats_merge(const float2 *part, int ldp, int V, int n_rows, float inv_temp, float2 *stats, hipStream_t st);
void launch_sample(const float2 *part, int ldp, int V, const float2 *stats, const float *draft_logit, const bf16_t *xsel,
                   const bf16_t *wlm, int K, const int *tok, const int *b_row0, const int *b_n, int NB, float inv_temp,
                   const float *u_accept, const float *u_sample, int prefill_mode, int *accept_len, int *next_token, hipStream_t st);
// k_lin / v_lin: bf16, linear [n_pos][Hkv][D]; mode 0 imports into the pages, mode 1 exports
void launch_kv_io(int mode, const int *page_row, int first_pos, int n_pos, f16_t *kpool_layer, f16_t *vpool_layer,
                  bf16_t *k_lin, bf16_t *v_lin, int Hkv, int D, int num_pages, unsigned long long *sat, hipStream_t st);
void launch_kv_synth(const int *page_row, int ctx, f16_t *kpool_layer, f16_t *vpool_layer, int Hkv, int D, int num_pages,
                     uint64_t seed, uint64_t seq_key, int layer, hipStream_t st);
void launch_copy(const void *src, void *dst, size_t bytes, hipStream_t st);
// dst[i] = bf16(sigma * z_i), z_i standard normal from the counter-based generator keyed by (seed, tensor_id, i); dst[i] = v
void launch_fill_normal(bf16_t *dst, size_t n, uint64_t seed, uint64_t tensor_id, double sigma, hipStream_t st);
void launch_fill_const(bf16_t *dst, size_t n, bf16_t v, hipStream_t st);
