/*
 * das.h -- C ABI of the MI355X (gfx950) batched speculative-verification library.
 *
 * The calls follow the paper's statement of one rollout round (Sec. 3; Fig. 3
 * right; Sec. 4.1.2): a drafter proposes a multi-token chain per sequence, the
 * target model verifies all of them in parallel in one batched pass, and the
 * accepted tokens advance generation -- with the guarantee (abstract, Sec. 5.1,
 * Sec. 6) that the emitted tokens are those that decoding without speculation
 * would have produced (greedy: token-identical; sampling: same distribution,
 * via the speculative-sampling rejection rule the paper cites in Sec. 2).
 *
 * Conventions
 *  - Every pointer argument is HOST memory owned by the caller unless a comment
 *    says otherwise; the library copies what it needs before returning and has
 *    written every output and synchronised its stream when a call returns.
 *  - Every call returns DAS_OK (0) or a negative DAS_ERR_* code.  All argument
 *    and state validation happens before any state change or kernel launch: a
 *    failed call leaves KV contents, page tables and sequence state untouched.
 *    No exception or abort crosses this boundary.
 *  - A sequence is (ctx_len committed KV positions, one pending token whose KV
 *    is not yet written).  das_verify_step scores the rows
 *    [pending, draft_1 .. draft_k] at positions ctx_len .. ctx_len+k and leaves
 *    the sequence SPECULATIVE; exactly one of das_kv_commit / das_kv_rollback
 *    must follow before the next verify step.
 *  - KV lives in pages of 16 tokens, values rounded to bf16, 2 bytes per element
 *    (see das_kv_import for the container).  Page ids are handed out from a
 *    stack whose first pop is page 0, in batch order then ascending position;
 *    pages are returned in batch order, highest page position first.
 *  - The library is not thread-safe per model: calls on one das_model must not
 *    overlap.
 */
#ifndef DAS_H
#define DAS_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DAS_OK            0
#define DAS_ERR_INVALID  (-1)   /* bad argument (null, out of range, duplicate id, over a configured maximum) */
#define DAS_ERR_STATE    (-2)   /* call not allowed in the sequence's state, or ctx_len mismatch */
#define DAS_ERR_NOMEM    (-3)   /* out of KV pages, sequence slots, or device/host memory */
#define DAS_ERR_DEVICE   (-4)   /* a HIP call failed; das_last_device_error() has the text */

typedef struct das_model das_model;   /* opaque: device weights, KV pool, page tables, sequence table, stream */

typedef struct {
    int32_t n_layers, d_model /* multiple of 64, <= 8192 */, n_q_heads, n_kv_heads, head_dim /* 64 or 128 */, d_ffn, vocab;
    float   rope_theta, rms_eps;
    int32_t page_size;      /* must be 16 */
    int32_t max_seqs;       /* sequence slots */
    int32_t max_ctx;        /* most positions one sequence may hold, drafts included */
    int32_t max_rows;       /* most rows (sum of 1+k_i) in one verify step; also the prefill pass size */
    int32_t max_draft;      /* largest k_i; (1+max_draft) * n_q_heads/n_kv_heads must be <= 256 */
    int64_t num_pages;      /* KV pool size in pages */
} das_config;

/* Sampling inputs for stochastic rollouts.  One uniform in [0,1) per ROW of the
 * step (row-aligned with [pending, drafts..] of every sequence, batch order):
 * u_accept[row j] decides draft j+1, u_sample[row j] draws the token emitted
 * after row j.  NULL das_sampling* means greedy decoding. */
typedef struct {
    float temperature;          /* > 0 */
    const float *u_accept;
    const float *u_sample;
} das_sampling;

/* The target model whose outputs the rollout must preserve (abstract; Sec. 5.1 names the 1.5B-8B decoder families).
 * Weights come either from the caller or from the library's own random initialisation:
 *  - `weights_bf16` != NULL: the canonical blob, every matrix [out_features][in_features] row-major, bf16 bit
 *    patterns:  embed[V][d]; per layer g1[d] Wq[Hq*D][d] Wk[Hkv*D][d] Wv[Hkv*D][d] Wo[d][Hq*D] g2[d] Wg[F][d]
 *    Wu[F][d] Wd[d][F]; then gf[d] Wlm[V][d].  `seed` is ignored.
 *  - `weights_bf16` == NULL: every matrix ~ N(0, 0.02^2), gains 1.0, generated ON THE DEVICE from `seed` by a
 *    counter-based generator: element i of tensor t (t counts the tensors of the blob above in order) is
 *    bf16(0.02 * sqrt(-2 ln u1) cos(2 pi u2)) with (u1, u2) the two 32-bit halves of
 *    mix(mix(mix(seed ^ 0x5745494748545321) ^ t) ^ i), u1 = (hi + 1) / 2^32, u2 = lo / 2^32, mix = splitmix64 step,
 *    arithmetic in fp64.  No host blob is needed (15 GB for the 7B shape).
 * The library repacks the matrices on the device.  `hip_stream` is a hipStream_t the library should run on, or NULL
 * to create its own.  Allocates all device memory here (weights, KV pool of num_pages, workspaces sized from
 * max_rows / max_seqs / max_ctx): no later call on the verification path allocates.  Cheap to call again: an RL
 * loop reloads the policy's weights every iteration (Sec. 1: the target model keeps changing during training). */
int das_model_load(const das_config *cfg, uint64_t seed, const uint16_t *weights_bf16, void *hip_stream, das_model **out);
int das_model_free(das_model *m);

/* Prefill: the prompt of a rollout request enters the KV cache before the first speculative round (Fig. 3: the
 * rollout phase starts from the prompts of the batch).  n NEW sequences (ids must be unused).  tokens =
 * concatenated prompts, lens[i] >= 1.  Writes KV for every prompt position and returns the first pending token
 * of each sequence (greedy argmax, lowest index on ties; or, with sampling, an inverse-CDF draw from
 * softmax(logits/T) using u_sample[i], one value per SEQUENCE; u_accept unused).  Sequences end COMMITTED with
 * ctx_len = lens[i].  The prompt runs through the same kernels as a verification pass, in blocks of rows that
 * attend causally to what is already written. */
int das_prefill(das_model *m, int32_t n, const int32_t *seq_ids, const int32_t *tokens, const int32_t *lens,
                const das_sampling *sampling, int32_t *next_token);

/* One batched verification pass (Sec. 3; Fig. 3 right).  seq_ids unique,
 * COMMITTED; ctx_lens[i] is checked against the library's committed length
 * (DAS_ERR_STATE on mismatch); draft_tokens = concatenated chains, draft_lens[i]
 * = k_i in [0, max_draft].
 * Greedy: g_j = argmax of row j's logits; accept_len = longest prefix with
 * draft_j == g_{j-1}; next_token = g_{accept_len}.
 * Sampling: for j = 0..k-1 accept draft_{j+1} iff u_accept[j]*Z_j < w_j(draft_{j+1})
 * with w = exp(logit/T - max), Z = sum w; on the first rejection next_token is
 * the inverse-CDF draw (ascending vocabulary order, u_sample[j]) from w with
 * the rejected token's weight zeroed; if all accepted, a draw from row k.
 * Leaves every sequence SPECULATIVE.  Nothing is committed. */
int das_verify_step(das_model *m, int32_t n, const int32_t *seq_ids, const int32_t *ctx_lens,
                    const int32_t *draft_tokens, const int32_t *draft_lens,
                    const das_sampling *sampling, int32_t *accept_len, int32_t *next_token);

/* Accepted tokens advance generation (Fig. 3 right): ctx_len += 1 + accept_lens[i]
 * (0 <= accept_lens[i] <= k_i of the pending step), pending = next_tokens[i],
 * pages past the new length are returned.  The caller normally passes the
 * step's own outputs; a parity harness may pass another decision (the KV rows
 * of the drafts depend only on the input tokens). */
int das_kv_commit(das_model *m, int32_t n, const int32_t *seq_ids, const int32_t *accept_lens,
                  const int32_t *next_tokens);
/* The other outcome of a round (Fig. 3 right: only accepted tokens advance generation): discard every row of the
 * pending step; ctx_len and the pending token are unchanged, the pages taken for the step are returned. */
int das_kv_rollback(das_model *m, int32_t n, const int32_t *seq_ids);
/* Truncate COMMITTED sequences to an earlier committed length new_lens[i] <= ctx_len (KV beyond it is
 * discarded, pages returned) and set their pending tokens: replaying a rollout from a checkpoint. */
int das_seq_rewind(das_model *m, int32_t n, const int32_t *seq_ids, const int32_t *new_lens,
                   const int32_t *pending_tokens);
/* A finished rollout leaves the batch (Sec. 3, Fig. 1: the effective batch shrinks as short responses end):
 * release sequences (any state) and their pages. */
int das_seq_free(das_model *m, int32_t n, const int32_t *seq_ids);

/* ---- state injection: contexts whose KV is an input rather than a prefill ---- */
/* New COMMITTED sequence of ctx_len positions (KV contents unspecified until imported) and a pending token. */
int das_seq_create(das_model *m, int32_t seq_id, int32_t ctx_len, int32_t pending_token);
/* Copy K and V rows [first_pos, first_pos+n_pos) of one layer; k, v are bf16 [n_pos][n_kv_heads][head_dim] in host
 * memory.  The pages keep bf16-rounded values in 16-bit IEEE binary16 containers: every bf16 value with
 * 2^-17 <= |x| <= 65280 (and zero) survives an import/export round trip bit for bit; larger magnitudes saturate at
 * the binary16 maximum 65504, smaller ones move to the nearest multiple of 2^-24 (at most 3e-8 away). */
int das_kv_import(das_model *m, int32_t seq_id, int32_t layer, int32_t first_pos, int32_t n_pos,
                  const uint16_t *k, const uint16_t *v);
int das_kv_export(das_model *m, int32_t seq_id, int32_t layer, int32_t first_pos, int32_t n_pos,
                  uint16_t *k, uint16_t *v);
/* Fill positions [0, ctx_len) of every layer on the device with the keyed synthetic
 * generator: element e of the [pos][kv_head][dim] tensor of (layer, which in {K=0,V=1}) is
 * bf16(s * 2^-15), s = centred sum of the four 16-bit fields of
 * mix(mix(mix(mix(seed ^ 0x4B5653594E544821) ^ seq_key) ^ (2*layer+which)) ^ e), mix = splitmix64 step. */
int das_kv_synth(das_model *m, int32_t seq_id, uint64_t seed, uint64_t seq_key);

/* ---- inspection (tests, parity harness, bench) ---- */
/* Row count of the last forward pass that produced logits. */
int das_debug_num_rows(das_model *m, int32_t *n_rows);
/* Greedy passes do not write their logits to memory by default (vocab >= 16384): the LM-head GEMM gathers each
 * row's argmax itself.  on != 0 makes every later pass write them, for das_debug_logits.  Passes with sampling
 * always write them. */
int das_debug_keep_logits(das_model *m, int32_t on);
/* fp32 logits of rows [first_row, first_row+n_rows) of the last pass; out[n_rows][vocab].
 * DAS_ERR_STATE if the last pass did not write them (see das_debug_keep_logits). */
int das_debug_logits(das_model *m, int32_t first_row, int32_t n_rows, float *out);
/* Greedy token of every row of the last pass; out[n_rows_of_pass].  DAS_ERR_STATE after a sampling pass unless
 * das_debug_keep_logits is on (sampling does not need the argmax). */
int das_debug_row_argmax(das_model *m, int32_t *out);
/* Sequence state: committed length, pending token, state (0 COMMITTED, 1 SPECULATIVE), page list.
 * pages may be NULL; *n_pages receives the count (pages must hold that many when non-NULL). */
int das_debug_seq(das_model *m, int32_t seq_id, int32_t *ctx_len, int32_t *pending, int32_t *state,
                  int32_t *pages, int32_t *n_pages);
int das_debug_free_pages(das_model *m, int64_t *n_free);
/* KV pages keep bf16-rounded values in binary16 containers (see das_kv_import): a K or V element whose bf16 value
 * exceeds 65504 in magnitude is stored as +-65504.  Every such store (by a verification / prefill pass or by
 * das_kv_import) is counted in a per-model counter that is never cleared; *count receives it.  Zero means that
 * the cache holds exactly the bf16 values that were computed. */
int das_debug_kv_saturated(das_model *m, int64_t *count);
/* Stand-alone run of the MFMA GEMM kernel the projections use: c[M][N] (fp32) = a[M][K] * w[N][K]^T,
 * a and w row-major bf16, K a multiple of 8.  Needs no model. */
int das_debug_gemm(int32_t M, int32_t N, int32_t K, const uint16_t *a, const uint16_t *w, float *c);
/* das_debug_gemm for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  c_dev[M][N] (fp32) = a_dev[M][K] * w_dev[N][K]^T with a_dev, w_dev row-major bf16 and
 * c_dev all DEVICE pointers owned by the caller (valid on the current device).  Calls no hipMalloc / hipFree and no
 * allocating library routine: the repacked operands and the K-slice partial sums live in a 14 MiB array that the library
 * keeps on every GPU it runs on until the process ends.  Limits: M <= 256, N <= 2048, K <= 2048 (K a multiple of 8);
 * anything larger is DAS_ERR_INVALID with a message in das_last_device_error().  The kernels are enqueued on
 * `hip_stream` (NULL: the default stream) and the call returns WITHOUT synchronising: c_dev is complete when the
 * stream reaches this point.  All calls on one GPU share that GPU's array: calls that overlap on one GPU (different
 * streams, different threads) race; calls on one stream are ordered.  Same kernels, same bits as das_debug_gemm. */
int das_gemm_noalloc(int32_t M, int32_t N, int32_t K, const uint16_t *a_dev, const uint16_t *w_dev, float *c_dev,
                     void *hip_stream);
/* The same kernel with its other two epilogues, on row-major bf16 host inputs a[M][K] (K a multiple of 64):
 * act[M][F] (host, fp32 values of the bf16 the kernel stores) = silu(a wg^T) * (a wu^T) with wg, wu [F][K], F a
 * multiple of 8 -- the gate/up projection (Sec. 3 names the model families; SwiGLU FFN);
 * col[M] (host) = lowest column holding the row maximum of a w^T, w [N][K], N >= 16384 -- the LM head of a greedy
 * pass, which writes no logits.  Pass F = 0 or N = 0 (and NULLs) to skip one of them.  Needs no model. */
int das_debug_gemm_epilogues(int32_t M, int32_t K, const uint16_t *a, int32_t F, const uint16_t *wg, const uint16_t *wu,
                             float *act, int32_t N, const uint16_t *w, int32_t *col);

/* Device time of the projection GEMM of one launch shape, as a verification pass launches it: epi 1 = residual add
 * (O, down: includes the kernel that adds the K-slice partials and applies the RMSNorm that follows), 2 = gate/up
 * with SiLU (N counts gate and up rows together), 3 = fp32 out (QKV), 4 = row maximum (LM head of a greedy pass).
 * Operands are random bf16 (N(0,1) activations, N(0,0.02^2) weights) generated on the device; `weight_sets`
 * distinct weight matrices are used in turn so that a launch does not find its weights in a cache left by the
 * previous one (a decoder touches each layer's weights once per pass).  *us_per_launch = mean over `iters`
 * launches after two warm-up launches.  copies_only != 0 times the same launches with their arithmetic switched
 * off: every workgroup moves the same tiles into LDS behind the same barriers and multiplies nothing (results are
 * meaningless), which shows how much of a shape's time is its copy stream.  Needs no model; not for use while
 * another thread launches verification passes (the switch is process-wide for the duration of the call). */
int das_debug_gemm_time(int32_t epi, int32_t M, int32_t N, int32_t K, int32_t iters, int32_t weight_sets,
                        int32_t copies_only, double *us_per_launch);

/* The HBM/L2 -> LDS copy ring that feeds the GEMM and attention kernels, run by itself over synthetic buffers: a
 * measurement of what the ring delivers, against which the kernels' copy streams are read.  `workgroups` workgroups of
 * 4 waves (one per compute unit: the launch reserves more than half of a CU's LDS) each pull `tiles` tiles through a
 * ring of `stages` stages; a tile is 4 * `copies` KiB, every wave issuing `copies` 1-KiB copies per tile, the first
 * `shared_copies` of them from a 64-tile region that all workgroups read (L2 hits), the others from the workgroup's
 * own stream (every line once: L2 misses; with the non-temporal hint if `non_temporal`).  Built (stages, copies,
 * shared_copies): (4,4,0) (9,4,0) (4,9,0) (4,4,4) (9,4,4) (4,9,9) (4,9,6) (4,9,3) (5,7,5) (3,7,5), anything else is
 * DAS_ERR_INVALID; tiles <= 4096, workgroups <= 1024.  *us = time of one launch (best of three after a
 * warm-up; every launch reads private bytes no earlier launch touched), *bytes_into_lds = bytes one launch copies.
 * Allocates and frees its buffers; needs no model. */
int das_debug_copy_ring(int32_t workgroups, int32_t stages, int32_t copies, int32_t shared_copies, int32_t tiles,
                        int32_t non_temporal, double *us, double *bytes_into_lds);

/* The matrix pipe by itself: 256 workgroups of 4 waves (one wave per SIMD, one workgroup per compute unit) each run
 * `iters` iterations of two k-steps of 16 independent v_mfma_f32_32x32x16_bf16, the inner loop of the 256x256-tile GEMM.
 * mode 0: operands constant, in registers; 1: every k-step's eight operand fragments read from LDS (pseudo-random bf16
 * bit patterns), requested one k-step ahead; 2: as 1 plus that GEMM's copy traffic (8 KiB per wave and k-tile from an
 * L2-resident region into a four-stage LDS ring, s_waitcnt + s_barrier per k-tile).  *ns_per_mfma = loop time of one
 * wave / its MFMAs (constant 100 MHz counter), *shader_ghz = shader-clock cycles of that loop / its time (the clock the
 * loop ran at: the chip lowers it under matrix load), *pflops = the launch's bf16 rate over its HIP-event duration.
 * This is the ceiling the GEMM kernels' MFMA fractions are read against.  Allocates and frees its buffers; needs no
 * model; iters <= 100000, anything else is DAS_ERR_INVALID. */
int das_debug_mfma_loop(int32_t mode, int32_t iters, double *ns_per_mfma, double *shader_ghz, double *pflops);

/* Device-to-device copy of `bytes` (multiple of 16) by a trivial kernel, `repeats` times: a dispatch of
 * known HBM traffic (bytes read + bytes written) against which profiler byte counters are scaled. */
int das_debug_copy(int64_t bytes, int32_t repeats);

/* ---- per-kernel timing with HIP events on the library's own stream ---- */
#define DAS_NUM_KERNEL_CLASSES 16
int das_profile_enable(das_model *m, int32_t on);          /* on: every launch is bracketed by events */
int das_profile_reset(das_model *m);
/* Accumulated device time (ms) and launch count of one kernel class since the last reset. */
int das_profile_read(das_model *m, int32_t kernel_class, double *ms, int64_t *launches);
const char *das_profile_name(int32_t kernel_class);        /* NULL past the last class */

const char *das_strerror(int code);
const char *das_last_device_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DAS_H */
