// Host side of the C ABI declared in include/das.h: model and KV-pool
// ownership, sequence table, page allocator, argument validation, and the
// orchestration of one forward pass (verify step or prefill pass) as a
// sequence of HIP kernel launches on one stream.
#include "das_internal.h"
#include "../../include/das.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <string>
#include <unordered_map>
#include <unordered_set>
#include <vector>

static thread_local std::string g_dev_err;

#define HIPCHK(expr)                                                                              \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess) {                                                                   \
            g_dev_err = std::string(#expr) + ": " + hipGetErrorString(e_);                        \
            return DAS_ERR_DEVICE;                                                                \
        }                                                                                         \
    } while (0)

static inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

enum { SEQ_FREE = -1, SEQ_COMMITTED = 0, SEQ_SPECULATIVE = 1 };

struct Seq {
    int id = -1, state = SEQ_FREE, ctx = 0, pending = -1, spec_rows = 0;
    std::vector<int> pages;
};

struct LayerW { bf16_t *g1, *wqkv, *wo, *g2, *wgu, *wd; };

struct PassBlock { int slot, start, n; const int32_t *toks; int want; /* 0 none, 1 last row, 2 all rows */ };

struct das_model {
    das_config cfg;
    DasDims dm;
    hipStream_t st = nullptr;
    bool own_stream = false;
    int max_pages = 0, Mp = 0;
    // weights
    bf16_t *embed = nullptr, *gf = nullptr, *wlm = nullptr;
    std::vector<LayerW> layers;
    std::vector<void *> allocs;             // everything to hipFree
    double *inv_freq = nullptr;
    // KV pool: [layer][page][Hkv][16*D] for K and for V
    f16_t *kpool = nullptr, *vpool = nullptr;      // bf16-rounded values in binary16 containers
    size_t layer_elems = 0;
    int *page_table = nullptr;
    // workspaces
    float *h = nullptr, *cs = nullptr, *logits = nullptr, *row_stats = nullptr;
    f16_t *q_h = nullptr;
    bf16_t *xn = nullptr, *attn = nullptr, *act = nullptr, *xsel = nullptr;
    float *qkv = nullptr;                  // fp32 projections of the pass: rounded to bf16 once, after RoPE
    float *gemm_ws = nullptr;        // slice partials of narrow few-row GEMMs
    size_t gemm_ws_floats = 0;
    uint16_t *part_o = nullptr;      // split-KV partial outputs (fp16, normalised per chunk)
    float *part_ml = nullptr;        // their (m, l) per row
    size_t part_rows_cap = 0;        // 16-row blocks the partial buffers hold (fixed at load)
    int max_blocks = 0;              // most blocks one pass may have (sequences + extra prompt blocks of a prefill pass)
    unsigned long long *d_kv_sat = nullptr;      // K/V elements that did not fit their container, ever
    int *d_g = nullptr, *d_accept = nullptr, *d_next = nullptr;
    // staging
    int *h_stage = nullptr, *d_stage = nullptr;
    size_t stage_ints = 0;
    int *h_out = nullptr;                   // pinned: g[max_rows], accept[max_seqs], next[max_seqs]
    // tables
    std::vector<Seq> slots;
    std::vector<int> free_slots;
    std::unordered_map<int, int> id2slot;
    std::vector<int> free_pages;
    std::vector<int> pending_upd;           // (index, page) pairs for the device page table
    int last_rows = 0;
    bool keep_logits = false;        // materialise fp32 logits of every greedy pass (inspection); sampling always does
    bool last_has_logits = false, last_has_argmax = false;
    unsigned long long *d_keys = nullptr;   // (row maximum, ~column) keys gathered by the LM-head GEMM
    // sampling passes: per-block softmax statistics [ceil(V/32)][max_rows] (m_b, z_b), then max_rows draft logits
    float2 *stat_part = nullptr;
    // profiling
    bool prof = false;
    struct Ev { int cls; hipEvent_t a, b; };
    std::vector<Ev> ev_used;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> ev_pool;
    double prof_ms[KC_COUNT] = {0};
    long long prof_n[KC_COUNT] = {0};
};

static const char *kClassNames[KC_COUNT] = {
    "meta", "embed", "rmsnorm", "gemm_qkv", "rope_kv_write", "attention", "attention_merge", "gemm_o",
    "gemm_gateup_silu", "gemm_down", "gemm_lm_head", "argmax", "accept_greedy", "accept_sample", "kv_io"};

// ------------------------------------------------------------------------------------------------ helpers

template <typename T>
static int dev_alloc(das_model *m, T **p, size_t count) {
    void *q = nullptr;
    hipError_t e = hipMalloc(&q, std::max<size_t>(count, 1) * sizeof(T));
    if (e != hipSuccess) { g_dev_err = std::string("hipMalloc: ") + hipGetErrorString(e); (void)hipGetLastError(); return DAS_ERR_NOMEM; }
    m->allocs.push_back(q);
    *p = reinterpret_cast<T *>(q);
    return DAS_OK;
}

struct ProfScope {
    das_model *m; int cls; hipEvent_t a = nullptr, b = nullptr;
    ProfScope(das_model *mm, int c) : m(mm), cls(c) {
        if (!m->prof) return;
        if (m->ev_pool.empty()) {
            hipEvent_t x, y;
            if (hipEventCreate(&x) != hipSuccess || hipEventCreate(&y) != hipSuccess) return;
            m->ev_pool.push_back({x, y});
        }
        a = m->ev_pool.back().first; b = m->ev_pool.back().second;
        m->ev_pool.pop_back();
        (void)hipEventRecord(a, m->st);
    }
    ~ProfScope() {
        if (!a) return;
        (void)hipEventRecord(b, m->st);
        m->ev_used.push_back({cls, a, b});
    }
};

static void prof_collect(das_model *m) {          // call after the stream is synchronised
    for (auto &e : m->ev_used) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, e.a, e.b) == hipSuccess) { m->prof_ms[e.cls] += ms; m->prof_n[e.cls] += 1; }
        m->ev_pool.push_back({e.a, e.b});
    }
    m->ev_used.clear();
}

static int pages_for(int tokens) { return (tokens + DAS_PAGE - 1) / DAS_PAGE; }

static void grow_pages(das_model *m, int slot, int tokens) {
    Seq &s = m->slots[slot];
    while ((int)s.pages.size() < pages_for(tokens)) {
        int pg = m->free_pages.back();
        m->free_pages.pop_back();
        m->pending_upd.push_back(slot * m->max_pages + (int)s.pages.size());
        m->pending_upd.push_back(pg);
        s.pages.push_back(pg);
    }
}
static void shrink_pages(das_model *m, int slot, int tokens) {
    Seq &s = m->slots[slot];
    while ((int)s.pages.size() > pages_for(tokens)) { m->free_pages.push_back(s.pages.back()); s.pages.pop_back(); }
}

// Size of a pass before anything is written or changed: ints of the staging block it needs (n_upd page-table
// updates, n_u uniforms per stream) and 16-row blocks of split-KV partials.  Partials are kept per 16-row block: 16 x D
// accumulators in the lane order the MFMA leaves them in, and (m, l) per row.
struct PassSize { size_t stage_ints, part_rows; };
static PassSize pass_size(const das_model *m, const std::vector<PassBlock> &blocks, size_t n_upd, size_t n_u) {
    const int chunk_tokens = das_attn_chunk(m->dm.Hkv);
    size_t T = 0, items = 0, mblk = 0, prow = 0;
    for (auto &b : blocks) {
        const size_t nrb = ((size_t)m->dm.G * b.n + 15) / 16, nchunk = ((size_t)b.start + b.n + chunk_tokens - 1) / chunk_tokens;
        T += b.n; items += nchunk; prow += nchunk * nrb;
        if (nchunk > 1) mblk += nrb;
    }
    return {5 * T + 6 * blocks.size() + 2 * items * m->dm.Hkv + 2 * mblk + 2 * n_upd + 2 * n_u, prow};
}
static int check_pass_size(const das_model *m, const PassSize &ps) {
    if (ps.stage_ints > m->stage_ints) return DAS_ERR_INVALID;        // over a configured maximum
    if (ps.part_rows > m->part_rows_cap) return DAS_ERR_NOMEM;
    return DAS_OK;
}

// ------------------------------------------------------------------------------------------------ one forward pass
// Rows of all blocks go through the layer stack; logits (+ argmax) are produced for the
// selected rows.  On return kernels are enqueued, nothing is synchronised.  The caller has checked pass_size() against
// the staging block and the partial buffers: nothing here allocates.
// inv_temp > 0: a sampling pass (1 / temperature): the logits' per-block softmax statistics and every row's draft logit
// are produced (m->stat_part), and the row statistics (m->row_stats); u_sample is then non-null.
static int run_pass(das_model *m, const std::vector<PassBlock> &blocks, const float *u_accept, const float *u_sample,
                    int n_u, float inv_temp, PassMeta *pm_out, const float **d_ua, const float **d_us) {
    const DasDims &dm = m->dm;
    const int NB = (int)blocks.size();
    int T = 0;
    for (auto &b : blocks) T += b.n;
    std::vector<int> items[3], mblk;
    size_t prow = 0;
    // ---- pack the metadata
    int *p = m->h_stage;
    int *tok = p; p += T;
    int *row_pos = p; p += T;
    int *row_b = p; p += T;
    int *sel = p; p += T;
    int *dtok = p; p += T;         // per selected row: the draft token its logits are tested against (-1: none)
    int *b_slot = p; p += NB;
    int *b_start = p; p += NB;
    int *b_n = p; p += NB;
    int *b_row0 = p; p += NB;
    int *b_prow = p; p += NB;
    int *b_nchunk = p; p += NB;
    int r = 0, n_sel = 0;
    const int chunk_tokens = das_attn_chunk(dm.Hkv);
    for (int b = 0; b < NB; ++b) {
        const PassBlock &pb = blocks[b];
        b_slot[b] = pb.slot; b_start[b] = pb.start; b_n[b] = pb.n; b_row0[b] = r;
        const int R = dm.G * pb.n, nrb = (R + 15) / 16;
        const int nchunk = (pb.start + pb.n + chunk_tokens - 1) / chunk_tokens;
        b_prow[b] = (int)prow; b_nchunk[b] = nchunk;
        prow += (size_t)nchunk * nrb;
        if (nchunk > 1)      // (one chunk: the attention kernel writes the finished rows itself)
            for (int rb = 0; rb < nrb; ++rb) { mblk.push_back(b); mblk.push_back(rb); }
        // two kernel shapes: up to 8 row blocks of 16 query rows per KV head (2 per wave), or up to 16 (4 per wave).
        // One launch for everything up to 8 blocks lets short sequences fill the tail of the long ones.
        const int cls = nrb <= 8 ? 1 : 2;
        for (int c = 0; c < nchunk; ++c) { items[cls].push_back(b); items[cls].push_back(c); }
        for (int j = 0; j < pb.n; ++j, ++r) {
            tok[r] = pb.toks[j]; row_pos[r] = pb.start + j; row_b[r] = b;
            if (pb.want == 2 || (pb.want == 1 && j == pb.n - 1)) {
                dtok[n_sel] = (pb.want == 2 && j + 1 < pb.n) ? pb.toks[j + 1] : -1;
                sel[n_sel++] = r;
            }
        }
    }
    if (prow > m->part_rows_cap) return DAS_ERR_NOMEM;
    // One work item per (sequence, chunk, KV head), longest first over the whole launch so that the short last
    // chunks fill its tail; among equal lengths one KV head's items run side by side (measured faster than the
    // heads of one chunk side by side).  Entry: sequence, chunk | head << 20.
    for (int c = 0; c < 3; ++c) {
        std::vector<std::pair<int, int>> v;
        for (int h = 0; h < dm.Hkv; ++h)
            for (size_t i = 0; i + 1 < items[c].size(); i += 2) v.push_back({items[c][i], items[c][i + 1] | (h << 20)});
        auto tokens = [&](const std::pair<int, int> &it) {
            const int total = blocks[it.first].start + blocks[it.first].n;
            return std::min(total - (it.second & 0xFFFFF) * chunk_tokens, chunk_tokens);
        };
        std::stable_sort(v.begin(), v.end(), [&](const std::pair<int, int> &a, const std::pair<int, int> &b) { return tokens(a) > tokens(b); });
        items[c].resize(2 * v.size());
        for (size_t i = 0; i < v.size(); ++i) { items[c][2 * i] = v[i].first; items[c][2 * i + 1] = v[i].second; }
    }
    int *item_ptr[3];
    for (int c = 0; c < 3; ++c) { item_ptr[c] = p; std::copy(items[c].begin(), items[c].end(), p); p += items[c].size(); }
    int *mblk_p = p; std::copy(mblk.begin(), mblk.end(), p); p += mblk.size();
    const int n_upd = (int)m->pending_upd.size() / 2;
    int *upd = p; std::copy(m->pending_upd.begin(), m->pending_upd.end(), p); p += 2 * n_upd;
    float *ua = reinterpret_cast<float *>(p);
    if (u_accept) { std::memcpy(p, u_accept, sizeof(float) * n_u); p += n_u; }
    float *us = reinterpret_cast<float *>(p);
    if (u_sample) { std::memcpy(p, u_sample, sizeof(float) * n_u); p += n_u; }
    const size_t used = (size_t)(p - m->h_stage);

    hipStream_t st = m->st;
    auto dptr = [&](const void *hp) { return m->d_stage + (reinterpret_cast<const int *>(hp) - m->h_stage); };
    PassMeta pm;
    pm.T = T; pm.NB = NB;
    pm.tok = dptr(tok); pm.row_pos = dptr(row_pos); pm.row_b = dptr(row_b); pm.sel = dptr(sel); pm.n_sel = n_sel;
    pm.b_slot = dptr(b_slot); pm.b_start = dptr(b_start); pm.b_n = dptr(b_n); pm.b_row0 = dptr(b_row0);
    pm.b_prow = dptr(b_prow); pm.b_nchunk = dptr(b_nchunk);
    pm.mblk = dptr(mblk_p); pm.n_mblk = (int)mblk.size() / 2;
    pm.page_table = m->page_table; pm.max_pages = m->max_pages; pm.num_pages = (int)m->cfg.num_pages; pm.chunk = chunk_tokens;
    {
        ProfScope ps(m, KC_META);
        HIPCHK(hipMemcpyAsync(m->d_stage, m->h_stage, used * sizeof(int), hipMemcpyHostToDevice, st));
        launch_pt_update(m->page_table, dptr(upd), n_upd, st);
        m->pending_upd.clear();
        launch_rope_table(pm, m->inv_freq, m->cs, dm.D, st);
    }
    { ProfScope ps(m, KC_EMBED); launch_embed(pm, m->embed, m->h, dm.d, st); }
    // A residual GEMM whose K slices are summed by a second kernel (passes of a few hundred rows) lets that kernel
    // normalise the finished rows as well: xn_ready says that the next RMSNorm has already been done.
    bool xn_ready = false;
    for (int l = 0; l < dm.L; ++l) {
        const LayerW &w = m->layers[l];
        f16_t *kl = m->kpool + (size_t)l * m->layer_elems, *vl = m->vpool + (size_t)l * m->layer_elems;
        if (!xn_ready) { ProfScope ps(m, KC_RMSNORM); launch_rmsnorm(m->h, w.g1, m->xn, nullptr, T, dm.d, dm.rms_eps, st); }
        // (few rows: the K-slice partials of QKV stay in the workspace and the rotation kernel adds them)
        int qkv_slices = 1;
        // (many rows, head dim 128: the GEMM's epilogue rotates and stores q, k, v itself and reports 0 slices left)
        const RopeEpi re = {pm.row_b, pm.row_pos, pm.b_slot, pm.page_table, pm.max_pages, reinterpret_cast<const float2 *>(m->cs),
                            m->q_h, kl, vl, dm.Hq, dm.Hkv, m->d_kv_sat};
        { ProfScope ps(m, KC_GEMM_QKV); launch_gemm(EPI_F32_ROWMAJOR, m->xn, w.wqkv, m->qkv, T, dm.qkvN, dm.d, dm.qkvN, st, m->gemm_ws, m->gemm_ws_floats, nullptr, &qkv_slices,
                                                    nullptr, 0.f, dm.D == 128 ? &re : nullptr); }
        if (qkv_slices > 0) { ProfScope ps(m, KC_ROPE_KV); launch_rope_kv(pm, qkv_slices > 1 ? m->gemm_ws : m->qkv, qkv_slices, m->q_h, m->cs, kl, vl, dm, m->d_kv_sat, st); }
        {
            ProfScope ps(m, KC_ATTN);
            for (int c = 0; c < 3; ++c)
                launch_attn(pm, dptr(item_ptr[c]), (int)items[c].size() / 2, 1 << c, m->q_h, kl, vl, m->part_o, m->part_ml, m->attn, dm, st);
        }
        { ProfScope ps(m, KC_ATTN_MERGE); launch_attn_merge(pm, m->part_o, m->part_ml, m->attn, dm, st); }
        {
            const GemmNormTail post_attn = {w.g2, m->xn, dm.rms_eps};
            ProfScope ps(m, KC_GEMM_O);
            xn_ready = launch_gemm(EPI_RESID_F32, m->attn, w.wo, m->h, T, dm.d, dm.Hq * dm.D, dm.d, st, m->gemm_ws, m->gemm_ws_floats, &post_attn);
        }
        if (!xn_ready) { ProfScope ps(m, KC_RMSNORM); launch_rmsnorm(m->h, w.g2, m->xn, nullptr, T, dm.d, dm.rms_eps, st); }
        { ProfScope ps(m, KC_GEMM_GATEUP); launch_gemm(EPI_SILU_FRAG, m->xn, w.wgu, m->act, T, 2 * dm.Fp, dm.d, dm.Fp, st, m->gemm_ws, m->gemm_ws_floats); }
        {
            // the next layer's input norm; the final norm gathers the rows that get logits and stays a kernel of its own
            const GemmNormTail next_input = {l + 1 < dm.L ? m->layers[l + 1].g1 : nullptr, m->xn, dm.rms_eps};
            ProfScope ps(m, KC_GEMM_DOWN);
            xn_ready = launch_gemm(EPI_RESID_F32, m->act, w.wd, m->h, T, dm.d, dm.Fp, dm.d, st, m->gemm_ws, m->gemm_ws_floats,
                                   l + 1 < dm.L ? &next_input : nullptr);
        }
    }
    if (n_sel > 0) {
        { ProfScope ps(m, KC_RMSNORM); launch_rmsnorm(m->h, m->gf, m->xsel, pm.sel, n_sel, dm.d, dm.rms_eps, st); }
        // Greedy passes need one number per row, the first column of the row maximum: the LM-head GEMM gathers it in
        // its epilogue and the [rows][vocab] logits never reach memory.  Sampling, inspection mode and small
        // vocabularies (narrow GEMM shapes) write the logits and scan them.
        const bool sampling = inv_temp > 0.f;
        const bool fused = !m->keep_logits && !sampling && dm.V >= 16384;
        const int nblk = (dm.V + 31) / 32, ldp = m->cfg.max_rows;
        float *draft_logit = reinterpret_cast<float *>(m->stat_part + (size_t)nblk * ldp);
        if (sampling && !m->keep_logits && gemm_rowstats_supported(n_sel, dm.V)) {
            // a sampling pass does not need its logits either: the LM-head GEMM leaves per-block softmax statistics and the
            // draft tokens' logits, and the one block a draw falls into is computed again by the kernel that draws
            { ProfScope ps(m, KC_GEMM_LMHEAD); launch_gemm(EPI_ROWSTATS, m->xsel, m->wlm, m->stat_part, n_sel, dm.V, dm.d, ldp, st, m->gemm_ws, m->gemm_ws_floats, nullptr, nullptr, dptr(dtok), inv_temp); }
            { ProfScope ps(m, KC_SAMPLE); launch_row_stats_merge(m->stat_part, ldp, dm.V, n_sel, inv_temp, reinterpret_cast<float2 *>(m->row_stats), st); }
            m->last_has_argmax = false;
            m->last_has_logits = false;
        } else if (fused) {
            { ProfScope ps(m, KC_ARGMAX); launch_rowmax_keys_clear(m->d_keys, n_sel, st); }
            { ProfScope ps(m, KC_GEMM_LMHEAD); launch_gemm(EPI_ROWMAX, m->xsel, m->wlm, m->d_keys, n_sel, dm.V, dm.d, dm.V, st, m->gemm_ws, m->gemm_ws_floats); }
            { ProfScope ps(m, KC_ARGMAX); launch_rowmax_keys_decode(m->d_keys, n_sel, m->d_g, st); }
        } else {
            { ProfScope ps(m, KC_GEMM_LMHEAD); launch_gemm(EPI_F32_ROWMAJOR, m->xsel, m->wlm, m->logits, n_sel, dm.V, dm.d, dm.V, st, m->gemm_ws, m->gemm_ws_floats); }
            // the row argmax is what greedy acceptance reads; a sampling pass needs it only for inspection
            if (!sampling || m->keep_logits) { ProfScope ps(m, KC_ARGMAX); launch_argmax(m->logits, n_sel, dm.V, m->d_g, st); }
            m->last_has_argmax = !sampling || m->keep_logits;
            m->last_has_logits = true;
            if (sampling) {
                ProfScope ps(m, KC_SAMPLE);
                launch_block_stats(m->logits, n_sel, dm.V, inv_temp, dptr(dtok), m->stat_part, ldp, draft_logit, st);
                launch_row_stats_merge(m->stat_part, ldp, dm.V, n_sel, inv_temp, reinterpret_cast<float2 *>(m->row_stats), st);
            }
        }
        if (fused) { m->last_has_argmax = true; m->last_has_logits = false; }
    }
    hipError_t le = hipGetLastError();
    if (le != hipSuccess) { g_dev_err = std::string("kernel launch: ") + hipGetErrorString(le); return DAS_ERR_DEVICE; }
    m->last_rows = n_sel;
    *pm_out = pm;
    if (d_ua) *d_ua = reinterpret_cast<const float *>(dptr(ua));
    if (d_us) *d_us = reinterpret_cast<const float *>(dptr(us));
    return DAS_OK;
}

// ------------------------------------------------------------------------------------------------ load / free

static int check_config(const das_config *c) {
    if (!c) return DAS_ERR_INVALID;
    if (c->n_layers < 1 || c->d_model < 64 || c->d_model % 64 || c->d_model > 8192 || c->n_q_heads < 1 || c->n_kv_heads < 1 ||
        c->n_q_heads % c->n_kv_heads || (c->head_dim != 64 && c->head_dim != 128) || c->d_ffn < 8 || c->d_ffn % 8 ||
        c->vocab < 2 || !(c->rope_theta > 0.f) || !(c->rms_eps > 0.f))
        return DAS_ERR_INVALID;
    if (c->page_size != DAS_PAGE || c->max_seqs < 1 || c->max_ctx < DAS_PAGE || c->max_rows < 1 || c->max_draft < 0 ||
        c->num_pages < 1 || c->num_pages > 0x3FFFFFFF)
        return DAS_ERR_INVALID;
    const int G = c->n_q_heads / c->n_kv_heads;
    if ((1 + c->max_draft) * G > 256 || 1 + c->max_draft > c->max_rows) return DAS_ERR_INVALID;
    if ((int64_t)c->max_rows * c->vocab > (int64_t)1 << 40) return DAS_ERR_INVALID;
    return DAS_OK;
}

extern "C" int das_model_free(das_model *m) {
    if (!m) return DAS_ERR_INVALID;
    (void)hipStreamSynchronize(m->st);
    for (void *p : m->allocs) (void)hipFree(p);
    if (m->h_stage) (void)hipHostFree(m->h_stage);
    if (m->h_out) (void)hipHostFree(m->h_out);
    for (auto &e : m->ev_pool) { (void)hipEventDestroy(e.first); (void)hipEventDestroy(e.second); }
    for (auto &e : m->ev_used) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
    if (m->own_stream && m->st) (void)hipStreamDestroy(m->st);
    delete m;
    return DAS_OK;
}

// One tensor of the canonical blob into `dst` on the device: copied from the caller's blob, or generated there
// (matrices N(0, 0.02^2) from the counter-based generator keyed by (seed, tensor index); gains 1.0).
struct WeightSource {
    const uint16_t *src; uint64_t seed, tensor = 0; hipStream_t st;
    int next(bf16_t *dst, size_t count, bool gain) {
        if (src) {
            HIPCHK(hipMemcpyAsync(dst, src, count * 2, hipMemcpyHostToDevice, st));
            HIPCHK(hipStreamSynchronize(st));
            src += count;
        } else if (gain) launch_fill_const(dst, count, (bf16_t)0x3F80, st);
        else launch_fill_normal(dst, count, seed, tensor, 0.02, st);
        ++tensor;
        return DAS_OK;
    }
};

static int load_impl(das_model *m, const uint16_t *wb, uint64_t seed) {
    const das_config &c = m->cfg;
    DasDims &dm = m->dm;
    dm.L = c.n_layers; dm.d = c.d_model; dm.Hq = c.n_q_heads; dm.Hkv = c.n_kv_heads; dm.D = c.head_dim;
    dm.F = c.d_ffn; dm.V = c.vocab; dm.G = dm.Hq / dm.Hkv; dm.Fp = round_up(dm.F, 64);
    dm.qkvN = (dm.Hq + 2 * dm.Hkv) * dm.D; dm.rope_theta = c.rope_theta; dm.rms_eps = c.rms_eps;
    m->max_pages = pages_for(c.max_ctx);
    // GEMM tiles may read activation rows past the last one (tile heights 64 ... 288 do not all divide 256): the row
    // count of every activation buffer is rounded up to 256 and one more tile of slack is added
    m->Mp = round_up(c.max_rows, 256) + 256;
    const int d = dm.d, qd = dm.Hq * dm.D, kd = dm.Hkv * dm.D, F = dm.F, Fp = dm.Fp, V = dm.V;
    const size_t Mp = m->Mp;
    int rc;
#define A(ptr, count) if ((rc = dev_alloc(m, &(ptr), (count))) != DAS_OK) return rc
    // ---- weights: upload tensor by tensor through one scratch buffer, repack on the device
    const size_t big = std::max((size_t)V * d, std::max((size_t)F * d * 2, (size_t)qd * d + 2 * (size_t)kd * d));
    bf16_t *tmp; A(tmp, big);
    A(m->embed, (size_t)V * d);
    A(m->gf, (size_t)d);
    const int Vp = round_up(V, 256), qkvNp = round_up(dm.qkvN, 256), dp = round_up(d, 256), gup = round_up(2 * Fp, 256);
    A(m->wlm, (size_t)Vp * d);
    m->layers.resize(dm.L);
    WeightSource ws{wb, seed, 0, m->st};
#define W(dst, count, gain) if ((rc = ws.next((dst), (count), (gain))) != DAS_OK) return rc
    W(m->embed, (size_t)V * d, false);
    for (int l = 0; l < dm.L; ++l) {
        LayerW &w = m->layers[l];
        A(w.g1, (size_t)d); A(w.g2, (size_t)d);
        A(w.wqkv, (size_t)qkvNp * d); A(w.wo, (size_t)dp * qd); A(w.wgu, (size_t)gup * d); A(w.wd, (size_t)dp * Fp);
        W(w.g1, (size_t)d, true);
        // Wq, Wk, Wv are adjacent in the blob: one [qkvN][d] matrix made of three tensors
        W(tmp, (size_t)qd * d, false); W(tmp + (size_t)qd * d, (size_t)kd * d, false); W(tmp + (size_t)(qd + kd) * d, (size_t)kd * d, false);
        launch_pack_weight(tmp, w.wqkv, dm.qkvN, d, qkvNp, d, m->st);
        W(tmp, (size_t)d * qd, false);
        launch_pack_weight(tmp, w.wo, d, qd, dp, qd, m->st);
        W(w.g2, (size_t)d, true);
        W(tmp, (size_t)F * d, false); W(tmp + (size_t)F * d, (size_t)F * d, false);
        HIPCHK(hipMemsetAsync(w.wgu, 0, (size_t)gup * d * 2, m->st));
        launch_pack_gateup(tmp, tmp + (size_t)F * d, w.wgu, F, d, Fp, m->st);
        W(tmp, (size_t)d * F, false);
        launch_pack_weight(tmp, w.wd, d, F, dp, Fp, m->st);
    }
    W(m->gf, (size_t)d, true);
    W(tmp, (size_t)V * d, false);
    launch_pack_weight(tmp, m->wlm, V, d, Vp, d, m->st);
    HIPCHK(hipStreamSynchronize(m->st));
#undef W
    // ---- RoPE inverse frequencies theta^(-2i/D), fp64
    {
        std::vector<double> f(dm.D / 2);
        for (int i = 0; i < dm.D / 2; ++i) f[i] = std::pow((double)c.rope_theta, -2.0 * i / dm.D);
        A(m->inv_freq, f.size());
        HIPCHK(hipMemcpy(m->inv_freq, f.data(), f.size() * sizeof(double), hipMemcpyHostToDevice));
    }
    // ---- KV pool (zeroed: every value ever read from it is finite), page table
    m->layer_elems = (size_t)c.num_pages * dm.Hkv * DAS_PAGE * dm.D;
    A(m->kpool, m->layer_elems * dm.L);
    A(m->vpool, m->layer_elems * dm.L);
    HIPCHK(hipMemsetAsync(m->kpool, 0, m->layer_elems * dm.L * 2, m->st));
    HIPCHK(hipMemsetAsync(m->vpool, 0, m->layer_elems * dm.L * 2, m->st));
    A(m->page_table, (size_t)c.max_seqs * m->max_pages);
    HIPCHK(hipMemsetAsync(m->page_table, 0, (size_t)c.max_seqs * m->max_pages * sizeof(int), m->st));
    // ---- workspaces (row counts padded to 256 so GEMM tiles may over-read)
    A(m->h, Mp * d); A(m->xn, Mp * d); A(m->qkv, Mp * dm.qkvN); A(m->q_h, Mp * qd); A(m->attn, Mp * qd); A(m->act, Mp * Fp); A(m->xsel, Mp * d);
    A(m->cs, Mp * dm.D); A(m->logits, (size_t)c.max_rows * V); A(m->row_stats, (size_t)c.max_rows * 2);
    A(m->d_g, (size_t)c.max_rows); A(m->d_accept, (size_t)c.max_seqs); A(m->d_next, (size_t)c.max_seqs); A(m->d_keys, (size_t)c.max_rows);
    A(m->stat_part, (size_t)((V + 31) / 32) * c.max_rows + ((size_t)c.max_rows + 1) / 2);
    {   // K-slice partials of the narrow GEMMs (QKV, O, down; a small LM head): whatever the largest pass can use
        const int rows = c.max_rows;
        size_t need = std::max(gemm_ws_floats_needed(rows, dm.qkvN, d), std::max(gemm_ws_floats_needed(rows, d, dm.Hq * dm.D), gemm_ws_floats_needed(rows, d, Fp)));
        if (V < 16384) need = std::max(need, gemm_ws_floats_needed(rows, V, d));
        m->gemm_ws_floats = std::max<size_t>(need, 4);
        A(m->gemm_ws, m->gemm_ws_floats);
    }
    HIPCHK(hipMemsetAsync(m->xn, 0, Mp * d * 2, m->st));
    HIPCHK(hipMemsetAsync(m->attn, 0, Mp * qd * 2, m->st));
    HIPCHK(hipMemsetAsync(m->act, 0, Mp * Fp * 2, m->st));
    HIPCHK(hipMemsetAsync(m->xsel, 0, Mp * d * 2, m->st));
    A(m->d_kv_sat, 1);
    HIPCHK(hipMemsetAsync(m->d_kv_sat, 0, sizeof(unsigned long long), m->st));
    // ---- split-KV partials, sized here once for every pass the configuration allows.  A block (a sequence's rows in
    // one pass) has at most 16 row blocks of 16 query rows per KV head and one partial per chunk it spans; the chunks of
    // distinct sequences together are bounded by the KV pool (a chunk is at most half empty per sequence).  A prefill
    // pass that takes several blocks of ONE prompt is cut to fit this capacity by its caller.
    const int chunk_tokens = das_attn_chunk(c.n_kv_heads);
    m->max_blocks = c.max_seqs + c.max_rows / std::max(1, std::min(256 / dm.G, c.max_rows)) + 1;
    {
        const size_t pool_chunks = (size_t)c.num_pages * DAS_PAGE / chunk_tokens + (size_t)c.max_seqs;
        const size_t per_seq_chunks = (size_t)c.max_ctx / chunk_tokens + 1;
        m->part_rows_cap = 16 * std::min(pool_chunks, per_seq_chunks * (size_t)c.max_seqs);
        A(m->part_o, m->part_rows_cap * dm.Hkv * 16 * dm.D);
        A(m->part_ml, m->part_rows_cap * dm.Hkv * 32);
    }
    // ---- staging (see pass_size)
    const size_t max_items = (size_t)m->max_blocks * (c.max_ctx / chunk_tokens + 2);
    m->stage_ints = 7 * (size_t)c.max_rows + 6 * (size_t)m->max_blocks + 2 * max_items * dm.Hkv +
                    2 * ((size_t)c.max_rows * dm.G / 16 + (size_t)m->max_blocks) +
                    2 * ((size_t)c.max_rows / DAS_PAGE + 2 * (size_t)c.max_seqs + 2) + 64;
    HIPCHK(hipHostMalloc((void **)&m->h_stage, m->stage_ints * sizeof(int), hipHostMallocDefault));
    A(m->d_stage, m->stage_ints);
    HIPCHK(hipHostMalloc((void **)&m->h_out, ((size_t)c.max_rows + 2 * (size_t)c.max_seqs) * sizeof(int), hipHostMallocDefault));
    // ---- tables
    m->slots.resize(c.max_seqs);
    for (int i = c.max_seqs - 1; i >= 0; --i) m->free_slots.push_back(i);
    m->free_pages.reserve((size_t)c.num_pages);
    for (int64_t i = c.num_pages - 1; i >= 0; --i) m->free_pages.push_back((int)i);   // pop_back() -> page 0 first
    HIPCHK(hipStreamSynchronize(m->st));
    // the upload scratch is no longer needed
    (void)hipFree(tmp);
    m->allocs.erase(std::find(m->allocs.begin(), m->allocs.end(), (void *)tmp));
#undef A
    return DAS_OK;
}

extern "C" int das_model_load(const das_config *cfg, uint64_t seed, const uint16_t *weights_bf16, void *hip_stream, das_model **out) {
    if (!out) return DAS_ERR_INVALID;
    *out = nullptr;
    int rc = check_config(cfg);
    if (rc != DAS_OK) return rc;
    int ndev = 0;
    HIPCHK(hipGetDeviceCount(&ndev));
    if (ndev < 1) { g_dev_err = "no HIP device"; return DAS_ERR_DEVICE; }
    das_model *m = new das_model();
    m->cfg = *cfg;
    if (hip_stream) m->st = reinterpret_cast<hipStream_t>(hip_stream);
    else {
        hipError_t e = hipStreamCreate(&m->st);
        if (e != hipSuccess) { g_dev_err = hipGetErrorString(e); delete m; return DAS_ERR_DEVICE; }
        m->own_stream = true;
    }
    rc = load_impl(m, weights_bf16, seed);
    if (rc != DAS_OK) { das_model_free(m); return rc; }
    *out = m;
    return DAS_OK;
}

// ------------------------------------------------------------------------------------------------ lookups / validation

static int find_slot(das_model *m, int id) {
    auto it = m->id2slot.find(id);
    return it == m->id2slot.end() ? -1 : it->second;
}
static bool unique_ids(int n, const int32_t *ids) {
    std::unordered_set<int> s;
    for (int i = 0; i < n; ++i) if (!s.insert(ids[i]).second) return false;
    return true;
}
static int new_seq(das_model *m, int id) {
    int slot = m->free_slots.back();
    m->free_slots.pop_back();
    Seq &s = m->slots[slot];
    s = Seq();
    s.id = id; s.state = SEQ_COMMITTED;
    m->id2slot[id] = slot;
    return slot;
}
static void purge_pending(das_model *m, int slot) {
    std::vector<int> keep;
    for (size_t i = 0; i + 1 < m->pending_upd.size(); i += 2)
        if (m->pending_upd[i] / m->max_pages != slot) { keep.push_back(m->pending_upd[i]); keep.push_back(m->pending_upd[i + 1]); }
    m->pending_upd.swap(keep);
}
static void drop_seq(das_model *m, int slot) {
    Seq &s = m->slots[slot];
    purge_pending(m, slot);
    shrink_pages(m, slot, 0);
    m->id2slot.erase(s.id);
    s = Seq();
    m->free_slots.push_back(slot);
}
static int upload_page_row(das_model *m, int slot) {
    Seq &s = m->slots[slot];
    purge_pending(m, slot);      // queued single-entry updates of this row: the whole row is written now
    HIPCHK(hipStreamSynchronize(m->st));
    if (!s.pages.empty())
        HIPCHK(hipMemcpy(m->page_table + (size_t)slot * m->max_pages, s.pages.data(), s.pages.size() * sizeof(int), hipMemcpyHostToDevice));
    return DAS_OK;
}

static int check_sampling(const das_sampling *s) {
    if (!s) return DAS_OK;
    if (!(s->temperature > 0.f) || !s->u_sample) return DAS_ERR_INVALID;
    return DAS_OK;
}

// ------------------------------------------------------------------------------------------------ prefill

extern "C" int das_prefill(das_model *m, int32_t n, const int32_t *seq_ids, const int32_t *tokens, const int32_t *lens,
                           const das_sampling *sampling, int32_t *next_token) {
    if (!m || n < 0) return DAS_ERR_INVALID;
    if (n == 0) return DAS_OK;
    if (!seq_ids || !tokens || !lens || !next_token || check_sampling(sampling) != DAS_OK) return DAS_ERR_INVALID;
    if (!unique_ids(n, seq_ids)) return DAS_ERR_INVALID;
    int64_t need_pages = 0, tot = 0;
    for (int i = 0; i < n; ++i) {
        if (lens[i] < 1 || lens[i] > m->cfg.max_ctx) return DAS_ERR_INVALID;
        if (find_slot(m, seq_ids[i]) >= 0) return DAS_ERR_STATE;
        need_pages += pages_for(lens[i]);
        tot += lens[i];
    }
    for (int64_t i = 0; i < tot; ++i) if (tokens[i] < 0 || tokens[i] >= m->dm.V) return DAS_ERR_INVALID;
    if ((int)m->free_slots.size() < n || need_pages > (int64_t)m->free_pages.size()) return DAS_ERR_NOMEM;

    std::vector<int> slot(n), done(n, 0);
    std::vector<const int32_t *> base(n);
    const int32_t *tp = tokens;
    for (int i = 0; i < n; ++i) {
        slot[i] = new_seq(m, seq_ids[i]);
        grow_pages(m, slot[i], lens[i]);
        base[i] = tp; tp += lens[i];
    }
    int rc = DAS_OK;
    for (int i = 0; i < n && rc == DAS_OK; ++i) rc = upload_page_row(m, slot[i]);
    // A pass takes up to max_rows prompt rows.  The attention kernel serves at most 256 query rows per KV head from one
    // sweep over the KV, so a prompt enters as blocks of floor(256 / G) rows; several blocks of the same prompt may share
    // a pass (a block attends to the KV that earlier blocks of the pass write in the same layer, kernel after kernel),
    // so a long prompt streams the weights once per max_rows rows, not once per block.
    const int per_blk = std::min(256 / m->dm.G, m->cfg.max_rows);
    int first = 0;                                   // first unfinished sequence
    while (rc == DAS_OK && first < n) {
        std::vector<PassBlock> blocks;
        std::vector<int> who;
        int T = 0, n_want = 0;
        bool full = false;
        for (int i = first; i < n && !full; ++i) {
            int d0 = done[i];
            while (d0 < lens[i]) {
                const int rows = std::min(std::min(lens[i] - d0, per_blk), m->cfg.max_rows - T);
                if (rows <= 0 || (int)blocks.size() >= m->max_blocks) { full = true; break; }
                blocks.push_back({slot[i], d0, rows, base[i] + d0, (d0 + rows == lens[i]) ? 1 : 0});
                if (check_pass_size(m, pass_size(m, blocks, m->pending_upd.size() / 2, (size_t)n_want + 1)) != DAS_OK) {
                    blocks.pop_back(); full = true; break;      // the staging block or the partial buffers are full
                }
                who.push_back(i);
                n_want += blocks.back().want ? 1 : 0;
                T += rows; d0 += rows;
            }
        }
        if (blocks.empty()) { rc = DAS_ERR_NOMEM; break; }      // (one block always fits a consistent configuration)
        PassMeta pm;
        const float *d_ua = nullptr, *d_us = nullptr;
        std::vector<float> us;
        int n_fin = 0;
        for (auto &b : blocks) n_fin += b.want ? 1 : 0;
        if (sampling && n_fin) for (size_t bi = 0; bi < blocks.size(); ++bi) if (blocks[bi].want) us.push_back(sampling->u_sample[who[bi]]);
        rc = run_pass(m, blocks, nullptr, us.empty() ? nullptr : us.data(), (int)us.size(), us.empty() ? 0.f : 1.f / sampling->temperature,
                      &pm, &d_ua, &d_us);
        if (rc != DAS_OK) break;
        if (n_fin) {
            if (sampling) {
                ProfScope ps(m, KC_SAMPLE);
                const int nblk = (m->dm.V + 31) / 32, ldp = m->cfg.max_rows;
                launch_sample(m->stat_part, ldp, m->dm.V, reinterpret_cast<const float2 *>(m->row_stats),
                              reinterpret_cast<const float *>(m->stat_part + (size_t)nblk * ldp), m->xsel, m->wlm, m->dm.d, pm.tok, pm.b_row0,
                              pm.b_n, n_fin, 1.f / sampling->temperature, nullptr, d_us, 1, m->d_accept, m->d_next, m->st);
                if (hipMemcpyAsync(m->h_out, m->d_next, n_fin * sizeof(int), hipMemcpyDeviceToHost, m->st) != hipSuccess) rc = DAS_ERR_DEVICE;
            } else {
                if (hipMemcpyAsync(m->h_out, m->d_g, n_fin * sizeof(int), hipMemcpyDeviceToHost, m->st) != hipSuccess) rc = DAS_ERR_DEVICE;
            }
        }
        if (hipStreamSynchronize(m->st) != hipSuccess) { g_dev_err = "stream synchronize failed in prefill"; rc = DAS_ERR_DEVICE; }
        prof_collect(m);
        if (rc != DAS_OK) break;
        int f = 0;
        for (size_t bi = 0; bi < blocks.size(); ++bi) {
            int i = who[bi];
            done[i] += blocks[bi].n;
            if (blocks[bi].want) next_token[i] = m->h_out[f++];
        }
        while (first < n && done[first] >= lens[first]) ++first;
    }
    if (rc != DAS_OK) {                              // undo: the sequences never existed
        for (int i = 0; i < n; ++i) drop_seq(m, slot[i]);
        return rc;
    }
    for (int i = 0; i < n; ++i) {
        Seq &s = m->slots[slot[i]];
        s.ctx = lens[i]; s.pending = next_token[i]; s.state = SEQ_COMMITTED; s.spec_rows = 0;
    }
    return DAS_OK;
}

// ------------------------------------------------------------------------------------------------ verify

extern "C" int das_verify_step(das_model *m, int32_t n, const int32_t *seq_ids, const int32_t *ctx_lens,
                               const int32_t *draft_tokens, const int32_t *draft_lens, const das_sampling *sampling,
                               int32_t *accept_len, int32_t *next_token) {
    if (!m || n < 0) return DAS_ERR_INVALID;
    if (n == 0) return DAS_OK;
    if (!seq_ids || !ctx_lens || !draft_lens || !accept_len || !next_token || n > m->cfg.max_seqs) return DAS_ERR_INVALID;
    if (check_sampling(sampling) != DAS_OK || (sampling && !sampling->u_accept)) return DAS_ERR_INVALID;
    if (!unique_ids(n, seq_ids)) return DAS_ERR_INVALID;
    int64_t T = 0, nd = 0, need_pages = 0;
    for (int i = 0; i < n; ++i) {
        if (draft_lens[i] < 0 || draft_lens[i] > m->cfg.max_draft) return DAS_ERR_INVALID;
        T += 1 + draft_lens[i]; nd += draft_lens[i];
    }
    if (T > m->cfg.max_rows || (nd > 0 && !draft_tokens)) return DAS_ERR_INVALID;
    for (int64_t i = 0; i < nd; ++i) if (draft_tokens[i] < 0 || draft_tokens[i] >= m->dm.V) return DAS_ERR_INVALID;
    std::vector<int> slot(n);
    for (int i = 0; i < n; ++i) {
        slot[i] = find_slot(m, seq_ids[i]);
        if (slot[i] < 0) return DAS_ERR_INVALID;
        const Seq &s = m->slots[slot[i]];
        if (s.state != SEQ_COMMITTED || s.ctx != ctx_lens[i]) return DAS_ERR_STATE;
        if (s.ctx + 1 + draft_lens[i] > m->cfg.max_ctx) return DAS_ERR_INVALID;
        need_pages += pages_for(s.ctx + 1 + draft_lens[i]) - (int64_t)s.pages.size();
    }
    if (need_pages > (int64_t)m->free_pages.size()) return DAS_ERR_NOMEM;
    std::vector<int32_t> rows((size_t)T);
    std::vector<PassBlock> blocks(n);
    {
        int r = 0; const int32_t *dp = draft_tokens;
        for (int i = 0; i < n; ++i) {
            const Seq &s = m->slots[slot[i]];
            blocks[i] = {slot[i], s.ctx, 1 + draft_lens[i], rows.data() + r, 2};
            rows[r++] = s.pending;
            for (int j = 0; j < draft_lens[i]; ++j) rows[r++] = *dp++;
        }
    }
    // the pass must fit the staging block and the partial buffers (both sized at load): checked like any other argument
    {
        const int rc0 = check_pass_size(m, pass_size(m, blocks, m->pending_upd.size() / 2 + (size_t)std::max<int64_t>(need_pages, 0),
                                                     sampling ? (size_t)T : 0));
        if (rc0 != DAS_OK) return rc0;
    }

    // ---- state changes start here
    const size_t upd_at_entry = m->pending_upd.size();
    for (int i = 0; i < n; ++i) grow_pages(m, slot[i], m->slots[slot[i]].ctx + 1 + draft_lens[i]);
    PassMeta pm;
    const float *d_ua = nullptr, *d_us = nullptr;
    int rc = run_pass(m, blocks, sampling ? sampling->u_accept : nullptr, sampling ? sampling->u_sample : nullptr, (int)T,
                      sampling ? 1.f / sampling->temperature : 0.f, &pm, &d_ua, &d_us);
    if (rc == DAS_OK) {
        if (sampling) {
            ProfScope ps(m, KC_SAMPLE);
            const int nblk = (m->dm.V + 31) / 32, ldp = m->cfg.max_rows;
            launch_sample(m->stat_part, ldp, m->dm.V, reinterpret_cast<const float2 *>(m->row_stats),
                          reinterpret_cast<const float *>(m->stat_part + (size_t)nblk * ldp), m->xsel, m->wlm, m->dm.d, pm.tok, pm.b_row0,
                          pm.b_n, n, 1.f / sampling->temperature, d_ua, d_us, 0, m->d_accept, m->d_next, m->st);
        } else {
            ProfScope ps(m, KC_ACCEPT);
            launch_accept_greedy(m->d_g, pm.b_row0, pm.b_n, pm.tok, n, m->d_accept, m->d_next, m->st);
        }
        if (hipMemcpyAsync(m->h_out, m->d_accept, n * sizeof(int), hipMemcpyDeviceToHost, m->st) != hipSuccess ||
            hipMemcpyAsync(m->h_out + n, m->d_next, n * sizeof(int), hipMemcpyDeviceToHost, m->st) != hipSuccess)
            rc = DAS_ERR_DEVICE;
    }
    if (hipStreamSynchronize(m->st) != hipSuccess) { g_dev_err = "stream synchronize failed in verify"; rc = DAS_ERR_DEVICE; }
    prof_collect(m);
    if (rc != DAS_OK) {      // give the freshly taken pages back, and forget their page-table updates if they are still queued
        if (m->pending_upd.size() > upd_at_entry) m->pending_upd.resize(upd_at_entry);
        for (int i = n - 1; i >= 0; --i) shrink_pages(m, slot[i], m->slots[slot[i]].ctx);
        return rc;
    }
    for (int i = 0; i < n; ++i) {
        accept_len[i] = m->h_out[i];
        next_token[i] = m->h_out[n + i];
        Seq &s = m->slots[slot[i]];
        s.state = SEQ_SPECULATIVE; s.spec_rows = 1 + draft_lens[i];
    }
    return DAS_OK;
}

extern "C" int das_kv_commit(das_model *m, int32_t n, const int32_t *seq_ids, const int32_t *accept_lens,
                             const int32_t *next_tokens) {
    if (!m || n < 0) return DAS_ERR_INVALID;
    if (n == 0) return DAS_OK;
    if (!seq_ids || !accept_lens || !next_tokens || !unique_ids(n, seq_ids)) return DAS_ERR_INVALID;
    std::vector<int> slot(n);
    for (int i = 0; i < n; ++i) {
        slot[i] = find_slot(m, seq_ids[i]);
        if (slot[i] < 0) return DAS_ERR_INVALID;
        const Seq &s = m->slots[slot[i]];
        if (s.state != SEQ_SPECULATIVE) return DAS_ERR_STATE;
        if (accept_lens[i] < 0 || accept_lens[i] > s.spec_rows - 1 || next_tokens[i] < 0 || next_tokens[i] >= m->dm.V)
            return DAS_ERR_INVALID;
    }
    for (int i = 0; i < n; ++i) {
        Seq &s = m->slots[slot[i]];
        s.ctx += 1 + accept_lens[i];
        s.pending = next_tokens[i];
        s.state = SEQ_COMMITTED; s.spec_rows = 0;
        shrink_pages(m, slot[i], s.ctx);
    }
    return DAS_OK;
}

extern "C" int das_kv_rollback(das_model *m, int32_t n, const int32_t *seq_ids) {
    if (!m || n < 0) return DAS_ERR_INVALID;
    if (n == 0) return DAS_OK;
    if (!seq_ids || !unique_ids(n, seq_ids)) return DAS_ERR_INVALID;
    std::vector<int> slot(n);
    for (int i = 0; i < n; ++i) {
        slot[i] = find_slot(m, seq_ids[i]);
        if (slot[i] < 0) return DAS_ERR_INVALID;
        if (m->slots[slot[i]].state != SEQ_SPECULATIVE) return DAS_ERR_STATE;
    }
    for (int i = 0; i < n; ++i) {
        Seq &s = m->slots[slot[i]];
        s.state = SEQ_COMMITTED; s.spec_rows = 0;
        shrink_pages(m, slot[i], s.ctx);
    }
    return DAS_OK;
}

extern "C" int das_seq_rewind(das_model *m, int32_t n, const int32_t *seq_ids, const int32_t *new_lens,
                              const int32_t *pending_tokens) {
    if (!m || n < 0) return DAS_ERR_INVALID;
    if (n == 0) return DAS_OK;
    if (!seq_ids || !new_lens || !pending_tokens || !unique_ids(n, seq_ids)) return DAS_ERR_INVALID;
    std::vector<int> slot(n);
    for (int i = 0; i < n; ++i) {
        slot[i] = find_slot(m, seq_ids[i]);
        if (slot[i] < 0) return DAS_ERR_INVALID;
        const Seq &s = m->slots[slot[i]];
        if (s.state != SEQ_COMMITTED) return DAS_ERR_STATE;
        if (new_lens[i] < 0 || new_lens[i] > s.ctx || pending_tokens[i] < 0 || pending_tokens[i] >= m->dm.V) return DAS_ERR_INVALID;
    }
    for (int i = 0; i < n; ++i) {
        Seq &s = m->slots[slot[i]];
        s.ctx = new_lens[i]; s.pending = pending_tokens[i];
        shrink_pages(m, slot[i], s.ctx);
    }
    return DAS_OK;
}

extern "C" int das_seq_free(das_model *m, int32_t n, const int32_t *seq_ids) {
    if (!m || n < 0) return DAS_ERR_INVALID;
    if (n == 0) return DAS_OK;
    if (!seq_ids || !unique_ids(n, seq_ids)) return DAS_ERR_INVALID;
    for (int i = 0; i < n; ++i) if (find_slot(m, seq_ids[i]) < 0) return DAS_ERR_INVALID;
    for (int i = 0; i < n; ++i) {
        drop_seq(m, find_slot(m, seq_ids[i]));
    }
    return DAS_OK;
}

// ------------------------------------------------------------------------------------------------ state injection

extern "C" int das_seq_create(das_model *m, int32_t seq_id, int32_t ctx_len, int32_t pending_token) {
    if (!m || ctx_len < 0 || ctx_len >= m->cfg.max_ctx || pending_token < 0 || pending_token >= m->dm.V) return DAS_ERR_INVALID;
    if (find_slot(m, seq_id) >= 0) return DAS_ERR_STATE;
    if (m->free_slots.empty() || pages_for(ctx_len) > (int)m->free_pages.size()) return DAS_ERR_NOMEM;
    int slot = new_seq(m, seq_id);
    grow_pages(m, slot, ctx_len);
    Seq &s = m->slots[slot];
    s.ctx = ctx_len; s.pending = pending_token;
    int rc = upload_page_row(m, slot);
    if (rc != DAS_OK) drop_seq(m, slot);
    return rc;
}

static int kv_io(das_model *m, int mode, int32_t seq_id, int32_t layer, int32_t first_pos, int32_t n_pos, uint16_t *k, uint16_t *v) {
    if (!m || !k || !v || layer < 0 || layer >= m->dm.L || first_pos < 0 || n_pos < 0) return DAS_ERR_INVALID;
    int slot = find_slot(m, seq_id);
    if (slot < 0) return DAS_ERR_INVALID;
    Seq &s = m->slots[slot];
    if (first_pos + n_pos > (int)s.pages.size() * DAS_PAGE) return DAS_ERR_INVALID;
    if (n_pos == 0) return DAS_OK;
    const size_t cnt = (size_t)n_pos * m->dm.Hkv * m->dm.D;
    bf16_t *dk = nullptr, *dv = nullptr;
    HIPCHK(hipStreamSynchronize(m->st));
    if (hipMalloc((void **)&dk, cnt * 2) != hipSuccess) { (void)hipGetLastError(); return DAS_ERR_NOMEM; }
    if (hipMalloc((void **)&dv, cnt * 2) != hipSuccess) { (void)hipGetLastError(); (void)hipFree(dk); return DAS_ERR_NOMEM; }
    int rc = DAS_OK;
    f16_t *kl = m->kpool + (size_t)layer * m->layer_elems, *vl = m->vpool + (size_t)layer * m->layer_elems;
    const int *prow = m->page_table + (size_t)slot * m->max_pages;
    auto fail = [&](hipError_t e) { if (e != hipSuccess) { g_dev_err = hipGetErrorString(e); rc = DAS_ERR_DEVICE; } return e != hipSuccess; };
    do {
        if (mode == 0) {
            if (fail(hipMemcpy(dk, k, cnt * 2, hipMemcpyHostToDevice))) break;
            if (fail(hipMemcpy(dv, v, cnt * 2, hipMemcpyHostToDevice))) break;
        }
        { ProfScope ps(m, KC_KVIO); launch_kv_io(mode, prow, first_pos, n_pos, kl, vl, dk, dv, m->dm.Hkv, m->dm.D, (int)m->cfg.num_pages, m->d_kv_sat, m->st); }
        if (fail(hipStreamSynchronize(m->st))) break;
        if (mode == 1) {
            if (fail(hipMemcpy(k, dk, cnt * 2, hipMemcpyDeviceToHost))) break;
            if (fail(hipMemcpy(v, dv, cnt * 2, hipMemcpyDeviceToHost))) break;
        }
    } while (0);
    prof_collect(m);
    (void)hipFree(dk); (void)hipFree(dv);
    return rc;
}

extern "C" int das_kv_import(das_model *m, int32_t seq_id, int32_t layer, int32_t first_pos, int32_t n_pos,
                             const uint16_t *k, const uint16_t *v) {
    return kv_io(m, 0, seq_id, layer, first_pos, n_pos, const_cast<uint16_t *>(k), const_cast<uint16_t *>(v));
}
extern "C" int das_kv_export(das_model *m, int32_t seq_id, int32_t layer, int32_t first_pos, int32_t n_pos,
                             uint16_t *k, uint16_t *v) {
    return kv_io(m, 1, seq_id, layer, first_pos, n_pos, k, v);
}

extern "C" int das_kv_synth(das_model *m, int32_t seq_id, uint64_t seed, uint64_t seq_key) {
    if (!m) return DAS_ERR_INVALID;
    int slot = find_slot(m, seq_id);
    if (slot < 0) return DAS_ERR_INVALID;
    Seq &s = m->slots[slot];
    if (s.state != SEQ_COMMITTED) return DAS_ERR_STATE;
    const int *prow = m->page_table + (size_t)slot * m->max_pages;
    {
        ProfScope ps(m, KC_KVIO);
        for (int l = 0; l < m->dm.L; ++l)
            launch_kv_synth(prow, s.ctx, m->kpool + (size_t)l * m->layer_elems, m->vpool + (size_t)l * m->layer_elems,
                            m->dm.Hkv, m->dm.D, (int)m->cfg.num_pages, seed, seq_key, l, m->st);
    }
    HIPCHK(hipStreamSynchronize(m->st));
    prof_collect(m);
    return DAS_OK;
}

// ------------------------------------------------------------------------------------------------ inspection

extern "C" int das_debug_num_rows(das_model *m, int32_t *n_rows) {
    if (!m || !n_rows) return DAS_ERR_INVALID;
    *n_rows = m->last_rows;
    return DAS_OK;
}
extern "C" int das_debug_logits(das_model *m, int32_t first_row, int32_t n_rows, float *out) {
    if (!m || !out || first_row < 0 || n_rows < 0 || first_row + n_rows > m->last_rows) return DAS_ERR_INVALID;
    if (n_rows == 0) return DAS_OK;
    if (!m->last_has_logits) return DAS_ERR_STATE;      // the last pass gathered its row maxima inside the GEMM
    HIPCHK(hipStreamSynchronize(m->st));
    HIPCHK(hipMemcpy(out, m->logits + (size_t)first_row * m->dm.V, (size_t)n_rows * m->dm.V * sizeof(float), hipMemcpyDeviceToHost));
    return DAS_OK;
}
extern "C" int das_debug_keep_logits(das_model *m, int32_t on) {
    if (!m) return DAS_ERR_INVALID;
    m->keep_logits = on != 0;
    return DAS_OK;
}
extern "C" int das_debug_row_argmax(das_model *m, int32_t *out) {
    if (!m || !out) return DAS_ERR_INVALID;
    if (m->last_rows == 0) return DAS_OK;
    if (!m->last_has_argmax) return DAS_ERR_STATE;      // a sampling pass outside inspection mode does not compute it
    HIPCHK(hipStreamSynchronize(m->st));
    HIPCHK(hipMemcpy(out, m->d_g, (size_t)m->last_rows * sizeof(int), hipMemcpyDeviceToHost));
    return DAS_OK;
}
extern "C" int das_debug_seq(das_model *m, int32_t seq_id, int32_t *ctx_len, int32_t *pending, int32_t *state,
                             int32_t *pages, int32_t *n_pages) {
    if (!m) return DAS_ERR_INVALID;
    int slot = find_slot(m, seq_id);
    if (slot < 0) return DAS_ERR_INVALID;
    const Seq &s = m->slots[slot];
    if (ctx_len) *ctx_len = s.ctx;
    if (pending) *pending = s.pending;
    if (state) *state = s.state;
    if (n_pages) *n_pages = (int)s.pages.size();
    if (pages) std::copy(s.pages.begin(), s.pages.end(), pages);
    return DAS_OK;
}
extern "C" int das_debug_kv_saturated(das_model *m, int64_t *count) {
    if (!m || !count) return DAS_ERR_INVALID;
    unsigned long long c = 0;
    HIPCHK(hipStreamSynchronize(m->st));
    HIPCHK(hipMemcpy(&c, m->d_kv_sat, sizeof(c), hipMemcpyDeviceToHost));
    *count = (int64_t)c;
    return DAS_OK;
}
extern "C" int das_debug_free_pages(das_model *m, int64_t *n_free) {
    if (!m || !n_free) return DAS_ERR_INVALID;
    *n_free = (int64_t)m->free_pages.size();
    return DAS_OK;
}

// Stand-alone check of the MFMA GEMM: C[M][N] = A[M][K] * W[N][K]^T from row-major bf16 host inputs.
extern "C" int das_debug_gemm(int32_t M, int32_t N, int32_t K, const uint16_t *a, const uint16_t *w, float *c) {
    if (M < 1 || N < 1 || K < 8 || (K % 8) || !a || !w || !c) return DAS_ERR_INVALID;
    const int Mp = round_up(M, 256) + 256, Np = round_up(N, 256), Kp = round_up(K, 64);
    bf16_t *da = nullptr, *dw = nullptr, *pa = nullptr, *pw = nullptr;
    float *dc = nullptr, *dws = nullptr;
    int rc = DAS_OK;
    auto bad = [&](hipError_t e) { if (e != hipSuccess) { g_dev_err = hipGetErrorString(e); rc = DAS_ERR_DEVICE; } return e != hipSuccess; };
    do {
        if (bad(hipMalloc((void **)&da, (size_t)M * K * 2)) || bad(hipMalloc((void **)&dw, (size_t)N * K * 2)) ||
            bad(hipMalloc((void **)&pa, (size_t)Mp * Kp * 2)) || bad(hipMalloc((void **)&pw, (size_t)Np * Kp * 2)) ||
            bad(hipMalloc((void **)&dc, (size_t)M * N * 4))) break;
        const size_t ws_floats = gemm_ws_floats_needed(M, N, Kp);
        if (ws_floats && bad(hipMalloc((void **)&dws, ws_floats * 4))) break;
        if (bad(hipMemcpy(da, a, (size_t)M * K * 2, hipMemcpyHostToDevice)) || bad(hipMemcpy(dw, w, (size_t)N * K * 2, hipMemcpyHostToDevice))) break;
        launch_pack_weight(da, pa, M, K, Mp, Kp, nullptr);
        launch_pack_weight(dw, pw, N, K, Np, Kp, nullptr);
        launch_gemm(EPI_F32_ROWMAJOR, pa, pw, dc, M, N, Kp, N, nullptr, dws, ws_floats);
        if (bad(hipDeviceSynchronize())) break;
        if (bad(hipMemcpy(c, dc, (size_t)M * N * 4, hipMemcpyDeviceToHost))) break;
    } while (0);
    (void)hipFree(da); (void)hipFree(dw); (void)hipFree(pa); (void)hipFree(pw); (void)hipFree(dc); (void)hipFree(dws);
    return rc;
}

// ------------------------------------------------------------------------------------------------ no-allocation GEMM
// das_debug_gemm for callers that cannot allocate: operands and result are DEVICE pointers, and everything the kernels
// need beyond them (both operands repacked into fragment order, the K-slice partial sums) lives in one file-scope
// device array.  Each GPU holds its own copy of the array at its own address; the address is asked for once per
// device and only that pointer, never the array's name, is handed to kernels.
#define DAS_NOALLOC_MAX_M 256
#define DAS_NOALLOC_MAX_N 2048
#define DAS_NOALLOC_MAX_K 2048
#define DAS_NOALLOC_PA_BYTES ((size_t)(DAS_NOALLOC_MAX_M + 256) * DAS_NOALLOC_MAX_K * 2)                 /* 2 MiB */
#define DAS_NOALLOC_PW_BYTES ((size_t)DAS_NOALLOC_MAX_N * DAS_NOALLOC_MAX_K * 2)                         /* 8 MiB */
#define DAS_NOALLOC_WS_BYTES ((size_t)2 * DAS_NOALLOC_MAX_M * DAS_NOALLOC_MAX_N * 4)                     /* 4 MiB: at most two K slices */
static __device__ __align__(256) unsigned char scratch[DAS_NOALLOC_PA_BYTES + DAS_NOALLOC_PW_BYTES + DAS_NOALLOC_WS_BYTES];
#define DAS_NOALLOC_MAX_DEVICES 64
static unsigned char *g_scratch_ptr[DAS_NOALLOC_MAX_DEVICES];      // device address of `scratch` on each GPU, filled on first use

extern "C" int das_gemm_noalloc(int32_t M, int32_t N, int32_t K, const uint16_t *a_dev, const uint16_t *w_dev, float *c_dev,
                                void *hip_stream) {
    if (M < 1 || N < 1 || K < 8 || (K % 8) || !a_dev || !w_dev || !c_dev) return DAS_ERR_INVALID;
    if (M > DAS_NOALLOC_MAX_M || N > DAS_NOALLOC_MAX_N || K > DAS_NOALLOC_MAX_K) {
        g_dev_err = "das_gemm_noalloc: at most 256 x 2048 x 2048 (M x N x K); larger products need das_debug_gemm";
        return DAS_ERR_INVALID;
    }
    int dev = -1;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= DAS_NOALLOC_MAX_DEVICES) { g_dev_err = "das_gemm_noalloc: device index out of range"; return DAS_ERR_DEVICE; }
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIPCHK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) { g_dev_err = "das_gemm_noalloc: no device address for the scratch array"; return DAS_ERR_DEVICE; }
        g_scratch_ptr[dev] = reinterpret_cast<unsigned char *>(p);
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    const int Mp = round_up(M, 256) + 256, Np = round_up(N, 256), Kp = round_up(K, 64);
    unsigned char *base = g_scratch_ptr[dev];
    bf16_t *pa = reinterpret_cast<bf16_t *>(base);
    bf16_t *pw = reinterpret_cast<bf16_t *>(base + DAS_NOALLOC_PA_BYTES);
    float *ws = reinterpret_cast<float *>(base + DAS_NOALLOC_PA_BYTES + DAS_NOALLOC_PW_BYTES);
    int slice_tiles = 0;
    const int slices = gemm_slices(Kp, &slice_tiles);
    const size_t ws_floats = (size_t)slices * M * N;
    if ((size_t)Mp * Kp * 2 > DAS_NOALLOC_PA_BYTES || (size_t)Np * Kp * 2 > DAS_NOALLOC_PW_BYTES || ws_floats * 4 > DAS_NOALLOC_WS_BYTES)
        return DAS_ERR_INVALID;      // (cannot happen inside the limits above)
    // the repacking kernels write every 16-byte slot of their padded outputs, zeros included, and the GEMM writes every
    // partial it later reads: nothing of the previous call's contents survives where it could be read
    launch_pack_weight(a_dev, pa, M, K, Mp, Kp, st);
    launch_pack_weight(w_dev, pw, N, K, Np, Kp, st);
    launch_gemm(EPI_F32_ROWMAJOR, pa, pw, c_dev, M, N, Kp, N, st, ws, ws_floats);
    hipError_t le = hipGetLastError();
    if (le != hipSuccess) { g_dev_err = std::string("das_gemm_noalloc launch: ") + hipGetErrorString(le); return DAS_ERR_DEVICE; }
    return DAS_OK;
}

// Stand-alone check of the GEMM's other two epilogues, from row-major bf16 host inputs:
//   act[M][F] = silu(a wg^T) * (a wu^T), rounded to bf16 as the kernel writes it, returned as fp32 (wg, wu: [F][K]);
//   col[M]    = lowest column of the row maximum of a w^T (w: [N][K], N >= 16384: the fused LM head).
// Either output may be NULL with its inputs.  K % 64 == 0.
extern "C" int das_debug_gemm_epilogues(int32_t M, int32_t K, const uint16_t *a, int32_t F, const uint16_t *wg, const uint16_t *wu,
                                        float *act, int32_t N, const uint16_t *w, int32_t *col) {
    const bool do_silu = F > 0 && wg && wu && act, do_max = N > 0 && w && col;
    if (M < 1 || K < 64 || (K % 64) || !a || (!do_silu && !do_max) || (do_silu && (F % 8)) || (do_max && N < 16384)) return DAS_ERR_INVALID;
    const int Mp = round_up(M, 256) + 256, Fp = do_silu ? round_up(F, 64) : 0, gup = round_up(2 * Fp, 256), Np = round_up(std::max(N, 1), 256);
    bf16_t *da = nullptr, *pa = nullptr, *dw = nullptr, *pw = nullptr, *dact = nullptr;
    unsigned long long *keys = nullptr;
    int *dcol = nullptr;
    int rc = DAS_OK;
    auto bad = [&](hipError_t e) { if (e != hipSuccess) { g_dev_err = hipGetErrorString(e); rc = DAS_ERR_DEVICE; } return e != hipSuccess; };
    do {
        if (bad(hipMalloc((void **)&da, (size_t)M * K * 2)) || bad(hipMalloc((void **)&pa, (size_t)Mp * K * 2))) break;
        if (bad(hipMemcpy(da, a, (size_t)M * K * 2, hipMemcpyHostToDevice))) break;
        launch_pack_weight(da, pa, M, K, Mp, K, nullptr);
        if (do_silu) {
            if (bad(hipMalloc((void **)&dw, (size_t)2 * F * K * 2)) || bad(hipMalloc((void **)&pw, (size_t)gup * K * 2)) ||
                bad(hipMalloc((void **)&dact, (size_t)Mp * Fp * 2))) break;
            if (bad(hipMemcpy(dw, wg, (size_t)F * K * 2, hipMemcpyHostToDevice)) ||
                bad(hipMemcpy(dw + (size_t)F * K, wu, (size_t)F * K * 2, hipMemcpyHostToDevice))) break;
            if (bad(hipMemset(pw, 0, (size_t)gup * K * 2)) || bad(hipMemset(dact, 0, (size_t)Mp * Fp * 2))) break;
            launch_pack_gateup(dw, dw + (size_t)F * K, pw, F, K, Fp, nullptr);
            launch_gemm(EPI_SILU_FRAG, pa, pw, dact, M, 2 * Fp, K, Fp, nullptr, nullptr, 0);
            if (bad(hipDeviceSynchronize())) break;
            std::vector<bf16_t> h((size_t)Mp * Fp);
            if (bad(hipMemcpy(h.data(), dact, h.size() * 2, hipMemcpyDeviceToHost))) break;
            for (int r = 0; r < M; ++r)
                for (int f = 0; f < F; ++f) {
                    const uint32_t u = (uint32_t)h[frag_off(r, f, Fp)] << 16;
                    float v; std::memcpy(&v, &u, 4);
                    act[(size_t)r * F + f] = v;
                }
            (void)hipFree(dw); (void)hipFree(pw); dw = pw = nullptr;
        }
        if (do_max) {
            if (bad(hipMalloc((void **)&dw, (size_t)N * K * 2)) || bad(hipMalloc((void **)&pw, (size_t)Np * K * 2)) ||
                bad(hipMalloc((void **)&keys, (size_t)M * 8)) || bad(hipMalloc((void **)&dcol, (size_t)M * 4))) break;
            if (bad(hipMemcpy(dw, w, (size_t)N * K * 2, hipMemcpyHostToDevice))) break;
            launch_pack_weight(dw, pw, N, K, Np, K, nullptr);
            launch_rowmax_keys_clear(keys, M, nullptr);
            launch_gemm(EPI_ROWMAX, pa, pw, keys, M, N, K, N, nullptr, nullptr, 0);
            launch_rowmax_keys_decode(keys, M, dcol, nullptr);
            if (bad(hipDeviceSynchronize())) break;
            if (bad(hipMemcpy(col, dcol, (size_t)M * 4, hipMemcpyDeviceToHost))) break;
        }
    } while (0);
    (void)hipFree(da); (void)hipFree(pa); (void)hipFree(dw); (void)hipFree(pw); (void)hipFree(dact); (void)hipFree(keys); (void)hipFree(dcol);
    return rc;
}

// Device time of one projection GEMM shape with the launch configuration a pass would use (see das.h).
extern "C" int das_debug_gemm_time(int32_t epi, int32_t M, int32_t N, int32_t K, int32_t iters, int32_t weight_sets, int32_t copies_only,
                                   double *us_per_launch) {
    if (M < 1 || N < 32 || K < 64 || (K % 64) || iters < 1 || weight_sets < 1 || weight_sets > 64 || !us_per_launch ||
        (epi != EPI_RESID_F32 && epi != EPI_SILU_FRAG && epi != EPI_F32_ROWMAJOR && epi != EPI_ROWMAX) ||
        (epi == EPI_SILU_FRAG && (N % 128)) || (epi == EPI_ROWMAX && N < 16384) || (epi != EPI_SILU_FRAG && epi != EPI_ROWMAX && (N % 4)))
        return DAS_ERR_INVALID;
    const size_t Mp = (size_t)round_up(M, 256) + 256, Np = (size_t)round_up(N, 256);
    const int Fp = N / 2;      // gate/up: N counts gate and up rows together (multiple of 128, so no padding of the FFN width)
    bf16_t *a = nullptr, *w = nullptr, *g = nullptr, *y = nullptr;
    float *c = nullptr, *ws = nullptr;
    unsigned long long *keys = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = DAS_OK;
    auto bad = [&](hipError_t e) { if (e != hipSuccess) { g_dev_err = hipGetErrorString(e); rc = DAS_ERR_DEVICE; } return e != hipSuccess; };
    do {
        const size_t ws_floats = std::max<size_t>(gemm_ws_floats_needed(M, N, K), 4);
        const size_t c_elems = epi == EPI_SILU_FRAG ? Mp * Fp / 2 + 1 : epi == EPI_ROWMAX ? 1 : (size_t)M * N;
        if (bad(hipMalloc((void **)&a, Mp * K * 2)) || bad(hipMalloc((void **)&w, Np * K * 2 * weight_sets)) ||
            bad(hipMalloc((void **)&c, c_elems * 4)) || bad(hipMalloc((void **)&ws, ws_floats * 4)) ||
            bad(hipMalloc((void **)&g, (size_t)N * 2)) || bad(hipMalloc((void **)&y, Mp * N * 2)) ||
            bad(hipMalloc((void **)&keys, (size_t)M * 8)) || bad(hipEventCreate(&e0)) || bad(hipEventCreate(&e1))) break;
        // operands are filled directly in fragment order: the values are i.i.d., so the order is immaterial
        launch_fill_normal(a, Mp * K, 1, 0, 1.0, nullptr);
        launch_fill_normal(w, Np * K * weight_sets, 1, 1, 0.02, nullptr);
        launch_fill_const(g, (size_t)N, (bf16_t)0x3F80, nullptr);
        if (bad(hipMemset(c, 0, c_elems * 4))) break;
        const GemmNormTail tail = {g, y, 1e-6f};
        auto once = [&](int it) {
            const bf16_t *wi = w + (size_t)(it % weight_sets) * Np * K;
            if (epi == EPI_ROWMAX) {
                launch_rowmax_keys_clear(keys, M, nullptr);
                launch_gemm(EPI_ROWMAX, a, wi, keys, M, N, K, N, nullptr, ws, ws_floats);
            } else if (epi == EPI_SILU_FRAG) launch_gemm(EPI_SILU_FRAG, a, wi, c, M, N, K, Fp, nullptr, ws, ws_floats);
            else if (epi == EPI_RESID_F32) launch_gemm(EPI_RESID_F32, a, wi, c, M, N, K, N, nullptr, ws, ws_floats, (N % 64) == 0 && N <= 8192 ? &tail : nullptr);
            else { int left = 1; launch_gemm(EPI_F32_ROWMAJOR, a, wi, c, M, N, K, N, nullptr, ws, ws_floats, nullptr, &left); }
        };
        gemm_debug_copies_only(copies_only != 0);
        once(0); once(1);
        if (bad(hipDeviceSynchronize())) { gemm_debug_copies_only(false); break; }
        if (bad(hipEventRecord(e0, nullptr))) { gemm_debug_copies_only(false); break; }
        for (int it = 0; it < iters; ++it) once(it + 2);
        gemm_debug_copies_only(false);
        if (bad(hipEventRecord(e1, nullptr)) || bad(hipEventSynchronize(e1))) break;
        float ms = 0.f;
        if (bad(hipEventElapsedTime(&ms, e0, e1))) break;
        if (bad(hipGetLastError())) break;
        *us_per_launch = (double)ms * 1e3 / iters;
    } while (0);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(a); (void)hipFree(w); (void)hipFree(c); (void)hipFree(ws); (void)hipFree(g); (void)hipFree(y); (void)hipFree(keys);
    return rc;
}

// Plain device-to-device copy of `bytes` (multiple of 16) with a trivial kernel: the known-traffic
// reference that scales the profiler's HBM byte counters.
extern "C" int das_debug_copy(int64_t bytes, int32_t repeats) {
    if (bytes < 16 || (bytes % 16) || repeats < 1) return DAS_ERR_INVALID;
    void *a = nullptr, *b = nullptr;
    if (hipMalloc(&a, (size_t)bytes) != hipSuccess) { (void)hipGetLastError(); return DAS_ERR_NOMEM; }
    if (hipMalloc(&b, (size_t)bytes) != hipSuccess) { (void)hipGetLastError(); (void)hipFree(a); return DAS_ERR_NOMEM; }
    int rc = DAS_OK;
    if (hipMemset(a, 1, (size_t)bytes) != hipSuccess) rc = DAS_ERR_DEVICE;
    for (int r = 0; r < repeats && rc == DAS_OK; ++r) launch_copy(a, b, (size_t)bytes, nullptr);
    if (hipDeviceSynchronize() != hipSuccess) rc = DAS_ERR_DEVICE;
    (void)hipFree(a); (void)hipFree(b);
    return rc;
}

// The copy ring of the kernels with nothing else in it (see k_probe.hip): time of one launch, best of three after a warm-up
// launch, each over a part of the private buffer that no earlier launch has touched.
extern "C" int das_debug_copy_ring(int32_t workgroups, int32_t stages, int32_t copies, int32_t shared_copies, int32_t tiles,
                                   int32_t non_temporal, double *us, double *bytes_into_lds) {
    if (workgroups < 1 || workgroups > 1024 || tiles < 1 || tiles > 4096 || shared_copies < 0 || shared_copies > copies ||
        !copy_ring_supported(stages, copies, shared_copies) || !us || !bytes_into_lds) return DAS_ERR_INVALID;
    const int reps = 4;
    const size_t per_launch = (size_t)workgroups * tiles * 4 * (copies - shared_copies) * 1024;      // private bytes of one launch
    const size_t shared_bytes = (size_t)64 * 4 * std::max(shared_copies, 1) * 1024;
    if (per_launch * reps > ((size_t)16 << 30)) return DAS_ERR_INVALID;
    void *priv = nullptr, *sh = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = DAS_OK;
    auto bad = [&](hipError_t e) { if (e != hipSuccess) { g_dev_err = hipGetErrorString(e); rc = DAS_ERR_DEVICE; } return e != hipSuccess; };
    do {
        if (bad(hipMalloc(&priv, std::max<size_t>(per_launch * reps, 1024))) || bad(hipMalloc(&sh, shared_bytes)) ||
            bad(hipMemset(priv, 1, std::max<size_t>(per_launch * reps, 1024))) || bad(hipMemset(sh, 1, shared_bytes)) ||
            bad(hipEventCreate(&e0)) || bad(hipEventCreate(&e1)) || bad(hipDeviceSynchronize())) break;
        float best = 0.f;
        for (int r = 0; r < reps && rc == DAS_OK; ++r) {
            const unsigned char *p = reinterpret_cast<const unsigned char *>(priv) + (size_t)r * per_launch;
            if (bad(hipEventRecord(e0, nullptr)) || bad(launch_copy_ring(p, sh, workgroups, stages, copies, shared_copies, tiles, non_temporal != 0, nullptr)) ||
                bad(hipEventRecord(e1, nullptr)) || bad(hipEventSynchronize(e1))) break;
            float ms = 0.f;
            if (bad(hipEventElapsedTime(&ms, e0, e1))) break;
            if (r >= 1 && (best == 0.f || ms < best)) best = ms;
        }
        *us = (double)best * 1e3;
        *bytes_into_lds = (double)workgroups * tiles * 4 * copies * 1024;
    } while (0);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(priv); (void)hipFree(sh);
    return rc;
}


// The matrix-pipe probe of k_probe.hip: best of three launches after a warm-up.
extern "C" int das_debug_mfma_loop(int32_t mode, int32_t iters, double *ns_per_mfma, double *shader_ghz, double *pflops) {
    if (mode < 0 || mode > 2 || iters < 1 || iters > 100000 || !ns_per_mfma || !shader_ghz || !pflops) return DAS_ERR_INVALID;
    const size_t src_bytes = (size_t)256 * 128 * 1024;
    void *src = nullptr, *aux = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = DAS_OK;
    auto bad = [&](hipError_t e) { if (e != hipSuccess) { g_dev_err = hipGetErrorString(e); rc = DAS_ERR_DEVICE; } return e != hipSuccess; };
    do {
        if (bad(hipMalloc(&src, src_bytes)) || bad(hipMalloc(&aux, 256)) || bad(hipMemset(src, 1, src_bytes)) || bad(hipMemset(aux, 0, 256)) ||
            bad(hipEventCreate(&e0)) || bad(hipEventCreate(&e1)) || bad(hipDeviceSynchronize())) break;
        float *sink = reinterpret_cast<float *>(aux);
        long long *clk = reinterpret_cast<long long *>(reinterpret_cast<unsigned char *>(aux) + 64);
        float best = 0.f;
        long long best_clk[2] = {0, 0};
        for (int r = 0; r < 4 && rc == DAS_OK; ++r) {
            if (bad(hipEventRecord(e0, nullptr)) || bad(launch_mfma_loop(mode, src, sink, iters, clk, nullptr)) ||
                bad(hipEventRecord(e1, nullptr)) || bad(hipEventSynchronize(e1))) break;
            float ms = 0.f;
            long long c[2];
            if (bad(hipEventElapsedTime(&ms, e0, e1)) || bad(hipMemcpy(c, clk, sizeof c, hipMemcpyDeviceToHost))) break;
            if (r >= 1 && (best == 0.f || ms < best)) { best = ms; best_clk[0] = c[0]; best_clk[1] = c[1]; }
        }
        if (rc != DAS_OK) break;
        const double mfmas_per_wave = (double)iters * 32.0;                       // 2 k-steps x 16 per iteration
        const double loop_ns = (double)best_clk[1] * 10.0;                        // 100 MHz ticks
        *ns_per_mfma = loop_ns / mfmas_per_wave;
        *shader_ghz = loop_ns > 0 ? (double)best_clk[0] / loop_ns : 0.0;
        // 256 CUs x 4 SIMDs, 32 x 32 x 16 x 2 flop per MFMA, over the launch's own duration (events)
        *pflops = 256.0 * 4.0 * mfmas_per_wave * 32768.0 / ((double)best * 1e-3) / 1e15;
    } while (0);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(src); (void)hipFree(aux);
    return rc;
}

// ------------------------------------------------------------------------------------------------ profiling / errors

extern "C" int das_profile_enable(das_model *m, int32_t on) {
    if (!m) return DAS_ERR_INVALID;
    m->prof = on != 0;
    return DAS_OK;
}
extern "C" int das_profile_reset(das_model *m) {
    if (!m) return DAS_ERR_INVALID;
    for (int i = 0; i < KC_COUNT; ++i) { m->prof_ms[i] = 0; m->prof_n[i] = 0; }
    return DAS_OK;
}
extern "C" int das_profile_read(das_model *m, int32_t kernel_class, double *ms, int64_t *launches) {
    if (!m || kernel_class < 0 || kernel_class >= KC_COUNT) return DAS_ERR_INVALID;
    if (ms) *ms = m->prof_ms[kernel_class];
    if (launches) *launches = m->prof_n[kernel_class];
    return DAS_OK;
}
extern "C" const char *das_profile_name(int32_t kernel_class) {
    return (kernel_class >= 0 && kernel_class < KC_COUNT) ? kClassNames[kernel_class] : nullptr;
}
extern "C" const char *das_strerror(int code) {
    switch (code) {
    case DAS_OK: return "ok";
    case DAS_ERR_INVALID: return "invalid argument";
    case DAS_ERR_STATE: return "call not allowed in this sequence state";
    case DAS_ERR_NOMEM: return "out of pages, sequence slots or memory";
    case DAS_ERR_DEVICE: return "HIP call failed";
    default: return "unknown error";
    }
}
extern "C" const char *das_last_device_error(void) { return g_dev_err.c_str(); }
