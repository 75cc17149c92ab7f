// Element-wise and data-movement kernels of the verify step: weight repacking,
// embedding gather, RMSNorm, RoPE + paged KV write, KV import/export.
#include "das_internal.h"
#include <algorithm>

__device__ __forceinline__ float bf2f(bf16_t x) { return __uint_as_float((uint32_t)x << 16); }
__device__ __forceinline__ bf16_t f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);      // round to nearest even
    return (bf16_t)(u >> 16);
}

// ---------------------------------------------------------------- weight repacking (load time)
// dst: fragment order [Np/32][Kp/16][64][8]; src row-major [N][K]; zero padding.
__global__ void pack_weight_kernel(const bf16_t *__restrict__ src, bf16_t *__restrict__ dst, int N, int K, int Np, int Kp) {
    size_t slot = (size_t)blockIdx.x * blockDim.x + threadIdx.x;        // one 16-byte lane slot
    size_t total = (size_t)Np * Kp / 8;
    if (slot >= total) return;
    int lane = (int)(slot & 63);
    size_t frag = slot >> 6;
    int kfr = Kp >> 4;
    int rb = (int)(frag / kfr), ks = (int)(frag % kfr);
    int row = rb * 32 + (lane & 31), k0 = ks * 16 + 8 * (lane >> 5);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row < N) {
        if (k0 + 8 <= K && (K & 7) == 0) {
            v = *reinterpret_cast<const uint4 *>(src + (size_t)row * K + k0);
        } else {
            bf16_t t[8];
            for (int e = 0; e < 8; ++e) t[e] = (k0 + e < K) ? src[(size_t)row * K + k0 + e] : (bf16_t)0;
            v = *reinterpret_cast<uint4 *>(t);
        }
    }
    reinterpret_cast<uint4 *>(dst)[slot] = v;
}

// gate and up projections interleaved in groups of 32 output features:
// packed row n' = b*64 + r  ->  r < 32 ? Wg[b*32 + r] : Wu[b*32 + r - 32]
__global__ void pack_gateup_kernel(const bf16_t *__restrict__ wg, const bf16_t *__restrict__ wu, bf16_t *__restrict__ dst,
                                   int F, int K, int Fp) {
    size_t slot = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)2 * Fp * K / 8;
    if (slot >= total) return;
    int lane = (int)(slot & 63);
    size_t frag = slot >> 6;
    int kfr = K >> 4;
    int rb = (int)(frag / kfr), ks = (int)(frag % kfr);
    int row = rb * 32 + (lane & 31), k0 = ks * 16 + 8 * (lane >> 5);
    int b = row >> 6, r = row & 63;
    int feat = b * 32 + (r & 31);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (feat < F) v = *reinterpret_cast<const uint4 *>((r < 32 ? wg : wu) + (size_t)feat * K + k0);
    reinterpret_cast<uint4 *>(dst)[slot] = v;
}

void launch_pack_weight(const bf16_t *src, bf16_t *dst, int N, int K, int Np, int Kp, hipStream_t st) {
    size_t total = (size_t)Np * Kp / 8;
    pack_weight_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(src, dst, N, K, Np, Kp);
}
void launch_pack_gateup(const bf16_t *wg, const bf16_t *wu, bf16_t *dst, int F, int K, int Fp, hipStream_t st) {
    size_t total = (size_t)2 * Fp * K / 8;
    pack_gateup_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(wg, wu, dst, F, K, Fp);
}

// ---------------------------------------------------------------- page-table updates
__global__ void pt_update_kernel(int *page_table, const int *upd, int n) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) page_table[upd[2 * i]] = upd[2 * i + 1];
}
void launch_pt_update(int *page_table, const int *upd, int n_upd, hipStream_t st) {
    if (n_upd > 0) pt_update_kernel<<<dim3((n_upd + 255) / 256), dim3(256), 0, st>>>(page_table, upd, n_upd);
}

// ---------------------------------------------------------------- embedding gather: h[r] = E[tok[r]]
__global__ void embed_kernel(const int *__restrict__ tok, const bf16_t *__restrict__ E, float *__restrict__ h, int d) {
    int r = blockIdx.x;
    const bf16_t *src = E + (size_t)tok[r] * d;
    float *dst = h + (size_t)r * d;
    for (int c = threadIdx.x; c < d / 8; c += blockDim.x) {
        uint4 v = reinterpret_cast<const uint4 *>(src)[c];
        const bf16_t *e = reinterpret_cast<const bf16_t *>(&v);
        float4 a = make_float4(bf2f(e[0]), bf2f(e[1]), bf2f(e[2]), bf2f(e[3]));
        float4 b = make_float4(bf2f(e[4]), bf2f(e[5]), bf2f(e[6]), bf2f(e[7]));
        reinterpret_cast<float4 *>(dst)[2 * c] = a;
        reinterpret_cast<float4 *>(dst)[2 * c + 1] = b;
    }
}
void launch_embed(const PassMeta &pm, const bf16_t *E, float *h, int d, hipStream_t st) {
    embed_kernel<<<dim3(pm.T), dim3(256), 0, st>>>(pm.tok, E, h, d);
}

// ---------------------------------------------------------------- RMSNorm -> bf16, fragment order
// y = x * rsqrt(mean(x^2) + eps) * g, fp32 accumulation; output row i of the
// fragment-ordered matrix [n][d] comes from h[sel ? sel[i] : i].
// Two launch shapes with the same arithmetic: four rows per workgroup, one wave each (many rows: the row stays in
// registers between the two passes, no LDS, no barrier, and the four 16-byte pieces that share a 64-byte line of the
// fragment layout leave the same workgroup together), or one row per workgroup spread over four waves (few rows: four
// times the loads in flight per row).  Lane l owns the 8-element groups c = l + 64 q; its sum of squares is
// ((s_0 + s_1) + s_2) + s_3 with s_w the sum over q = w, w + 4, ... in ascending order, then a butterfly over the
// lanes: the order depends on d alone, so a row's bits do not depend on how many rows the pass has.
// FUSED: the row is first produced here, as the tail of a GEMM whose K slices went to separate workgroups: the slice
// partials ws[slices][n][d] are added in ascending order, the sum is added to the residual row h[i] (which is written
// back), and the new row is normalised -- the arithmetic of gemm_reduce_kernel<EPI_RESID_F32> followed by this kernel,
// bit for bit, in one launch instead of two.
template <int MAXC, int WPR, bool FUSED = false>      // 8-element groups per lane the registers can hold (d <= MAXC * 512); waves per row
__global__ __launch_bounds__(256) void rmsnorm_kernel(float *__restrict__ h, const bf16_t *__restrict__ g,
                                                      bf16_t *__restrict__ y, const int *__restrict__ sel, int n, int d, float eps,
                                                      const float4 *__restrict__ ws = nullptr, int slices = 0, size_t slab4 = 0, int group = 0) {
    static_assert(MAXC % 4 == 0 && (WPR == 1 || WPR == 4), "four partial sums per lane");
    __shared__ float part[WPR == 4 ? 4 * 64 : 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = WPR == 4 ? blockIdx.x : blockIdx.x * 4 + wave;
    if (i >= n) return;
    float *x = h + (size_t)((!FUSED && sel) ? sel[i] : i) * d;
    const int nc = d / 8;
    constexpr int NQ = MAXC / WPR;                 // groups this thread holds: q = q0 + QS * t
    const int q0 = WPR == 4 ? wave : 0;
    constexpr int QS = WPR == 4 ? 4 : 1;
    float4 a[NQ], b[NQ];
    float s4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < NQ; ++t) {
        const int q = q0 + QS * t, c = lane + q * 64;
        if (c < nc) {
            a[t] = reinterpret_cast<const float4 *>(x)[2 * c]; b[t] = reinterpret_cast<const float4 *>(x)[2 * c + 1];
            if (FUSED) {
                const float4 *p = ws + (size_t)i * (d / 4) + 2 * c;
                const int n1 = group > 0 ? group : slices;      // (group > 0: two runs, [0, group) and [group, slices), then their sum)
                float4 ta = p[0], tb = p[1];
                for (int s2 = 1; s2 < n1; ++s2) {
                    const float4 va = p[(size_t)s2 * slab4], vb = p[(size_t)s2 * slab4 + 1];
                    ta.x += va.x; ta.y += va.y; ta.z += va.z; ta.w += va.w;
                    tb.x += vb.x; tb.y += vb.y; tb.z += vb.z; tb.w += vb.w;
                }
                if (n1 < slices) {
                    float4 ua = p[(size_t)n1 * slab4], ub = p[(size_t)n1 * slab4 + 1];
                    for (int s2 = n1 + 1; s2 < slices; ++s2) {
                        const float4 va = p[(size_t)s2 * slab4], vb = p[(size_t)s2 * slab4 + 1];
                        ua.x += va.x; ua.y += va.y; ua.z += va.z; ua.w += va.w;
                        ub.x += vb.x; ub.y += vb.y; ub.z += vb.z; ub.w += vb.w;
                    }
                    ta.x += ua.x; ta.y += ua.y; ta.z += ua.z; ta.w += ua.w;
                    tb.x += ub.x; tb.y += ub.y; tb.z += ub.z; tb.w += ub.w;
                }
                a[t].x += ta.x; a[t].y += ta.y; a[t].z += ta.z; a[t].w += ta.w;
                b[t].x += tb.x; b[t].y += tb.y; b[t].z += tb.z; b[t].w += tb.w;
                reinterpret_cast<float4 *>(x)[2 * c] = a[t]; reinterpret_cast<float4 *>(x)[2 * c + 1] = b[t];
            }
            s4[WPR == 4 ? 0 : (t & 3)] += a[t].x * a[t].x + a[t].y * a[t].y + a[t].z * a[t].z + a[t].w * a[t].w
                                        + b[t].x * b[t].x + b[t].y * b[t].y + b[t].z * b[t].z + b[t].w * b[t].w;
        }
    }
    float ss;
    if (WPR == 4) {
        part[wave * 64 + lane] = s4[0];
        __syncthreads();
        ss = ((part[lane] + part[64 + lane]) + part[128 + lane]) + part[192 + lane];
    } else {
        ss = ((s4[0] + s4[1]) + s4[2]) + s4[3];
    }
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    const float inv = rsqrtf(ss / (float)d + eps);
#pragma unroll
    for (int t = 0; t < NQ; ++t) {
        const int q = q0 + QS * t, c = lane + q * 64;
        if (c < nc) {
            uint4 gv = reinterpret_cast<const uint4 *>(g)[c];
            const bf16_t *ge = reinterpret_cast<const bf16_t *>(&gv);
            bf16_t o[8];
            o[0] = f2bf(a[t].x * inv * bf2f(ge[0])); o[1] = f2bf(a[t].y * inv * bf2f(ge[1]));
            o[2] = f2bf(a[t].z * inv * bf2f(ge[2])); o[3] = f2bf(a[t].w * inv * bf2f(ge[3]));
            o[4] = f2bf(b[t].x * inv * bf2f(ge[4])); o[5] = f2bf(b[t].y * inv * bf2f(ge[5]));
            o[6] = f2bf(b[t].z * inv * bf2f(ge[6])); o[7] = f2bf(b[t].w * inv * bf2f(ge[7]));
            *reinterpret_cast<uint4 *>(y + frag_off(i, c * 8, d)) = *reinterpret_cast<uint4 *>(o);
        }
    }
}
template <int WPR>
static void launch_rmsnorm_shape(float *h, const bf16_t *g, bf16_t *y, const int *sel, int n, int d, float eps, hipStream_t st) {
    const dim3 grid(WPR == 4 ? n : (n + 3) / 4), block(256);
    if (d <= 2048) rmsnorm_kernel<4, WPR><<<grid, block, 0, st>>>(h, g, y, sel, n, d, eps);
    else if (d <= 4096) rmsnorm_kernel<8, WPR><<<grid, block, 0, st>>>(h, g, y, sel, n, d, eps);
    else rmsnorm_kernel<16, WPR><<<grid, block, 0, st>>>(h, g, y, sel, n, d, eps);      // d <= 8192 (checked at model load)
}
void launch_rmsnorm(const float *h, const bf16_t *g, bf16_t *y, const int *sel, int n, int d, float eps, hipStream_t st) {
    if (n <= 0) return;
    float *hh = const_cast<float *>(h);      // only the FUSED instantiation writes through it
    if (n >= 1024) launch_rmsnorm_shape<1>(hh, g, y, sel, n, d, eps, st);
    else launch_rmsnorm_shape<4>(hh, g, y, sel, n, d, eps, st);
}
// h[i] += sum of the slice partials ws[s][i] (ascending s; in two runs when group > 0), then y = rmsnorm(h[i]) in fragment order
void launch_reduce_resid_rmsnorm(const float *ws, int slices, int group, float *h, const bf16_t *g, bf16_t *y, int n, int d, float eps, hipStream_t st) {
    if (n <= 0) return;
    const dim3 grid(n), block(256);
    const float4 *w4 = reinterpret_cast<const float4 *>(ws);
    const size_t slab4 = (size_t)n * d / 4;
    if (d <= 2048) rmsnorm_kernel<4, 4, true><<<grid, block, 0, st>>>(h, g, y, nullptr, n, d, eps, w4, slices, slab4, group);
    else if (d <= 4096) rmsnorm_kernel<8, 4, true><<<grid, block, 0, st>>>(h, g, y, nullptr, n, d, eps, w4, slices, slab4, group);
    else rmsnorm_kernel<16, 4, true><<<grid, block, 0, st>>>(h, g, y, nullptr, n, d, eps, w4, slices, slab4, group);
}

// ---------------------------------------------------------------- RoPE angles, once per pass
// cs[r][i] = (cos, sin)(pos_r * inv_freq_i), computed in fp64 so that positions
// up to 64k lose nothing before the fp32 rotation.
__global__ void rope_table_kernel(const int *__restrict__ row_pos, const double *__restrict__ inv_freq,
                                  float2 *__restrict__ cs, int T, int half) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= T * half) return;
    int r = idx / half, i = idx % half;
    double ang = (double)row_pos[r] * inv_freq[i];
    double s, c;
    sincos(ang, &s, &c);
    cs[idx] = make_float2((float)c, (float)s);
}
void launch_rope_table(const PassMeta &pm, const double *inv_freq, float *cs, int D, hipStream_t st) {
    int n = pm.T * (D / 2);
    rope_table_kernel<<<dim3((n + 255) / 256), dim3(256), 0, st>>>(pm.row_pos, inv_freq, reinterpret_cast<float2 *>(cs), pm.T, D / 2);
}

// ---------------------------------------------------------------- RoPE on q and k; K/V rows -> pages
__device__ __forceinline__ f16_t f2h(float x) { return das_f2h(x); }
__device__ __forceinline__ float h2f(f16_t u) { return (float)__builtin_bit_cast(_Float16, u); }
// a K or V element: rounded to bf16 exactly once (the cache precision), then kept in a binary16 container, which is
// exact for every bf16 value with 2^-17 <= |x| <= 65504 (smaller ones move by at most 3e-8, larger ones saturate).
// The attention kernel's matrix instructions are the f16 ones: next to these values the rotated query and the
// probabilities then carry 11 significant bits in one term.
__device__ __forceinline__ f16_t kv_elem(float x) { return f2h(bf2f(f2bf(x))); }
// the same store, counted in *sat when the bf16 value does not fit the container (das_debug_kv_saturated)
__device__ __forceinline__ f16_t kv_elem_counted(float x, unsigned long long *sat) { return das_kv_elem_counted(x, sat); }

// grid (T, heads / heads per workgroup), block 256 = 256 / (D/2) heads: thread i of a head owns the rotate-half pair
// (i, i + D/2).  The projections arrive in fp32 and are rounded exactly once, after the rotation: q to binary16, k and
// v to bf16.
__global__ void rope_kv_kernel(PassMeta pm, const float *__restrict__ qkv, int slices, size_t slab, f16_t *__restrict__ q_h,
                               const float2 *__restrict__ cs, f16_t *__restrict__ kpool, f16_t *__restrict__ vpool,
                               int Hq, int Hkv, int D, int qkvN, unsigned long long *__restrict__ sat) {
    const int half = D >> 1, r = blockIdx.x, hh = blockIdx.y * (256 / half) + threadIdx.x / half, i = threadIdx.x % half;
    if (hh >= Hq + 2 * Hkv) return;
    const float *row = qkv + (size_t)r * qkvN + (size_t)hh * D;
    float x1 = row[i], x2 = row[i + half];
    for (int s = 1; s < slices; ++s) { x1 += row[s * slab + i]; x2 += row[s * slab + i + half]; }      // K-slice partials, in order
    if (hh < Hq + Hkv) {
        float2 c = cs[r * half + i];
        float y1 = das_rope_first(x1, x2, c), y2 = das_rope_second(x1, x2, c);
        x1 = y1; x2 = y2;
    }
    if (hh < Hq) {
        const size_t o = (size_t)r * Hq * D + (size_t)hh * D;
        q_h[o + i] = f2h(x1); q_h[o + i + half] = f2h(x2);
        return;
    }
    int b = pm.row_b[r], pos = pm.row_pos[r];
    int page = pm.page_table[(size_t)pm.b_slot[b] * pm.max_pages + (pos >> 4)];
    int t = pos & 15;
    if (hh < Hq + Hkv) {
        f16_t *blk = kpool + ((size_t)page * Hkv + (hh - Hq)) * (size_t)(DAS_PAGE * D);
        blk[kpage_off(t, i)] = kv_elem_counted(x1, sat);
        blk[kpage_off(t, i + half)] = kv_elem_counted(x2, sat);
    } else {
        f16_t *blk = vpool + ((size_t)page * Hkv + (hh - Hq - Hkv)) * (size_t)(DAS_PAGE * D);
        blk[vpage_off(t, i)] = kv_elem_counted(x1, sat);
        blk[vpage_off(t, i + half)] = kv_elem_counted(x2, sat);
    }
}
void launch_rope_kv(const PassMeta &pm, const float *qkv, int slices, f16_t *q_h, const float *cs,
                    f16_t *kpool_layer, f16_t *vpool_layer, const DasDims &dm, unsigned long long *sat, hipStream_t st) {
    const int heads_per_wg = 256 / (dm.D / 2);
    rope_kv_kernel<<<dim3(pm.T, (dm.Hq + 2 * dm.Hkv + heads_per_wg - 1) / heads_per_wg), dim3(256), 0, st>>>(
        pm, qkv, slices, (size_t)pm.T * dm.qkvN, q_h, reinterpret_cast<const float2 *>(cs), kpool_layer, vpool_layer, dm.Hq, dm.Hkv, dm.D, dm.qkvN, sat);
}

// ---------------------------------------------------------------- KV import / export / synthetic fill
// linear layout [n_pos][Hkv][D] in bf16; grid (n_pos, Hkv), block D
__global__ void kv_io_kernel(int mode, const int *__restrict__ page_row, int first_pos, f16_t *kpool, f16_t *vpool,
                             bf16_t *k_lin, bf16_t *v_lin, int Hkv, int D, int num_pages, unsigned long long *sat) {
    int p = blockIdx.x, hd = blockIdx.y, d = threadIdx.x;
    int pos = first_pos + p;
    size_t blk = ((size_t)page_row[pos >> 4] * Hkv + hd) * (size_t)(DAS_PAGE * D);
    size_t lin = ((size_t)p * Hkv + hd) * D + d;
    int t = pos & 15;
    if (mode == 0) {
        kpool[blk + kpage_off(t, d)] = kv_elem_counted(bf2f(k_lin[lin]), sat);
        vpool[blk + vpage_off(t, d)] = kv_elem_counted(bf2f(v_lin[lin]), sat);
    } else {
        k_lin[lin] = f2bf(h2f(kpool[blk + kpage_off(t, d)]));
        v_lin[lin] = f2bf(h2f(vpool[blk + vpage_off(t, d)]));
    }
}
void launch_kv_io(int mode, const int *page_row, int first_pos, int n_pos, f16_t *kpool_layer, f16_t *vpool_layer,
                  bf16_t *k_lin, bf16_t *v_lin, int Hkv, int D, int num_pages, unsigned long long *sat, hipStream_t st) {
    if (n_pos > 0)
        kv_io_kernel<<<dim3(n_pos, Hkv), dim3(D), 0, st>>>(mode, page_row, first_pos, kpool_layer, vpool_layer, k_lin, v_lin, Hkv, D, num_pages, sat);
}

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
__device__ __forceinline__ f16_t synth_value(uint64_t base, uint64_t e) {
    uint64_t h = mix64(base ^ e);
    int s = (int)(h & 0xFFFF) + (int)((h >> 16) & 0xFFFF) + (int)((h >> 32) & 0xFFFF) + (int)(h >> 48) - 131070;
    return kv_elem((float)s * (1.0f / 32768.0f));
}
__global__ void kv_synth_kernel(const int *__restrict__ page_row, f16_t *kpool, f16_t *vpool, int Hkv, int D, int num_pages,
                                uint64_t base_k, uint64_t base_v) {
    int pos = blockIdx.x, hd = blockIdx.y, d = threadIdx.x;
    size_t blk = ((size_t)page_row[pos >> 4] * Hkv + hd) * (size_t)(DAS_PAGE * D);
    uint64_t e = ((uint64_t)pos * Hkv + hd) * D + d;
    int t = pos & 15;
    kpool[blk + kpage_off(t, d)] = synth_value(base_k, e);
    vpool[blk + vpage_off(t, d)] = synth_value(base_v, e);
}
static uint64_t host_mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
void launch_kv_synth(const int *page_row, int ctx, f16_t *kpool_layer, f16_t *vpool_layer, int Hkv, int D, int num_pages,
                     uint64_t seed, uint64_t seq_key, int layer, hipStream_t st) {
    if (ctx <= 0) return;
    uint64_t b = host_mix64(host_mix64(seed ^ 0x4B5653594E544821ull) ^ seq_key);
    uint64_t bk = host_mix64(b ^ ((uint64_t)layer * 2u)), bv = host_mix64(b ^ ((uint64_t)layer * 2u + 1u));
    kv_synth_kernel<<<dim3(ctx, Hkv), dim3(D), 0, st>>>(page_row, kpool_layer, vpool_layer, Hkv, D, num_pages, bk, bv);
}

// ---------------------------------------------------------------- random initialisation on the device
// Element i of a tensor is bf16(sigma * z), z = sqrt(-2 ln u1) cos(2 pi u2) in fp64, (u1, u2) from the two halves of
// mix64(base ^ i): the counter-based generator that das.h states for das_model_load without a weight blob.
__device__ __forceinline__ double normal_from_bits(uint64_t h) {
    const double u1 = ((double)(uint32_t)(h >> 32) + 1.0) * (1.0 / 4294967296.0);      // (0, 1]
    const double u2 = (double)(uint32_t)h * (1.0 / 4294967296.0);
    return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
}
__global__ void fill_normal_kernel(bf16_t *__restrict__ dst, size_t n, uint64_t base, double sigma) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = f2bf((float)(sigma * normal_from_bits(mix64(base ^ (uint64_t)i))));
}
__global__ void fill_const_kernel(bf16_t *__restrict__ dst, size_t n, bf16_t v) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = v;
}
void launch_fill_normal(bf16_t *dst, size_t n, uint64_t seed, uint64_t tensor_id, double sigma, hipStream_t st) {
    if (n == 0) return;
    const uint64_t base = host_mix64(host_mix64(seed ^ 0x5745494748545321ull) ^ tensor_id);
    const unsigned grid = (unsigned)std::min<size_t>((n + 255) / 256, 256 * 64);
    fill_normal_kernel<<<dim3(grid), dim3(256), 0, st>>>(dst, n, base, sigma);
}
void launch_fill_const(bf16_t *dst, size_t n, bf16_t v, hipStream_t st) {
    if (n == 0) return;
    const unsigned grid = (unsigned)std::min<size_t>((n + 255) / 256, 256 * 64);
    fill_const_kernel<<<dim3(grid), dim3(256), 0, st>>>(dst, n, v);
}

// ---------------------------------------------------------------- plain copy (counter calibration)
__global__ void plain_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = src[i];
}
void launch_copy(const void *src, void *dst, size_t bytes, hipStream_t st) {
    const size_t n = bytes / 16;
    const unsigned grid = (unsigned)std::min<size_t>((n + 255) / 256, 256 * 32);
    plain_copy_kernel<<<dim3(grid), dim3(256), 0, st>>>(reinterpret_cast<const uint4 *>(src), reinterpret_cast<uint4 *>(dst), n);
}
