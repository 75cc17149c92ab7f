// Decision kernels of the verify step: per-row argmax (wavefront reduction,
// lowest index wins ties), greedy prefix acceptance, and the rejection-sampling
// acceptance for stochastic rollouts.
#include "das_internal.h"

// ---------------------------------------------------------------- argmax over the vocabulary
__global__ __launch_bounds__(1024) void argmax_kernel(const float *__restrict__ logits, int V, int *__restrict__ out) {
    __shared__ float sv[16];
    __shared__ int si[16];
    const float *x = logits + (size_t)blockIdx.x * V;
    float best = -INFINITY;
    int bi = 0x7FFFFFFF;
    const int nv4 = V >> 2;
    for (int c = threadIdx.x; c < nv4; c += 1024) {
        float4 v = reinterpret_cast<const float4 *>(x)[c];
        int i = c * 4;
        if (v.x > best) { best = v.x; bi = i; }
        if (v.y > best) { best = v.y; bi = i + 1; }
        if (v.z > best) { best = v.z; bi = i + 2; }
        if (v.w > best) { best = v.w; bi = i + 3; }
    }
    for (int i = (nv4 << 2) + threadIdx.x; i < V; i += 1024)
        if (x[i] > best) { best = x[i]; bi = i; }
    // thread-local scan is in ascending index, so bi is already the lowest index of its maximum
    for (int o = 32; o > 0; o >>= 1) {
        float ov = __shfl_xor(best, o);
        int oi = __shfl_xor(bi, o);
        if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
    }
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = best; si[threadIdx.x >> 6] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; ++w)
            if (sv[w] > best || (sv[w] == best && si[w] < bi)) { best = sv[w]; bi = si[w]; }
        out[blockIdx.x] = bi;
    }
}
void launch_argmax(const float *logits, int n_rows, int V, int *out, hipStream_t st) {
    if (n_rows > 0) argmax_kernel<<<dim3(n_rows), dim3(1024), 0, st>>>(logits, V, out);
}

// ---------------------------------------------------------------- greedy acceptance
// Block b holds rows [pending, d_1..d_k]; g[r] is the target's token after row r.
// accept = longest prefix with d_j == g[row j-1]; next = g[row accept].
__global__ void accept_greedy_kernel(const int *__restrict__ g, const int *__restrict__ b_row0, const int *__restrict__ b_n,
                                     const int *__restrict__ tok, int NB, int *__restrict__ accept_len,
                                     int *__restrict__ next_token) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= NB) return;
    const int r0 = b_row0[b], k = b_n[b] - 1;
    int a = 0;
    while (a < k && tok[r0 + 1 + a] == g[r0 + a]) ++a;
    accept_len[b] = a;
    next_token[b] = g[r0 + a];
}
void launch_accept_greedy(const int *g, const int *b_row0, const int *b_n, const int *tok, int NB,
                          int *accept_len, int *next_token, hipStream_t st) {
    if (NB > 0) accept_greedy_kernel<<<dim3((NB + 63) / 64), dim3(64), 0, st>>>(g, b_row0, b_n, tok, NB, accept_len, next_token);
}

// ---------------------------------------------------------------- stochastic acceptance
// Everything here is DEFINED on per-block statistics of the logits, so that a pass that never writes its logits (the
// LM-head GEMM emits the statistics from its accumulators) and a pass that does (inspection, small vocabularies) take
// the same decisions bit for bit.  Block b = columns 32b .. 32b+31 of a row; the block is seen as two halves, half h
// holding the columns c with (c >> 2) & 1 == h in ascending order (the registers of one lane of a 32x32 MFMA block):
//     m_h = running maximum of half h,  m_b = max(m_0, m_1),
//     z_h = sum over half h, in that order, of exp((l - m_b) / T),  z_b = z_0 + z_1.
// Columns past the vocabulary take no part.  Row statistics (M, Z): 32 chains, chain c merging the blocks
// b = c, c+32, ... in ascending order, then the chains merged in ascending order, where merging (m, z) with (m', z')
// gives (max, z e^{(m-max)/T} + z' e^{(m'-max)/T}).

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

__device__ __forceinline__ void stats_merge(float &m, float &z, float om, float oz, float inv_temp) {
    const float nm = fmaxf(m, om);
    if (nm == -INFINITY) return;                                          // both empty
    z = z * __expf((m - nm) * inv_temp) + oz * __expf((om - nm) * inv_temp);
    m = nm;
}

// block statistics from written logits; grid (ceil(nblk / 256), rows), one thread per (row, block)
__global__ __launch_bounds__(256) void block_stats_kernel(const float *__restrict__ logits, int V, int nblk, float inv_temp,
                                                          const int *__restrict__ dtok, float2 *__restrict__ part, int ldp,
                                                          float *__restrict__ draft_logit) {
    const int row = blockIdx.y, b = blockIdx.x * 256 + threadIdx.x;
    const float *x = logits + (size_t)row * V;
    if (b == 0) { const int dt = dtok ? dtok[row] : -1; draft_logit[row] = dt >= 0 ? x[dt] : 0.f; }
    if (b >= nblk) return;
    float v[32];
#pragma unroll
    for (int c = 0; c < 32; ++c) v[c] = 32 * b + c < V ? x[32 * b + c] : -INFINITY;
    float mh[2] = {-INFINITY, -INFINITY};
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int r = 0; r < 16; ++r) { const int c = 8 * (r >> 2) + 4 * h + (r & 3); if (32 * b + c < V) mh[h] = fmaxf(mh[h], v[c]); }
    const float mb = fmaxf(mh[0], mh[1]);
    float zh[2] = {0.f, 0.f};
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int r = 0; r < 16; ++r) { const int c = 8 * (r >> 2) + 4 * h + (r & 3); if (32 * b + c < V) zh[h] += __expf((v[c] - mb) * inv_temp); }
    part[(size_t)b * ldp + row] = make_float2(mb, zh[0] + zh[1]);
}

// row statistics from the block statistics; grid ceil(rows / 8), block 256 = 32 chains x 8 rows (8 rows = one 64-byte
// run of the [block][row] layout).  A chain's loads are independent of its arithmetic: eight are requested at a time.
__global__ __launch_bounds__(256) void row_stats_merge_kernel(const float2 *__restrict__ part, int ldp, int nblk, int n_rows,
                                                              float inv_temp, float2 *__restrict__ stats) {
    __shared__ float2 chain[32][8];
    const int rl = threadIdx.x & 7, c = threadIdx.x >> 3, row = blockIdx.x * 8 + rl;
    float m = -INFINITY, z = 0.f;
    if (row < n_rows) {
        for (int b0 = c; b0 < nblk; b0 += 32 * 8) {
            float2 p[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) { const int b = b0 + 32 * q; p[q] = b < nblk ? part[(size_t)b * ldp + row] : make_float2(-INFINITY, 0.f); }
#pragma unroll
            for (int q = 0; q < 8; ++q) stats_merge(m, z, p[q].x, p[q].y, inv_temp);
        }
    }
    chain[c][rl] = make_float2(m, z);
    __syncthreads();
    if (c == 0 && row < n_rows) {
        for (int k = 1; k < 32; ++k) stats_merge(m, z, chain[k][rl].x, chain[k][rl].y, inv_temp);
        stats[row] = make_float2(m, z);
    }
}

// One workgroup (256 threads) per sequence.
//  1. Rows j = 0..k-1 (one per lane of wave 0): accept draft j+1 iff u_accept * Z < w(draft), w = exp((l_draft - M) / T);
//     the first rejection is taken from a ballot: a = accepted drafts, `rejected` = the token that failed (-1: none).
//  2. The token after row a is the inverse-CDF draw (ascending vocabulary order) from the row's weights with the rejected
//     token's weight removed.  First the BLOCK that holds the crossing, from the block weights
//         W_b = z_b e^{(m_b - M)/T}   (minus w(rejected), floored at zero, for the block that holds the rejected token):
//     thread t adds its ceil(nblk/256) consecutive blocks in ascending order, the 256 sums are added in ascending order
//     (total), target = u_sample * total, and the crossing is the first block at which the running sum exceeds the target.
//  3. Then the column inside that block: wave 0 computes the block's 32 logits of that row again with the MFMA sequence of
//     the LM-head GEMM (one pass over K, 16 at a time, from zero: the same bits) and walks them in ascending order from
//     the running sum in front of the block.  If rounding keeps the walk below the target, the block's last column of
//     non-zero weight is taken; the rejected token is never returned.
// xsel: the normalised rows that got logits (fragment order, K = d); wlm: the LM head (fragment order).
__global__ __launch_bounds__(256) void accept_sample_kernel(const float2 *__restrict__ part, int ldp, int nblk, int V,
                                                            const float2 *__restrict__ stats, const float *__restrict__ draft_logit,
                                                            const bf16_t *__restrict__ xsel, const bf16_t *__restrict__ wlm, int K,
                                                            const int *__restrict__ tok, const int *__restrict__ b_row0,
                                                            const int *__restrict__ b_n, float inv_temp,
                                                            const float *__restrict__ u_accept, const float *__restrict__ u_sample,
                                                            int prefill_mode, int *__restrict__ accept_len, int *__restrict__ next_token) {
    __shared__ int walk[2];            // accepted drafts, rejected token
    __shared__ float tsum[256];
    __shared__ float found[4];         // crossing block, running sum in front of it, target, (flag)
    __shared__ int last_nz_blk[256];
    const int s = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r0 = prefill_mode ? s : b_row0[s];
    const int k = prefill_mode ? 0 : b_n[s] - 1;
    if (wave == 0) {
        int a = k, rejected = -1;
        for (int base = 0; base < k && a == k; base += 64) {
            const int jrow = base + lane;
            bool rej = false;
            int d = -1;
            if (jrow < k) {
                const int r = r0 + jrow;
                d = tok[r + 1];
                const float2 st = stats[r];
                const float wd = __expf((draft_logit[r] - st.x) * inv_temp);
                rej = !(u_accept[r] * st.y < wd);
            }
            const unsigned long long mk = __ballot(rej);
            if (mk) {
                const int first = __ffsll((long long)mk) - 1;
                a = base + first;
                rejected = __shfl(d, first);
            }
        }
        if (lane == 0) { walk[0] = a; walk[1] = rejected; }
    }
    __syncthreads();
    const int a = walk[0], rejected = walk[1];
    const int r = r0 + a;
    const float M = stats[r].x;
    const float u = prefill_mode ? u_sample[s] : u_sample[r];
    const float wrej = rejected >= 0 ? __expf((draft_logit[r] - M) * inv_temp) : 0.f;
    const int rej_blk = rejected >= 0 ? rejected >> 5 : -1;
    auto block_weight = [&](int b) -> float {
        const float2 p = part[(size_t)b * ldp + r];
        float w = p.x == -INFINITY ? 0.f : p.y * __expf((p.x - M) * inv_temp);
        if (b == rej_blk) w = fmaxf(w - wrej, 0.f);
        return w;
    };
    const int per = (nblk + 255) / 256;
    const int b_lo = min(tid * per, nblk), b_hi = min(b_lo + per, nblk);
    {
        float acc = 0.f;
        int nz = -1;
        for (int b0 = b_lo; b0 < b_hi; b0 += 8) {      // (the loads of eight blocks in flight together; added in ascending order)
            float w[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) w[q] = b0 + q < b_hi ? block_weight(b0 + q) : 0.f;
#pragma unroll
            for (int q = 0; q < 8; ++q) if (b0 + q < b_hi) { acc += w[q]; if (w[q] > 0.f) nz = b0 + q; }
        }
        tsum[tid] = acc;
        last_nz_blk[tid] = nz;
    }
    __syncthreads();
    if (tid == 0) {
        float total = 0.f;
        for (int t = 0; t < 256; ++t) total += tsum[t];
        const float target = u * total;
        float c = 0.f;
        int owner = -1;
        for (int t = 0; t < 256 && owner < 0; ++t) { if (c + tsum[t] > target) owner = t; else c += tsum[t]; }
        found[2] = target;
        found[3] = (float)owner;
        found[1] = c;                  // running sum in front of the owner's first block
    }
    __syncthreads();
    const float target = found[2];
    const int owner = (int)found[3];
    if (owner >= 0) {
        if (tid == owner) {
            float c = found[1];
            int bsel = -1;
            for (int b = b_lo; b < b_hi; ++b) {
                const float w = block_weight(b);
                if (c + w > target) { bsel = b; break; }
                c += w;
            }
            if (bsel < 0) {            // the thread's total crossed but its walk did not (cannot differ: same additions); keep its last non-zero block
                bsel = last_nz_blk[tid];
                c = found[1];
                for (int b = b_lo; b < bsel; ++b) c += block_weight(b);
            }
            found[0] = (float)bsel;
            found[1] = c;
        }
    } else if (tid == 0) {             // rounding pushed the target past the total: the last block of non-zero weight
        int tl = -1, bsel = -1;
        for (int t = 0; t < 256; ++t) if (last_nz_blk[t] >= 0) tl = t;
        float c = 0.f;
        if (tl >= 0) {
            bsel = last_nz_blk[tl];
            for (int t = 0; t < tl; ++t) c += tsum[t];
            for (int b = min(tl * per, nblk); b < bsel; ++b) c += block_weight(b);
        }
        found[0] = (float)bsel;
        found[1] = c;
    }
    __syncthreads();
    if (wave != 0) return;
    const int bsel = (int)found[0];
    float c = found[1];
    // the 32 logits of row r in block bsel: transposed 32x32 block (rows = weight rows = columns of the logits)
    const int KF = K >> 4;
    const uint4 *wp = reinterpret_cast<const uint4 *>(wlm) + (size_t)max(bsel, 0) * KF * 64 + lane;
    const uint4 *ap = reinterpret_cast<const uint4 *>(xsel) + (size_t)(r >> 5) * KF * 64 + lane;
    f32x16_t acc;
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[q] = 0.f;
    for (int ks0 = 0; ks0 < KF; ks0 += 16) {      // sixteen k-steps' loads in flight together (past the end: the last one again, unused)
        uint4 wv[16], av[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) { const size_t o = (size_t)min(ks0 + q, KF - 1) * 64; wv[q] = wp[o]; av[q] = ap[o]; }
#pragma unroll
        for (int q = 0; q < 16; ++q)
            if (ks0 + q < KF)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8_t *>(&wv[q]), *reinterpret_cast<const bf16x8_t *>(&av[q]), acc, 0, 0, 0);
    }
    // lane (lr, lh) holds, of activation row lr, the block's columns 8q + 4lh + e in register 4q + e: bring row r % 32 to every lane
    float l[32];
    const int src0 = r & 31, src1 = 32 + (r & 31);
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            l[8 * q + e] = __shfl(acc[4 * q + e], src0);
            l[8 * q + 4 + e] = __shfl(acc[4 * q + e], src1);
        }
    if (lane == 0) {
        int pick = -1, last_nz = -1, first_ok = -1;
        if (bsel >= 0) {
#pragma unroll
            for (int cc = 0; cc < 32; ++cc) {
                const int col = 32 * bsel + cc;
                if (col >= V || col == rejected) continue;
                if (first_ok < 0) first_ok = col;
                const float w = __expf((l[cc] - M) * inv_temp);
                if (w > 0.f) last_nz = col;
                c += w;
                if (pick < 0 && c > target) pick = col;
            }
            if (pick < 0) pick = last_nz >= 0 ? last_nz : first_ok;
        }
        if (pick < 0) pick = rejected == 0 ? 1 : 0;      // (a row without any weight: cannot happen for finite logits)
        accept_len[s] = a;
        next_token[s] = pick;
    }
}

void launch_block_stats(const float *logits, int n_rows, int V, float inv_temp, const int *dtok, float2 *part, int ldp,
                        float *draft_logit, hipStream_t st) {
    if (n_rows <= 0) return;
    const int nblk = (V + 31) / 32;
    block_stats_kernel<<<dim3((nblk + 255) / 256, n_rows), dim3(256), 0, st>>>(logits, V, nblk, inv_temp, dtok, part, ldp, draft_logit);
}
void launch_row_stats_merge(const float2 *part, int ldp, int V, int n_rows, float inv_temp, float2 *stats, hipStream_t st) {
    if (n_rows <= 0) return;
    row_stats_merge_kernel<<<dim3((n_rows + 7) / 8), dim3(256), 0, st>>>(part, ldp, (V + 31) / 32, n_rows, inv_temp, stats);
}
void launch_sample(const float2 *part, int ldp, int V, const float2 *stats, const float *draft_logit, const bf16_t *xsel,
                   const bf16_t *wlm, int K, const int *tok, const int *b_row0, const int *b_n, int NB, float inv_temp,
                   const float *u_accept, const float *u_sample, int prefill_mode, int *accept_len, int *next_token, hipStream_t st) {
    if (NB <= 0) return;
    accept_sample_kernel<<<dim3(NB), dim3(256), 0, st>>>(part, ldp, (V + 31) / 32, V, stats, draft_logit, xsel, wlm, K, tok, b_row0, b_n,
                                                       inv_temp, u_accept, u_sample, prefill_mode, accept_len, next_token);
}

// ---------------------------------------------------------------- row maxima gathered by the LM-head GEMM itself
// key = (order-preserving integer image of the value) << 32 | ~column: the largest key is the largest value at its
// lowest column.  Keys start at zero (below the image of every float).
__global__ void rowmax_keys_clear_kernel(unsigned long long *keys, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) keys[i] = 0ull;
}
__global__ void rowmax_keys_decode_kernel(const unsigned long long *keys, int n, int *out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = (int)(0xFFFFFFFFu - (uint32_t)(keys[i] & 0xFFFFFFFFull));
}
void launch_rowmax_keys_clear(unsigned long long *keys, int n_rows, hipStream_t st) {
    if (n_rows > 0) rowmax_keys_clear_kernel<<<(n_rows + 255) / 256, 256, 0, st>>>(keys, n_rows);
}
void launch_rowmax_keys_decode(const unsigned long long *keys, int n_rows, int *out, hipStream_t st) {
    if (n_rows > 0) rowmax_keys_decode_kernel<<<(n_rows + 255) / 256, 256, 0, st>>>(keys, n_rows, out);
}
