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
// row_stats[r] = (max logit, Z = sum exp((l - max)/T))
__global__ __launch_bounds__(1024) void row_stats_kernel(const float *__restrict__ logits, int V, float inv_temp,
                                                         float *__restrict__ stats) {
    // one pass over the row: every thread keeps a running (max, sum of exp relative to that max) over its elements and
    // the pairs are then combined in a fixed order (lanes by butterfly, waves in index order)
    __shared__ float red_m[16], red_z[16];
    const float *x = logits + (size_t)blockIdx.x * V;
    float mx = -INFINITY, z = 0.f;
    auto add = [&](float v) {
        if (v > mx) { z = z * __expf((mx - v) * inv_temp) + 1.f; mx = v; }      // exp(-inf) = 0 on the first element
        else z += __expf((v - mx) * inv_temp);
    };
    const int nv4 = V >> 2;
    for (int c = threadIdx.x; c < nv4; c += 1024) {
        const float4 v = reinterpret_cast<const float4 *>(x)[c];
        add(v.x); add(v.y); add(v.z); add(v.w);
    }
    for (int i = (nv4 << 2) + threadIdx.x; i < V; i += 1024) add(x[i]);
    auto merge = [&](float om, float oz) {
        const float nm = fmaxf(mx, om);
        if (nm == -INFINITY) return;                                          // both empty
        z = z * __expf((mx - nm) * inv_temp) + oz * __expf((om - nm) * inv_temp);
        mx = nm;
    };
    for (int o = 32; o > 0; o >>= 1) {
        const float om = __shfl_xor(mx, o), oz = __shfl_xor(z, o);
        merge(om, oz);
    }
    if ((threadIdx.x & 63) == 0) { red_m[threadIdx.x >> 6] = mx; red_z[threadIdx.x >> 6] = z; }
    __syncthreads();
    if (threadIdx.x == 0) {
        mx = red_m[0]; z = red_z[0];
        for (int w = 1; w < 16; ++w) merge(red_m[w], red_z[w]);
        stats[2 * blockIdx.x] = mx;
        stats[2 * blockIdx.x + 1] = z;
    }
}

// One workgroup (16 waves) per sequence.  Rows j = 0..k-1: accept draft j+1 iff u_accept*Z < w(draft); the rows are tested
// side by side, one per lane, and the first rejection is taken from a ballot.  Then an inverse-CDF draw (ascending
// vocabulary order) from the row where the walk stopped, with the rejected draft's weight removed: wave w owns the
// contiguous segment [w*seg, (w+1)*seg) and walks it in blocks of 256 consecutive columns (four per lane), recording the
// total of every block; the 16 segment totals are added in order, and the wave whose segment holds the crossing finds
// the block from its recorded totals and reads that block a second time to name the column.
__device__ __forceinline__ float wave_inclusive_scan(float v, int lane) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const float t = __shfl_up(v, o);
        if (lane >= o) v += t;
    }
    return v;
}
#define SAMPLE_GROUPS 64
__global__ __launch_bounds__(1024) void accept_sample_kernel(const float *__restrict__ logits, int V,
                                                             const int *__restrict__ tok, const int *__restrict__ b_row0,
                                                             const int *__restrict__ b_n, float inv_temp,
                                                             const float *__restrict__ u_accept,
                                                             const float *__restrict__ u_sample, int prefill_mode,
                                                             const float *__restrict__ stats, int *__restrict__ accept_len,
                                                             int *__restrict__ next_token) {
    __shared__ float seg_total[16];
    __shared__ int seg_lastnz[16];
    __shared__ int walk[2];          // accepted drafts, rejected token
    __shared__ float grp_total[16][SAMPLE_GROUPS];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r0 = prefill_mode ? b : b_row0[b];
    const int k = prefill_mode ? 0 : b_n[b] - 1;
    if (wave == 0) {
        int a = k, rejected = -1;
        for (int base = 0; base < k && a == k; base += 64) {
            const int jrow = base + lane;
            bool rej = false;
            int d = -1;
            if (jrow < k) {
                const int r = r0 + jrow;
                d = tok[r + 1];
                const float mx = stats[2 * r], Z = stats[2 * r + 1];
                const float wd = __expf((logits[(size_t)r * V + d] - mx) * inv_temp);
                rej = !(u_accept[r] * Z < wd);
            }
            const unsigned long long m = __ballot(rej);
            if (m) {
                const int first = __ffsll((long long)m) - 1;
                a = base + first;
                rejected = __shfl(d, first);
            }
        }
        if (lane == 0) { walk[0] = a; walk[1] = rejected; }
    }
    __syncthreads();
    const int a = walk[0], rejected = walk[1];
    const int r = r0 + a;
    const float *x = logits + (size_t)r * V;
    const float mx = stats[2 * r];
    const float u = prefill_mode ? u_sample[b] : u_sample[r];
    // Columns per wave: a multiple of 256.  A wave walks its segment in blocks of 256 columns, four columns per lane (one
    // 16-byte load when V is a multiple of 4), four blocks in flight.  The weights of a block are added as: each lane its four
    // columns in order, then an inclusive scan over the lanes, so a running sum in index order exists at every column.
    const int seg = (((V + 15) / 16) + 255) & ~255;
    const int lo = wave * seg, hi = min(lo + seg, V);
    const int nblk = hi > lo ? (hi - lo + 255) >> 8 : 0;          // blocks of this wave that hold columns
    const int grp = ((seg >> 8) + SAMPLE_GROUPS - 1) / SAMPLE_GROUPS;      // blocks per recorded total (1 up to V = 262144)
    const bool vec = (V & 3) == 0;
    auto weights4 = [&](int i, float w[4]) {
        float l[4];
        if (vec && i + 3 < hi) {
            const float4 v = *reinterpret_cast<const float4 *>(x + i);
            l[0] = v.x; l[1] = v.y; l[2] = v.z; l[3] = v.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) l[e] = i + e < hi ? x[i + e] : -INFINITY;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (i + e < hi && i + e != rejected) ? __expf((l[e] - mx) * inv_temp) : 0.f;
    };
    float run = 0.f, gsum = 0.f;
    int nz = -1;
    for (int b0 = 0; b0 < nblk; b0 += 4) {
        float w[4][4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (b0 + q < nblk) weights4(lo + ((b0 + q) << 8) + 4 * lane, w[q]);
            else w[q][0] = w[q][1] = w[q][2] = w[q][3] = 0.f;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int blk = b0 + q;
            if (blk >= nblk) break;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (w[q][e] > 0.f) nz = lo + (blk << 8) + 4 * lane + e;
            const float ls = ((w[q][0] + w[q][1]) + w[q][2]) + w[q][3];
            gsum += __shfl(wave_inclusive_scan(ls, lane), 63);
            if (blk % grp == grp - 1 || blk == nblk - 1) {
                if (lane == 0) grp_total[wave][blk / grp] = gsum;
                run += gsum;
                gsum = 0.f;
            }
        }
    }
    for (int o = 32; o > 0; o >>= 1) nz = max(nz, __shfl_xor(nz, o));
    if (lane == 0) { seg_total[wave] = run; seg_lastnz[wave] = nz; }
    __syncthreads();
    float before = 0.f, total = 0.f;
    int owner = -1;
    {
        float c = 0.f;
        for (int w = 0; w < 16; ++w) {
            if (w == wave) before = c;
            c += seg_total[w];
        }
        total = c;
        const float target = u * total;
        c = 0.f;
        for (int w = 0; w < 16; ++w) {
            c += seg_total[w];
            if (owner < 0 && c > target) owner = w;
        }
    }
    const float target = u * total;
    if (wave == (owner < 0 ? 0 : owner)) {
        int pick = -1;
        if (owner >= 0) {
            // the recorded totals name the group of blocks that holds the crossing; only that group is read again
            float c = before;
            const int ngrp = (nblk + grp - 1) / grp;
            int g = 0;
            for (; g < ngrp; ++g) {
                const float t = grp_total[wave][g];
                if (c + t > target) break;
                c += t;
            }
            for (int blk = g * grp; g < ngrp && blk < min((g + 1) * grp, nblk) && pick < 0; ++blk) {
                float w[4];
                const int i = lo + (blk << 8) + 4 * lane;
                weights4(i, w);
                const float p0 = w[0], p1 = p0 + w[1], p2 = p1 + w[2], ls = p2 + w[3];
                const float sc = wave_inclusive_scan(ls, lane);
                float ex = __shfl_up(sc, 1);
                if (lane == 0) ex = 0.f;
                // this lane's candidate: its first column whose running sum passes the target, else its last non-zero one
                const float pre[4] = {p0, p1, p2, ls};
                int cand = -1;
#pragma unroll
                for (int e = 3; e >= 0; --e)
                    if (w[e] > 0.f && (cand < 0 || c + (ex + pre[e]) > target)) cand = e;
                const unsigned long long m = __ballot(c + sc > target);
                if (m) {
                    const int L = __ffsll((long long)m) - 1;
                    // (a lane of zero weights cannot be the first to pass, except by rounding in the scan: then the
                    // nearest lane below it that holds a weight)
                    const unsigned long long have = __ballot(cand >= 0) & ((2ull << L) - 1ull);
                    if (have) pick = __shfl(i + cand, 63 - __clzll((long long)have));
                }
                c += __shfl(sc, 63);
            }
            // the running sum starts at the segments before this one here and at zero in the first walk: if that rounds
            // the last step below the target, the crossing is the segment's last non-zero weight
            if (pick < 0) pick = seg_lastnz[wave];
        }
        if (pick < 0) {                                  // rounding pushed the target past the total: last non-zero weight
            for (int w = 0; w < 16; ++w) pick = max(pick, seg_lastnz[w]);
        }
        if (lane == 0) {
            accept_len[b] = a;
            next_token[b] = pick;
        }
    }
}

void launch_sample(const float *logits, int V, const int *tok, const int *b_row0, const int *b_n, int NB,
                   float inv_temp, const float *u_accept, const float *u_sample, int prefill_mode,
                   float *row_stats, int *accept_len, int *next_token, hipStream_t st) {
    // the caller passes the number of logit rows through b_n/b_row0 (verify) or NB (prefill: one row per sequence)
    (void)row_stats;
    accept_sample_kernel<<<dim3(NB), dim3(1024), 0, st>>>(logits, V, tok, b_row0, b_n, inv_temp, u_accept, u_sample,
                                                        prefill_mode, row_stats, accept_len, next_token);
}

void launch_row_stats(const float *logits, int n_rows, int V, float inv_temp, float *stats, hipStream_t st) {
    if (n_rows > 0) row_stats_kernel<<<dim3(n_rows), dim3(1024), 0, st>>>(logits, V, inv_temp, stats);
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
