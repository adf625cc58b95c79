// Quality diagnostic of libdhsa: per-row recall of the routed key sets against
// exact top-k attention (App. "Theoretical Analysis", Setup and Notation:
// Recall_i = |I*_i n I_hat_i| / |I*_i|, I*_i = the k keys j <= i with the largest
// attention scores, k = min(N_b, i + 1), equal scores by lower index).
//
// One workgroup per sampled row:
//   1. logits q_i . k_j, j <= i, in fp64, summed in the order d = 0, 1, ... by one
//      thread per key (the products of bf16 / fp32 values are exact in fp64, so the
//      value is the same on any machine that sums in that order), stored as
//      order-preserving 64-bit integers in the caller's workspace;
//   2. the k-th largest of them by a most-significant-digit radix select (8 passes
//      of 8 bits, LDS histograms);
//   3. the row's selected keys (walked from the plan like the attention kernels do)
//      are counted if their logit is above that threshold, or equal to it and among
//      the lowest-indexed equal ones that still fit into the top k.
#include "dhsa_internal.h"

namespace dhsa {

__device__ __forceinline__ double recall_elem(const float *p, int d) { return (double)p[d]; }
__device__ __forceinline__ double recall_elem(const uint16_t *p, int d) {
    return (double)__uint_as_float((uint32_t)p[d] << 16);
}

template <typename T>
__global__ __launch_bounds__(256) void k_recall(PlanView pv, const T *__restrict__ Q, const T *__restrict__ K,
                                                int N_b, int G, int D, int head, const int64_t *__restrict__ rows,
                                                int64_t L, unsigned long long *__restrict__ ws,
                                                int32_t *__restrict__ hits_out, int32_t *__restrict__ size_out,
                                                int64_t qs_h, int64_t qs_l, int64_t ks_h, int64_t ks_l) {
    __shared__ double s_q[128];
    __shared__ int s_hist[256];
    __shared__ int s_wave[4];
    __shared__ int s_digit, s_above, s_equal;
    if (!plan_matches(pv)) return;   // not this problem's plan: nothing is written
    const int t = blockIdx.x, tid = threadIdx.x;
    const int64_t i = rows[t];
    const int n = (int)(i + 1);
    const int k_top = N_b < n ? N_b : n;
    unsigned long long *key = ws + (int64_t)t * L;
    const T *q = Q + (int64_t)head * qs_h + i * qs_l;
    const T *Kg = K + (int64_t)(head / G) * ks_h;
    if (tid < D) s_q[tid] = recall_elem(q, tid);
    __syncthreads();

    // ---- 1. logits ----
    for (int j = tid; j < n; j += 256) {
        const T *kr = Kg + (int64_t)j * ks_l;
        double acc = 0.0;
        for (int d = 0; d < D; ++d) acc += s_q[d] * recall_elem(kr, d);
        if (acc == 0.0) acc = 0.0;                           // -0.0 ties with +0.0
        unsigned long long u = (unsigned long long)__double_as_longlong(acc);
        key[j] = (u >> 63) ? ~u : (u | 0x8000000000000000ull);
    }
    __threadfence_block();
    __syncthreads();

    // ---- 2. threshold = the k_top-th largest key; above = keys larger than it; equal = keys equal to it ----
    unsigned long long prefix = 0ull;
    int above = 0, equal = n;
    for (int pass = 0; pass < 8; ++pass) {
        const int shift = 56 - 8 * pass;
        s_hist[tid] = 0;
        __syncthreads();
        for (int j = tid; j < n; j += 256) {
            const unsigned long long u = key[j];
            if (pass == 0 || (u >> (shift + 8)) == prefix) atomicAdd(&s_hist[(int)((u >> shift) & 255ull)], 1);
        }
        __syncthreads();
        const int d = 255 - tid, cnt = s_hist[d];            // suffix counts: thread t looks at digit 255 - t
        int total;
        const int gt = block_excl_scan(cnt, s_wave, &total); // keys of the region with a larger digit
        const int want = k_top - above;                      // still to be found inside the region (>= 1)
        if (gt < want && gt + cnt >= want) { s_digit = d; s_above = gt; s_equal = cnt; }
        __syncthreads();
        above += s_above;
        equal = s_equal;
        prefix = (prefix << 8) | (unsigned long long)s_digit;
        __syncthreads();
    }
    const unsigned long long thr = prefix;
    const int need_eq = k_top - above;                       // equal keys that belong to the top set: the lowest-indexed

    // ---- 3. the row's selected keys ----
    const int l = chunk_of_row(pv.RB, pv.N_q, i);
    const int v = (int)(i + 1 - pv.RB[l]);
    const int E = pv.count[(int64_t)head * pv.N_q + l];
    const int32_t *ent = pv.entries + ((int64_t)head * pv.N_q + l) * pv.stride * 2;
    int hits = 0;
    for (int e = 0; e < E; ++e) {
        const int w0 = ent[2 * e], rem = ent[2 * e + 1];
        const int k = w0 & kChunkMask, pos = w0 >> kPosShift;
        const int b0 = pv.B[k];
        int take = entry_take(pos, rem, pv.B[k + 1] - b0, v);
        if (pos == 3) {                                      // row-block form: listed keys above the row are masked
            const int64_t vis = i + 1 - b0;
            if (vis < take) take = vis > 0 ? (int)vis : 0;
        }
        for (int x = tid; x < take; x += 256) {
            const int j = b0 + x;
            const unsigned long long u = key[j];
            if (u > thr) ++hits;
            else if (u == thr) {
                if (need_eq >= equal) ++hits;                // every equal key is in the top set
                else {                                       // a tie cut by the budget: rank among the equal keys
                    int r = 0;
                    for (int jj = 0; jj < j; ++jj) r += key[jj] == thr;
                    if (r < need_eq) ++hits;
                }
            }
        }
    }
    int total;
    (void)block_excl_scan(hits, s_wave, &total);
    if (tid == 0) {
        hits_out[t] = total;
        size_out[t] = k_top;
    }
}

hipError_t launch_recall(const Prob &p, const PlanView &pv, const void *Q, const void *K, int head,
                         const int64_t *rows_dev, int n_rows, unsigned long long *ws, int32_t *hits, int32_t *size,
                         hipStream_t s) {
    if (n_rows == 0) return hipSuccess;
    if (p.dtype == DHSA_F32)
        hipLaunchKernelGGL(k_recall<float>, dim3(n_rows), dim3(256), 0, s, pv, (const float *)Q, (const float *)K,
                           p.N_b, p.G, p.D, head, rows_dev, p.L, ws, hits, size, p.qs_h, p.qs_l, p.ks_h, p.ks_l);
    else
        hipLaunchKernelGGL(k_recall<uint16_t>, dim3(n_rows), dim3(256), 0, s, pv, (const uint16_t *)Q,
                           (const uint16_t *)K, p.N_b, p.G, p.D, head, rows_dev, p.L, ws, hits, size, p.qs_h, p.qs_l,
                           p.ks_h, p.ks_l);
    return hipGetLastError();
}

}  // namespace dhsa
