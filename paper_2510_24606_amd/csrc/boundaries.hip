// Boundary finalisation of libdhsa: boundary scores -> chunk boundaries B
// (Sec. 3.2 "Inference Pipeline"; App. "Inference of the Boundary Predictor":
// drop the positions whose score does not exceed a threshold, visit the rest by
// descending score, keep a position and remove every other candidate within W
// tokens of it).
//
// The greedy is sequential as stated; its result is the unique set in which a
// candidate is kept iff no better candidate within W tokens of it is kept
// ("better" = higher score, equal scores: lower position).  That set is built
// in rounds, all positions in parallel: a still undecided candidate that is
// better than every undecided candidate within W tokens is kept (nothing can
// remove it any more), then every undecided candidate within W tokens of a
// newly kept one is removed.  The best undecided candidate of the whole
// sequence is decided in every round, so the loop ends; on scores without long
// monotone runs it takes a handful of rounds.  One workgroup of 1024 threads
// does all of it (the state is one byte per position in the caller's
// workspace and stays in L2); it runs once per prompt, not once per layer.
#include "dhsa_internal.h"

namespace dhsa {

constexpr int kNmsThreads = 1024;
enum : uint8_t { kOut = 0, kUndecided = 1, kKept = 2, kNewKept = 3 };

__global__ __launch_bounds__(kNmsThreads) void k_finalize_boundaries(const float *__restrict__ p, int64_t L,
                                                                     float tau, int W, uint8_t *st,
                                                                     int32_t *__restrict__ B_out,
                                                                     int32_t *__restrict__ N_c_out) {
    __shared__ int s_cnt[kNmsThreads / 64];
    __shared__ int s_total;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // candidates: score strictly above the threshold (a NaN never is)
    int undecided = 0;
    for (int64_t i = tid; i < L; i += kNmsThreads) {
        const bool c = p[i] > tau;
        st[i] = c ? kUndecided : kOut;
        undecided += c;
    }
    for (;;) {
        // ---- how many candidates are still undecided (block-wide sum; also orders the state writes) ----
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) undecided += __shfl_xor(undecided, off);
        __syncthreads();                       // s_cnt free again; state writes of the last phase visible
        if (lane == 0) s_cnt[wave] = undecided;
        __syncthreads();
        if (tid == 0) {
            int t = 0;
            for (int w = 0; w < kNmsThreads / 64; ++w) t += s_cnt[w];
            s_total = t;
        }
        __syncthreads();
        if (s_total == 0) break;               // block-uniform

        // ---- phase 1: an undecided candidate that beats every undecided neighbour is kept ----
        for (int64_t i = tid; i < L; i += kNmsThreads) {
            if (st[i] != kUndecided) continue;
            const float pi = p[i];
            const int64_t lo = i - W < 0 ? 0 : i - W, hi = i + W > L - 1 ? L - 1 : i + W;
            bool best = true;
            for (int64_t j = lo; j <= hi && best; ++j) {
                if (j == i) continue;
                const uint8_t sj = st[j];      // a neighbour marked kNewKept in this phase still counts as a rival
                if (sj != kUndecided && sj != kNewKept) continue;
                const float pj = p[j];
                if (pj > pi || (pj == pi && j < i)) best = false;
            }
            if (best) st[i] = kNewKept;
        }
        __threadfence_block();
        __syncthreads();
        // ---- phase 2: undecided candidates within W tokens of a newly kept one are removed ----
        undecided = 0;
        for (int64_t i = tid; i < L; i += kNmsThreads) {
            if (st[i] != kUndecided) continue;
            const int64_t lo = i - W < 0 ? 0 : i - W, hi = i + W > L - 1 ? L - 1 : i + W;
            bool hit = false;
            for (int64_t j = lo; j <= hi && !hit; ++j) hit = st[j] == kNewKept;
            if (hit) st[i] = kOut; else ++undecided;
        }
        __threadfence_block();
        __syncthreads();
        for (int64_t i = tid; i < L; i += kNmsThreads)
            if (st[i] == kNewKept) st[i] = kKept;
        __threadfence_block();
    }

    // ---- boundaries in the half-open convention: 0, (kept end + 1) ..., L; ascending ----
    // consecutive slabs of kNmsThreads positions, exclusive scan of the kept flags within a slab
    int base = 1;                              // B_out[0] = 0
    for (int64_t s0 = 0; s0 < L - 1; s0 += kNmsThreads) {   // position L-1 is the end of the sequence anyway
        const int64_t i = s0 + tid;
        const int flag = (i < L - 1) && st[i] == kKept;
        int inc = flag;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int t = __shfl_up(inc, off);
            if (lane >= off) inc += t;
        }
        __syncthreads();
        if (lane == 63) s_cnt[wave] = inc;
        __syncthreads();
        int before = 0, total = 0;
        for (int w = 0; w < kNmsThreads / 64; ++w) {
            const int x = s_cnt[w];
            if (w < wave) before += x;
            total += x;
        }
        if (flag) B_out[base + before + inc - 1] = (int32_t)(i + 1);
        base += total;
    }
    if (tid == 0) {
        B_out[0] = 0;
        B_out[base] = (int32_t)L;
        *N_c_out = base;
    }
}

}  // namespace dhsa

extern "C" __attribute__((visibility("default"))) size_t dhsa_finalize_boundaries_workspace_bytes(int64_t L) {
    return L >= 1 && L < ((int64_t)1 << 31) ? (size_t)((L + 255) / 256 * 256) : 0;
}

extern "C" __attribute__((visibility("default"))) dhsa_status dhsa_finalize_boundaries(
    const float *scores_dev, int64_t L, float threshold, int32_t window, int32_t *B_dev, int32_t *N_c_dev,
    void *ws_dev, size_t ws_bytes, void *stream) {
    using namespace dhsa;
    if (!scores_dev || !B_dev || !N_c_dev || !ws_dev) return DHSA_ERR_NULL;
    if (L < 1 || L >= ((int64_t)1 << 31) || window < 0 || threshold != threshold) return DHSA_ERR_SHAPE;
    if (ws_bytes < dhsa_finalize_boundaries_workspace_bytes(L)) return DHSA_ERR_WORKSPACE;
    hipLaunchKernelGGL(k_finalize_boundaries, dim3(1), dim3(kNmsThreads), 0, (hipStream_t)stream, scores_dev, L,
                       threshold, (int)window, (uint8_t *)ws_dev, B_dev, N_c_dev);
    return hipGetLastError() == hipSuccess ? DHSA_OK : DHSA_ERR_HIP;
}
