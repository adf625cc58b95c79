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
// monotone runs it takes a handful of rounds.  A round only visits the 64-position
// blocks in which something can change: a candidate can become the best of its
// neighbourhood only after a better neighbour was removed, so the blocks within W
// of a removal are the next round's work list (three bitmaps in the workspace);
// a long monotone run then costs one cheap round per chunk end instead of a pass
// over the sequence.  One workgroup of 1024 threads does all of it (the state is
// one byte per position in the caller's workspace and stays in L2); it runs once
// per prompt, not once per layer.
#include "dhsa_internal.h"

namespace dhsa {

constexpr int kNmsThreads = 1024;
constexpr int kNmsWaves = kNmsThreads / 64;
enum : uint8_t { kOut = 0, kUndecided = 1, kKept = 2, kNewKept = 3 };

// set the bits of the 64-position blocks that intersect positions [lo, hi]
__device__ __forceinline__ void nms_mark(unsigned *bits, int64_t lo, int64_t hi) {
    for (int64_t b = lo >> 6; b <= (hi >> 6); ++b) atomicOr(&bits[b >> 5], 1u << (b & 31));
}

// Calls body(block) for every block whose bit is set, a whole wave per block, the
// waves sharing the blocks in groups of 64.
#define DHSA_NMS_FOR_BLOCKS(bits, ...)                                                           \
    for (int64_t g0_ = (int64_t)wave * 64; g0_ < NB; g0_ += (int64_t)kNmsWaves * 64) {           \
        const int64_t mine_ = g0_ + lane;                                                        \
        const bool set_ = mine_ < NB && ((bits[mine_ >> 5] >> (mine_ & 31)) & 1u);               \
        unsigned long long m_ = __ballot(set_);                                                  \
        while (m_) {                                                                             \
            const int64_t blk = g0_ + __builtin_ctzll(m_);                                       \
            m_ &= m_ - 1;                                                                        \
            __VA_ARGS__                                                                          \
        }                                                                                        \
    }

__global__ __launch_bounds__(kNmsThreads) void k_finalize_boundaries(const float *__restrict__ p, int64_t L,
                                                                     float tau, int W, uint8_t *st,
                                                                     unsigned *bits0, unsigned *bits1,
                                                                     unsigned *bits2, int32_t *__restrict__ B_out,
                                                                     int32_t *__restrict__ N_c_out) {
    __shared__ int s_cnt[kNmsWaves];
    __shared__ int s_und;          // candidates still undecided
    __shared__ int s_any;          // does the next round have a block to visit?
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t NB = (L + 63) >> 6, NW = (NB + 31) >> 5;   // 64-position blocks, bitmap words
    unsigned *dirtyA = bits0, *dirtyB = bits1, *dirtyN = bits2;   // visit now / near a new chunk end / visit next

    // candidates: score strictly above the threshold (a NaN never is); every block is visited in the first pass
    int und = 0;
    for (int64_t i = tid; i < L; i += kNmsThreads) {
        const bool c = p[i] > tau;
        st[i] = c ? kUndecided : kOut;
        und += c;
    }
    for (int64_t w = tid; w < NW; w += kNmsThreads) { dirtyA[w] = 0xffffffffu; dirtyB[w] = 0u; dirtyN[w] = 0u; }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) und += __shfl_xor(und, off);
    if (lane == 0) s_cnt[wave] = und;
    __syncthreads();
    if (tid == 0) {
        int t = 0;
        for (int w = 0; w < kNmsWaves; ++w) t += s_cnt[w];
        s_und = t;
    }
    __syncthreads();
    int und_now = s_und;           // read between two barriers: nobody changes s_und before the second one,
    __syncthreads();               // so every thread takes the same decision at the loop head

    while (und_now > 0) {
        if (tid == 0) s_any = 0;   // set again only in phase 2, behind the next barrier
        // ---- phase 1: an undecided candidate that beats every undecided neighbour becomes a chunk end ----
        DHSA_NMS_FOR_BLOCKS(dirtyA, {
            const int64_t i = blk * 64 + lane;
            bool best = false;
            if (i < L && st[i] == kUndecided) {
                const float pi = p[i];
                const int64_t lo = i - W < 0 ? 0 : i - W, hi = i + W > L - 1 ? L - 1 : i + W;
                best = true;
                for (int64_t j = lo; j <= hi && best; ++j) {
                    if (j == i) continue;
                    const uint8_t sj = st[j];   // a neighbour marked in this phase still counts as a rival
                    if (sj != kUndecided && sj != kNewKept) continue;
                    const float pj = p[j];
                    if (pj > pi || (pj == pi && j < i)) best = false;
                }
                if (best) {
                    st[i] = kNewKept;
                    nms_mark(dirtyB, lo, hi);
                }
            }
            const int n_ = __popcll(__ballot(best));
            if (lane == 0 && n_) atomicSub(&s_und, n_);
        })
        __threadfence_block();
        __syncthreads();
        // ---- phase 2: undecided candidates within W tokens of a new chunk end are removed ----
        DHSA_NMS_FOR_BLOCKS(dirtyB, {
            const int64_t j = blk * 64 + lane;
            bool hit = false;
            if (j < L && st[j] == kUndecided) {
                const int64_t lo = j - W < 0 ? 0 : j - W, hi = j + W > L - 1 ? L - 1 : j + W;
                for (int64_t x = lo; x <= hi && !hit; ++x) hit = st[x] == kNewKept;
                if (hit) {
                    st[j] = kOut;
                    nms_mark(dirtyN, lo, hi);   // its neighbours may now be the best of their neighbourhood
                }
            }
            const int n_ = __popcll(__ballot(hit));
            if (lane == 0 && n_) { atomicSub(&s_und, n_); s_any = 1; }
        })
        __threadfence_block();
        __syncthreads();
        // ---- phase 3: the new chunk ends become plain ones; rotate the work lists ----
        DHSA_NMS_FOR_BLOCKS(dirtyA, {
            const int64_t i = blk * 64 + lane;
            if (i < L && st[i] == kNewKept) st[i] = kKept;
        })
        __threadfence_block();
        __syncthreads();
        {
            unsigned *t_ = dirtyA;
            dirtyA = dirtyN;
            dirtyN = t_;
        }
        // no removal but candidates left cannot happen (the best undecided candidate is always
        // visited); should it, every block is visited again rather than looping forever
        und_now = s_und;
        const unsigned fill = (s_any || und_now == 0) ? 0u : 0xffffffffu;
        for (int64_t w = tid; w < NW; w += kNmsThreads) {
            dirtyB[w] = 0u;
            dirtyN[w] = 0u;
            if (fill) dirtyA[w] = fill;
        }
        __threadfence_block();
        __syncthreads();
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

namespace {
// workspace: one state byte per position, then three bitmaps with one bit per 64 positions
int64_t nms_state_bytes(int64_t L) { return (L + 255) / 256 * 256; }
int64_t nms_bitmap_bytes(int64_t L) { return (((((L + 63) >> 6) + 31) >> 5) * 4 + 255) / 256 * 256; }
}  // namespace

extern "C" __attribute__((visibility("default"))) size_t dhsa_finalize_boundaries_workspace_bytes(int64_t L) {
    return L >= 1 && L < ((int64_t)1 << 31) ? (size_t)(nms_state_bytes(L) + 3 * nms_bitmap_bytes(L)) : 0;
}

extern "C" __attribute__((visibility("default"))) dhsa_status dhsa_finalize_boundaries(
    const float *scores_dev, int64_t L, float threshold, int32_t window, int32_t *B_dev, int32_t *N_c_dev,
    void *ws_dev, size_t ws_bytes, void *stream) {
    using namespace dhsa;
    if (!scores_dev || !B_dev || !N_c_dev || !ws_dev) return DHSA_ERR_NULL;
    if (L < 1 || L >= ((int64_t)1 << 31) || window < 0 || threshold != threshold) return DHSA_ERR_SHAPE;
    if (ws_bytes < dhsa_finalize_boundaries_workspace_bytes(L)) return DHSA_ERR_WORKSPACE;
    uint8_t *st = (uint8_t *)ws_dev;
    unsigned *bits = (unsigned *)(st + nms_state_bytes(L));
    const int64_t bw = nms_bitmap_bytes(L) / 4;
    hipLaunchKernelGGL(k_finalize_boundaries, dim3(1), dim3(kNmsThreads), 0, (hipStream_t)stream, scores_dev, L,
                       threshold, (int)window, st, bits, bits + bw, bits + 2 * bw, B_dev, N_c_dev);
    return hipGetLastError() == hipSuccess ? DHSA_OK : DHSA_ERR_HIP;
}
