// Internal declarations shared by the HIP translation units of libdhsa.
// Nothing here is part of the C ABI (see include/dhsa.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dhsa.h"

namespace dhsa {

constexpr int kRowTile = DHSA_ROW_TILE;  // query rows per attention workgroup
constexpr int kMaxChunks = 8192;         // N_c limit (LDS ranking of one query chunk)
constexpr int kPosShift = 28;            // plan entry word 0 = chunk id | pos << 28
constexpr int kChunkMask = (1 << kPosShift) - 1;

// Resolved problem: strides filled in, budget clamped, scale chosen.
struct Prob {
    int64_t L;
    int H_q, H_kv, G, D, N_c, N_b;  // N_b already clamped to L
    int B_r, N_q;                   // row-block size (0 = query groups are the chunks), query groups
    int pooling;                    // dhsa_pooling
    int dtype;
    float scale;
    int64_t qs_h, qs_l, ks_h, ks_l, vs_h, vs_l, os_h, os_l;
};

constexpr int kPlanHeaderWords = DHSA_PLAN_HEADER_WORDS;

// Word offsets inside the plan buffer (see the layout comment in dhsa.h).
struct PlanLayout {
    int stride;       // entries per (h, l)
    int T1;           // row tiles per head
    int T_big;        // ... of which have more than 64 rows (listed first)
    int T_cls[4];     // tiles of > 96, 65..96, 33..64 and <= 32 rows: the order of the tile table
    int N_q;          // query groups (chunks, or row blocks)
    int guess;        // chunks the ranking kernel lists first (see first_list_guess in dhsa_api.hip)
    int b_sum;        // checksum of the boundaries (header word 17)
    int64_t off_B, off_RB, off_count, off_entries, off_tiles, words;
};

// What the caller's problem says a plan must have been built for.  Every kernel that reads a plan
// compares this with the plan's header first and leaves without writing anything if they differ
// (a plan routed for another budget, row-block size, representation or boundary array of equal
// size would otherwise be used silently).
struct PlanSig {
    int32_t H_q, N_c, N_b, L, B_r, N_q, pooling, b_sum, stride, T1;
};

// Device-side view of a plan.
struct PlanView {
    const int32_t *hdr;      // [kPlanHeaderWords]
    PlanSig sig;
    const int32_t *B;        // [N_c + 1] key chunk boundaries
    const int32_t *RB;       // [N_q + 1] query group boundaries (== B when the groups are the chunks)
    const int32_t *count;    // [H_q][N_q]
    const int32_t *entries;  // [H_q][N_q][stride][2]
    const int32_t *tiles;    // [T1][2]: tiles of > 96 rows, then 65..96, 33..64, <= 32 rows (T_cls of each)
    int stride, T1, T_big, N_q;
    int T_cls[4];
};

// Workspace layout in doubles.
struct WsLayout {
    int64_t off_Qc, off_Kc, off_Sc, doubles;
};

// Decode workspace (byte offsets).  Kc persists between steps; the rest is scratch of one step.
// The "plan" is a one-group plan: B [N_c_cap + 1], RB [2], count [H_q], entries [H_q][stride][2]
// (room for stride = N_c_cap), laid out by `pl` in words from off_plan.
struct DecodeLayout {
    int64_t off_Kc, off_Qc, off_Sc, off_plan, off_part, bytes;
    PlanLayout pl;
    int S_cap;   // most key slices (workgroups per head) of the attention step
};
constexpr int kDecSlice = 128;   // selected keys per workgroup of the decode attention step
// Boundaries B[kc_valid .. kc_valid + n] of the chunks a decoding step pools anew, passed by
// value when they are few (n = 0: the kernels read all boundaries from the workspace).
constexpr int kBoundaryTailMax = 6;
struct BoundaryTail {
    int n;
    int32_t b[kBoundaryTailMax + 1];
};

// Up to kBoundaryBlockMax boundaries passed by value to a kernel (a launch argument block
// holds at most 4 KiB), for callers whose boundary array must not go through a host copy.
constexpr int kBoundaryBlockMax = 960;
struct BoundaryBlock {
    int32_t first, n;
    int32_t b[kBoundaryBlockMax];
};

// ---- launchers (each enqueues on `s` and returns the launch status) ----
// B_host[0 .. n) -> B_dev, carried by kernel arguments (no copy engine, no staging buffer)
hipError_t launch_put_boundaries(const int32_t *B_host, int n, int32_t *B_dev, hipStream_t s);
hipError_t launch_setup(const Prob &p, const PlanLayout &pl, int32_t *plan, hipStream_t s);
hipError_t launch_pool(const Prob &p, const void *Q, const void *K, const int32_t *B_dev, const int32_t *RB_dev,
                       double *Qc, double *Kc, hipStream_t s);
hipError_t launch_scores(const Prob &p, const double *Qc, const double *Kc, const int32_t *B_dev,
                         const int32_t *RB_dev, double *Sc, hipStream_t s);
hipError_t launch_select(const Prob &p, const PlanLayout &pl, const double *Sc, int32_t *plan, hipStream_t s);
// query groups [l_first, l_first + n_groups) only; `pl`, `Sc` and `plan` are indexed by group - l_first
hipError_t launch_select_groups(const Prob &p, const PlanLayout &pl, const double *Sc, int32_t *plan, int l_first,
                                int n_groups, hipStream_t s);
// one decoding step: the kernels of decode.hip (pooling of the new chunks and the open query group,
// scores of that group, and after the ranking the attention of the newest row)
// rb0 = first row of the open query group; the boundaries are already in the step's plan
hipError_t launch_decode_route(const Prob &p, const DecodeLayout &dl, int N_c_cap, int kc_valid, int rb0,
                               const BoundaryTail &tail, const void *Q, const void *K, void *ws, hipStream_t s);
hipError_t launch_decode_attend(const Prob &p, const DecodeLayout &dl, int rb0, const void *Q, const void *K,
                                const void *V, void *ws, void *O_row, int32_t *idx, int32_t *cnt, hipStream_t s);
hipError_t launch_expand(const Prob &p, const PlanView &pv, int head, const int64_t *rows_dev, int n_rows,
                         int32_t *idx, int cap, int32_t *cnt, hipStream_t s);
hipError_t launch_recall(const Prob &p, const PlanView &pv, const void *Q, const void *K, int head,
                         const int64_t *rows_dev, int n_rows, unsigned long long *ws, int32_t *hits, int32_t *size,
                         hipStream_t s);
hipError_t launch_attn_rowwise(const Prob &p, const PlanView &pv, const void *Q, const void *K, const void *V,
                               void *O, hipStream_t s);
// ev (may be null): three events recorded after the launches of the tiles of more than 64 rows, of
// 33..64 rows and of at most 32 rows
hipError_t launch_attn_mfma(const Prob &p, const PlanView &pv, const void *Q, const void *K, const void *V,
                            void *O, hipStream_t s, hipEvent_t *ev = nullptr);

// ---- small device helpers ----
// bf16 storage type (a bare 16-bit pattern; the kernels convert by hand)
struct bf16_t { uint16_t bits; };

// 16 bytes of a row as fp64 addends (the pooling kernels accumulate in fp64)
template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kPer16 = 4;
    __device__ static void unpack(const uint4 &u, double *acc) {
        acc[0] += (double)__uint_as_float(u.x);
        acc[1] += (double)__uint_as_float(u.y);
        acc[2] += (double)__uint_as_float(u.z);
        acc[3] += (double)__uint_as_float(u.w);
    }
};
template <> struct Elem<bf16_t> {
    static constexpr int kPer16 = 8;
    __device__ static void unpack(const uint4 &u, double *acc) {
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[2 * i] += (double)__uint_as_float(w[i] << 16);
            acc[2 * i + 1] += (double)__uint_as_float(w[i] & 0xffff0000u);
        }
    }
};

__device__ __forceinline__ int chunk_of_row(const int32_t *__restrict__ B, int N_c, int64_t i) {
    int lo = 0, hi = N_c;  // B[lo] <= i < B[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if ((int64_t)B[mid] <= i) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ bool plan_matches(const PlanView &pv) {
    const int32_t *w = pv.hdr;
    return w[0] == DHSA_PLAN_MAGIC && w[1] == DHSA_PLAN_VERSION && w[2] == pv.sig.H_q && w[3] == pv.sig.N_c &&
           w[4] == pv.sig.N_b && w[5] == pv.sig.stride && w[6] == pv.sig.L && w[7] == pv.sig.T1 &&
           w[14] == pv.sig.N_q && w[15] == pv.sig.B_r && w[16] == pv.sig.pooling && w[17] == pv.sig.b_sum;
}

// Class of a row tile by its number of rows (1..128): the attention kernels give each class its
// own arrangement of waves.  0: more than 96 rows, 1: 65..96, 2: 33..64, 3: at most 32.
__host__ __device__ __forceinline__ int tile_class(int rows) {
    return rows > 96 ? 0 : rows > 64 ? 1 : rows > 32 ? 2 : 3;
}

// Tokens row (visible own-chunk count v) takes from a plan entry.  For pos = 3
// (row-block form) rem is the number of listed tokens, never above len_k; the
// causal mask is applied per token by the caller.
__device__ __forceinline__ int entry_take(int pos, int rem, int len_k, int v) {
    int lim = (pos == 1) ? v : len_k;
    int room = (pos == 2) ? rem - v : rem;
    int t = room < lim ? room : lim;
    return t > 0 ? t : 0;
}

// Exclusive prefix sum of one int per thread over a 256-thread block (wave
// shuffles + one LDS slot per wave).  `total` receives the block sum.  Contains
// two block barriers; s_wave is an int[4] in LDS.
__device__ __forceinline__ int block_excl_scan(int val, int *s_wave, int *total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = val;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int t = __shfl_up(inc, off);
        if (lane >= off) inc += t;
    }
    __syncthreads();  // protects s_wave from its previous use
    if (lane == 63) s_wave[wave] = inc;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        int x = s_wave[w];
        if (w < wave) base += x;
        tot += x;
    }
    *total = tot;
    return base + inc - val;
}

// Two exclusive prefix sums at once (same barriers as one).
__device__ __forceinline__ void block_excl_scan2(int a, int b, int *s_wave8, int *excl_a, int *excl_b, int *total_a,
                                                 int *total_b) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int ia = a, ib = b;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int ta = __shfl_up(ia, off), tb = __shfl_up(ib, off);
        if (lane >= off) { ia += ta; ib += tb; }
    }
    __syncthreads();  // protects s_wave8 from its previous use
    if (lane == 63) { s_wave8[wave] = ia; s_wave8[4 + wave] = ib; }
    __syncthreads();
    int base_a = 0, base_b = 0, tot_a = 0, tot_b = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const int xa = s_wave8[w], xb = s_wave8[4 + w];
        if (w < wave) { base_a += xa; base_b += xb; }
        tot_a += xa; tot_b += xb;
    }
    *total_a = tot_a; *total_b = tot_b;
    *excl_a = base_a + ia - a;
    *excl_b = base_b + ib - b;
}

}  // namespace dhsa
