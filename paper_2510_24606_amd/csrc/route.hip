// Routing kernels of libdhsa: plan set-up, chunk pooling (Sec. 3.3 Eq. 4),
// chunk similarity S_c = Q_c K_c^T (Sec. 3.3), ranking and per-row budget
// (Sec. 3.1 Step 2, Alg. 1), and the plan -> index-set expansion hook.
//
// All routing arithmetic is fp64: pooled sums of bf16 inputs are then exact
// (order-free), and S_c carries ~1e-14 absolute error, so the ranking does not
// hinge on summation order.
#include <algorithm>
#include "dhsa_internal.h"

namespace dhsa {

typedef double f64x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// Plan header, query-group boundaries and row-tile table.  One block; B is
// already in the plan.  The query groups are the chunks themselves, or (Alg. 1
// as printed) row blocks of B_r rows, RB[i] = min(i B_r, L).  Tiles are the
// <= 128-row pieces of the query groups; the table lists them by class -- more
// than 96 rows, 65..96, 33..64, at most 32 -- each class ordered by row.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_setup(int32_t *__restrict__ plan, PlanLayout pl, int H_q, int H_kv, int D,
                                               int N_c, int N_b, int64_t L, int B_r, int pooling) {
    __shared__ int s_n[4][256];    // tiles of each class per query group of the slab (scanned in place)
    __shared__ int s_carry[4];
    const int tid = threadIdx.x;
    const int N_q = pl.N_q;
    int32_t *tiles = plan + pl.off_tiles;
    if (B_r > 0) {
        int32_t *RBw = plan + pl.off_RB;
        for (int i = tid; i <= N_q; i += 256) {
            const int64_t b = (int64_t)i * B_r;
            RBw[i] = (int32_t)(b < L ? b : L);
        }
        __syncthreads();
    }
    const int32_t *B = plan + pl.off_RB;   // the boundaries the rows are grouped by
    if (tid < kPlanHeaderWords) {
        int32_t w = 0;
        switch (tid) {
            case 0: w = DHSA_PLAN_MAGIC; break;
            case 1: w = DHSA_PLAN_VERSION; break;
            case 2: w = H_q; break;
            case 3: w = N_c; break;
            case 4: w = N_b; break;
            case 5: w = pl.stride; break;
            case 6: w = (int32_t)L; break;
            case 7: w = pl.T1; break;
            case 8: w = (int32_t)pl.off_B; break;
            case 9: w = (int32_t)pl.off_count; break;
            case 10: w = (int32_t)pl.off_entries; break;
            case 11: w = (int32_t)pl.off_tiles; break;
            case 12: w = pl.T_big; break;
            case 13: w = (int32_t)pl.off_RB; break;
            case 14: w = N_q; break;
            case 15: w = B_r; break;
            case 16: w = pooling; break;
            case 17: w = pl.b_sum; break;
            case 18: w = H_kv; break;
            case 19: w = D; break;
            case 20: case 21: case 22: case 23: w = pl.T_cls[tid - 20]; break;
            default: break;
        }
        plan[tid] = w;
    }
    if (tid == 0) {   // where each class starts in the table
        s_carry[0] = 0;
        s_carry[1] = pl.T_cls[0];
        s_carry[2] = pl.T_cls[0] + pl.T_cls[1];
        s_carry[3] = pl.T_cls[0] + pl.T_cls[1] + pl.T_cls[2];
    }
    __syncthreads();
    for (int base = 0; base < N_q; base += 256) {
        const int l = base + tid;
        int b0 = 0, nfull = 0, rem = 0;
        if (l < N_q) {
            b0 = B[l];
            const int len = B[l + 1] - b0;
            nfull = len / kRowTile;
            rem = len % kRowTile;
        }
        const int rem_cls = rem > 0 ? tile_class(rem) : -1;
        int mine[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            mine[c] = (c == 0 ? nfull : 0) + (rem_cls == c);
            s_n[c][tid] = mine[c];
        }
        __syncthreads();
        // Hillis-Steele inclusive scans over the 256 slab entries
        for (int off = 1; off < 256; off <<= 1) {
            int v[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) v[c] = (tid >= off) ? s_n[c][tid - off] : 0;
            __syncthreads();
#pragma unroll
            for (int c = 0; c < 4; ++c) s_n[c][tid] += v[c];
            __syncthreads();
        }
        int at = s_carry[0] + s_n[0][tid] - mine[0];
        for (int t = 0; t < nfull; ++t) {
            tiles[2 * (at + t)] = l;
            tiles[2 * (at + t) + 1] = b0 + t * kRowTile;
        }
        if (rem_cls >= 0) {
            at = s_carry[rem_cls] + s_n[rem_cls][tid] - 1;
            tiles[2 * at] = l;
            tiles[2 * at + 1] = b0 + nfull * kRowTile;
        }
        __syncthreads();
        if (tid == 255) {
#pragma unroll
            for (int c = 0; c < 4; ++c) s_carry[c] += s_n[c][255];
        }
        __syncthreads();
    }
}

hipError_t launch_setup(const Prob &p, const PlanLayout &pl, int32_t *plan, hipStream_t s) {
    hipLaunchKernelGGL(k_setup, dim3(1), dim3(256), 0, s, plan, pl, p.H_q, p.H_kv, p.D, p.N_c, p.N_b, p.L, p.B_r,
                       p.pooling);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Boundaries into the plan without a copy from host memory: each launch carries
// up to kBoundaryBlockMax of them as kernel arguments.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_put_boundaries(int32_t *__restrict__ dst, BoundaryBlock blk) {
    for (int i = threadIdx.x; i < blk.n; i += 256) dst[blk.first + i] = blk.b[i];
}

hipError_t launch_put_boundaries(const int32_t *B_host, int n, int32_t *B_dev, hipStream_t s) {
    BoundaryBlock blk;
    for (int first = 0; first < n; first += kBoundaryBlockMax) {
        blk.first = first;
        blk.n = std::min(kBoundaryBlockMax, n - first);
        for (int i = 0; i < blk.n; ++i) blk.b[i] = B_host[first + i];
        for (int i = blk.n; i < kBoundaryBlockMax; ++i) blk.b[i] = 0;
        hipLaunchKernelGGL(k_put_boundaries, dim3(1), dim3(256), 0, s, B_dev, blk);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---------------------------------------------------------------------------
// Chunk pooling, Eq. 4: X_c[h, k, :] = (sqrt(len)/len) * sum_{i in chunk k} X[h, i, :].
// One block per (chunk, head); a row of D elements is read by D*sizeof(T)/16
// threads with 16-byte loads, row groups are summed through LDS.  HBM-bound.
// Keys are pooled over the chunks B; queries over the query groups RB (the
// chunks again, or with B_r > 0 the row blocks of Alg. 1, whose representation
// is sqrt(B_r) * mean of the block's rows).
// ---------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void k_pool(const T *__restrict__ Q, const T *__restrict__ K,
                                              const int32_t *__restrict__ B, const int32_t *__restrict__ RB,
                                              double *__restrict__ Qc, double *__restrict__ Kc, int H_q, int N_c,
                                              int N_q, int B_r, int pooling, int64_t qs_h, int64_t qs_l,
                                              int64_t ks_h, int64_t ks_l) {
    constexpr int EPT = Elem<T>::kPer16;   // elements per thread per row
    constexpr int TPR = D / EPT;           // threads per row
    constexpr int RG = 256 / TPR;          // rows in flight
    __shared__ double s_sum[RG][D];
    const int k = blockIdx.x;
    int h = blockIdx.y;
    const T *X;
    double *Xc;
    int64_t s_l;
    const bool is_q = h < H_q;
    if (k >= (is_q ? N_q : N_c)) return;   // block-uniform: the grid spans max(N_q, N_c)
    if (is_q) {
        X = Q + (int64_t)h * qs_h; s_l = qs_l; Xc = Qc + ((int64_t)h * N_q + k) * D;
    } else {
        h -= H_q;
        X = K + (int64_t)h * ks_h; s_l = ks_l; Xc = Kc + ((int64_t)h * N_c + k) * D;
    }
    const int32_t *Bx = is_q ? RB : B;
    const int b0 = Bx[k], b1 = Bx[k + 1];
    const int tid = threadIdx.x;
    const int rg = tid / TPR, col = (tid % TPR) * EPT;
    double acc[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) acc[e] = 0.0;
    for (int i = b0 + rg; i < b1; i += RG) {
        uint4 u = *reinterpret_cast<const uint4 *>(X + (int64_t)i * s_l + col);
        Elem<T>::unpack(u, acc);
    }
#pragma unroll
    for (int e = 0; e < EPT; ++e) s_sum[rg][col + e] = acc[e];
    __syncthreads();
    if (tid < D) {
        double sum = 0.0;
#pragma unroll 4
        for (int r = 0; r < RG; ++r) sum += s_sum[r][tid];
        const double len = (double)(b1 - b0);
        Xc[tid] = pooling == DHSA_POOL_MEAN ? sum / len                                  // plain average (ablation)
                  : (is_q && B_r > 0)      ? sqrt((double)B_r) * (sum / len)            // Alg. 1 row blocks
                                           : (sqrt(len) / len) * sum;                   // Eq. 4
    }
}

hipError_t launch_pool(const Prob &p, const void *Q, const void *K, const int32_t *B_dev, const int32_t *RB_dev,
                       double *Qc, double *Kc, hipStream_t s) {
    dim3 grid(p.N_q > p.N_c ? p.N_q : p.N_c, p.H_q + p.H_kv), block(256);
#define DHSA_POOL(T, DD)                                                                                  \
    hipLaunchKernelGGL((k_pool<T, DD>), grid, block, 0, s, (const T *)Q, (const T *)K, B_dev, RB_dev, Qc, \
                       Kc, p.H_q, p.N_c, p.N_q, p.B_r, p.pooling, p.qs_h, p.qs_l, p.ks_h, p.ks_l)
    if (p.dtype == DHSA_F32) {
        if (p.D == 64) DHSA_POOL(float, 64); else DHSA_POOL(float, 128);
    } else {
        if (p.D == 64) DHSA_POOL(bf16_t, 64); else DHSA_POOL(bf16_t, 128);
    }
#undef DHSA_POOL
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Chunk similarity S_c[h, l, k] = <Q_c[h, l], K_c[h / G, k]> for the key chunks
// k that some row of query group l can see (B[k] < RB[l+1]; with the chunks as
// query groups that is k <= l), fp64 MFMA (16x16x4).  A 64 x 64 output tile per
// block; four waves in a 2 x 2 arrangement, each 32 x 32 = 2 x 2 MFMA blocks.
// Tiles none of whose pairs is visible are skipped.
// ---------------------------------------------------------------------------
constexpr int kScTile = 64;
constexpr int kScKc = 32;   // reduction slab staged in LDS
constexpr int kScPad = 1;

__global__ __launch_bounds__(256) void k_scores(const double *__restrict__ Qc, const double *__restrict__ Kc,
                                                const int32_t *__restrict__ B, const int32_t *__restrict__ RB,
                                                double *__restrict__ Sc, int N_c, int N_q, int D, int G) {
    const int k0 = blockIdx.x * kScTile, l0 = blockIdx.y * kScTile, h = blockIdx.z;
    {
        const int l_last = (l0 + kScTile < N_q ? l0 + kScTile : N_q) - 1;   // last query group of the tile
        if (B[k0] >= RB[l_last + 1]) return;                                // its first chunk starts past every row
    }
    __shared__ double sA[kScTile][kScKc + kScPad];
    __shared__ double sB[kScTile][kScKc + kScPad];
    const double *A = Qc + (int64_t)h * N_q * D;
    const double *Bm = Kc + (int64_t)(h / G) * N_c * D;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wl = (wave >> 1) * 32, wk = (wave & 1) * 32;
    f64x4 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = (f64x4){0.0, 0.0, 0.0, 0.0};

    // 64 x 32 slabs of both operands go through registers into LDS (rows past the end read as
    // zero); the next slab is requested from memory before the current one is multiplied
    constexpr int kPerThread = kScTile * kScKc / 256;
    double ra[kPerThread], rb[kPerThread];
#define DHSA_SC_FETCH(d0_)                                                                      \
    _Pragma("unroll") for (int i = 0; i < kPerThread; ++i) {                                    \
        const int x = tid + 256 * i, r = x / kScKc, c = x % kScKc;                              \
        ra[i] = (l0 + r < N_q) ? A[(int64_t)(l0 + r) * D + (d0_) + c] : 0.0;                    \
        rb[i] = (k0 + r < N_c) ? Bm[(int64_t)(k0 + r) * D + (d0_) + c] : 0.0;                   \
    }
    DHSA_SC_FETCH(0)
    for (int d0 = 0; d0 < D; d0 += kScKc) {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const int x = tid + 256 * i, r = x / kScKc, c = x % kScKc;
            sA[r][c] = ra[i];
            sB[r][c] = rb[i];
        }
        __syncthreads();
        if (d0 + kScKc < D) DHSA_SC_FETCH(d0 + kScKc)
#pragma unroll
        for (int kk = 0; kk < kScKc; kk += 4) {
            double a[2], b[2];
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                a[m] = sA[wl + 16 * m + (lane & 15)][kk + (lane >> 4)];
                b[m] = sB[wk + 16 * m + (lane & 15)][kk + (lane >> 4)];
            }
#pragma unroll
            for (int m = 0; m < 2; ++m)
#pragma unroll
                for (int n = 0; n < 2; ++n)
                    acc[m][n] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[m], b[n], acc[m][n], 0, 0, 0);
        }
        __syncthreads();
    }
#undef DHSA_SC_FETCH
    // D[i][j]: accumulator element v of a lane is row 4*v + lane/16, column lane % 16
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                int l = l0 + wl + 16 * m + 4 * v + (lane >> 4);
                int k = k0 + wk + 16 * n + (lane & 15);
                if (l < N_q && k < N_c) Sc[((int64_t)h * N_q + l) * N_c + k] = acc[m][n][v];
            }
}

hipError_t launch_scores(const Prob &p, const double *Qc, const double *Kc, const int32_t *B_dev,
                         const int32_t *RB_dev, double *Sc, hipStream_t s) {
    const int ntk = (p.N_c + kScTile - 1) / kScTile, ntl = (p.N_q + kScTile - 1) / kScTile;
    hipLaunchKernelGGL(k_scores, dim3(ntk, ntl, p.H_q), dim3(256), 0, s, Qc, Kc, B_dev, RB_dev, Sc, p.N_c, p.N_q,
                       p.D, p.G);
    return hipGetLastError();
}

// Value of lane (lane ^ J) of the wave, J a power of two below 64: lane-crossing moves of the
// vector unit where there is one (quads, rows of 16), the LDS crossbar otherwise.
template <int J>
__device__ __forceinline__ int lane_xor(int v) {
    if constexpr (J == 1) return __builtin_amdgcn_mov_dpp(v, 0xB1, 0xf, 0xf, true);        // quad_perm [1,0,3,2]
    else if constexpr (J == 2) return __builtin_amdgcn_mov_dpp(v, 0x4E, 0xf, 0xf, true);   // quad_perm [2,3,0,1]
    else if constexpr (J == 4) return __builtin_amdgcn_ds_swizzle(v, 0x101F);              // xor 4 inside 32 lanes
    else if constexpr (J == 8) return __builtin_amdgcn_mov_dpp(v, 0x128, 0xf, 0xf, true);  // row_ror 8 == xor 8
    else if constexpr (J == 16) return __builtin_amdgcn_ds_swizzle(v, 0x401F);             // xor 16 inside 32 lanes
    else return __shfl_xor(v, 32);
}

// Bitonic sort of PS <= 256 (key, id) pairs, one per thread of the first PS threads, "first"
// = larger key, or equal key and smaller id.  In: skey[0..PS), sid[0..PS); out: the same
// arrays, sorted.  Exchanges at distances below 64 stay inside a wave, the few at 64 and 128
// go through the arrays.  Called by all 256 threads (barriers).
template <int PS, int SIZE, int J>
__device__ __forceinline__ void sort_step(unsigned long long &k, int &ci, unsigned long long *skey, int *sid,
                                          int tid, bool active) {
    unsigned long long pk = 0ull;
    int pi = 0;
    if constexpr (J < 64) {
        if (active) {
            const int lo = lane_xor<J>((int)(unsigned)k), hi = lane_xor<J>((int)(unsigned)(k >> 32));
            pk = ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo;
            pi = lane_xor<J>(ci);
        }
    } else {
        __syncthreads();           // the previous exchange has been read
        if (active) { skey[tid] = k; sid[tid] = ci; }
        __syncthreads();
        if (active) { pk = skey[tid ^ J]; pi = sid[tid ^ J]; }
    }
    if (active) {
        const bool first = (k > pk) || (k == pk && ci < pi);
        const bool want_first = ((tid & J) == 0) == ((tid & SIZE) == 0);
        if (first != want_first) { k = pk; ci = pi; }
    }
    if constexpr (J > 1) sort_step<PS, SIZE, J / 2>(k, ci, skey, sid, tid, active);
    else if constexpr (SIZE < PS) sort_step<PS, SIZE * 2, SIZE>(k, ci, skey, sid, tid, active);
}

template <int PS>
__device__ __forceinline__ void sort_in_registers(unsigned long long *skey, int *sid, int tid) {
    const bool active = tid < PS;      // PS is a multiple of 64: whole waves; the others only keep the barriers company
    unsigned long long k = active ? skey[tid] : 0ull;
    int ci = active ? sid[tid] : 0x7fffffff;
    sort_step<PS, 2, 1>(k, ci, skey, sid, tid, active);
    __syncthreads();
    if (active) { skey[tid] = k; sid[tid] = ci; }
    __syncthreads();
}

// ---------------------------------------------------------------------------
// Ranking + per-row budget for one (head, query chunk l): Alg. 1's Argsort and
// walk, done once for all rows of the chunk.
//   1. scores of key chunks 0..l -> LDS as order-preserving 64-bit integers;
//   2. only the best `stride` chunks can ever be listed (stride bounds the number
//      of chunks whose tokens fit the budget), so for rows of more than 256 chunks a
//      most-significant-digit radix select (8-bit digits, LDS histograms, prefix
//      scans) first cuts the row down to a candidate list: at first a short one,
//      sized for chunks of about the mean length (it is the answer whenever its
//      chunks hold the budget), else one of <= 512 that holds `stride` chunks;
//   3. bitonic sort of the candidates (of the whole row if there was no select),
//      larger score first, equal scores lower id first; up to 256 elements are
//      sorted in registers, one per thread, more in LDS;
//   4. exclusive prefix sum of chunk lengths along the ranking, chunk l left out
//      -> rem = N_b - (tokens of other chunks before this rank);
//   5. a chunk is kept if some row takes a token of it; kept chunks are
//      compacted in ascending chunk id (prefix sum of flags) into the plan.
// Row-block form (B_r > 0, Alg. 1 as printed): query group l is a row block,
// the candidates are the chunks that start before the block's end q_max, their
// lengths are clipped to q_max, there is no "own chunk", and an entry records
// how many tokens of the chunk the block's list holds (pos = 3).
// ---------------------------------------------------------------------------
constexpr int kMaxCand = 512;     // candidates kept by the radix select
constexpr int kSelectMin = 256;   // rows with more chunks than this use it; shorter rows are sorted whole, in registers

__global__ __launch_bounds__(256) void k_select(const double *__restrict__ Sc, int32_t *__restrict__ plan,
                                                PlanLayout pl, int N_c, int N_b, int B_r, int smem_bytes,
                                                int guess, int l_first) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int s_wave[4];
    __shared__ int s_p;
    __shared__ int s_hist[256];
    __shared__ int s_digit, s_above, s_equal;
    const int l = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
    const int32_t *B = plan + pl.off_B;
    const bool blocks = B_r > 0;
    const int q_max = blocks ? (plan + pl.off_RB)[l + 1] : 0x7fffffff;   // clip of the chunk lengths
    // l indexes Sc, RB and the plan; the group's number in the sequence is l_first + l (a launch
    // may cover a suffix of the groups, laid out from 0)
    const int own = blocks ? -1 : l_first + l;                            // the query group's own chunk
    const int n = blocks ? chunk_of_row(B, N_c, (int64_t)q_max - 1) + 1 : l_first + l + 1;   // visible chunks 0..n-1
    int P = 64;
    while (P < n) P <<= 1;
    unsigned long long *key = reinterpret_cast<unsigned long long *>(smem);  // [P]
    int *id = reinterpret_cast<int *>(smem + (size_t)P * 8);                 // [P]
    const double *row = Sc + ((int64_t)h * pl.N_q + l) * N_c;

    // eight scores per thread are requested before the first is used (one memory latency per
    // 2048 scores instead of one per 256)
    for (int x0 = tid; x0 < P; x0 += 8 * 256) {
        double sc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int x = x0 + e * 256;
            sc[e] = (x < n) ? row[x] : 0.0;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int x = x0 + e * 256;
            if (x >= P) break;
            unsigned long long u = 0ull;
            int k = 0x7fffffff;
            if (x < n) {
                double s = sc[e];
                if (s == 0.0) s = 0.0;  // -0.0 ties with +0.0
                u = (unsigned long long)__double_as_longlong(s);
                u = (u >> 63) ? ~u : (u | 0x8000000000000000ull);
                k = x;
            }
            key[x] = u;
            id[x] = k;
        }
    }
    __syncthreads();

    // What gets sorted: the whole row in place, or the candidates of a radix select.  The select
    // is tried first with `guess` chunks (the number that holds the budget if the best chunks
    // have about the mean length): the sorted candidates are exactly the head of the full
    // ranking, so if their lengths add up to the budget no later chunk can be listed and the
    // short sort is the answer.  Otherwise the select is redone with `stride` chunks, the bound
    // that always suffices.
    const bool can_select = n > kSelectMin && pl.stride <= kMaxCand - 64 && P * 8 + kMaxCand * 12 <= smem_bytes;
    int cap0 = 64;
    while (cap0 < guess) cap0 <<= 1;
    unsigned long long *skey = key;
    int *sid = id;
    int Ps = P, ns = n;
    int p = 0x7fffffff, run = 0;
    int lens[32];
    bool id_intact = true;
    for (int attempt = (can_select && guess < pl.stride && cap0 < kMaxCand) ? 0 : 1;; ++attempt) {
        skey = key;
        sid = id;
        Ps = P;
        ns = n;
        if (can_select) {
            // ---- radix select: smallest set {key >= threshold prefix} holding the best `need` ----
            const int cap = attempt == 0 ? cap0 : kMaxCand;
            const int goal = attempt == 0 ? guess : pl.stride;
            const int need = goal < n ? goal : n;
            unsigned long long prefix = 0ull;
            int above = 0, equal = n, shift = 64;
            for (int pass = 0; pass < 8 && above + equal > cap; ++pass) {
                shift = 56 - 8 * pass;
                s_hist[tid] = 0;
                __syncthreads();
                for (int x = tid; x < n; x += 256) {
                    const unsigned long long k = key[x];
                    if (pass == 0 || (k >> (shift + 8)) == prefix)
                        atomicAdd(&s_hist[(int)((k >> shift) & 255ull)], 1);
                }
                __syncthreads();
                // suffix counts over digits: thread t looks at digit 255 - t
                const int d = 255 - tid, cnt = s_hist[d];
                int total;
                const int gt = block_excl_scan(cnt, s_wave, &total);   // elements of the region with a larger digit
                const int want = need - above;                         // still to be found inside the region
                if (gt < want && gt + cnt >= want) { s_digit = d; s_above = gt; s_equal = cnt; }
                __syncthreads();
                above += s_above;
                equal = s_equal;
                prefix = (prefix << 8) | (unsigned long long)s_digit;
                __syncthreads();
            }
            if (above + equal <= cap) {
                // ---- compact the candidates, in chunk-id order, into their own arrays ----
                unsigned long long *ckey = reinterpret_cast<unsigned long long *>(smem + (size_t)P * 8);  // over id[]
                int *cid = reinterpret_cast<int *>(ckey + kMaxCand);
                const int per = (n + 255) / 256;
                const bool all = shift == 64;   // no radix pass ran (n <= cap): every element is a candidate
                int local = 0;
                for (int e = 0; e < per; ++e) {
                    const int x = tid * per + e;
                    if (x < n && (all || (key[x] >> shift) >= prefix)) ++local;
                }
                int total;
                int slot = block_excl_scan(local, s_wave, &total);
                __syncthreads();               // id[] is dead (ids are positions), its space is reused now
                id_intact = false;
                for (int e = 0; e < per; ++e) {
                    const int x = tid * per + e;
                    if (x < n && (all || (key[x] >> shift) >= prefix)) { ckey[slot] = key[x]; cid[slot] = x; ++slot; }
                }
                ns = total;
                Ps = 64;
                while (Ps < ns) Ps <<= 1;
                for (int x = ns + tid; x < Ps; x += 256) { ckey[x] = 0ull; cid[x] = 0x7fffffff; }
                skey = ckey;
                sid = cid;
                __syncthreads();
            } else if (attempt == 0) {
                continue;                      // too many equal scores for the short sort
            } else if (!id_intact) {           // whole-row sort after a first attempt: ids are positions
                for (int x = tid; x < P; x += 256) id[x] = x < n ? x : 0x7fffffff;
                __syncthreads();
            }
        }

        // ---- bitonic network; "a goes first" iff key larger, or equal and id smaller ----
        if (Ps <= 256) {
            if (Ps == 64) sort_in_registers<64>(skey, sid, tid);
            else if (Ps == 128) sort_in_registers<128>(skey, sid, tid);
            else sort_in_registers<256>(skey, sid, tid);
        } else
        for (int size = 2; size <= Ps; size <<= 1) {
            for (int j = size >> 1, lj = 31 - __clz(size >> 1); j > 0; j >>= 1, --lj) {   // j = 1 << lj
                for (int t = tid; t < (Ps >> 1); t += 256) {
                    int lo = ((t >> lj) << (lj + 1)) + (t & (j - 1));
                    int hi = lo + j;
                    bool up = (lo & size) == 0;
                    unsigned long long ka = skey[lo], kb = skey[hi];
                    int ia = sid[lo], ib = sid[hi];
                    bool a_first = (ka > kb) || (ka == kb && ia < ib);
                    if (a_first != up) {
                        skey[lo] = kb; skey[hi] = ka;
                        sid[lo] = ib; sid[hi] = ia;
                    }
                }
                __syncthreads();
            }
        }
        // rank of chunk l (beyond every candidate if it is not one of them)
        if (tid == 0) s_p = 0x7fffffff;
        __syncthreads();
        for (int x = tid; x < ns; x += 256)
            if (sid[x] == own) s_p = x;
        __syncthreads();
        p = s_p;
        // chunk lengths along the ranking (chunk l left out) and their exclusive prefix sum
        const int per = Ps / 256 > 0 ? Ps / 256 : 1;           // consecutive ranks per thread
        int local = 0;
        for (int e = 0; e < per; ++e) {
            int r = tid * per + e;
            int len = 0;
            if (r < ns) {
                int k = sid[r];
                const int end = B[k + 1] < q_max ? B[k + 1] : q_max;
                len = (k == own) ? 0 : end - B[k];
            }
            lens[e] = len;
            local += len;
        }
        int total;
        run = block_excl_scan(local, s_wave, &total);
        if (attempt == 0 && ns < n && total < N_b) {
            __syncthreads();                   // every thread is done with the candidates
            continue;
        }
        break;
    }
    // the row's key array is dead now: reuse it as rem_by_id / pos_by_id
    int *rem_by_id = reinterpret_cast<int *>(smem);        // [P]
    int *pos_by_id = rem_by_id + P;                        // [P]
    if (skey != key) {                                     // chunks that are no candidates are not listed
        for (int x = tid; x < n; x += 256) rem_by_id[x] = 0;
    }
    __syncthreads();  // the zero fill is complete
    {
        const int per = Ps / 256 > 0 ? Ps / 256 : 1;
        for (int e = 0; e < per; ++e) {
            int r = tid * per + e;
            if (r < ns) {
                int k = sid[r];
                int pos = blocks ? 3 : ((r < p) ? 0 : (r == p ? 1 : 2));
                int rem = N_b - run;                      // may be <= 0: not needed
                bool need = (pos == 2) ? (rem > 1) : (rem > 0);
                if (blocks && rem > lens[e]) rem = lens[e];   // tokens of the chunk in the block's list
                rem_by_id[k] = need ? rem : 0;
                pos_by_id[k] = pos;
            }
            run += lens[e];
        }
    }
    __syncthreads();
    // compact in ascending chunk id
    int32_t *entries = plan + pl.off_entries + ((int64_t)h * pl.N_q + l) * pl.stride * 2;
    {
        const int per_id = P / 256 > 0 ? P / 256 : 1;
        int local = 0;
        for (int e = 0; e < per_id; ++e) {
            int k = tid * per_id + e;
            if (k < n && rem_by_id[k] != 0) ++local;
        }
        int total;
        int slot = block_excl_scan(local, s_wave, &total);
        for (int e = 0; e < per_id; ++e) {
            int k = tid * per_id + e;
            if (k < n && rem_by_id[k] != 0) {
                if (slot < pl.stride) {
                    entries[2 * slot] = k | (pos_by_id[k] << kPosShift);
                    entries[2 * slot + 1] = rem_by_id[k];
                }
                ++slot;
            }
        }
        if (tid == 0) plan[pl.off_count + (int64_t)h * pl.N_q + l] = total < pl.stride ? total : pl.stride;
    }
}

hipError_t launch_select(const Prob &p, const PlanLayout &pl, const double *Sc, int32_t *plan, hipStream_t s) {
    return launch_select_groups(p, pl, Sc, plan, 0, p.N_q, s);
}

hipError_t launch_select_groups(const Prob &p, const PlanLayout &pl, const double *Sc, int32_t *plan, int l_first,
                                int n_groups, hipStream_t s) {
    int P = 64;
    while (P < p.N_c) P <<= 1;
    size_t shmem = (size_t)P * 8 + std::max<size_t>((size_t)P * 4, (size_t)kMaxCand * 12);   // keys + (ids | candidates)
    if (shmem > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_select),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k_select, dim3(n_groups, p.H_q), dim3(256), shmem, s, Sc, plan, pl, p.N_c, p.N_b, p.B_r,
                       (int)shmem, pl.guess > 0 ? pl.guess : 1, l_first);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Plan -> explicit index sets (Alg. 1's output) for a list of rows of one head.
// One wave per row.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_expand(PlanView pv, int N_c, int head, const int64_t *__restrict__ rows,
                                               int32_t *__restrict__ idx, int cap, int32_t *__restrict__ cnt) {
    if (!plan_matches(pv)) return;   // not this problem's plan: nothing is written
    const int t = blockIdx.x, lane = threadIdx.x;
    const int64_t i = rows[t];
    const int l = chunk_of_row(pv.RB, pv.N_q, i);
    const int v = (int)(i + 1 - pv.RB[l]);
    const int E = pv.count[(int64_t)head * pv.N_q + l];
    const int32_t *ent = pv.entries + ((int64_t)head * pv.N_q + l) * pv.stride * 2;
    int32_t *out = idx + (int64_t)t * cap;
    int n = 0;
    for (int e = 0; e < E; ++e) {
        int w0 = ent[2 * e], rem = ent[2 * e + 1];
        int k = w0 & kChunkMask, pos = w0 >> kPosShift;
        int b0 = pv.B[k];
        int take = entry_take(pos, rem, pv.B[k + 1] - b0, v);
        for (int x = lane; x < take; x += 64)
            if (n + x < cap) out[n + x] = b0 + x;
        n += take;
    }
    for (int x = n + lane; x < cap; x += 64) out[x] = -1;
    if (lane == 0) cnt[t] = n;
}

hipError_t launch_expand(const Prob &p, const PlanView &pv, int head, const int64_t *rows_dev, int n_rows,
                         int32_t *idx, int cap, int32_t *cnt, hipStream_t s) {
    if (n_rows == 0) return hipSuccess;
    hipLaunchKernelGGL(k_expand, dim3(n_rows), dim3(64), 0, s, pv, p.N_c, head, rows_dev, idx, cap, cnt);
    return hipGetLastError();
}

}  // namespace dhsa
