// One decoding step of libdhsa (Sec. 3.4, the remark on decoding: the same sparse
// attention applied to each newly generated token by restricting the keys it
// attends).  The newest token is row i = L - 1 of a sequence whose K / V rows are
// cached; its key set is what the prefill path gives that row: its query group
// (the open chunk, or with B_r > 0 the open row block) is pooled, scored against
// every key chunk, ranked and walked with the budget N_b (Alg. 1), and the row
// attends to the selected keys (Alg. 2).
//
// Kernels of this file:
//   k_pool_decode     pooled keys (Eq. 4) of the chunks not pooled by an earlier
//                     step, pooled queries of the open group;
//   k_scores_decode   that group's scores against every key chunk (one wave per pooled key);
//   (the ranking and the walk are k_select of route.hip, launched for one group)
//   k_attn_decode     the selected keys are split into slices of 128; one workgroup
//                     per (slice, head) streams its K and V rows once, 16 bytes per
//                     lane, several rows in flight, and keeps an online-softmax
//                     state per row group; memory bound;
//   k_decode_combine  merges the slices' states into the output row.
#include "dhsa_internal.h"

namespace dhsa {

// ---------------------------------------------------------------------------
// Pooling.  grid (max(N_c - kc_valid, 1), H_kv + H_q): y < H_kv pools key chunk
// kc_valid + x of kv-head y into Kc [H_kv][N_c_cap][D]; y >= H_kv (x = 0 only)
// pools the rows [rb0, L) of query head y - H_kv into Qc [H_q][D].  Same row
// traversal as the prefill pooling kernel.
// ---------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void k_pool_decode(const T *__restrict__ Q, const T *__restrict__ K,
                                                     int32_t *__restrict__ B, BoundaryTail tail,
                                                     int32_t *__restrict__ RBw,
                                                     double *__restrict__ Qc, double *__restrict__ Kc, int H_kv,
                                                     int N_c, int N_c_cap, int kc_valid, int rb0, int L, int B_r,
                                                     int pooling, int64_t qs_h, int64_t qs_l, int64_t ks_h,
                                                     int64_t ks_l) {
    constexpr int EPT = Elem<T>::kPer16;   // elements per thread per row
    constexpr int TPR = D / EPT;           // threads per row
    constexpr int RG = 256 / TPR;          // rows in flight
    __shared__ double s_sum[RG][D];
    const int tid = threadIdx.x;
    const bool is_q = (int)blockIdx.y >= H_kv;
    const T *X;
    double *Xc;
    int64_t s_l;
    int b0, b1;
    if (is_q) {
        if (blockIdx.x != 0) return;
        const int h = blockIdx.y - H_kv;
        X = Q + (int64_t)h * qs_h; s_l = qs_l; Xc = Qc + (int64_t)h * D;
        b0 = rb0; b1 = L;
        if (h == 0 && tid == 0) { RBw[0] = rb0; RBw[1] = L; }   // the one query group of the step's plan
        // boundaries that came as arguments go into the workspace for the kernels after this one
        if (h == 0 && tid <= tail.n && tail.n > 0) B[kc_valid + tid] = tail.b[tid];
    } else {
        const int k = kc_valid + blockIdx.x, g = blockIdx.y;
        if (k >= N_c) return;
        X = K + (int64_t)g * ks_h; s_l = ks_l; Xc = Kc + ((int64_t)g * N_c_cap + k) * D;
        if (tail.n > 0) { b0 = tail.b[blockIdx.x]; b1 = tail.b[blockIdx.x + 1]; }   // not yet in B (see below)
        else { b0 = B[k]; b1 = B[k + 1]; }
    }
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

// ---------------------------------------------------------------------------
// Scores of the open query group: Sc[h][k] = <Qc[h], Kc[h / G][k]>, k < N_c.
// One wave per (kv-head g, chunk k): it reads the pooled key once and forms the
// scores of the G query heads of the group.  grid (ceil(N_c / 4), H_kv).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_scores_decode(const double *__restrict__ Qc, const double *__restrict__ Kc,
                                                       double *__restrict__ Sc, int N_c, int N_c_cap, int D, int G) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int k = blockIdx.x * 4 + wave, g = blockIdx.y;
    if (k >= N_c) return;   // wave-uniform
    const double *kc = Kc + ((int64_t)g * N_c_cap + k) * D;
    const double k0 = kc[lane], k1 = D > 64 ? kc[lane + 64] : 0.0;
    for (int hh = 0; hh < G; ++hh) {
        const int h = g * G + hh;
        const double *q = Qc + (int64_t)h * D;
        double acc = q[lane] * k0;
        if (D > 64) acc += q[lane + 64] * k1;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
        if (lane == 0) Sc[(int64_t)h * N_c + k] = acc;
    }
}

// ---------------------------------------------------------------------------
// Attention of the newest row over slice blockIdx.x of its selected keys.
// The plan entries of (h, the open group) are walked like in the prefill
// kernels (ascending key position); packed positions [128 s, 128 s + 128) are
// this workgroup's.  A key row is read by TPR = D sizeof(T) / 16 adjacent lanes
// (16 bytes each: coalesced), NG = 256 / TPR rows at a time, U batches in
// flight.  Partial state of the slice -> part[h][s] = (m, l, o[D]).
// ---------------------------------------------------------------------------
template <typename T> struct DecIO;
template <> struct DecIO<float> {
    __device__ static void unpack(const uint4 &u, float *x) {
        x[0] = __uint_as_float(u.x); x[1] = __uint_as_float(u.y);
        x[2] = __uint_as_float(u.z); x[3] = __uint_as_float(u.w);
    }
    __device__ static void store(float *p, float x) { *p = x; }
};
template <> struct DecIO<bf16_t> {
    __device__ static void unpack(const uint4 &u, float *x) {
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __uint_as_float(w[i] << 16);
            x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ static void store(bf16_t *p, float x) {   // round to nearest even
        uint32_t u = __float_as_uint(x);
        u += 0x7fffu + ((u >> 16) & 1u);
        p->bits = (uint16_t)(u >> 16);
    }
};

template <typename T, int D>
__global__ __launch_bounds__(256) void k_attn_decode(const int32_t *__restrict__ B, const int32_t *__restrict__ count,
                                                     const int32_t *__restrict__ entries, int stride, int rb0, int L,
                                                     const T *__restrict__ Q, const T *__restrict__ K,
                                                     const T *__restrict__ V, float *__restrict__ part, int S,
                                                     int32_t *__restrict__ idx, int cap, int32_t *__restrict__ cnt,
                                                     int G, float scale, int64_t qs_h, int64_t qs_l, int64_t ks_h,
                                                     int64_t ks_l, int64_t vs_h, int64_t vs_l) {
    constexpr int EPT = 16 / (int)sizeof(T);   // elements per 16 bytes
    constexpr int TPR = D / EPT;               // lanes per key row (8, 16 or 32)
    constexpr int NG = 256 / TPR;              // key rows per batch
    constexpr int U = 4;                       // batches in flight
    __shared__ int s_keys[kDecSlice];
    __shared__ int s_wave[4];
    __shared__ float s_m[NG], s_l[NG];
    __shared__ float s_o[NG][D];
    const int s = blockIdx.x, h = blockIdx.y, g = h / G, tid = threadIdx.x;
    const int i = L - 1;
    const int v = L - rb0;   // rows of the query group up to and including the newest
    const int E = count[h];
    const int32_t *ent = entries + (int64_t)h * stride * 2;
    const int x_lo = s * kDecSlice, x_hi = x_lo + kDecSlice;

    if (tid < kDecSlice) s_keys[tid] = -1;
    __syncthreads();
    int base = 0;   // selected keys of the entries walked so far (block-uniform)
    for (int e0 = 0; e0 < E; e0 += 256) {
        int take = 0, b0 = 0;
        if (e0 + tid < E) {
            const int w0 = ent[2 * (e0 + tid)], rem = ent[2 * (e0 + tid) + 1];
            const int k = w0 & kChunkMask, pos = w0 >> kPosShift;
            b0 = B[k];
            take = entry_take(pos, rem, B[k + 1] - b0, v);
            if (pos == 3) {   // row-block form: of the block's list, the keys up to the row itself
                const int vis = i + 1 - b0;
                if (vis < take) take = vis > 0 ? vis : 0;
            }
        }
        int total;
        const int start = base + block_excl_scan(take, s_wave, &total);
        const int lo = start > x_lo ? start : x_lo;
        const int hi = start + take < x_hi ? start + take : x_hi;
        for (int x = lo; x < hi; ++x) s_keys[x - x_lo] = b0 + (x - start);
        base += total;
        if (base >= x_hi && s != 0) break;   // slice 0 walks on: it reports the row's key count
    }
    __syncthreads();
    if (s == 0 && tid == 0 && cnt) cnt[h] = base;
    int n_mine = base - x_lo;
    n_mine = n_mine < 0 ? 0 : (n_mine > kDecSlice ? kDecSlice : n_mine);
    if (idx && tid < kDecSlice && x_lo + tid < cap) idx[(int64_t)h * cap + x_lo + tid] = s_keys[tid];

    const int gi = tid / TPR, r = tid % TPR;
    float q[EPT];
    DecIO<T>::unpack(*reinterpret_cast<const uint4 *>(Q + (int64_t)h * qs_h + (int64_t)i * qs_l + r * EPT), q);
    const T *Kg = K + (int64_t)g * ks_h + r * EPT;
    const T *Vg = V + (int64_t)g * vs_h + r * EPT;
    float m = -INFINITY, l = 0.f, o[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) o[e] = 0.f;
    for (int j0 = gi; j0 < n_mine; j0 += NG * U) {
        uint4 kf[U], vf[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int jj = j0 + u * NG;
            ok[u] = jj < n_mine;
            const int key = ok[u] ? s_keys[jj] : s_keys[j0];   // a valid row either way
            kf[u] = *reinterpret_cast<const uint4 *>(Kg + (int64_t)key * ks_l);
            vf[u] = *reinterpret_cast<const uint4 *>(Vg + (int64_t)key * vs_l);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kx[EPT], vx[EPT];
            DecIO<T>::unpack(kf[u], kx);
            DecIO<T>::unpack(vf[u], vx);
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < EPT; ++e) d += q[e] * kx[e];
#pragma unroll
            for (int off = TPR / 2; off > 0; off >>= 1) d += __shfl_xor(d, off);
            if (ok[u]) {
                const float sc = d * scale;
                const float m_new = fmaxf(m, sc);
                const float alpha = __expf(m - m_new), p = __expf(sc - m_new);
                l = l * alpha + p;
#pragma unroll
                for (int e = 0; e < EPT; ++e) o[e] = o[e] * alpha + p * vx[e];
                m = m_new;
            }
        }
    }
    if (r == 0) { s_m[gi] = m; s_l[gi] = l; }
#pragma unroll
    for (int e = 0; e < EPT; ++e) s_o[gi][r * EPT + e] = o[e];
    __syncthreads();
    if (tid < D) {
        float M = -INFINITY;
        for (int x = 0; x < NG; ++x) M = fmaxf(M, s_m[x]);
        float ls = 0.f, acc = 0.f;
        for (int x = 0; x < NG; ++x) {
            const float w = (s_m[x] == -INFINITY) ? 0.f : __expf(s_m[x] - M);
            ls += s_l[x] * w;
            acc += s_o[x][tid] * w;
        }
        float *pp = part + ((int64_t)h * S + s) * (D + 2);
        pp[2 + tid] = acc;
        if (tid == 0) { pp[0] = M; pp[1] = ls; }
    }
}

// Merge of the S slice states of one head into the output row.  grid H_q, block 512:
// the slices are dealt to 512 / D groups of D threads (thread = output column), whose
// partial sums meet in LDS.
template <typename T, int D>
__global__ __launch_bounds__(512) void k_decode_combine(const float *__restrict__ part, int S, T *__restrict__ O_row) {
    constexpr int NSG = 512 / D;
    __shared__ float s_red[8];
    __shared__ float s_ls[NSG];
    __shared__ float s_acc[NSG][D];
    const int h = blockIdx.x, tid = threadIdx.x, d = tid % D, sg = tid / D;
    const float *pp = part + (int64_t)h * S * (D + 2);
    // reference exponent: the largest slice maximum
    float M = -INFINITY;
    for (int s = tid; s < S; s += 512) M = fmaxf(M, pp[(int64_t)s * (D + 2)]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
    if ((tid & 63) == 0) s_red[tid >> 6] = M;
    __syncthreads();
    M = s_red[0];
#pragma unroll
    for (int x = 1; x < 8; ++x) M = fmaxf(M, s_red[x]);
    float ls = 0.f, acc = 0.f;
    for (int s = sg; s < S; s += NSG) {
        const float *ps = pp + (int64_t)s * (D + 2);
        const float w = (ps[0] == -INFINITY) ? 0.f : __expf(ps[0] - M);
        ls += ps[1] * w;
        acc += ps[2 + d] * w;
    }
    s_acc[sg][d] = acc;
    if (d == 0) s_ls[sg] = ls;
    __syncthreads();
    if (tid < D) {
        float L = 0.f, A = 0.f;
#pragma unroll
        for (int x = 0; x < NSG; ++x) { L += s_ls[x]; A += s_acc[x][tid]; }
        DecIO<T>::store(O_row + (int64_t)h * D + tid, L > 0.f ? A / L : 0.f);
    }
}

hipError_t launch_decode_route(const Prob &p, const DecodeLayout &dl, int N_c_cap, int kc_valid, int rb0,
                               const BoundaryTail &tail, const void *Q, const void *K, void *ws, hipStream_t s) {
    char *w8 = static_cast<char *>(ws);
    double *Kc = reinterpret_cast<double *>(w8 + dl.off_Kc), *Qc = reinterpret_cast<double *>(w8 + dl.off_Qc);
    double *Sc = reinterpret_cast<double *>(w8 + dl.off_Sc);
    int32_t *plan = reinterpret_cast<int32_t *>(w8 + dl.off_plan);
    const int n_new = p.N_c - kc_valid;
    dim3 grid(n_new > 1 ? n_new : 1, p.H_kv + p.H_q), block(256);
#define DHSA_POOLD(T, DD)                                                                                      \
    hipLaunchKernelGGL((k_pool_decode<T, DD>), grid, block, 0, s, (const T *)Q, (const T *)K,                  \
                       plan + dl.pl.off_B, tail, plan + dl.pl.off_RB, Qc, Kc, p.H_kv, p.N_c, N_c_cap, kc_valid, rb0, \
                       (int)p.L, p.B_r, p.pooling, p.qs_h, p.qs_l, p.ks_h, p.ks_l)
    if (p.dtype == DHSA_F32) {
        if (p.D == 64) DHSA_POOLD(float, 64); else DHSA_POOLD(float, 128);
    } else {
        if (p.D == 64) DHSA_POOLD(bf16_t, 64); else DHSA_POOLD(bf16_t, 128);
    }
#undef DHSA_POOLD
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_scores_decode, dim3((p.N_c + 3) / 4, p.H_kv), dim3(256), 0, s, Qc, Kc, Sc, p.N_c, N_c_cap,
                       p.D, p.G);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    // ranking + walk of the one open group: group number N_q - 1 of the sequence, group 0 of this plan
    return launch_select_groups(p, dl.pl, Sc, plan, p.N_q - 1, 1, s);
}

hipError_t launch_decode_attend(const Prob &p, const DecodeLayout &dl, int rb0, const void *Q, const void *K,
                                const void *V, void *ws, void *O_row, int32_t *idx, int32_t *cnt, hipStream_t s) {
    char *w8 = static_cast<char *>(ws);
    const int32_t *plan = reinterpret_cast<const int32_t *>(w8 + dl.off_plan);
    float *part = reinterpret_cast<float *>(w8 + dl.off_part);
    const int S = (p.N_b + kDecSlice - 1) / kDecSlice;   // N_b is clamped to L: the row takes exactly N_b keys
    dim3 grid(S, p.H_q), block(256);
#define DHSA_ATTD(T, DD)                                                                                          \
    do {                                                                                                          \
        hipLaunchKernelGGL((k_attn_decode<T, DD>), grid, block, 0, s, plan + dl.pl.off_B, plan + dl.pl.off_count, \
                           plan + dl.pl.off_entries, dl.pl.stride, rb0, (int)p.L, (const T *)Q, (const T *)K,     \
                           (const T *)V, part, S, idx, p.N_b, cnt, p.G, p.scale, p.qs_h, p.qs_l, p.ks_h, p.ks_l,  \
                           p.vs_h, p.vs_l);                                                                       \
        hipLaunchKernelGGL((k_decode_combine<T, DD>), dim3(p.H_q), dim3(512), 0, s, part, S, (T *)O_row);         \
    } while (0)
    if (p.dtype == DHSA_F32) {
        if (p.D == 64) DHSA_ATTD(float, 64); else DHSA_ATTD(float, 128);
    } else {
        if (p.D == 64) DHSA_ATTD(bf16_t, 64); else DHSA_ATTD(bf16_t, 128);
    }
#undef DHSA_ATTD
    return hipGetLastError();
}

}  // namespace dhsa
