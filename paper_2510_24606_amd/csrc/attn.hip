// Sparse attention kernels of libdhsa: exact softmax attention over the keys
// the routing plan selects (Alg. 2 / Alg. 3 of the paper, App. C "Backend
// implementations").  Two kernels:
//   k_attn_rowwise  fp32 arithmetic, one wavefront per query row (DHSA_F32 path)
//   k_attn_mfma     bf16 MFMA 32x32x16, fp32 online softmax, one workgroup per
//                   (query head, tile of <= 128 rows of one query chunk)
#include "dhsa_internal.h"

namespace dhsa {

struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// ---------------------------------------------------------------------------
// Row-wise fp32 kernel.  Each wave owns one query row: lanes compute the scores
// of 64 selected keys at a time (online softmax over batches, Alg. 3 with
// B_r = 1, B_c = 64), then lanes own output columns for the PV sum.
// ---------------------------------------------------------------------------
template <typename T> struct RowIO;
template <> struct RowIO<float> {
    static constexpr int kPer16 = 4;
    __device__ static float dot16(const uint4 &u, const float *q) {
        return __uint_as_float(u.x) * q[0] + __uint_as_float(u.y) * q[1] + __uint_as_float(u.z) * q[2] +
               __uint_as_float(u.w) * q[3];
    }
    __device__ static float load(const float *p) { return *p; }
    __device__ static void store(float *p, float x) { *p = x; }
};
template <> struct RowIO<bf16_t> {
    static constexpr int kPer16 = 8;
    __device__ static float dot16(const uint4 &u, const float *q) {
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            s += __uint_as_float(w[i] << 16) * q[2 * i] + __uint_as_float(w[i] & 0xffff0000u) * q[2 * i + 1];
        return s;
    }
    __device__ static float load(const bf16_t *p) { return bf16_to_f32(p->bits); }
    __device__ static void store(bf16_t *p, float x) {
        uint32_t u = __float_as_uint(x);
        u += 0x7fffu + ((u >> 16) & 1u);
        p->bits = (uint16_t)(u >> 16);
    }
};

template <typename T, int D>
__global__ __launch_bounds__(256) void k_attn_rowwise(PlanView pv, const T *__restrict__ Q,
                                                      const T *__restrict__ K, const T *__restrict__ V,
                                                      T *__restrict__ O, int64_t L, int N_c, int G, float scale,
                                                      int64_t qs_h, int64_t qs_l, int64_t ks_h, int64_t ks_l,
                                                      int64_t vs_h, int64_t vs_l, int64_t os_h, int64_t os_l) {
    constexpr int EP = RowIO<T>::kPer16;
    constexpr int NC = D / 64;  // output columns per lane
    __shared__ float s_q[4][D];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = blockIdx.y, g = h / G;
    const int64_t i = (int64_t)blockIdx.x * 4 + wave;
    const bool live = i < L;
    if (live)
        for (int d = lane; d < D; d += 64) s_q[wave][d] = RowIO<T>::load(Q + (int64_t)h * qs_h + i * qs_l + d);
    __syncthreads();
    if (!live) return;
    const T *Kg = K + (int64_t)g * ks_h;
    const T *Vg = V + (int64_t)g * vs_h;
    const int l = chunk_of_row(pv.B, N_c, i);
    const int v = (int)(i + 1 - pv.B[l]);
    const int E = pv.count[(int64_t)h * N_c + l];
    const int32_t *ent = pv.entries + ((int64_t)h * N_c + l) * pv.stride * 2;
    float m_run = -INFINITY, l_lane = 0.f;
    float o[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) o[c] = 0.f;
    for (int e = 0; e < E; ++e) {
        const int w0 = ent[2 * e], rem = ent[2 * e + 1];
        const int k = w0 & kChunkMask, pos = w0 >> kPosShift;
        const int b0 = pv.B[k];
        const int take = entry_take(pos, rem, pv.B[k + 1] - b0, v);
        for (int t0 = 0; t0 < take; t0 += 64) {
            const int nv = (take - t0 < 64) ? take - t0 : 64;
            float s = -INFINITY;
            if (lane < nv) {
                const T *kr = Kg + (int64_t)(b0 + t0 + lane) * ks_l;
                float acc = 0.f;
#pragma unroll
                for (int d = 0; d < D; d += EP)
                    acc += RowIO<T>::dot16(*reinterpret_cast<const uint4 *>(kr + d), &s_q[wave][d]);
                s = acc * scale;
            }
            float mx = s;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
            const float m_new = fmaxf(m_run, mx);  // finite: nv >= 1
            const float alpha = __expf(m_run - m_new);
            const float p = (lane < nv) ? __expf(s - m_new) : 0.f;
            l_lane = l_lane * alpha + p;
#pragma unroll
            for (int c = 0; c < NC; ++c) o[c] *= alpha;
            for (int jj = 0; jj < nv; ++jj) {
                const float pj = __shfl(p, jj);
                const T *vr = Vg + (int64_t)(b0 + t0 + jj) * vs_l;
#pragma unroll
                for (int c = 0; c < NC; ++c) o[c] += pj * RowIO<T>::load(vr + lane + 64 * c);
            }
            m_run = m_new;
        }
    }
    float lsum = l_lane;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) lsum += __shfl_xor(lsum, off);
    const float inv = 1.f / lsum;
#pragma unroll
    for (int c = 0; c < NC; ++c)
        RowIO<T>::store(O + (int64_t)h * os_h + i * os_l + lane + 64 * c, o[c] * inv);
}

hipError_t launch_attn_rowwise(const Prob &p, const PlanView &pv, const void *Q, const void *K, const void *V,
                               void *O, hipStream_t s) {
    dim3 grid((unsigned)((p.L + 3) / 4), p.H_q), block(256);
#define DHSA_ROWWISE(T, DD)                                                                                  \
    hipLaunchKernelGGL((k_attn_rowwise<T, DD>), grid, block, 0, s, pv, (const T *)Q, (const T *)K,           \
                       (const T *)V, (T *)O, p.L, p.N_c, p.G, p.scale, p.qs_h, p.qs_l, p.ks_h, p.ks_l,       \
                       p.vs_h, p.vs_l, p.os_h, p.os_l)
    if (p.dtype == DHSA_F32) {
        if (p.D == 64) DHSA_ROWWISE(float, 64); else DHSA_ROWWISE(float, 128);
    } else {
        if (p.D == 64) DHSA_ROWWISE(bf16_t, 64); else DHSA_ROWWISE(bf16_t, 128);
    }
#undef DHSA_ROWWISE
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// MFMA kernel (bf16).
//
// Work unit: (query head h, row tile): up to 128 consecutive rows of ONE query
// chunk l.  All rows of the tile share the plan entries of (h, l); they differ
// only through v = i + 1 - B[l].  The selected keys are walked in ascending
// position (softmax is order-free) and packed densely into tiles of 64 keys;
// a packed key carries (j, lo, hi) with "row takes key  <=>  lo < v < hi".
//
// Four waves; wave w owns rows 32w .. 32w+31.  Scores are computed transposed,
// S^T = K Q^T (keys are the MFMA M dimension), so a lane holds 16 keys of ONE
// query row per 32-key block: the row max / sum stay in the lane (one exchange
// with lane ^ 32), and the exponentiated scores are already laid out as the B
// operand of O^T = V^T P^T.  V is transposed on its way into LDS.
// ---------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kKT = 64;      // keys per tile
constexpr int kSegB = 256;   // plan entries handled per batch
constexpr int kIntMax = 0x7fffffff;

template <int D>
struct AttnSmem {
    static constexpr int KS = D + 8;    // K row stride in bf16 (272 B: conflict-free b128 row reads)
    static constexpr int VS = kKT + 4;  // V^T row stride in bf16 (136 B: conflict-free b64 row reads)
    alignas(16) uint16_t K[kKT * KS];
    alignas(16) uint16_t Vt[D * VS];
    alignas(16) int key_j[3][kKT];
    alignas(16) int key_lo[3][kKT];
    alignas(16) int key_hi[3][kKT];
    int seg_start[kSegB + 1];
    int seg_b0[kSegB];
    int seg_pos[kSegB];
    int seg_rem[kSegB];
    int flags[4];
    int s_wave[4];
};

// blockIdx -> (head, tile).  Workgroups are dealt to the 8 XCDs round-robin, each
// XCD has its own L2: give one XCD the heads of one kv-group and neighbouring
// row tiles, so that the K/V slabs its workgroups stream overlap in that L2.
// Tiles are issued from the end of the sequence (most keys) to the start.
__device__ __forceinline__ bool decode_block(int b, int H_q, int H_kv, int G, int T1, int *h, int *tile) {
    if (H_kv % 8 == 0) {
        const int x = b & 7, j = b >> 3;
        const int s = j / (G * T1), r = j % (G * T1);
        *tile = T1 - 1 - r / G;
        *h = (x + 8 * s) * G + r % G;
        return true;
    }
    if (8 % H_kv == 0) {
        const int S = 8 / H_kv;
        const int x = b & 7, j = b >> 3;
        const int g = x % H_kv, s = x / H_kv;
        const int rank = (j / G) * S + s;
        if (rank >= T1) return false;
        *tile = T1 - 1 - rank;
        *h = g * G + j % G;
        return true;
    }
    *tile = T1 - 1 - b / H_q;
    *h = b % H_q;
    return true;
}

static int attn_grid(int H_q, int H_kv, int G, int T1) {
    if (H_kv % 8 == 0) return H_q * T1;
    if (8 % H_kv == 0) {
        const int S = 8 / H_kv;
        return 8 * G * ((T1 + S - 1) / S);
    }
    return H_q * T1;
}

template <int D>
__global__ __launch_bounds__(256, 2) void k_attn_mfma(PlanView pv, const uint16_t *__restrict__ Q,
                                                      const uint16_t *__restrict__ K,
                                                      const uint16_t *__restrict__ V, uint16_t *__restrict__ O,
                                                      int N_c, int H_q, int H_kv, int G, float scale_log2e,
                                                      int64_t qs_h, int64_t qs_l, int64_t ks_h, int64_t ks_l,
                                                      int64_t vs_h, int64_t vs_l, int64_t os_h, int64_t os_l) {
    using Smem = AttnSmem<D>;
    constexpr int OPR = D / 8;          // 16-byte pieces per row
    constexpr int KPT = OPR / 4;        // K pieces per thread per tile
    constexpr int NS = D / 16;          // MFMA k-steps of Q K^T
    constexpr int NDB = D / 32;         // 32-wide output column blocks
    __shared__ Smem sm;

    int h, tile;
    if (!decode_block(blockIdx.x, H_q, H_kv, G, pv.T1, &h, &tile)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lr = lane & 31, g2 = lane >> 5;
    const int g = h / G;
    const int l = pv.tiles[2 * tile], row0 = pv.tiles[2 * tile + 1];
    const int b_l = pv.B[l];
    const int rows_left = pv.B[l + 1] - row0;
    const int nrows = rows_left < kRowTile ? rows_left : kRowTile;
    const int v_lo = row0 + 1 - b_l, v_hi = v_lo + nrows - 1;
    const bool wave_live = wave * 32 < nrows;
    const int v_i = v_lo + wave * 32 + lr;  // this lane's query row (may be a padding row)

    const uint16_t *Kg = K + (int64_t)g * ks_h;
    const uint16_t *Vg = V + (int64_t)g * vs_h;

    // Q fragments: B operand of S^T = K Q^T; lane holds row lr, d = 16 s + 8 g2 .. + 7
    bf16x8 qf[NS];
    {
        int r = wave * 32 + lr;
        if (r >= nrows) r = nrows - 1;  // padding rows read a valid row; never stored
        const uint16_t *qp = Q + (int64_t)h * qs_h + (int64_t)(row0 + r) * qs_l + 8 * g2;
#pragma unroll
        for (int s = 0; s < NS; ++s) qf[s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);
    }

    f32x16 oacc[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int x = 0; x < 16; ++x) oacc[db][x] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const int E = pv.count[(int64_t)h * N_c + l];
    const int32_t *ent = pv.entries + ((int64_t)h * N_c + l) * pv.stride * 2;

    // staging assignment
    const int k_key = tid / OPR, k_oct = tid % OPR;        // + (256 / OPR) keys per extra piece
    const int v_q = tid / OPR, v_oct = tid % OPR;          // key quad, d octet
    const bool v_live = tid < 16 * OPR;
    uint4 kreg[KPT];
    uint4 vreg[4];

    for (int e0 = 0; e0 < E; e0 += kSegB) {
        // ---- segment table of this batch of plan entries ----
        int n_e = 0;
        if (e0 + tid < E) {
            const int w0 = ent[2 * (e0 + tid)], rem = ent[2 * (e0 + tid) + 1];
            const int k = w0 & kChunkMask, pos = w0 >> kPosShift;
            const int b0 = pv.B[k];
            // most tokens any row of the tile takes from this chunk
            n_e = entry_take(pos, rem, pv.B[k + 1] - b0, pos == 1 ? v_hi : v_lo);
            sm.seg_b0[tid] = b0;
            sm.seg_pos[tid] = pos;
            sm.seg_rem[tid] = rem;
        }
        int total;
        const int start = block_excl_scan(n_e, sm.s_wave, &total);
        sm.seg_start[tid] = start;
        if (tid == 255) sm.seg_start[kSegB] = total;
        __syncthreads();
        const int nseg = (E - e0 < kSegB) ? E - e0 : kSegB;
        const int ntiles = (total + kKT - 1) / kKT;
        if (ntiles == 0) continue;

        auto make_meta = [&](int n) {
            // wave 0: packed position -> (key index, lo, hi) of tile n
            if (wave == 0) {
                const int buf = n % 3;
                int x = n * kKT + lane;
                const bool pad = x >= total;
                if (pad) x = total - 1;
                int lo_s = 0, hi_s = nseg;  // seg_start[lo_s] <= x < seg_start[hi_s]
                while (hi_s - lo_s > 1) {
                    const int mid = (lo_s + hi_s) >> 1;
                    if (sm.seg_start[mid] <= x) lo_s = mid; else hi_s = mid;
                }
                const int t = x - sm.seg_start[lo_s];
                const int pos = sm.seg_pos[lo_s];
                int lo = (pos == 1) ? t : 0;
                int hi = (pos == 2) ? sm.seg_rem[lo_s] - t : kIntMax;
                if (pad) { lo = kIntMax; hi = kIntMax; }
                sm.key_j[buf][lane] = sm.seg_b0[lo_s] + t;
                sm.key_lo[buf][lane] = lo;
                sm.key_hi[buf][lane] = hi;
                const bool need = (lo >= v_lo) || (hi <= v_hi);
                const unsigned long long any = __ballot(need);
                if (lane == 0) sm.flags[buf] = any != 0ull;
            }
        };
        auto gload = [&](int n) {
            const int buf = n % 3;
#pragma unroll
            for (int c = 0; c < KPT; ++c) {
                const int key = k_key + c * (256 / OPR);
                kreg[c] = *reinterpret_cast<const uint4 *>(Kg + (int64_t)sm.key_j[buf][key] * ks_l + 8 * k_oct);
            }
            if (v_live) {
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    vreg[jj] = *reinterpret_cast<const uint4 *>(Vg + (int64_t)sm.key_j[buf][4 * v_q + jj] * vs_l +
                                                                8 * v_oct);
            }
        };
        auto lstore = [&]() {
#pragma unroll
            for (int c = 0; c < KPT; ++c) {
                const int key = k_key + c * (256 / OPR);
                *reinterpret_cast<uint4 *>(&sm.K[key * Smem::KS + 8 * k_oct]) = kreg[c];
            }
            if (v_live) {
                const uint32_t a[4] = {vreg[0].x, vreg[0].y, vreg[0].z, vreg[0].w};
                const uint32_t b[4] = {vreg[1].x, vreg[1].y, vreg[1].z, vreg[1].w};
                const uint32_t c[4] = {vreg[2].x, vreg[2].y, vreg[2].z, vreg[2].w};
                const uint32_t d[4] = {vreg[3].x, vreg[3].y, vreg[3].z, vreg[3].w};
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    uint2 even, odd;  // four keys of one d
                    even.x = __builtin_amdgcn_perm(b[w], a[w], 0x05040100u);
                    even.y = __builtin_amdgcn_perm(d[w], c[w], 0x05040100u);
                    odd.x = __builtin_amdgcn_perm(b[w], a[w], 0x07060302u);
                    odd.y = __builtin_amdgcn_perm(d[w], c[w], 0x07060302u);
                    *reinterpret_cast<uint2 *>(&sm.Vt[(8 * v_oct + 2 * w) * Smem::VS + 4 * v_q]) = even;
                    *reinterpret_cast<uint2 *>(&sm.Vt[(8 * v_oct + 2 * w + 1) * Smem::VS + 4 * v_q]) = odd;
                }
            }
        };

        make_meta(0);
        if (ntiles > 1) make_meta(1);
        __syncthreads();
        gload(0);
        for (int n = 0; n < ntiles; ++n) {
            lstore();
            if (n + 2 < ntiles) make_meta(n + 2);
            __syncthreads();
            if (n + 1 < ntiles) gload(n + 1);
            if (wave_live) {
                const int buf = n % 3;
                // ---- S^T = K Q^T : two 32-key blocks ----
                f32x16 sacc[2];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int x = 0; x < 16; ++x) sacc[kb][x] = 0.f;
#pragma unroll
                for (int s = 0; s < NS; ++s)
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb) {
                        const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(
                            &sm.K[(kb * 32 + lr) * Smem::KS + 16 * s + 8 * g2]);
                        sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sacc[kb], 0, 0, 0);
                    }
                // ---- mask: key taken by this row iff lo < v_i < hi ----
                if (sm.flags[buf]) {
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) {
                            const int key = kb * 32 + q4 * 8 + g2 * 4;
                            const int4 lo = *reinterpret_cast<const int4 *>(&sm.key_lo[buf][key]);
                            const int4 hi = *reinterpret_cast<const int4 *>(&sm.key_hi[buf][key]);
                            if (!(v_i > lo.x && v_i < hi.x)) sacc[kb][q4 * 4 + 0] = -INFINITY;
                            if (!(v_i > lo.y && v_i < hi.y)) sacc[kb][q4 * 4 + 1] = -INFINITY;
                            if (!(v_i > lo.z && v_i < hi.z)) sacc[kb][q4 * 4 + 2] = -INFINITY;
                            if (!(v_i > lo.w && v_i < hi.w)) sacc[kb][q4 * 4 + 3] = -INFINITY;
                        }
                }
                // ---- online softmax (base 2), statistics per lane = per query row ----
                float mx = -INFINITY;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int x = 0; x < 16; ++x) mx = fmaxf(mx, sacc[kb][x]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run, mx);
                const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
                const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * scale_log2e);
                const float mc = m_use * scale_log2e;
                float psum = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int x = 0; x < 16; ++x) {
                        const float pexp = __builtin_amdgcn_exp2f(sacc[kb][x] * scale_log2e - mc);
                        sacc[kb][x] = pexp;
                        psum += pexp;
                    }
                l_run = l_run * alpha + psum;
                m_run = m_new;
#pragma unroll
                for (int db = 0; db < NDB; ++db)
#pragma unroll
                    for (int x = 0; x < 16; ++x) oacc[db][x] *= alpha;
                // ---- O^T += V^T P^T ----
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk) {
                        bf16x8 pf;
#pragma unroll
                        for (int x = 0; x < 8; ++x) pf[x] = (__bf16)sacc[kb][8 * kk + x];
#pragma unroll
                        for (int db = 0; db < NDB; ++db) {
                            const uint16_t *vp = &sm.Vt[(db * 32 + lr) * Smem::VS + kb * 32 + 16 * kk + 4 * g2];
                            union { uint2 u[2]; bf16x8 v; } vf;
                            vf.u[0] = *reinterpret_cast<const uint2 *>(vp);
                            vf.u[1] = *reinterpret_cast<const uint2 *>(vp + 8);
                            oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf, oacc[db], 0, 0, 0);
                        }
                    }
            }
            __syncthreads();
        }
    }

    // ---- epilogue: normalise, round to bf16, store ----
    if (wave_live) {
        const float l_tot = l_run + __shfl_xor(l_run, 32);
        const int r = wave * 32 + lr;
        if (r < nrows) {
            const float inv = 1.f / l_tot;
            uint16_t *op = O + (int64_t)h * os_h + (int64_t)(row0 + r) * os_l;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    union { __bf16 b[4]; uint2 u; } pk;
#pragma unroll
                    for (int x = 0; x < 4; ++x) pk.b[x] = (__bf16)(oacc[db][q4 * 4 + x] * inv);
                    *reinterpret_cast<uint2 *>(op + db * 32 + q4 * 8 + g2 * 4) = pk.u;
                }
        }
    }
}

hipError_t launch_attn_mfma(const Prob &p, const PlanView &pv, const void *Q, const void *K, const void *V,
                            void *O, hipStream_t s) {
    const int grid = attn_grid(p.H_q, p.H_kv, p.G, pv.T1);
    const float c = p.scale * 1.4426950408889634f;
#define DHSA_MFMA(DD)                                                                                       \
    hipLaunchKernelGGL((k_attn_mfma<DD>), dim3(grid), dim3(256), 0, s, pv, (const uint16_t *)Q,             \
                       (const uint16_t *)K, (const uint16_t *)V, (uint16_t *)O, p.N_c, p.H_q, p.H_kv, p.G,  \
                       c, p.qs_h, p.qs_l, p.ks_h, p.ks_l, p.vs_h, p.vs_l, p.os_h, p.os_l)
    if (p.D == 64) DHSA_MFMA(64); else DHSA_MFMA(128);
#undef DHSA_MFMA
    return hipGetLastError();
}

}  // namespace dhsa
