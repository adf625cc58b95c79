// Sparse attention kernels of libdhsa: exact softmax attention over the keys
// the routing plan selects (Alg. 2 / Alg. 3 of the paper, App. C "Backend
// implementations").  This file: k_attn_rowwise, fp32 arithmetic, one wavefront
// per query row (the DHSA_F32 path).  The bf16 MFMA kernel is in attn_mfma.hip.
#include "dhsa_internal.h"

namespace dhsa {

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
                                                      T *__restrict__ O, int64_t L, int G, float scale,
                                                      int64_t qs_h, int64_t qs_l, int64_t ks_h, int64_t ks_l,
                                                      int64_t vs_h, int64_t vs_l, int64_t os_h, int64_t os_l) {
    constexpr int EP = RowIO<T>::kPer16;
    constexpr int NC = D / 64;  // output columns per lane
    __shared__ float s_q[4][D];
    if (!plan_matches(pv)) return;   // not this problem's plan: O is not written
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
    const int l = chunk_of_row(pv.RB, pv.N_q, i);   // the row's query group
    const int v = (int)(i + 1 - pv.RB[l]);
    const int E = pv.count[(int64_t)h * pv.N_q + l];
    const int32_t *ent = pv.entries + ((int64_t)h * pv.N_q + l) * pv.stride * 2;
    float m_run = -INFINITY, l_lane = 0.f;
    float o[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) o[c] = 0.f;
    for (int e = 0; e < E; ++e) {
        const int w0 = ent[2 * e], rem = ent[2 * e + 1];
        const int k = w0 & kChunkMask, pos = w0 >> kPosShift;
        const int b0 = pv.B[k];
        int take = entry_take(pos, rem, pv.B[k + 1] - b0, v);
        if (pos == 3) {   // row-block form: of the block's list, the keys up to the row itself
            const int64_t vis = i + 1 - b0;
            if (vis < take) take = vis > 0 ? (int)vis : 0;
        }
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
    const float inv = lsum > 0.f ? 1.f / lsum : 0.f;   // a row that sees no key of its block's list: zeros
#pragma unroll
    for (int c = 0; c < NC; ++c)
        RowIO<T>::store(O + (int64_t)h * os_h + i * os_l + lane + 64 * c, o[c] * inv);
}

hipError_t launch_attn_rowwise(const Prob &p, const PlanView &pv, const void *Q, const void *K, const void *V,
                               void *O, hipStream_t s) {
    dim3 grid((unsigned)((p.L + 3) / 4), p.H_q), block(256);
#define DHSA_ROWWISE(T, DD)                                                                                  \
    hipLaunchKernelGGL((k_attn_rowwise<T, DD>), grid, block, 0, s, pv, (const T *)Q, (const T *)K,           \
                       (const T *)V, (T *)O, p.L, p.G, p.scale, p.qs_h, p.qs_l, p.ks_h, p.ks_l,              \
                       p.vs_h, p.vs_l, p.os_h, p.os_l)
    if (p.dtype == DHSA_F32) {
        if (p.D == 64) DHSA_ROWWISE(float, 64); else DHSA_ROWWISE(float, 128);
    } else {
        if (p.D == 64) DHSA_ROWWISE(bf16_t, 64); else DHSA_ROWWISE(bf16_t, 128);
    }
#undef DHSA_ROWWISE
    return hipGetLastError();
}

}  // namespace dhsa
