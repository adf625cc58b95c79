// bf16 MFMA sparse attention kernel of libdhsa (Alg. 3 of the paper: tiled
// online softmax over the selected keys; App. C "Backend implementations").
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
// operand of O^T = V^T P^T.  K and V tiles sit row-major in LDS; the V^T
// operand is fetched with the LDS transpose read (ds_read_b64_tr_b16).
//
// K/V rows go from global memory straight into LDS (global_load_lds_dwordx4:
// lane L of a wave fills bytes [16 L, 16 L + 16) of a 1 KiB LDS window), so
// rows are unpadded; bank conflicts are avoided by an XOR swizzle of the
// 16-byte pieces of a row, applied through the choice of which piece each
// lane fetches.
//
// Pipeline per key tile n (one barrier per tile): LDS buffer n%2 holds tile n;
//   issue the loads of tile n+1 into buffer (n+1)%2;  every fourth tile each
//   wave prepares the key list of one later tile;  MFMA + softmax on buffer
//   n%2;  wait for the loads;  barrier
#include <stdlib.h>

#include "dhsa_internal.h"

namespace dhsa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kKT = 64;      // keys per tile
constexpr int kSegB = 256;   // plan entries handled per batch
constexpr int kIntMax = 0x7fffffff;

// XOR swizzle of the 16-byte pieces of LDS row r (only r mod 16 matters).  Eight
// (sixteen for 256-byte rows) consecutive rows get distinct values, so a column
// of 16-byte reads spreads over all banks; rows r..r+3 with r % 4 == 0 differ
// in bits 1-2, so the 32-byte row segments of a transpose read do too.
__device__ __forceinline__ int piece_swizzle(int r, int pieces_per_row) {
    int f = ((r & 3) << 1) | ((r >> 2) & 1);
    if (pieces_per_row == 16) f |= ((r >> 3) & 1) << 3;
    return f;
}

// 16 bytes per lane from global memory straight into LDS: lane L of the wave
// writes bytes [16 L, 16 L + 16) of the window starting at `lds_window`, which
// must be wave-uniform.  Completion is tracked by vmcnt.  (The builtin only
// exists in the device pass.)
__device__ __forceinline__ void load16_to_lds(const uint16_t *g, uint16_t *lds_window) {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_global_load_lds(g, (__attribute__((address_space(3))) void *)lds_window, 16, 0, 0);
#else
    (void)g; (void)lds_window;
#endif
}

template <int D>
struct AttnSmem {
    static constexpr int kTileBytes = kKT * D * 2;   // one K (or V) tile, rows unpadded
    alignas(1024) uint16_t K[2][kKT * D];
    alignas(1024) uint16_t V[2][kKT * D];
    alignas(16) int key_j[8][kKT];
    alignas(16) int key_lo[8][kKT];
    alignas(16) int key_hi[8][kKT];
    alignas(16) int seg_start[kSegB + 16];
    int seg_b0[kSegB];
    int seg_pos[kSegB];
    int seg_rem[kSegB];
    int flags[8];
    int s_wave[4];
};

// blockIdx -> (head, tile).  Workgroups are dealt to the 8 XCDs round-robin and
// each XCD has its own L2.  mode 0: one XCD serves the heads of one kv-group
// and neighbouring row tiles (K/V slabs shared in that L2).  mode 1: plain
// order, all XCDs on the same row tiles, heads fastest.  Tiles are issued from
// the end of the sequence (most keys) to the start.
__device__ __forceinline__ bool decode_block(int mode, int b, int H_q, int H_kv, int G, int T1, int *h,
                                             int *tile) {
    if (mode == 0 && H_kv % 8 == 0) {
        const int x = b & 7, j = b >> 3;
        const int s = j / (G * T1), r = j % (G * T1);
        *tile = T1 - 1 - r / G;
        *h = (x + 8 * s) * G + r % G;
        return true;
    }
    if (mode == 0 && 8 % H_kv == 0) {
        const int S = 8 / H_kv;
        const int x = b & 7, j = b >> 3;
        const int g = x % H_kv, s = x / H_kv;
        const int rank = (j / G) * S + s;
        if (rank >= T1) return false;
        *tile = T1 - 1 - rank;
        *h = g * G + j % G;
        return true;
    }
    if (mode == 2) {  // kv-group major in time: every XCD works on the same kv-head
        const int per = G * T1;
        const int g = b / per, r = b % per;
        *tile = T1 - 1 - r / G;
        *h = g * G + r % G;
        return true;
    }
    *tile = T1 - 1 - b / H_q;
    *h = b % H_q;
    return true;
}

static int attn_grid(int mode, int H_q, int H_kv, int G, int T1) {
    if (mode == 0 && H_kv % 8 != 0 && 8 % H_kv == 0) {
        const int S = 8 / H_kv;
        return 8 * G * ((T1 + S - 1) / S);
    }
    return H_q * T1;
}

template <int D>
__global__ __launch_bounds__(256, 2) void k_attn_mfma(PlanView pv, const uint16_t *__restrict__ Q,
                                                      const uint16_t *__restrict__ K,
                                                      const uint16_t *__restrict__ V, uint16_t *__restrict__ O,
                                                      int N_c, int H_q, int H_kv, int G, int mode,
                                                      float scale_log2e, int64_t qs_h, int64_t qs_l,
                                                      int64_t ks_h, int64_t ks_l, int64_t vs_h, int64_t vs_l,
                                                      int64_t os_h, int64_t os_l) {
    using Smem = AttnSmem<D>;
    constexpr int OPR = D / 8;          // 16-byte pieces per row
    constexpr int KPT = OPR / 4;        // pieces per thread per tile (K and V each)
    constexpr int NS = D / 16;          // MFMA k-steps of Q K^T
    constexpr int NDB = D / 32;         // 32-wide output column blocks
    __shared__ Smem sm;

    int h, tile;
    if (!decode_block(mode, blockIdx.x, H_q, H_kv, G, pv.T1, &h, &tile)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);   // wave-uniform copy (LDS window base goes to M0)
    const int lr = lane & 31, g2 = lane >> 5;
    const int g = h / G;
    const int l = pv.tiles[2 * tile], row0 = pv.tiles[2 * tile + 1];
    const int b_l = pv.B[l];
    const int rows_left = pv.B[l + 1] - row0;
    const int nrows = rows_left < kRowTile ? rows_left : kRowTile;
    const int v_lo = row0 + 1 - b_l, v_hi = v_lo + nrows - 1;
    // which 32-row block this wave owns: rotated per workgroup so that the waves
    // left without rows (short chunks) do not always sit on the same SIMD
    const int rb = (wave + (blockIdx.x >> 3)) & 3;
    const bool wave_live = rb * 32 < nrows;
    const int v_i = v_lo + rb * 32 + lr;  // this lane's query row (may be a padding row)

    const uint16_t *Kg = K + (int64_t)g * ks_h;
    const uint16_t *Vg = V + (int64_t)g * vs_h;

    // Q fragments: B operand of S^T = K Q^T; lane holds row lr, d = 16 s + 8 g2 .. + 7
    bf16x8 qf[NS];
    {
        int r = rb * 32 + lr;
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

    // staging: load instruction c of this wave fills LDS window (4 c + wave) of a
    // tile (1 KiB = 64 pieces); this lane's piece there is row ld_row(c), physical
    // piece lane % OPR, i.e. logical piece (lane % OPR) ^ swizzle(row)
    constexpr int RPW = 64 / OPR;                                     // rows per window
    const int ld_row0 = wave * RPW + lane / OPR;                      // + c * 4 * RPW
    int ld_piece[KPT];
#pragma unroll
    for (int c = 0; c < KPT; ++c) ld_piece[c] = (lane % OPR) ^ piece_swizzle(ld_row0 + c * 4 * RPW, OPR);
    // operand fragments (element offsets inside a tile)
    //   K: row kb*32 + lr, logical piece 2 s + g2
    //   V (transpose read): row kb*32 + 16 kk + 8 half + 4 g2 + c, elements db*32 + 16 dhalf + 4 r
    const int k_sw = piece_swizzle(lr, OPR);
    int k_off[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) k_off[s] = lr * D + 8 * ((2 * s + g2) ^ k_sw);
    const int tr_c = (lane & 15) >> 2, tr_r = lane & 3, tr_dh = (lane >> 4) & 1;
    int v_off[2][NDB];
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
            const int row = 8 * half + 4 * g2 + tr_c;
            const int piece = (4 * db + 2 * tr_dh + (tr_r >> 1)) ^ piece_swizzle(row, OPR);
            v_off[half][db] = row * D + 8 * piece + 4 * (tr_r & 1);
        }

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
        sm.seg_start[tid] = start;                 // entries past the last segment hold `total`
        if (tid < 16) sm.seg_start[kSegB + tid] = total;
        __syncthreads();
        const int nseg = (E - e0 < kSegB) ? E - e0 : kSegB;
        const int ntiles = (total + kKT - 1) / kKT;
        if (ntiles == 0) continue;

// one wave: packed position -> (key index, lo, hi) of tile n.  The segment of a
// position is found with two 16-way steps over the sorted segment starts.
#define DHSA_MAKE_META(n)                                                                       \
    {                                                                                           \
        const int buf_ = (n) & 7;                                                               \
        int x_ = (n) * kKT + lane;                                                              \
        const bool pad_ = x_ >= total;                                                          \
        if (pad_) x_ = total - 1;                                                               \
        int c_ = -1;                                                                            \
        _Pragma("unroll") for (int i_ = 0; i_ < 16; ++i_) c_ += (sm.seg_start[16 * i_] <= x_);  \
        int f_ = -1;                                                                            \
        _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_) {                                      \
            const int4 q_ = *reinterpret_cast<const int4 *>(&sm.seg_start[16 * c_ + 4 * i_]);   \
            f_ += (q_.x <= x_) + (q_.y <= x_) + (q_.z <= x_) + (q_.w <= x_);                    \
        }                                                                                       \
        const int seg_ = 16 * c_ + f_;                                                          \
        const int t_ = x_ - sm.seg_start[seg_];                                                 \
        const int pos_ = sm.seg_pos[seg_];                                                      \
        int lo_ = (pos_ == 1) ? t_ : 0;                                                         \
        int hi_ = (pos_ == 2) ? sm.seg_rem[seg_] - t_ : kIntMax;                                \
        if (pad_) { lo_ = kIntMax; hi_ = kIntMax; }                                             \
        sm.key_j[buf_][lane] = sm.seg_b0[seg_] + t_;                                            \
        sm.key_lo[buf_][lane] = lo_;                                                            \
        sm.key_hi[buf_][lane] = hi_;                                                            \
        const unsigned long long any_ = __ballot((lo_ >= v_lo) || (hi_ <= v_hi));               \
        if (lane == 0) sm.flags[buf_] = any_ != 0ull;                                           \
    }
// issue the global -> LDS loads of tile n into buffer b (completion: vmcnt)
#define DHSA_GLOAD(n, b)                                                                        \
    {                                                                                           \
        const int buf_ = (n) & 7;                                                               \
        _Pragma("unroll") for (int c = 0; c < KPT; ++c) {                                       \
            const int64_t j_ = sm.key_j[buf_][ld_row0 + c * 4 * RPW];                           \
            const int win_ = (4 * c + wave_u) * 512;          /* window offset in elements */   \
            load16_to_lds(Kg + j_ * ks_l + 8 * ld_piece[c], &sm.K[b][win_]);                    \
            load16_to_lds(Vg + j_ * vs_l + 8 * ld_piece[c], &sm.V[b][win_]);                    \
        }                                                                                       \
    }

        if (wave < ntiles) DHSA_MAKE_META(wave);
        __syncthreads();
        DHSA_GLOAD(0, 0);
        __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): this wave's pieces are in LDS
        __syncthreads();
        for (int n = 0; n < ntiles; ++n) {
            const int cur = n & 1;
            if (n + 1 < ntiles) DHSA_GLOAD(n + 1, cur ^ 1);
            if ((n & 3) == 0 && n + 4 + wave < ntiles) DHSA_MAKE_META(n + 4 + wave);
            if (wave_live) {
                const int buf = n & 7;
                const uint16_t *Ks = sm.K[cur];
                const uint16_t *Vs = sm.V[cur];
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
                        const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(&Ks[k_off[s] + kb * 32 * D]);
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
                            sacc[kb][q4 * 4 + 0] = ((v_i > lo.x) & (v_i < hi.x)) ? sacc[kb][q4 * 4 + 0] : -INFINITY;
                            sacc[kb][q4 * 4 + 1] = ((v_i > lo.y) & (v_i < hi.y)) ? sacc[kb][q4 * 4 + 1] : -INFINITY;
                            sacc[kb][q4 * 4 + 2] = ((v_i > lo.z) & (v_i < hi.z)) ? sacc[kb][q4 * 4 + 2] : -INFINITY;
                            sacc[kb][q4 * 4 + 3] = ((v_i > lo.w) & (v_i < hi.w)) ? sacc[kb][q4 * 4 + 3] : -INFINITY;
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
                const float mc = m_use * scale_log2e;
                if (__any(m_new != m_run)) {  // rescale only when some row's maximum moved
                    const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * scale_log2e);
                    l_run *= alpha;
#pragma unroll
                    for (int db = 0; db < NDB; ++db)
#pragma unroll
                        for (int x = 0; x < 16; ++x) oacc[db][x] *= alpha;
                    m_run = m_new;
                }
                float psum = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int x = 0; x < 16; ++x) {
                        const float pexp = __builtin_amdgcn_exp2f(sacc[kb][x] * scale_log2e - mc);
                        sacc[kb][x] = pexp;
                        psum += pexp;
                    }
                l_run += psum;
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
                            // keys kb*32 + 16 kk + 4 g2 + {0..3} and the same + 8; columns db*32 + lr
                            const uint16_t *vb = &Vs[(kb * 32 + 16 * kk) * D];
                            union { s16x4 h[2]; bf16x8 v; } vf;
                            vf.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                (s16x4 __attribute__((address_space(3))) *)(vb + v_off[0][db]));
                            vf.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                (s16x4 __attribute__((address_space(3))) *)(vb + v_off[1][db]));
                            oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf, oacc[db], 0, 0, 0);
                        }
                    }
            }
            __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): the next tile's pieces have landed
            __syncthreads();
        }
#undef DHSA_MAKE_META
#undef DHSA_GLOAD
    }

    // ---- epilogue: normalise, round to bf16, store ----
    if (wave_live) {
        const float l_tot = l_run + __shfl_xor(l_run, 32);
        const int r = rb * 32 + lr;
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
    static const int mode = [] {
        const char *e = getenv("DHSA_ATTN_ORDER");
        return e ? atoi(e) : 2;
    }();
    const int grid = attn_grid(mode, p.H_q, p.H_kv, p.G, pv.T1);
    const float c = p.scale * 1.4426950408889634f;
#define DHSA_MFMA(DD)                                                                                       \
    hipLaunchKernelGGL((k_attn_mfma<DD>), dim3(grid), dim3(256), 0, s, pv, (const uint16_t *)Q,             \
                       (const uint16_t *)K, (const uint16_t *)V, (uint16_t *)O, p.N_c, p.H_q, p.H_kv, p.G,  \
                       mode, c, p.qs_h, p.qs_l, p.ks_h, p.ks_l, p.vs_h, p.vs_l, p.os_h, p.os_l)
    if (p.D == 64) DHSA_MFMA(64); else DHSA_MFMA(128);
#undef DHSA_MFMA
    return hipGetLastError();
}

}  // namespace dhsa
