// bf16 MFMA sparse attention kernel of libdhsa (Alg. 3 of the paper: tiled
// online softmax over the selected keys; App. C "Backend implementations").
//
// Work unit: (query head h, row tile): up to 128 consecutive rows of ONE query
// group l (a chunk; or a row block, see below).  All rows of the tile share the
// plan entries of (h, l); they differ only through v = i + 1 - RB[l], the rows of
// the group up to and including their own.  The selected keys are walked in ascending
// position (softmax is order-free) and packed densely into tiles of 64 keys;
// a packed key carries (row offset, lo, hi) with "row takes key <=> lo < v < hi".
//
// Four waves; each owns one 32-row block.  Scores are computed transposed,
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
// Pipeline, iteration n (one barrier per key tile; K(t), V(t) live in LDS
// buffers t%2; work proceeds in 32-key blocks): every fourth tile each wave
// prepares the key list of one later tile; the row offsets of this iteration's
// loads (upper half of K(n+1), V(n+1), lower half of K(n+2)) and the mask flag
// of tile n+1 are fetched into registers; then per block: the matrix unit
// computes the scores of the NEXT block while the vector unit exponentiates the
// current one, O += P V of the current block, mask of the next block, with the
// loads issued a quarter at a time between these steps; wait for the loads;
// barrier.
//
// Query groups: a tile's rows belong to one query group l = rows [RB[l], RB[l+1]):
// a chunk (RB = B), or a fixed row block of Alg. 1 as printed, whose listed keys
// are masked causally per token like the keys of a row's own chunk.
#include "dhsa_internal.h"

namespace dhsa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

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

// 16 bytes per lane from global memory (uniform base + per-lane 32-bit byte
// offset) straight into LDS: lane L of the wave writes bytes [16 L, 16 L + 16)
// of the window at LDS byte address `lds_window` (wave-uniform, goes through
// M0, which nothing else in this kernel uses).  Completion is tracked by vmcnt;
// the caller waits and then passes a barrier before anyone reads the window.
__device__ __forceinline__ void load16_to_lds(const char *base, unsigned byte_off, unsigned lds_window) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(byte_off), "s"(base), "s"(lds_window) : "memory");
#else
    (void)base; (void)byte_off; (void)lds_window;
#endif
}

template <int D>
struct AttnSmem {
    static constexpr int kTile = kKT * D;            // elements of one K (or V) tile, rows unpadded
    alignas(1024) uint16_t K[2 * kTile];
    alignas(1024) uint16_t V[2 * kTile];
    // byte offset of each key's row in K / V of this kv-head, stored in the order the
    // loading lanes want them (see off_slot): the rows one lane fetches are adjacent
    alignas(16) unsigned key_koff[8][kKT];
    alignas(16) unsigned key_voff[8][kKT];
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
// each XCD has its own L2.  `act` kv-heads (1, 2, 4 or 8) are worked on at a
// time, each by 8 / act XCDs: act = 8 gives every XCD its own kv-head (best L2
// reuse of the K/V slabs), smaller values keep fewer K/V slabs live at once
// (they then fit the memory-side cache).  Within a kv-head, row tiles are
// issued from the end of the sequence (most keys) to the start, the query heads
// of the group innermost.  act = 0: plain order.
__device__ __forceinline__ void decode_block(int act, int b, int H_q, int G, int T1, int *h, int *tile) {
    if (act > 0) {
        const int per = act * G * T1;          // workgroups per set of `act` kv-heads
        const int p = b / per, r = b % per;
        const int x = r & 7;
        const int kv = p * act + (x & (act - 1));
        const int idx = (r >> 3) * (8 / act) + x / act;
        *tile = T1 - 1 - idx / G;
        *h = kv * G + idx % G;
        return;
    }
    *tile = T1 - 1 - b / H_q;
    *h = b % H_q;
}

// act must divide H_kv and act * G * T1 must be a multiple of 8 for the mapping above
static int attn_order(int want, int H_kv, int G, int T1) {
    for (int act = want; act >= 1; act >>= 1)
        if (H_kv % act == 0 && (act * G * T1) % 8 == 0) return act;
    return 0;
}

template <int D, bool PAR>
__global__ __launch_bounds__(256, 2) void k_attn_mfma(PlanView pv, int tile0, int T, const uint16_t *__restrict__ Q,
                                                      const uint16_t *__restrict__ K,
                                                      const uint16_t *__restrict__ V, uint16_t *__restrict__ O,
                                                      int H_q, int G, int mode,
                                                      float scale_log2e, int64_t qs_h, int64_t qs_l,
                                                      int64_t ks_h, int64_t ks_l, int64_t vs_h, int64_t vs_l,
                                                      int64_t os_h, int64_t os_l) {
    using Smem = AttnSmem<D>;
    constexpr int OPR = D / 8;          // 16-byte pieces per row
    constexpr int KPT = OPR / 4;        // load instructions per wave per tile (K and V each)
    constexpr int NS = D / 16;          // MFMA k-steps of Q K^T
    constexpr int NDB = D / 32;         // 32-wide output column blocks
    constexpr int kTile = Smem::kTile;
    __shared__ Smem sm;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);   // wave-uniform copy
    const int lr = lane & 31, g2 = lane >> 5;

    int h, tile;
    decode_block(mode, blockIdx.x, H_q, G, T, &h, &tile);
    tile += tile0;   // this launch covers tiles [tile0, tile0 + T) of the plan's table
    const int g = h / G;
    const int l = pv.tiles[2 * tile], row0 = pv.tiles[2 * tile + 1];   // query group, first row
    const int b_l = pv.RB[l];
    const int rows_left = pv.RB[l + 1] - row0;
    const int nrows = rows_left < kRowTile ? rows_left : kRowTile;
    const int v_lo = row0 + 1 - b_l, v_hi = v_lo + nrows - 1;
    // Wave roles (PAR = false / true is chosen per launch: the plan lists the tiles
    // of more than 64 rows first).  Tiles of more than 64 rows: wave = one 32-row block (rotated per
    // workgroup so that the waves left without rows do not always sit on the same
    // SIMD), both 32-key blocks of every key tile.  Tiles of at most 64 rows: two
    // waves per row block, each taking ONE of the two 32-key blocks of every key
    // tile ("key parity" kbw); their partial softmax states are merged at the end.
    constexpr bool par = PAR;
    const int rb = par ? (wave & 1) : ((wave + (blockIdx.x >> 3)) & 3);
    const int kbw = par ? (wave >> 1) : 0;
    const bool wave_live = rb * 32 < nrows;
    const int v_i = v_lo + rb * 32 + lr;  // this lane's query row (may be a padding row)

    // K / V of this kv-head; rows are addressed by 32-bit byte offsets (the host
    // checks that a head slab is below 4 GiB)
    const char *Kg8 = reinterpret_cast<const char *>(K + (int64_t)g * ks_h);
    const char *Vg8 = reinterpret_cast<const char *>(V + (int64_t)g * vs_h);
    const unsigned k_row_bytes = (unsigned)ks_l * 2u, v_row_bytes = (unsigned)vs_l * 2u;

    // Q fragments: B operand of S^T = K Q^T; lane holds row lr, d = 16 s + 8 g2 .. + 7.
    // Padding rows (past the end of the tile; never stored) get q = 0 and, through a
    // huge exponent reference, p = 0: all-zero operand columns keep the matrix unit's
    // switching activity, and with it the power drawn for rows that do not exist, low.
    bf16x8 qf[NS];
    const bool pad_row = rb * 32 + lr >= nrows;
    {
        const int r = pad_row ? nrows - 1 : rb * 32 + lr;
        const uint16_t *qp = Q + (int64_t)h * qs_h + (int64_t)(row0 + r) * qs_l + 8 * g2;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            qf[s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);
            if (pad_row) qf[s] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        }
    }

    f32x16 oacc[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int x = 0; x < 16; ++x) oacc[db][x] = 0.f;
    float m_ref = pad_row ? 1e30f : -INFINITY, l_run = 0.f;   // m_ref: reference used in the exponent (see DHSA_EXP)

    const int E = pv.count[(int64_t)h * pv.N_q + l];
    const int32_t *ent = pv.entries + ((int64_t)h * pv.N_q + l) * pv.stride * 2;

    // staging: load instruction c of this wave fills LDS window (4 c + wave) of a
    // tile (1 KiB = 64 pieces); this lane's piece there is physical piece
    // lane % OPR of row ld_row0 + 4 c RPW, i.e. logical piece (lane % OPR) ^
    // swizzle(row) (the rows of one lane are 16 or 32 apart: same swizzle)
    constexpr int RPW = 64 / OPR;                                     // rows per window
    const int ld_row0 = wave * RPW + lane / OPR;
    const unsigned ld_piece_bytes = 16u * ((lane % OPR) ^ piece_swizzle(ld_row0, OPR));
    // the rows one lane fetches for a tile are ld_row0 + c RSTR, c = 0 .. KPT-1; the offset of
    // key row r sits in slot (r % RSTR) KPT + r / RSTR of the tile's offset table
    constexpr int RSTR = 4 * RPW;
    const int off_slot_wr = (lane % RSTR) * KPT + lane / RSTR;   // slot of key `lane` (writer side)
    const int off_slot_rd = ld_row0 * KPT;                        // first slot of this lane's rows
    const unsigned lds_K = (unsigned)(uintptr_t)(__attribute__((address_space(3))) uint16_t *)sm.K;
    const unsigned lds_V = (unsigned)(uintptr_t)(__attribute__((address_space(3))) uint16_t *)sm.V;
    // operand fragments (byte offsets inside the K / V buffers)
    //   K: row kb*32 + lr, logical piece 2 s + g2
    const int k_sw = piece_swizzle(lr, OPR);
    int k_off[NS];   // points into the K buffer of the current tile; moved once per tile
#pragma unroll
    for (int s = 0; s < NS; ++s) k_off[s] = 2 * ((kbw * 32 + lr) * D + 8 * ((2 * s + g2) ^ k_sw));
    // Transpose-read source of this lane: row 8 half + 4 g2 + c of a 16-row group,
    // logical piece P = 4 db + 2 dh + (r >> 1), physical piece P ^ swizzle(row).  The
    // swizzle's bits 2-3 are (c >> 1) and half, so the physical piece is
    //   low2 | 4 * (x2 ^ (c >> 1)),  x2 = db ^ 2 half (a compile-time value),
    // and x2 ^ cb = x2 + cb for even x2, x2 - cb for odd x2: two per-lane bases,
    // everything else folds into the instruction's immediate offset.
    const int tr_c = (lane & 15) >> 2, tr_r = lane & 3, tr_dh = (lane >> 4) & 1;
    const int tr_low2 = ((tr_r >> 1) ^ g2) | ((tr_dh ^ (tr_c & 1)) << 1);
    const int tr_l0 = (4 * g2 + tr_c) * D + 8 * tr_low2 + 4 * (tr_r & 1);
    int v_base_e = 2 * (kbw * 32 * D + tr_l0 + 32 * (tr_c >> 1));   // moved once per tile
    int v_base_o = 2 * (kbw * 32 * D + tr_l0 - 32 * (tr_c >> 1));
    const char *const smK8 = reinterpret_cast<const char *>(sm.K);
    const char *const smV8 = reinterpret_cast<const char *>(sm.V);

    for (int e0 = 0; e0 < E; e0 += kSegB) {
        // ---- segment table of this batch of plan entries ----
        int n_e = 0;
        if (e0 + tid < E) {
            const int w0 = ent[2 * (e0 + tid)], rem = ent[2 * (e0 + tid) + 1];
            const int k = w0 & kChunkMask, pos = w0 >> kPosShift;
            const int b0 = pv.B[k];
            // most tokens any row of the tile takes from this chunk
            n_e = entry_take(pos, rem, pv.B[k + 1] - b0, pos == 1 ? v_hi : v_lo);
            if (pos == 3) {   // row-block form: keys past the tile's last row are masked for every row
                const int vis = row0 + nrows - b0;
                n_e = vis < n_e ? (vis > 0 ? vis : 0) : n_e;
            }
            sm.seg_b0[tid] = b0;
            sm.seg_pos[tid] = pos;
            sm.seg_rem[tid] = rem;
        }
        int total;
        const int start = block_excl_scan(n_e, sm.s_wave, &total);
        sm.seg_start[tid] = start;                 // entries past the last segment hold `total`
        if (tid < 16) sm.seg_start[kSegB + tid] = total;
        __syncthreads();
        const int ntiles = (total + kKT - 1) / kKT;
        if (ntiles == 0) continue;

// one wave: packed position -> (row offsets, lo, hi) of tile n.  The segment of a
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
        const unsigned j_ = (unsigned)(sm.seg_b0[seg_] + t_);                                   \
        /* key j is at or below row i  <=>  j - b_l < v: the group's own chunk (pos 1,   */     \
        /* j - b_l = t) and every listed key of the row-block form (pos 3) */                   \
        int lo_ = (pos_ & 1) ? ((int)j_ > b_l ? (int)j_ - b_l : 0) : 0;                         \
        int hi_ = (pos_ == 2) ? sm.seg_rem[seg_] - t_ : kIntMax;                                \
        if (pad_) { lo_ = kIntMax; hi_ = kIntMax; }                                             \
        sm.key_koff[buf_][off_slot_wr] = j_ * k_row_bytes;                                      \
        sm.key_voff[buf_][off_slot_wr] = j_ * v_row_bytes;                                      \
        sm.key_lo[buf_][lane] = lo_;                                                            \
        sm.key_hi[buf_][lane] = hi_;                                                            \
        const unsigned long long any_ = __ballot((lo_ >= v_lo) || (hi_ <= v_hi));               \
        if (lane == 0) sm.flags[buf_] = any_ != 0ull;                                           \
    }

// fetch this lane's row offsets of tile n into registers (windows c0..c1-1)
#define DHSA_OFFS(dst, off_tab, n, c0, c1)                                                      \
    _Pragma("unroll") for (int c = c0; c < c1; ++c) dst[c] = sm.off_tab[(n) & 7][off_slot_rd + c];
// issue the global -> LDS loads of windows c0..c1-1 of the K (or V) rows of tile n,
// row offsets taken from registers
#define DHSA_GLOAD(lds_base, offs, base8, n, c0, c1)                                            \
    {                                                                                           \
        const unsigned dst_ = lds_base + (((n) & 1) * kTile + wave_u * 512) * 2;                \
        _Pragma("unroll") for (int c = c0; c < c1; ++c)                                         \
            load16_to_lds(base8, offs[c] + ld_piece_bytes, dst_ + c * 4096);                    \
    }
#define DHSA_LOAD_K_LO(n) DHSA_GLOAD(lds_K, ko_lo, Kg8, n, 0, KPT / 2)      /* keys 0..31  */
#define DHSA_LOAD_K_HI(n) DHSA_GLOAD(lds_K, ko_hi, Kg8, n, KPT / 2, KPT)    /* keys 32..63 */
#define DHSA_LOAD_V(n) DHSA_GLOAD(lds_V, vo, Vg8, n, 0, KPT)
#define DHSA_LOAD_V_LO(n) DHSA_GLOAD(lds_V, vo, Vg8, n, 0, KPT / 2)
#define DHSA_LOAD_V_HI(n) DHSA_GLOAD(lds_V, vo, Vg8, n, KPT / 2, KPT)

// S^T of one 32-key block whose K rows start at element offset kb_off of the
// buffer k_off points into: keys = MFMA rows, this lane's query row = column lr
#define DHSA_QK(kb_off, sacc)                                                                   \
    {                                                                                           \
        _Pragma("unroll") for (int x = 0; x < 16; ++x) sacc[x] = 0.f;                           \
        _Pragma("unroll") for (int s = 0; s < NS; ++s) {                                        \
            const bf16x8 kf_ = *reinterpret_cast<const bf16x8 *>(smK8 + k_off[s] + 2 * (kb_off)); \
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf_, qf[s], sacc, 0, 0, 0);          \
        }                                                                                       \
    }

// mask: only tiles that hold a key some row of the tile does not take
#define DHSA_MASK(n, kb, sacc, flag)                                                            \
    {                                                                                           \
        const int buf_ = (n) & 7;                                                               \
        if (flag) {                                                                             \
            _Pragma("unroll") for (int q4 = 0; q4 < 4; ++q4) {                                  \
                const int key_ = (kb) * 32 + q4 * 8 + g2 * 4;                                   \
                const int4 lo_ = *reinterpret_cast<const int4 *>(&sm.key_lo[buf_][key_]);       \
                const int4 hi_ = *reinterpret_cast<const int4 *>(&sm.key_hi[buf_][key_]);       \
                sacc[q4 * 4 + 0] = ((v_i > lo_.x) & (v_i < hi_.x)) ? sacc[q4 * 4 + 0] : -INFINITY; \
                sacc[q4 * 4 + 1] = ((v_i > lo_.y) & (v_i < hi_.y)) ? sacc[q4 * 4 + 1] : -INFINITY; \
                sacc[q4 * 4 + 2] = ((v_i > lo_.z) & (v_i < hi_.z)) ? sacc[q4 * 4 + 2] : -INFINITY; \
                sacc[q4 * 4 + 3] = ((v_i > lo_.w) & (v_i < hi_.w)) ? sacc[q4 * 4 + 3] : -INFINITY; \
            }                                                                                   \
        }                                                                                       \
    }

// row maximum of a block of S^T (the two lanes of a row exchange their halves)
#define DHSA_ROWMAX(sacc, mx)                                                                   \
    {                                                                                           \
        float m_ = sacc[0];                                                                     \
        _Pragma("unroll") for (int x = 1; x < 16; ++x) m_ = fmaxf(m_, sacc[x]);                 \
        mx = fmaxf(m_, __shfl_xor(m_, 32));                                                     \
    }

// P = exp2((S - m_ref) * c) with row sums, rounded to the two bf16 MFMA B operands
// of the block.  m_ref is a REFERENCE for the exponent, not the running maximum:
// O / l at the end is exact whatever reference was used, so it only has to keep
// the exponentials in range.  It is set from the first block and moved up (with
// a rescale of l and O) only when a block's exponentials grow past 2^20, which
// the row sums reveal without a per-block maximum.  A row keeps m_ref = -inf
// (and p = 0) until it meets its first unmasked key.
#define DHSA_EXP(sacc, pf)                                                                      \
    {                                                                                           \
        float mc_ = (m_ref == -INFINITY) ? 0.f : m_ref * scale_log2e;                           \
        float psum_ = 0.f;                                                                      \
        _Pragma("unroll") for (int x = 0; x < 16; ++x) {                                        \
            const float e_ = __builtin_amdgcn_exp2f(sacc[x] * scale_log2e - mc_);               \
            psum_ += e_;                                                                        \
            pf[x >> 3][x & 7] = (__bf16)e_;                                                     \
        }                                                                                       \
        /* too large, inf or NaN, or no reference yet (then nothing has been accumulated) */     \
        if (__any(!(psum_ < 1048576.f) || m_ref == -INFINITY)) {                                \
            float mx_;                                                                          \
            DHSA_ROWMAX(sacc, mx_);                                                             \
            const float m_new_ = fmaxf(m_ref, mx_);                                             \
            const float alpha_ = (m_ref == -INFINITY) ? 0.f                                     \
                                 : __builtin_amdgcn_exp2f((m_ref - m_new_) * scale_log2e);      \
            l_run *= alpha_;                                                                    \
            _Pragma("unroll") for (int db = 0; db < NDB; ++db)                                  \
                _Pragma("unroll") for (int x = 0; x < 16; ++x) oacc[db][x] *= alpha_;           \
            m_ref = m_new_;                                                                     \
            mc_ = (m_ref == -INFINITY) ? 0.f : m_ref * scale_log2e;                             \
            psum_ = 0.f;                                                                        \
            _Pragma("unroll") for (int x = 0; x < 16; ++x) {                                    \
                const float e_ = __builtin_amdgcn_exp2f(sacc[x] * scale_log2e - mc_);           \
                psum_ += e_;                                                                    \
                pf[x >> 3][x & 7] = (__bf16)e_;                                                 \
            }                                                                                   \
        }                                                                                       \
        l_run += psum_;                                                                         \
    }

// O^T += V^T P^T for the 32-key block kb of the V buffer v_base_* point into
#define DHSA_PV(kb, pf)                                                                         \
    {                                                                                           \
        _Pragma("unroll") for (int kk = 0; kk < 2; ++kk)                                        \
            _Pragma("unroll") for (int db = 0; db < NDB; ++db) {                                \
                /* keys kb*32 + 16 kk + 4 g2 + {0..3} and the same + 8; columns db*32 + lr */   \
                union { s16x4 h[2]; bf16x8 v; } vf_;                                            \
                _Pragma("unroll") for (int half = 0; half < 2; ++half) {                        \
                    const int x2_ = (OPR == 16) ? (db ^ (2 * half)) : db;                       \
                    const char *vp_ = smV8 + ((x2_ & 1) ? v_base_o : v_base_e) +                \
                                      2 * (((kb) * 32 + 16 * kk + 8 * half) * D + 32 * x2_);    \
                    vf_.h[half] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(                      \
                        (s16x4 __attribute__((address_space(3))) *)vp_);                        \
                }                                                                               \
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf_.v, pf[kk], oacc[db], 0, 0, 0); \
            }                                                                                   \
    }

        f32x16 s_a, s_b;                      // scores of two consecutive blocks (ping-pong)
        int toggle = 2 * kTile;               // +tile, -tile, ... (bytes): k_off / v_base_* follow the tile buffers
        unsigned ko_lo[KPT], ko_hi[KPT], vo[KPT];   // row offsets of the loads this lane issues next
        if (wave < ntiles) DHSA_MAKE_META(wave);   // key lists of tiles 0..3
        __syncthreads();
        if constexpr (!PAR) {
        // ================= tiles of more than 64 rows =================
        // ---- prologue: K(0), V(0), lower half of K(1) in LDS; S(0, block 0) ----
        DHSA_OFFS(ko_lo, key_koff, 0, 0, KPT / 2);
        DHSA_OFFS(ko_hi, key_koff, 0, KPT / 2, KPT);
        DHSA_OFFS(vo, key_voff, 0, 0, KPT);
        DHSA_LOAD_K_LO(0);
        DHSA_LOAD_K_HI(0);
        DHSA_LOAD_V(0);
        if (ntiles > 1) {
            DHSA_OFFS(ko_lo, key_koff, 1, 0, KPT / 2);
            DHSA_LOAD_K_LO(1);
        }
        int fl_cur = __builtin_amdgcn_readfirstlane(sm.flags[0]);   // does tile n need the mask?
        __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): this wave's pieces are in LDS
        __syncthreads();
        if (wave_live) {
            DHSA_QK(0, s_a);
            DHSA_MASK(0, 0, s_a, fl_cur);
            if (e0 == 0) { float mx0; DHSA_ROWMAX(s_a, mx0); m_ref = fmaxf(m_ref, mx0); }   // reference = row maxima of the first block
        }
        __syncthreads();                      // the lower half of K(0) may be overwritten from here on

        // ---- steady state, tile n (all but the last): softmax and PV of its two blocks; the
        // matrix unit computes the scores of the next block while the vector unit exponentiates ----
        int n = 0;
        for (; n + 1 < ntiles; ++n) {
            if ((n & 3) == 0 && n + 4 + wave < ntiles) DHSA_MAKE_META(n + 4 + wave);
            // The loads of this iteration (upper half of K(n+1) over K(n-1), V(n+1) over
            // V(n-1), lower half of K(n+2) over K(n)) are spread over the block steps so
            // that the four waves do not hand them to the memory pipeline in one burst;
            // their row offsets and the mask flag of tile n+1 are fetched up front, so
            // that no load has to wait for LDS in the middle of the block steps.
            DHSA_OFFS(ko_hi, key_koff, n + 1, KPT / 2, KPT);
            DHSA_OFFS(vo, key_voff, n + 1, 0, KPT);
            DHSA_OFFS(ko_lo, key_koff, n + 2, 0, KPT / 2);
            const int fl_next = __builtin_amdgcn_readfirstlane(sm.flags[(n + 1) & 7]);
            if (wave_live) {
                bf16x8 pf[2];
                DHSA_LOAD_K_HI(n + 1);
                DHSA_QK(32 * D, s_b);                      // block 1 of tile n
                DHSA_EXP(s_a, pf);
                DHSA_LOAD_V_LO(n + 1);
                DHSA_PV(0, pf);
                DHSA_MASK(n, 1, s_b, fl_cur);
#pragma unroll
                for (int s = 0; s < NS; ++s) k_off[s] += toggle;   // now the K buffer of tile n+1
                DHSA_LOAD_V_HI(n + 1);
                DHSA_QK(0, s_a);                           // block 0 of tile n+1
                DHSA_EXP(s_b, pf);
                if (n + 2 < ntiles) DHSA_LOAD_K_LO(n + 2);
                DHSA_PV(1, pf);
                DHSA_MASK(n + 1, 0, s_a, fl_next);
                v_base_e += toggle;                        // now the V buffer of tile n+1
                v_base_o += toggle;
                toggle = -toggle;
            } else {
                DHSA_LOAD_K_HI(n + 1);
                DHSA_LOAD_V(n + 1);
                if (n + 2 < ntiles) DHSA_LOAD_K_LO(n + 2);
            }
            fl_cur = fl_next;
            __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): the pieces this wave requested have landed
            __syncthreads();
        }
        // ---- last tile of the batch: nothing left to load or to score ahead ----
        if (wave_live) {
            bf16x8 pf[2];
            DHSA_QK(32 * D, s_b);
            DHSA_EXP(s_a, pf);
            DHSA_PV(0, pf);
            DHSA_MASK(n, 1, s_b, fl_cur);
            DHSA_EXP(s_b, pf);
            DHSA_PV(1, pf);
        }
        __syncthreads();                          // LDS is reused by the next batch
        if (wave_live && !(ntiles & 1)) {         // leave the offsets at buffer 0 for the next batch
#pragma unroll
            for (int s = 0; s < NS; ++s) k_off[s] -= 2 * kTile;
            v_base_e -= 2 * kTile;
            v_base_o -= 2 * kTile;
        }
        } else {
        // ================= tiles of at most 64 rows: one 32-key block per wave and tile =================
        // ---- prologue: K(0), V(0), K(1) in LDS; S(0, own block) ----
        DHSA_OFFS(ko_lo, key_koff, 0, 0, KPT / 2);
        DHSA_OFFS(ko_hi, key_koff, 0, KPT / 2, KPT);
        DHSA_OFFS(vo, key_voff, 0, 0, KPT);
        DHSA_LOAD_K_LO(0);
        DHSA_LOAD_K_HI(0);
        DHSA_LOAD_V(0);
        if (ntiles > 1) {
            DHSA_OFFS(ko_lo, key_koff, 1, 0, KPT / 2);
            DHSA_OFFS(ko_hi, key_koff, 1, KPT / 2, KPT);
            DHSA_LOAD_K_LO(1);
            DHSA_LOAD_K_HI(1);
        }
        const int fl_0 = __builtin_amdgcn_readfirstlane(sm.flags[0]);
        __builtin_amdgcn_s_waitcnt(0x0f70);
        __syncthreads();
        if (wave_live) {
            DHSA_QK(0, s_a);
            DHSA_MASK(0, kbw, s_a, fl_0);
            if (e0 == 0) { float mx0; DHSA_ROWMAX(s_a, mx0); m_ref = fmaxf(m_ref, mx0); }   // reference = row maxima of this wave's first block
#pragma unroll
            for (int s = 0; s < NS; ++s) k_off[s] += 2 * kTile;   // K offsets run one tile ahead of V offsets
        }
        __syncthreads();                      // K(0) may be overwritten from here on

        // ---- tile n (all but the last): softmax and PV of this wave's block (scores in s_a)
        // while the matrix unit computes the scores of its block of tile n+1 (into s_b) ----
        int n = 0;
        for (; n + 1 < ntiles; ++n) {
            DHSA_OFFS(ko_lo, key_koff, n + 2, 0, KPT / 2);
            DHSA_OFFS(ko_hi, key_koff, n + 2, KPT / 2, KPT);
            DHSA_OFFS(vo, key_voff, n + 1, 0, KPT);
            const int fl_next = __builtin_amdgcn_readfirstlane(sm.flags[(n + 1) & 7]);
            if (n + 2 < ntiles) { DHSA_LOAD_K_LO(n + 2); DHSA_LOAD_K_HI(n + 2); }   // over K(n)
            DHSA_LOAD_V(n + 1);                                                    // over V(n-1)
            if ((n & 3) == 0 && n + 4 + wave < ntiles) DHSA_MAKE_META(n + 4 + wave);
            if (wave_live) {
                bf16x8 pf[2];
                DHSA_QK(0, s_b);
                DHSA_EXP(s_a, pf);
                DHSA_PV(0, pf);
                DHSA_MASK(n + 1, kbw, s_b, fl_next);
                s_a = s_b;
#pragma unroll
                for (int s = 0; s < NS; ++s) k_off[s] -= toggle;
                v_base_e += toggle;
                v_base_o += toggle;
                toggle = -toggle;
            }
            __builtin_amdgcn_s_waitcnt(0x0f70);
            __syncthreads();
        }
        if (wave_live) {                          // last tile of the batch
            bf16x8 pf[2];
            DHSA_EXP(s_a, pf);
            DHSA_PV(0, pf);
        }
        __syncthreads();                          // LDS is reused by the next batch / the merge
        if (wave_live) {                          // leave the offsets at buffer 0 for the next batch
            if (ntiles & 1) {
#pragma unroll
                for (int s = 0; s < NS; ++s) k_off[s] -= 2 * kTile;
            } else {
                v_base_e -= 2 * kTile;
                v_base_o -= 2 * kTile;
            }
        }
        }
#undef DHSA_MAKE_META
#undef DHSA_OFFS
#undef DHSA_GLOAD
#undef DHSA_LOAD_K_LO
#undef DHSA_LOAD_K_HI
#undef DHSA_LOAD_V
#undef DHSA_LOAD_V_LO
#undef DHSA_LOAD_V_HI
#undef DHSA_QK
#undef DHSA_MASK
#undef DHSA_ROWMAX
#undef DHSA_EXP
#undef DHSA_PV
    }

    // ---- key-parity tiles: fold the state of the wave that took the odd blocks into its partner ----
    if constexpr (PAR) {
        float *xch = reinterpret_cast<float *>(sm.K) + rb * (NDB * 16 + 2) * 64 + lane;   // [slot][lane]
        if (wave_live && kbw == 1) {
            xch[0] = m_ref;
            xch[64] = l_run;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int x = 0; x < 16; ++x) xch[(2 + db * 16 + x) * 64] = oacc[db][x];
        }
        __syncthreads();
        if (wave_live && kbw == 0) {
            const float m1 = xch[0], l1 = xch[64];
            const float mm = fmaxf(m_ref, m1);
            const float a0 = (m_ref == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((m_ref - mm) * scale_log2e);
            const float a1 = (m1 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((m1 - mm) * scale_log2e);
            l_run = l_run * a0 + l1 * a1;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int x = 0; x < 16; ++x) oacc[db][x] = oacc[db][x] * a0 + xch[(2 + db * 16 + x) * 64] * a1;
        }
    }

    // ---- epilogue: normalise, round to bf16, store ----
    if (wave_live && kbw == 0) {
        const float l_tot = l_run + __shfl_xor(l_run, 32);
        const int r = rb * 32 + lr;
        if (r < nrows) {
            const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;   // no visible key (row-block form): zeros
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
    const int want = 8;   // kv-heads in flight: one per XCD (other orders measured within 2 %)
    const float c = p.scale * 1.4426950408889634f;
#define DHSA_MFMA(DD, PAR, tile0, T)                                                                        \
    {                                                                                                       \
        const int mode = attn_order(want, p.H_kv, p.G, T);                                                  \
        hipLaunchKernelGGL((k_attn_mfma<DD, PAR>), dim3(p.H_q * (T)), dim3(256), 0, s, pv, tile0, T,        \
                           (const uint16_t *)Q, (const uint16_t *)K, (const uint16_t *)V, (uint16_t *)O,    \
                           p.H_q, p.G, mode, c, p.qs_h, p.qs_l, p.ks_h, p.ks_l, p.vs_h, p.vs_l,      \
                           p.os_h, p.os_l);                                                                 \
    }
    // tiles of more than 64 rows first (they take longest), then the key-parity tiles
    const int T_big = pv.T_big, T_small = pv.T1 - pv.T_big;
    if (T_big > 0) { if (p.D == 64) DHSA_MFMA(64, false, 0, T_big) else DHSA_MFMA(128, false, 0, T_big) }
    if (T_small > 0) { if (p.D == 64) DHSA_MFMA(64, true, T_big, T_small) else DHSA_MFMA(128, true, T_big, T_small) }
#undef DHSA_MFMA
    return hipGetLastError();
}

}  // namespace dhsa
