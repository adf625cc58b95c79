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
// Row tiles are launched by height: tiles of more than 64 rows on the body
// described next (attn_tile_32), tiles of at most 64 and at most 32 rows on 16-row
// MFMA blocks (attn_tile_16, described at that function), one launch each.
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
#include <stddef.h>

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
    alignas(16) int seg_start[kSegB + 80];   // the entries past the last segment hold the batch's key count
    int meta_tmp[4][kKT];                   // per wave: marks of the segment starts inside a tile
    int seg_b0[kSegB];
    int seg_pos[kSegB];
    int seg_rem[kSegB];
    int flags[8];
    int s_wave[8];
};

// blockIdx -> (head, tile).  Workgroups are dealt to the 8 XCDs round-robin and
// each XCD has its own L2.  `act` kv-heads (1, 2, 4 or 8) are worked on at a
// time, each by 8 / act XCDs: act = 8 gives every XCD its own kv-head (best L2
// reuse of the K/V slabs), smaller values keep fewer K/V slabs live at once
// (they then fit the memory-side cache).  Within a kv-head the query heads of
// the group are innermost; *tile is the tile's position in the order of issue
// (0 = first), which the kernel maps to a row tile.  act = 0: plain order.
__device__ __forceinline__ void decode_block(int act, int b, int H_q, int G, int T1, int *h, int *tile) {
    if (act > 0) {
        const int per = act * G * T1;          // workgroups per set of `act` kv-heads
        const int p = b / per, r = b % per;
        const int x = r & 7;
        const int kv = p * act + (x & (act - 1));
        const int idx = (r >> 3) * (8 / act) + x / act;
        *tile = idx / G;
        *h = kv * G + idx % G;
        return;
    }
    *tile = b / H_q;
    *h = b % H_q;
}

// act must divide H_kv and act * G * T1 must be a multiple of 8 for the mapping above
static int attn_order(int want, int H_kv, int G, int T1) {
    for (int act = want; act >= 1; act >>= 1)
        if (H_kv % act == 0 && (act * G * T1) % 8 == 0) return act;
    return 0;
}

// ---------------------------------------------------------------------------
// Key lists and loads, shared by the two kernels below (they use the same names
// for the variables these macros touch: sm, lane, tid, wave_u, total, v_lo, v_hi,
// b_l, row0, nrows, k_row_bytes, v_row_bytes, off_slot_wr, off_slot_rd, lds_K,
// lds_V, Kg8, Vg8, ld_piece_bytes_k / _v, ko_lo, ko_hi, vo, KPT, kTile).
// ---------------------------------------------------------------------------
// Segment table of the batch of plan entries [e0, e0 + kSegB) for this tile.  A segment is an entry
// some row of the tile takes a key from; segments are stored compacted, in entry order: the first
// packed position of their keys (an exclusive scan of the most tokens any row of the tile takes
// from the entry; for the row-block form keys past the tile's last row are dropped), the chunk's
// first token, pos and rem.  Defines `total` (packed keys of the batch), `nseg` and the wave's
// segment cursor.  Contains block barriers.
#define DHSA_SEGMENT_TABLE(e0) \
    int n_e = 0, b0_e = 0, pos_e = 0, rem_e = 0; \
    if (e0 + tid < E) { \
        const int w0 = ent[2 * (e0 + tid)]; \
        rem_e = ent[2 * (e0 + tid) + 1]; \
        const int k = w0 & kChunkMask; \
        pos_e = w0 >> kPosShift; \
        b0_e = pv.B[k]; \
        n_e = entry_take(pos_e, rem_e, pv.B[k + 1] - b0_e, pos_e == 1 ? v_hi : v_lo); \
        if (pos_e == 3) { \
            const int vis = row0 + nrows - b0_e; \
            n_e = vis < n_e ? (vis > 0 ? vis : 0) : n_e; \
        } \
    } \
    int total, nseg, start, slot; \
    block_excl_scan2(n_e, n_e > 0 ? 1 : 0, sm.s_wave, &start, &slot, &total, &nseg); \
    if (n_e > 0) { \
        sm.seg_start[slot] = start; \
        sm.seg_b0[slot] = b0_e; \
        sm.seg_pos[slot] = pos_e; \
        sm.seg_rem[slot] = rem_e; \
    } \
    for (int i_ = nseg + tid; i_ < kSegB + 80; i_ += 256) sm.seg_start[i_] = total; \
    int seg_cur = 0; \
    __syncthreads();

// one wave: packed position -> (row offsets, lo, hi) of tile n.  The tiles a wave prepares come in
// ascending order, so the segment of the tile's first key is found by moving the wave's cursor
// forward (64 segment starts per look); the starts that fall inside the tile then mark their
// position, and a key's segment is the first one plus the marks at or before the key.
#define DHSA_MAKE_META(n)                                                                       \
    {                                                                                           \
        const int buf_ = (n) & 7;                                                               \
        const int x0_ = (n) * kKT;                                                              \
        int s0_ = seg_cur;                                                                      \
        for (;;) {                                                                              \
            const int a_ = __popcll(__ballot(sm.seg_start[s0_ + 1 + lane] <= x0_));             \
            s0_ += a_;                                                                          \
            if (a_ < 64) break;                                                                 \
        }                                                                                       \
        seg_cur = s0_;                                                                          \
        const int p_ = sm.seg_start[s0_ + 1 + lane] - x0_;                                      \
        /* lanes talk through LDS without a block barrier: volatile keeps the three accesses  */ \
        /* in program order (the LDS executes one wave's operations in order)                 */ \
        volatile int *const mt_ = sm.meta_tmp[wave_u];                                          \
        mt_[lane] = 0;                                                                          \
        if (p_ > 0 && p_ < kKT) mt_[p_] = 1;                                                    \
        const unsigned long long marks_ = __ballot(mt_[lane] != 0);                             \
        int x_ = x0_ + lane;                                                                    \
        int seg_ = s0_ + __popcll(marks_ & ((2ull << lane) - 1ull));                            \
        const bool pad_ = x_ >= total;                                                          \
        if (pad_) { x_ = total - 1; seg_ = nseg - 1; }                                          \
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
#define DHSA_GLOAD(lds_base, offs, base8, piece_bytes, n, c0, c1)                               \
    {                                                                                           \
        const unsigned dst_ = lds_base + (((n) & 1) * kTile + wave_u * 512) * 2;                \
        _Pragma("unroll") for (int c = c0; c < c1; ++c)                                         \
            load16_to_lds(base8, offs[c] + piece_bytes, dst_ + c * 4096);                       \
    }
#define DHSA_LOAD_K_LO(n) DHSA_GLOAD(lds_K, ko_lo, Kg8, ld_piece_bytes_k, n, 0, KPT / 2)      /* keys 0..31  */
#define DHSA_LOAD_K_HI(n) DHSA_GLOAD(lds_K, ko_hi, Kg8, ld_piece_bytes_k, n, KPT / 2, KPT)    /* keys 32..63 */
#define DHSA_LOAD_V(n) DHSA_GLOAD(lds_V, vo, Vg8, ld_piece_bytes_v, n, 0, KPT)
#define DHSA_LOAD_V_LO(n) DHSA_GLOAD(lds_V, vo, Vg8, ld_piece_bytes_v, n, 0, KPT / 2)
#define DHSA_LOAD_V_HI(n) DHSA_GLOAD(lds_V, vo, Vg8, ld_piece_bytes_v, n, KPT / 2, KPT)


// Everything the tile bodies need beside the plan (kernel arguments, passed on by reference).
struct AttnArgs {
    const uint16_t *Q, *K, *V;
    uint16_t *O;
    int G;
    float scale_log2e;
    int64_t qs_h, qs_l, ks_h, ks_l, vs_h, vs_l, os_h, os_l;
};

// One row tile of more than 64 rows (any tile of up to 128 rows is handled correctly): see the
// header of this file.
template <int D>
__device__ __forceinline__ void attn_tile_32(AttnSmem<D> &sm, const PlanView &pv, const AttnArgs &a, const int h,
                                             const int tile) {
    using Smem = AttnSmem<D>;
    constexpr int OPR = D / 8;          // 16-byte pieces per row
    constexpr int KPT = OPR / 4;        // load instructions per wave per tile (K and V each)
    constexpr int NS = D / 16;          // MFMA k-steps of Q K^T
    constexpr int NDB = D / 32;         // 32-wide output column blocks
    constexpr int kTile = Smem::kTile;
    const uint16_t *__restrict__ Q = a.Q;
    const uint16_t *__restrict__ K = a.K;
    const uint16_t *__restrict__ V = a.V;
    uint16_t *__restrict__ O = a.O;
    const int G = a.G;
    const float scale_log2e = a.scale_log2e;
    const int64_t qs_h = a.qs_h, qs_l = a.qs_l, ks_h = a.ks_h, ks_l = a.ks_l, vs_h = a.vs_h, vs_l = a.vs_l,
                  os_h = a.os_h, os_l = a.os_l;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);   // wave-uniform copy
    const int lr = lane & 31, g2 = lane >> 5;

    const int g = h / G;
    const int l = pv.tiles[2 * tile], row0 = pv.tiles[2 * tile + 1];   // query group, first row
    const int b_l = pv.RB[l];
    const int rows_left = pv.RB[l + 1] - row0;
    const int nrows = rows_left < kRowTile ? rows_left : kRowTile;
    const int v_lo = row0 + 1 - b_l, v_hi = v_lo + nrows - 1;
    // Wave = one 32-row block of the tile (rotated per workgroup so that the waves left without
    // rows do not always sit on the same SIMD), every 32-key block of the key list.
    const int rb = (wave + (blockIdx.x >> 3)) & 3;
    constexpr int kbw = 0;
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
    const unsigned ld_piece_bytes_k = 16u * ((lane % OPR) ^ piece_swizzle(ld_row0, OPR));
    const unsigned ld_piece_bytes_v = ld_piece_bytes_k;
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
        DHSA_SEGMENT_TABLE(e0);
        const int ntiles = (total + kKT - 1) / kKT;
        if (ntiles == 0) continue;

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
        {
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
        }
#undef DHSA_QK
#undef DHSA_MASK
#undef DHSA_ROWMAX
#undef DHSA_EXP
#undef DHSA_PV
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

// ---------------------------------------------------------------------------
// Row tiles of at most 96 rows: 16-row MFMA blocks (v_mfma_f32_16x16x32_bf16).
//
// The tile's rows are cut into two row groups of 16 RW rows (RW = 1, 2, 3: tiles
// of at most 32, 64, 96 rows); a wave owns one row group and ONE of the two
// 32-key blocks of every 64-key tile ("key parity" kbw), so all four waves work
// whatever the tile's height, and the two waves of a row group merge their
// partial softmax states at the end.  A K or V fragment read from LDS serves the
// RW row blocks of the wave (at RW = 3 a third less LDS traffic per product
// than one 32-row block per wave).
//
// Lane l = 16 q + n of a wave.  S^T block = K (16 keys x 32 d) Q^T (32 d x 16
// rows): the lane holds, per row block r and key half kh, the scores of row n of
// the block against keys 16 kh + 4 q + {0..3} of the wave's key block -- 8 keys
// of ONE query row per row block, which after the exponential are exactly the B
// operand of O^T (16 d x 16 rows) += V^T (16 d x 32 keys) P^T (32 keys x 16
// rows) when the contraction index 8 q + i is read as key 4 q + i (i < 4) or
// 16 + 4 q + i - 4: the V^T operand is fetched in that key order with two
// transpose reads.  The four lanes of a row (same n) share the exponent
// reference; their row sums are added at the very end.
//
// K rows are swizzled by row & 15 here (16-byte column reads of 16 rows x 4
// pieces; the swizzle of the 32-row kernel would make two lanes of a bank group
// collide), V rows as in the kernel above.  Loads, key lists and the pipeline
// (scores of this wave's block of tile n + 1 on the matrix unit while the block
// of tile n is exponentiated) are those of the key-parity path above.
// ---------------------------------------------------------------------------
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int piece_swizzle_k16(int r, int pieces_per_row) {
    return pieces_per_row == 16 ? (r & 15) : piece_swizzle(r, pieces_per_row);
}

template <int D, int RW>
__device__ __forceinline__ void attn_tile_16(AttnSmem<D> &sm, const PlanView &pv, const AttnArgs &a, const int h,
                                             const int tile) {
    using Smem = AttnSmem<D>;
    constexpr int OPR = D / 8;          // 16-byte pieces per row
    constexpr int KPT = OPR / 4;        // load instructions per wave per tile (K and V each)
    constexpr int NT = D / 32;          // MFMA k-steps of K Q^T
    constexpr int NJ = D / 16;          // 16-wide blocks of the head dimension (rows of O^T)
    constexpr int kTile = Smem::kTile;
    const uint16_t *__restrict__ Q = a.Q;
    const uint16_t *__restrict__ K = a.K;
    const uint16_t *__restrict__ V = a.V;
    uint16_t *__restrict__ O = a.O;
    const int G = a.G;
    const float scale_log2e = a.scale_log2e;
    const int64_t qs_h = a.qs_h, qs_l = a.qs_l, ks_h = a.ks_h, ks_l = a.ks_l, vs_h = a.vs_h, vs_l = a.vs_l,
                  os_h = a.os_h, os_l = a.os_l;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int n16 = lane & 15, q = lane >> 4;

    const int g = h / G;
    const int l = pv.tiles[2 * tile], row0 = pv.tiles[2 * tile + 1];
    const int b_l = pv.RB[l];
    const int rows_left = pv.RB[l + 1] - row0;
    const int nrows = rows_left < 32 * RW ? rows_left : 32 * RW;   // only tiles of <= 32 RW rows come here
    const int v_lo = row0 + 1 - b_l, v_hi = v_lo + nrows - 1;
    const int rg = wave & 1, kbw = wave >> 1;        // row group, key parity
    const int rbase = rg * 16 * RW;
    const bool wave_live = rbase < nrows;

    const char *Kg8 = reinterpret_cast<const char *>(K + (int64_t)g * ks_h);
    const char *Vg8 = reinterpret_cast<const char *>(V + (int64_t)g * vs_h);
    const unsigned k_row_bytes = (unsigned)ks_l * 2u, v_row_bytes = (unsigned)vs_l * 2u;

    // Q fragments (B operand of K Q^T): row n of row block r, d = 32 t + 8 q .. + 7.  Padding rows
    // get q = 0 and, through a huge exponent reference, p = 0.
    bf16x8 qf[RW][NT];
    int v_i[RW];
    float m_ref[RW], l_run[RW];
    f32x4 oacc[RW][NJ];
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        const int rr = rbase + 16 * r + n16;
        const bool pad_row = rr >= nrows;
        v_i[r] = v_lo + rr;
        const uint16_t *qp = Q + (int64_t)h * qs_h + (int64_t)(row0 + (pad_row ? nrows - 1 : rr)) * qs_l + 8 * q;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            qf[r][t] = *reinterpret_cast<const bf16x8 *>(qp + 32 * t);
            if (pad_row) qf[r][t] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        }
        m_ref[r] = pad_row ? 1e30f : -INFINITY;
        l_run[r] = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j) oacc[r][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    const int E = pv.count[(int64_t)h * pv.N_q + l];
    const int32_t *ent = pv.entries + ((int64_t)h * pv.N_q + l) * pv.stride * 2;

    // staging (as in the kernel above; K with its own swizzle)
    constexpr int RPW = 64 / OPR;
    const int ld_row0 = wave * RPW + lane / OPR;
    const unsigned ld_piece_bytes_k = 16u * ((lane % OPR) ^ piece_swizzle_k16(ld_row0, OPR));
    const unsigned ld_piece_bytes_v = 16u * ((lane % OPR) ^ piece_swizzle(ld_row0, OPR));
    constexpr int RSTR = 4 * RPW;
    const int off_slot_wr = (lane % RSTR) * KPT + lane / RSTR;
    const int off_slot_rd = ld_row0 * KPT;
    const unsigned lds_K = (unsigned)(uintptr_t)(__attribute__((address_space(3))) uint16_t *)sm.K;
    const unsigned lds_V = (unsigned)(uintptr_t)(__attribute__((address_space(3))) uint16_t *)sm.V;
    // K fragment of k-step t: key row kbw 32 + 16 kh + n, logical piece 4 t + q (byte offsets; kh by immediate)
    int k_off[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
        k_off[t] = 2 * (kbw * 32 + n16) * D + 16 * ((4 * t + q) ^ piece_swizzle_k16(n16, OPR));
    // V^T fragment of head-dimension block j: the 16 lanes of group q read keys 4 q + rho (rho = n >> 2),
    // four lanes per key covering d = 16 j + 4 (n & 3) .. + 3; the transpose read hands lane n element
    // d = 16 j + n of the four keys
    int v_off[NJ];
    {
        const int key = 4 * q + (n16 >> 2), c = n16 & 3;
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            v_off[j] = 2 * (kbw * 32 + key) * D + 16 * ((2 * j + (c >> 1)) ^ piece_swizzle(key, OPR)) + 8 * (c & 1);
    }
    const char *const smK8 = reinterpret_cast<const char *>(sm.K);
    const char *const smV8 = reinterpret_cast<const char *>(sm.V);

    for (int e0 = 0; e0 < E; e0 += kSegB) {
        DHSA_SEGMENT_TABLE(e0);
        const int ntiles = (total + kKT - 1) / kKT;
        if (ntiles == 0) continue;

// S^T of this wave's 32-key block of the K buffer k_off points into, all row blocks
#define DHSA_QK16(sacc)                                                                         \
    {                                                                                           \
        _Pragma("unroll") for (int kh = 0; kh < 2; ++kh) {                                      \
            _Pragma("unroll") for (int r = 0; r < RW; ++r) sacc[r][kh] = f32x4{0.f, 0.f, 0.f, 0.f}; \
            _Pragma("unroll") for (int t = 0; t < NT; ++t) {                                    \
                const bf16x8 kf_ = *reinterpret_cast<const bf16x8 *>(smK8 + k_off[t] + kh * 32 * D); \
                _Pragma("unroll") for (int r = 0; r < RW; ++r)                                  \
                    sacc[r][kh] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf_, qf[r][t], sacc[r][kh], 0, 0, 0); \
            }                                                                                   \
        }                                                                                       \
    }

#define DHSA_MASK16(n, sacc, flag)                                                              \
    {                                                                                           \
        if (flag) {                                                                             \
            _Pragma("unroll") for (int kh = 0; kh < 2; ++kh) {                                  \
                const int key_ = kbw * 32 + kh * 16 + 4 * q;                                    \
                const int4 lo_ = *reinterpret_cast<const int4 *>(&sm.key_lo[(n) & 7][key_]);    \
                const int4 hi_ = *reinterpret_cast<const int4 *>(&sm.key_hi[(n) & 7][key_]);    \
                _Pragma("unroll") for (int r = 0; r < RW; ++r) {                                \
                    sacc[r][kh][0] = ((v_i[r] > lo_.x) & (v_i[r] < hi_.x)) ? sacc[r][kh][0] : -INFINITY; \
                    sacc[r][kh][1] = ((v_i[r] > lo_.y) & (v_i[r] < hi_.y)) ? sacc[r][kh][1] : -INFINITY; \
                    sacc[r][kh][2] = ((v_i[r] > lo_.z) & (v_i[r] < hi_.z)) ? sacc[r][kh][2] : -INFINITY; \
                    sacc[r][kh][3] = ((v_i[r] > lo_.w) & (v_i[r] < hi_.w)) ? sacc[r][kh][3] : -INFINITY; \
                }                                                                               \
            }                                                                                   \
        }                                                                                       \
    }

// maximum over the 32 keys of the block for this lane's row of row block r (four lanes per row)
#define DHSA_ROWMAX16(sa, mx)                                                                   \
    {                                                                                           \
        float m_ = fmaxf(fmaxf(sa[0][0], sa[0][1]), fmaxf(sa[0][2], sa[0][3]));                 \
        m_ = fmaxf(m_, fmaxf(fmaxf(sa[1][0], sa[1][1]), fmaxf(sa[1][2], sa[1][3])));            \
        m_ = fmaxf(m_, __shfl_xor(m_, 16));                                                     \
        mx = fmaxf(m_, __shfl_xor(m_, 32));                                                     \
    }

// P = exp2((S - m_ref) c) per row block, with the lazily moved exponent reference of the kernel above
#define DHSA_EXP16(sacc, pf)                                                                    \
    _Pragma("unroll") for (int r = 0; r < RW; ++r) {                                            \
        float mc_ = (m_ref[r] == -INFINITY) ? 0.f : m_ref[r] * scale_log2e;                     \
        float psum_ = 0.f;                                                                      \
        _Pragma("unroll") for (int x = 0; x < 8; ++x) {                                         \
            const float e_ = __builtin_amdgcn_exp2f(sacc[r][x >> 2][x & 3] * scale_log2e - mc_); \
            psum_ += e_;                                                                        \
            pf[r][x] = (__bf16)e_;                                                              \
        }                                                                                       \
        if (__any(!(psum_ < 1048576.f) || m_ref[r] == -INFINITY)) {                             \
            float mx_;                                                                          \
            DHSA_ROWMAX16(sacc[r], mx_);                                                        \
            const float m_new_ = fmaxf(m_ref[r], mx_);                                          \
            const float alpha_ = (m_ref[r] == -INFINITY) ? 0.f                                  \
                                 : __builtin_amdgcn_exp2f((m_ref[r] - m_new_) * scale_log2e);   \
            l_run[r] *= alpha_;                                                                 \
            _Pragma("unroll") for (int j = 0; j < NJ; ++j)                                      \
                _Pragma("unroll") for (int x = 0; x < 4; ++x) oacc[r][j][x] *= alpha_;          \
            m_ref[r] = m_new_;                                                                  \
            mc_ = (m_ref[r] == -INFINITY) ? 0.f : m_ref[r] * scale_log2e;                       \
            psum_ = 0.f;                                                                        \
            _Pragma("unroll") for (int x = 0; x < 8; ++x) {                                     \
                const float e_ = __builtin_amdgcn_exp2f(sacc[r][x >> 2][x & 3] * scale_log2e - mc_); \
                psum_ += e_;                                                                    \
                pf[r][x] = (__bf16)e_;                                                          \
            }                                                                                   \
        }                                                                                       \
        l_run[r] += psum_;                                                                      \
    }

// O^T += V^T P^T for this wave's 32-key block of the V buffer v_off points into
#define DHSA_PV16(pf)                                                                           \
    _Pragma("unroll") for (int j = 0; j < NJ; ++j) {                                            \
        union { s16x4 h[2]; bf16x8 v; } vf_;                                                    \
        _Pragma("unroll") for (int kh = 0; kh < 2; ++kh)                                        \
            vf_.h[kh] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(                                \
                (s16x4 __attribute__((address_space(3))) *)(smV8 + v_off[j] + kh * 32 * D));    \
        _Pragma("unroll") for (int r = 0; r < RW; ++r)                                          \
            oacc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf_.v, pf[r], oacc[r][j], 0, 0, 0); \
    }

        f32x4 s_a[RW][2], s_b[RW][2];
        int toggle = 2 * kTile;
        unsigned ko_lo[KPT], ko_hi[KPT], vo[KPT];
        if (wave < ntiles) DHSA_MAKE_META(wave);
        __syncthreads();
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
        __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0)
        __syncthreads();
        if (wave_live) {
            DHSA_QK16(s_a);
            DHSA_MASK16(0, s_a, fl_0);
            if (e0 == 0) {   // reference = row maxima of this wave's first block
#pragma unroll
                for (int r = 0; r < RW; ++r) { float mx0; DHSA_ROWMAX16(s_a[r], mx0); m_ref[r] = fmaxf(m_ref[r], mx0); }
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) k_off[t] += 2 * kTile;   // K offsets run one tile ahead of V offsets
        }
        __syncthreads();                      // K(0) may be overwritten from here on

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
                bf16x8 pf[RW];
                DHSA_QK16(s_b);
                DHSA_EXP16(s_a, pf);
                DHSA_PV16(pf);
                DHSA_MASK16(n + 1, s_b, fl_next);
#pragma unroll
                for (int r = 0; r < RW; ++r) { s_a[r][0] = s_b[r][0]; s_a[r][1] = s_b[r][1]; }
#pragma unroll
                for (int t = 0; t < NT; ++t) k_off[t] -= toggle;
#pragma unroll
                for (int j = 0; j < NJ; ++j) v_off[j] += toggle;
                toggle = -toggle;
            }
            __builtin_amdgcn_s_waitcnt(0x0f70);
            __syncthreads();
        }
        if (wave_live) {                          // last tile of the batch
            bf16x8 pf[RW];
            DHSA_EXP16(s_a, pf);
            DHSA_PV16(pf);
        }
        __syncthreads();                          // LDS is reused by the next batch / the merge
        if (wave_live) {                          // leave the offsets at buffer 0 for the next batch
            if (ntiles & 1) {
#pragma unroll
                for (int t = 0; t < NT; ++t) k_off[t] -= 2 * kTile;
            } else {
#pragma unroll
                for (int j = 0; j < NJ; ++j) v_off[j] -= 2 * kTile;
            }
        }
#undef DHSA_QK16
#undef DHSA_MASK16
#undef DHSA_ROWMAX16
#undef DHSA_EXP16
#undef DHSA_PV16
    }

    // ---- fold the state of the wave that took the odd key blocks into its partner ----
    {
        constexpr int SLOTS = RW * (2 + 4 * NJ);
        // the exchange area starts at K and runs on into V, which follows it in AttnSmem; both are dead here
        static_assert(offsetof(Smem, V) == sizeof(sm.K) && 2 * SLOTS * 64 * sizeof(float) <= sizeof(sm.K) + sizeof(sm.V),
                      "merge scratch must fit K + V");
        float *xch = reinterpret_cast<float *>(sm.K) + rg * SLOTS * 64 + lane;   // [slot][lane]
        if (wave_live && kbw == 1) {
#pragma unroll
            for (int r = 0; r < RW; ++r) {
                xch[(r * (2 + 4 * NJ)) * 64] = m_ref[r];
                xch[(r * (2 + 4 * NJ) + 1) * 64] = l_run[r];
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int x = 0; x < 4; ++x) xch[(r * (2 + 4 * NJ) + 2 + 4 * j + x) * 64] = oacc[r][j][x];
            }
        }
        __syncthreads();
        if (wave_live && kbw == 0) {
#pragma unroll
            for (int r = 0; r < RW; ++r) {
                const float m1 = xch[(r * (2 + 4 * NJ)) * 64], l1 = xch[(r * (2 + 4 * NJ) + 1) * 64];
                const float mm = fmaxf(m_ref[r], m1);
                const float a0 = (m_ref[r] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((m_ref[r] - mm) * scale_log2e);
                const float a1 = (m1 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((m1 - mm) * scale_log2e);
                l_run[r] = l_run[r] * a0 + l1 * a1;
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int x = 0; x < 4; ++x)
                        oacc[r][j][x] = oacc[r][j][x] * a0 + xch[(r * (2 + 4 * NJ) + 2 + 4 * j + x) * 64] * a1;
            }
        }
    }

    // ---- epilogue: normalise, round to bf16, store (lane: row n of each row block, d = 16 j + 4 q .. + 3) ----
    if (wave_live && kbw == 0) {
#pragma unroll
        for (int r = 0; r < RW; ++r) {
            float l_tot = l_run[r] + __shfl_xor(l_run[r], 16);
            l_tot += __shfl_xor(l_tot, 32);
            const int rr = rbase + 16 * r + n16;
            if (rr < nrows) {
                const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;   // no visible key (row-block form): zeros
                uint16_t *op = O + (int64_t)h * os_h + (int64_t)(row0 + rr) * os_l + 4 * q;
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    union { __bf16 b[4]; uint2 u; } pk;
#pragma unroll
                    for (int x = 0; x < 4; ++x) pk.b[x] = (__bf16)(oacc[r][j][x] * inv);
                    *reinterpret_cast<uint2 *>(op + 16 * j) = pk.u;
                }
            }
        }
    }
}

// One launch per tile class (a kernel that holds all three bodies measured 3-10 % slower than
// the sum of these).  CLS 0: tiles of more than 64 rows (table classes 0 and 1), 1: 33..64 rows,
// 2: at most 32 rows.  Inside a launch tiles are issued from the end of the sequence (most keys)
// to its start, so that the launch ends with the cheapest workgroups.
template <int D, int CLS>
__global__ __launch_bounds__(256, 2) void k_attn_mfma(PlanView pv, AttnArgs a, int H_q, int mode, int tile0, int T) {
    __shared__ AttnSmem<D> sm;
    if (!plan_matches(pv)) return;   // not this problem's plan: nothing is read further, O is not written
    int h, pos;
    decode_block(mode, blockIdx.x, H_q, a.G, T, &h, &pos);
    const int tile = tile0 + T - 1 - pos;
    if constexpr (CLS == 0) attn_tile_32<D>(sm, pv, a, h, tile);
    else if constexpr (CLS == 1) attn_tile_16<D, 2>(sm, pv, a, h, tile);
    else attn_tile_16<D, 1>(sm, pv, a, h, tile);
}

hipError_t launch_attn_mfma(const Prob &p, const PlanView &pv, const void *Q, const void *K, const void *V,
                            void *O, hipStream_t s, hipEvent_t *ev) {
    // kv-heads in flight: one per XCD (most workgroups walking the same K / V per L2).  Row blocks of
    // full tile height whose K and V of eight heads exceed the 256 MB memory-side cache while those of
    // four fit: four in flight, each on two XCDs -- the L2s then miss more often (53 % hits instead of
    // 56 % on c3) but mostly into that cache, and the step measures 4-5 % faster; the row form on the
    // dynamic chunks, which is bound by what crosses the fabric, gains nothing from it (0-1 %) and asks
    // the fabric for 30 % more, so it keeps eight.  Two or one in flight are slower in both forms.
    const double kv_head_bytes = 2.0 * (double)p.L * (double)(p.ks_l + p.vs_l);
    const int want = (p.B_r >= kRowTile && 8 * kv_head_bytes > 288e6 && 4 * kv_head_bytes <= 288e6) ? 4 : 8;
    AttnArgs a;
    a.Q = (const uint16_t *)Q; a.K = (const uint16_t *)K; a.V = (const uint16_t *)V; a.O = (uint16_t *)O;
    a.G = p.G;
    a.scale_log2e = p.scale * 1.4426950408889634f;
    a.qs_h = p.qs_h; a.qs_l = p.qs_l; a.ks_h = p.ks_h; a.ks_l = p.ks_l;
    a.vs_h = p.vs_h; a.vs_l = p.vs_l; a.os_h = p.os_h; a.os_l = p.os_l;
#define DHSA_LAUNCH(CLS, tile0, T)                                                                           \
    if ((T) > 0) {                                                                                          \
        const int mode = attn_order(want, p.H_kv, p.G, T);                                                  \
        if (p.D == 64)                                                                                      \
            hipLaunchKernelGGL((k_attn_mfma<64, CLS>), dim3(p.H_q * (T)), dim3(256), 0, s, pv, a, p.H_q, mode, tile0, T);  \
        else                                                                                                \
            hipLaunchKernelGGL((k_attn_mfma<128, CLS>), dim3(p.H_q * (T)), dim3(256), 0, s, pv, a, p.H_q, mode, tile0, T); \
    }
    // tallest tiles first (they take longest)
    DHSA_LAUNCH(0, 0, pv.T_big)
    if (ev && hipEventRecord(ev[0], s) != hipSuccess) return hipErrorUnknown;
    DHSA_LAUNCH(1, pv.T_big, pv.T_cls[2])
    if (ev && hipEventRecord(ev[1], s) != hipSuccess) return hipErrorUnknown;
    DHSA_LAUNCH(2, pv.T_big + pv.T_cls[2], pv.T_cls[3])
    if (ev && hipEventRecord(ev[2], s) != hipSuccess) return hipErrorUnknown;
#undef DHSA_LAUNCH
    return hipGetLastError();
}

#undef DHSA_SEGMENT_TABLE
#undef DHSA_MAKE_META
#undef DHSA_OFFS
#undef DHSA_GLOAD
#undef DHSA_LOAD_K_LO
#undef DHSA_LOAD_K_HI
#undef DHSA_LOAD_V
#undef DHSA_LOAD_V_LO
#undef DHSA_LOAD_V_HI

}  // namespace dhsa
