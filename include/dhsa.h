/*
 * libdhsa -- the prefill hot path of Dynamic Hierarchical Sparse Attention
 * (arXiv 2510.24606) for AMD MI355X (gfx950).  C ABI: plain pointers and sizes.
 *
 * One attention layer, batch 1 (a batch is a caller-side loop, as in the
 * paper's Sec. 4 "batch handling").  Per query head h (GQA: kv-head g = h / G,
 * G = H_q / H_kv) the path is
 *   1. pool Q and K over the variable-length chunks given by the boundaries B
 *      (Sec. 3.3, Eq. 4: x_C = sqrt(len)/len * sum of the chunk's vectors);
 *   2. chunk similarity S_c = Q_c K_c^T, unscaled (Sec. 3.3);
 *   3. rank the key chunks of every query chunk by S_c, larger first, equal
 *      scores by lower chunk id (Sec. 3.1 Step 2; Alg. 1 "Argsort");
 *   4. per query ROW i take tokens in ranked order, clipped to keys j <= i,
 *      until exactly min(N_b, i+1) are taken; the last chunk taken keeps its
 *      lowest indices (Alg. 1 walk/append/truncate with q_max = i + 1);
 *   5. softmax(q_i . k_j * scale) over the selected keys only, times V
 *      (Alg. 2 / Alg. 3; App. C "Backend implementations").
 * Steps 1-4 are dhsa_route (result: a compact routing plan), step 5 is
 * dhsa_sparse_prefill, dhsa_prefill runs both on one stream.
 * Beside the path: dhsa_finalize_boundaries (boundary scores -> B, Sec. 3.2),
 * dhsa_recall_rows (recall of the routed sets against exact top-k attention),
 * dhsa_decode_step (the newest token's row alone, over cached K / V), and the
 * inspection hooks dhsa_plan_expand_rows, dhsa_debug_routing, dhsa_mfma_probe.
 *
 * With B_r > 0 in the problem struct the same entry points run Alg. 1 as it is
 * printed (App. C) instead of the per-row form above: queries are grouped in
 * fixed row blocks of B_r rows, q_i = sqrt(B_r) * AvgPool(Q_i) (mean over the
 * rows the block has), S_c is N_r x N_c with N_r = ceil(L / B_r), every key
 * chunk is ranked, ONE index list per row block is built with q_max = the
 * block's end (at most N_b tokens, the last chunk taken truncated to its lowest
 * indices), and attention applies the causal mask per token (Alg. 2 / Alg. 3:
 * row u of block i attends the listed keys j <= i B_r + u).  A row that sees
 * none of its block's keys gets O = 0.
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses, "host" pointers host addresses.
 *   - Q is [H_q, L, D], K and V are [H_kv, L, D], O is [H_q, L, D]; D contiguous;
 *     element strides between heads and rows are in the problem struct (0 means
 *     packed).  Row starts must be 16-byte aligned.
 *   - B is a HOST array of N_c+1 int32 with B[0] = 0 < B[1] < ... < B[N_c] = L;
 *     chunk k holds tokens [B[k], B[k+1]).  It is validated on the host before
 *     any device work and travels into the plan as kernel arguments (no copy from
 *     host memory, which could make the call wait).
 *   - The caller owns every buffer (plan and workspace included, sized by the
 *     *_bytes calls, 256-byte aligned).  The library allocates nothing, keeps
 *     no state between calls, and never synchronises: work is enqueued on
 *     `stream` (a hipStream_t passed as void*; NULL = the default stream) and
 *     results are valid once the caller has synchronised that stream.  (Two
 *     calls beside the path do wait for the stream and say so below:
 *     dhsa_plan_expand_rows, which reads the plan header back, and
 *     dhsa_mfma_probe, which times a kernel.)
 *   - Every entry point returns a dhsa_status; arguments are validated before
 *     the first device call and on error nothing is written or launched.
 *   - Inputs must be finite; N_b > L behaves as N_b = L.
 *   - Limits: D in {64, 128}; 1 <= N_c <= 8192; L < 2^31; for DHSA_BF16 one K or V
 *     head must span at most 4 GiB (L * row stride * 2 bytes); with B_r > 0 at
 *     most 2^20 row blocks.
 *   - Routing arithmetic (pooling, S_c, ranking) is fp64 so that the chosen
 *     index sets do not depend on summation order beyond ~1e-13 score gaps.
 *     Attention: DHSA_BF16 uses bf16 MFMA with fp32 softmax and accumulators
 *     (probabilities are rounded to bf16 before the PV product); DHSA_F32 uses
 *     fp32 arithmetic throughout.  O has the input dtype.
 */
#ifndef DHSA_H
#define DHSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DHSA_OK = 0,
    DHSA_ERR_NULL = 1,        /* a required pointer is NULL                               */
    DHSA_ERR_SHAPE = 2,       /* L, H_q, H_kv, D, N_c or a stride out of the stated range */
    DHSA_ERR_BOUNDARIES = 3,  /* B not strictly increasing from 0 to L                    */
    DHSA_ERR_BUDGET = 4,      /* N_b < 1                                                  */
    DHSA_ERR_DTYPE = 5,       /* dtype not DHSA_F32 / DHSA_BF16                           */
    DHSA_ERR_WORKSPACE = 6,   /* plan or workspace smaller than *_bytes() says            */
    DHSA_ERR_HIP = 7,         /* a HIP runtime call or launch failed                      */
    DHSA_ERR_PLAN = 8,        /* the plan does not belong to this problem                 */
    DHSA_ERR_ALIGN = 9        /* a pointer or stride breaks the 16-byte row alignment     */
} dhsa_status;

typedef enum { DHSA_F32 = 0, DHSA_BF16 = 1 } dhsa_dtype;

/* Chunk representation.  DHSA_POOL_ROBUST: Sec. 3.3 Eq. 4, sqrt(len)/len * sum (and
 * sqrt(B_r) * AvgPool for the row blocks of Alg. 1).  DHSA_POOL_MEAN: plain average,
 * the ablation "without robust chunk representation" (App. D); with fixed-size
 * chunks on top (uniform boundaries) the method is conventional block-sparse
 * attention, as that appendix notes. */
typedef enum { DHSA_POOL_ROBUST = 0, DHSA_POOL_MEAN = 1 } dhsa_pooling;

/* Problem statement of Sec. 3.1 / Alg. 1-3: sequence length L, chunk count N_c
 * (boundaries passed separately), per-row token budget N_b, GQA head counts. */
typedef struct {
    int64_t L;
    int32_t H_q, H_kv, D;
    int32_t N_c;
    int32_t N_b;
    int32_t dtype;            /* dhsa_dtype of Q, K, V and O                       */
    float scale;              /* softmax scale of step 5; 0 means 1/sqrt(D)        */
    int64_t q_stride_h, q_stride_l;   /* in elements; 0 = packed [H, L, D]         */
    int64_t k_stride_h, k_stride_l;
    int64_t v_stride_h, v_stride_l;
    int64_t o_stride_h, o_stride_l;
    int32_t B_r;              /* 0: per-row budgets on the dynamic chunks (steps 1-5 above);
                                 > 0: Alg. 1 as printed with row blocks of B_r rows        */
    int32_t pooling;          /* dhsa_pooling: how chunks (and row blocks) are represented  */
} dhsa_problem;

/*
 * Layout of the routing plan (device memory, int32 words, little endian).  It
 * is the sparsity mask M of Sec. 3.1 in compact form: all rows of query chunk l
 * share one ranking and differ only in v = i + 1 - B[l], the visible part of
 * their own chunk.
 *   words [0, 32)            header: magic 'DHSA', version, H_q, N_c, N_b (clamped to L),
 *                            stride, L, T1 (row tiles per head), off_B, off_count,
 *                            off_entries, off_tiles (word offsets), T_big, off_RB, N_q, B_r,
 *                            pooling, checksum of B (32-bit FNV-1a over its N_c + 1 words),
 *                            H_kv, D, tiles of more than 96 / 65..96 / 33..64 / at most 32
 *                            rows (4 words), 8 words zero
 *   off_B      int32[N_c+1]  the boundaries of the key chunks
 *   off_RB     int32[N_q+1]  the boundaries of the query groups: the same array as
 *                            off_B (N_q = N_c) when B_r = 0; else RB[i] = min(i B_r, L),
 *                            N_q = ceil(L / B_r).  Below, "chunk l" on the query side
 *                            means query group l and v = i + 1 - RB[l].
 *   off_count  int32[H_q][N_c]          number of entries of (h, l)
 *   off_entries int32[H_q][N_c][stride][2]   entries, ascending chunk id:
 *        word 0: key chunk id k | (pos << 28), pos = 0 ranked before chunk l,
 *                1 = chunk l itself, 2 ranked after chunk l, 3 = row-block form
 *        word 1: rem = N_b - (tokens of other chunks taken before chunk k); for
 *                pos = 3 the number of tokens of chunk k in the block's list
 *      Row i of chunk l takes from entry (k, pos, rem) the tokens B[k] + t with
 *        t < min(len_k, rem)            if pos = 0
 *        t < min(v, rem)                if pos = 1
 *        t < min(len_k, rem - v)        if pos = 2
 *        t < rem and B[k] + t <= i      if pos = 3 (the block's list, causal mask per token)
 *      Only chunks some row of l takes a token from are listed.
 *   off_tiles  int32[T1][2]  row tiles of one head: (chunk l, first row), rows
 *                            [row, min(row + 128, B[l+1])), listed by height: tiles of
 *                            more than 96 rows, then 65..96, 33..64, at most 32 rows
 *                            (the first T_big have more than 64), each class by row
 */
#define DHSA_PLAN_MAGIC 0x41534844
#define DHSA_PLAN_VERSION 3
#define DHSA_PLAN_HEADER_WORDS 32
#define DHSA_ROW_TILE 128

/* Device bytes the plan / the routing workspace need.  0 on invalid arguments. */
size_t dhsa_plan_bytes(const dhsa_problem *prob, const int32_t *B_host);
size_t dhsa_workspace_bytes(const dhsa_problem *prob, const int32_t *B_host);

/* Steps 1-4 (Sec. 3.1, 3.3; Alg. 1): Q_dev, K_dev -> plan_dev.  ws_dev is
 * scratch (pooled vectors and S_c); its contents after the call are readable
 * through the dhsa_debug_* hooks until the next call that uses it. */
dhsa_status dhsa_route(const dhsa_problem *prob, const void *Q_dev, const void *K_dev,
                       const int32_t *B_host, void *plan_dev, size_t plan_bytes, void *ws_dev,
                       size_t ws_bytes, void *stream);

/* Step 5 (Alg. 2 / Alg. 3): exact softmax attention over the keys the plan
 * selects, O_dev[h, i, :] for every row.  The plan must come from dhsa_route on
 * the same problem and boundaries (it may be reused across calls, as the paper
 * caches routing results).  On the host only the plan's size can be checked
 * (DHSA_ERR_PLAN if too small) since the call never waits for the device; the
 * kernels compare the plan's header -- H_q, N_c, N_b, L, B_r, pooling, a checksum
 * of B -- with the problem and, if they differ, leave without reading further or
 * writing O.  dhsa_plan_check reports such a mismatch to the host. */
dhsa_status dhsa_sparse_prefill(const dhsa_problem *prob, const void *Q_dev, const void *K_dev,
                                const void *V_dev, const int32_t *B_host, const void *plan_dev,
                                size_t plan_bytes, void *O_dev, void *stream);

/* Does plan_dev belong to this problem and these boundaries?  Reads the plan's
 * header back (so it WAITS for `stream`) and compares it with what dhsa_route
 * would write: DHSA_OK, or DHSA_ERR_PLAN.  For callers that keep plans across
 * calls (Sec. 3.4 caches routing results) and want the check on the host. */
dhsa_status dhsa_plan_check(const dhsa_problem *prob, const int32_t *B_host, const void *plan_dev,
                            size_t plan_bytes, void *stream);

/* Steps 1-5 on one stream (Sec. 3.4 "Workflow"). */
dhsa_status dhsa_prefill(const dhsa_problem *prob, const void *Q_dev, const void *K_dev, const void *V_dev,
                         const int32_t *B_host, void *O_dev, void *plan_dev, size_t plan_bytes,
                         void *ws_dev, size_t ws_bytes, void *stream);

/* For callers that cannot allocate device memory -- code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc: dhsa_prefill without a
 * workspace argument.  The routing scratch (pooled vectors and S_c) lives in a
 * static device array of DHSA_STATIC_SCRATCH_BYTES inside the library (one copy
 * per GPU the library runs on, held until the process ends), and the boundaries
 * reach the device as kernel arguments instead of a copy from host memory, so
 * the call issues kernel launches only: no hipMalloc / hipFree, no copy.
 * Everything else is dhsa_prefill: same arguments, same kernels, same results
 * (plan_dev and O_dev are the caller's).  A problem whose
 * dhsa_workspace_bytes() exceeds dhsa_static_scratch_bytes() is rejected with
 * DHSA_ERR_WORKSPACE before anything is launched (64 MiB holds e.g. L = 32768
 * with 32 query heads and ~410 chunks).  All calls on one GPU share that GPU's
 * array: calls that may overlap on one GPU (different streams, different host
 * threads) race on it and must be ordered by the caller; the array keeps the
 * last call's contents and nothing in it has to start at zero. */
#define DHSA_STATIC_SCRATCH_BYTES (64u << 20)
dhsa_status dhsa_prefill_static(const dhsa_problem *prob, const void *Q_dev, const void *K_dev,
                                const void *V_dev, const int32_t *B_host, void *O_dev, void *plan_dev,
                                size_t plan_bytes, void *stream);
size_t dhsa_static_scratch_bytes(void);

/* The step just before the path: boundary scores -> chunk boundaries (Sec. 3.2
 * "Inference Pipeline"; App. "Inference of the Boundary Predictor").
 * scores_dev[i], i in [0, L), is the predictor's score that position i marks the
 * END of a chunk (fp32, device; the predictor network itself is not part of this
 * library).  Positions whose score does not exceed `threshold` are dropped; the
 * others are visited by descending score (equal scores: lower position first); a
 * visited position that has not been removed becomes a chunk end and removes
 * every other candidate within `window` tokens of it (0 < |j - i| <= window).
 * Output, in the half-open convention of the rest of the ABI:
 * B_dev = {0} u {i + 1 : i kept} u {L}, ascending, no repeats (the sequence end is
 * always a chunk end), N_c + 1 int32 entries, capacity L + 1; *N_c_dev = N_c.
 * Both are DEVICE memory: copy them to the host after synchronising `stream`
 * (the other entry points take B as a host array; boundaries are made once per
 * prompt).  ws_dev: device scratch of dhsa_finalize_boundaries_workspace_bytes(L)
 * bytes.  Asynchronous like the path itself.  A NaN score never exceeds the
 * threshold.  Errors: NULL pointers, L outside [1, 2^31), window < 0 or a NaN
 * threshold (DHSA_ERR_SHAPE), workspace too small. */
dhsa_status dhsa_finalize_boundaries(const float *scores_dev, int64_t L, float threshold, int32_t window,
                                     int32_t *B_dev, int32_t *N_c_dev, void *ws_dev, size_t ws_bytes,
                                     void *stream);
size_t dhsa_finalize_boundaries_workspace_bytes(int64_t L);

/* ---- inspection hooks (tests, stage-wise parity) ---- */

/* Expand the plan into explicit index sets I_{h,i} (Alg. 1's output) for one
 * head and a HOST list of rows: idx_dev[n_rows][cap] ascending, padded with -1,
 * cnt_dev[n_rows]; cap >= min(N_b, L).  With B_r > 0 a row gets the list of its
 * row block as Alg. 1 returns it (not yet masked causally).  The call reads the
 * plan header back to check it against `prob`, so it waits for `stream`.  rows are copied to rows_dev_scratch
 * (device, n_rows int64) by the call. */
dhsa_status dhsa_plan_expand_rows(const dhsa_problem *prob, const void *plan_dev, size_t plan_bytes,
                                  int32_t head, const int64_t *rows_host, int32_t n_rows,
                                  int64_t *rows_dev_scratch, int32_t *idx_dev, int32_t cap,
                                  int32_t *cnt_dev, void *stream);

/* Copy the pooled vectors (fp64, Qc_dev [H_q][N_q][D], Kc_dev [H_kv][N_c][D])
 * and/or S_c (fp64, Sc_dev [H_q][N_q][N_c]; entries of chunks no row of the
 * query group can see are not written) out of a workspace dhsa_route has
 * filled.  N_q = N_c, or ceil(L / B_r) when B_r > 0.  NULL skips. */
dhsa_status dhsa_debug_routing(const dhsa_problem *prob, const int32_t *B_host, const void *ws_dev,
                               size_t ws_bytes, double *Qc_dev, double *Kc_dev, double *Sc_dev, void *stream);

/* S_c alone (Sec. 3.3), fp64 [H_q][N_q][N_c], out of a workspace dhsa_route has
 * filled: dhsa_debug_routing with only the scores asked for. */
dhsa_status dhsa_debug_scores(const dhsa_problem *prob, const int32_t *B_host, const void *ws_dev,
                              size_t ws_bytes, double *Sc_dev, void *stream);

/* Measurement aid (not a step of the method): dhsa_prefill run once with events
 * between its kernels.  ms_host[0..7] (HOST floats) receive the milliseconds of:
 * 0 boundaries + plan set-up, 1 chunk pooling (Eq. 4), 2 S_c, 3 ranking + budget
 * (Alg. 1), 4 / 5 / 6 attention (Alg. 3) over the row tiles of more than 64 rows /
 * of 33..64 rows / of at most 32 rows (fp32 inputs: all rows in slot 4), 7 the
 * whole call.  Creates and destroys events and BLOCKS until the work is done;
 * arguments and results otherwise as dhsa_prefill. */
dhsa_status dhsa_prefill_stage_times(const dhsa_problem *prob, const void *Q_dev, const void *K_dev,
                                     const void *V_dev, const int32_t *B_host, void *O_dev, void *plan_dev,
                                     size_t plan_bytes, void *ws_dev, size_t ws_bytes, float *ms_host,
                                     void *stream);

/* Measurement aid (not a step of the method): the sustained rate of the bf16
 * matrix instruction the attention kernel (Alg. 3's QK^T and PV products) is
 * built on, alone in a loop on every CU, for `iters` x 16 instructions per
 * wave.  random_operands = 0: operands never change (the chip reaches its
 * published rate); 1: eight rotating sets of random operands (the chip lowers
 * its clock to stay inside its power limit, as it does under real attention
 * data).  scratch_dev: device memory of at least dhsa_mfma_probe_scratch_bytes()
 * bytes, contents overwritten.  Results go to HOST doubles: TFLOP/s over the
 * whole chip and (may be NULL) the average shader clock of one wave in MHz.
 * Unlike the other entry points this one BLOCKS until the kernel has run (it
 * times it with two events on `stream`).  iters in [1, 2^22]. */
dhsa_status dhsa_mfma_probe(int random_operands, int iters, void *scratch_dev, size_t scratch_bytes,
                            double *tflops_host, double *shader_mhz_host, void *stream);
size_t dhsa_mfma_probe_scratch_bytes(void);

/* Quality diagnostic (App. "Theoretical Analysis", Setup and Notation; the
 * quantity behind "Overlap with Top-K Attention" in Sec. 4): per-row recall of
 * the routed key sets of one head against exact top-k attention.  For every row
 * i of the HOST list: I*_i = the k = min(N_b, i + 1) keys j <= i with the largest
 * logits q_i . k_j (fp64, summed over d in ascending order; equal logits: lower
 * index), I_hat_i = the keys the plan gives row i (row-block form: the keys of
 * its block's list at or below the row).  hits_dev[t] = |I* n I_hat|,
 * size_dev[t] = |I*| (device int32[n_rows]); recall = hits / size.
 * plan_dev must come from dhsa_route on the same problem and boundaries.
 * rows_dev_scratch: device int64[n_rows]; ws_dev: device scratch of
 * dhsa_recall_workspace_bytes(prob, n_rows) bytes (8 L per row).  Asynchronous;
 * cost O(L D) per row -- a diagnostic for sampled rows, not a step of the path. */
dhsa_status dhsa_recall_rows(const dhsa_problem *prob, const void *Q_dev, const void *K_dev,
                             const int32_t *B_host, const void *plan_dev, size_t plan_bytes, int32_t head,
                             const int64_t *rows_host, int32_t n_rows, int64_t *rows_dev_scratch,
                             void *ws_dev, size_t ws_bytes, int32_t *hits_dev, int32_t *size_dev,
                             void *stream);
size_t dhsa_recall_workspace_bytes(const dhsa_problem *prob, int32_t n_rows);

/* One decoding step (Sec. 3.4, the remark on decoding: the same sparse attention
 * applied to a newly generated token by restricting the keys it attends).  The
 * paper gives the step no algorithm of its own; the reading taken here is that
 * the newest token is row L - 1 of the sequence and gets exactly what the prefill
 * path gives that row: its query group -- the open chunk [B[N_c-1], L), or with
 * B_r > 0 the open row block -- is pooled (Eq. 4; the row block as in Alg. 1),
 * scored against all N_c key chunks, ranked and walked with the budget N_b
 * (Alg. 1), and the row attends to the min(N_b, L) selected keys (Alg. 2).
 *
 * prob / B_host describe the sequence INCLUDING the newest token (L tokens,
 * N_c chunks; how a new token extends the boundaries -- joins the open chunk or
 * starts a chunk -- is the caller's boundary rule).  Q_dev, K_dev, V_dev are
 * addressed with the problem's strides like in dhsa_prefill; of Q only the rows
 * of the open query group are read (rows below it may be unset), K and V are
 * the caches, rows [0, L).  o_stride_* are not used: the output is
 *   O_row_dev  [H_q][D], contiguous, input dtype;
 * optional (either may be NULL):
 *   idx_dev    int32 [H_q][min(N_b, L)]: the selected key positions, ascending;
 *   cnt_dev    int32 [H_q]: their number.
 * Workspace: ws_dev of dhsa_decode_workspace_bytes(prob, N_c_cap, L_cap) bytes,
 * 16-byte aligned, whose layout depends only on the caps (and on H_q, H_kv, D,
 * N_b), so one allocation serves a whole generation with N_c <= N_c_cap <= 8192
 * and L <= L_cap.  It keeps the pooled keys between calls: kc_valid says that
 * the pooled keys of chunks [0, kc_valid) are already in ws_dev from earlier
 * calls with the same caps, the same K rows and the same boundaries B[0..kc_valid];
 * they are not read again.  0 <= kc_valid <= N_c - 1 (the open chunk is always
 * pooled anew); pass 0 on the first call.  Asynchronous on `stream`; calls that
 * share a workspace must be ordered.  Errors as for dhsa_prefill; caps below
 * the problem's sizes or kc_valid out of range: DHSA_ERR_SHAPE. */
dhsa_status dhsa_decode_step(const dhsa_problem *prob, const void *Q_dev, const void *K_dev, const void *V_dev,
                             const int32_t *B_host, int32_t N_c_cap, int64_t L_cap, int32_t kc_valid,
                             void *O_row_dev, int32_t *idx_dev, int32_t *cnt_dev, void *ws_dev, size_t ws_bytes,
                             void *stream);
/* 0 if the problem's scalar fields or the caps are out of range. */
size_t dhsa_decode_workspace_bytes(const dhsa_problem *prob, int32_t N_c_cap, int64_t L_cap);

const char *dhsa_status_string(dhsa_status s);
int dhsa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DHSA_H */
