// Host side of libdhsa: argument validation, plan/workspace layout, launches.
// See include/dhsa.h for the contract of every entry point.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <vector>

#include "dhsa_internal.h"

using namespace dhsa;

namespace {

int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// Validate the problem and the boundaries (host only, no device call).
dhsa_status resolve(const dhsa_problem *in, const int32_t *B, Prob *p) {
    if (!in || !B) return DHSA_ERR_NULL;
    if (in->dtype != DHSA_F32 && in->dtype != DHSA_BF16) return DHSA_ERR_DTYPE;
    if (in->L < 1 || in->L >= (int64_t)1 << 31) return DHSA_ERR_SHAPE;
    if (in->H_q < 1 || in->H_kv < 1 || in->H_q % in->H_kv != 0 || in->H_q > 65535 - in->H_kv) return DHSA_ERR_SHAPE;
    if (in->D != 64 && in->D != 128) return DHSA_ERR_SHAPE;
    if (in->N_c < 1 || in->N_c > kMaxChunks || in->N_c > in->L) return DHSA_ERR_SHAPE;
    if (in->N_b < 1) return DHSA_ERR_BUDGET;
    if (in->B_r < 0) return DHSA_ERR_SHAPE;
    if (in->pooling != DHSA_POOL_ROBUST && in->pooling != DHSA_POOL_MEAN) return DHSA_ERR_SHAPE;
    // row-block form: N_r = ceil(L / B_r) query groups, one workgroup each in the ranking kernel
    if (in->B_r > 0 && (in->L + in->B_r - 1) / in->B_r > (int64_t)1 << 20) return DHSA_ERR_SHAPE;
    if (!(in->scale >= 0.f) || !isfinite(in->scale)) return DHSA_ERR_SHAPE;
    if (B[0] != 0 || (int64_t)B[in->N_c] != in->L) return DHSA_ERR_BOUNDARIES;
    for (int k = 0; k < in->N_c; ++k)
        if (B[k + 1] <= B[k]) return DHSA_ERR_BOUNDARIES;
    p->L = in->L; p->H_q = in->H_q; p->H_kv = in->H_kv; p->G = in->H_q / in->H_kv; p->D = in->D;
    p->N_c = in->N_c;
    p->B_r = in->B_r;
    p->pooling = in->pooling;
    p->N_q = in->B_r > 0 ? (int)((in->L + in->B_r - 1) / in->B_r) : in->N_c;
    p->N_b = (int)std::min<int64_t>(in->N_b, in->L);
    p->dtype = in->dtype;
    p->scale = in->scale > 0.f ? in->scale : 1.0f / sqrtf((float)in->D);
    const int64_t row = in->D, head = in->L * in->D;
    const int esz = in->dtype == DHSA_F32 ? 4 : 2;
    struct { int64_t in_h, in_l, *out_h, *out_l; } st[4] = {
        {in->q_stride_h, in->q_stride_l, &p->qs_h, &p->qs_l}, {in->k_stride_h, in->k_stride_l, &p->ks_h, &p->ks_l},
        {in->v_stride_h, in->v_stride_l, &p->vs_h, &p->vs_l}, {in->o_stride_h, in->o_stride_l, &p->os_h, &p->os_l}};
    for (auto &s : st) {
        *s.out_l = s.in_l ? s.in_l : row;
        *s.out_h = s.in_h ? s.in_h : head;
        if (*s.out_l < row || *s.out_h < 0) return DHSA_ERR_SHAPE;
        if ((*s.out_l * esz) % 16 != 0 || (*s.out_h * esz) % 16 != 0) return DHSA_ERR_ALIGN;
    }
    // the bf16 attention kernel addresses the rows of one K / V head with 32-bit byte offsets
    if (in->dtype == DHSA_BF16 && (p->L * p->ks_l * 2 > ((int64_t)1 << 32) || p->L * p->vs_l * 2 > ((int64_t)1 << 32)))
        return DHSA_ERR_SHAPE;
    return DHSA_OK;
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Most chunks any query group can list: the chunks taken before the budget is
// met number at most 1 + (how many of the shortest chunks sum to < N_b), plus
// the query chunk itself (in the row-block form the chunk cut by the block's end
// may count with any shorter length: it is the "+ 1" that is not among the whole
// chunks).
int listed_bound(const Prob &p, std::vector<int32_t> &lens) {
    const int32_t longest = *std::max_element(lens.begin(), lens.end());
    int64_t acc = 0;
    int n = 0;
    if (longest <= 1 << 16) {
        // shortest first without a sort: count the chunks of every length (this runs once per
        // decoding step, where a sort of the lengths would cost more than the rest of the host side)
        std::vector<int32_t> hist((size_t)longest + 1, 0);
        for (int32_t len : lens) ++hist[len];
        for (int32_t len = 1; len <= longest && acc + len < p.N_b; ++len) {
            const int64_t fit = std::min<int64_t>(hist[len], (p.N_b - 1 - acc) / len);   // acc + fit len < N_b
            n += (int)fit;
            acc += fit * len;
            if (fit < hist[len]) break;
        }
    } else {
        std::sort(lens.begin(), lens.end());
        while (n < p.N_c && acc + lens[n] < p.N_b) acc += lens[n++];
    }
    return std::min(p.N_c, n + 2);
}

// How many chunks the ranking kernel puts on its first, short candidate list: enough to hold the
// budget if the best chunks were drawn at random from the length distribution, m mu - z sigma sqrt(m)
// >= N_b with z = 2.5 (the kernel checks the list it gets and falls back to the safe bound
// `stride`, so this only trades a rare second pass against a longer first sort).
int first_list_guess(const Prob &p, const std::vector<int32_t> &lens) {
    double sum = 0.0, sq = 0.0;
    for (int32_t len : lens) { sum += len; sq += (double)len * len; }
    const double mu = sum / p.N_c, var = std::max(0.0, sq / p.N_c - mu * mu), zs = 2.5 * sqrt(var);
    const double rt = (zs + sqrt(zs * zs + 4.0 * mu * p.N_b)) / (2.0 * mu);
    return (int)std::min(rt * rt + 3.0, 1048576.0);
}

PlanLayout plan_layout(const Prob &p, const int32_t *B) {
    PlanLayout pl;
    std::vector<int32_t> lens(p.N_c);
    for (int k = 0; k < p.N_c; ++k) lens[k] = B[k + 1] - B[k];
    pl.guess = first_list_guess(p, lens);
    uint32_t fnv = 2166136261u;                   // FNV-1a over the words of B
    for (int k = 0; k <= p.N_c; ++k) fnv = (fnv ^ (uint32_t)B[k]) * 16777619u;
    pl.b_sum = (int32_t)fnv;
    // row tiles: every query group is cut into pieces of 128 rows and a remainder
    int64_t cls[4] = {0, 0, 0, 0};
    auto add_group = [&cls](int64_t len, int64_t times) {
        cls[0] += times * (len / kRowTile);
        if (len % kRowTile) cls[tile_class((int)(len % kRowTile))] += times;
    };
    if (p.B_r > 0) {
        add_group(p.B_r, p.L / p.B_r);            // row blocks of B_r rows, one shorter block
        if (p.L % p.B_r) add_group(p.L % p.B_r, 1);
    } else {
        for (int k = 0; k < p.N_c; ++k) add_group(lens[k], 1);
    }
    const int64_t T1 = cls[0] + cls[1] + cls[2] + cls[3], T_big = cls[0] + cls[1];
    for (int c = 0; c < 4; ++c) pl.T_cls[c] = (int)cls[c];
    pl.stride = listed_bound(p, lens);
    pl.T1 = (int)T1;
    pl.T_big = (int)T_big;
    pl.N_q = p.N_q;
    pl.off_B = kPlanHeaderWords;
    pl.off_RB = p.B_r > 0 ? align_up(pl.off_B + p.N_c + 1, 4) : pl.off_B;
    pl.off_count = align_up(pl.off_RB + p.N_q + 1, 4);
    pl.off_entries = align_up(pl.off_count + (int64_t)p.H_q * p.N_q, 4);
    pl.off_tiles = align_up(pl.off_entries + (int64_t)p.H_q * p.N_q * pl.stride * 2, 4);
    pl.words = align_up(pl.off_tiles + (int64_t)T1 * 2, 64);
    return pl;
}

WsLayout ws_layout(const Prob &p) {
    WsLayout w;
    w.off_Qc = 0;
    w.off_Kc = align_up(w.off_Qc + (int64_t)p.H_q * p.N_q * p.D, 32);
    w.off_Sc = align_up(w.off_Kc + (int64_t)p.H_kv * p.N_c * p.D, 32);
    w.doubles = align_up(w.off_Sc + (int64_t)p.H_q * p.N_q * p.N_c, 32);
    return w;
}

// Workspace of the decoding step for up to N_c_cap chunks and L_cap tokens (the
// layout does not depend on the step's own N_c and L, so the pooled keys stay put).
DecodeLayout decode_layout(int H_q, int H_kv, int D, int64_t N_b, int N_c_cap, int64_t L_cap) {
    DecodeLayout dl;
    dl.off_Kc = 0;
    dl.off_Qc = align_up((int64_t)H_kv * N_c_cap * D * 8, 256);
    dl.off_Sc = align_up(dl.off_Qc + (int64_t)H_q * D * 8, 256);
    dl.off_plan = align_up(dl.off_Sc + (int64_t)H_q * N_c_cap * 8, 256);
    PlanLayout &pl = dl.pl;
    pl.stride = pl.guess = pl.b_sum = 0;   // set per step
    pl.T1 = pl.T_big = 0;
    pl.T_cls[0] = pl.T_cls[1] = pl.T_cls[2] = pl.T_cls[3] = 0;
    pl.N_q = 1;
    pl.off_B = 0;
    pl.off_RB = align_up((int64_t)N_c_cap + 1, 4);
    pl.off_count = pl.off_RB + 4;
    pl.off_entries = align_up(pl.off_count + H_q, 4);
    pl.off_tiles = pl.words = pl.off_entries + (int64_t)H_q * N_c_cap * 2;
    dl.off_part = align_up(dl.off_plan + pl.words * 4, 256);
    dl.S_cap = (int)((std::min<int64_t>(N_b, L_cap) + kDecSlice - 1) / kDecSlice);
    dl.bytes = align_up(dl.off_part + (int64_t)H_q * dl.S_cap * (D + 2) * 4, 256);
    return dl;
}

bool decode_caps_ok(const dhsa_problem *prob, int32_t N_c_cap, int64_t L_cap) {
    return prob && (prob->dtype == DHSA_F32 || prob->dtype == DHSA_BF16) && prob->H_q >= 1 && prob->H_kv >= 1 &&
           prob->H_q % prob->H_kv == 0 && prob->H_q <= 65535 - prob->H_kv && (prob->D == 64 || prob->D == 128) &&
           prob->N_b >= 1 && N_c_cap >= 1 && N_c_cap <= kMaxChunks && L_cap >= 1 && L_cap < (int64_t)1 << 31;
}

PlanView plan_view(const Prob &p, const PlanLayout &pl, const void *plan) {
    const int32_t *w = static_cast<const int32_t *>(plan);
    PlanView v;
    v.hdr = w;
    v.sig.H_q = p.H_q; v.sig.N_c = p.N_c; v.sig.N_b = p.N_b; v.sig.L = (int32_t)p.L; v.sig.B_r = p.B_r;
    v.sig.N_q = pl.N_q; v.sig.pooling = p.pooling; v.sig.b_sum = pl.b_sum; v.sig.stride = pl.stride; v.sig.T1 = pl.T1;
    v.B = w + pl.off_B;
    v.RB = w + pl.off_RB;
    v.count = w + pl.off_count;
    v.entries = w + pl.off_entries;
    v.tiles = w + pl.off_tiles;
    v.stride = pl.stride;
    v.T1 = pl.T1;
    v.T_big = pl.T_big;
    for (int c = 0; c < 4; ++c) v.T_cls[c] = pl.T_cls[c];
    v.N_q = pl.N_q;
    return v;
}

dhsa_status hip_status(hipError_t e) { return e == hipSuccess ? DHSA_OK : DHSA_ERR_HIP; }

// ev (may be null): events recorded after set-up, pooling, scores and ranking
dhsa_status route_impl(const Prob &p, const PlanLayout &pl, const WsLayout &wl, const void *Q, const void *K,
                       const int32_t *B_host, void *plan, void *ws, hipStream_t s, hipEvent_t *ev = nullptr) {
    int32_t *pw = static_cast<int32_t *>(plan);
    double *wd = static_cast<double *>(ws);
    // the boundaries travel as kernel arguments: no copy from (pageable) host memory, nothing that can wait
    if (launch_put_boundaries(B_host, p.N_c + 1, pw + pl.off_B, s) != hipSuccess) return DHSA_ERR_HIP;
    if (launch_setup(p, pl, pw, s) != hipSuccess) return DHSA_ERR_HIP;
    if (ev && hipEventRecord(ev[0], s) != hipSuccess) return DHSA_ERR_HIP;
    if (launch_pool(p, Q, K, pw + pl.off_B, pw + pl.off_RB, wd + wl.off_Qc, wd + wl.off_Kc, s) != hipSuccess)
        return DHSA_ERR_HIP;
    if (ev && hipEventRecord(ev[1], s) != hipSuccess) return DHSA_ERR_HIP;
    if (launch_scores(p, wd + wl.off_Qc, wd + wl.off_Kc, pw + pl.off_B, pw + pl.off_RB, wd + wl.off_Sc, s) !=
        hipSuccess)
        return DHSA_ERR_HIP;
    if (ev && hipEventRecord(ev[2], s) != hipSuccess) return DHSA_ERR_HIP;
    if (launch_select(p, pl, wd + wl.off_Sc, pw, s) != hipSuccess) return DHSA_ERR_HIP;
    if (ev && hipEventRecord(ev[3], s) != hipSuccess) return DHSA_ERR_HIP;
    return DHSA_OK;
}

// ev (may be null): three events, see launch_attn_mfma
dhsa_status attend_impl(const Prob &p, const PlanLayout &pl, const void *Q, const void *K, const void *V,
                        const void *plan, void *O, hipStream_t s, hipEvent_t *ev = nullptr) {
    const PlanView pv = plan_view(p, pl, plan);
    if (p.dtype == DHSA_BF16) return hip_status(launch_attn_mfma(p, pv, Q, K, V, O, s, ev));
    hipError_t e = launch_attn_rowwise(p, pv, Q, K, V, O, s);
    for (int i = 0; ev && i < 3 && e == hipSuccess; ++i) e = hipEventRecord(ev[i], s);
    return hip_status(e);
}

// ---- routing scratch of dhsa_prefill_static ----
// One array per GPU, created when the code object is loaded there and held until the process
// ends.  Host code never uses the array's name as an address: the device address is looked up
// once per device (with that device current) and kept.
constexpr size_t kStaticScratchBytes = (size_t)DHSA_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
void *g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device; nullptr if it cannot be had.
void *static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

__attribute__((visibility("default"))) size_t dhsa_plan_bytes(const dhsa_problem *prob, const int32_t *B_host) {
    Prob p;
    if (resolve(prob, B_host, &p) != DHSA_OK) return 0;
    return (size_t)plan_layout(p, B_host).words * sizeof(int32_t);
}

__attribute__((visibility("default"))) size_t dhsa_workspace_bytes(const dhsa_problem *prob,
                                                                   const int32_t *B_host) {
    Prob p;
    if (resolve(prob, B_host, &p) != DHSA_OK) return 0;
    return (size_t)ws_layout(p).doubles * sizeof(double);
}

__attribute__((visibility("default"))) dhsa_status dhsa_route(const dhsa_problem *prob, const void *Q_dev,
                                                              const void *K_dev, const int32_t *B_host,
                                                              void *plan_dev, size_t plan_bytes, void *ws_dev,
                                                              size_t ws_bytes, void *stream) {
    Prob p;
    dhsa_status st = resolve(prob, B_host, &p);
    if (st != DHSA_OK) return st;
    if (!Q_dev || !K_dev || !plan_dev || !ws_dev) return DHSA_ERR_NULL;
    if (misaligned(Q_dev) || misaligned(K_dev) || misaligned(plan_dev) || misaligned(ws_dev)) return DHSA_ERR_ALIGN;
    const PlanLayout pl = plan_layout(p, B_host);
    const WsLayout wl = ws_layout(p);
    if (plan_bytes < (size_t)pl.words * 4 || ws_bytes < (size_t)wl.doubles * 8) return DHSA_ERR_WORKSPACE;
    return route_impl(p, pl, wl, Q_dev, K_dev, B_host, plan_dev, ws_dev, static_cast<hipStream_t>(stream));
}

__attribute__((visibility("default"))) dhsa_status dhsa_sparse_prefill(const dhsa_problem *prob, const void *Q_dev,
                                                                       const void *K_dev, const void *V_dev,
                                                                       const int32_t *B_host, const void *plan_dev,
                                                                       size_t plan_bytes, void *O_dev,
                                                                       void *stream) {
    Prob p;
    dhsa_status st = resolve(prob, B_host, &p);
    if (st != DHSA_OK) return st;
    if (!Q_dev || !K_dev || !V_dev || !plan_dev || !O_dev) return DHSA_ERR_NULL;
    if (misaligned(Q_dev) || misaligned(K_dev) || misaligned(V_dev) || misaligned(plan_dev) || misaligned(O_dev))
        return DHSA_ERR_ALIGN;
    const PlanLayout pl = plan_layout(p, B_host);
    if (plan_bytes < (size_t)pl.words * 4) return DHSA_ERR_PLAN;
    return attend_impl(p, pl, Q_dev, K_dev, V_dev, plan_dev, O_dev, static_cast<hipStream_t>(stream));
}

__attribute__((visibility("default"))) dhsa_status dhsa_prefill(const dhsa_problem *prob, const void *Q_dev,
                                                                const void *K_dev, const void *V_dev,
                                                                const int32_t *B_host, void *O_dev, void *plan_dev,
                                                                size_t plan_bytes, void *ws_dev, size_t ws_bytes,
                                                                void *stream) {
    Prob p;
    dhsa_status st = resolve(prob, B_host, &p);
    if (st != DHSA_OK) return st;
    if (!Q_dev || !K_dev || !V_dev || !plan_dev || !O_dev || !ws_dev) return DHSA_ERR_NULL;
    if (misaligned(Q_dev) || misaligned(K_dev) || misaligned(V_dev) || misaligned(plan_dev) ||
        misaligned(O_dev) || misaligned(ws_dev))
        return DHSA_ERR_ALIGN;
    const PlanLayout pl = plan_layout(p, B_host);
    const WsLayout wl = ws_layout(p);
    if (plan_bytes < (size_t)pl.words * 4 || ws_bytes < (size_t)wl.doubles * 8) return DHSA_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = route_impl(p, pl, wl, Q_dev, K_dev, B_host, plan_dev, ws_dev, s);
    if (st != DHSA_OK) return st;
    return attend_impl(p, pl, Q_dev, K_dev, V_dev, plan_dev, O_dev, s);
}

__attribute__((visibility("default"))) size_t dhsa_static_scratch_bytes(void) { return kStaticScratchBytes; }

__attribute__((visibility("default"))) dhsa_status dhsa_prefill_static(const dhsa_problem *prob, const void *Q_dev,
                                                                       const void *K_dev, const void *V_dev,
                                                                       const int32_t *B_host, void *O_dev,
                                                                       void *plan_dev, size_t plan_bytes,
                                                                       void *stream) {
    Prob p;
    dhsa_status st = resolve(prob, B_host, &p);
    if (st != DHSA_OK) return st;
    if (!Q_dev || !K_dev || !V_dev || !plan_dev || !O_dev) return DHSA_ERR_NULL;
    if (misaligned(Q_dev) || misaligned(K_dev) || misaligned(V_dev) || misaligned(plan_dev) || misaligned(O_dev))
        return DHSA_ERR_ALIGN;
    const PlanLayout pl = plan_layout(p, B_host);
    const WsLayout wl = ws_layout(p);
    if (plan_bytes < (size_t)pl.words * 4) return DHSA_ERR_WORKSPACE;
    if ((size_t)wl.doubles * 8 > kStaticScratchBytes) return DHSA_ERR_WORKSPACE;   // beyond the static scratch
    void *ws = static_scratch();
    if (!ws) return DHSA_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // nothing in the scratch has to start at zero: the pooled vectors and every score the ranking
    // reads are written by this call before they are read
    st = route_impl(p, pl, wl, Q_dev, K_dev, B_host, plan_dev, ws, s);
    if (st != DHSA_OK) return st;
    return attend_impl(p, pl, Q_dev, K_dev, V_dev, plan_dev, O_dev, s);
}

__attribute__((visibility("default"))) dhsa_status dhsa_plan_check(const dhsa_problem *prob, const int32_t *B_host,
                                                                   const void *plan_dev, size_t plan_bytes,
                                                                   void *stream) {
    Prob p;
    dhsa_status st = resolve(prob, B_host, &p);
    if (st != DHSA_OK) return st;
    if (!plan_dev) return DHSA_ERR_NULL;
    if (misaligned(plan_dev)) return DHSA_ERR_ALIGN;
    const PlanLayout pl = plan_layout(p, B_host);
    if (plan_bytes < (size_t)pl.words * 4) return DHSA_ERR_PLAN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t hdr[kPlanHeaderWords];
    if (hipMemcpyAsync(hdr, plan_dev, sizeof(hdr), hipMemcpyDeviceToHost, s) != hipSuccess) return DHSA_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return DHSA_ERR_HIP;
    const int32_t want[18] = {DHSA_PLAN_MAGIC, DHSA_PLAN_VERSION, p.H_q, p.N_c, p.N_b, pl.stride, (int32_t)p.L, pl.T1,
                              (int32_t)pl.off_B, (int32_t)pl.off_count, (int32_t)pl.off_entries,
                              (int32_t)pl.off_tiles, pl.T_big, (int32_t)pl.off_RB, pl.N_q, p.B_r, p.pooling, pl.b_sum};
    for (int i = 0; i < 18; ++i)
        if (hdr[i] != want[i]) return DHSA_ERR_PLAN;
    return DHSA_OK;
}

__attribute__((visibility("default"))) dhsa_status dhsa_prefill_stage_times(
    const dhsa_problem *prob, const void *Q_dev, const void *K_dev, const void *V_dev, const int32_t *B_host,
    void *O_dev, void *plan_dev, size_t plan_bytes, void *ws_dev, size_t ws_bytes, float *ms_host, void *stream) {
    Prob p;
    dhsa_status st = resolve(prob, B_host, &p);
    if (st != DHSA_OK) return st;
    if (!Q_dev || !K_dev || !V_dev || !plan_dev || !O_dev || !ws_dev || !ms_host) return DHSA_ERR_NULL;
    if (misaligned(Q_dev) || misaligned(K_dev) || misaligned(V_dev) || misaligned(plan_dev) ||
        misaligned(O_dev) || misaligned(ws_dev))
        return DHSA_ERR_ALIGN;
    const PlanLayout pl = plan_layout(p, B_host);
    const WsLayout wl = ws_layout(p);
    if (plan_bytes < (size_t)pl.words * 4 || ws_bytes < (size_t)wl.doubles * 8) return DHSA_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t ev[8];   // start, then the end of each of the seven stages
    int made = 0;
    for (; made < 8; ++made)
        if (hipEventCreate(&ev[made]) != hipSuccess) break;
    st = made == 8 ? DHSA_OK : DHSA_ERR_HIP;
    if (st == DHSA_OK && hipEventRecord(ev[0], s) != hipSuccess) st = DHSA_ERR_HIP;
    if (st == DHSA_OK) st = route_impl(p, pl, wl, Q_dev, K_dev, B_host, plan_dev, ws_dev, s, ev + 1);
    if (st == DHSA_OK) st = attend_impl(p, pl, Q_dev, K_dev, V_dev, plan_dev, O_dev, s, ev + 5);
    if (st == DHSA_OK && hipEventSynchronize(ev[7]) != hipSuccess) st = DHSA_ERR_HIP;
    if (st == DHSA_OK) {
        for (int i = 0; i < 7 && st == DHSA_OK; ++i)
            if (hipEventElapsedTime(&ms_host[i], ev[i], ev[i + 1]) != hipSuccess) st = DHSA_ERR_HIP;
        if (st == DHSA_OK && hipEventElapsedTime(&ms_host[7], ev[0], ev[7]) != hipSuccess) st = DHSA_ERR_HIP;
    }
    for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
    return st;
}

__attribute__((visibility("default"))) dhsa_status dhsa_plan_expand_rows(
    const dhsa_problem *prob, const void *plan_dev, size_t plan_bytes, int32_t head, const int64_t *rows_host,
    int32_t n_rows, int64_t *rows_dev_scratch, int32_t *idx_dev, int32_t cap, int32_t *cnt_dev, void *stream) {
    if (!prob || !plan_dev || !rows_host || !rows_dev_scratch || !idx_dev || !cnt_dev) return DHSA_ERR_NULL;
    // the boundaries live in the plan; only the scalar fields of the problem are checked here
    if (prob->L < 1 || prob->N_c < 1 || prob->N_c > kMaxChunks || prob->H_q < 1 || prob->N_b < 1 || prob->B_r < 0)
        return DHSA_ERR_SHAPE;
    if (head < 0 || head >= prob->H_q || n_rows < 0) return DHSA_ERR_SHAPE;
    const int nb = (int)std::min<int64_t>(prob->N_b, prob->L);
    if (cap < nb) return DHSA_ERR_WORKSPACE;
    for (int t = 0; t < n_rows; ++t)
        if (rows_host[t] < 0 || rows_host[t] >= prob->L) return DHSA_ERR_SHAPE;
    if (plan_bytes < sizeof(int32_t) * kPlanHeaderWords) return DHSA_ERR_PLAN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // read the header back: the layout offsets are part of the plan
    int32_t hdr[kPlanHeaderWords];
    if (hipMemcpyAsync(hdr, plan_dev, sizeof(hdr), hipMemcpyDeviceToHost, s) != hipSuccess) return DHSA_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return DHSA_ERR_HIP;
    if (hdr[0] != DHSA_PLAN_MAGIC || hdr[1] != DHSA_PLAN_VERSION || hdr[2] != prob->H_q || hdr[3] != prob->N_c ||
        hdr[4] != nb || (int64_t)hdr[6] != prob->L || hdr[15] != prob->B_r ||
        hdr[14] != (prob->B_r > 0 ? (int32_t)((prob->L + prob->B_r - 1) / prob->B_r) : prob->N_c))
        return DHSA_ERR_PLAN;
    PlanLayout pl;
    pl.stride = hdr[5]; pl.T1 = hdr[7]; pl.T_big = hdr[12]; pl.N_q = hdr[14]; pl.guess = 0;
    pl.b_sum = hdr[17];                                          // no boundaries here to check it against
    pl.T_cls[0] = pl.T_cls[1] = pl.T_cls[2] = pl.T_cls[3] = 0;   // the expansion does not use the tile table
    pl.off_B = hdr[8]; pl.off_RB = hdr[13]; pl.off_count = hdr[9]; pl.off_entries = hdr[10]; pl.off_tiles = hdr[11];
    pl.words = pl.off_tiles + 2 * (int64_t)pl.T1;
    if (plan_bytes < (size_t)pl.words * 4) return DHSA_ERR_PLAN;
    Prob p;
    memset(&p, 0, sizeof(p));
    p.L = prob->L; p.H_q = prob->H_q; p.N_c = prob->N_c; p.N_b = nb; p.B_r = prob->B_r; p.N_q = pl.N_q;
    p.pooling = hdr[16];
    if (n_rows == 0) return DHSA_OK;
    if (hipMemcpyAsync(rows_dev_scratch, rows_host, sizeof(int64_t) * (size_t)n_rows, hipMemcpyHostToDevice, s) !=
        hipSuccess)
        return DHSA_ERR_HIP;
    return hip_status(launch_expand(p, plan_view(p, pl, plan_dev), head, rows_dev_scratch, n_rows, idx_dev, cap,
                                    cnt_dev, s));
}

__attribute__((visibility("default"))) size_t dhsa_decode_workspace_bytes(const dhsa_problem *prob,
                                                                          int32_t N_c_cap, int64_t L_cap) {
    if (!decode_caps_ok(prob, N_c_cap, L_cap)) return 0;
    return (size_t)decode_layout(prob->H_q, prob->H_kv, prob->D, prob->N_b, N_c_cap, L_cap).bytes;
}

__attribute__((visibility("default"))) dhsa_status dhsa_decode_step(
    const dhsa_problem *prob, const void *Q_dev, const void *K_dev, const void *V_dev, const int32_t *B_host,
    int32_t N_c_cap, int64_t L_cap, int32_t kc_valid, void *O_row_dev, int32_t *idx_dev, int32_t *cnt_dev,
    void *ws_dev, size_t ws_bytes, void *stream) {
    Prob p;
    dhsa_status st = resolve(prob, B_host, &p);
    if (st != DHSA_OK) return st;
    if (!Q_dev || !K_dev || !V_dev || !O_row_dev || !ws_dev) return DHSA_ERR_NULL;
    if (misaligned(Q_dev) || misaligned(K_dev) || misaligned(V_dev) || misaligned(O_row_dev) || misaligned(ws_dev))
        return DHSA_ERR_ALIGN;
    if (!decode_caps_ok(prob, N_c_cap, L_cap) || p.N_c > N_c_cap || p.L > L_cap) return DHSA_ERR_SHAPE;
    if (kc_valid < 0 || kc_valid >= p.N_c) return DHSA_ERR_SHAPE;   // the open chunk is always pooled anew
    DecodeLayout dl = decode_layout(p.H_q, p.H_kv, p.D, prob->N_b, N_c_cap, L_cap);
    if (ws_bytes < (size_t)dl.bytes) return DHSA_ERR_WORKSPACE;
    std::vector<int32_t> lens(p.N_c);
    for (int k = 0; k < p.N_c; ++k) lens[k] = B_host[k + 1] - B_host[k];
    dl.pl.guess = first_list_guess(p, lens);
    dl.pl.stride = listed_bound(p, lens);
    // first row of the open query group: the last chunk, or the last row block
    const int rb0 = p.B_r > 0 ? (int)(((p.L - 1) / p.B_r) * p.B_r) : B_host[p.N_c - 1];
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t *plan = reinterpret_cast<int32_t *>(static_cast<char *>(ws_dev) + dl.off_plan);
    // The boundaries B[0 .. kc_valid] are in the workspace already (the caller vouches for it).  The
    // others travel as kernel arguments when they are few (the usual step adds one or two), so that a
    // steady-state step needs no launch for them; otherwise all of B is sent (as arguments of small kernels).
    BoundaryTail tail;
    tail.n = 0;
    if (kc_valid > 0 && p.N_c - kc_valid <= kBoundaryTailMax) {
        tail.n = p.N_c - kc_valid;
        for (int j = 0; j <= tail.n; ++j) tail.b[j] = B_host[kc_valid + j];
    } else if (launch_put_boundaries(B_host, p.N_c + 1, plan + dl.pl.off_B, s) != hipSuccess) {
        return DHSA_ERR_HIP;
    }
    if (launch_decode_route(p, dl, N_c_cap, kc_valid, rb0, tail, Q_dev, K_dev, ws_dev, s) != hipSuccess)
        return DHSA_ERR_HIP;
    return hip_status(launch_decode_attend(p, dl, rb0, Q_dev, K_dev, V_dev, ws_dev, O_row_dev, idx_dev, cnt_dev, s));
}

__attribute__((visibility("default"))) size_t dhsa_recall_workspace_bytes(const dhsa_problem *prob,
                                                                        int32_t n_rows) {
    if (!prob || prob->L < 1 || prob->L >= (int64_t)1 << 31 || n_rows < 0) return 0;
    return (size_t)std::max<int64_t>((int64_t)n_rows * prob->L * 8, 256);
}

__attribute__((visibility("default"))) dhsa_status dhsa_recall_rows(
    const dhsa_problem *prob, const void *Q_dev, const void *K_dev, const int32_t *B_host, const void *plan_dev,
    size_t plan_bytes, int32_t head, const int64_t *rows_host, int32_t n_rows, int64_t *rows_dev_scratch,
    void *ws_dev, size_t ws_bytes, int32_t *hits_dev, int32_t *size_dev, void *stream) {
    Prob p;
    dhsa_status st = resolve(prob, B_host, &p);
    if (st != DHSA_OK) return st;
    if (!Q_dev || !K_dev || !plan_dev || !rows_host || !rows_dev_scratch || !ws_dev || !hits_dev || !size_dev)
        return DHSA_ERR_NULL;
    if (misaligned(Q_dev) || misaligned(K_dev) || misaligned(plan_dev) || misaligned(ws_dev)) return DHSA_ERR_ALIGN;
    if (head < 0 || head >= p.H_q || n_rows < 0) return DHSA_ERR_SHAPE;
    for (int t = 0; t < n_rows; ++t)
        if (rows_host[t] < 0 || rows_host[t] >= p.L) return DHSA_ERR_SHAPE;
    const PlanLayout pl = plan_layout(p, B_host);
    if (plan_bytes < (size_t)pl.words * 4) return DHSA_ERR_PLAN;
    if (ws_bytes < dhsa_recall_workspace_bytes(prob, n_rows)) return DHSA_ERR_WORKSPACE;
    if (n_rows == 0) return DHSA_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(rows_dev_scratch, rows_host, sizeof(int64_t) * (size_t)n_rows, hipMemcpyHostToDevice, s) !=
        hipSuccess)
        return DHSA_ERR_HIP;
    return hip_status(launch_recall(p, plan_view(p, pl, plan_dev), Q_dev, K_dev, head, rows_dev_scratch, n_rows,
                                    static_cast<unsigned long long *>(ws_dev), hits_dev, size_dev, s));
}

__attribute__((visibility("default"))) dhsa_status dhsa_debug_routing(const dhsa_problem *prob,
                                                                      const int32_t *B_host, const void *ws_dev,
                                                                      size_t ws_bytes, double *Qc_dev,
                                                                      double *Kc_dev, double *Sc_dev,
                                                                      void *stream) {
    Prob p;
    dhsa_status st = resolve(prob, B_host, &p);
    if (st != DHSA_OK) return st;
    if (!ws_dev) return DHSA_ERR_NULL;
    const WsLayout wl = ws_layout(p);
    if (ws_bytes < (size_t)wl.doubles * 8) return DHSA_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const double *wd = static_cast<const double *>(ws_dev);
    hipError_t e = hipSuccess;
    if (Qc_dev)
        e = hipMemcpyAsync(Qc_dev, wd + wl.off_Qc, sizeof(double) * (size_t)p.H_q * p.N_q * p.D,
                           hipMemcpyDeviceToDevice, s);
    if (e == hipSuccess && Kc_dev)
        e = hipMemcpyAsync(Kc_dev, wd + wl.off_Kc, sizeof(double) * (size_t)p.H_kv * p.N_c * p.D,
                           hipMemcpyDeviceToDevice, s);
    if (e == hipSuccess && Sc_dev)
        e = hipMemcpyAsync(Sc_dev, wd + wl.off_Sc, sizeof(double) * (size_t)p.H_q * p.N_q * p.N_c,
                           hipMemcpyDeviceToDevice, s);
    return hip_status(e);
}

__attribute__((visibility("default"))) dhsa_status dhsa_debug_scores(const dhsa_problem *prob, const int32_t *B_host,
                                                                     const void *ws_dev, size_t ws_bytes,
                                                                     double *Sc_dev, void *stream) {
    if (!Sc_dev) return DHSA_ERR_NULL;
    return dhsa_debug_routing(prob, B_host, ws_dev, ws_bytes, nullptr, nullptr, Sc_dev, stream);
}

__attribute__((visibility("default"))) const char *dhsa_status_string(dhsa_status s) {
    switch (s) {
        case DHSA_OK: return "ok";
        case DHSA_ERR_NULL: return "null pointer";
        case DHSA_ERR_SHAPE: return "shape out of range";
        case DHSA_ERR_BOUNDARIES: return "boundaries not strictly increasing from 0 to L";
        case DHSA_ERR_BUDGET: return "token budget below 1";
        case DHSA_ERR_DTYPE: return "unsupported dtype";
        case DHSA_ERR_WORKSPACE: return "plan or workspace too small";
        case DHSA_ERR_HIP: return "HIP runtime error";
        case DHSA_ERR_PLAN: return "plan does not match the problem";
        case DHSA_ERR_ALIGN: return "pointer or stride not 16-byte aligned";
    }
    return "unknown status";
}

__attribute__((visibility("default"))) int dhsa_version(void) { return 200; }

}  // extern "C"
