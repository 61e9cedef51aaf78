// C-ABI entry points of libvlcache: argument validation, cache bookkeeping, kernel sequencing.
// Every entry point validates on the host first and only then enqueues kernels, so a bad call
// never reaches the device.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <initializer_list>
#include <mutex>
#include <new>

#include "internal.h"

namespace {

thread_local char g_err[512] = "";

vlc_status fail(vlc_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

vlc_status hip_fail(hipError_t e, const char* where) {
    return fail(VLC_ERR_HIP, "%s: %s", where, hipGetErrorString(e));
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

size_t elem_size(int dtype) { return dtype == VLC_F32 ? 4 : 2; }

vlc_status check_shape(const vlc_shape* s) {
    if (!s) return fail(VLC_ERR_INVALID_ARG, "shape is NULL");
    if (s->dtype != VLC_F32 && s->dtype != VLC_BF16) return fail(VLC_ERR_DTYPE, "dtype %d is neither VLC_F32 nor VLC_BF16", s->dtype);
    if (s->B < 1 || s->L < 1 || s->Hq < 1 || s->Hkv < 1 || s->m < 1 || s->tau < 1)
        return fail(VLC_ERR_SHAPE, "B, L, Hq, Hkv, m, tau must be positive");
    if (s->d != 64 && s->d != 128) return fail(VLC_ERR_SHAPE, "d = %d: only 64 and 128 are built", s->d);
    if (s->Hq % s->Hkv != 0) return fail(VLC_ERR_SHAPE, "Hq = %d is not a multiple of Hkv = %d", s->Hq, s->Hkv);
    const int g = s->Hq / s->Hkv;
    if (g > 8) return fail(VLC_ERR_SHAPE, "g = Hq/Hkv = %d: at most 8 query heads per KV head", g);
    if (s->tau > s->m) return fail(VLC_ERR_SHAPE, "tau = %d exceeds m = %d", s->tau, s->m);
    if (s->tau > 4096) return fail(VLC_ERR_SHAPE, "tau = %d exceeds 4096 window rows", s->tau);
    if (s->L > vlc::kMaxLayers) return fail(VLC_ERR_SHAPE, "L = %d exceeds %d", s->L, vlc::kMaxLayers);
    if ((int64_t)s->B * s->L * s->Hkv > 65535) return fail(VLC_ERR_SHAPE, "B * L * Hkv = %lld exceeds 65535", (long long)s->B * s->L * s->Hkv);
    if ((double)s->B * s->L * s->Hq * ((s->m + 255) / 256) > 2.0e9) return fail(VLC_ERR_SHAPE, "B * L * Hq * m exceeds the grid of the scoring sweeps");
    if ((int64_t)s->B * s->L > 2048) return fail(VLC_ERR_SHAPE, "B * L = %lld exceeds 2048", (long long)s->B * s->L);
    if ((double)s->m * s->d * s->Hkv * s->L * s->B > 4.0e12) return fail(VLC_ERR_SHAPE, "K tensor larger than 4e12 elements");
    if ((s->flags & ~VLC_SHAPE_SCORE_PLAIN_ALU) != 0 || s->reserved != 0)
        return fail(VLC_ERR_INVALID_ARG, "shape flags %#x / reserved %d: unknown bits", s->flags, s->reserved);
    return VLC_OK;
}

double region_size(const vlc_shape& s) {
    return (double)s.tau * (s.m - s.tau) + (double)s.tau * (s.tau + 1) / 2.0;
}

// Workspace layout: [partial row statistics][3 arrays of B L Hq tau floats: two hold the row max and row sum of a
// standalone vlc_sparsity sweep]
struct WsPlan { size_t part, stats, total; bool mfma; };

WsPlan ws_plan(const vlc_shape& s) {
    WsPlan w;
    w.mfma = vlc::score_mfma_supported(s) && !(s.flags & VLC_SHAPE_SCORE_PLAIN_ALU);
    const size_t a = vlc::score_simple_workspace_bytes(s), b = vlc::score_mfma_workspace_bytes(s);
    w.part = align_up(a > b ? a : b, 256);
    w.stats = align_up((size_t)s.B * s.L * s.Hq * s.tau * sizeof(float), 256);
    w.total = w.part + 3 * w.stats;
    return w;
}

vlc::ScoreArgs score_args(const vlc_shape* s, const void* q_win, const void* k, const float* sm_scale, float p,
                          float* scores, float* row_max, float* row_sum, uint64_t* nnz, void* ws, vlc_stream st) {
    vlc::ScoreArgs a;
    a.s = *s; a.q_win = q_win; a.k = k; a.sm_scale = sm_scale; a.p = p; a.scores = scores;
    a.row_max = row_max; a.row_sum = row_sum; a.nnz = nnz; a.workspace = ws; a.stream = (hipStream_t)st;
    return a;
}

// ---- scratch of vlc_score_static: one array per GPU, held until the process ends ----------------
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};      // device address of `scratch` on each GPU, resolved on first use

// The address of this GPU's copy of `scratch` (the array's name is a host-side handle, not a device
// address: only the pointer resolved here may reach a kernel).
vlc_status static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(VLC_ERR_INVALID_ARG, "device ordinal %d is outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!p) return fail(VLC_ERR_HIP, "hipGetSymbolAddress(scratch) returned a null address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return VLC_OK;
}

hipError_t run_rowstats(const vlc::ScoreArgs& a, bool mfma) {
    return mfma ? vlc::launch_rowstats_mfma(a) : vlc::launch_rowstats_simple(a);
}
hipError_t run_colsweep(const vlc::ScoreArgs& a, bool mfma, bool after_rowstats) {
    return mfma ? vlc::launch_colsweep_mfma(a, after_rowstats) : vlc::launch_colsweep_simple(a);
}

}  // namespace

extern "C" {

const char* vlc_last_error_string(void) { return g_err; }
const char* vlc_version(void) { return "vlcache-mi355x 0.1 (gfx950)"; }

size_t vlc_workspace_bytes(const vlc_shape* shape) {
    if (check_shape(shape) != VLC_OK) return 0;
    return ws_plan(*shape).total;
}

vlc_status vlc_score(const vlc_shape* shape, const void* q_win, const void* k, const float* sm_scale, float p,
                     float* scores, float* row_max, float* row_sum, uint64_t* nnz, void* workspace,
                     size_t workspace_bytes, vlc_stream stream) {
    if (vlc_status st = check_shape(shape)) return st;
    if (!q_win || !k || !scores || !row_max || !row_sum || !workspace)
        return fail(VLC_ERR_INVALID_ARG, "vlc_score: q_win, k, scores, row_max, row_sum and workspace must not be NULL");
    if (nnz && !(p > 0.f && p < 1.f)) return fail(VLC_ERR_INVALID_ARG, "vlc_score: p = %g is outside (0, 1)", p);
    if (workspace_bytes < vlc_workspace_bytes(shape))
        return fail(VLC_ERR_CAPACITY, "vlc_score: workspace of %zu bytes, %zu needed", workspace_bytes, vlc_workspace_bytes(shape));
    vlc::ScoreArgs a = score_args(shape, q_win, k, sm_scale, p, scores, row_max, row_sum, nnz, workspace, stream);
    const bool mfma = ws_plan(*shape).mfma;
    hipError_t e = run_rowstats(a, mfma);
    if (e != hipSuccess) return hip_fail(e, "vlc_score row statistics");
    e = run_colsweep(a, mfma, true);              // the counters were zeroed by the row-statistics sweep
    if (e != hipSuccess) return hip_fail(e, "vlc_score column sweep");
    return VLC_OK;
}

size_t vlc_score_static_max_workspace(void) { return kStaticScratchBytes; }

vlc_status vlc_score_static(const vlc_shape* shape, const void* q_win, const void* k, const float* sm_scale, float p,
                            float* scores, float* row_max, float* row_sum, uint64_t* nnz, vlc_stream stream) {
    if (vlc_status st = check_shape(shape)) return st;
    if (!q_win || !k || !scores || !row_max || !row_sum)
        return fail(VLC_ERR_INVALID_ARG, "vlc_score_static: q_win, k, scores, row_max and row_sum must not be NULL");
    if (nnz && !(p > 0.f && p < 1.f)) return fail(VLC_ERR_INVALID_ARG, "vlc_score_static: p = %g is outside (0, 1)", p);
    const WsPlan wp = ws_plan(*shape);
    if (wp.part > kStaticScratchBytes)          // only the partial row statistics: the tail of a caller's workspace serves vlc_sparsity
        return fail(VLC_ERR_CAPACITY, "vlc_score_static: this shape needs %zu bytes of partial row statistics, the built-in scratch holds %zu; "
                                      "use vlc_score with a workspace", wp.part, kStaticScratchBytes);
    void* ws = nullptr;
    if (vlc_status st = static_scratch(&ws)) return st;
    // Every partial the column sweep reads is written by the row-statistics sweep of the same call, so
    // what an earlier call left in the array is never seen and nothing has to be cleared.
    vlc::ScoreArgs a = score_args(shape, q_win, k, sm_scale, p, scores, row_max, row_sum, nnz, ws, stream);
    hipError_t e = run_rowstats(a, wp.mfma);
    if (e != hipSuccess) return hip_fail(e, "vlc_score_static row statistics");
    e = run_colsweep(a, wp.mfma, true);
    if (e != hipSuccess) return hip_fail(e, "vlc_score_static column sweep");
    return VLC_OK;
}

vlc_status vlc_sparsity(const vlc_shape* shape, const void* q_win, const void* k, const float* sm_scale,
                        const float* row_max, float p, uint64_t* nnz, float* gamma, void* workspace,
                        size_t workspace_bytes, vlc_stream stream) {
    if (vlc_status st = check_shape(shape)) return st;
    if (!nnz) return fail(VLC_ERR_INVALID_ARG, "vlc_sparsity: nnz must not be NULL");
    hipStream_t hs = (hipStream_t)stream;
    if (q_win) {
        if (!k || !workspace) return fail(VLC_ERR_INVALID_ARG, "vlc_sparsity: k and workspace are needed for a sweep");
        if (!(p > 0.f && p < 1.f)) return fail(VLC_ERR_INVALID_ARG, "vlc_sparsity: p = %g is outside (0, 1)", p);
        if (workspace_bytes < vlc_workspace_bytes(shape))
            return fail(VLC_ERR_CAPACITY, "vlc_sparsity: workspace of %zu bytes, %zu needed", workspace_bytes, vlc_workspace_bytes(shape));
        vlc::ScoreArgs a = score_args(shape, q_win, k, sm_scale, p, nullptr, nullptr, nullptr, nnz, workspace, stream);
        const WsPlan wp = ws_plan(*shape);
        bool have_t = false;
        if (row_max) {
            a.row_max = const_cast<float*>(row_max);
        } else {
            char* tail = (char*)workspace + wp.part + wp.stats;
            a.row_max = (float*)tail;
            a.row_sum = (float*)(tail + wp.stats);
            hipError_t e = run_rowstats(a, wp.mfma);
            if (e != hipSuccess) return hip_fail(e, "vlc_sparsity row statistics");
            a.row_sum = nullptr;
            have_t = true;                          // that pass also zeroed the counters
        }
        hipError_t e = hipSuccess;
        if (!have_t) e = vlc::launch_fill_u64(nnz, (size_t)shape->B * shape->L * shape->Hq, 0, hs);
        if (e != hipSuccess) return hip_fail(e, "vlc_sparsity clear counts");
        e = run_colsweep(a, wp.mfma, have_t);
        if (e != hipSuccess) return hip_fail(e, "vlc_sparsity count sweep");
    }
    if (gamma) {
        hipError_t e = vlc::launch_gamma(*shape, nnz, gamma, hs);
        if (e != hipSuccess) return hip_fail(e, "vlc_sparsity gamma");
    }
    return VLC_OK;
}

// The matrix-core attention kernel takes bf16 storage with d = 128; every other shape, and that one too when the
// shape asks for the plain-ALU route, goes to the generic kernel, which needs no workspace.
static bool window_attn_on_matrix_cores(const vlc_shape& s) {
    return vlc::window_attn_supported(s) && !(s.flags & VLC_SHAPE_SCORE_PLAIN_ALU);
}

vlc_status vlc_window_attn_workspace_bytes(const vlc_shape* shape, size_t* bytes_out) {
    if (!bytes_out) return fail(VLC_ERR_INVALID_ARG, "vlc_window_attn_workspace_bytes: bytes_out is NULL");
    *bytes_out = 0;
    if (vlc_status st = check_shape(shape)) return st;
    if (window_attn_on_matrix_cores(*shape)) *bytes_out = vlc::window_attn_workspace_bytes(*shape);
    return VLC_OK;
}

vlc_status vlc_window_attn(const vlc_shape* shape, const void* q_win, const void* k, const void* v,
                           const float* sm_scale, void* out, float* row_max, float* row_sum,
                           void* workspace, size_t workspace_bytes, vlc_stream stream) {
    if (vlc_status st = check_shape(shape)) return st;
    if (!q_win || !k || !v || !out || !row_max || !row_sum)
        return fail(VLC_ERR_INVALID_ARG, "vlc_window_attn: q_win, k, v, out, row_max and row_sum must not be NULL");
    const bool mfma = window_attn_on_matrix_cores(*shape);
    const size_t need = mfma ? vlc::window_attn_workspace_bytes(*shape) : 0;
    if (need && !workspace) return fail(VLC_ERR_INVALID_ARG, "vlc_window_attn: workspace must not be NULL for this shape");
    if (workspace_bytes < need)
        return fail(VLC_ERR_CAPACITY, "vlc_window_attn: workspace of %zu bytes, %zu needed", workspace_bytes, need);
    vlc::WindowAttnArgs a;
    a.s = *shape; a.q_win = q_win; a.k = k; a.v = v; a.sm_scale = sm_scale; a.out = out;
    a.row_max = row_max; a.row_sum = row_sum; a.workspace = workspace; a.stream = (hipStream_t)stream;
    const hipError_t e = mfma ? vlc::launch_window_attn(a) : vlc::launch_window_attn_simple(a);
    if (e != hipSuccess) return hip_fail(e, "vlc_window_attn");
    return VLC_OK;
}

vlc_status vlc_score_from_stats(const vlc_shape* shape, const void* q_win, const void* k, const float* sm_scale,
                                float p, const float* row_max, const float* row_sum, float* scores, uint64_t* nnz,
                                vlc_stream stream) {
    if (vlc_status st = check_shape(shape)) return st;
    if (!q_win || !k || !row_max || !row_sum || !scores)
        return fail(VLC_ERR_INVALID_ARG, "vlc_score_from_stats: q_win, k, row_max, row_sum and scores must not be NULL");
    if (nnz && !(p > 0.f && p < 1.f)) return fail(VLC_ERR_INVALID_ARG, "vlc_score_from_stats: p = %g is outside (0, 1)", p);
    vlc::ScoreArgs a;
    a.s = *shape; a.q_win = q_win; a.k = k; a.sm_scale = sm_scale; a.p = nnz ? p : 0.5f; a.scores = scores;
    a.row_max = const_cast<float*>(row_max); a.row_sum = const_cast<float*>(row_sum);
    a.nnz = nnz; a.workspace = nullptr; a.stream = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    if (nnz) e = vlc::launch_fill_u64(nnz, (size_t)shape->B * shape->L * shape->Hq, 0, a.stream);
    if (e != hipSuccess) return hip_fail(e, "vlc_score_from_stats clear counts");
    e = run_colsweep(a, ws_plan(*shape).mfma, false);
    if (e != hipSuccess) return hip_fail(e, "vlc_score_from_stats column sweep");
    return VLC_OK;
}

vlc_status vlc_allocate(const vlc_shape* shape, const uint64_t* nnz, int64_t alpha_num, int64_t alpha_den,
                        int32_t* k_out, float* beta_out, vlc_stream stream) {
    if (vlc_status st = check_shape(shape)) return st;
    if (!nnz || !k_out) return fail(VLC_ERR_INVALID_ARG, "vlc_allocate: nnz and k_out must not be NULL");
    if (alpha_num < 1 || alpha_den < 1 || alpha_num > alpha_den)
        return fail(VLC_ERR_INVALID_ARG, "vlc_allocate: alpha = %lld/%lld is outside (0, 1]", (long long)alpha_num, (long long)alpha_den);
    const double lm = (double)shape->L * shape->m;
    if ((double)alpha_num * lm > 9.0e18) return fail(VLC_ERR_INVALID_ARG, "vlc_allocate: alpha_num * L * m overflows");
    const int64_t B_tot = (alpha_num * (int64_t)shape->L * shape->m) / alpha_den;
    // n_l * B_tot must fit 64 bits: n_l <= Hq * region size
    if ((double)shape->Hq * region_size(*shape) * (double)B_tot > 1.8e19)
        return fail(VLC_ERR_SHAPE, "vlc_allocate: Hq * region * budget exceeds 64-bit arithmetic");
    hipError_t e = vlc::launch_allocate(*shape, nnz, alpha_num, alpha_den, k_out, beta_out, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "vlc_allocate");
    return VLC_OK;
}

struct ArenaPlan {
    vlc_cache_layout lay;
    vlc_cache_options opt;      // resolved
    size_t items_off[vlc::kNumLists], layer_start_off[vlc::kNumLists], row_first_off[vlc::kNumLists], partials_off, counters_off, readers_off, lens_off;
    int64_t cap[vlc::kNumLists];
};

static bool one_of(int v, std::initializer_list<int> ok) {
    for (int x : ok) if (v == x) return true;
    return false;
}

// Upper bound on the units of a list that cuts rows into u_big units followed by u_small units (internal.h):
// a row of k kept slots has floor(k / u_big) + ceil((k mod u_big + T_max) / u_small) units, a rejected row one.
static int64_t list_capacity(const vlc_shape* s, int32_t T_max, int64_t spr, int ub, int us) {
    const int64_t BL = (int64_t)s->B * s->L;
    const int64_t by_small = (int64_t)s->B * spr / us + BL;
    const int64_t by_big = (int64_t)s->B * spr / ub + BL * (((int64_t)ub + T_max + us - 1) / us + 1);
    return (int64_t)s->Hkv * (by_small < by_big ? by_small : by_big);
}

static vlc_status cache_layout(const vlc_shape* s, int32_t T_max, int64_t sum_k_max, const vlc_cache_options* in, ArenaPlan* plan) {
    if (vlc_status st = check_shape(s)) return st;
    vlc_cache_options o;
    memset(&o, 0, sizeof(o));
    if (in) o = *in;
    const bool fp8 = o.kv_fp8 != 0;
    if (!one_of(o.kv_fp8, {0, 1})) return fail(VLC_ERR_INVALID_ARG, "options: kv_fp8 = %d", o.kv_fp8);
    if (fp8 && s->dtype != VLC_BF16) return fail(VLC_ERR_DTYPE, "an FP8 cache needs bf16 storage of Q, K and V");
    if (T_max < 0 || T_max > (1 << 24)) return fail(VLC_ERR_INVALID_ARG, "T_max = %d is out of range", T_max);
    if (sum_k_max < s->L || sum_k_max > (int64_t)s->L * s->m)
        return fail(VLC_ERR_INVALID_ARG, "sum_k_max = %lld is outside [L, L*m]", (long long)sum_k_max);
    if (!one_of(o.unit_slots, {0, 128, 256, 512, 1024, 2048}) || !one_of(o.tail_unit_slots, {0, 128, 256, 512, 1024, 2048}) ||
        !one_of(o.layer_unit_slots, {0, 128, 256, 512, 1024, 2048}))
        return fail(VLC_ERR_INVALID_ARG, "options: unit sizes %d / %d / %d are not among 128, 256, 512, 1024, 2048", o.unit_slots,
                    o.tail_unit_slots, o.layer_unit_slots);
    if (!one_of(o.decode_order, {0, 1, 2}) || !one_of(o.decode_merge, {0, 1, 2}) || !one_of(o.decode_zigzag, {0, 1, 2, 3}) ||
        !one_of(o.gather_rows, {0, 16, 32, 64, 128}) || !one_of(o.select_fold, {0, 1, 2}))
        return fail(VLC_ERR_INVALID_ARG, "options: decode_order %d, decode_merge %d, decode_zigzag %d, gather_rows %d or select_fold %d "
                                         "is not a listed value", o.decode_order, o.decode_merge, o.decode_zigzag, o.gather_rows, o.select_fold);
    vlc_cache_layout* lay = &plan->lay;
    const size_t es = fp8 ? 1 : elem_size(s->dtype);          // bytes per cached K/V element
    const size_t BL = (size_t)s->B * s->L;
    const int64_t spr = sum_k_max + (int64_t)s->L * T_max;
    const int64_t mean_row = sum_k_max / s->L + T_max / 2;    // slots of an average row half-way through decode
    // ---- the library's own choices
    // Launches over all layers (measured on the ragged budgets of the 7B and 34B shapes at batch 1 to 64, on an
    // MI355X: 256 CUs, three blocks of this kernel per CU, two when a KV head serves more than four query heads).
    // The walk is by size class with the partly filled units longest first, so balance comes from the order; what
    // the unit size trades is the cost of a unit's start, merge and cross-block chain against having enough units.
    //   rows >= 4 x the resident blocks: 2048-slot units (most rows are one unit: no partials at all);
    //   rows >= 1.3 x: the power of two above the mean row, so that an average row is one unit (at most 1024 slots
    //     below 2.5 x when a KV head serves more than four query heads: 960 rows of the 34B shape lose 20 % with 2048);
    //   fewer rows: whole units of the largest power of two below the slots per resident block (at least 512 slots
    //     for long rows, 256 for short ones, so that the chip still fills), and the rest of a row in units of at most
    //     512 slots, which the longest-first order then spreads behind the whole units.
    if (!o.unit_slots) {
        const int64_t rows = (int64_t)BL * s->Hkv;
        const int g = s->Hq / s->Hkv;
        const int64_t resident = 256 * ((g <= 4 && (s->dtype != VLC_F32 || s->d == 64)) ? 3 : 2);
        int u, tail;
        if (rows >= 4 * resident) {
            u = tail = vlc::kMaxUnitSlots;
        } else if (rows * 10 >= resident * 13) {
            u = 256;
            while (u < mean_row && u < vlc::kMaxUnitSlots) u <<= 1;
            if (g > 4 && rows * 2 < resident * 5 && u > 1024) u = 1024;
            tail = u;
        } else {
            u = mean_row >= 768 ? 512 : 256;
            while ((int64_t)u * 2 * resident <= rows * mean_row && u < vlc::kMaxUnitSlots) u <<= 1;
            tail = u < 512 ? u : 512;
        }
        o.unit_slots = u;
        if (!o.tail_unit_slots) o.tail_unit_slots = tail;
        if (o.tail_unit_slots > o.unit_slots) o.unit_slots = o.tail_unit_slots;
    }
    if (!o.tail_unit_slots) o.tail_unit_slots = o.unit_slots;
    if (o.tail_unit_slots > o.unit_slots)
        return fail(VLC_ERR_INVALID_ARG, "options: tail_unit_slots = %d exceeds unit_slots = %d", o.tail_unit_slots, o.unit_slots);
    // launches over a layer range: units fine enough that one layer of the batch spreads over the chip (measured:
    // 128 slots for rows of a few hundred slots, 256 beyond, where more units per row make the merge the longer wait)
    if (!o.layer_unit_slots) {
        const int64_t layer_slots = (int64_t)s->B * s->Hkv * mean_row;
        o.layer_unit_slots = mean_row < 512 ? 128 : (layer_slots / 256 <= 2048 ? 256 : 512);
    }
    plan->cap[0] = list_capacity(s, T_max, spr, o.layer_unit_slots, o.layer_unit_slots);
    plan->cap[1] = list_capacity(s, T_max, spr, o.unit_slots, o.tail_unit_slots);
    plan->cap[2] = list_capacity(s, T_max, spr, vlc::kGatherUnit, vlc::kGatherUnit);
    // a launch over all layers whose units are all resident at once (768 blocks fit the chip) gains nothing from the
    // size-class order, which only moves the units of a row apart
    if (!o.decode_order) o.decode_order = plan->cap[1] > 1536 ? 2 : 1;
    if (!o.decode_merge) o.decode_merge = 1;
    if (!o.decode_zigzag) o.decode_zigzag = 3;
    if (!o.gather_rows) o.gather_rows = 64;
    {
        // The layout rides along as one more block of the selection while all rows are resident at once and short
        // (m <= 4096), which is where a one-block kernel and its launch gap show.  With more rows the LDS the
        // layout needs would halve the selecting blocks per CU, and with longer rows, whose keys fill the register
        // file, the extra code costs registers (spills at 64 keys per lane).
        const bool short_rows = s->m <= 4096;
        if (!o.select_fold) o.select_fold = (BL * s->Hkv <= 512 && short_rows) ? 2 : 1;
        if (o.select_fold == 2 && !short_rows) o.select_fold = 1;
    }
    for (int i = 0; i < vlc::kNumLists; ++i)
        if (plan->cap[i] > (int64_t)1 << 30)
            return fail(VLC_ERR_SHAPE, "cache of %lld decode units: budgets plus reserved appends are too large", (long long)plan->cap[i]);
    plan->opt = o;
    const int g = s->Hq / s->Hkv;
    const int64_t cap_max = plan->cap[0] > plan->cap[1] ? plan->cap[0] : plan->cap[1];      // the gather's list leaves no partial results
    size_t off = 0;
    lay->status_off = off;      off = align_up(off + 4 * sizeof(int32_t), 256);
    lay->slot_off_off = off;    off = align_up(off + BL * sizeof(int64_t), 256);
    lay->kept_off = off;        off = align_up(off + BL * sizeof(int32_t), 256);
    lay->appended_off = off;    off = align_up(off + (size_t)s->L * sizeof(int32_t), 256);
    lay->kv_off = off;          off = align_up(off + (size_t)s->B * spr * 2 * s->Hkv * s->d * es, 256);
    lay->idx_off = off;         off = align_up(off + (size_t)s->B * spr * s->Hkv * sizeof(int32_t), 256);
    lay->scratch_off = off;
    for (int i = 0; i < vlc::kNumLists; ++i) {
        plan->items_off[i] = off;        off = align_up(off + (size_t)plan->cap[i] * sizeof(vlc::WorkItem), 256);
        plan->layer_start_off[i] = off;  off = align_up(off + (size_t)(s->L + 2) * sizeof(int32_t), 256);
        plan->row_first_off[i] = off;    off = align_up(off + BL * s->Hkv * sizeof(int32_t), 256);
    }
    plan->partials_off = off;     off = align_up(off + (size_t)cap_max * g * (s->d + 2) * sizeof(float), 256);
    plan->counters_off = off;     off = align_up(off + BL * s->Hkv * sizeof(int32_t), 256);
    plan->readers_off = off;      off = align_up(off + (size_t)(s->L + 1) * vlc::kReaderStride * sizeof(int32_t), 256);
    plan->lens_off = off;         off = align_up(off + (size_t)s->B * 2 * sizeof(int32_t), 256);
    lay->scale_off = off;
    if (fp8) off = align_up(off + (size_t)s->B * spr * 2 * s->Hkv * sizeof(float), 256);
    lay->kv_fp8 = fp8 ? 1 : 0;
    lay->unit_slots = o.unit_slots; lay->tail_unit_slots = o.tail_unit_slots; lay->layer_unit_slots = o.layer_unit_slots;
    lay->total_bytes = off;
    lay->slots_per_request = spr;
    return VLC_OK;
}

static vlc_cache_options options_fp8(bool fp8) {
    vlc_cache_options o;
    memset(&o, 0, sizeof(o));
    o.kv_fp8 = fp8 ? 1 : 0;
    return o;
}

static size_t cache_bytes_common(const vlc_shape* shape, int32_t T_max, int64_t sum_k_max, const vlc_cache_options* opt) {
    ArenaPlan plan;
    if (cache_layout(shape, T_max, sum_k_max, opt, &plan) != VLC_OK) return 0;
    return plan.lay.total_bytes;
}

static vlc_status cache_create_common(const char* who, const vlc_shape* shape, int32_t T_max, int64_t sum_k_max,
                                      const vlc_cache_options* opt, void* arena, size_t arena_bytes, vlc_cache** out) {
    if (!out) return fail(VLC_ERR_INVALID_ARG, "%s: out is NULL", who);
    *out = nullptr;
    ArenaPlan plan;
    if (vlc_status st = cache_layout(shape, T_max, sum_k_max, opt, &plan)) return st;
    const vlc_cache_layout& lay = plan.lay;
    if (!arena) return fail(VLC_ERR_INVALID_ARG, "%s: arena is NULL", who);
    if (((uintptr_t)arena & 255) != 0) return fail(VLC_ERR_INVALID_ARG, "%s: arena must be 256-byte aligned", who);
    if (arena_bytes < lay.total_bytes)
        return fail(VLC_ERR_CAPACITY, "%s: arena of %zu bytes, %zu needed", who, arena_bytes, lay.total_bytes);
    vlc_cache* c = new (std::nothrow) vlc_cache;
    if (!c) return fail(VLC_ERR_INVALID_ARG, "%s: out of host memory", who);
    memset(c, 0, sizeof(*c));
    c->shape = *shape;
    c->T_max = T_max;
    c->sum_k_max = sum_k_max;
    c->slots_per_request = lay.slots_per_request;
    c->arena = (char*)arena;
    c->layout = lay;
    c->opt = plan.opt;
    c->dev.status = (int32_t*)(c->arena + lay.status_off);
    c->dev.slot_off = (int64_t*)(c->arena + lay.slot_off_off);
    c->dev.kept = (int32_t*)(c->arena + lay.kept_off);
    c->dev.appended = (int32_t*)(c->arena + lay.appended_off);
    c->dev.kv = c->arena + lay.kv_off;
    c->dev.idx = (int32_t*)(c->arena + lay.idx_off);
    for (int i = 0; i < vlc::kNumLists; ++i) {
        vlc::WorkList& wl = c->dev.list[i];
        wl.items = (vlc::WorkItem*)(c->arena + plan.items_off[i]);
        wl.layer_start = (int32_t*)(c->arena + plan.layer_start_off[i]);
        wl.row_first = (int32_t*)(c->arena + plan.row_first_off[i]);
        wl.u_big = i == 0 ? plan.opt.layer_unit_slots : (i == 1 ? plan.opt.unit_slots : vlc::kGatherUnit);
        wl.u_small = i == 0 ? plan.opt.layer_unit_slots : (i == 1 ? plan.opt.tail_unit_slots : vlc::kGatherUnit);
        wl.by_size = i == 1 && plan.opt.decode_order == 2;
        wl.cap = (int32_t)plan.cap[i];
    }
    // the gather walks uniform 256-slot units in layer order: a decode list of that very form serves it too
    for (int i = 1; i >= 0; --i) {
        const vlc::WorkList& wl = c->dev.list[i];
        if (wl.u_big == vlc::kGatherUnit && wl.u_small == vlc::kGatherUnit && !wl.by_size) c->dev.list[2] = wl;
    }
    for (int i = 0; i < vlc::kNumLists; ++i) {
        c->layout.list_items_off[i] = (size_t)((char*)c->dev.list[i].items - c->arena);
        c->layout.list_index_off[i] = (size_t)((char*)c->dev.list[i].layer_start - c->arena);
        c->layout.list_by_size[i] = c->dev.list[i].by_size;
    }
    c->layout.list_reserved = 0;
    c->dev.partials = (float*)(c->arena + plan.partials_off);
    c->dev.counters = (int32_t*)(c->arena + plan.counters_off);
    c->dev.readers = (int32_t*)(c->arena + plan.readers_off);
    c->dev.lens = (int32_t*)(c->arena + plan.lens_off);
    c->dev.scales = (float*)(c->arena + lay.scale_off);
    c->kv_fp8 = plan.opt.kv_fp8 != 0;
    c->ragged = false;
    c->compacted = false;
    {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
            (void)hipGetLastError();
            cus = 256;
        }
        c->num_cus = cus;
    }
    *out = c;
    return VLC_OK;
}

size_t vlc_cache_bytes(const vlc_shape* shape, int32_t T_max, int64_t sum_k_max) {
    return cache_bytes_common(shape, T_max, sum_k_max, nullptr);
}
size_t vlc_cache_bytes_fp8(const vlc_shape* shape, int32_t T_max, int64_t sum_k_max) {
    const vlc_cache_options o = options_fp8(true);
    return cache_bytes_common(shape, T_max, sum_k_max, &o);
}
size_t vlc_cache_bytes_opt(const vlc_shape* shape, int32_t T_max, int64_t sum_k_max, const vlc_cache_options* options) {
    return cache_bytes_common(shape, T_max, sum_k_max, options);
}
vlc_status vlc_cache_create(const vlc_shape* shape, int32_t T_max, int64_t sum_k_max, void* arena,
                            size_t arena_bytes, vlc_cache** out) {
    return cache_create_common("vlc_cache_create", shape, T_max, sum_k_max, nullptr, arena, arena_bytes, out);
}
vlc_status vlc_cache_create_fp8(const vlc_shape* shape, int32_t T_max, int64_t sum_k_max, void* arena,
                                size_t arena_bytes, vlc_cache** out) {
    const vlc_cache_options o = options_fp8(true);
    return cache_create_common("vlc_cache_create_fp8", shape, T_max, sum_k_max, &o, arena, arena_bytes, out);
}
vlc_status vlc_cache_create_opt(const vlc_shape* shape, int32_t T_max, int64_t sum_k_max, const vlc_cache_options* options,
                                void* arena, size_t arena_bytes, vlc_cache** out) {
    return cache_create_common("vlc_cache_create_opt", shape, T_max, sum_k_max, options, arena, arena_bytes, out);
}

void vlc_cache_destroy(vlc_cache* cache) { delete cache; }

vlc_status vlc_cache_get_layout(const vlc_cache* cache, vlc_cache_layout* out) {
    if (!cache || !out) return fail(VLC_ERR_INVALID_ARG, "vlc_cache_get_layout: NULL argument");
    *out = cache->layout;
    return VLC_OK;
}

vlc_status vlc_cache_status(vlc_cache* cache, vlc_stream stream) {
    if (!cache) return fail(VLC_ERR_INVALID_ARG, "vlc_cache_status: cache is NULL");
    if (!cache->compacted) return VLC_OK;
    int32_t st[4] = {0, 0, 0, 0};
    hipError_t e = hipMemcpyAsync(st, cache->dev.status, sizeof(st), hipMemcpyDeviceToHost, (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "vlc_cache_status");
    if (st[0] == VLC_ERR_INVALID_ARG && st[2] == -2)
        return fail(VLC_ERR_INVALID_ARG, "request %d: per-request lengths (m_b = %d) are outside 1 <= tau_b <= min(tau, m_b), m_b <= m", st[1], st[3]);
    if (st[0] == VLC_ERR_INVALID_ARG) return fail(VLC_ERR_INVALID_ARG, "budget k[%d][%d] = %d is outside [1, m]", st[1], st[2], st[3]);
    if (st[0] == VLC_ERR_CAPACITY && st[1] == -3)
        return fail(VLC_ERR_CAPACITY, "decode step on layer %d after %d appends: only %d were reserved; the step attended without appending",
                    st[2], st[3], cache->T_max);
    if (st[0] == VLC_ERR_CAPACITY) return fail(VLC_ERR_CAPACITY, "request %d: budgets plus reserved appends need %d slots, arena has %lld",
                                               st[1], st[3], (long long)cache->slots_per_request);
    return (vlc_status)st[0];
}

static vlc_status topk_compact_common(const char* who, vlc_cache* cache, const int32_t* lens, const float* scores, const int32_t* k,
                                      int32_t n_recent, int32_t recent_num, int32_t recent_den, const void* k_full,
                                      const void* v_full, int32_t* idx_out, vlc_stream stream) {
    if (!cache) return fail(VLC_ERR_INVALID_ARG, "%s: cache is NULL", who);
    if (!scores || !k || !k_full || !v_full)
        return fail(VLC_ERR_INVALID_ARG, "%s: scores, k, k_full and v_full must not be NULL", who);
    hipStream_t hs = (hipStream_t)stream;
    hipError_t e = vlc::launch_topk_compact(*cache, lens, scores, k, n_recent, recent_num, recent_den, k_full, v_full, idx_out, hs);
    if (e != hipSuccess) return hip_fail(e, who);
    cache->compacted = true;
    cache->ragged = lens != nullptr;
    memset(cache->appended, 0, sizeof(cache->appended));
    return VLC_OK;
}

vlc_status vlc_topk_compact(vlc_cache* cache, const float* scores, const int32_t* k, int32_t n_recent,
                            const void* k_full, const void* v_full, int32_t* idx_out, vlc_stream stream) {
    const int32_t* lens = cache ? cache->shape.lens : nullptr;      // the array given at vlc_cache_create, read at every compaction
    if (n_recent < 0) return fail(VLC_ERR_INVALID_ARG, "vlc_topk_compact: n_recent = %d is negative", n_recent);
    return topk_compact_common("vlc_topk_compact", cache, lens, scores, k, n_recent, 0, 0, k_full, v_full, idx_out, stream);
}

vlc_status vlc_topk_compact_recent_frac(vlc_cache* cache, const float* scores, const int32_t* k, int32_t recent_num,
                                        int32_t recent_den, const void* k_full, const void* v_full,
                                        int32_t* idx_out, vlc_stream stream) {
    const int32_t* lens = cache ? cache->shape.lens : nullptr;      // the array given at vlc_cache_create, read at every compaction
    if (recent_den < 1 || recent_num < 0 || recent_num > recent_den)
        return fail(VLC_ERR_INVALID_ARG, "vlc_topk_compact_recent_frac: fraction %d/%d is outside [0, 1]", recent_num, recent_den);
    return topk_compact_common("vlc_topk_compact_recent_frac", cache, lens, scores, k, 0, recent_num, recent_den, k_full, v_full,
                               idx_out, stream);
}

vlc_status vlc_cache_hit_rate(vlc_cache* cache, const float* scores_star, int32_t* hits_out, float* rate_out,
                              vlc_stream stream) {
    if (!cache) return fail(VLC_ERR_INVALID_ARG, "vlc_cache_hit_rate: cache is NULL");
    if (!cache->compacted) return fail(VLC_ERR_INVALID_ARG, "vlc_cache_hit_rate: the cache has not been filled by vlc_topk_compact");
    if (!scores_star || !hits_out) return fail(VLC_ERR_INVALID_ARG, "vlc_cache_hit_rate: scores_star and hits_out must not be NULL");
    hipError_t e = vlc::launch_cache_hit_count(*cache, scores_star, hits_out, rate_out, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "vlc_cache_hit_rate");
    return VLC_OK;
}

vlc_status vlc_decode_attn(vlc_cache* cache, int32_t layer_begin, int32_t layer_end, const void* q,
                           const void* k_new, const void* v_new, const float* sm_scale, void* out,
                           vlc_stream stream) {
    if (!cache) return fail(VLC_ERR_INVALID_ARG, "vlc_decode_attn: cache is NULL");
    if (!cache->compacted) return fail(VLC_ERR_INVALID_ARG, "vlc_decode_attn: the cache has not been filled by vlc_topk_compact");
    if (layer_begin < 0 || layer_end > cache->shape.L || layer_begin >= layer_end)
        return fail(VLC_ERR_INVALID_ARG, "vlc_decode_attn: layer range [%d, %d) is outside [0, %d)", layer_begin, layer_end, cache->shape.L);
    if (!q || !out) return fail(VLC_ERR_INVALID_ARG, "vlc_decode_attn: q and out must not be NULL");
    if ((k_new == nullptr) != (v_new == nullptr))
        return fail(VLC_ERR_INVALID_ARG, "vlc_decode_attn: k_new and v_new must both be given or both be NULL");
    const int appended = cache->appended[layer_begin];
    for (int l = layer_begin; l < layer_end; ++l)
        if (cache->appended[l] != appended)
            return fail(VLC_ERR_INVALID_ARG, "vlc_decode_attn: layers %d and %d have %d and %d appends; call them separately",
                        layer_begin, l, appended, cache->appended[l]);
    if (k_new && appended >= cache->T_max)
        return fail(VLC_ERR_CAPACITY, "vlc_decode_attn: layer %d already holds the %d appends reserved", layer_begin, cache->T_max);
    vlc::DecodeArgs a;
    a.c = cache; a.layer_begin = layer_begin; a.n_layers = layer_end - layer_begin;
    a.q = q; a.k_new = k_new; a.v_new = v_new; a.sm_scale = sm_scale; a.out = out;
    a.stream = (hipStream_t)stream;
    hipError_t e = vlc::launch_decode(a);
    if (e != hipSuccess) return hip_fail(e, "vlc_decode_attn");
    if (k_new)
        for (int l = layer_begin; l < layer_end; ++l) cache->appended[l] += 1;
    return VLC_OK;
}

vlc_status vlc_probe_read_stream(const void* buf, size_t bytes, uint32_t* sink, int32_t blocks, vlc_stream stream) {
    if (!buf || !sink) return fail(VLC_ERR_INVALID_ARG, "vlc_probe_read_stream: buf and sink must not be NULL");
    if (bytes < 16 || (bytes & 15) != 0 || ((uintptr_t)buf & 15) != 0)
        return fail(VLC_ERR_INVALID_ARG, "vlc_probe_read_stream: %zu bytes at %p: size and address must be multiples of 16", bytes, buf);
    if (blocks < 1 || blocks > (1 << 20)) return fail(VLC_ERR_INVALID_ARG, "vlc_probe_read_stream: blocks = %d", blocks);
    const hipError_t e = vlc::launch_read_stream(buf, bytes, sink, blocks, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "vlc_probe_read_stream");
    return VLC_OK;
}

vlc_status vlc_decode_attn_steps(vlc_cache* cache, int32_t layer_begin, int32_t layer_end, int32_t n_steps,
                                 const void* q, const void* k_new, const void* v_new, const float* sm_scale,
                                 void* out, vlc_stream stream) {
    if (!cache) return fail(VLC_ERR_INVALID_ARG, "vlc_decode_attn_steps: cache is NULL");
    if (n_steps < 1) return fail(VLC_ERR_INVALID_ARG, "vlc_decode_attn_steps: n_steps = %d", n_steps);
    if (!q || !k_new || !v_new || !out)
        return fail(VLC_ERR_INVALID_ARG, "vlc_decode_attn_steps: q, k_new, v_new and out must not be NULL");
    if (layer_begin < 0 || layer_end > cache->shape.L || layer_begin >= layer_end)
        return fail(VLC_ERR_INVALID_ARG, "vlc_decode_attn_steps: layer range [%d, %d) is outside [0, %d)", layer_begin, layer_end, cache->shape.L);
    const vlc_shape& s = cache->shape;
    const size_t es = elem_size(s.dtype);
    const size_t nl = (size_t)(layer_end - layer_begin);
    const size_t q_step = nl * s.B * s.Hq * s.d * es, kv_step = nl * s.B * s.Hkv * s.d * es;
    for (int t = 0; t < n_steps; ++t) {
        vlc_status st = vlc_decode_attn(cache, layer_begin, layer_end, (const char*)q + t * q_step,
                                        (const char*)k_new + t * kv_step, (const char*)v_new + t * kv_step, sm_scale,
                                        (char*)out + t * q_step, stream);
        if (st != VLC_OK) return st;
    }
    return VLC_OK;
}

}  // extern "C"
