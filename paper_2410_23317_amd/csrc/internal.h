// Host-side internals of libvlcache: the cache bookkeeping and the kernel launchers that the
// C-ABI entry points (api.hip) call after validating their arguments.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "vlcache.h"

namespace vlc {

constexpr int kMaxLayers = 1024;
constexpr int kScoreChunk = 256;       // keys per block of the generic scoring sweeps
constexpr int kReaderStride = 64;      // ints between the ticket counters of two layers: a cache line each (measured: counters that share a
                                       // line cost a launch over all layers of the 7B shape 1.7 of 16 us)

// One block-unit of decode work: consecutive cache slots [key0, key0 + ucap) of one (b, l, kv head) row.
// vlc_topk_compact builds three lists of them on the device.  A row is cut into floor(kept / u_big) units of
// u_big slots followed by units of u_small slots that hold the end of the row and the append reserve.
//   list 0 (launches over a layer range): ordered by (layer, request, kv head, unit), so that a layer
//           range is a contiguous slice;
//   list 2 (the gather of the compaction): the same order, uniform fine units;
//   list 1 (launches over all layers): the same order, or by size class (all u_big units, then the small
//           units that hold kept rows, the (request, layer) entries with the most slots beyond their u_big
//           units first, then the units that only hold append reserve), so that the blocks dispatched last
//           are the short ones.
struct WorkItem {
    int32_t row_abs;                   // (b*L + l)*Hkv + hkv
    int32_t key0;                      // first slot of the unit
    int32_t kept;                      // validated k[b][l]; 0 marks a rejected row
    int32_t unit;                      // index of the unit inside its row
    int64_t kbase;                     // element offset of the row's K slab inside the kv region
    int64_t idx_base;                  // offset of the row's kept-index list inside the idx region
    int32_t b, l;
    int32_t canon;                     // index of this unit in the (layer, request, kv head, unit) order of its list
    int32_t ucap;                      // slots of the unit
    int32_t hkv;                       // the row's KV head
    int32_t layer_units;               // units of layer l in this list (every one of them takes a ticket in a launch that appends)
    int32_t pad[2];
};
static_assert(sizeof(WorkItem) == 64, "WorkItem layout: one 64-byte scalar load");

constexpr int kMaxUnitSlots = 2048;     // largest block-unit of a work list (the options admit 128 .. 2048)
constexpr int kNumLists = 3;
constexpr int kGatherUnit = 256;        // slots per unit of the gather's list

struct WorkList {
    WorkItem* items;                   // [cap]
    int32_t* layer_start;              // [L+2]: canon index of each layer's first unit, [L] the number of units, [L+1] the number of u_big units
    int32_t* row_first;                // [B*L*Hkv]: canon index of each row's first unit
    int32_t u_big, u_small;            // powers of two, u_small <= u_big
    int32_t by_size;                   // items are stored by size class (else in canon order)
    int32_t cap;                       // capacity in units
};

struct CacheDev {                      // device pointers into the caller's arena
    int32_t* status;                   // [4]
    int64_t* slot_off;                 // [B*L]
    int32_t* kept;                     // [B*L]
    char* kv;
    int32_t* idx;
    WorkList list[kNumLists];         // 0: launches over a layer range, 1: launches over all layers, 2: the gather
    float* partials;                   // [max list cap][g][d + 2]
    int32_t* counters;                 // [B*L*Hkv] units of a row that have left their partial result
    int32_t* appended;                 // [L] appends each layer has received since the last compaction
    int32_t* readers;                  // [(L + 1) * kReaderStride] blocks of a launch that have read the append count: per layer, and per launch after the last layer
    int32_t* lens;                     // [B][2] copy of the per-request (m_b, tau_b) of the last compaction
    float* scales;                     // FP8 caches: one fp32 scale per K row and per V row, laid out like the rows
};

}  // namespace vlc

struct vlc_cache {
    vlc_shape shape;
    int32_t T_max;
    int64_t sum_k_max;
    int64_t slots_per_request;
    vlc_cache_options opt;             // every field resolved (no zeros left)
    char* arena;
    vlc_cache_layout layout;
    vlc::CacheDev dev;
    bool compacted;
    bool kv_fp8;                       // rows stored as E4M3 codes + per-row scale
    bool ragged;                       // the last compaction had per-request lengths (dev.lens is valid)
    int32_t num_cus;                   // compute units of the device the cache was created on
    int32_t appended[vlc::kMaxLayers]; // decode appends enqueued so far, per layer (the device keeps the count the kernels use)
};

namespace vlc {

// ---- scoring sweeps (score_simple.hip: any dtype; score_mfma.hip: bf16 matrix-core path) ----
struct ScoreArgs {
    vlc_shape s;
    const void* q_win;
    const void* k;
    const float* sm_scale;      // may be null
    float p;
    float* scores;              // null: count only
    float* row_max;
    float* row_sum;
    uint64_t* nnz;              // null: no counting
    void* workspace;
    hipStream_t stream;
};
size_t score_simple_workspace_bytes(const vlc_shape& s);
hipError_t launch_rowstats_simple(const ScoreArgs& a);     // fills row_max, row_sum; zeroes nnz if given
hipError_t launch_colsweep_simple(const ScoreArgs& a);     // scores and/or nnz from row_max,row_sum
bool score_mfma_supported(const vlc_shape& s);            // bf16, d = 128
size_t score_mfma_workspace_bytes(const vlc_shape& s);
hipError_t launch_rowstats_mfma(const ScoreArgs& a);       // leaves per-split partial statistics in the workspace; zeroes nnz if given
hipError_t launch_colsweep_mfma(const ScoreArgs& a, bool merge_partials);   // merge_partials: statistics come from the sweep just run (row_max, row_sum are then outputs)
hipError_t launch_fill_u64(uint64_t* p, size_t n, uint64_t v, hipStream_t st);
hipError_t launch_gamma(const vlc_shape& s, const uint64_t* nnz, float* gamma, hipStream_t st);

// ---- window attention with row statistics (matrix-core path only: bf16, d = 128) ----
struct WindowAttnArgs {
    vlc_shape s;
    const void* q_win;
    const void* k;
    const void* v;
    const float* sm_scale;      // may be null
    void* out;                  // [B,L,Hq,tau,d]
    float* row_max;
    float* row_sum;
    void* workspace;
    hipStream_t stream;
};
bool window_attn_supported(const vlc_shape& s);
size_t window_attn_workspace_bytes(const vlc_shape& s);
hipError_t launch_window_attn(const WindowAttnArgs& a);
hipError_t launch_window_attn_simple(const WindowAttnArgs& a);      // any dtype and d (window_attn_simple.hip); no workspace

// ---- allocation ----
hipError_t launch_allocate(const vlc_shape& s, const uint64_t* nnz, int64_t alpha_num, int64_t alpha_den,
                           int32_t* k_out, float* beta_out, hipStream_t st);

// ---- eviction ----
// recent_den > 0: the recent window is floor(k * recent_num / recent_den) per (b, l), n_recent is ignored
// lens: per-request (m_b, tau_b) of this compaction (device, may be null); copied into the cache
hipError_t launch_topk_compact(const vlc_cache& c, const int32_t* lens, const float* scores, const int32_t* k,
                               int32_t n_recent, int32_t recent_num, int32_t recent_den,
                               const void* k_full, const void* v_full, int32_t* idx_out, hipStream_t st);

// |kept positions of the cache ∩ top-k of scores_star| per (b, l, kv head) row, k = the row's budget
hipError_t launch_cache_hit_count(const vlc_cache& c, const float* scores_star, int32_t* hits_out, float* rate_out,
                                  hipStream_t st);

// ---- decode ----
struct DecodeArgs {
    const vlc_cache* c;
    int layer_begin, n_layers;
    const void* q;
    const void* k_new;
    const void* v_new;
    const float* sm_scale;
    void* out;
    hipStream_t stream;
};
hipError_t launch_decode(const DecodeArgs& a);

// ---- measurement aid: a kernel that only reads `bytes` bytes (a multiple of 16) once
hipError_t launch_read_stream(const void* buf, size_t bytes, uint32_t* sink, int blocks, hipStream_t st);

}  // namespace vlc
