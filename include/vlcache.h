/*
 * vlcache.h -- C ABI of the VL-Cache hot path for AMD MI355X (gfx950).
 *
 * The path runs once after prefill (score -> sparsity -> allocate -> topk_compact) and then
 * on every decode step (decode_attn over the compressed, ragged, per-layer cache).
 *
 * Notation is the paper's: m prompt tokens, tau rows of the post-vision query window
 * (the last tau prompt tokens), L layers, Hq query heads, Hkv key/value heads,
 * g = Hq / Hkv, d head dimension, p the ThresholdFilter threshold, alpha the whole-model
 * cache budget, k_l the token budget of layer l.
 *
 * Conventions shared by every call
 *   - Tensor arguments are DEVICE pointers owned by the caller, contiguous (row-major) in
 *     the stated layout, 16-byte aligned.  The library keeps no pointer after a call returns,
 *     except for the arena and the shape's optional lens array handed to vlc_cache_create
 *     (lens is read again by every vlc_topk_compact on that cache).
 *   - Every call only enqueues work on the given HIP stream and returns; no call
 *     synchronises, allocates or frees device memory (vlc_cache_status synchronises, and says so).
 *   - Calls return a vlc_status; nothing throws or aborts.  vlc_last_error_string() holds a
 *     description of the calling thread's last failure.
 *   - Errors that only the device can see (a budget outside [1, m], a cache arena too
 *     small for the budgets) set a sticky flag inside the cache; the offending rows are skipped
 *     without touching memory, and vlc_cache_status reports the flag.
 *   - Query head h reads key/value head h / g (consecutive query heads share a KV head).
 *   - A vlc_cache owns device scratch (partial results, counters, the per-layer append counts):
 *     calls on one cache come from one thread at a time, on one stream or on streams the caller
 *     orders; calls that overlap on the device race.  Different caches are independent.  The
 *     scoring calls keep their intermediates in the caller's workspace: calls that may overlap on
 *     the device need workspaces of their own.
 *   - No call reads the process environment; behaviour depends on the arguments only.
 *   - Every call may be recorded into a HIP graph (stream capture) and replayed: the kernels take
 *     everything that changes from step to step (budgets, cache layout, append counts) from device
 *     memory, never from values fixed at enqueue time.
 */
#ifndef VLCACHE_H
#define VLCACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    VLC_OK = 0,
    VLC_ERR_INVALID_ARG = 1,   /* null pointer, value out of range, inconsistent call order */
    VLC_ERR_SHAPE = 2,         /* shape the kernels do not cover (see vlc_shape)             */
    VLC_ERR_DTYPE = 3,
    VLC_ERR_CAPACITY = 4,      /* arena / workspace too small, or more appends than reserved  */
    VLC_ERR_HIP = 5,           /* a HIP runtime call failed (message in vlc_last_error_string)*/
    VLC_ERR_UNIMPLEMENTED = 6
} vlc_status;

typedef enum { VLC_F32 = 0, VLC_BF16 = 1 } vlc_dtype;

/* A hipStream_t, passed as a plain pointer so that C callers need no HIP headers.
 * NULL is the device's default stream. */
typedef void* vlc_stream;

/* Problem shape.  m and tau are the prompt length and the post-vision window length (paper Sec. 3.2),
 * and the strides of every tensor: K, V [B,L,Hkv,m,d], Q' [B,L,Hq,tau,d], scores [B,L,Hkv,m], ...
 * Supported: d in {64, 128}; Hq % Hkv == 0 with g <= 8; 1 <= tau <= min(m, 4096);
 * L <= 1024; B * L <= 2048; B * L * Hkv <= 65535; dtype is the storage type of Q, K, V and of the decode output.
 *
 * lens == NULL: every request has prompt length m and window tau.
 * lens != NULL (ragged batch): DEVICE array int32 [B][2] = (m_b, tau_b) with 1 <= tau_b <= tau,
 * tau_b <= m_b <= m.  Request b then uses keys [0, m_b) of its K/V rows and rows [0, tau_b) of its
 * window (row i is prompt position m_b - tau_b + i); the rest of the padded tensors is never read.
 * Outputs beyond a request's lengths: scores[b,..,j >= m_b] = 0; row_max / row_sum rows >= tau_b are
 * left untouched; budgets are computed from m_b (total floor(alpha L m_b), clips ceil(m_b/100) and m_b).
 * The array is read when a call's kernels run (it must stay valid until then); values outside
 * the ranges above are clamped into them by the scoring calls and reported as VLC_ERR_INVALID_ARG by
 * vlc_cache_status after vlc_topk_compact, which also copies the array into the cache. */
typedef struct {
    int32_t B, L, Hq, Hkv, d, m, tau;
    int32_t dtype;             /* vlc_dtype */
    const int32_t* lens;       /* device, [B][2], or NULL */
    int32_t flags;             /* 0, or VLC_SHAPE_* bits */
    int32_t reserved;          /* 0 */
} vlc_shape;

/* vlc_shape.flags: take the plain-ALU scoring sweeps, and the generic window-attention kernel, even where the
 * matrix-core kernels cover the shape (bf16, d = 128).  Same results to the stated tolerances; a cross-check
 * for tests.  The workspace queries and the calls read the flag from the same shape, so a size query and the
 * call it is for always agree. */
#define VLC_SHAPE_SCORE_PLAIN_ALU 1

const char* vlc_last_error_string(void);
const char* vlc_version(void);

/* Bytes of scratch vlc_score / vlc_sparsity need for this shape (partial row statistics). */
size_t vlc_workspace_bytes(const vlc_shape* shape);

/*
 * vlc_score -- accumulated post-vision attention (paper Sec. 3.2; Alg. 1 ComputeSparsity for
 * the softmax; App. A.3 for the two-sweep schedule that never writes the attention matrix).
 *
 *   s_ij  = sm_scale[l] * <q_win[b,l,h,i,:], k[b,l,h/g,j,:]>,  valid iff j <= m - tau + i
 *   A'_ij = exp(s_ij - M_i) / Z_i over the valid j of row i   (M_i = row max, Z_i = row sum)
 *   scores[b,l,hkv,j] = sum over the g query heads of the group and over rows i of A'_ij
 *   nnz[b,l,h]        = #{valid (i,j): s_ij - M_i >= ln p}     (only if nnz != NULL; Eq. 1)
 *
 * q_win   [B,L,Hq,tau,d]  in   storage dtype
 * k       [B,L,Hkv,m,d]   in   storage dtype
 * sm_scale[L] float       in   per-layer logit scale, or NULL for 1/sqrt(d)
 * p                       in   threshold in (0,1); ignored when nnz == NULL
 * scores  [B,L,Hkv,m]     out  fp32
 * row_max [B,L,Hq,tau]    out  fp32, M_i (natural-log domain)
 * row_sum [B,L,Hq,tau]    out  fp32, Z_i
 * nnz     [B,L,Hq]        out  uint64, may be NULL (counting rides on the score sweep)
 * workspace               scratch of at least vlc_workspace_bytes(shape) bytes
 */
vlc_status vlc_score(const vlc_shape* shape, const void* q_win, const void* k,
                     const float* sm_scale, float p,
                     float* scores, float* row_max, float* row_sum, uint64_t* nnz,
                     void* workspace, size_t workspace_bytes, vlc_stream stream);

/*
 * vlc_score_static -- vlc_score for callers that cannot allocate device memory or hold a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same
 * arguments, outputs and errors as vlc_score, without the workspace: the partial row statistics live
 * in an array built into the library, vlc_score_static_max_workspace() bytes (16 MiB) per GPU, which
 * the GPU holds until the process ends.  A shape whose partial statistics need more is rejected with
 * VLC_ERR_CAPACITY (use vlc_score).  The call allocates and frees nothing.  All calls on one GPU share
 * that array: calls that may overlap on the device (different streams) race; calls ordered on one
 * stream are fine, and nothing an earlier call left in the array is read.
 */
size_t     vlc_score_static_max_workspace(void);
vlc_status vlc_score_static(const vlc_shape* shape, const void* q_win, const void* k,
                            const float* sm_scale, float p,
                            float* scores, float* row_max, float* row_sum, uint64_t* nnz,
                            vlc_stream stream);

/*
 * vlc_sparsity -- ThresholdFilter sparsity of the post-vision attention (paper Eq. 1, Eq. 2,
 * Alg. 1 ComputeSparsity):  gamma = 1 - nnz / D,  D = tau (m - tau) + tau (tau + 1) / 2.
 *
 * Two modes:
 *   q_win != NULL: standalone sweep.  Counts nnz as defined under vlc_score; row_max may be
 *                  the array vlc_score produced, or NULL to recompute the row statistics.
 *   q_win == NULL: finalise only.  nnz is an INPUT (as filled by vlc_score) and gamma is
 *                  computed from it; k, sm_scale, row_max and workspace are ignored.
 * nnz   [B,L,Hq] uint64   out (in, when finalising)
 * gamma [B,L,Hq] float    out, may be NULL
 */
vlc_status vlc_sparsity(const vlc_shape* shape, const void* q_win, const void* k,
                        const float* sm_scale, const float* row_max, float p,
                        uint64_t* nnz, float* gamma,
                        void* workspace, size_t workspace_bytes, vlc_stream stream);

/*
 * vlc_window_attn -- causal prefill attention of the post-vision window rows that also hands out
 * its row statistics (paper Sec. 2.1, prefill phase, for the last tau prompt positions; App. A.3:
 * the first scoring kernel computes the two reductions a fused-softmax attention kernel carries
 * anyway).  With it the row-statistics sweep of vlc_score is not needed: a model runs this call as
 * the attention of its last tau prompt rows and then vlc_score_from_stats.
 *
 *   out[b,l,h,i,:] = sum over valid j of A'_ij * v[b,l,h/g,j,:]     (A', validity as under vlc_score)
 *   row_max, row_sum = M_i, Z_i of the same softmax
 *
 * q_win   [B,L,Hq,tau,d]  in   storage dtype
 * k, v    [B,L,Hkv,m,d]   in   storage dtype
 * out     [B,L,Hq,tau,d]  out  storage dtype (fp32 accumulation)
 * row_max, row_sum [B,L,Hq,tau] out fp32
 * workspace               scratch of at least vlc_window_attn_workspace_bytes(shape) bytes; may be NULL when
 *                         that is 0
 * Two kernels: bf16 storage with d = 128 runs on the matrix cores (probabilities rounded to bf16 for the
 * P.V product; key range split over blocks, partial results in the workspace); every other dtype / d, and
 * that shape too when shape->flags has VLC_SHAPE_SCORE_PLAIN_ALU, runs a generic kernel (one wave per window
 * row, fp32 probabilities, no workspace: the query stores 0), written for coverage rather than speed.
 * With shape->lens, rows >= tau_b of request b are left untouched.
 */
vlc_status vlc_window_attn_workspace_bytes(const vlc_shape* shape, size_t* bytes_out);
vlc_status vlc_window_attn(const vlc_shape* shape, const void* q_win, const void* k, const void* v,
                           const float* sm_scale, void* out, float* row_max, float* row_sum,
                           void* workspace, size_t workspace_bytes, vlc_stream stream);

/*
 * vlc_score_from_stats -- the column sweep of vlc_score alone (paper App. A.3, second kernel), for
 * row statistics the caller already has (from vlc_window_attn, or from its own prefill attention):
 * scores and nnz exactly as defined under vlc_score, with row_max (natural-log domain) and row_sum
 * as INPUTS.  Any dtype and d the scoring path supports; needs no workspace.  nnz may be NULL.
 */
vlc_status vlc_score_from_stats(const vlc_shape* shape, const void* q_win, const void* k,
                                const float* sm_scale, float p,
                                const float* row_max, const float* row_sum,
                                float* scores, uint64_t* nnz, vlc_stream stream);

/*
 * vlc_allocate -- sparsity-aware layer budgets (paper Alg. 1, SkewedCacheBudgetAllocation),
 * in integers.  Per request: n_l = sum_h nnz[b,l,h] (proportional to 1 - gamma'_l),
 * N = sum_l n_l, B_tot = floor(alpha_num * L * m / alpha_den); floor quotas
 * q_l = floor(n_l * B_tot / N), then +1 to the B_tot - sum q_l layers with the largest
 * remainders (ties to the lower layer); k_l = clip(q_l, max(1, ceil(m/100)), m), the token
 * form of the paper's clip(beta, 0.01, 1).  No renormalisation after the clip.
 *
 * nnz      [B,L,Hq] uint64  in
 * alpha    as a rational alpha_num / alpha_den, 0 < alpha <= 1
 * k_out    [B,L] int32      out
 * beta_out [B,L] float      out, k_l / m, may be NULL
 */
vlc_status vlc_allocate(const vlc_shape* shape, const uint64_t* nnz,
                        int64_t alpha_num, int64_t alpha_den,
                        int32_t* k_out, float* beta_out, vlc_stream stream);

/*
 * The compressed cache.  The caller owns one device arena; the library lays out inside it
 * the ragged per-layer K/V slabs (layer l of request b holds k[b][l] + T_max slots per KV
 * head), the kept indices, per-layer offsets, and the split-KV scratch of decode.
 *
 * T_max      decode appends reserved per layer
 * sum_k_max  upper bound on sum_l k[b][l] of one request (e.g. B_tot + L * ceil(m/100))
 */
typedef struct vlc_cache vlc_cache;

size_t     vlc_cache_bytes(const vlc_shape* shape, int32_t T_max, int64_t sum_k_max);
vlc_status vlc_cache_create(const vlc_shape* shape, int32_t T_max, int64_t sum_k_max,
                            void* arena, size_t arena_bytes, vlc_cache** out);

/* The same cache with its K/V rows stored as FP8 (paper App. A.2 names FP8 KV-cache quantisation as an
 * orthogonal technique that combines with sparsification; this halves the bytes a decode step reads).
 * Format: OCP E4M3 codes, one fp32 scale per row (slot and KV head): scale = absmax(row) / 448
 * (1 for an all-zero row), code = nearest E4M3 value to fp32(x / scale), ties to even.  Rows are
 * quantised when vlc_topk_compact gathers them and when a decode step appends; decode attends over
 * the dequantised values code * scale.  bf16 storage only (VLC_ERR_DTYPE otherwise).  Every other
 * call takes such a cache unchanged. */
size_t     vlc_cache_bytes_fp8(const vlc_shape* shape, int32_t T_max, int64_t sum_k_max);
vlc_status vlc_cache_create_fp8(const vlc_shape* shape, int32_t T_max, int64_t sum_k_max,
                                void* arena, size_t arena_bytes, vlc_cache** out);

/* Cache creation with explicit options: everything the two calls above decide by themselves.  A zero in a
 * field (or options == NULL) keeps the library's choice for that field; a value outside a field's list is
 * VLC_ERR_INVALID_ARG.  The options only move work between blocks and kernels: results are the same to the
 * decode tolerance, and they are fixed for the cache's lifetime.
 *   kv_fp8            1: rows stored as E4M3 codes + per-row scale (vlc_cache_create_fp8)
 *   unit_slots        decode launches over ALL layers cut every cached row into block-units; slots of a unit
 *                     that lies wholly inside the kept rows: 128, 256, 512, 1024 or 2048
 *   tail_unit_slots   slots of the units that hold the end of a row and the slots reserved for appends:
 *                     128 .. 2048, not above unit_slots
 *   layer_unit_slots  slots per unit for launches over a layer range (how a model calls decode): 128 .. 2048
 *   decode_order      1: launches over all layers walk the units layer by layer; 2: by size class (whole
 *                     units first, then row ends with the longest first, then append reserve), so the blocks
 *                     dispatched last are short
 *   decode_merge      1: the unit of a row that finishes last merges the row's partial results inside the
 *                     decode kernel; 2: a second kernel merges
 *   decode_zigzag     1: off; 2: a wave walks its tiles backwards on odd steps; 3: also the whole units of a
 *                     size-class walk (what the previous step read last is what the caches still hold)
 *   gather_rows       rows of K and of V one block of the compaction moves: 16, 32, 64 or 128
 *   select_fold       1: the cache layout always runs as a kernel of its own; 2: always inside one more block
 *                     of the selection kernel (B * L <= 2048 in either case) */
typedef struct {
    int32_t kv_fp8;
    int32_t unit_slots, tail_unit_slots, layer_unit_slots;
    int32_t decode_order, decode_merge, decode_zigzag;
    int32_t gather_rows, select_fold;
    int32_t reserved[7];       /* 0 */
} vlc_cache_options;
size_t     vlc_cache_bytes_opt(const vlc_shape* shape, int32_t T_max, int64_t sum_k_max,
                               const vlc_cache_options* options);
vlc_status vlc_cache_create_opt(const vlc_shape* shape, int32_t T_max, int64_t sum_k_max,
                                const vlc_cache_options* options,
                                void* arena, size_t arena_bytes, vlc_cache** out);
void       vlc_cache_destroy(vlc_cache* cache);      /* frees host bookkeeping only */

/* Where things live inside the arena (byte offsets from its base), for tests and tools.
 * Slab of (b,l): cap = k[b][l] + T_max slots; K rows of KV head h start at
 *   kv_off + ((slot_off[b][l] * 2 * Hkv) + h * cap) * d * elem_size,
 * V rows at the same plus Hkv * cap * d * elem_size; kept indices of head h at
 *   idx_off + (slot_off[b][l] * Hkv + h * cap) * 4.   Appended slots hold index m + t.
 * FP8 caches: elem_size is 1, and the fp32 scale of the K row in slot r of head h sits at
 *   scale_off + (slot_off[b][l] * 2 * Hkv + h * cap + r) * 4, that of the V row Hkv * cap floats later. */
typedef struct {
    size_t status_off;     /* int32[4]: sticky vlc_status, request, layer, detail */
    size_t slot_off_off;   /* int64[B*L]: first slot of (b,l), in slots            */
    size_t kept_off;       /* int32[B*L]: validated k[b][l]                        */
    size_t kv_off;
    size_t idx_off;
    size_t scratch_off;
    size_t total_bytes;
    int64_t slots_per_request;
    size_t scale_off;      /* FP8 caches only */
    int32_t kv_fp8;        /* 1 if the rows are FP8 E4M3 codes */
    int32_t unit_slots, tail_unit_slots, layer_unit_slots;   /* the block-unit sizes in effect (see vlc_cache_options) */
    size_t appended_off;   /* int32[L]: appends each layer has received since the last compaction */
    /* The work lists the kernels walk, written by vlc_topk_compact: list 0 for decode launches over a layer range,
     * list 1 for decode launches over all layers, list 2 for the gather (it may be the same memory as list 0 or 1).
     * A list is an array of 64-byte records, one per block-unit of a cached row:
     *   int32 row ((b*L + l)*Hkv + kv head), first slot, kept (k[b][l]; 0 = rejected request), unit index in its row;
     *   int64 K slab offset (elements), int64 kept-index offset; int32 b, l, position in (layer, request, kv head, unit)
     *   order, slots of the unit, kv head, units of layer l in this list; 8 bytes of padding.
     * list_index_off[i] points at int32[L+2]: the position of each layer's first unit in that order, then the number of
     * units, then the number of whole unit_slots units.  With list_by_size[i] = 1 the records are stored by size class:
     * the whole units, then the other units that hold kept rows ((request, layer) entries with the most slots beyond
     * their whole units first), then the units that only hold append reserve; else in (layer, request, kv head, unit) order. */
    size_t list_items_off[3];
    size_t list_index_off[3];
    int32_t list_by_size[3];
    int32_t list_reserved;
} vlc_cache_layout;
vlc_status vlc_cache_get_layout(const vlc_cache* cache, vlc_cache_layout* out);

/* Synchronises the stream and returns the cache's sticky device-side status. */
vlc_status vlc_cache_status(vlc_cache* cache, vlc_stream stream);

/*
 * vlc_topk_compact -- token eviction (paper Sec. 2.2 top-k set; Sec. 4.2; App. A.4 copy of the
 * survivors into contiguous memory).  For every (b,l,hkv): keep the k[b][l] positions with the
 * largest score (ties to the lower position), in ascending position, and gather their K and
 * V rows into the cache.  With n_recent = r > 0 the last min(r, k) positions are kept
 * unconditionally and TopK fills the rest.  Resets the cache's decode step count to 0.
 *
 * scores  [B,L,Hkv,m] float  in
 * k       [B,L] int32        in (device; e.g. vlc_allocate's output), each in [1, m]
 * k_full, v_full [B,L,Hkv,m,d] in, storage dtype
 * idx_out [B,L,Hkv,m] int32  out, may be NULL: first k[b][l] entries of a row are the kept
 *                             positions, the rest are left untouched
 */
vlc_status vlc_topk_compact(vlc_cache* cache, const float* scores, const int32_t* k,
                            int32_t n_recent, const void* k_full, const void* v_full,
                            int32_t* idx_out, vlc_stream stream);

/*
 * vlc_topk_compact_recent_frac -- vlc_topk_compact with the forced recent window given as a
 * fraction of each layer's own budget (paper Sec. 5, implementation details: the recent window is
 * 10 % of the budget): n_recent[b][l] = floor(k[b][l] * recent_num / recent_den), computed on the
 * device from the same k array.  0 <= recent_num <= recent_den, recent_den >= 1
 * (VLC_ERR_INVALID_ARG otherwise); all other arguments, layouts and errors as vlc_topk_compact.
 */
vlc_status vlc_topk_compact_recent_frac(vlc_cache* cache, const float* scores, const int32_t* k,
                                        int32_t recent_num, int32_t recent_den, const void* k_full,
                                        const void* v_full, int32_t* idx_out, vlc_stream stream);

/*
 * vlc_cache_hit_rate -- CacheHitRate of paper Def. 3.1 for the set the cache holds.  For every
 * (b,l,hkv): S* = the k[b][l] positions with the largest scores_star (ties to the lower position,
 * no recent window), hits = |kept positions of the cache ∩ S*|, rate = hits / k[b][l].
 * scores_star is the attention of the first decode query over the m prompt keys, summed over the
 * query heads of the KV group: vlc_score on a shape with tau = 1 and q_win = that query computes it
 * (a one-row window placed at the last position sees every key).  Positions appended by decode steps
 * are not counted.
 *
 * scores_star [B,L,Hkv,m] float in;  hits_out [B,L,Hkv] int32 out;  rate_out [B,L,Hkv] float out or NULL.
 * VLC_ERR_INVALID_ARG if the cache has not been filled; rows of a rejected request report 0.
 */
vlc_status vlc_cache_hit_rate(vlc_cache* cache, const float* scores_star, int32_t* hits_out,
                              float* rate_out, vlc_stream stream);

/*
 * vlc_decode_attn -- one decode step of GQA attention over the compressed cache (paper
 * Sec. 2.1 decoding phase), for layers [layer_begin, layer_end).  If k_new != NULL the new
 * key/value of every (b, hkv) is appended first and attended; nothing is evicted.
 *
 *   out[l,b,h,:] = sum_r softmax_r(sm_scale[l] * <q[l,b,h,:], Kc[b,l,h/g,r,:]>) Vc[b,l,h/g,r,:]
 *
 * q            [layers in range, B, Hq, d]   in, storage dtype
 * k_new, v_new [layers in range, B, Hkv, d]  in, or both NULL (no append)
 * sm_scale     [L] float (indexed by absolute layer) or NULL for 1/sqrt(d)
 * out          [layers in range, B, Hq, d]   out, storage dtype
 * All layers of one call must have received the same number of appends so far
 * (VLC_ERR_INVALID_ARG otherwise); appending beyond T_max is VLC_ERR_CAPACITY.
 *
 * The number of appends a layer has received lives in the cache's device memory: the kernel reads it,
 * appends at slot k[b][l] + count and the launch leaves count + 1 behind.  A HIP graph that holds ONE
 * decode step (one call over all layers, or one call per layer) can therefore be replayed once per
 * generated token, with the new q / k_new / v_new written into the same buffers before each replay.
 * The host keeps a count of its own for the two errors above; it advances once per call, not per replay,
 * so replays are checked on the device only: a step beyond T_max attends without appending and sets the
 * cache's sticky status to VLC_ERR_CAPACITY (vlc_cache_status).  vlc_topk_compact resets both counts.
 */
vlc_status vlc_decode_attn(vlc_cache* cache, int32_t layer_begin, int32_t layer_end,
                           const void* q, const void* k_new, const void* v_new,
                           const float* sm_scale, void* out, vlc_stream stream);

/*
 * vlc_decode_attn_steps -- n_steps consecutive vlc_decode_attn calls (paper Sec. 2.1, one appended
 * token per step) enqueued from one C loop, for callers whose per-call overhead would otherwise
 * exceed the kernel time.  Step t uses slice t of every tensor:
 * q, out [n_steps, layers in range, B, Hq, d];  k_new, v_new [n_steps, layers in range, B, Hkv, d].
 * Same errors as vlc_decode_attn; steps enqueued before a failing one stay enqueued.
 */
vlc_status vlc_decode_attn_steps(vlc_cache* cache, int32_t layer_begin, int32_t layer_end, int32_t n_steps,
                                 const void* q, const void* k_new, const void* v_new,
                                 const float* sm_scale, void* out, vlc_stream stream);

/*
 * vlc_probe_read_stream -- measurement aid, not a step of the path: one kernel that reads `bytes` bytes of
 * device memory once (16-byte loads, eight per lane in flight, `blocks` blocks of 256 threads each reading a
 * contiguous share) and writes nothing.  The benchmark times it next to the decode launch, on a buffer of the
 * same size, to state what a pure read stream reaches on the device at hand (paper Sec. 2.1: decoding is
 * bound by the bytes of the cache it reads).  buf and bytes must be multiples of 16; sink is one uint32 of
 * device memory (practically never written).
 */
vlc_status vlc_probe_read_stream(const void* buf, size_t bytes, uint32_t* sink, int32_t blocks, vlc_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* VLCACHE_H */
