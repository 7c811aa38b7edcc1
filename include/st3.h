/*
 * st3.h - C ABI of the ST3 attention / visual-token-trimming hot path for AMD MI355X (gfx950).
 *
 * The calls follow the problem statement of the ST3 paper (spatial-temporal visual token
 * trimming; Alg. 3, the KV-cache form of PVTP with VTA): per decoder layer, causal attention over a
 * sequence laid out [S, V, I, O] (Eq. 1) whose visual segment V shrinks over layers at prefill
 * (Progressive Visual Token Pruning, Eq. 3) and over decode steps (Visual Token Annealing,
 * Eq. 7-8), driven by the attention the last query row pays to each visual key (Sec. 3.2).
 *
 * Conventions (all entry points unless stated otherwise)
 *   - extern "C"; every pointer documented as DEVICE points to HIP device memory owned by the
 *     caller; every pointer documented as HOST is ordinary host memory.  The library never
 *     allocates or frees device memory and never synchronises: work is enqueued on `stream` (a
 *     hipStream_t passed as void*; NULL = the null stream) and results are valid once the caller
 *     has synchronised that stream.  Nothing a call computes is kept on the host between calls.
 *     What the library does keep, process-wide: the last HIP error (thread-local), per-device
 *     caches of device properties (compute units, resident workgroups per kernel build; written
 *     once, same value from every thread), the device address of the st3_decode_attention_noalloc
 *     array, and the diagnostic switches of the st3_debug_* / st3_profile_* block at the end of
 *     this header, which stay at their defaults unless ST3_DEBUG=1 was in the environment when
 *     the library was loaded.  Calls from several threads are safe as long as they do not share
 *     buffers.
 *   - Arguments are checked on the host before anything is enqueued.  On an error the call
 *     returns a non-zero st3_status and enqueues nothing.  A failed HIP launch returns
 *     ST3_ERR_HIP and st3_last_hip_error() gives the hipError_t (thread-local).
 *   - Element types: ST3_F32 (4 bytes) or ST3_BF16 (2 bytes, upper half of an IEEE float32).
 *     Arithmetic is float32 throughout; outputs are rounded to the element type (nearest even).
 *   - head_dim must be 64 or 128.  Rows of head_dim elements are contiguous and 16-byte aligned;
 *     strides are given in ELEMENTS unless a parameter says bytes.
 *   - Counts of kept tokens are integers chosen by the caller (see the schedule helpers below);
 *     no ratio is ever rounded on the device.
 */
#ifndef ST3_H
#define ST3_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Symbols below are the only ones the shared library exports. */
#define ST3_EXPORT __attribute__((visibility("default")))

typedef enum {
    ST3_OK = 0,
    ST3_ERR_INVALID_ARG = 1,        /* null pointer, negative size, k > n, length > capacity ... */
    ST3_ERR_UNSUPPORTED = 2,        /* head_dim / dtype / size outside what the kernels handle  */
    ST3_ERR_WORKSPACE_TOO_SMALL = 3,
    ST3_ERR_HIP = 4
} st3_status;

typedef enum { ST3_F32 = 0, ST3_BF16 = 1, ST3_E4M3 = 2 /* one byte; cache element of ST3_KV_E4M3, st3_kv_bytes only */ } st3_dtype;

/* How select-and-compact rearranges a layer's cache (see st3_select_compact_layer). */
typedef enum { ST3_STABLE = 0, ST3_HOLE_FILL = 1 } st3_compact_mode;

/* Attenuation function of Eq. 8 / Sec. 4.4, plus the fixed per-step drop used by the tiny case. */
typedef enum { ST3_ANNEAL_COS = 0, ST3_ANNEAL_LINEAR = 1, ST3_ANNEAL_EXP = 2, ST3_ANNEAL_DROP = 3,
               ST3_ANNEAL_NONE = 4 } st3_anneal_kind;

typedef struct {
    int32_t batch;          /* B  */
    int32_t heads;          /* H  (multi-head attention: as many KV heads as query heads) */
    int32_t head_dim;       /* d: 64 or 128 */
    int32_t dtype;          /* st3_dtype of q/k/v/out */
    float   softmax_scale;  /* logits are (q.k)*softmax_scale; 0 means 1/sqrt(d) (Eq. 2) */
} st3_attn_shape;

/* A [B, H, n, d] tensor on the DEVICE; element (b,h,t,c) at data + b*stride_b + h*stride_h + t*stride_t + c. */
typedef struct {
    void*   data;
    int64_t stride_b, stride_h, stride_t;
} st3_tensor4;

/* How a cache row is stored.  ST3_KV_PLAIN: d elements of shape->dtype.  ST3_KV_E4M3 (an
 * implementation variant of the KV cache of Sec. 4.3, not part of the paper): d bytes, each an OCP
 * FP8 E4M3 code (bias 7, no infinities, S.1111.111 = NaN, largest finite 448); the value of an
 * element of strip (b,h) is its code value times k_scale[b*H+h] (v_scale for V).  Rows enter such
 * a cache through st3_quantize_rows, st3_kv_append and the fused step calls, which divide by the
 * scale in float32, saturate at +-448 and round to nearest, ties to the even code.  Requires
 * shape->dtype == ST3_BF16. */
typedef enum { ST3_KV_PLAIN = 0, ST3_KV_E4M3 = 1 } st3_kv_format;

/* One layer's KV cache on the DEVICE: K and V share strides (in cache elements); `capacity` rows
 * exist per (b,h).  k_scale / v_scale: DEVICE float32 [B*H], positive, read only for ST3_KV_E4M3. */
typedef struct {
    void*   k;
    void*   v;
    int64_t stride_b, stride_h, stride_t;
    int32_t capacity;
    int32_t format;         /* st3_kv_format */
    const float* k_scale;
    const float* v_scale;
} st3_kv_layer;

/* Where the visual keys sit in a layer's cache.  For sequence b the cache holds rows up to
 * kv_len[b]; rows [sys_len, sys_len + vis_len[b]) are visual keys; everything else (system prompt,
 * instruction, generated tokens) is never pruned.  kv_len and vis_len live on the DEVICE because the
 * kernels update them; max_kv_len / max_vis_len are HOST-side upper bounds used to size launches and
 * to index the workspace (kv_len[b] <= max_kv_len <= capacity, vis_len[b] <= max_vis_len).
 * tail_start (DEVICE [B], may be NULL) chooses between two layouts of the rows behind the visual
 * segment (instruction + generated tokens, "the tail"):
 *   NULL      the tail follows the visual rows directly; an eviction closes the cache up again
 *             (up to two row moves per evicted row) and lowers kv_len[b];
 *   non-NULL  the tail starts at row tail_start[b] >= sys_len + vis_len[b] and stays there; rows
 *             [sys_len + vis_len[b], tail_start[b]) hold nothing and no call reads them.  An
 *             eviction only refills holes inside the visual segment (at most one row move per
 *             evicted row) and leaves kv_len[b], the END of the tail, alone.  Requires
 *             kv_len[b] >= tail_start[b].  Keys attended: kv_len[b] - (tail_start[b] - sys_len - vis_len[b]).
 * A prefill leaves [system | kept visual | instruction] contiguous, so tail_start[b] =
 * sys_len + vis_len[b] at that moment is where the fixed-tail layout begins.
 * vis_len_hint / tail_start_hint (HOST values; tail_start_hint <= 0: none) are the caller's guess at
 * the value most sequences have in vis_len[b] / tail_start[b] right now.  The decode attention
 * addresses its first loads with them while the device values are still on their way; a sequence
 * whose values differ has those loads repeated, so a wrong guess costs time and never changes a
 * result.  Ignored when tail_start is NULL. */
typedef struct {
    int32_t  sys_len;
    int32_t  max_vis_len;
    int32_t  max_kv_len;
    int32_t* vis_len;       /* DEVICE [B] */
    int32_t* kv_len;        /* DEVICE [B] */
    const int32_t* tail_start;  /* DEVICE [B] or NULL */
    int32_t  vis_len_hint;
    int32_t  tail_start_hint;
} st3_segments;

ST3_EXPORT const char* st3_status_string(st3_status s);
ST3_EXPORT int st3_last_hip_error(void);
ST3_EXPORT uint32_t st3_version(void);                 /* major<<16 | minor<<8 | patch */

/* Bytes of DEVICE workspace (256-byte aligned base expected) that any call below needs for a
 * layer whose cache has `kv_capacity` rows per (b,h), prefill sequences with at most max_vis_len
 * visual tokens and a score window of at most `score_window` rows.  The decode-path calls lay the
 * workspace out from the cache capacity alone. */
ST3_EXPORT size_t st3_workspace_bytes(const st3_attn_shape* shape, int32_t kv_capacity, int32_t max_vis_len,
                                      int32_t score_window);

/* Prepares a workspace for the decode-path calls: clears the per-sequence "mass pending"
 * descriptors (a few integers) with a small kernel on `stream`.  Required once before the first
 * st3_decode_layer_step / st3_select_compact_layer on a workspace that was not zero-filled.
 * Prefill scratch lives at the end of the workspace and never overlaps those descriptors. */
ST3_EXPORT st3_status st3_workspace_init(const st3_attn_shape* shape, int32_t kv_capacity, void* workspace,
                                         size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Prefill attention with visual-mass output (Eq. 2; score extraction of Sec. 3.2).
 *   out[b,h,i,:] = sum_{j<=i} softmax_j((q_i . k_j) * scale) v_j          for i in [0, n)
 *   vis_mass[b,j] = (1/H) sum_h sum_{i in last `score_window` rows} A_h[i, sys_len + j],  j in [0, vis_len)
 * q, k, v, out: DEVICE [B,H,n,d] with their own strides (k/v may point straight into a layer's
 * cache so that they become its first n rows).  vis_mass: DEVICE float32, row b at
 * vis_mass + b*mass_stride (mass_stride >= vis_len), may be NULL.
 * The paper takes the last row only (score_window = 1).  Requires 1 <= score_window <= min(n, 16),
 * sys_len + vis_len <= n <= 32768.
 * ------------------------------------------------------------------------------------------- */
ST3_EXPORT st3_status st3_prefill_attention(const st3_attn_shape* shape, const st3_tensor4* q, const st3_tensor4* k,
                                 const st3_tensor4* v, int32_t n, int32_t sys_len, int32_t vis_len,
                                 int32_t score_window, const st3_tensor4* out, float* vis_mass,
                                 int64_t mass_stride, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Writes rows [0, n) of a [B,H,n,d] tensor of shape->dtype into rows [0, n) of a cache's K
 * (which = 0) or V (which = 1) in the cache's own format: a copy for ST3_KV_PLAIN, the E4M3
 * quantiser described at st3_kv_format otherwise.  Used after prefill, whose attention runs on
 * the unquantised prompt.  n <= capacity.
 * ------------------------------------------------------------------------------------------- */
ST3_EXPORT st3_status st3_quantize_rows(const st3_attn_shape* shape, const st3_tensor4* src, const st3_kv_layer* kv,
                                        int32_t which, int32_t n, void* stream);

/* ---------------------------------------------------------------------------------------------
 * KV append (KV-cache use of Sec. 4.3): writes k_new/v_new (DEVICE, contiguous [B,H,d]) at row
 * kv_len[b] of the layer's cache, then kv_len[b] += 1.  Host check: max_kv_len < capacity.
 * A sequence with kv_len[b] >= capacity is left unchanged (device-side guard).
 * A layer that caches values only (a lazy layer of Alg. 2, which never forms K) passes
 * kv->k == NULL and k_new == NULL.
 * ------------------------------------------------------------------------------------------- */
ST3_EXPORT st3_status st3_kv_append(const st3_attn_shape* shape, const st3_kv_layer* kv, const st3_segments* seg,
                         const void* k_new, const void* v_new, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Decode attention with visual-mass output (Eq. 2 with one query row that follows every cached
 * key; score extraction of Sec. 3.2 applied to that row).
 *   out[b,h,:]   = sum_{j<kv_len[b]} p_j v_j,  p = softmax over the kv_len[b] cached keys
 *   vis_mass[b,j] = (1/H) sum_h p_h[sys_len + j],  j in [0, vis_len[b])
 * q, out: DEVICE contiguous [B,H,d].  vis_mass: DEVICE float32 with row stride `mass_stride`
 * (>= max_vis_len) or NULL; entries j >= vis_len[b] are left untouched.  The cache is read once;
 * when B*H alone does not fill the chip each (b,h) strip is cut into chunks handled by different
 * workgroups whose partial results a second kernel merges in a fixed order, so results are
 * reproducible run to run.
 * A sequence with kv_len[b] == 0 gets out = 0.
 * The call leaves the scaled logit of every cached key and the softmax normalisers in the
 * workspace (Alg. 2's attention cache U): st3_decode_attention_inherit reads them from there.
 * ------------------------------------------------------------------------------------------- */
ST3_EXPORT st3_status st3_decode_attention(const st3_attn_shape* shape, const void* q, const st3_kv_layer* kv,
                                const st3_segments* seg, void* out, float* vis_mass, int64_t mass_stride,
                                void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * st3_decode_attention for callers that cannot allocate device memory or hand over a workspace:
 * code that runs under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results and kernels as st3_decode_attention, without the workspace: the chunk
 * partials, logits and descriptors of the call live in a device array of
 * ST3_NOALLOC_SCRATCH_BYTES that is part of the library's code object (every GPU the process uses
 * holds one copy until the process ends).  The call allocates and frees nothing, on the host or
 * on the device.  A shape whose workspace (st3_workspace_bytes(shape, kv->capacity, 0, 1)) exceeds
 * the array returns ST3_ERR_WORKSPACE_TOO_SMALL and enqueues nothing; at the LLaVA-1.5-13B shape
 * (H = 40, d = 128) a batch of 64 sequences with 1251 cache rows each needs 15 MB.
 * All calls on one GPU share that GPU's array, which keeps whatever the last call left in it
 * (nothing in it has to be cleared between calls): two calls whose kernels may overlap on one GPU -
 * different streams, or different threads - race; serialise them.  What the call leaves in the
 * array is not available to st3_decode_attention_inherit.
 * ------------------------------------------------------------------------------------------- */
#define ST3_NOALLOC_SCRATCH_BYTES (32u << 20)
ST3_EXPORT st3_status st3_decode_attention_noalloc(const st3_attn_shape* shape, const void* q, const st3_kv_layer* kv,
                                                   const st3_segments* seg, void* out, float* vis_mass,
                                                   int64_t mass_stride, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Decode attention of a lazy layer (QK heredity, Eq. 6 and Alg. 2): the layer inherits the softmax
 * probabilities of its source layer l-n and applies them to its own values,
 *   out[b,h,:] = sum_{j<kv_len[b]} p^{src}_j v_j .
 * `src_workspace` is the workspace of the source layer's most recent st3_decode_attention (or
 * fused step) call, made with the same shape and for the same step; `src_kv_capacity` is the
 * capacity of the source layer's cache.  The lazy layer's cache must hold the same tokens in the
 * same row order as the source's did during that call (same lengths, same evictions applied
 * with the same ranking column).  Only kv->v is read (kv->k may be NULL): half the bytes of
 * st3_decode_attention.  The visual mass of a lazy layer is its source's and is not recomputed.
 * A sequence whose source call saw no keys gets out = 0.
 * ------------------------------------------------------------------------------------------- */
ST3_EXPORT st3_status st3_decode_attention_inherit(const st3_attn_shape* shape, const st3_kv_layer* kv,
                                                   const st3_segments* seg, const void* src_workspace,
                                                   size_t src_workspace_bytes, int32_t src_kv_capacity, void* out,
                                                   void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Top-k selection (Eq. 3: indices of the G highest scores).  Total order: higher score first,
 * then lower tie id first (tie_ids == NULL: the position itself).  -0.0 ranks equal to +0.0.
 *   scores:  DEVICE float32, row b at scores + b*score_stride, n_dev[b] valid entries
 *            (n_dev == NULL: every row has n entries).  n <= 16384.
 *   tie_ids: DEVICE int32 with row stride id_stride, distinct non-negative values per row, or NULL.
 *   k:       entries to keep; row b keeps min(k, n_b).
 *   keep_mask: DEVICE uint8 [B, n]  (1 = kept; entries >= n_b are written 0), may be NULL.
 *   keep_idx:  DEVICE int32, row b at keep_idx + b*idx_stride (idx_stride >= k): positions of the
 *              kept entries in ascending order, padded with -1 up to k entries; may be NULL.
 * ------------------------------------------------------------------------------------------- */
ST3_EXPORT st3_status st3_select_topk(const float* scores, int64_t score_stride, const int32_t* tie_ids, int64_t id_stride,
                           int32_t batch, const int32_t* n_dev, int32_t n, int32_t k,
                           uint8_t* keep_mask, int32_t* keep_idx, int64_t idx_stride, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Stable in-place row compaction (Alg. 1/3: V = V[T]; X = [S, V, I] rebuilt, order preserved).
 * For every (b, i) with b < batch, i < inner, on the strip that starts at
 * rows + b*stride_b_bytes + i*stride_inner_bytes:
 *   row[r] <- row[keep_idx[b][r]]   for r in [0, k_b)    (keep_idx row b at keep_idx + b*idx_stride,
 *                                                          ascending)
 *   row[k_b + j] <- row[n + j]      for j in [0, tail_rows)
 * where k_b <= k is the length of the leading run of entries inside [0, n): an index list is its
 * valid entries followed by padding (the -1 entries st3_select_topk appends for a row with fewer
 * than k candidates); whatever follows the first entry outside [0, n) is ignored.
 * Rows are row_bytes long (multiple of 4), stride_row_bytes apart.  Used for Q/K/V rows of a
 * layer's input, hidden rows, and the score / id columns (row_bytes = 4).
 * ------------------------------------------------------------------------------------------- */
ST3_EXPORT st3_status st3_compact_rows(void* rows, int32_t batch, int32_t inner, int64_t stride_b_bytes,
                            int64_t stride_inner_bytes, int64_t stride_row_bytes, int32_t row_bytes,
                            const int32_t* keep_idx, int64_t idx_stride, int32_t k, int32_t n, int32_t tail_rows,
                            void* stream);

/* ---------------------------------------------------------------------------------------------
 * Out-of-place gather of the rows a prune event keeps, for several tensors in ONE launch
 * (Alg. 1: V = V[T]; X = [S, V, I] - one index list applied to a layer's Q, K and V rows alike,
 * or to hidden rows of full width; Alg. 3, PVTP branch).  For every pair p < n_pairs, b < batch,
 * i < inner, on the strips src_p + b*src_stride_b + i*src_stride_inner and dst_p + ... alike:
 *   dst row r                 <- src row r                              r in [0, head_rows)
 *   dst row head_rows + j     <- src row head_rows + keep_idx[b][j]     j in [0, k)
 *   dst row head_rows + k + j <- src row head_rows + n + j              j in [0, tail_rows)
 * keep_idx: DEVICE int32, row b at keep_idx + b*idx_stride, entries in [0, n) (a destination row
 * whose entry lies outside is left untouched); NULL means the identity and requires k == n, which
 * makes the call a strided copy.  Rows are row_bytes long (multiple of 16); all strides are in
 * bytes and multiples of 16, all pointers 16-byte aligned; no dst strip may overlap a src strip.
 * At most ST3_MAX_GATHER pairs per call.
 * ------------------------------------------------------------------------------------------- */
#define ST3_MAX_GATHER 4
typedef struct {
    const void* src;
    int64_t     src_stride_b, src_stride_inner, src_stride_row;
    void*       dst;
    int64_t     dst_stride_b, dst_stride_inner, dst_stride_row;
} st3_gather_pair;
ST3_EXPORT st3_status st3_gather_rows(const st3_gather_pair* pairs, int32_t n_pairs, int32_t batch, int32_t inner,
                                      int32_t row_bytes, int32_t head_rows, const int32_t* keep_idx,
                                      int64_t idx_stride, int32_t k, int32_t n, int32_t tail_rows, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Select-and-compact for one layer at one decode step (Eq. 7: C_v <- C_v[: |V^{l,0}| * beta^t];
 * Alg. 3, VTA branch; eviction semantics of Sec. 4.3).  For every sequence b with
 * vis_len[b] > keep_count: ranks the layer's visual keys by score_col (total order of
 * st3_select_topk, ties by id_col), keeps the best keep_count, evicts the rest from K and V,
 * applies the same rearrangement to score_col and id_col, and updates vis_len[b] / kv_len[b].
 *   score_col: DEVICE float32, row stride col_stride; entry p ranks cache row sys_len + p.
 *   id_col:    DEVICE int32,  same layout; original visual token ids (distinct per row).
 *   mode ST3_STABLE:    survivors keep their relative order and the rows after the visual segment
 *                       move down by the number evicted (what a slice assignment would do).
 *   mode ST3_HOLE_FILL: survivors from the evicted tail of the segment move into the holes, and
 *                       the vacated end of the segment is refilled from the END of the cache, so
 *                       at most 2*(evicted) rows move.  Valid for decode only, where softmax
 *                       attention does not depend on the order of cached keys.
 * max_vis_len / max_kv_len in `seg` must bound the lengths BEFORE the call.
 * kv->k may be NULL for a layer that caches values only (lazy layer, Alg. 2).  The rearrangement
 * is a function of (score_col, id_col, lengths, keep_count, mode) alone, so layers that hold
 * equal columns end up with equal row orders.
 * ------------------------------------------------------------------------------------------- */
ST3_EXPORT st3_status st3_select_compact_layer(const st3_attn_shape* shape, const st3_kv_layer* kv, const st3_segments* seg,
                                    float* score_col, int32_t* id_col, int64_t col_stride, int32_t keep_count,
                                    int32_t mode, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * One layer of one decode step (Alg. 3, VTA branch):
 *   (1) append k_new/v_new and attend: q over the cache plus the new token, with visual mass;
 *   (2) count the appended row (kv_len[b] += 1) and select-and-compact down to `keep_after`
 *       visual rows, i.e. the eviction Alg. 3 performs at the START of the layer's NEXT step is
 *       done here, right after this step's attention (the cache is not touched in between, so
 *       the result is the same; keep_after < 0: no eviction).  The eviction that precedes the
 *       very first decode step is a stand-alone st3_select_compact_layer call.
 * Two kernels: the attention kernel reads the new token's row from k_new/v_new and stores it
 * into the cache while streaming K and V once; then one workgroup per sequence finishes the visual
 * mass (head reduction), ranks, evicts (moving the few affected rows itself) and publishes the
 * lengths.  max_* in `seg` bound the lengths BEFORE the call; host check: max_kv_len < capacity.
 * vis_mass (may be NULL: no mass) holds this step's mass, in the cache order the attention saw,
 * once the stream is synchronised.  With vis_mass == score_col the eviction ranks by that mass
 * (and compacts it along with id_col).  The workspace must be the layer's own (st3_workspace_init).
 * ------------------------------------------------------------------------------------------- */
ST3_EXPORT st3_status st3_decode_layer_step(const st3_attn_shape* shape, const st3_kv_layer* kv,
                                            const st3_segments* seg, float* score_col, int32_t* id_col,
                                            int64_t col_stride, int32_t keep_after, int32_t mode, const void* q,
                                            const void* k_new, const void* v_new, void* out, float* vis_mass,
                                            int64_t mass_stride, void* workspace, size_t workspace_bytes,
                                            void* stream);

/* ---------------------------------------------------------------------------------------------
 * One whole decode step over `n_layers` layers from a single host call (Alg. 3, VTA branch, the
 * loop over l).  `layers` is a HOST array; entry i carries exactly the arguments
 * st3_decode_layer_step takes for that layer.  The result is the same as calling
 * st3_decode_layer_step for i = 0 .. n_layers-1 in order.  Step (2) of a layer depends on that
 * layer's attention only, so all layers attend first (one launch each) and their steps (2) then
 * run side by side in one launch (up to 64 layers; each attention launch leaves its layer's
 * step-(2) arguments in the layer's workspace, where that launch reads them).  Every layer needs
 * buffers and a workspace of its own.
 * Lazy layers (inherit_from >= 0) are available through this call only: a group's evictions must
 * wait until its last lazy layer has attended, which the per-layer call cannot arrange.
 * ------------------------------------------------------------------------------------------- */
typedef struct {
    st3_kv_layer kv;
    st3_segments seg;
    float*       score_col;
    int32_t*     id_col;
    int64_t      col_stride;
    int32_t      keep_after;        /* visual rows to keep after this step's attention; < 0: all */
    int32_t      inherit_from;      /* < 0: ordinary layer.  Else this is a lazy layer (Eq. 6, Alg. 2) and the
                                       value is the index, in the same array and before this entry, of its
                                       source layer: q and k_new are ignored, kv.k may be NULL, the attention
                                       applies the source's probabilities of this step to kv.v and v_new.
                                       The source must be an ordinary layer with the same sys_len, max_*
                                       bounds and keep_after, and must pass a vis_mass of its own when
                                       this layer passes one; score_col/id_col/lengths are this layer's own
                                       copies and must equal the source's, so that both evict alike.
                                       vis_mass (may be NULL) receives the source's mass. */
    const void*  q;
    const void*  k_new;
    const void*  v_new;
    void*        out;
    float*       vis_mass;
    int64_t      mass_stride;
    void*        workspace;         /* this layer's own workspace */
    size_t       workspace_bytes;
} st3_layer_step;

ST3_EXPORT st3_status st3_decode_step(const st3_attn_shape* shape, int32_t n_layers, const st3_layer_step* layers,
                                      int32_t mode, void* stream);

/* ---------------------------------------------------------------------------------------------
 * The same step in the two parts a decoder with a data dependency between its layers can call
 * (Alg. 3, VTA branch: the loop over l visits the layers in order, and layer l+1's query exists
 * only once layer l's output does).
 *   st3_decode_layer_attend   part (1) of layer `layer` of the array: append k_new/v_new and attend
 *                             (a lazy layer: inherit from its source, which must have attended in
 *                             this step already).  Only that entry (and its source's) is read and
 *                             checked, plus inherit_from of the later entries, so the q / k_new /
 *                             v_new of later layers need not exist yet.  out is valid, and complete, as soon as
 *                             the stream has run the call; the visual mass stays pending in the
 *                             layer's workspace; kv_len[b] does not yet count the appended row.
 *   st3_decode_plans          part (2) of ALL layers, once per step after the last layer has
 *                             attended: finishes the masses, counts the appended rows, ranks and
 *                             evicts down to keep_after, 16 layers per launch.
 * Calling st3_decode_layer_attend for layer = 0 .. n_layers-1 and then st3_decode_plans, with the
 * same array, is what st3_decode_step does.  Between the first attend and the plans of a step the
 * arrays max_* bounds, keep_after and the buffers of every entry must stay as they are.
 * ------------------------------------------------------------------------------------------- */
ST3_EXPORT st3_status st3_decode_layer_attend(const st3_attn_shape* shape, int32_t n_layers, const st3_layer_step* layers,
                                              int32_t layer, int32_t mode, void* stream);
ST3_EXPORT st3_status st3_decode_plans(const st3_attn_shape* shape, int32_t n_layers, const st3_layer_step* layers,
                                       int32_t mode, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Retention schedules: HOST-only pure functions that fill integer tables.
 * ------------------------------------------------------------------------------------------- */

/* Strided progressive pruning (Sec. 3.2: layers 0..2 keep every visual token; Alg. 1: prune
 * events at layers l >= 3 with (l-3) % S == 0; Eq. 9 with P the first event's ratio and R each
 * later event's, both relative to the original count).  Ratios in basis points.  keep_l: HOST [L]. */
ST3_EXPORT st3_status st3_schedule_pvtp(int32_t L, int32_t n_vis, int32_t first_layer, int32_t stride_S,
                             int32_t P_bp, int32_t R_bp, int32_t* keep_l);

/* Keep ratio 1 up to last_full_layer, then falling linearly to end_ratio_bp at layer L-1. */
ST3_EXPORT st3_status st3_schedule_linear(int32_t L, int32_t n_vis, int32_t last_full_layer, int32_t end_ratio_bp,
                               int32_t* keep_l);

/* Eq. 7-8: keep_lt[l*(T+1) + t] = floor(keep_l0[l] * beta(t)), t = 0..T; beta per `kind` with
 * param = tau (COS, LINEAR), sigma (EXP) or tokens dropped per step (DROP).  HOST arrays. */
ST3_EXPORT st3_status st3_schedule_anneal(int32_t kind, double param, int32_t T, const int32_t* keep_l0, int32_t L,
                               int32_t* keep_lt);

/* KV-cache bytes held by `batch` sequences whose layer l caches kv_lens[l] keys (HOST array [L]). */
ST3_EXPORT int64_t st3_kv_bytes(int32_t batch, int32_t heads, int32_t head_dim, int32_t dtype, const int32_t* kv_lens,
                     int32_t L);

/* ---------------------------------------------------------------------------------------------
 * Diagnostics on score (mass) vectors, as the paper uses them to motivate the method.
 *
 * st3_overlap_topk - Eq. 10: overlap[b] = |TopK(a) ^ TopK(b)| and topk_a[b] = |TopK(a)|, where
 *   TopK(x) is the set of token ids of the k best entries of x under the order of st3_select_topk
 *   (Overlap_n is their quotient).  a and b are score vectors with id columns (DEVICE, row b at
 *   +b*stride, n_x_dev[b] valid entries or n_x when the pointer is NULL); they may hold different
 *   token sets in different orders, e.g. the same layer's mass at two decode steps.
 *   ids in [0, id_space), id_space <= 16384, n <= 8192.
 * st3_cosine_similarity - Eq. 4-5: cosine[b] = <a,b> / (|a| |b|), entries matched by token id
 *   (ids NULL: by position); a token missing on one side counts as zero there.  Zero vectors give 0.
 * ------------------------------------------------------------------------------------------- */
ST3_EXPORT st3_status st3_overlap_topk(const float* score_a, const int32_t* ids_a, int64_t stride_a,
                                       const int32_t* n_a_dev, int32_t n_a, const float* score_b,
                                       const int32_t* ids_b, int64_t stride_b, const int32_t* n_b_dev, int32_t n_b,
                                       int32_t batch, int32_t k, int32_t id_space, int32_t* overlap, int32_t* topk_a,
                                       void* stream);
ST3_EXPORT st3_status st3_cosine_similarity(const float* va, const int32_t* ids_a, int64_t stride_a,
                                            const int32_t* n_a_dev, int32_t n_a, const float* vb,
                                            const int32_t* ids_b, int64_t stride_b, const int32_t* n_b_dev,
                                            int32_t n_b, int32_t batch, int32_t id_space, float* cosine, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Diagnostic block.  Compiled into every build, inert by default: unless the environment held
 * ST3_DEBUG=1 when the library was loaded, every call below returns ST3_ERR_UNSUPPORTED and
 * changes nothing (st3_debug_enabled tells which).  The switches are process-wide and meant for
 * tests and benchmarks: set them while no other thread is inside a library call.
 *
 * st3_profile_enable(n) creates (host-side) hipEvents for up to n launches and makes the decode
 *   calls launch the decode attention kernel (the kernel that streams K and V) with an event pair
 *   attached that receives the kernel's own start and end on the caller's stream; this stops
 *   silently once n launches are used.
 * st3_profile_read waits for the recorded events, returns the summed / min / max kernel time in
 *   milliseconds and the number of launches timed, and switches recording off.  HOST pointers, any
 *   may be NULL.
 * st3_debug_set_prefill_path: which kernel st3_prefill_attention uses for bf16 inputs.  0 =
 *   automatic (MFMA kernel), 1 = the float32 row kernel, 2 = MFMA or fail.  Lets the two be
 *   compared on one input.
 * st3_debug_set_attend_tile: the decode attention kernel is built for several tile sizes (16-byte
 *   loads of K, and of V, per lane and tile) and picks one per launch from the launch's size.
 *   tile_loads != 0 makes every later launch use that build when the cache type has it (plain
 *   caches: 1, 4, 6, 8; E4M3: 1, 3, 4; any other value: automatic choice, as with 0).  Results do
 *   not depend on the tile size beyond float32 rounding order.
 * ------------------------------------------------------------------------------------------- */
ST3_EXPORT int st3_debug_enabled(void);
ST3_EXPORT st3_status st3_profile_enable(int32_t max_launches);
ST3_EXPORT st3_status st3_profile_read(double* total_ms, int64_t* launches, double* min_ms, double* max_ms);
ST3_EXPORT st3_status st3_debug_set_prefill_path(int path);
ST3_EXPORT st3_status st3_debug_set_attend_tile(int tile_loads);

#ifdef __cplusplus
}
#endif
#endif /* ST3_H */
