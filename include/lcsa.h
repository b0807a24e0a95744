/*
 * lcsa.h -- C ABI of the MI355X (gfx950) library for locality-constrained
 * block-sparse spatiotemporal attention, the self-attention of FlashVSR's
 * one-step streaming diffusion transformer (arXiv 2510.12747).
 *
 * One layer call for one chunk of latent frames is, in this order,
 *     lcsa_kv_cache_append   keys/values of the chunk join the sliding-window cache
 *     lcsa_pool_blocks       block means of the chunk's queries
 *     lcsa_select_blocks     coarse block map, spatial window, per-row top-k
 *     lcsa_sparse_attn_fwd   exact softmax attention on the kept block pairs
 *
 * General rules
 *   - Every pointer named "device" is GPU memory owned by the caller.  The
 *     library never allocates or frees device memory and never synchronises:
 *     each call validates its arguments on the host, enqueues kernels on the
 *     given stream (a hipStream_t passed as void*, NULL = default stream) and
 *     returns.  The number of visible frames advances on the host at enqueue time
 *     and the slot positions advance on the device in stream order, so all calls
 *     that touch one cache must be issued in program order on one stream.
 *   - HIP graphs: a sequence of calls recorded by stream capture replays correctly,
 *     chunk after chunk, provided the cache was FULL (valid frames = cache_frames)
 *     when it was recorded: from then on every layer call has the same arguments and
 *     launch shapes, and where the new frames go is decided on the device (sliding
 *     window: a ring position the append launch advances; importance policies: the
 *     slot table the eviction launch rewrites).  lcsa_kv_cache_append on a capturing
 *     stream with a cache that is not full returns LCSA_EUNSUPPORTED.  Replays do not
 *     move the host's copy of the ring position (lcsa_cache_frame_slot).
 *   - Tokens of a tensor are in raster order: token = (frame*grid_h + row)*grid_w + col.
 *     Element (token, head, c) of x is x[token*stride_tok + head*stride_head + c];
 *     strides are in elements, c is contiguous.  Base pointers must be 16-byte
 *     aligned and strides multiples of 16 bytes.
 *   - A block is tile_t consecutive frames x one tile_h x tile_w tile (Sec. 3.2 uses
 *     (2,8,8); tile_t = 1 gives single-frame tiles); tiles on the right and bottom
 *     edge of a grid the tile does not divide hold fewer (valid) tokens.  Frame counts
 *     (q_frames, cache_frames, every append) are multiples of tile_t; a "group" is
 *     tile_t consecutive frames.  nb = ceil(grid_h/tile_h)*ceil(grid_w/tile_w) blocks
 *     per group.  Block id = group*nb + tile_row*ceil(grid_w/tile_w) + tile_col.  For
 *     key blocks group 0 holds the OLDEST frames currently visible in the cache and the
 *     chunk's own frames come last; for query blocks group 0 starts the chunk.
 *   - Return value: LCSA_OK or a negative lcsa_status.  Nothing is enqueued
 *     when a call fails validation.  No call aborts, throws or prints.
 */
#ifndef LCSA_H
#define LCSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum lcsa_status {
    LCSA_OK = 0,
    LCSA_EINVAL = -1,       /* null pointer, non-positive size, bad stride/alignment, wrong state   */
    LCSA_EUNSUPPORTED = -2, /* valid request that no kernel of this build covers                    */
    LCSA_EHIP = -3          /* the HIP runtime reported an error at launch                          */
} lcsa_status;

enum { LCSA_F32 = 0, LCSA_BF16 = 1 };
enum { LCSA_WINDOW_TRUNCATED = 0, LCSA_WINDOW_PRESERVED = 1 };
/* KV-cache eviction (appendix on KV-cache eviction): sliding window (the paper's default), or by
 * importance, decided per head or once for all heads of the layer */
/* arithmetic of lcsa_sparse_attn_bwd: matrix cores where a kernel exists for the shape, or float FMA everywhere */
enum { LCSA_BWD_AUTO = 0, LCSA_BWD_FLOAT = 1 };
enum { LCSA_EVICT_SLIDING = 0, LCSA_EVICT_IMPORTANCE_HEADWISE = 1, LCSA_EVICT_IMPORTANCE_UNIFORM = 2 };

/* Problem geometry.  Plain data, passed by pointer, validated on every call. */
typedef struct lcsa_geom {
    int32_t heads;         /* attention heads                                                        */
    int32_t head_dim;      /* d; multiple of 8 (bf16) / 4 (f32), at most 256                         */
    int32_t grid_h;        /* latent tokens per frame: rows                                          */
    int32_t grid_w;        /*                          columns                                       */
    int32_t tile_h;        /* block = tile_t frames x tile_h x tile_w tokens (Sec. 3.2)              */
    int32_t tile_w;
    int32_t tile_t;        /* frames per block; divides q_frames and cache_frames                    */
    int32_t q_frames;      /* frames per chunk (queries)                                             */
    int32_t cache_frames;  /* sliding-window capacity in frames, the current chunk included          */
    int32_t radius_h;      /* local window: max distance of block centres in tokens, per axis;       */
    int32_t radius_w;      /*   negative = unbounded (Sec. 3.3)                                      */
    int32_t window_mode;   /* LCSA_WINDOW_TRUNCATED: window cut at the frame border;                 */
                           /* LCSA_WINDOW_PRESERVED: window keeps its size and slides inward (Fig. 3)*/
    int32_t topk;          /* key blocks kept per (head, query block) (Sec. 3.2)                     */
    int32_t dtype;         /* LCSA_F32 or LCSA_BF16: element type of Q, K, V, O and of the cache     */
} lcsa_geom;

/* ---- sliding-window KV cache (appendix "Discussion on Stream VSR Pipelines") ---------------- */

typedef struct lcsa_cache lcsa_cache; /* host-side handle; the storage it describes is the caller's */

/* Device bytes the caller must provide for one layer's cache; 0 if *geom is invalid. */
size_t lcsa_cache_device_bytes(const lcsa_geom *geom);

/*
 * Creates a handle over caller-owned device memory (256-byte aligned, at least
 * lcsa_cache_device_bytes(geom) bytes, contents irrelevant).  The cache starts empty.
 * Host-only call.  LCSA_EINVAL on bad geometry, misaligned or undersized memory.
 */
int32_t lcsa_cache_init(lcsa_cache **out, const lcsa_geom *geom, void *device_mem, size_t bytes);
/* Forgets all frames (start of a new video).  Host-only. */
int32_t lcsa_cache_reset(lcsa_cache *cache);
/* Frees the host handle; the device memory stays the caller's.  NULL is allowed. */
void lcsa_cache_free(lcsa_cache *cache);
/* Frames currently visible (0 .. cache_frames); negative status on NULL. */
int32_t lcsa_cache_valid_frames(const lcsa_cache *cache);
/*
 * Inspection helpers for tests.  Pooled keys live in the cache as float
 * [heads][(cache_frames/tile_t)*nb][head_dim], indexed by ring slot: the block `tile` of the
 * group that holds visible frame f (0 = oldest) is row lcsa_cache_frame_slot(cache, f)*nb + tile.
 */
const float *lcsa_cache_pooled_k_device(const lcsa_cache *cache);
int32_t lcsa_cache_frame_slot(const lcsa_cache *cache, int32_t frame);   /* sliding-window policy only; counts enqueued
                                                                            appends, not replays of a captured one */
/*
 * device uint32 [heads][(cache_frames/tile_t)*nb], by ring slot like the pooled keys: how many values of V
 * the append clamped to +-65504 when it stored that block (see lcsa_kv_cache_append; always 0 for layouts
 * that store V as given).  Entries of slots that hold no visible group are undefined.
 */
const uint32_t *lcsa_cache_v_clamped_device(const lcsa_cache *cache);

/*
 * Appends the keys and values of n_frames new frames (device, raster order, the cache's
 * dtype, shared strides) and evicts frames beyond the capacity: the oldest ones under
 * sliding-window eviction, the paper's default (see lcsa_cache_set_eviction for the alternative).  Also stores the block means of the new keys (Sec. 3.2
 * average pooling) for lcsa_select_blocks.  1 <= n_frames <= cache_frames, a multiple of tile_t.
 *
 * Range of V.  For bf16 with head_dim = 128 and 128-token blocks (the matrix-core path) V is stored as
 * IEEE half, which the second matrix product of lcsa_sparse_attn_fwd runs in: every bf16 value with
 * 2^-14 <= |v| <= 65280 is stored exactly; smaller magnitudes round to the nearest multiple of 2^-24
 * (absolute error at most 2^-25, zero below that); |v| >= 65536 and infinities are CLAMPED to +-65504 and
 * counted per block (lcsa_cache_v_clamped_device), NaN stays NaN.  Attention over clamped values is the
 * attention of eq. (1) on the clamped V.  Every other configuration stores V as given.
 */
int32_t lcsa_kv_cache_append(lcsa_cache *cache, const void *k, const void *v,
                             int64_t stride_tok, int64_t stride_head,
                             int32_t n_frames, void *stream);

/* ---- importance-based eviction (appendix on KV-cache eviction; a preliminary exploration there) --- */

/*
 * Chooses how lcsa_kv_cache_append makes room once the cache is full.  Allowed only while the
 * cache is empty (after init or reset), else LCSA_EINVAL.  Under an importance policy an entry
 * is one group of tile_t frames; an append that does not fit drops the visible groups with the
 * lowest importance (equal importance: the older group first; arriving groups are never
 * candidates), surviving groups stay in temporal order (key-block ids count in that order), and
 * the scores are forgotten.  Groups that were never scored count as 0, so without calls to
 * lcsa_block_importance the cache behaves like the sliding window.  HEADWISE: every head decides
 * for itself (heads may then hold different frames); UNIFORM: by the sum over heads, one decision.
 * The decision is taken on the device in stream order.  At most 64 groups of capacity
 * (LCSA_EUNSUPPORTED beyond).
 */
int32_t lcsa_cache_set_eviction(lcsa_cache *cache, int32_t policy);
int32_t lcsa_cache_eviction(const lcsa_cache *cache);
/*
 * Scores the visible groups from the coarse block-to-block attention map of the current chunk:
 * for every (head, query block) the softmax (eq. 1; scale <= 0 selects 1/sqrt(head_dim)) of the
 * pooled-Q . pooled-K scores (Sec. 3.2) over the key blocks inside the spatial window (Sec. 3.3);
 * the importance of a group is the attention its blocks receive, summed over the chunk's query
 * blocks.  Result: device float [heads][cache_frames/tile_t] indexed by visible group (0 =
 * oldest), kept inside the cache (lcsa_cache_importance_device) for the next append.  Call it
 * after the chunk's own append, with the pooled queries lcsa_select_blocks was given.
 */
int32_t lcsa_block_importance(const lcsa_geom *geom, const float *pooled_q, lcsa_cache *cache, float scale, void *stream);
/*
 * lcsa_block_importance for callers that cannot allocate or size a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): identical results, but the per-row partial sums live
 * in a static device array inside the library (1 MiB, held on every GPU the library runs on until the process
 * ends) instead of in the cache's own memory.  Allocates nothing.  Needs heads * n_qb * (cache_frames/tile_t)
 * <= 262144, else LCSA_EUNSUPPORTED.  Runs on the CURRENT device, to which the stream and all pointers must
 * belong.  Every call on one GPU uses the same array: calls that overlap on one GPU (different streams) race.
 */
int32_t lcsa_block_importance_static(const lcsa_geom *geom, const float *pooled_q, lcsa_cache *cache, float scale, void *stream);
/* Inspection helpers for tests: the scores above, and under an importance policy the device table
 * int32 [heads][cache_frames/tile_t], visible group (0 = oldest) -> slot (NULL under the sliding window,
 * where lcsa_cache_frame_slot answers on the host). */
const float *lcsa_cache_importance_device(const lcsa_cache *cache);
const int32_t *lcsa_cache_order_device(const lcsa_cache *cache);

/* ---- block pooling (Sec. 3.2: average pooling inside each block) ------------------------------ */

/*
 * pooled[head][group*nb + tile][c] = mean of x over the VALID tokens of the block
 * (device float [heads][(n_frames/tile_t)*nb][head_dim], written in full).  x: device,
 * geom->dtype; n_frames a multiple of tile_t.
 */
int32_t lcsa_pool_blocks(const lcsa_geom *geom, const void *x,
                         int64_t stride_tok, int64_t stride_head,
                         int32_t n_frames, float *pooled, void *stream);

/*
 * Rotary position embedding fused with the pooling, for the tensors on their way into this library (Q before
 * lcsa_select_blocks / lcsa_sparse_attn_fwd, K before lcsa_kv_cache_append): one pass over x instead of two.
 * Sec. 3.3 rests its local window on the relative formulation of RoPE; the paper does not print the channel
 * layout of its backbone, so the split is the caller's: the channels of a head are consecutive pairs
 * (2i, 2i+1); the first pairs_t pairs turn with the frame index first_frame + (frame within x), the next
 * pairs_h with the row, the last pairs_w with the column (pairs_t + pairs_h + pairs_w = head_dim/2); pair i of
 * an axis that owns n pairs turns by position * base^(-i/n) (base <= 0 selects 10000).
 *   x_rot    device, geom->dtype, own strides, may be x itself: the rotated tokens (float arithmetic, rounded
 *            to the element type)
 *   pooled   as lcsa_pool_blocks would compute it on x_rot, bit for bit
 * 0 <= first_frame, first_frame + n_frames <= 2^24.
 */
int32_t lcsa_rope_pool_blocks(const lcsa_geom *geom, const void *x, int64_t stride_tok, int64_t stride_head, int32_t n_frames,
                              int32_t pairs_t, int32_t pairs_h, int32_t pairs_w, float base, int32_t first_frame,
                              void *x_rot, int64_t rot_stride_tok, int64_t rot_stride_head, float *pooled, void *stream);

/* ---- block selection (Sec. 3.2 coarse map + top-k, Sec. 3.3 / Fig. 3 local window) ----------- */

/*
 * For every (head, query block qb): scores S = <pooled_q[qb], pooled_k[kb]> (float
 * accumulation) for every key block kb of every visible frame whose tile lies inside
 * qb's spatial window; keeps the m = min(topk, #admissible) best, equal scores going to
 * the lower key-block id.
 *   sel_idx  device int32 [heads][n_qb][topk], n_qb = (q_frames/tile_t)*nb: kept ids ascending, then -1
 *   sel_cnt  device int32 [heads][n_qb]: m
 *   gap      device float [heads][n_qb] or NULL: score of the weakest kept block
 *            minus the best admissible score left out (+inf if none is left out)
 * pooled_q: device float [heads][n_qb][head_dim] from lcsa_pool_blocks.
 * The cache must hold at least q_frames frames.  At most 8192 admissible key blocks
 * per row (LCSA_EUNSUPPORTED beyond).
 */
int32_t lcsa_select_blocks(const lcsa_geom *geom, const float *pooled_q, const lcsa_cache *cache,
                           int32_t *sel_idx, int32_t *sel_cnt, float *gap, void *stream);

/*
 * lcsa_pool_blocks and lcsa_select_blocks in one launch, for the chunk's queries (q: device,
 * geom->dtype, raster order over q_frames frames): every workgroup pools its own query block, with
 * the arithmetic of lcsa_pool_blocks (pooled_q, device float [heads][n_qb][head_dim], receives the
 * same values, bit for bit), then selects.  Saves one launch and the round trip of the pooled queries.
 * Arguments, limits and results otherwise as for the two calls.
 */
int32_t lcsa_pool_select_blocks(const lcsa_geom *geom, const void *q, int64_t q_stride_tok, int64_t q_stride_head,
                                const lcsa_cache *cache, float *pooled_q,
                                int32_t *sel_idx, int32_t *sel_cnt, float *gap, void *stream);

/* ---- block-sparse attention (Sec. 3.2: full attention on the kept pairs; eq. 1) --------------- */

/*
 * o[token][head][:] = sum_j softmax_j(q_token . k_j * scale) v_j over the valid tokens j of
 * the blocks sel_idx[head][block(token)][0 .. sel_cnt) (ids as produced against the cache's
 * CURRENT contents).  q, o: device, geom->dtype, raster order over the chunk's q_frames
 * frames, each with its own strides.  lse: device float [token][head] or NULL, natural
 * log of the softmax denominator.  scale <= 0 selects 1/sqrt(head_dim).  Products are
 * formed from the stored element type with float accumulation and a float online
 * softmax; on the matrix-core path probabilities and V enter the second product as IEEE half
 * (range of V: see lcsa_kv_cache_append).
 * Rows with sel_cnt = 0 produce zeros (lse = -inf).  Counts outside [0, topk] and ids outside the
 * visible blocks are clamped into range by the kernels (the row's result is then meaningless, but
 * nothing outside the cache is read).
 */
int32_t lcsa_sparse_attn_fwd(const lcsa_geom *geom,
                             const void *q, int64_t q_stride_tok, int64_t q_stride_head,
                             const lcsa_cache *cache,
                             const int32_t *sel_idx, const int32_t *sel_cnt,
                             void *o, int64_t o_stride_tok, int64_t o_stride_head,
                             float *lse, float scale, void *stream);

/* ---- backward of the block-sparse attention (Sec. 3.2 "Stage 2": the model is trained with it) --------- */

/*
 * Gradients of lcsa_sparse_attn_fwd with respect to q, k and v, the selection held fixed: the top-k choice is a
 * discrete decision and carries no gradient, so this is the backward of eq. (1) over the kept block pairs.
 *   q, d_o      device, geom->dtype, raster order over the chunk's q_frames frames, each with its own strides;
 *               d_o is the gradient of the loss with respect to the forward's output
 *   k, v        device, geom->dtype, raster order over the kv_frames frames that were visible at the forward,
 *               oldest first (the order key-block ids count in), shared strides; kv_frames a multiple of tile_t.
 *               They are read from these tensors, not from a cache: no cache is needed for a backward
 *   sel_idx, sel_cnt   as given to the forward;   lse: device float [token][head] as written by the forward
 *   d_q         device float [q_frames*grid_h*grid_w][heads][head_dim], contiguous
 *   d_k, d_v    device float [kv_frames*grid_h*grid_w][heads][head_dim], contiguous
 *   delta       device float [q_frames*grid_h*grid_w][heads]: receives D_i = sum_j p_ij (d_o_i . v_j), the quantity
 *               usually taken as d_o_i . o_i; it is formed from the kernel's own probabilities instead, because the
 *               forward's output rounded to bf16 would put a relative error of several 1e-3 into d_q and d_k
 * All results are written in full (zeros where no kept pair reaches).  scale <= 0 selects 1/sqrt(head_dim).
 * arithmetic = LCSA_BWD_AUTO: for bf16, head_dim 128 and 128-token blocks the products run on the matrix cores (bf16
 * operands, float accumulation; probabilities and their gradients are rounded to bf16 between the two levels of
 * products: results within a few 1e-3 of the largest gradient), every other shape in float FMA arithmetic.
 * LCSA_BWD_FLOAT: float FMA arithmetic for every shape (results within 2e-5 of the largest gradient; slow).
 * Either way the summation orders are fixed: results are reproducible bit for bit.
 * The float kernels return LCSA_EUNSUPPORTED if 2 * (tokens per block) * head_dim floats (a key block's
 * accumulators) exceed the LDS.
 */
int32_t lcsa_sparse_attn_bwd(const lcsa_geom *geom,
                             const void *q, int64_t q_stride_tok, int64_t q_stride_head,
                             const void *k, const void *v, int64_t kv_stride_tok, int64_t kv_stride_head, int32_t kv_frames,
                             const int32_t *sel_idx, const int32_t *sel_cnt,
                             const void *d_o, int64_t o_stride_tok, int64_t o_stride_head, const float *lse,
                             float *d_q, float *d_k, float *d_v, float *delta, float scale, int32_t arithmetic, void *stream);

/* Static, human-readable text for a status code. */
const char *lcsa_status_string(int32_t status);
/* Text of the last HIP error seen by this thread's most recent LCSA_EHIP ("" if none). */
const char *lcsa_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LCSA_H */
