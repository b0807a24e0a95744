// Internal interface between the C-ABI host layer and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lcsa {

// Geometry as the kernels see it (derived once per call on the host).
struct KGeom {
    int heads, d;
    int H, W;          // token grid per frame
    int tt, th, tw;    // block shape: frames x rows x cols
    int ty, tx, nb;    // spatial tiles per frame: rows, cols, total (= blocks per group of tt frames)
    int ts, bt;        // tokens per full spatial tile = th*tw, per full block = tt*ts
    int q_groups, cap; // chunk length and ring capacity, both in groups of tt frames
    int rh, rw, wmode;
    int topk;
    int bf16;          // element type of Q,K,V,O and cache: 1 = bf16, 0 = f32
};

// Ring cache as the kernels see it.
//   K tiles : [heads][cap][nb][tile image]   element type = geometry dtype; cap ring slots, one per group
//   V tiles : same extent
//   pooled  : float [heads][cap*nb][d], indexed by ring slot
// Tokens of a block are ordered (frame in group, tile row, tile col) over the block's valid extent:
// a clipped block holds its valid tokens first and padding after them.
// Tile image, generic layout: K and V row-major [bt][d], padded tokens zero.
// Tile image, matrix-core layout (bf16, d = 128, bt = 128): 128 rows of 256 bytes,
//   the 16-byte chunk j of row r stored at chunk position j ^ (r & 15);
//   K rows = tile tokens (contents: d), V rows = channels (contents: tile tokens),
//   i.e. V is stored transposed, and converted to IEEE half.  Padded tokens are zero in both.
struct KCache {
    void *k, *v;
    float *pooled;
    uint32_t *v_clamped;   // [heads][cap*nb] by ring slot: V values of the block that the matrix-core layout clamped to half's range
    // Sliding-window eviction: two device words.  ring[0] = slot the next appended group goes to (so the oldest
    // visible group sits `valid` slots before it); ring[1] = arrival counter of the append launch in flight.
    // Only the append kernels write them, in stream order, which is what lets a captured layer call replay.
    int32_t *ring;
    int valid;   // visible groups
    int mfma_layout;
    // importance-based eviction: device table [heads][cap], visible group (0 = oldest) -> slot, per head;
    // null under sliding-window eviction, where the slot follows from ring[0]
    const int32_t *order;
};

__host__ __device__ inline int slot_of_frame(int start, int cap, int f) {
    int s = start + f;
    return s >= cap ? s - cap : s;
}

// Ring slot of the oldest visible group under sliding-window eviction; read once per kernel (no kernel that
// reads it runs while an append on the same stream is still writing it).
__device__ inline int ring_start(const KCache &c, const KGeom &g) {
    if (c.order) return 0;
    const int s = c.ring[0] - c.valid;
    return s < 0 ? s + g.cap : s;
}

// Slot that holds visible group f (0 = oldest) of a head; start = ring_start(c, g).
__device__ inline int cache_slot(const KCache &c, const KGeom &g, int start, int head, int f) {
    return c.order ? c.order[head * g.cap + f] : slot_of_frame(start, g.cap, f);
}

// Block token i -> (frame within the group, row, col inside the tile) of a tile clipped to vh x vw.
// The valid tokens of a block come first, in (frame, row, col) order over the clipped extent;
// positions tt*vh*vw .. bt-1 are padding (false is returned for them).
__host__ __device__ inline bool block_token(const KGeom &g, int i, int vh, int vw, int &ft, int &r, int &c) {
    const int per_frame = vh * vw;
    ft = i / per_frame;
    const int rem = i - ft * per_frame;
    r = rem / vw;
    c = rem - r * vw;
    return i < g.tt * per_frame;
}
// block_token for many tokens of one block: the two divisions become multiplications by reciprocals prepared once
// per block.  q = (i * ceil(2^32 / d)) >> 32 equals i / d for i < 65536 and 2 <= d <= 32768 (a block has at most
// 1024 tokens); d = 1 is passed through.
struct BlockTokens {
    uint32_t m_frame, m_row;
    int per_frame, vw, n_valid;
    __device__ BlockTokens(const KGeom &g, int vh, int vw_) : per_frame(vh * vw_), vw(vw_), n_valid(g.tt * vh * vw_) {
        m_frame = 0xFFFFFFFFu / (uint32_t)per_frame + 1u;
        m_row = 0xFFFFFFFFu / (uint32_t)vw + 1u;
    }
    __device__ bool at(int i, int &ft, int &r, int &c) const {
        ft = per_frame == 1 ? i : (int)__umulhi((uint32_t)i, m_frame);
        const int rem = i - ft * per_frame;
        r = vw == 1 ? rem : (int)__umulhi((uint32_t)rem, m_row);
        c = rem - r * vw;
        return i < n_valid;
    }
};
// Raster token index of (group, frame in group, absolute row, absolute col).
__host__ __device__ inline int64_t raster_token(const KGeom &g, int group, int ft, int row, int col) {
    return ((int64_t)(group * g.tt + ft) * g.H + row) * g.W + col;
}

// Every launcher enqueues on `stream` and returns hipGetLastError().
hipError_t launch_pool(const KGeom &g, const void *x, int64_t stride_tok, int64_t stride_head,
                       int n_groups, float *pooled, hipStream_t stream);

// Rotary position embedding per (frame, row, column) axis + block pooling of the rotated tokens in one pass;
// pairs_t + pairs_h + pairs_w = d/2 channel pairs; x_rot may be x itself.
hipError_t launch_rope_pool(const KGeom &g, const void *x, int64_t st, int64_t sh, int n_groups,
                            int pairs_t, int pairs_h, float base, int first_frame,
                            void *x_rot, int64_t rot_st, int64_t rot_sh, float *pooled, hipStream_t stream);

// Writes n_groups groups of frames: tiles of K, V and pooled K.  Importance-based eviction (c.order set):
// group i into the slot that c.order gives visible group first + i of each head.  Sliding window (c.order
// null): into ring slots ring[0].. (mod cap), and the launch advances ring[0] by n_groups once every
// workgroup has read it; fresh = the cache is empty and the ring words hold nothing yet: the groups go to
// slots 0.. and the words are initialised.
hipError_t launch_append(const KGeom &g, const KCache &c, const void *k, const void *v,
                         int64_t stride_tok, int64_t stride_head, int n_groups, int first, bool fresh,
                         hipStream_t stream);

// Importance of the visible groups from the coarse attention map of one chunk (appendix on KV-cache
// eviction): imp[heads][cap] by visible group; row_group is scratch [heads][n_qb][cap].
hipError_t launch_importance(const KGeom &g, const KCache &c, const float *pooled_q, float scale,
                             float *row_group, float *imp, int max_cand, hipStream_t stream);

// The same with the scratch in a static device array of kStaticScratchFloats floats that the library holds on
// every GPU it runs on (no caller memory beyond inputs and outputs); needs heads*n_qb*cap <= that many floats.
// Runs on the current device, to which `stream` must belong.
constexpr int kStaticScratchFloats = 1 << 18;
hipError_t launch_importance_static(const KGeom &g, const KCache &c, const float *pooled_q, float scale,
                                    float *imp, int max_cand, hipStream_t stream);

// Importance-based eviction before an append of n_new groups: drops the n_evict least important of the
// `valid` visible groups of every head (uniform: by the sum over heads), gives the arrivals the free
// slots, and rewrites order[heads][cap].  scored = false: imp is not read and every group counts as 0
// (oldest first).  cap <= kMaxEvictGroups.
constexpr int kMaxEvictGroups = 64;
hipError_t launch_evict(const KGeom &g, int32_t *order, const float *imp, int valid, int n_new, int n_evict,
                        bool uniform, bool scored, hipStream_t stream);

hipError_t launch_select(const KGeom &g, const KCache &c, const float *pooled_q,
                         int32_t *sel_idx, int32_t *sel_cnt, float *gap, int max_cand,
                         hipStream_t stream);

// The same with the pooling of the chunk's queries folded in: q is pooled per block (written to pooled_q too).
hipError_t launch_pool_select(const KGeom &g, const KCache &c, const void *q, int64_t q_st, int64_t q_sh, float *pooled_q,
                              int32_t *sel_idx, int32_t *sel_cnt, float *gap, int max_cand, hipStream_t stream);

hipError_t launch_attn_generic(const KGeom &g, const KCache &c, const void *q, int64_t q_st, int64_t q_sh,
                               const int32_t *sel_idx, const int32_t *sel_cnt,
                               void *o, int64_t o_st, int64_t o_sh, float *lse, float scale,
                               hipStream_t stream);

hipError_t launch_attn_mfma(const KGeom &g, const KCache &c, const void *q, int64_t q_st, int64_t q_sh,
                            const int32_t *sel_idx, const int32_t *sel_cnt,
                            void *o, int64_t o_st, int64_t o_sh, float *lse, float scale,
                            hipStream_t stream);

// Backward of the attention on the kept pairs (selection held fixed): d_q [q tokens][heads][d], d_k, d_v
// [kv_groups*tt*H*W][heads][d], float, contiguous, written in full.  k, v: raster tensors of the visible frames,
// oldest first; delta: float [q tokens][heads], receives D_i = sum_j p_ij (dO_i.v_j).  attn_bwd_supported: the key-block accumulators (2 * bt * d floats) must fit in LDS.
bool attn_bwd_supported(const KGeom &g);
hipError_t launch_attn_bwd(const KGeom &g, int kv_groups, const void *q, int64_t q_st, int64_t q_sh,
                           const void *k, const void *v, int64_t kv_st, int64_t kv_sh,
                           const int32_t *sel_idx, const int32_t *sel_cnt,
                           const void *d_o, int64_t o_st, int64_t o_sh, const float *lse,
                           float *d_q, float *d_k, float *d_v, float *delta, float scale, hipStream_t stream);

// The same on the matrix cores (bf16, d = 128, 128-token blocks, at most 8192 query blocks per chunk): products in
// bf16 with float accumulation, probabilities and their gradients rounded to bf16 between the two product levels.
bool attn_bwd_mfma_supported(const KGeom &g);
hipError_t launch_attn_bwd_mfma(const KGeom &g, int kv_groups, const void *q, int64_t q_st, int64_t q_sh,
                                const void *k, const void *v, int64_t kv_st, int64_t kv_sh,
                                const int32_t *sel_idx, const int32_t *sel_cnt,
                                const void *d_o, int64_t o_st, int64_t o_sh, const float *lse,
                                float *d_q, float *d_k, float *d_v, float *delta, float scale, hipStream_t stream);

// Largest number of admissible key blocks of any query block (host arithmetic).
int max_candidates(const KGeom &g, int valid_groups);

// Window of tile index b along one axis: [*lo, *hi).
__host__ __device__ inline void axis_window(int b, int tile, int n, int radius, int mode, int *lo, int *hi) {
    if (radius < 0) { *lo = 0; *hi = n; return; }
    int r = radius / tile;              // centres are (b + 1/2)*tile apart by whole tiles
    if (mode == 0) {
        *lo = b - r < 0 ? 0 : b - r;
        *hi = b + r + 1 > n ? n : b + r + 1;
    } else {
        int size = 2 * r + 1;
        if (size >= n) { *lo = 0; *hi = n; return; }
        int s = b - r;
        if (s < 0) s = 0;
        if (s > n - size) s = n - size;
        *lo = s; *hi = s + size;
    }
}

} // namespace lcsa

