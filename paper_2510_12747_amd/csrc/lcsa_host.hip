// C ABI of the library (see include/lcsa.h): argument validation, the host-side ring
// state of the sliding-window cache, and kernel dispatch.  No device allocation, no
// synchronisation, no host<->device copies happen here.
#include "../../include/lcsa.h"
#include "lcsa_kernels.h"
#include "lcsa_cache_handle.h"

#include <new>
#include <string>

using namespace lcsa;

namespace {

thread_local std::string g_last_hip_error;

int32_t hip_status(hipError_t e) {
    if (e == hipSuccess) return LCSA_OK;
    g_last_hip_error = hipGetErrorString(e);
    return LCSA_EHIP;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Is `stream` being recorded into a HIP graph?  (No GPU, or an error from the query: no.)
bool stream_is_capturing(hipStream_t stream) {
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &st) != hipSuccess) { (void)hipGetLastError(); return false; }
    return st != hipStreamCaptureStatusNone;
}

bool geom_ok(const lcsa_geom *g) {
    if (!g) return false;
    if (g->dtype != LCSA_F32 && g->dtype != LCSA_BF16) return false;
    const int vec = g->dtype == LCSA_BF16 ? 8 : 4;
    if (g->heads < 1 || g->head_dim < 1 || g->head_dim > 256 || g->head_dim % vec) return false;
    if (g->grid_h < 1 || g->grid_w < 1 || g->tile_h < 1 || g->tile_w < 1 || g->tile_t < 1) return false;
    if ((int64_t)g->tile_h * g->tile_w * g->tile_t > 1024) return false;
    if (g->q_frames < 1 || g->cache_frames < g->q_frames) return false;
    if (g->q_frames % g->tile_t || g->cache_frames % g->tile_t) return false;
    if (g->window_mode != LCSA_WINDOW_TRUNCATED && g->window_mode != LCSA_WINDOW_PRESERVED) return false;
    if (g->topk < 1) return false;
    // index arithmetic in the kernels is 32-bit for block ids and 64-bit for elements
    const int64_t ty = (g->grid_h + g->tile_h - 1) / g->tile_h, tx = (g->grid_w + g->tile_w - 1) / g->tile_w;
    if (ty * tx * g->cache_frames > (1 << 24)) return false;
    if (ty * tx * g->cache_frames * g->heads > (1ll << 30)) return false;      // one workgroup per (block, head) in a 1-D grid
    if ((int64_t)g->grid_h * g->grid_w * g->cache_frames > (1ll << 30)) return false;
    return true;
}

KGeom derive(const lcsa_geom &g) {
    KGeom k;
    k.heads = g.heads; k.d = g.head_dim;
    k.H = g.grid_h; k.W = g.grid_w; k.tt = g.tile_t; k.th = g.tile_h; k.tw = g.tile_w;
    k.ty = (g.grid_h + g.tile_h - 1) / g.tile_h;
    k.tx = (g.grid_w + g.tile_w - 1) / g.tile_w;
    k.nb = k.ty * k.tx;
    k.ts = g.tile_h * g.tile_w;
    k.bt = k.ts * g.tile_t;
    k.q_groups = g.q_frames / g.tile_t; k.cap = g.cache_frames / g.tile_t;
    k.rh = g.radius_h; k.rw = g.radius_w; k.wmode = g.window_mode;
    k.topk = g.topk;
    k.bf16 = g.dtype == LCSA_BF16;
    return k;
}

bool same_geom(const lcsa_geom *a, const lcsa_geom &b) {
    return a->heads == b.heads && a->head_dim == b.head_dim && a->grid_h == b.grid_h && a->grid_w == b.grid_w &&
           a->tile_h == b.tile_h && a->tile_w == b.tile_w && a->tile_t == b.tile_t && a->q_frames == b.q_frames &&
           a->cache_frames == b.cache_frames && a->dtype == b.dtype;
}

struct Layout { size_t k_off, v_off, pooled_off, order_off, imp_off, row_group_off, ring_off, clamped_off, total; };

Layout cache_layout(const KGeom &k) {
    const size_t elt = k.bf16 ? 2 : 4;
    const size_t tiles = (size_t)k.heads * k.cap * k.nb;
    const size_t kv = align_up(tiles * k.bt * k.d * elt, 256);
    Layout l;
    l.k_off = 0;
    l.v_off = kv;
    l.pooled_off = 2 * kv;
    l.order_off = l.pooled_off + align_up(tiles * k.d * sizeof(float), 256);
    l.imp_off = l.order_off + align_up((size_t)k.heads * k.cap * sizeof(int32_t), 256);
    l.row_group_off = l.imp_off + align_up((size_t)k.heads * k.cap * sizeof(float), 256);
    l.ring_off = l.row_group_off + align_up((size_t)k.heads * k.q_groups * k.nb * k.cap * sizeof(float), 256);
    l.clamped_off = l.ring_off + 256;
    l.total = l.clamped_off + align_up(tiles * sizeof(uint32_t), 256);
    return l;
}

bool tensor_ok(const void *p, int64_t st, int64_t sh, const KGeom &k) {
    const int vec = k.bf16 ? 8 : 4;
    if (!p || ((uintptr_t)p & 15)) return false;
    if (st < k.d || sh < k.d || st % vec || sh % vec) return false;
    return true;
}

} // namespace

extern "C" {

size_t lcsa_cache_device_bytes(const lcsa_geom *geom) {
    if (!geom_ok(geom)) return 0;
    return cache_layout(derive(*geom)).total;
}

int32_t lcsa_cache_init(lcsa_cache **out, const lcsa_geom *geom, void *device_mem, size_t bytes) {
    if (!out || !geom_ok(geom) || !device_mem || ((uintptr_t)device_mem & 255)) return LCSA_EINVAL;
    KGeom kg = derive(*geom);
    Layout l = cache_layout(kg);
    if (bytes < l.total) return LCSA_EINVAL;
    lcsa_cache *c = new (std::nothrow) lcsa_cache;
    if (!c) return LCSA_EINVAL;
    c->geom = *geom;
    c->kg = kg;
    c->bytes = bytes;
    char *base = (char *)device_mem;
    c->kc.k = base + l.k_off;
    c->kc.v = base + l.v_off;
    c->kc.pooled = (float *)(base + l.pooled_off);
    c->kc.v_clamped = (uint32_t *)(base + l.clamped_off);
    c->kc.ring = (int32_t *)(base + l.ring_off);
    c->start = 0;
    c->kc.valid = 0;
    c->kc.mfma_layout = kg.bf16 && kg.d == 128 && kg.bt == 128;
    c->kc.order = nullptr;
    c->policy = LCSA_EVICT_SLIDING;
    c->order = (int32_t *)(base + l.order_off);
    c->importance = (float *)(base + l.imp_off);
    c->row_group = (float *)(base + l.row_group_off);
    c->scored = false;
    *out = c;
    return LCSA_OK;
}

int32_t lcsa_cache_reset(lcsa_cache *cache) {
    if (!cache) return LCSA_EINVAL;
    cache->start = 0;
    cache->kc.valid = 0;
    cache->scored = false;
    return LCSA_OK;
}

void lcsa_cache_free(lcsa_cache *cache) { delete cache; }

int32_t lcsa_cache_set_eviction(lcsa_cache *cache, int32_t policy) {
    if (!cache || cache->kc.valid != 0) return LCSA_EINVAL;
    if (policy != LCSA_EVICT_SLIDING && policy != LCSA_EVICT_IMPORTANCE_HEADWISE && policy != LCSA_EVICT_IMPORTANCE_UNIFORM)
        return LCSA_EINVAL;
    if (policy != LCSA_EVICT_SLIDING && cache->kg.cap > kMaxEvictGroups) return LCSA_EUNSUPPORTED;
    cache->policy = policy;
    cache->kc.order = policy == LCSA_EVICT_SLIDING ? nullptr : cache->order;
    cache->start = 0;
    return LCSA_OK;
}

int32_t lcsa_cache_eviction(const lcsa_cache *cache) { return cache ? cache->policy : (int32_t)LCSA_EINVAL; }

const int32_t *lcsa_cache_order_device(const lcsa_cache *cache) { return cache ? cache->kc.order : nullptr; }

const float *lcsa_cache_importance_device(const lcsa_cache *cache) { return cache ? cache->importance : nullptr; }

int32_t lcsa_cache_valid_frames(const lcsa_cache *cache) {
    return cache ? cache->kc.valid * cache->kg.tt : (int32_t)LCSA_EINVAL;
}

const float *lcsa_cache_pooled_k_device(const lcsa_cache *cache) { return cache ? cache->kc.pooled : nullptr; }

const uint32_t *lcsa_cache_v_clamped_device(const lcsa_cache *cache) { return cache ? cache->kc.v_clamped : nullptr; }

int32_t lcsa_cache_frame_slot(const lcsa_cache *cache, int32_t frame) {
    if (!cache || frame < 0 || frame >= cache->kc.valid * cache->kg.tt) return LCSA_EINVAL;
    if (cache->policy != LCSA_EVICT_SLIDING) return LCSA_EINVAL;      // per head, on the device: lcsa_cache_order_device
    return slot_of_frame(cache->start, cache->kg.cap, frame / cache->kg.tt);
}

int32_t lcsa_kv_cache_append(lcsa_cache *cache, const void *k, const void *v,
                             int64_t stride_tok, int64_t stride_head, int32_t n_frames, void *stream) {
    if (!cache) return LCSA_EINVAL;
    const KGeom &kg = cache->kg;
    if (n_frames < 1 || n_frames % kg.tt || n_frames / kg.tt > kg.cap) return LCSA_EINVAL;
    if (!tensor_ok(k, stride_tok, stride_head, kg) || !tensor_ok(v, stride_tok, stride_head, kg)) return LCSA_EINVAL;
    if ((int64_t)n_frames * kg.H * kg.W > (1ll << 30)) return LCSA_EINVAL;
    KCache &kc = cache->kc;
    const int n_groups = n_frames / kg.tt;
    const int evict = kc.valid + n_groups > kg.cap ? kc.valid + n_groups - kg.cap : 0;
    // The number of visible groups travels by value in every launch, so a captured call replays correctly only
    // if that number no longer changes: the cache must be full when it is recorded.
    if (kc.valid != kg.cap && stream_is_capturing((hipStream_t)stream)) return LCSA_EUNSUPPORTED;
    if (cache->policy != LCSA_EVICT_SLIDING) {
        // The least important visible groups make room (per head, or for all heads alike); the table of
        // slots is rewritten on the device, in stream order, before the tiles are written.
        hipError_t e = launch_evict(kg, cache->order, cache->importance, kc.valid, n_groups, evict,
                                    cache->policy == LCSA_EVICT_IMPORTANCE_UNIFORM, cache->scored, (hipStream_t)stream);
        if (e != hipSuccess) return hip_status(e);
        cache->scored = false;
        e = launch_append(kg, kc, k, v, stride_tok, stride_head, n_groups, kc.valid - evict, false, (hipStream_t)stream);
        if (e != hipSuccess) return hip_status(e);
        kc.valid = kc.valid - evict + n_groups;
        return LCSA_OK;
    }
    // New groups go into the slots right after the newest one; once the ring is full those are the slots of
    // the oldest groups, which thereby leave the window.  The position is a device word that the launch
    // itself advances; the first append into an empty cache initialises it.
    hipError_t e = launch_append(kg, kc, k, v, stride_tok, stride_head, n_groups, 0, kc.valid == 0, (hipStream_t)stream);
    if (e != hipSuccess) return hip_status(e);
    cache->start = slot_of_frame(cache->start, kg.cap, evict);
    kc.valid = kc.valid + n_groups - evict;
    return LCSA_OK;
}

int32_t lcsa_pool_blocks(const lcsa_geom *geom, const void *x, int64_t stride_tok, int64_t stride_head,
                         int32_t n_frames, float *pooled, void *stream) {
    if (!geom_ok(geom) || !pooled || n_frames < 1 || n_frames % geom->tile_t) return LCSA_EINVAL;
    KGeom kg = derive(*geom);
    if (!tensor_ok(x, stride_tok, stride_head, kg)) return LCSA_EINVAL;
    if ((int64_t)n_frames * kg.H * kg.W > (1ll << 30)) return LCSA_EINVAL;
    return hip_status(launch_pool(kg, x, stride_tok, stride_head, n_frames / kg.tt, pooled, (hipStream_t)stream));
}

int32_t lcsa_rope_pool_blocks(const lcsa_geom *geom, const void *x, int64_t stride_tok, int64_t stride_head, int32_t n_frames,
                              int32_t pairs_t, int32_t pairs_h, int32_t pairs_w, float base, int32_t first_frame,
                              void *x_rot, int64_t rot_stride_tok, int64_t rot_stride_head, float *pooled, void *stream) {
    if (!geom_ok(geom) || !pooled || n_frames < 1 || n_frames % geom->tile_t) return LCSA_EINVAL;
    KGeom kg = derive(*geom);
    if (!tensor_ok(x, stride_tok, stride_head, kg) || !tensor_ok(x_rot, rot_stride_tok, rot_stride_head, kg)) return LCSA_EINVAL;
    if ((int64_t)n_frames * kg.H * kg.W > (1ll << 30)) return LCSA_EINVAL;
    if (pairs_t < 0 || pairs_h < 0 || pairs_w < 0 || 2 * ((int64_t)pairs_t + pairs_h + pairs_w) != kg.d) return LCSA_EINVAL;
    if (first_frame < 0 || (int64_t)first_frame + n_frames > (1 << 24)) return LCSA_EINVAL;     // positions are exact in float
    if (!(base > 0.f)) base = 10000.f;
    return hip_status(launch_rope_pool(kg, x, stride_tok, stride_head, n_frames / kg.tt, pairs_t, pairs_h, base, first_frame,
                                       x_rot, rot_stride_tok, rot_stride_head, pooled, (hipStream_t)stream));
}

int32_t lcsa_select_blocks(const lcsa_geom *geom, const float *pooled_q, const lcsa_cache *cache,
                           int32_t *sel_idx, int32_t *sel_cnt, float *gap, void *stream) {
    if (!geom_ok(geom) || !cache || !pooled_q || !sel_idx || !sel_cnt) return LCSA_EINVAL;
    if (!same_geom(geom, cache->geom)) return LCSA_EINVAL;
    if (cache->kc.valid * geom->tile_t < geom->q_frames) return LCSA_EINVAL;
    KGeom kg = derive(*geom);   // window, top-k may differ from the cache's own copy
    const int mc = max_candidates(kg, cache->kc.valid);
    if (mc > 8192) return LCSA_EUNSUPPORTED;
    return hip_status(launch_select(kg, cache->kc, pooled_q, sel_idx, sel_cnt, gap, mc, (hipStream_t)stream));
}

int32_t lcsa_pool_select_blocks(const lcsa_geom *geom, const void *q, int64_t q_stride_tok, int64_t q_stride_head,
                                const lcsa_cache *cache, float *pooled_q, int32_t *sel_idx, int32_t *sel_cnt, float *gap,
                                void *stream) {
    if (!geom_ok(geom) || !cache || !pooled_q || !sel_idx || !sel_cnt) return LCSA_EINVAL;
    if (!same_geom(geom, cache->geom)) return LCSA_EINVAL;
    if (cache->kc.valid * geom->tile_t < geom->q_frames) return LCSA_EINVAL;
    KGeom kg = derive(*geom);
    if (!tensor_ok(q, q_stride_tok, q_stride_head, kg)) return LCSA_EINVAL;
    if ((int64_t)geom->q_frames * kg.H * kg.W > (1ll << 30)) return LCSA_EINVAL;
    const int mc = max_candidates(kg, cache->kc.valid);
    if (mc > 8192) return LCSA_EUNSUPPORTED;
    return hip_status(launch_pool_select(kg, cache->kc, q, q_stride_tok, q_stride_head, pooled_q, sel_idx, sel_cnt, gap, mc,
                                         (hipStream_t)stream));
}

int32_t lcsa_block_importance(const lcsa_geom *geom, const float *pooled_q, lcsa_cache *cache, float scale, void *stream) {
    if (!geom_ok(geom) || !cache || !pooled_q) return LCSA_EINVAL;
    if (!same_geom(geom, cache->geom)) return LCSA_EINVAL;
    if (cache->kc.valid * geom->tile_t < geom->q_frames) return LCSA_EINVAL;
    KGeom kg = derive(*geom);   // the window may differ from the cache's own copy
    const int mc = max_candidates(kg, cache->kc.valid);
    if (mc > 8192 || kg.cap > 1024) return LCSA_EUNSUPPORTED;
    if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)kg.d);
    const hipError_t e = launch_importance(kg, cache->kc, pooled_q, scale, cache->row_group, cache->importance, mc,
                                           (hipStream_t)stream);
    if (e == hipSuccess) cache->scored = true;
    return hip_status(e);
}

int32_t lcsa_block_importance_static(const lcsa_geom *geom, const float *pooled_q, lcsa_cache *cache, float scale, void *stream) {
    if (!geom_ok(geom) || !cache || !pooled_q) return LCSA_EINVAL;
    if (!same_geom(geom, cache->geom)) return LCSA_EINVAL;
    KGeom kg = derive(*geom);
    // the limit of the static array is a property of the geometry: checked before the state of the cache
    if ((int64_t)kg.heads * kg.q_groups * kg.nb * kg.cap > kStaticScratchFloats) return LCSA_EUNSUPPORTED;
    if (cache->kc.valid * geom->tile_t < geom->q_frames) return LCSA_EINVAL;
    const int mc = max_candidates(kg, cache->kc.valid);
    if (mc > 8192 || kg.cap > 1024) return LCSA_EUNSUPPORTED;
    if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)kg.d);
    const hipError_t e = launch_importance_static(kg, cache->kc, pooled_q, scale, cache->importance, mc, (hipStream_t)stream);
    if (e == hipSuccess) cache->scored = true;
    return hip_status(e);
}

int32_t lcsa_sparse_attn_fwd(const lcsa_geom *geom, const void *q, int64_t q_stride_tok, int64_t q_stride_head,
                             const lcsa_cache *cache, const int32_t *sel_idx, const int32_t *sel_cnt,
                             void *o, int64_t o_stride_tok, int64_t o_stride_head,
                             float *lse, float scale, void *stream) {
    if (!geom_ok(geom) || !cache || !sel_idx || !sel_cnt) return LCSA_EINVAL;
    if (!same_geom(geom, cache->geom)) return LCSA_EINVAL;
    if (cache->kc.valid * geom->tile_t < geom->q_frames) return LCSA_EINVAL;
    KGeom kg = derive(*geom);
    if (!tensor_ok(q, q_stride_tok, q_stride_head, kg) || !tensor_ok(o, o_stride_tok, o_stride_head, kg))
        return LCSA_EINVAL;
    if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)kg.d);
    hipError_t e = cache->kc.mfma_layout
        ? launch_attn_mfma(kg, cache->kc, q, q_stride_tok, q_stride_head, sel_idx, sel_cnt,
                           o, o_stride_tok, o_stride_head, lse, scale, (hipStream_t)stream)
        : launch_attn_generic(kg, cache->kc, q, q_stride_tok, q_stride_head, sel_idx, sel_cnt,
                              o, o_stride_tok, o_stride_head, lse, scale, (hipStream_t)stream);
    return hip_status(e);
}

int32_t lcsa_sparse_attn_bwd(const lcsa_geom *geom, const void *q, int64_t q_stride_tok, int64_t q_stride_head,
                             const void *k, const void *v, int64_t kv_stride_tok, int64_t kv_stride_head, int32_t kv_frames,
                             const int32_t *sel_idx, const int32_t *sel_cnt,
                             const void *d_o, int64_t o_stride_tok, int64_t o_stride_head, const float *lse,
                             float *d_q, float *d_k, float *d_v, float *delta, float scale, int32_t arithmetic, void *stream) {
    if (!geom_ok(geom) || !sel_idx || !sel_cnt || !lse || !d_q || !d_k || !d_v || !delta) return LCSA_EINVAL;
    if (arithmetic != LCSA_BWD_AUTO && arithmetic != LCSA_BWD_FLOAT) return LCSA_EINVAL;
    KGeom kg = derive(*geom);
    if (kv_frames < geom->q_frames || kv_frames % kg.tt) return LCSA_EINVAL;
    if (!tensor_ok(q, q_stride_tok, q_stride_head, kg) || !tensor_ok(k, kv_stride_tok, kv_stride_head, kg) ||
        !tensor_ok(v, kv_stride_tok, kv_stride_head, kg) || !tensor_ok(d_o, o_stride_tok, o_stride_head, kg))
        return LCSA_EINVAL;
    const int kv_groups = kv_frames / kg.tt;
    if ((int64_t)kv_frames * kg.H * kg.W > (1ll << 30) || (int64_t)kv_groups * kg.nb * kg.heads > (1ll << 30)) return LCSA_EINVAL;
    if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)kg.d);
    if (arithmetic == LCSA_BWD_AUTO && attn_bwd_mfma_supported(kg))
        return hip_status(launch_attn_bwd_mfma(kg, kv_groups, q, q_stride_tok, q_stride_head, k, v, kv_stride_tok, kv_stride_head,
                                               sel_idx, sel_cnt, d_o, o_stride_tok, o_stride_head, lse, d_q, d_k, d_v, delta, scale,
                                               (hipStream_t)stream));
    if (!attn_bwd_supported(kg)) return LCSA_EUNSUPPORTED;
    return hip_status(launch_attn_bwd(kg, kv_groups, q, q_stride_tok, q_stride_head, k, v, kv_stride_tok, kv_stride_head,
                                      sel_idx, sel_cnt, d_o, o_stride_tok, o_stride_head, lse, d_q, d_k, d_v, delta, scale,
                                      (hipStream_t)stream));
}

const char *lcsa_status_string(int32_t status) {
    switch (status) {
    case LCSA_OK: return "ok";
    case LCSA_EINVAL: return "invalid argument";
    case LCSA_EUNSUPPORTED: return "unsupported configuration";
    case LCSA_EHIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

const char *lcsa_last_hip_error(void) { return g_last_hip_error.c_str(); }

} // extern "C"
