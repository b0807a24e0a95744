// Block selection: coarse block-to-block scores (Sec. 3.2) restricted to the spatial local
// window (Sec. 3.3, Fig. 3), then the per-row top-k with ties going to the lower key-block
// id.  One workgroup owns one (head, query block) row: four lanes share each dot product
// against an admissible key block, then one wavefront finds the k-th largest score by a 32-step
// bitwise search over order-preserving integer keys with ballot/popcount and emits the kept ids
// in ascending order with ballot prefix counts.  No sort, no atomics, fully deterministic.
#include "lcsa_kernels.h"
#include "lcsa_pool.h"

namespace lcsa {
namespace {

// Monotone map float -> uint32 (larger float = larger key); -0 is folded into +0 first so
// that equal floats always get equal keys.
__device__ inline uint32_t order_key(float s) {
    uint32_t u = __float_as_uint(s + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ inline float key_to_float(uint32_t key) {
    return __uint_as_float((key & 0x80000000u) ? (key ^ 0x80000000u) : ~key);
}

__device__ inline int wave_count(bool p) { return __popcll(__ballot(p)); }

constexpr int kSelThreads = 256;
static_assert(kSelThreads == pooling::kThreads, "the fused kernel pools with the pooling kernel's thread layout");

// VEC = 0: the pooled queries are given.  VEC = 8 (bf16) or 4 (f32): the kernel first pools its own query
// block from q, exactly as the pooling kernel would (same code, same summation order), and also writes
// the mean to pooled_out: one launch and one pass over Q less per layer call.
template <int VEC>
__global__ __launch_bounds__(kSelThreads) void select_kernel(KGeom g, KCache c, const float *__restrict__ pooled_q,
                                                             const char *__restrict__ x, int64_t st, int64_t sh,
                                                             float *__restrict__ pooled_out,
                                                             int32_t *__restrict__ sel_idx, int32_t *__restrict__ sel_cnt,
                                                             float *__restrict__ gap) {
    extern __shared__ float smem[];
    float *qs = smem;                                  // [d] pooled query of this row
    uint32_t *keys = (uint32_t *)(smem + g.d);         // [n] ordered keys of the admissible blocks (after pooling's partial sums)
    const int qb = blockIdx.x / g.heads, head = blockIdx.x - qb * g.heads;     // head-fastest, like the pooling kernels
    const int tid = threadIdx.x, lane = tid & 63;
    const int n_qb = g.q_groups * g.nb;
    const int tile = qb % g.nb, by = tile / g.tx, bx = tile - by * g.tx;
    int y0, y1, x0, x1;
    axis_window(by, g.th, g.ty, g.rh, g.wmode, &y0, &y1);
    axis_window(bx, g.tw, g.tx, g.rw, g.wmode, &x0, &x1);
    const int wx = x1 - x0, nwin = (y1 - y0) * wx;
    const int n = c.valid * nwin;                      // admissible key blocks, in ascending id order
    const int64_t row = (int64_t)head * n_qb + qb;
    const int start = ring_start(c, g);                // requested here, needed after the pooling

    if constexpr (VEC == 0) {
        for (int i = tid; i < g.d; i += kSelThreads) qs[i] = pooled_q[row * g.d + i];
    } else {
        float *red = smem + g.d;                       // [kSelThreads * VEC] partial sums per row group
        const pooling::TileRef t = pooling::tile_ref(g, qb);
        const int lpr = g.d / VEC, rows_par = kSelThreads / lpr;
        const int rg = tid / lpr, j = tid - rg * lpr;
        float acc[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
        if (rg < rows_par) {
            pooling::accumulate_block<VEC>(g, t, x, st, sh, head, rg, j, rows_par, acc);
#pragma unroll
            for (int e = 0; e < VEC; ++e) red[rg * g.d + j * VEC + e] = acc[e];
        }
        __syncthreads();
        const int count = g.tt * t.vh * t.vw;
        for (int ch = tid; ch < g.d; ch += kSelThreads) {
            float sum = 0.f;
            for (int r = 0; r < rows_par; ++r) sum += red[r * g.d + ch];
            const float mean = sum / (float)count;
            qs[ch] = mean;
            pooled_out[row * g.d + ch] = mean;
        }
    }
    __syncthreads();

    // candidate ci -> (visible group f, tile t); key-block id = f*nb + t grows with ci
    auto tile_of = [&](int ci, int &f) {
        f = ci / nwin;
        int w = ci - f * nwin, wy = w / wx;
        return (y0 + wy) * g.tx + x0 + (w - wy * wx);
    };

    // ---- scores: four lanes per candidate, each a quarter of the channels (interleaved float4s so
    // that the four lanes read one contiguous 64-byte piece at a time); all loads of a lane are
    // issued before the first FMA
    {
        const int part = tid & 3, n4 = g.d / 4;
        for (int ci = tid >> 2; ci < ((n + 63) & ~63); ci += kSelThreads / 4) {
            float s = 0.f;
            if (ci < n) {
                int f;
                const int t = tile_of(ci, f);
                const int slot = cache_slot(c, g, start, head, f);
                const float4 *kr = (const float4 *)(c.pooled + (((int64_t)head * g.cap + slot) * g.nb + t) * g.d);
                for (int e0 = part; e0 < n4; e0 += 4 * 16) {
                    float4 kk[16];
#pragma unroll
                    for (int u = 0; u < 16; ++u) kk[u] = e0 + 4 * u < n4 ? kr[e0 + 4 * u] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                    for (int u = 0; u < 16; ++u) {
                        const int e = (e0 + 4 * u < n4 ? e0 + 4 * u : 0) * 4;
                        s = fmaf(qs[e], kk[u].x, s);
                        s = fmaf(qs[e + 1], kk[u].y, s);
                        s = fmaf(qs[e + 2], kk[u].z, s);
                        s = fmaf(qs[e + 3], kk[u].w, s);
                    }
                }
            }
            s += __shfl_xor(s, 1);
            s += __shfl_xor(s, 2);
            if (ci < n && part == 0) keys[ci] = order_key(s);
        }
    }
    __syncthreads();
    if (tid >= 64) return;                             // the selection itself is one wavefront's work

    int32_t *out = sel_idx + row * g.topk;
    const int k = g.topk;
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    int written = 0;
    float row_gap = __builtin_inff();

    if (n <= k) {
        for (int base = 0; base < n; base += 64) {
            const int ci = base + lane;
            if (ci < n) { int f; const int t = tile_of(ci, f); out[ci] = f * g.nb + t; }
        }
        written = n;
    } else {
        // T = k-th largest key: the largest value with at least k keys >= it (32-step bitwise search)
        uint32_t T = 0;
        if (n <= 128) {
            // the common case (a window of at most 21 tiles over 6 frames): two keys per lane in registers
            const uint32_t k0 = lane < n ? keys[lane] : 0u, k1 = lane + 64 < n ? keys[lane + 64] : 0u;   // finite floats map to keys > 0
            for (int bit = 31; bit >= 0; --bit) {
                const uint32_t trial = T | (1u << bit);
                if (wave_count(k0 >= trial) + wave_count(k1 >= trial) >= k) T = trial;
            }
        } else {
            for (int bit = 31; bit >= 0; --bit) {
                const uint32_t trial = T | (1u << bit);
                int cnt = 0;
                for (int base = 0; base < n; base += 64) {
                    const int ci = base + lane;
                    cnt += wave_count(ci < n && keys[ci] >= trial);
                }
                if (cnt >= k) T = trial;
            }
        }
        int n_gt = 0, n_ge = 0;
        uint32_t below = 0;                              // largest key < T (0 if none; keys of finite floats are > 0)
        for (int base = 0; base < n; base += 64) {
            const int ci = base + lane;
            const uint32_t key = ci < n ? keys[ci] : 0u;
            n_gt += wave_count(ci < n && key > T);
            n_ge += wave_count(ci < n && key >= T);
            if (ci < n && key < T && key > below) below = key;
        }
        const int need = k - n_gt;                       // how many of the blocks tied at T are kept (>= 1)
        int eq_seen = 0;
        for (int base = 0; base < n; base += 64) {
            const int ci = base + lane;
            const uint32_t key = ci < n ? keys[ci] : 0u;
            const bool gt = ci < n && key > T, eq = ci < n && key == T;
            const uint64_t eq_mask = __ballot(eq);
            const bool keep = gt || (eq && eq_seen + __popcll(eq_mask & lt_mask) < need);
            const uint64_t keep_mask = __ballot(keep);
            if (keep) { int f; const int t = tile_of(ci, f); out[written + __popcll(keep_mask & lt_mask)] = f * g.nb + t; }
            written += __popcll(keep_mask);
            eq_seen += __popcll(eq_mask);
        }
        if (gap) {
            if (n_ge > k) row_gap = 0.f;
            else {
                for (int off = 32; off > 0; off >>= 1) {
                    const uint32_t o = __shfl_xor(below, off);
                    below = o > below ? o : below;
                }
                row_gap = key_to_float(T) - key_to_float(below);
            }
        }
    }
    for (int i = written + lane; i < k; i += 64) out[i] = -1;
    if (lane == 0) {
        sel_cnt[row] = written;
        if (gap) gap[row] = row_gap;
    }
}

} // namespace

int max_candidates(const KGeom &g, int valid_groups) {
    int my = 0, mx = 0;
    for (int b = 0; b < g.ty; ++b) { int lo, hi; axis_window(b, g.th, g.ty, g.rh, g.wmode, &lo, &hi); if (hi - lo > my) my = hi - lo; }
    for (int b = 0; b < g.tx; ++b) { int lo, hi; axis_window(b, g.tw, g.tx, g.rw, g.wmode, &lo, &hi); if (hi - lo > mx) mx = hi - lo; }
    return my * mx * valid_groups;
}

hipError_t launch_select(const KGeom &g, const KCache &c, const float *pooled_q,
                         int32_t *sel_idx, int32_t *sel_cnt, float *gap, int max_cand, hipStream_t stream) {
    dim3 grid(g.q_groups * g.nb * g.heads);
    const size_t lds = (size_t)(g.d + max_cand) * sizeof(float);
    select_kernel<0><<<grid, kSelThreads, lds, stream>>>(g, c, pooled_q, nullptr, 0, 0, nullptr, sel_idx, sel_cnt, gap);
    return hipGetLastError();
}

hipError_t launch_pool_select(const KGeom &g, const KCache &c, const void *q, int64_t q_st, int64_t q_sh, float *pooled_q,
                              int32_t *sel_idx, int32_t *sel_cnt, float *gap, int max_cand, hipStream_t stream) {
    dim3 grid(g.q_groups * g.nb * g.heads);
    const int vec = g.bf16 ? 8 : 4;
    const size_t lds = (size_t)(g.d + (max_cand > kSelThreads * vec ? max_cand : kSelThreads * vec)) * sizeof(float);
    if (g.bf16)
        select_kernel<8><<<grid, kSelThreads, lds, stream>>>(g, c, nullptr, (const char *)q, q_st, q_sh, pooled_q, sel_idx, sel_cnt, gap);
    else
        select_kernel<4><<<grid, kSelThreads, lds, stream>>>(g, c, nullptr, (const char *)q, q_st, q_sh, pooled_q, sel_idx, sel_cnt, gap);
    return hipGetLastError();
}

} // namespace lcsa
