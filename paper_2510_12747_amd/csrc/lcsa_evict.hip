// Importance-based KV-cache eviction (appendix on KV-cache eviction; the paper's default is the
// sliding window and it reports this variant as a preliminary exploration).
//
// Importance of a cached group of frames = attention its key blocks receive in the coarse
// block-to-block attention map of the chunk attended last: row softmax (eq. 1 scale) of the
// pooled-Q . pooled-K scores (Sec. 3.2) over the blocks of the row's spatial window (Sec. 3.3),
// summed over the chunk's query blocks and over the blocks of the group.
//
//   importance_rows_kernel   one workgroup per (head, query block): scores of the admissible
//                            blocks, row max, exponentials, one sum per visible group
//   importance_sum_kernel    per (head, group): sum over query blocks, in a fixed order
//   evict_kernel             one wavefront per head: drops the least important visible groups
//                            (ties: older first), hands the free slots to the arriving groups,
//                            rewrites the head's visible-group -> slot table
// Everything is deterministic: no atomics, fixed summation orders.
#include "lcsa_kernels.h"

#include <mutex>

namespace lcsa {
namespace {

constexpr int kThreads = 256;

// Scratch of the entry point that allocates nothing: the per-row partial sums of the importance kernels,
// held by every GPU the library runs on until the process ends.  The name below is only a host-side handle
// of the symbol; host code uses the per-device address that hipGetSymbolAddress returns.
__device__ __align__(256) float scratch[kStaticScratchFloats];

constexpr int kMaxDevices = 64;
float *g_scratch_ptr[kMaxDevices];      // address of `scratch` on each device, looked up once
std::mutex g_scratch_mutex;

__global__ __launch_bounds__(kThreads) void importance_rows_kernel(KGeom g, KCache c, const float *__restrict__ pooled_q,
                                                                   float scale, float *__restrict__ row_group) {
    extern __shared__ float smem[];
    float *qs = smem;                       // [d] pooled query of this row
    float *gsum = smem + g.d;               // [cap] per-group sums of exponentials
    float *red = gsum + g.cap;              // [4] per-wavefront partial results
    float *sc = red + 4;                    // [n] scaled scores, then exponentials
    const int qb = blockIdx.x, head = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_qb = g.q_groups * g.nb;
    const int tile = qb % g.nb, by = tile / g.tx, bx = tile - by * g.tx;
    int y0, y1, x0, x1;
    axis_window(by, g.th, g.ty, g.rh, g.wmode, &y0, &y1);
    axis_window(bx, g.tw, g.tx, g.rw, g.wmode, &x0, &x1);
    const int wx = x1 - x0, nwin = (y1 - y0) * wx;
    const int n = c.valid * nwin;           // admissible key blocks; those of visible group f are [f*nwin, (f+1)*nwin)
    const int64_t row = (int64_t)head * n_qb + qb;
    const int start = ring_start(c, g);

    for (int i = tid; i < g.d; i += kThreads) qs[i] = pooled_q[row * g.d + i];
    __syncthreads();

    // scores: four lanes per candidate, each a quarter of the channels
    {
        const int part = tid & 3, n4 = g.d / 4;
        for (int ci = tid >> 2; ci < ((n + 63) & ~63); ci += kThreads / 4) {
            float s = 0.f;
            if (ci < n) {
                const int f = ci / nwin, w = ci - f * nwin, wy = w / wx;
                const int t = (y0 + wy) * g.tx + x0 + (w - wy * wx);
                const int slot = cache_slot(c, g, start, head, f);
                const float4 *kr = (const float4 *)(c.pooled + (((int64_t)head * g.cap + slot) * g.nb + t) * g.d);
                for (int e4 = part; e4 < n4; e4 += 4) {
                    const float4 kk = kr[e4];
                    s = fmaf(qs[4 * e4], kk.x, s);
                    s = fmaf(qs[4 * e4 + 1], kk.y, s);
                    s = fmaf(qs[4 * e4 + 2], kk.z, s);
                    s = fmaf(qs[4 * e4 + 3], kk.w, s);
                }
            }
            s += __shfl_xor(s, 1);
            s += __shfl_xor(s, 2);
            if (ci < n && part == 0) sc[ci] = s * scale;
        }
    }
    __syncthreads();

    // row maximum
    float mx = -__builtin_inff();
    for (int ci = tid; ci < n; ci += kThreads) mx = fmaxf(mx, sc[ci]);
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));

    // per visible group: sum of exp(score - max); wavefront w takes groups w, w+4, ...
    for (int f = wave; f < c.valid; f += kThreads / 64) {
        float s = 0.f;
        for (int w = lane; w < nwin; w += 64) s += expf(sc[f * nwin + w] - mx);
        for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
        if (lane == 0) gsum[f] = s;
    }
    __syncthreads();
    float den = 0.f;
    for (int f = 0; f < c.valid; ++f) den += gsum[f];
    for (int f = tid; f < g.cap; f += kThreads) row_group[row * g.cap + f] = f < c.valid && den > 0.f ? gsum[f] / den : 0.f;
}

__global__ void importance_sum_kernel(const float *__restrict__ row_group, float *__restrict__ imp, int n_qb, int cap) {
    const int head = blockIdx.x, f = threadIdx.x;
    if (f >= cap) return;
    float s = 0.f;
    for (int i = 0; i < n_qb; ++i) s += row_group[((int64_t)head * n_qb + i) * cap + f];
    imp[head * cap + f] = s;
}

// One wavefront per head, lane f = visible group f (cap <= 64).
__global__ __launch_bounds__(64) void evict_kernel(int32_t *__restrict__ order, const float *__restrict__ imp, int heads, int cap,
                                                   int valid, int n_new, int n_evict, int uniform, int scored) {
    __shared__ int used[kMaxEvictGroups];
    const int head = blockIdx.x, lane = threadIdx.x;
    bool alive = lane < valid;
    const int slot = alive ? order[head * cap + lane] : 0;
    float w = 0.f;                                   // groups that were never scored count as zero
    if (alive && scored) {
        if (uniform) {
            for (int h = 0; h < heads; ++h) w += imp[h * cap + lane];     // same order for every head: same decision
        } else {
            w = imp[head * cap + lane];
        }
    }
    // the least important visible group goes, n_evict times; equal importance: the older one.  Importance
    // is a sum of softmax weights (>= 0), so its bit pattern orders like an integer; the lane index breaks ties.
    for (int e = 0; e < n_evict; ++e) {
        unsigned long long key = alive ? ((unsigned long long)__float_as_uint(w + 0.0f) << 32) | (unsigned)lane : ~0ull;
        for (int off = 32; off > 0; off >>= 1) {
            const unsigned long long other = __shfl_xor(key, off);
            key = other < key ? other : key;
        }
        if (lane == (int)(key & 0xffffffffu)) alive = false;
    }
    used[lane] = 0;
    __syncthreads();
    const uint64_t keep = __ballot(alive);
    const int m = __popcll(keep);
    if (alive) {
        order[head * cap + __popcll(keep & ((1ull << lane) - 1ull))] = slot;      // survivors stay in temporal order
        used[slot] = 1;
    }
    __syncthreads();
    // arrivals take the free slots in ascending order
    const uint64_t free_slots = __ballot(lane < cap && !used[lane]);
    if (lane < n_new) {
        uint64_t f = free_slots;
        for (int i = 0; i < lane; ++i) f &= f - 1;                                  // drop the lane lowest set bits
        order[head * cap + m + lane] = __ffsll((unsigned long long)f) - 1;
    }
}

} // namespace

hipError_t launch_importance(const KGeom &g, const KCache &c, const float *pooled_q, float scale,
                             float *row_group, float *imp, int max_cand, hipStream_t stream) {
    const int n_qb = g.q_groups * g.nb;
    const size_t smem = (size_t)(g.d + g.cap + 4 + max_cand) * sizeof(float);
    importance_rows_kernel<<<dim3(n_qb, g.heads), kThreads, smem, stream>>>(g, c, pooled_q, scale, row_group);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    importance_sum_kernel<<<dim3(g.heads), dim3((g.cap + 63) / 64 * 64), 0, stream>>>(row_group, imp, n_qb, g.cap);
    return hipGetLastError();
}

hipError_t launch_importance_static(const KGeom &g, const KCache &c, const float *pooled_q, float scale,
                                    float *imp, int max_cand, hipStream_t stream) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    float *ptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {          // first call on this device, which is the current one
            void *p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return e;
            g_scratch_ptr[dev] = (float *)p;
        }
        ptr = g_scratch_ptr[dev];
    }
    // every row of the scratch that the second kernel reads is written in full by the first: nothing to clear
    return launch_importance(g, c, pooled_q, scale, ptr, imp, max_cand, stream);
}

hipError_t launch_evict(const KGeom &g, int32_t *order, const float *imp, int valid, int n_new, int n_evict,
                        bool uniform, bool scored, hipStream_t stream) {
    evict_kernel<<<dim3(g.heads), 64, 0, stream>>>(order, imp, g.heads, g.cap, valid, n_new, n_evict, uniform, scored);
    return hipGetLastError();
}

} // namespace lcsa
