// Block-sparse attention, generic path: any head_dim <= 256, any tile shape, f32 or bf16
// storage, plain FMA arithmetic in float.  Used where the matrix-core kernel's shape
// constraints do not hold (e.g. the 16-token / d = 32 / f32 toy configuration).
//
// One workgroup per (head, query block), four wavefronts, each owning one query token at a
// time.  Keys of a selected block are taken 64 at a time: lane-per-key dot products against
// the query held in LDS, wavefront max/sum for the online softmax (eq. 1), probabilities
// through LDS, then lane-per-channel accumulation of P*V with coalesced V reads.
#include "lcsa_kernels.h"

namespace lcsa {
namespace {

constexpr int kWaves = 4;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <typename T> struct Elt;
template <> struct Elt<float> {
    static constexpr int VEC = 4;
    static __device__ float load(const float *p) { return *p; }
    static __device__ void store(float *p, float x) { *p = x; }
    static __device__ void load_vec(const float *p, float *f) {
        const float4 u = *(const float4 *)p;
        f[0] = u.x; f[1] = u.y; f[2] = u.z; f[3] = u.w;
    }
};
template <> struct Elt<__bf16> {
    static constexpr int VEC = 8;
    static __device__ float load(const __bf16 *p) { return (float)*p; }
    static __device__ void store(__bf16 *p, float x) { *p = (__bf16)x; }
    static __device__ void load_vec(const __bf16 *p, float *f) {
        const uint4 u = *(const uint4 *)p;
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};

__device__ inline float wave_max(float x) {
    for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
    return x;
}
__device__ inline float wave_sum(float x) {
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
}

template <typename T>
__global__ __launch_bounds__(64 * kWaves) void attn_generic_kernel(
    KGeom g, KCache c, const T *__restrict__ q, int64_t q_st, int64_t q_sh,
    const int32_t *__restrict__ sel_idx, const int32_t *__restrict__ sel_cnt,
    T *__restrict__ o, int64_t o_st, int64_t o_sh, float *__restrict__ lse, float scale_log2) {
    __shared__ float qs[kWaves][256];
    __shared__ float ps[kWaves][64];
    constexpr int VEC = Elt<T>::VEC;
    constexpr int DPL = 4;                                  // channels per lane: e = lane + 64*jj
    const int qb = blockIdx.x, head = blockIdx.y;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n_qb = g.q_groups * g.nb;
    const int fq = qb / g.nb, tile = qb - fq * g.nb, by = tile / g.tx, bx = tile - by * g.tx;
    const int qvh = min(g.th, g.H - by * g.th), qvw = min(g.tw, g.W - bx * g.tw);
    const int64_t row = (int64_t)head * n_qb + qb;
    const int cnt = min(max(sel_cnt[row], 0), g.topk);       // a row holds at most topk ids
    const int32_t *sel = sel_idx + row * g.topk;
    const T *kc = (const T *)c.k, *vc = (const T *)c.v;
    const int start = ring_start(c, g);

    // every wavefront walks the same loop structure so that workgroup barriers line up;
    // wavefronts whose token is padding compute on a clamped token and store nothing
    for (int t0 = 0; t0 < g.bt; t0 += kWaves) {
        const int tq = t0 + wave;
        int qft, r, cc;
        const bool q_valid = block_token(g, tq, qvh, qvw, qft, r, cc);
        const int64_t token = q_valid ? raster_token(g, fq, qft, by * g.th + r, bx * g.tw + cc)
                                      : raster_token(g, fq, 0, by * g.th, bx * g.tw);
        __syncthreads();                                     // previous token's readers of qs are done
        for (int e = lane; e < g.d; e += 64) qs[wave][e] = Elt<T>::load(q + token * q_st + (int64_t)head * q_sh + e);
        __syncthreads();
        float m = -__builtin_inff(), l = 0.f, acc[DPL] = {0.f, 0.f, 0.f, 0.f};
        for (int b = 0; b < cnt; ++b) {
            const int kb = min(max(sel[b], 0), c.valid * g.nb - 1);   // ids outside the cache must not become wild addresses
            const int f = kb / g.nb, kt = kb - f * g.nb, kby = kt / g.tx, kbx = kt - kby * g.tx;
            const int vh = min(g.th, g.H - kby * g.th), vw = min(g.tw, g.W - kbx * g.tw);
            const int slot = cache_slot(c, g, start, head, f);
            const int64_t tbase = (((int64_t)head * g.cap + slot) * g.nb + kt) * g.bt * g.d;
            for (int base = 0; base < g.bt; base += 64) {
                const int key = base + lane;
                int kft, kr, kcc;
                const bool k_valid = block_token(g, key, vh, vw, kft, kr, kcc);
                float s = -__builtin_inff();
                if (k_valid) {
                    const T *kp = kc + tbase + (int64_t)key * g.d;
                    float dot = 0.f;
                    for (int e = 0; e < g.d; e += VEC) {
                        float kv[VEC];
                        Elt<T>::load_vec(kp + e, kv);
#pragma unroll
                        for (int i = 0; i < VEC; ++i) dot = fmaf(qs[wave][e + i], kv[i], dot);
                    }
                    s = dot * scale_log2;
                }
                const float cmax = wave_max(s);
                // a 64-key group made only of padding is skipped by all wavefronts alike
                if (cmax == -__builtin_inff()) continue;
                const float m_new = fmaxf(m, cmax);
                const float p = k_valid ? __builtin_amdgcn_exp2f(s - m_new) : 0.f;
                const float alpha = __builtin_amdgcn_exp2f(m - m_new);
                l = l * alpha + wave_sum(p);
                m = m_new;
                __syncthreads();                             // previous group's readers of ps are done
                ps[wave][lane] = p;
                __syncthreads();
                const int nk = min(64, g.bt - base);
#pragma unroll
                for (int jj = 0; jj < DPL; ++jj) {
                    const int e = lane + 64 * jj;
                    if (e < g.d) {
                        float a = acc[jj] * alpha;
                        const T *vp = vc + tbase + (int64_t)base * g.d + e;
                        for (int j = 0; j < nk; ++j) a = fmaf(ps[wave][j], Elt<T>::load(vp + (int64_t)j * g.d), a);
                        acc[jj] = a;
                    }
                }
            }
        }
        if (q_valid) {
            const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
            for (int jj = 0; jj < DPL; ++jj) {
                const int e = lane + 64 * jj;
                if (e < g.d) Elt<T>::store(o + token * o_st + (int64_t)head * o_sh + e, acc[jj] * inv);
            }
            if (lse && lane == 0)
                lse[token * g.heads + head] = l > 0.f ? (m + __builtin_amdgcn_logf(l)) * kLn2 : -__builtin_inff();
        }
    }
}

} // namespace

hipError_t launch_attn_generic(const KGeom &g, const KCache &c, const void *q, int64_t q_st, int64_t q_sh,
                               const int32_t *sel_idx, const int32_t *sel_cnt,
                               void *o, int64_t o_st, int64_t o_sh, float *lse, float scale, hipStream_t stream) {
    dim3 grid(g.q_groups * g.nb, g.heads);
    const float scale_log2 = scale * kLog2e;
    if (g.bf16)
        attn_generic_kernel<__bf16><<<grid, 64 * kWaves, 0, stream>>>(g, c, (const __bf16 *)q, q_st, q_sh, sel_idx, sel_cnt,
                                                                      (__bf16 *)o, o_st, o_sh, lse, scale_log2);
    else
        attn_generic_kernel<float><<<grid, 64 * kWaves, 0, stream>>>(g, c, (const float *)q, q_st, q_sh, sel_idx, sel_cnt,
                                                                     (float *)o, o_st, o_sh, lse, scale_log2);
    return hipGetLastError();
}

} // namespace lcsa
