// Backward of the block-sparse attention (Sec. 3.2 "Stage 2": the model is trained with this attention).
// The discrete top-k choice carries no gradient, so this is the backward of eq. (1) restricted to the kept
// block pairs: with s_ij = scale q_i.k_j, p_ij = exp(s_ij - lse_i), g_i = dL/do_i,
//     t_ij = g_i.v_j,  D_i = sum_j p_ij t_ij (= g_i.o_i),  u_ij = p_ij (t_ij - D_i),
//     dq_i = scale sum_j u_ij k_j,   dk_j = scale sum_i u_ij q_i,   dv_j = sum_i p_ij g_i.
//
// Two kernels, plain float FMA arithmetic, any shape the generic forward covers, no atomics and fixed
// summation orders (results are reproducible bit for bit):
//   bwd_dq_kernel    one workgroup per (head, query block), a wavefront per query token: lane-per-key dot
//                    products for s and t, first to form D_i from the kernel's own p and t (the forward's
//                    output, rounded to its element type, would put an error of ~2^-9 |o| |g| sqrt(d) into D
//                    and through it into dq and dk; D_i is also stored for the second kernel), then again
//                    for u, with lane-per-channel accumulation of u k over the keys.
//   bwd_dkv_kernel   one workgroup per (head, key block): finds the query blocks that kept this block (their
//                    id lists are ascending: one binary search per row), walks them in ascending order, four
//                    query tokens at a time (one per wavefront), and accumulates dk and dv of the block in LDS;
//                    every key token belongs to exactly one block, so dk and dv are written in full.
// K and V are read from the caller's raster tensors (the frames the cache held at the forward, oldest first):
// the backward needs them in token-major form for both operands, which the cache's tile images do not give.
#include "lcsa_kernels.h"

namespace lcsa {
namespace {

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;

template <typename T> struct In;
template <> struct In<float> {
    static constexpr int VEC = 4;
    static __device__ float load(const float *p) { return *p; }
    static __device__ void load_vec(const float *p, float *f) {
        const float4 u = *(const float4 *)p;
        f[0] = u.x; f[1] = u.y; f[2] = u.z; f[3] = u.w;
    }
};
template <> struct In<__bf16> {
    static constexpr int VEC = 8;
    static __device__ float load(const __bf16 *p) { return (float)*p; }
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

__device__ inline float wave_sum(float x) {
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
}

struct BlockRef { int group, by, bx, vh, vw, n_valid; };
__device__ inline BlockRef block_ref(const KGeom &g, int block) {
    BlockRef b;
    b.group = block / g.nb;
    const int tile = block - b.group * g.nb;
    b.by = tile / g.tx;
    b.bx = tile - b.by * g.tx;
    b.vh = min(g.th, g.H - b.by * g.th);
    b.vw = min(g.tw, g.W - b.bx * g.tw);
    b.n_valid = g.tt * b.vh * b.vw;
    return b;
}
// raster token of valid block token i (i < n_valid)
__device__ inline int64_t token_of(const KGeom &g, const BlockRef &b, int i) {
    int ft, r, c;
    block_token(g, i, b.vh, b.vw, ft, r, c);
    return raster_token(g, b.group, ft, b.by * g.th + r, b.bx * g.tw + c);
}

// s = q.k_j and t = g.v_j for this lane's key row (q, g in LDS as floats)
template <typename T>
__device__ inline void key_dots(const float *qv, const float *gv, const T *krow, const T *vrow, int d, float &s, float &t) {
    constexpr int VEC = In<T>::VEC;
    s = 0.f; t = 0.f;
    for (int e = 0; e < d; e += VEC) {
        float kf[VEC], vf[VEC];
        In<T>::load_vec(krow + e, kf);
        In<T>::load_vec(vrow + e, vf);
#pragma unroll
        for (int i = 0; i < VEC; ++i) { s = fmaf(qv[e + i], kf[i], s); t = fmaf(gv[e + i], vf[i], t); }
    }
}

// ---------------------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void bwd_dq_kernel(
    KGeom g, int kv_groups, const T *__restrict__ q, int64_t q_st, int64_t q_sh,
    const T *__restrict__ k, const T *__restrict__ v, int64_t kv_st, int64_t kv_sh,
    const int32_t *__restrict__ sel_idx, const int32_t *__restrict__ sel_cnt,
    const T *__restrict__ d_o, int64_t o_st, int64_t o_sh, const float *__restrict__ lse,
    float *__restrict__ d_q, float *__restrict__ delta, float scale) {
    __shared__ float qv[kWaves][256], gv[kWaves][256];
    constexpr int DPL = 4;                                   // channels per lane: e = lane + 64*jj
    const int qb = blockIdx.x / g.heads, head = blockIdx.x - qb * g.heads;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n_qb = g.q_groups * g.nb;
    const BlockRef qr = block_ref(g, qb);
    const int64_t row = (int64_t)head * n_qb + qb;
    const int cnt = min(max(sel_cnt[row], 0), g.topk);
    const int32_t *sel = sel_idx + row * g.topk;

    // every wavefront walks the same loop structure so that workgroup barriers line up; wavefronts whose token
    // is padding compute on a clamped token and store nothing
    for (int t0 = 0; t0 < qr.n_valid; t0 += kWaves) {
        const bool q_valid = t0 + wave < qr.n_valid;
        const int64_t token = token_of(g, qr, q_valid ? t0 + wave : 0);
        __syncthreads();                                     // the previous token's readers of qv, gv are done
        for (int e = lane; e < g.d; e += 64) {
            qv[wave][e] = In<T>::load(q + token * q_st + (int64_t)head * q_sh + e);
            gv[wave][e] = In<T>::load(d_o + token * o_st + (int64_t)head * o_sh + e);
        }
        const float l = lse[token * g.heads + head];
        __syncthreads();
        // first pass over the kept keys: D_i = sum_j p_ij t_ij
        float dsum = 0.f;
        for (int b = 0; b < cnt; ++b) {
            const int kb = min(max(sel[b], 0), kv_groups * g.nb - 1);      // ids outside the visible blocks must not become wild addresses
            const BlockRef kr = block_ref(g, kb);
            for (int j = lane; j < kr.n_valid; j += 64) {
                const int64_t kt = token_of(g, kr, j);
                float s, t;
                key_dots<T>(qv[wave], gv[wave], k + kt * kv_st + (int64_t)head * kv_sh, v + kt * kv_st + (int64_t)head * kv_sh, g.d, s, t);
                dsum = fmaf(__expf(s * scale - l), t, dsum);
            }
        }
        const float D = wave_sum(dsum);
        if (q_valid && lane == 0) delta[token * g.heads + head] = D;
        float acc[DPL] = {0.f, 0.f, 0.f, 0.f};
        for (int b = 0; b < cnt; ++b) {
            const int kb = min(max(sel[b], 0), kv_groups * g.nb - 1);
            const BlockRef kr = block_ref(g, kb);
            for (int base = 0; base < kr.n_valid; base += 64) {
                const int j = base + lane;
                float u = 0.f;
                if (j < kr.n_valid) {
                    const int64_t kt = token_of(g, kr, j);
                    float s, t;
                    key_dots<T>(qv[wave], gv[wave], k + kt * kv_st + (int64_t)head * kv_sh, v + kt * kv_st + (int64_t)head * kv_sh, g.d, s, t);
                    u = __expf(s * scale - l) * (t - D);
                }
                const int nk = min(64, kr.n_valid - base);
                for (int jj = 0; jj < nk; ++jj) {            // lane-per-channel: coalesced reads of one key row at a time
                    const float uj = __shfl(u, jj);
                    const T *krow = k + token_of(g, kr, base + jj) * kv_st + (int64_t)head * kv_sh;
#pragma unroll
                    for (int c = 0; c < DPL; ++c) {
                        const int e = lane + 64 * c;
                        if (e < g.d) acc[c] = fmaf(uj, In<T>::load(krow + e), acc[c]);
                    }
                }
            }
        }
        if (q_valid) {
#pragma unroll
            for (int c = 0; c < DPL; ++c) {
                const int e = lane + 64 * c;
                if (e < g.d) d_q[(token * g.heads + head) * g.d + e] = acc[c] * scale;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------------
// dynamic LDS: float dk[bt*d], dv[bt*d], ps[kWaves][bt], us[kWaves][bt], qv[kWaves][d], gv[kWaves][d]; then one flag byte per query block
template <typename T>
__global__ __launch_bounds__(kThreads) void bwd_dkv_kernel(
    KGeom g, int kv_groups, const T *__restrict__ q, int64_t q_st, int64_t q_sh,
    const T *__restrict__ k, const T *__restrict__ v, int64_t kv_st, int64_t kv_sh,
    const int32_t *__restrict__ sel_idx, const int32_t *__restrict__ sel_cnt,
    const T *__restrict__ d_o, int64_t o_st, int64_t o_sh, const float *__restrict__ lse, const float *__restrict__ delta,
    float *__restrict__ d_k, float *__restrict__ d_v, float scale) {
    extern __shared__ float smem[];
    float *dk = smem, *dv = dk + g.bt * g.d, *ps = dv + g.bt * g.d, *us = ps + kWaves * g.bt;
    float *qv = us + kWaves * g.bt, *gv = qv + kWaves * g.d;
    unsigned char *kept_by = (unsigned char *)(gv + kWaves * g.d);
    const int kb = blockIdx.x / g.heads, head = blockIdx.x - kb * g.heads;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n_qb = g.q_groups * g.nb;
    const BlockRef kr = block_ref(g, kb);

    for (int i = tid; i < g.bt * g.d; i += kThreads) { dk[i] = 0.f; dv[i] = 0.f; }
    // which query blocks kept this key block?  (ascending id lists: binary search)
    for (int qb = tid; qb < n_qb; qb += kThreads) {
        const int64_t row = (int64_t)head * n_qb + qb;
        const int32_t *sel = sel_idx + row * g.topk;
        int lo = 0, hi = min(max(sel_cnt[row], 0), g.topk);
        while (lo < hi) { const int mid = (lo + hi) >> 1; if (sel[mid] < kb) lo = mid + 1; else hi = mid; }
        kept_by[qb] = lo < min(max(sel_cnt[row], 0), g.topk) && sel[lo] == kb;
    }
    __syncthreads();

    for (int qb = 0; qb < n_qb; ++qb) {
        if (!kept_by[qb]) continue;                          // uniform
        const BlockRef qr = block_ref(g, qb);
        for (int t0 = 0; t0 < qr.n_valid; t0 += kWaves) {
            const int nw = min(kWaves, qr.n_valid - t0);     // query tokens of this round, one per wavefront
            if (wave < nw) {
                const int64_t token = token_of(g, qr, t0 + wave);
                for (int e = lane; e < g.d; e += 64) {
                    qv[wave * g.d + e] = In<T>::load(q + token * q_st + (int64_t)head * q_sh + e);
                    gv[wave * g.d + e] = In<T>::load(d_o + token * o_st + (int64_t)head * o_sh + e);
                }
                const float D = delta[token * g.heads + head];   // written by bwd_dq_kernel, earlier on the stream
                const float l = lse[token * g.heads + head];
                // this wavefront reads what its own lanes wrote: LDS operations of one wavefront complete in order
                __builtin_amdgcn_s_waitcnt(0xc07f);          // lgkmcnt(0)
                __builtin_amdgcn_wave_barrier();
                for (int j = lane; j < kr.n_valid; j += 64) {
                    const int64_t kt = token_of(g, kr, j);
                    float s, t;
                    key_dots<T>(qv + wave * g.d, gv + wave * g.d, k + kt * kv_st + (int64_t)head * kv_sh,
                                v + kt * kv_st + (int64_t)head * kv_sh, g.d, s, t);
                    const float p = __expf(s * scale - l);
                    ps[wave * g.bt + j] = p;
                    us[wave * g.bt + j] = p * (t - D) * scale;
                }
            }
            __syncthreads();
            for (int idx = tid; idx < kr.n_valid * g.d; idx += kThreads) {
                const int j = idx / g.d, c = idx - j * g.d;
                float av = dv[idx], ak = dk[idx];
                for (int w = 0; w < nw; ++w) {               // fixed order: query tokens ascending
                    av = fmaf(ps[w * g.bt + j], gv[w * g.d + c], av);
                    ak = fmaf(us[w * g.bt + j], qv[w * g.d + c], ak);
                }
                dv[idx] = av; dk[idx] = ak;
            }
            __syncthreads();
        }
    }
    for (int idx = tid; idx < kr.n_valid * g.d; idx += kThreads) {
        const int j = idx / g.d, c = idx - j * g.d;
        const int64_t kt = token_of(g, kr, j);
        d_k[(kt * g.heads + head) * g.d + c] = dk[idx];
        d_v[(kt * g.heads + head) * g.d + c] = dv[idx];
    }
}

size_t dkv_lds_bytes(const KGeom &g) {
    return ((size_t)2 * g.bt * g.d + 2 * kWaves * g.bt + 2 * kWaves * g.d) * sizeof(float) + (size_t)g.q_groups * g.nb;
}

} // namespace

bool attn_bwd_supported(const KGeom &g) { return dkv_lds_bytes(g) <= 160 * 1024; }

hipError_t launch_attn_bwd(const KGeom &g, int kv_groups, const void *q, int64_t q_st, int64_t q_sh,
                           const void *k, const void *v, int64_t kv_st, int64_t kv_sh,
                           const int32_t *sel_idx, const int32_t *sel_cnt,
                           const void *d_o, int64_t o_st, int64_t o_sh, const float *lse,
                           float *d_q, float *d_k, float *d_v, float *delta, float scale, hipStream_t stream) {
    const dim3 grid_q(g.q_groups * g.nb * g.heads), grid_k(kv_groups * g.nb * g.heads);
    const size_t lds = dkv_lds_bytes(g);
    hipError_t e;
    if (g.bf16) {
        e = hipFuncSetAttribute((const void *)bwd_dkv_kernel<__bf16>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        bwd_dq_kernel<__bf16><<<grid_q, kThreads, 0, stream>>>(g, kv_groups, (const __bf16 *)q, q_st, q_sh, (const __bf16 *)k, (const __bf16 *)v,
                                                               kv_st, kv_sh, sel_idx, sel_cnt, (const __bf16 *)d_o, o_st, o_sh,
                                                               lse, d_q, delta, scale);
        bwd_dkv_kernel<__bf16><<<grid_k, kThreads, lds, stream>>>(g, kv_groups, (const __bf16 *)q, q_st, q_sh, (const __bf16 *)k, (const __bf16 *)v,
                                                                  kv_st, kv_sh, sel_idx, sel_cnt, (const __bf16 *)d_o, o_st, o_sh,
                                                                  lse, delta, d_k, d_v, scale);
    } else {
        e = hipFuncSetAttribute((const void *)bwd_dkv_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        bwd_dq_kernel<float><<<grid_q, kThreads, 0, stream>>>(g, kv_groups, (const float *)q, q_st, q_sh, (const float *)k, (const float *)v,
                                                              kv_st, kv_sh, sel_idx, sel_cnt, (const float *)d_o, o_st, o_sh,
                                                              lse, d_q, delta, scale);
        bwd_dkv_kernel<float><<<grid_k, kThreads, lds, stream>>>(g, kv_groups, (const float *)q, q_st, q_sh, (const float *)k, (const float *)v,
                                                                 kv_st, kv_sh, sel_idx, sel_cnt, (const float *)d_o, o_st, o_sh,
                                                                 lse, delta, d_k, d_v, scale);
    }
    return hipGetLastError();
}

} // namespace lcsa
