// Block mean pooling (Sec. 3.2), shared by the pooling kernel, the cache append and the fused
// pool + select kernel, so that a block mean is the same bit pattern whichever kernel formed it.
#pragma once
#include "lcsa_kernels.h"

namespace lcsa {
namespace pooling {

constexpr int kThreads = 256;

template <int VEC> struct Unpack;
template <> struct Unpack<8> {   // 8 x bf16 in 16 bytes
    static __device__ void to_float(const uint4 &u, float *f) {
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};
template <> struct Unpack<4> {   // 4 x f32
    static __device__ void to_float(const uint4 &u, float *f) {
        f[0] = __uint_as_float(u.x); f[1] = __uint_as_float(u.y);
        f[2] = __uint_as_float(u.z); f[3] = __uint_as_float(u.w);
    }
};

struct TileRef {
    int group, by, bx;   // group of tt frames within the call's tensor, tile coordinates
    int vh, vw;          // valid rows / cols of the tile
};

__device__ inline TileRef tile_ref(const KGeom &g, int block) {
    TileRef t;
    t.group = block / g.nb;
    int tile = block - t.group * g.nb;
    t.by = tile / g.tx;
    t.bx = tile - t.by * g.tx;
    t.vh = min(g.th, g.H - t.by * g.th);
    t.vw = min(g.tw, g.W - t.bx * g.tw);
    return t;
}

// Sum over the row-groups held in LDS and write the mean of the block.
template <int VEC>
__device__ inline void finish_pool(float *red, const float *acc, int rg, int j, int lpr, int rows_par,
                                   bool active, int d, int count, float *out) {
    if (active) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) red[rg * d + j * VEC + e] = acc[e];
    }
    __syncthreads();
    for (int c = threadIdx.x; c < d; c += kThreads) {
        float s = 0.f;
        for (int r = 0; r < rows_par; ++r) s += red[r * d + c];
        out[c] = s / (float)count;
    }
}

// What accumulate_block does to a 16-byte vector between loading and summing it: nothing, by default.
struct NoTransform {
    __device__ uint4 apply(const uint4 &u, int frame, int row, int col, int64_t token) const { return u; }
};

// Sums this thread's share of one block of x into acc[VEC]: lanes j cover a token row with 16-byte
// vectors, rows_par = kThreads / lpr token rows are in flight, 8 rows per lane are requested before any
// is consumed so that the loads overlap.  xf may change (and store elsewhere) every vector on its way
// into the sum; the order of the summation does not depend on it.
template <int VEC, class X = NoTransform>
__device__ inline void accumulate_block(const KGeom &g, const TileRef &t, const char *x, int64_t st, int64_t sh, int head,
                                        int rg, int j, int rows_par, float *acc, const X &xf = X()) {
    constexpr int ELT = 16 / VEC;
    const BlockTokens bt(g, t.vh, t.vw);
    for (int tok0 = rg; tok0 < g.bt; tok0 += 8 * rows_par) {
        uint4 u[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int tok = tok0 + i * rows_par;
            int ft, r, c;
            u[i] = make_uint4(0, 0, 0, 0);
            if (bt.at(tok, ft, r, c)) {
                const int64_t token = raster_token(g, t.group, ft, t.by * g.th + r, t.bx * g.tw + c);
                u[i] = *(const uint4 *)(x + (token * st + (int64_t)head * sh + j * VEC) * ELT);
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if constexpr (!__is_same(X, NoTransform)) {
                const int tok = tok0 + i * rows_par;
                int ft, r, c;
                if (bt.at(tok, ft, r, c))
                    u[i] = xf.apply(u[i], t.group * g.tt + ft, t.by * g.th + r, t.bx * g.tw + c,
                                    raster_token(g, t.group, ft, t.by * g.th + r, t.bx * g.tw + c));
            }
            float f[VEC];
            Unpack<VEC>::to_float(u[i], f);       // zeros for padding add nothing
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] += f[e];
        }
    }
}

} // namespace pooling
} // namespace lcsa
