// Bandwidth-bound kernels: block mean pooling (Sec. 3.2) and the sliding-window cache
// append, which re-tiles K and V into the layout the attention kernels read and pools
// the new keys on the way.  One workgroup per (block, head); every global access is a
// 16-byte vector per lane, consecutive lanes covering consecutive bytes of a token row.
#include "lcsa_kernels.h"
#include "lcsa_pool.h"

namespace lcsa {
namespace {

using namespace pooling;

// ---------------------------------------------------------------------------------------------
// pooled[head][block][c] = mean over the block's valid tokens.      grid (n_groups*nb, heads)
template <int VEC>
__global__ __launch_bounds__(kThreads) void pool_kernel(KGeom g, const char *x, int64_t st, int64_t sh,
                                                        int n_blocks, float *pooled) {
    __shared__ float red[kThreads * VEC];
    const int block = blockIdx.x, head = blockIdx.y;
    const TileRef t = tile_ref(g, block);
    const int lpr = g.d / VEC;                 // lanes per token row
    const int rows_par = kThreads / lpr;       // token rows in flight
    const int rg = threadIdx.x / lpr, j = threadIdx.x - rg * lpr;
    const bool active = rg < rows_par;
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
    if (active) accumulate_block<VEC>(g, t, x, st, sh, head, rg, j, rows_par, acc);
    finish_pool<VEC>(red, acc, rg, j, lpr, rows_par, active, g.d, g.tt * t.vh * t.vw,
                     pooled + ((int64_t)head * n_blocks + block) * g.d);
}

// ---------------------------------------------------------------------------------------------
// Cache append, generic tile image: K and V tiles row-major [bt][d], padded tokens zero;
// pooled K written beside them.                                      grid (n_groups*nb, heads)
template <int VEC>
__global__ __launch_bounds__(kThreads) void append_generic_kernel(KGeom g, KCache c, const char *k, const char *v,
                                                                  int64_t st, int64_t sh, int first) {
    __shared__ float red[kThreads * VEC];
    const int block = blockIdx.x, head = blockIdx.y;
    const TileRef t = tile_ref(g, block);
    const int slot = c.order ? c.order[head * g.cap + first + t.group] : (first + t.group) % g.cap;
    const int tile = block - t.group * g.nb;
    constexpr int ELT = 16 / VEC;
    const int64_t tile_index = ((int64_t)head * g.cap + slot) * g.nb + tile;
    char *kt = (char *)c.k + tile_index * g.bt * g.d * ELT;
    char *vt = (char *)c.v + tile_index * g.bt * g.d * ELT;
    const int lpr = g.d / VEC, rows_par = kThreads / lpr;
    const int rg = threadIdx.x / lpr, j = threadIdx.x - rg * lpr;
    const bool active = rg < rows_par;
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
    if (active) {
        for (int tok = rg; tok < g.bt; tok += rows_par) {
            int ft, r, cc;
            uint4 uk = make_uint4(0, 0, 0, 0), uv = uk;
            if (block_token(g, tok, t.vh, t.vw, ft, r, cc)) {
                const int64_t token = raster_token(g, t.group, ft, t.by * g.th + r, t.bx * g.tw + cc);
                const int64_t off = (token * st + (int64_t)head * sh + j * VEC) * ELT;
                uk = *(const uint4 *)(k + off);
                uv = *(const uint4 *)(v + off);
                float f[VEC];
                Unpack<VEC>::to_float(uk, f);
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] += f[e];
            }
            *(uint4 *)(kt + ((int64_t)tok * g.d + j * VEC) * ELT) = uk;
            *(uint4 *)(vt + ((int64_t)tok * g.d + j * VEC) * ELT) = uv;
        }
    }
    finish_pool<VEC>(red, acc, rg, j, lpr, rows_par, active, g.d, g.tt * t.vh * t.vw,
                     c.pooled + tile_index * g.d);
}

// bf16 bit pattern -> IEEE half bit pattern, round to nearest even, saturating (NaN stays NaN)
__device__ inline uint32_t bf16_bits_to_half_bits(uint32_t b) {
    float f = __uint_as_float(b << 16);
    f = fminf(fmaxf(f, -65504.f), 65504.f);          // fmin/fmax return the non-NaN operand: map NaN below
    if ((b & 0x7fffu) > 0x7f80u) return 0x7e00u;      // NaN
    const _Float16 h = (_Float16)f;
    return (uint32_t)__builtin_bit_cast(unsigned short, h);
}

// ---------------------------------------------------------------------------------------------
// Cache append, matrix-core tile image (bf16, d = 128, 128 tokens per tile).  Each tile is
// 128 rows of 256 bytes whose 16-byte chunk j sits at chunk position j ^ (row & 15), so the
// attention kernel can copy a tile into LDS byte for byte and read matrix operands without
// bank conflicts.  K rows are tokens (bf16 as given); V is transposed through LDS so that its
// rows are channels and its columns tokens, and is stored as IEEE half: every bf16 value with
// magnitude in [2^-14, 65504] converts exactly (8 significant bits into 11), smaller ones round
// to half subnormals (absolute error < 2^-25), larger ones saturate to +-65504.  Half is what the
// second matrix product runs in, because softmax probabilities need mantissa, not range.
//                                                                    grid (n_groups*nb, heads)
constexpr int kVPitchWords = 65;   // LDS pitch of a staged V token row (128 bf16 = 64 words, +1)

__global__ __launch_bounds__(kThreads) void append_mfma_kernel(KGeom g, KCache c, const char *k, const char *v,
                                                               int64_t st, int64_t sh, int first) {
    __shared__ float red[16 * 128];
    __shared__ uint32_t vs[128 * kVPitchWords];
    const int block = blockIdx.x, head = blockIdx.y;
    const TileRef t = tile_ref(g, block);
    const int slot = c.order ? c.order[head * g.cap + first + t.group] : (first + t.group) % g.cap;
    const int tile = block - t.group * g.nb;
    const int64_t tile_index = ((int64_t)head * g.cap + slot) * g.nb + tile;
    char *kt = (char *)c.k + tile_index * (128 * 256);
    char *vt = (char *)c.v + tile_index * (128 * 256);
    const int rg = threadIdx.x >> 4, j = threadIdx.x & 15;   // 16 token rows in flight, 16 chunks per row
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        const int tok = rg + 16 * it;
        int ft, r, cc;
        uint4 uk = make_uint4(0, 0, 0, 0), uv = uk;
        if (block_token(g, tok, t.vh, t.vw, ft, r, cc)) {
            const int64_t token = raster_token(g, t.group, ft, t.by * g.th + r, t.bx * g.tw + cc);
            const int64_t off = (token * st + (int64_t)head * sh + j * 8) * 2;
            uk = *(const uint4 *)(k + off);
            uv = *(const uint4 *)(v + off);
            float f[8];
            Unpack<8>::to_float(uk, f);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += f[e];
        }
        *(uint4 *)(kt + tok * 256 + ((j ^ (tok & 15)) << 4)) = uk;
        uint32_t *row = vs + tok * kVPitchWords + j * 4;
        row[0] = uv.x; row[1] = uv.y; row[2] = uv.z; row[3] = uv.w;
    }
    __syncthreads();
    // transposed write-out: this lane produces the 16-byte piece at (channel dd, chunk position pos)
    const unsigned short *vh = (const unsigned short *)vs;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        const int dd = rg + 16 * it, pos = j;
        const int chunk = pos ^ (dd & 15);           // tokens 8*chunk .. 8*chunk+7
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t lo = vh[(8 * chunk + 2 * i) * (2 * kVPitchWords) + dd];
            const uint32_t hi = vh[(8 * chunk + 2 * i + 1) * (2 * kVPitchWords) + dd];
            w[i] = bf16_bits_to_half_bits(lo) | (bf16_bits_to_half_bits(hi) << 16);
        }
        *(uint4 *)(vt + dd * 256 + (pos << 4)) = make_uint4(w[0], w[1], w[2], w[3]);
    }
    finish_pool<8>(red, acc, rg, j, 16, 16, true, 128, g.tt * t.vh * t.vw, c.pooled + tile_index * 128);
}

} // namespace

hipError_t launch_pool(const KGeom &g, const void *x, int64_t stride_tok, int64_t stride_head,
                       int n_groups, float *pooled, hipStream_t stream) {
    dim3 grid(n_groups * g.nb, g.heads);
    if (g.bf16)
        pool_kernel<8><<<grid, kThreads, 0, stream>>>(g, (const char *)x, stride_tok, stride_head, n_groups * g.nb, pooled);
    else
        pool_kernel<4><<<grid, kThreads, 0, stream>>>(g, (const char *)x, stride_tok, stride_head, n_groups * g.nb, pooled);
    return hipGetLastError();
}

hipError_t launch_append(const KGeom &g, const KCache &c, const void *k, const void *v,
                         int64_t stride_tok, int64_t stride_head, int n_groups, int first,
                         hipStream_t stream) {
    dim3 grid(n_groups * g.nb, g.heads);
    if (c.mfma_layout)
        append_mfma_kernel<<<grid, kThreads, 0, stream>>>(g, c, (const char *)k, (const char *)v, stride_tok, stride_head, first);
    else if (g.bf16)
        append_generic_kernel<8><<<grid, kThreads, 0, stream>>>(g, c, (const char *)k, (const char *)v, stride_tok, stride_head, first);
    else
        append_generic_kernel<4><<<grid, kThreads, 0, stream>>>(g, c, (const char *)k, (const char *)v, stride_tok, stride_head, first);
    return hipGetLastError();
}

} // namespace lcsa
