// Bandwidth-bound kernels: block mean pooling (Sec. 3.2) and the sliding-window cache
// append, which re-tiles K and V into the layout the attention kernels read and pools
// the new keys on the way.  One workgroup per (block, head); every global access is a
// 16-byte vector per lane, consecutive lanes covering consecutive bytes of a token row.
// Workgroups are numbered head-fastest: the workgroups that are dispatched together then read
// neighbouring pieces of the same token rows ([token][head][d] storage), which keeps the DRAM
// pages they open busy.
#include "lcsa_kernels.h"
#include "lcsa_pool.h"

namespace lcsa {
namespace {

using namespace pooling;

// Sliding-window eviction keeps its ring position in device memory (KCache::ring) so that a captured append
// replays into the right slots.  Thread 0 of every workgroup of an append launch reads ring[0] (the slot the
// launch's first group goes to), hands it to the workgroup through LDS, and then draws a ticket; the workgroup
// that drew the last ticket, knowing that every other workgroup has read the word, advances it when it is done.
// The ticket is requested at the start and looked at only at the end, so its latency hides behind the tile.
// A launch into an empty cache (fresh) reads nothing: it starts at slot 0 and initialises both words.
struct RingPos { int head_slot, ticket; };

// Called by every thread (holds a workgroup barrier unless the ring is not in use); word = one int of LDS.
__device__ inline RingPos ring_enter(const KCache &c, bool fresh, int *word) {
    RingPos p = {0, -1};
    if (c.order || fresh) return p;
    if (threadIdx.x == 0) *word = c.ring[0];
    __syncthreads();
    p.head_slot = *word;
    if (threadIdx.x == 0) p.ticket = atomicAdd(&c.ring[1], 1);
    return p;
}
__device__ inline void ring_leave(const KCache &c, const KGeom &g, const RingPos &p, int n_groups, bool fresh) {
    if (c.order || threadIdx.x != 0) return;
    const int next = (p.head_slot + n_groups) % g.cap;
    if (fresh) {
        if (blockIdx.x == 0) { c.ring[0] = next; c.ring[1] = 0; }
    } else if (p.ticket == (int)gridDim.x - 1) {
        c.ring[0] = next;
        c.ring[1] = 0;
    }
}

// ---------------------------------------------------------------------------------------------
// pooled[head][block][c] = mean over the block's valid tokens.      grid n_groups*nb*heads
template <int VEC>
__global__ __launch_bounds__(kThreads) void pool_kernel(KGeom g, const char *x, int64_t st, int64_t sh,
                                                        int n_blocks, float *pooled) {
    __shared__ float red[kThreads * VEC];
    const int block = blockIdx.x / g.heads, head = blockIdx.x - block * g.heads;
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
// Rotary position embedding fused with the pooling (the producer-side fusion for Q and K): one pass reads x,
// turns every channel pair (2i, 2i+1) by the angle its axis gives it (RoFormer's relative formulation, per
// (frame, row, column) axis: pair i of an axis that owns n pairs turns by position * base^(-i/n)), stores the
// rotated token in the element type and sums the STORED values, in the pooling kernel's order: the means are
// the bits lcsa_pool_blocks would give on the rotated tensor.  Frequencies and angles are formed in double: a
// streamed video reaches frame indices in the thousands, and an angle of thousands of radians formed in float
// would be off by 1e-4 and more.  The angle is reduced to [-pi, pi] in double; sine and cosine are then taken in float.
//
// A block spans tt frames, th rows and tw columns, so its tokens need only pairs_t * tt + pairs_h * th + pairs_w * tw
// distinct (cosine, sine) values: the workgroup computes that table into LDS once and every vector looks its four
// (or two) pairs up (TABLE).  A block whose table would exceed kRopeTableMax entries computes each value where it
// is used, by the same arithmetic: both paths give the same bits.
constexpr int kRopeTableMax = 4096;

struct RopeParams { int pairs_t, pairs_h, pairs_w, first_frame; double log2_base; };

// (cosine, sine) of pair i (of n on its axis) at position pos
__device__ inline float2 rope_cos_sin(int i, int n, int pos, double log2_base) {
    const double freq = exp2(-(double)i / (double)n * log2_base);
    double angle = (double)pos * freq;
    angle -= 6.283185307179586 * rint(angle * 0.15915494309189535);
    float sn, cs;
    sincosf((float)angle, &sn, &cs);
    return make_float2(cs, sn);
}

template <int VEC, bool TABLE> struct RopeTransform {
    RopeParams rp;
    const float2 *tab;           // TABLE: [pairs_t][tt], [pairs_h][th], [pairs_w][tw] one after the other
    int axis[VEC / 2];           // 0: frame, 1: row, 2: column
    int index[VEC / 2];          // pair index on its axis
    int entry[VEC / 2];          // TABLE: where this pair's positions start in tab
    int origin[3];               // first frame, row, column of the block
    char *out;
    int64_t st, sh;
    int head, j;
    __device__ uint4 apply(const uint4 &u, int frame, int row, int col, int64_t token) const {
        float f[VEC];
        Unpack<VEC>::to_float(u, f);
#pragma unroll
        for (int p = 0; p < VEC / 2; ++p) {
            const int pos = axis[p] == 0 ? frame : axis[p] == 1 ? row : col;
            float2 cs;
            if constexpr (TABLE) {
                cs = tab[entry[p] + pos - origin[axis[p]]];
            } else {
                const int n = axis[p] == 0 ? rp.pairs_t : axis[p] == 1 ? rp.pairs_h : rp.pairs_w;
                cs = rope_cos_sin(index[p], n, pos + (axis[p] == 0 ? rp.first_frame : 0), rp.log2_base);
            }
            const float a = f[2 * p], b = f[2 * p + 1];
            f[2 * p] = a * cs.x - b * cs.y;
            f[2 * p + 1] = a * cs.y + b * cs.x;
        }
        uint4 r;
        if constexpr (VEC == 8) {
            uint32_t w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                w[i] = (uint32_t)__builtin_bit_cast(unsigned short, (__bf16)f[2 * i]) |
                       (uint32_t)__builtin_bit_cast(unsigned short, (__bf16)f[2 * i + 1]) << 16;
            r = make_uint4(w[0], w[1], w[2], w[3]);
        } else {
            r = make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
        }
        *(uint4 *)(out + (token * st + (int64_t)head * sh + j * VEC) * (16 / VEC)) = r;
        return r;
    }
};

template <int VEC, bool TABLE>
__global__ __launch_bounds__(kThreads) void rope_pool_kernel(KGeom g, const char *x, int64_t st, int64_t sh, int n_blocks,
                                                             RopeParams rp, char *x_rot, int64_t rot_st, int64_t rot_sh, float *pooled) {
    __shared__ float red[kThreads * VEC];
    extern __shared__ float2 rope_table[];
    const int block = blockIdx.x / g.heads, head = blockIdx.x - block * g.heads;
    const TileRef t = tile_ref(g, block);
    const int lpr = g.d / VEC, rows_par = kThreads / lpr;
    const int rg = threadIdx.x / lpr, j = threadIdx.x - rg * lpr;
    const bool active = rg < rows_par;
    RopeTransform<VEC, TABLE> xf;
    xf.rp = rp;
    xf.tab = rope_table;
    xf.origin[0] = t.group * g.tt; xf.origin[1] = t.by * g.th; xf.origin[2] = t.bx * g.tw;
    const int len[3] = {g.tt, g.th, g.tw}, pairs[3] = {rp.pairs_t, rp.pairs_h, rp.pairs_w};
    const int start[3] = {0, rp.pairs_t * g.tt, rp.pairs_t * g.tt + rp.pairs_h * g.th};
    if (TABLE) {
        const int n_entries = start[2] + rp.pairs_w * g.tw;
        for (int e = threadIdx.x; e < n_entries; e += kThreads) {
            const int a = e < start[1] ? 0 : e < start[2] ? 1 : 2;
            const int i = (e - start[a]) / len[a], p = (e - start[a]) - i * len[a];
            rope_table[e] = rope_cos_sin(i, pairs[a], xf.origin[a] + p + (a == 0 ? rp.first_frame : 0), rp.log2_base);
        }
        __syncthreads();
    }
#pragma unroll
    for (int p = 0; p < VEC / 2; ++p) {
        const int ip = j * (VEC / 2) + p;                    // pair index within the head
        const int a = ip < rp.pairs_t ? 0 : ip < rp.pairs_t + rp.pairs_h ? 1 : 2;
        xf.axis[p] = a;
        xf.index[p] = a == 0 ? ip : a == 1 ? ip - rp.pairs_t : ip - rp.pairs_t - rp.pairs_h;
        xf.entry[p] = start[a] + xf.index[p] * len[a];
    }
    xf.out = x_rot; xf.st = rot_st; xf.sh = rot_sh; xf.head = head; xf.j = j;
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
    if (active) accumulate_block<VEC>(g, t, x, st, sh, head, rg, j, rows_par, acc, xf);
    finish_pool<VEC>(red, acc, rg, j, lpr, rows_par, active, g.d, g.tt * t.vh * t.vw,
                     pooled + ((int64_t)head * n_blocks + block) * g.d);
}

// ---------------------------------------------------------------------------------------------
// Cache append, generic tile image: K and V tiles row-major [bt][d], padded tokens zero;
// pooled K written beside them.                                      grid n_groups*nb*heads
template <int VEC>
__global__ __launch_bounds__(kThreads) void append_generic_kernel(KGeom g, KCache c, const char *k, const char *v,
                                                                  int64_t st, int64_t sh, int first, int n_groups, bool fresh) {
    __shared__ float red[kThreads * VEC];
    __shared__ int ring_word;
    const int block = blockIdx.x / g.heads, head = blockIdx.x - block * g.heads;
    const TileRef t = tile_ref(g, block);
    const RingPos ring = ring_enter(c, fresh, &ring_word);
    const int slot = c.order ? c.order[head * g.cap + first + t.group] : (ring.head_slot + t.group) % g.cap;
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
        const BlockTokens bt(g, t.vh, t.vw);
        for (int tok = rg; tok < g.bt; tok += rows_par) {
            int ft, r, cc;
            uint4 uk = make_uint4(0, 0, 0, 0), uv = uk;
            if (bt.at(tok, ft, r, cc)) {
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
    if (threadIdx.x == 0) c.v_clamped[tile_index] = 0;     // this layout stores V as given
    ring_leave(c, g, ring, n_groups, fresh);
}

// bf16 bit pattern -> IEEE half bit pattern, round to nearest even, saturating (NaN stays NaN);
// clamped counts the values that did not fit (|v| >= 65536 in bf16, infinities included)
__device__ inline uint32_t bf16_bits_to_half_bits(uint32_t b, int &clamped) {
    float f = __uint_as_float(b << 16);
    f = fminf(fmaxf(f, -65504.f), 65504.f);          // fmin/fmax return the non-NaN operand: map NaN below
    if ((b & 0x7fffu) > 0x7f80u) return 0x7e00u;      // NaN
    clamped += (b & 0x7fffu) >= 0x4780u;              // 0x4780 = 65536, the smallest bf16 magnitude above 65504
    const _Float16 h = (_Float16)f;
    return (uint32_t)__builtin_bit_cast(unsigned short, h);
}

// ---------------------------------------------------------------------------------------------
// Cache append, matrix-core tile image (bf16, d = 128, 128 tokens per tile).  Each tile is
// 128 rows of 256 bytes whose 16-byte chunk j sits at chunk position j ^ (row & 15), so the
// attention kernel can copy a tile into LDS byte for byte and read matrix operands without
// bank conflicts.  K rows are tokens (bf16 as given); V is stored transposed, rows = channels and
// columns = tokens, and as IEEE half: every bf16 value with
// magnitude in [2^-14, 65504] converts exactly (8 significant bits into 11), smaller ones round
// to half subnormals (absolute error < 2^-25), larger ones saturate to +-65504.  Half is what the
// second matrix product runs in, because softmax probabilities need mantissa, not range.  The number of
// clamped values of the block is stored beside the tile (v_clamped) so that a caller can tell.
//
// K: thread (token row rg, chunk j) moves 16-byte chunks, 16 lanes per 256-byte token row, in and out.
// V: thread (token chunk vc, channel group vj) loads an 8-token x 8-channel square (8 x 16 bytes),
// transposes it in registers and stores 8 chunks of the transposed image; vc is the fast lane index, so
// 16 lanes complete one 256-byte row of the image per store.  All 16 loads of a thread are requested before
// anything is stored.                                                grid n_groups*nb*heads
__global__ __launch_bounds__(kThreads) void append_mfma_kernel(KGeom g, KCache c, const char *__restrict__ k,
                                                               const char *__restrict__ v,
                                                               int64_t st, int64_t sh, int first, int n_groups, bool fresh) {
    __shared__ float red[16 * 128];
    __shared__ int n_clamped, ring_word;
    const int block = blockIdx.x / g.heads, head = blockIdx.x - block * g.heads;
    const TileRef t = tile_ref(g, block);
    const int rg = threadIdx.x >> 4, j = threadIdx.x & 15;     // K: 16 token rows in flight, 16 chunks per row
    const int vc = threadIdx.x & 15, vj = threadIdx.x >> 4;    // V: tokens 8vc..8vc+7, channels 8vj..8vj+7
    const bool use_ring = !c.order && !fresh;
    if (threadIdx.x == 0) {
        n_clamped = 0;
        if (use_ring) ring_word = c.ring[0];
    }
    uint4 uk[8], uv[8];
    const BlockTokens bt(g, t.vh, t.vw);
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        int ft, r, cc;
        uk[it] = make_uint4(0, 0, 0, 0);
        if (bt.at(rg + 16 * it, ft, r, cc)) {
            const int64_t token = raster_token(g, t.group, ft, t.by * g.th + r, t.bx * g.tw + cc);
            uk[it] = *(const uint4 *)(k + (token * st + (int64_t)head * sh + j * 8) * 2);
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int ft, r, cc;
        uv[i] = make_uint4(0, 0, 0, 0);
        if (bt.at(8 * vc + i, ft, r, cc)) {
            const int64_t token = raster_token(g, t.group, ft, t.by * g.th + r, t.bx * g.tw + cc);
            uv[i] = *(const uint4 *)(v + (token * st + (int64_t)head * sh + vj * 8) * 2);
        }
    }
    __syncthreads();                                   // ring_word and n_clamped are set
    RingPos ring = {use_ring ? ring_word : 0, -1};
    if (use_ring && threadIdx.x == 0) ring.ticket = atomicAdd(&c.ring[1], 1);      // looked at in ring_leave
    const int slot = c.order ? c.order[head * g.cap + first + t.group] : (ring.head_slot + t.group) % g.cap;
    const int tile = block - t.group * g.nb;
    const int64_t tile_index = ((int64_t)head * g.cap + slot) * g.nb + tile;
    char *kt = (char *)c.k + tile_index * (128 * 256);
    char *vt = (char *)c.v + tile_index * (128 * 256);

    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        const int tok = rg + 16 * it;
        float f[8];
        Unpack<8>::to_float(uk[it], f);                // zeros for padding add nothing
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += f[e];
        *(uint4 *)(kt + tok * 256 + ((j ^ (tok & 15)) << 4)) = uk[it];
    }
    // V: channel e of this thread's eight tokens -> one 16-byte chunk of row 8vj+e, at chunk position vc ^ (row & 15).
    // Whether any value needs clamping (magnitude bits >= 0x4780: 65536 and up, infinities, NaN) is looked at two
    // values per word first: x + 0x3880 carries into bit 15 exactly then.  Wavefronts that hold none, the usual case,
    // convert pairs with the packed instruction and skip the per-value range handling.
    uint32_t big = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t w4[4] = {uv[i].x, uv[i].y, uv[i].z, uv[i].w};
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) big |= ((w4[q4] & 0x7fff7fffu) + 0x38803880u) & 0x80008000u;
    }
    const bool plain = __ballot(big != 0) == 0;                // wavefront-uniform
    int clamped = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int dd = vj * 8 + e;
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint4 &a = uv[2 * i], &b = uv[2 * i + 1];
            const uint32_t wa = e < 2 ? a.x : e < 4 ? a.y : e < 6 ? a.z : a.w;
            const uint32_t wb = e < 2 ? b.x : e < 4 ? b.y : e < 6 ? b.z : b.w;
            if (plain) {
                typedef __attribute__((ext_vector_type(2))) float f32x2;
                typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
                const f32x2 f = {__uint_as_float((e & 1) ? wa & 0xffff0000u : wa << 16), __uint_as_float((e & 1) ? wb & 0xffff0000u : wb << 16)};
                w[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, f16x2));
            } else {
                const uint32_t lo = (e & 1) ? wa >> 16 : wa & 0xffffu, hi = (e & 1) ? wb >> 16 : wb & 0xffffu;
                w[i] = bf16_bits_to_half_bits(lo, clamped) | (bf16_bits_to_half_bits(hi, clamped) << 16);
            }
        }
        *(uint4 *)(vt + dd * 256 + ((vc ^ (dd & 15)) << 4)) = make_uint4(w[0], w[1], w[2], w[3]);
    }
    if (__ballot(clamped != 0)) {                      // rare: one LDS atomic per wavefront that saw any
        for (int off = 32; off > 0; off >>= 1) clamped += __shfl_xor(clamped, off);
        if ((threadIdx.x & 63) == 0) atomicAdd(&n_clamped, clamped);
    }
    finish_pool<8>(red, acc, rg, j, 16, 16, true, 128, g.tt * t.vh * t.vw, c.pooled + tile_index * 128);   // holds a barrier
    if (threadIdx.x == 0) c.v_clamped[tile_index] = (uint32_t)n_clamped;
    ring_leave(c, g, ring, n_groups, fresh);
}

} // namespace

hipError_t launch_pool(const KGeom &g, const void *x, int64_t stride_tok, int64_t stride_head,
                       int n_groups, float *pooled, hipStream_t stream) {
    dim3 grid(n_groups * g.nb * g.heads);
    if (g.bf16)
        pool_kernel<8><<<grid, kThreads, 0, stream>>>(g, (const char *)x, stride_tok, stride_head, n_groups * g.nb, pooled);
    else
        pool_kernel<4><<<grid, kThreads, 0, stream>>>(g, (const char *)x, stride_tok, stride_head, n_groups * g.nb, pooled);
    return hipGetLastError();
}

hipError_t launch_rope_pool(const KGeom &g, const void *x, int64_t st, int64_t sh, int n_groups,
                            int pairs_t, int pairs_h, float base, int first_frame,
                            void *x_rot, int64_t rot_st, int64_t rot_sh, float *pooled, hipStream_t stream) {
    dim3 grid(n_groups * g.nb * g.heads);
    const RopeParams rp = {pairs_t, pairs_h, g.d / 2 - pairs_t - pairs_h, first_frame, log2((double)base)};
    const int n_entries = rp.pairs_t * g.tt + rp.pairs_h * g.th + rp.pairs_w * g.tw;
    const bool table = n_entries <= kRopeTableMax;
    const size_t lds = table ? n_entries * sizeof(float2) : 0;
    const char *in = (const char *)x;
    char *out = (char *)x_rot;
    const int n_blocks = n_groups * g.nb;
    if (g.bf16 && table) rope_pool_kernel<8, true><<<grid, kThreads, lds, stream>>>(g, in, st, sh, n_blocks, rp, out, rot_st, rot_sh, pooled);
    else if (g.bf16) rope_pool_kernel<8, false><<<grid, kThreads, 0, stream>>>(g, in, st, sh, n_blocks, rp, out, rot_st, rot_sh, pooled);
    else if (table) rope_pool_kernel<4, true><<<grid, kThreads, lds, stream>>>(g, in, st, sh, n_blocks, rp, out, rot_st, rot_sh, pooled);
    else rope_pool_kernel<4, false><<<grid, kThreads, 0, stream>>>(g, in, st, sh, n_blocks, rp, out, rot_st, rot_sh, pooled);
    return hipGetLastError();
}

hipError_t launch_append(const KGeom &g, const KCache &c, const void *k, const void *v,
                         int64_t stride_tok, int64_t stride_head, int n_groups, int first, bool fresh,
                         hipStream_t stream) {
    dim3 grid(n_groups * g.nb * g.heads);
    if (c.mfma_layout)
        append_mfma_kernel<<<grid, kThreads, 0, stream>>>(g, c, (const char *)k, (const char *)v, stride_tok, stride_head, first, n_groups, fresh);
    else if (g.bf16)
        append_generic_kernel<8><<<grid, kThreads, 0, stream>>>(g, c, (const char *)k, (const char *)v, stride_tok, stride_head, first, n_groups, fresh);
    else
        append_generic_kernel<4><<<grid, kThreads, 0, stream>>>(g, c, (const char *)k, (const char *)v, stride_tok, stride_head, first, n_groups, fresh);
    return hipGetLastError();
}

} // namespace lcsa
