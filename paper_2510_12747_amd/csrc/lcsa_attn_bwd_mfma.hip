// Backward of the block-sparse attention on the gfx950 matrix cores (bf16, d = 128, 128-token blocks).
// Same mathematics as lcsa_attn_bwd.hip (selection held fixed; Sec. 3.2 "Stage 2", eq. 1):
//     p_ij = exp(scale q_i.k_j - lse_i),  t_ij = g_i.v_j,  D_i = sum_j p_ij t_ij,  u_ij = scale p_ij (t_ij - D_i),
//     dq_i = sum_j u_ij k_j,   dk_j = sum_i u_ij q_i,   dv_j = sum_i p_ij g_i          (g = dL/do)
// with every product a v_mfma_f32_32x32x16_bf16 (float accumulation); p and u enter the second-level products
// rounded to bf16, everything else (exponentials, D, the accumulators, the results) is float.  Fixed summation
// orders, no atomics: results are reproducible bit for bit.
//
// Tiles.  A 128-token x 128-channel bf16 tile lives in LDS as 128 rows of 256 bytes, the 16-byte chunk j of row r
// at chunk position j ^ sw(r), sw(r) = the low four bits of r rotated left by one.  It is copied there straight
// from the raster tensor by direct-to-LDS loads (a wavefront instruction moves 4 rows: lane t lands at byte 16 t of
// them and fetches the chunk that belongs there; rows beyond the block's valid tokens fetch zeros), two tiles per
// step into one of two buffers, so that the next block's tiles arrive while the current block is computed.
// All products have the form C[m][n] = sum_k A[m][k] B[n][k].  Where the summed index runs along the rows of the
// tile (first level: over channels), an operand fragment is one ds_read_b128 of a row; where it runs down the
// columns (second level: over keys or queries), the fragment comes from two transposing reads (ds_read_b64_tr_b16:
// 16 lanes fetch 4 rows x 16 columns and each receives 4 consecutive rows of one column), so no transposed copy of
// a tile is ever built.  sw() spreads both kinds of read over the banks: 16 rows with distinct low bits map to 16
// distinct chunk positions (the row reads are conflict free by the hardware counters), and 4 consecutive rows map to
// 4 distinct 32-byte positions (the transposing reads still show about one conflict cycle in four).
//
// Operand reuse without LDS round trips: the rows fed to the matrix rows of a first-level product (S or S^T) are
// permuted (bits 2 and 3 of the row index swapped), which makes the 8 accumulator registers 8s..8s+7 of a lane
// hold 8 consecutive indices of the summed dimension of the second-level product: the accumulator, rounded to
// bf16, IS the A operand of that product.
//
//   bwd_delta_mfma_kernel workgroup = (head, query block): D_i = sum_j p_ij t_ij over the kept key blocks (stored in
//                         `delta`), formed from unrounded p and t in float.
//   bwd_dq_mfma_kernel    workgroup = (head, query block), wavefront w owns queries 32w..32w+31 (their Q and dO
//                         fragments stay in registers as B operands): u from D, dQ += u K.
//   bwd_dkv_mfma_kernel   workgroup = (head, key block), wavefront w owns keys 32w..32w+31 (K and V fragments in
//                         registers).  Walks the query blocks that kept this block (ascending), per query block
//                         the Q and dO tiles: dV += P^T dO, dK += U^T Q.
// Every matrix instruction takes one 1 KB operand fragment from LDS (the 64-bit transposing reads at less than half
// the rate of the 128-bit row reads), and every kernel fetches 64 KB of tiles per block pair from L2.
#include "lcsa_kernels.h"

#include <type_traits>

namespace lcsa {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short i16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kThreads = 256;
constexpr int kTileBytes = 128 * 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr int kMaxQueryBlocks = 8192;        // flags of the key-block kernel

#define LCSA_LDS __attribute__((address_space(3)))

// what padding rows of a tile are copied from
__device__ __attribute__((aligned(256))) const unsigned char zero_row[256] = {};

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
// raster token of the first token of a block; token i of the block lies rel_token(i) further on
__device__ inline int64_t block_origin(const KGeom &g, const BlockRef &b) { return raster_token(g, b.group, 0, b.by * g.th, b.bx * g.tw); }
// distance, in raster tokens, from a block's first token to its i-th valid token (valid tokens first, in
// (frame, row, column) order over the block's clipped extent vh x vw); -1 beyond the valid tokens
__device__ inline int rel_token(const KGeom &g, int vh, int vw, int i) {
    int ft, r, c;
    return block_token(g, i, vh, vw, ft, r, c) ? (ft * g.H + r) * g.W + c : -1;
}
__device__ inline int64_t token_of(const KGeom &g, const BlockRef &b, int i) { return block_origin(g, b) + rel_token(g, b.vh, b.vw, i); }

// chunk position swizzle of a tile image and the byte offset of 16-byte chunk `chunk` of row `row`
__device__ inline int sw(int row) { return ((row & 7) << 1) | ((row >> 3) & 1); }
__device__ inline int img_off(int row, int chunk) { return row * 256 + ((chunk ^ sw(row)) << 4); }
// matrix row m of a first-level product reads tile row swap23(m)
__device__ inline int swap23(int m) { return (m & 0x13) | ((m & 4) << 1) | ((m & 8) >> 1); }

// operand fragment along a row: elements 8 chunk .. 8 chunk + 7 of row `row`
__device__ inline bf16x8 frag(const unsigned char *img, int row, int chunk) { return *(const bf16x8 *)(img + img_off(row, chunk)); }

// Operand fragment down a column.  Lane (n = lane & 31, half = lane >> 5) receives column col0 + n, rows
// row0 + 8 half .. + 7.  A transposing read serves 16 lanes at a time: lane i of the 16 points at 4 elements of row
// (first + i / 4), columns (c16 + 4 (i % 4) ..), and receives rows first .. first + 3 of column c16 + i.
__device__ inline bf16x8 frag_down(const unsigned char *img, int row0, int col0, int lane) {
    const int i = lane & 15, c16 = col0 + (lane & 16), half = lane >> 5;
    const int chunk = (c16 >> 3) + ((i >> 1) & 1), sub = (i & 1) * 8;
    const int ra = row0 + 8 * half + (i >> 2), rb = ra + 4;
    const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LCSA_LDS i16x4 *)(img + img_off(ra, chunk) + sub));
    const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LCSA_LDS i16x4 *)(img + img_off(rb, chunk) + sub));
    typedef __attribute__((ext_vector_type(8))) short i16x8;
    const i16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, both);
}

// B-operand fragments of the 32 rows a wavefront owns, straight from the raster tensor: lane (n, half) holds
// x[token(first + n)][16 ks + 8 half .. + 8] for ks = 0..7; rows beyond the block's valid tokens are zeros
__device__ inline void load_own_rows(const KGeom &g, const BlockRef &b, const __bf16 *__restrict__ x, int64_t st, int64_t sh, int head,
                                     int first, int lane, bf16x8 (&f)[8]) {
    const int n = lane & 31, half = lane >> 5;
    const bool ok = first + n < b.n_valid;
    const __bf16 *p = x + (ok ? token_of(g, b, first + n) : 0) * st + (int64_t)head * sh + half * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const uint4 u = ok ? *(const uint4 *)(p + ks * 16) : make_uint4(0, 0, 0, 0);
        f[ks] = __builtin_bit_cast(bf16x8, u);
    }
}

// ---- tile copies -------------------------------------------------------------------------------------------------
// A wavefront copies rows 32 wave .. 32 wave + 31 of a tile with 8 instructions; instruction i moves rows
// 32 wave + 4 i .. + 3, lane t supplying row (t >> 4), chunk position (t & 15).  RowPlan holds, for the 8 rows of a
// lane, the distance of the row's token from the block's first token (-1: padding row) for one block extent; the
// plan of the unclipped extent is made once, clipped blocks make their own.
template <int WAVES> struct RowPlan { int rel[32 / WAVES]; };
template <int WAVES>
__device__ inline RowPlan<WAVES> plan_rows(const KGeom &g, int vh, int vw, int wave, int lane) {
    RowPlan<WAVES> p;
#pragma unroll
    for (int i = 0; i < 32 / WAVES; ++i) p.rel[i] = rel_token(g, vh, vw, (128 / WAVES) * wave + 4 * i + (lane >> 4));
    return p;
}
// One copy instruction: 64 lanes x 16 bytes from per-lane addresses to LDS bytes lds_rows + 16 lane.  The load
// stays in flight (counted by vmcnt) until waited for; nothing else orders it.
__device__ inline void copy_rows_to_lds(const void *src, uint32_t lds_rows) {
    lds_rows = __builtin_amdgcn_readfirstlane(lds_rows);     // wavefront-uniform already; this pins it to a scalar register
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" :: "v"(src), "s"(lds_rows) : "memory", "m0");
}
// Copies this wavefront's rows (128 / WAVES of them) of the tiles of block `b` of two tensors (K and V, or Q and dO);
// x1 = the second tensor moved so that the first tensor's strides reach its elements too when the two share
// strides (`same`, the usual case: one address computation serves both), else its own base with strides st1, sh1.
template <int WAVES>
__device__ inline void copy_tiles(const KGeom &g, const BlockRef &b, const RowPlan<WAVES> &full, int wave, int lane,
                                  const __bf16 *__restrict__ x0, const __bf16 *__restrict__ x1, int64_t st, int64_t sh, int head,
                                  uint32_t lds0, uint32_t lds1, bool same = true, int64_t st1 = 0, int64_t sh1 = 0) {
    RowPlan<WAVES> plan = full;
    if (b.vh != g.th || b.vw != g.tw) plan = plan_rows<WAVES>(g, b.vh, b.vw, wave, lane);     // workgroup-uniform
    const int64_t origin = block_origin(g, b);
    const int slot = lane & 15, q4 = lane >> 4;
    const int first = (128 / WAVES) * wave;                  // a multiple of 16: its low bits do not enter sw()
#pragma unroll
    for (int i = 0; i < 32 / WAVES; ++i) {
        const int chunk = slot ^ sw(4 * i + q4);
        const int64_t at = ((origin + plan.rel[i]) * st + (int64_t)head * sh + chunk * 8) * 2;
        const int64_t at1 = same ? at : ((origin + plan.rel[i]) * st1 + (int64_t)head * sh1 + chunk * 8) * 2;      // `same` is workgroup-uniform
        const bool ok = plan.rel[i] >= 0;
        const void *s0 = ok ? (const void *)((const char *)x0 + at) : (const void *)(zero_row + chunk * 16);
        const void *s1 = ok ? (const void *)((const char *)x1 + at1) : (const void *)(zero_row + chunk * 16);
        const uint32_t rows = (uint32_t)(first + 4 * i) * 256;
        copy_rows_to_lds(s0, lds0 + rows);
        copy_rows_to_lds(s1, lds1 + rows);
    }
}
__device__ inline uint32_t lds_address(const unsigned char *p) { return (uint32_t)(uintptr_t)((LCSA_LDS unsigned char *)p); }

// all of this wavefront's tile copies have landed; then a workgroup barrier: everybody's have, and everybody is
// done with the buffer that the next copies will overwrite
__device__ inline void tiles_ready() { asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Launch order.  Workgroups are dealt to the 8 XCDs round-robin, each with an L2 of its own; workgroup ids are
// mapped so that an XCD walks a contiguous run of (head, tile, frame group) items: neighbouring tiles of a head keep
// (or are kept by) nearly the same blocks, whose tiles are then found in that XCD's L2.
__device__ inline bool work_item(const KGeom &g, int groups, int per_xcd, int &head, int &block) {
    const int item = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (item >= g.heads * groups * g.nb) return false;
    head = item / (groups * g.nb);
    const int rem = item - head * groups * g.nb;
    const int tile = rem / groups, grp = rem - tile * groups;
    block = grp * g.nb + tile;
    return true;
}

__device__ inline void zero(f32x16 &a) {
#pragma unroll
    for (int i = 0; i < 16; ++i) a[i] = 0.f;
}

// ---------------------------------------------------------------------------------------------------------------
// D_i = sum_j p_ij t_ij.  Eight wavefronts, two per SIMD, so that one wavefront's matrix products run beside the
// other's LDS reads and exponentials: wavefront w owns queries 32 (w & 3) .. + 31 and, of every kept key block, the
// 32-key units 2 (w >> 2) and 2 (w >> 2) + 1; the two partial sums of a query meet in LDS at the end.
__global__ __launch_bounds__(512) void bwd_delta_mfma_kernel(
    KGeom g, int kv_groups, const __bf16 *__restrict__ q, int64_t q_st, int64_t q_sh,
    const __bf16 *__restrict__ k, const __bf16 *__restrict__ v, int64_t kv_st, int64_t kv_sh,
    const int32_t *__restrict__ sel_idx, const int32_t *__restrict__ sel_cnt,
    const __bf16 *__restrict__ d_o, int64_t o_st, int64_t o_sh, const float *__restrict__ lse,
    float *__restrict__ delta, float scale, int per_xcd) {
    __shared__ __attribute__((aligned(16))) unsigned char img[2][2][kTileBytes];      // [buffer][K, V]
    __shared__ float part[128];
    int qb, head;
    if (!work_item(g, g.q_groups, per_xcd, head, qb)) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), qg = wave & 3, kh = wave >> 2;
    const int ql = lane & 31, half = lane >> 5;
    const int n_qb = g.q_groups * g.nb;
    const BlockRef qr = block_ref(g, qb);
    const int64_t row = (int64_t)head * n_qb + qb;
    const int cnt = min(max(sel_cnt[row], 0), g.topk);
    const int32_t *sel = sel_idx + row * g.topk;
    const float scale_log2 = scale * kLog2e;
    const uint32_t lds_img = lds_address(&img[0][0][0]);
    const RowPlan<8> full = plan_rows<8>(g, g.th, g.tw, wave, lane);

    bf16x8 qf[8], gf[8];
    load_own_rows(g, qr, q, q_st, q_sh, head, 32 * qg, lane, qf);
    load_own_rows(g, qr, d_o, o_st, o_sh, head, 32 * qg, lane, gf);
    const bool q_ok = 32 * qg + ql < qr.n_valid;
    const int64_t q_token = token_of(g, qr, q_ok ? 32 * qg + ql : 0);
    const float l2 = q_ok ? lse[q_token * g.heads + head] * kLog2e : __builtin_inff();   // padding queries: probability zero
    auto key_block = [&](int b) { return block_ref(g, min(max(sel[b], 0), kv_groups * g.nb - 1)); };
    auto copy_block = [&](const BlockRef &kr, int buf) {
        copy_tiles<8>(g, kr, full, wave, lane, k, v, kv_st, kv_sh, head, lds_img + buf * 2 * kTileBytes, lds_img + (buf * 2 + 1) * kTileBytes);
    };
    __builtin_amdgcn_s_waitcnt(0x0F70);                      // vmcnt(0), where the compiler sees it: no wait of its own inside the loop

    float dsum = 0.f;
    BlockRef kr = key_block(0);
    if (cnt > 0) copy_block(kr, 0);
    for (int b = 0; b < cnt; ++b) {
        tiles_ready();
        const int n_keys = kr.n_valid;
        if (b + 1 < cnt) { kr = key_block(b + 1); copy_block(kr, (b + 1) & 1); }
        const unsigned char *k_img = img[b & 1][0], *v_img = img[b & 1][1];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int mt = 2 * kh + u;
            if (mt * 32 < n_keys) {
                const int arow = mt * 32 + swap23(ql);
                bf16x8 ka[8], va[8];
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) { ka[ks] = frag(k_img, arow, 2 * ks + half); va[ks] = frag(v_img, arow, 2 * ks + half); }
                __builtin_amdgcn_sched_barrier(0);
                f32x16 st_, dpt;
                zero(st_); zero(dpt);
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    st_ = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qf[ks], st_, 0, 0, 0);
                    dpt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ks], gf[ks], dpt, 0, 0, 0);
                }
                // register 8 kk + j = key mt*32 + 16 kk + 8 half + j; keys beyond the valid ones get probability zero
                const int left = n_keys - (mt * 32 + 8 * half);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(st_[r], scale_log2, -l2));
                    dsum = fmaf((r >> 3) * 16 + (r & 7) < left ? p : 0.f, dpt[r], dsum);
                }
            }
        }
    }
    const float d = dsum + __shfl_xor(dsum, 32);             // the two half-waves hold the two halves of a unit's keys
    if (kh == 1 && half == 0) part[32 * qg + ql] = d;
    __syncthreads();
    if (kh == 0 && half == 0 && q_ok) delta[q_token * g.heads + head] = d + part[32 * qg + ql];
}

// ---------------------------------------------------------------------------------------------------------------
// dQ += u K over the kept key blocks, with D_i read from `delta`.  Four wavefronts, one per SIMD (the accumulators
// and both operand sets of a unit do not fit twice), software-pipelined instead.
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void bwd_dq_mfma_kernel(
    KGeom g, int kv_groups, const __bf16 *__restrict__ q, int64_t q_st, int64_t q_sh,
    const __bf16 *__restrict__ k, const __bf16 *__restrict__ v, int64_t kv_st, int64_t kv_sh,
    const int32_t *__restrict__ sel_idx, const int32_t *__restrict__ sel_cnt,
    const __bf16 *__restrict__ d_o, int64_t o_st, int64_t o_sh, const float *__restrict__ lse,
    float *__restrict__ d_q, const float *__restrict__ delta, float scale, int per_xcd) {
    __shared__ __attribute__((aligned(16))) unsigned char img[2][2][kTileBytes];      // [buffer][K, V]
    int qb, head;
    if (!work_item(g, g.q_groups, per_xcd, head, qb)) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ql = lane & 31, half = lane >> 5;
    const int n_qb = g.q_groups * g.nb;
    const BlockRef qr = block_ref(g, qb);
    const int64_t row = (int64_t)head * n_qb + qb;
    const int cnt = min(max(sel_cnt[row], 0), g.topk);
    const int32_t *sel = sel_idx + row * g.topk;
    const float scale_log2 = scale * kLog2e;
    const uint32_t lds_img = lds_address(&img[0][0][0]);
    const RowPlan<4> full = plan_rows<4>(g, g.th, g.tw, wave, lane);

    // this wavefront's queries: Q and dO fragments (B operands), lse and the token to write to
    bf16x8 qf[8], gf[8];
    load_own_rows(g, qr, q, q_st, q_sh, head, 32 * wave, lane, qf);
    load_own_rows(g, qr, d_o, o_st, o_sh, head, 32 * wave, lane, gf);
    const bool q_ok = 32 * wave + ql < qr.n_valid;
    const int64_t q_token = token_of(g, qr, q_ok ? 32 * wave + ql : 0);
    // padding queries: an infinite reference makes every probability zero
    const float l2 = q_ok ? lse[q_token * g.heads + head] * kLog2e : __builtin_inff();

    auto key_block = [&](int b) {
        return block_ref(g, min(max(sel[b], 0), kv_groups * g.nb - 1));   // ids outside the visible blocks must not become wild addresses
    };
    auto copy_block = [&](const BlockRef &kr, int buf) {
        copy_tiles<4>(g, kr, full, wave, lane, k, v, kv_st, kv_sh, head, lds_img + buf * 2 * kTileBytes, lds_img + (buf * 2 + 1) * kTileBytes);
    };
    const float D = q_ok ? delta[q_token * g.heads + head] : 0.f;
    // All loads so far are waited for here, where the compiler sees it: left to itself it would wait at their first
    // use inside the loop, on every trip, and each such wait also drains the tile copies in flight (they share the counter).
    __builtin_amdgcn_s_waitcnt(0x0F70);                      // vmcnt(0)
    f32x16 dq[4];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) zero(dq[nt]);

    // Operand reads of the 32-key unit mt of the tiles in `k_img`, `v_img`.
    auto read_a = [&](const unsigned char *k_img, const unsigned char *v_img, int mt, bf16x8 (&ka)[8], bf16x8 (&va)[8]) {
        const int arow = mt * 32 + swap23(ql);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) { ka[ks] = frag(k_img, arow, 2 * ks + half); va[ks] = frag(v_img, arow, 2 * ks + half); }
    };
    auto read_b = [&](const unsigned char *k_img, int mt, bf16x8 (&kb_)[8]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) kb_[i] = frag_down(k_img, mt * 32 + 16 * (i & 1), (i >> 1) * 32, lane);
    };
    // first level: S^T = K Q^T and (dO V^T)^T = V dO^T for 32 keys x this wavefront's 32 queries
    auto first_level = [&](const bf16x8 (&ka)[8], const bf16x8 (&va)[8], f32x16 &st_, f32x16 &dpt) {
        zero(st_); zero(dpt);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            st_ = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qf[ks], st_, 0, 0, 0);
            dpt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ks], gf[ks], dpt, 0, 0, 0);
        }
    };
    // lane = query ql; register 8 kk + j = key mt*32 + 16 kk + 8 half + j.  Keys beyond the block's valid ones (zero
    // rows of the tiles) must get probability zero; only a block's last unit can hold any (MASK): `left` = valid keys
    // from this lane's first one on.
    auto prob = [&](float s_, bool mask, int idx, int left) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s_, scale_log2, -l2));
        return mask && idx >= left ? 0.f : p;
    };

    // A block is walked in 32-key units, software-pipelined so that the matrix pipe, the vector pipe and the LDS reads
    // of neighbouring units run side by side:
    //     first level(mt), reads A(mt+1) | element-wise(mt) || second level(mt-1) | reads B(mt)
    auto block_units = [&](auto n_tag, const unsigned char *k_img, const unsigned char *v_img, int n_keys) {
        constexpr int N = decltype(n_tag)::value;
        bf16x8 ka[8], va[8], kb_[8], ua[2];
        f32x16 st_, dpt;
        const float d_scaled = D * scale;
        read_a(k_img, v_img, 0, ka, va);
#pragma unroll
        for (int mt = 0; mt <= N; ++mt) {
            if (mt < N) {
                __builtin_amdgcn_sched_barrier(0);
                first_level(ka, va, st_, dpt);
                __builtin_amdgcn_sched_barrier(0);
                if (mt + 1 < N) read_a(k_img, v_img, mt + 1, ka, va);
            }
            __builtin_amdgcn_sched_barrier(0);
            bf16x8 un[2];
            if (mt < N) {
                const int left = n_keys - (mt * 32 + 8 * half);
#pragma unroll
                for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const int r = kk * 8 + j;
                        un[kk][j] = (__bf16)(prob(st_[r], mt == N - 1, 16 * kk + j, left) * fmaf(dpt[r], scale, -d_scaled));
                    }
            }
            if (mt > 0) {
#pragma unroll
                for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk)
                        dq[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua[kk], kb_[nt * 2 + kk], dq[nt], 0, 0, 0);
            }
            if (mt > 0 && mt < N) {
#pragma unroll
                for (int n = 0; n < 8; ++n) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 9, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (mt < N) { read_b(k_img, mt, kb_); ua[0] = un[0]; ua[1] = un[1]; }
        }
    };

    BlockRef kr = key_block(0);
    if (cnt > 0) copy_block(kr, 0);
    for (int b = 0; b < cnt; ++b) {
        tiles_ready();                                       // block b is in buffer b & 1; nobody reads the other buffer any more
        const int n_keys = kr.n_valid;
        if (b + 1 < cnt) { kr = key_block(b + 1); copy_block(kr, (b + 1) & 1); }
        const unsigned char *k_img = img[b & 1][0], *v_img = img[b & 1][1];
        auto units = [&](auto n_tag) { block_units(n_tag, k_img, v_img, n_keys); };
        switch ((n_keys + 31) >> 5) {                        // 32-key units that hold valid keys
        case 4: units(std::integral_constant<int, 4>()); break;
        case 3: units(std::integral_constant<int, 3>()); break;
        case 2: units(std::integral_constant<int, 2>()); break;
        default: units(std::integral_constant<int, 1>()); break;
        }
    }
    // dq tile nt: lane = channel nt*32 + ql, register r = query row 8 (r >> 2) + 4 half + (r & 3) of this wavefront
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int qi = 32 * wave + 8 * (r >> 2) + 4 * half + (r & 3);
        if (qi < qr.n_valid) {
            float *out = d_q + (token_of(g, qr, qi) * g.heads + head) * 128 + ql;
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) out[nt * 32] = dq[nt][r];
        }
    }
}

// ---------------------------------------------------------------------------------------------------------------
// SAME_STRIDES: Q and dO share their strides (the usual case: one address computation per copied row serves both).
template <bool SAME_STRIDES>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void bwd_dkv_mfma_kernel(
    KGeom g, int kv_groups, const __bf16 *__restrict__ q, int64_t q_st, int64_t q_sh,
    const __bf16 *__restrict__ k, const __bf16 *__restrict__ v, int64_t kv_st, int64_t kv_sh,
    const int32_t *__restrict__ sel_idx, const int32_t *__restrict__ sel_cnt,
    const __bf16 *__restrict__ d_o, int64_t o_st, int64_t o_sh, const float *__restrict__ lse, const float *__restrict__ delta,
    float *__restrict__ d_k, float *__restrict__ d_v, float scale, int per_xcd) {
    __shared__ __attribute__((aligned(16))) unsigned char img[2][2][kTileBytes];      // [buffer][Q, dO]
    __shared__ float l2_s[2][128], D_s[2][128];
    __shared__ unsigned char kept_by[kMaxQueryBlocks];
    int kb, head;
    if (!work_item(g, kv_groups, per_xcd, head, kb)) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ql = lane & 31, half = lane >> 5;
    const int n_qb = g.q_groups * g.nb;
    const BlockRef kr = block_ref(g, kb);
    const float scale_log2 = scale * kLog2e;
    const uint32_t lds_img = lds_address(&img[0][0][0]);
    const RowPlan<4> full = plan_rows<4>(g, g.th, g.tw, wave, lane);

    // which query blocks kept this key block?  (ascending id lists: binary search)
    for (int qb = tid; qb < n_qb; qb += kThreads) {
        const int64_t row = (int64_t)head * n_qb + qb;
        const int32_t *sel = sel_idx + row * g.topk;
        const int c = min(max(sel_cnt[row], 0), g.topk);
        int lo = 0, hi = c;
        while (lo < hi) { const int mid = (lo + hi) >> 1; if (sel[mid] < kb) lo = mid + 1; else hi = mid; }
        kept_by[qb] = lo < c && sel[lo] == kb;
    }
    // this wavefront's keys: K and V fragments (B operands of the first-level products)
    bf16x8 kf[8], vf[8];
    load_own_rows(g, kr, k, kv_st, kv_sh, head, 32 * wave, lane, kf);
    load_own_rows(g, kr, v, kv_st, kv_sh, head, 32 * wave, lane, vf);
    const bool key_ok = 32 * wave + ql < kr.n_valid;
    f32x16 dk[4], dv[4];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) { zero(dk[nt]); zero(dv[nt]); }
    __builtin_amdgcn_s_waitcnt(0x0F70);                      // vmcnt(0), where the compiler sees it (see the query-side kernel)
    __syncthreads();

    auto next_kept = [&](int from) { while (from < n_qb && !kept_by[from]) ++from; return from; };   // uniform
    int qb = next_kept(0);
    float l2_next = 0.f, D_next = 0.f;
    auto request = [&](int qb_, int buf) {                   // a query block's tiles, lse and D
        const BlockRef qr = block_ref(g, qb_);
        copy_tiles<4>(g, qr, full, wave, lane, q, d_o, q_st, q_sh, head, lds_img + buf * 2 * kTileBytes, lds_img + (buf * 2 + 1) * kTileBytes,
                      SAME_STRIDES, o_st, o_sh);
        if (tid < 128) {
            const bool ok = tid < qr.n_valid;
            const int64_t token = token_of(g, qr, ok ? tid : 0);
            l2_next = ok ? lse[token * g.heads + head] * kLog2e : __builtin_inff();   // padding queries: probability zero
            D_next = ok ? delta[token * g.heads + head] : 0.f;
        }
    };
    int buf = 0;
    if (qb < n_qb) request(qb, 0);
    while (qb < n_qb) {
        const int n_queries = block_ref(g, qb).n_valid;
        // buffer `buf` of the per-query values was last read two blocks ago, before the previous barrier
        if (tid < 128) { l2_s[buf][tid] = l2_next; D_s[buf][tid] = D_next; }
        tiles_ready();
        qb = next_kept(qb + 1);
        if (qb < n_qb) request(qb, buf ^ 1);                 // lands while this block is computed
        const unsigned char *q_img = img[buf][0], *g_img = img[buf][1];
        const float *l2_b = l2_s[buf], *D_b = D_s[buf];
        const int n_units = (n_queries + 31) >> 5;           // 32-query units that hold valid queries
        // Software pipeline over the units (a wavefront has its SIMD to itself): the element-wise work of unit mt
        // runs beside the second-level products of unit mt - 1:
        //     first level(mt), reads A(mt+1) | element-wise(mt) || second level(mt-1) | reads B(mt)
        bf16x8 qa[8], ga[8], gb[8], qb_[8], pa[2], ua[2];
        auto read_a = [&](int mt) {
            const int arow = mt * 32 + swap23(ql);
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) { qa[ks] = frag(q_img, arow, 2 * ks + half); ga[ks] = frag(g_img, arow, 2 * ks + half); }
        };
        // lane = key ql of this wavefront; register 8 kk + j = query mt*32 + 16 kk + 8 half + j
        auto element_wise = [&](int mt, const f32x16 &s, const f32x16 &dp, bf16x8 (&pn)[2], bf16x8 (&un)[2]) {
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const int q0 = mt * 32 + 16 * kk + 8 * half;
                const float4 la = *(const float4 *)(l2_b + q0), lb = *(const float4 *)(l2_b + q0 + 4);
                const float4 da = *(const float4 *)(D_b + q0), db = *(const float4 *)(D_b + q0 + 4);
                const float l8[8] = {la.x, la.y, la.z, la.w, lb.x, lb.y, lb.z, lb.w};
                const float d8[8] = {da.x, da.y, da.z, da.w, db.x, db.y, db.z, db.w};
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int r = kk * 8 + j;
                    float p = __builtin_amdgcn_exp2f(fmaf(s[r], scale_log2, -l8[j]));
                    p = key_ok ? p : 0.f;
                    pn[kk][j] = (__bf16)p;
                    un[kk][j] = (__bf16)(p * ((dp[r] - d8[j]) * scale));
                }
            }
        };
        auto second_level = [&]() {
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    dv[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa[kk], gb[nt * 2 + kk], dv[nt], 0, 0, 0);
                    dk[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua[kk], qb_[nt * 2 + kk], dk[nt], 0, 0, 0);
                }
        };
        read_a(0);
        for (int mt = 0; mt < n_units; ++mt) {
            __builtin_amdgcn_sched_barrier(0);
            f32x16 s, dp;
            zero(s); zero(dp);
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[ks], kf[ks], s, 0, 0, 0);
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga[ks], vf[ks], dp, 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (mt + 1 < n_units) read_a(mt + 1);            // arrives under the element-wise part and the second-level products
            __builtin_amdgcn_sched_barrier(0);
            bf16x8 pn[2], un[2];
            if (mt > 0) {
                element_wise(mt, s, dp, pn, un);
                second_level();
#pragma unroll
                for (int n = 0; n < 16; ++n) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
                }
            } else {
                element_wise(mt, s, dp, pn, un);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                gb[i] = frag_down(g_img, mt * 32 + 16 * (i & 1), (i >> 1) * 32, lane);
                qb_[i] = frag_down(q_img, mt * 32 + 16 * (i & 1), (i >> 1) * 32, lane);
            }
            pa[0] = pn[0]; pa[1] = pn[1]; ua[0] = un[0]; ua[1] = un[1];
        }
        __builtin_amdgcn_sched_barrier(0);
        second_level();                                      // of the block's last unit
        buf ^= 1;
    }
    // tile nt: lane = channel nt*32 + ql, register r = key row 8 (r >> 2) + 4 half + (r & 3) of this wavefront
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int ki = 32 * wave + 8 * (r >> 2) + 4 * half + (r & 3);
        if (ki < kr.n_valid) {
            const int64_t o = (token_of(g, kr, ki) * g.heads + head) * 128 + ql;
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) { d_k[o + nt * 32] = dk[nt][r]; d_v[o + nt * 32] = dv[nt][r]; }
        }
    }
}

} // namespace

bool attn_bwd_mfma_supported(const KGeom &g) {
    return g.bf16 && g.d == 128 && g.bt == 128 && g.q_groups * g.nb <= kMaxQueryBlocks;
}

hipError_t launch_attn_bwd_mfma(const KGeom &g, int kv_groups, const void *q, int64_t q_st, int64_t q_sh,
                                const void *k, const void *v, int64_t kv_st, int64_t kv_sh,
                                const int32_t *sel_idx, const int32_t *sel_cnt,
                                const void *d_o, int64_t o_st, int64_t o_sh, const float *lse,
                                float *d_q, float *d_k, float *d_v, float *delta, float scale, hipStream_t stream) {
    const int q_per_xcd = (g.q_groups * g.nb * g.heads + 7) / 8, k_per_xcd = (kv_groups * g.nb * g.heads + 7) / 8;
    const dim3 grid_q(q_per_xcd * 8), grid_k(k_per_xcd * 8);
    bwd_delta_mfma_kernel<<<grid_q, 512, 0, stream>>>(g, kv_groups, (const __bf16 *)q, q_st, q_sh, (const __bf16 *)k, (const __bf16 *)v,
                                                      kv_st, kv_sh, sel_idx, sel_cnt, (const __bf16 *)d_o, o_st, o_sh, lse, delta, scale, q_per_xcd);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    bwd_dq_mfma_kernel<<<grid_q, kThreads, 0, stream>>>(g, kv_groups, (const __bf16 *)q, q_st, q_sh, (const __bf16 *)k, (const __bf16 *)v,
                                                           kv_st, kv_sh, sel_idx, sel_cnt, (const __bf16 *)d_o, o_st, o_sh, lse, d_q, delta, scale, q_per_xcd);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (q_st == o_st && q_sh == o_sh)
        bwd_dkv_mfma_kernel<true><<<grid_k, kThreads, 0, stream>>>(g, kv_groups, (const __bf16 *)q, q_st, q_sh, (const __bf16 *)k, (const __bf16 *)v,
                                                                   kv_st, kv_sh, sel_idx, sel_cnt, (const __bf16 *)d_o, o_st, o_sh, lse, delta,
                                                                   d_k, d_v, scale, k_per_xcd);
    else
        bwd_dkv_mfma_kernel<false><<<grid_k, kThreads, 0, stream>>>(g, kv_groups, (const __bf16 *)q, q_st, q_sh, (const __bf16 *)k, (const __bf16 *)v,
                                                                    kv_st, kv_sh, sel_idx, sel_cnt, (const __bf16 *)d_o, o_st, o_sh, lse, delta,
                                                                    d_k, d_v, scale, k_per_xcd);
    return hipGetLastError();
}

} // namespace lcsa
