// Block-sparse flash attention on the gfx950 matrix cores (bf16, d = 128, 128-token blocks).
//
// One workgroup (4 wavefronts) owns one (head, query block); wavefront w owns query rows
// 32w .. 32w+31.  For each selected key block the K tile and the transposed V tile (each a
// 32 KB byte-for-byte LDS image prepared by the cache append) are streamed into LDS with
// direct-to-LDS loads, and the wavefront computes
//     S^T = K Q^T          v_mfma_f32_32x32x16_bf16  (keys on the row axis, queries on lanes)
//     O^T += V^T P^T       v_mfma_f32_32x32x16_f16   (channels on the row axis, queries on lanes)
// The second product runs in IEEE half (same matrix-core rate as bf16): probabilities lie in
// [0,1] and need mantissa rather than range, which cuts the kernel's dominant rounding error
// (bf16 P) by 8x; V was converted to half, exactly for all normal-range values, at append time.
// so that every query column lives in one lane (and its partner lane+32): the online-softmax
// statistics (eq. 1, scale folded into exp2) need no cross-lane traffic beyond one exchange
// with lane^32, the accumulator of S^T is already in B-operand layout for the second product,
// and the rescale factor of O is a per-lane scalar.
//
// The K rows fed to MFMA row m are permuted (bits 2 and 3 of m swapped) so that accumulator
// registers 8s..8s+7 of a lane hold 8 consecutive keys: the bf16 P fragment for k-step s is
// then just those registers packed, and the matching V^T fragment is one 16-byte LDS read.
#include "lcsa_kernels.h"

namespace lcsa {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kTileBytes = 128 * 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

#define LCSA_GLOBAL __attribute__((address_space(1)))
#define LCSA_LDS __attribute__((address_space(3)))

// Synchronisation inside the main loop is written as inline assembly on purpose.  The tile
// copies are direct-to-LDS loads that stay in flight across workgroup barriers; __syncthreads()
// and the compiler's own bookkeeping for LDS-writing loads would drain them (vmcnt(0)) at every
// barrier and before unrelated LDS reads, which serialises copy and compute.  Here arrival of a
// tile is established by an explicit vmcnt wait, and the barrier only orders LDS traffic.
//   vm_allow = number of newer vector-memory loads that may still be in flight.
template <int VM_ALLOW>
__device__ inline void wait_tiles_and_barrier() {
    static_assert(VM_ALLOW == 0 || VM_ALLOW == 8, "encodable cases used by the kernel");
    if (VM_ALLOW == 0) asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
__device__ inline void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Each wavefront copies its quarter (8 KB) of a 32 KB tile image: 8 loads of 64 lanes x 16
// bytes; lane t of a load lands at LDS address M0 + 16*t.
__device__ inline void tile_to_lds(const char *gsrc, unsigned char *lds, int wave, int lane) {
    const char *gp = gsrc + wave * 8192 + lane * 16;
    uint32_t dst = (uint32_t)(uintptr_t)((LCSA_LDS unsigned char *)lds) + wave * 8192;
    dst = __builtin_amdgcn_readfirstlane(dst);
#pragma unroll
    for (int i = 0; i < 8; ++i)
        asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off"
                     :: "v"(gp + i * 1024), "s"(dst + i * 1024) : "memory", "m0");
}

__global__ __launch_bounds__(256, 2) void attn_mfma_kernel(
    KGeom g, KCache c, const __bf16 *__restrict__ q, int64_t q_st, int64_t q_sh,
    const int32_t *__restrict__ sel_idx, const int32_t *__restrict__ sel_cnt,
    __bf16 *__restrict__ o, int64_t o_st, int64_t o_sh, float *__restrict__ lse,
    float scale_log2, int total_items, int items_per_xcd) {
    __shared__ __attribute__((aligned(16))) unsigned char k_lds[kTileBytes];
    __shared__ __attribute__((aligned(16))) unsigned char v_lds[kTileBytes];

    // Workgroups are dealt to the 8 XCDs round-robin; give each XCD a contiguous run of work
    // items (same head, neighbouring tiles, both query frames) so that K/V tiles shared by
    // neighbouring windows are found in that XCD's L2.
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int item = xcd * items_per_xcd + idx;
    if (item >= total_items) return;
    const int head = item / (g.nb * g.q_frames);
    const int rem = item - head * (g.nb * g.q_frames);
    const int tile = rem / g.q_frames, fq = rem - tile * g.q_frames;
    const int qb = fq * g.nb + tile;
    const int by = tile / g.tx, bx = tile - by * g.tx;
    const int qvh = min(g.th, g.H - by * g.th), qvw = min(g.tw, g.W - bx * g.tw);

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int ql = lane & 31, grp = lane >> 5;
    const int n_qb = g.q_frames * g.nb;
    const int64_t row = (int64_t)head * n_qb + qb;
    const int cnt = sel_cnt[row];
    const int32_t *sel = sel_idx + row * g.topk;

    // tile-token coordinates of keys `lane` and `lane + 64`, for the validity ballots of clipped tiles
    const int kr0 = lane / g.tw, kc0 = lane - kr0 * g.tw;
    const int kr1 = (lane + 64) / g.tw, kc1 = (lane + 64) - kr1 * g.tw;

    // ---- Q fragments (B operand of S^T = K Q^T): lane holds query ql of this wavefront, channels 16s+8grp..+8
    const int tq = wave * 32 + ql;
    const int qr = tq / g.tw, qc = tq - qr * g.tw;
    const bool q_valid = qr < qvh && qc < qvw;
    const int64_t token = q_valid ? ((int64_t)fq * g.H + by * g.th + qr) * g.W + bx * g.tw + qc
                                  : ((int64_t)fq * g.H + by * g.th) * g.W + bx * g.tw;   // clamp padding rows
    bf16x8 bq[8];
    {
        const __bf16 *qp = q + token * q_st + (int64_t)head * q_sh + grp * 8;
#pragma unroll
        for (int s = 0; s < 8; ++s) bq[s] = *(const bf16x8 *)(qp + s * 16);
    }

    // selected ids of this row, 64 at a time, one per lane
    int sel_chunk = lane < cnt ? sel[lane] : 0;

    // ---- per-lane LDS offsets
    // K operand: MFMA row m = ql reads key row pi(ql) of each 32-key group (bits 2,3 swapped)
    const int krow = (ql & 0x13) | ((ql & 4) << 1) | ((ql & 8) >> 1);
    int k_off[8], v_off[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        k_off[s] = krow * 256 + ((((s * 2 + grp) ^ (krow & 15))) << 4);    // + 8192 * key group
        v_off[s] = ql * 256 + ((((s * 2 + grp) ^ (ql & 15))) << 4);        // + 8192 * channel group; s = chunk pair
    }

    f32x16 oacc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[dt][i] = 0.f;
    float m_run = -__builtin_inff(), l_run = 0.f;

    auto tile_ptr = [&](const void *base, int kb) {
        const int f = kb / g.nb, kt = kb - f * g.nb;
        const int slot = slot_of_frame(c.start, g.cap, f);
        return (const char *)base + (((int64_t)head * g.cap + slot) * g.nb + kt) * (int64_t)kTileBytes;
    };

    if (cnt > 0) {
        const int kb0 = __builtin_amdgcn_readlane(sel_chunk, 0);
        tile_to_lds(tile_ptr(c.k, kb0), k_lds, wave, lane);
    }

    for (int it = 0; it < cnt; ++it) {
        const int kb = __builtin_amdgcn_readlane(sel_chunk, it & 63);
        // K tile of this iteration has landed (this wavefront's part), and after the barrier
        // everyone's; the barrier also says that all wavefronts left the previous P*V, so the
        // V buffer may be overwritten.
        wait_tiles_and_barrier<0>();
        tile_to_lds(tile_ptr(c.v, kb), v_lds, wave, lane);

        // ---- S^T = K Q^T : 4 key groups x 8 k-steps
        f32x16 sacc[4];
#pragma unroll
        for (int kg = 0; kg < 4; ++kg) {
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[kg][i] = 0.f;
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const bf16x8 a = *(const bf16x8 *)(k_lds + kg * 8192 + k_off[s]);
                sacc[kg] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bq[s], sacc[kg], 0, 0, 0);
            }
        }

        // id of the next block; every 64 iterations the per-lane chunk of ids is refilled
        // (the read of the fresh value sits inside the branch so that the wait for that load
        // does too, instead of draining the tile copies on every iteration)
        int kb_next = -1;
        if (it + 1 < cnt) {
            if (((it + 1) & 63) == 0) {
                sel_chunk = (it + 1 + lane) < cnt ? sel[it + 1 + lane] : 0;
                kb_next = __builtin_amdgcn_readlane(sel_chunk, 0);
            } else {
                kb_next = __builtin_amdgcn_readlane(sel_chunk, (it + 1) & 63);
            }
        }
        // all wavefronts are done reading K: stream in the next K tile behind the V tile
        lds_barrier();
        if (kb_next >= 0) tile_to_lds(tile_ptr(c.k, kb_next), k_lds, wave, lane);

        // ---- padding keys of clipped tiles get weight exactly zero
        {
            const int f = kb / g.nb, kt = kb - f * g.nb, kby = kt / g.tx, kbx = kt - kby * g.tx;
            const int kvh = min(g.th, g.H - kby * g.th), kvw = min(g.tw, g.W - kbx * g.tw);
            if (kvh < g.th || kvw < g.tw) {                 // wavefront-uniform
                const uint64_t b0 = __ballot(kr0 < kvh && kc0 < kvw);   // keys 0..63
                const uint64_t b1 = __ballot(kr1 < kvh && kc1 < kvw);   // keys 64..127
                const uint32_t key_ok[4] = {(uint32_t)b0, (uint32_t)(b0 >> 32), (uint32_t)b1, (uint32_t)(b1 >> 32)};
#pragma unroll
                for (int kg = 0; kg < 4; ++kg) {
                    // accumulator register i of key group kg is key kg*32 + (i>>3)*16 + grp*8 + (i&7)
                    const uint32_t mbits = key_ok[kg] >> (grp * 8);
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (!((mbits >> ((i >> 3) * 16 + (i & 7))) & 1u)) sacc[kg][i] = -__builtin_inff();
                }
            }
        }

        // ---- online softmax over this block's 128 keys, per query column
        float mx = sacc[0][0];
#pragma unroll
        for (int kg = 0; kg < 4; ++kg)
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[kg][i]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx * scale_log2);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        float psum = 0.f;
#pragma unroll
        for (int kg = 0; kg < 4; ++kg)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kg][i], scale_log2, -m_new));
                sacc[kg][i] = p;
                psum += p;
            }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[dt][i] *= alpha;

        // V tile has landed (the 8 newer loads in flight are the next K tile, if any)
        __builtin_amdgcn_sched_barrier(0);
        if (kb_next >= 0) wait_tiles_and_barrier<8>();
        else wait_tiles_and_barrier<0>();
        __builtin_amdgcn_sched_barrier(0);

        // ---- O^T += V^T P^T : 8 k-steps of 16 keys x 4 channel groups
#pragma unroll
        for (int kg = 0; kg < 4; ++kg)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                f16x8 pb;
#pragma unroll
                for (int j = 0; j < 8; ++j) pb[j] = (_Float16)sacc[kg][s2 * 8 + j];
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) {
                    const f16x8 a = *(const f16x8 *)(v_lds + dt * 8192 + v_off[kg * 2 + s2]);
                    oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, pb, oacc[dt], 0, 0, 0);
                }
            }
    }

    // ---- epilogue: normalise, transpose through LDS, store rows of 256 bytes
    __syncthreads();                                        // all P*V reads of LDS are done
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    {
        // lane owns query row tq; accumulator register i of channel group dt is channel
        // dt*32 + (i>>2)*8 + grp*4 + (i&3): 4 consecutive channels = 8 bytes
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
                bf16x4 w;
#pragma unroll
                for (int j = 0; j < 4; ++j) w[j] = (__bf16)(oacc[dt][i4 * 4 + j] * inv);
                const int chunk = dt * 4 + i4;
                *(bf16x4 *)(k_lds + tq * 256 + ((chunk ^ (tq & 15)) << 4) + grp * 8) = w;
            }
    }
    if (lse && grp == 0 && q_valid)
        lse[token * g.heads + head] = l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -__builtin_inff();
    __syncthreads();
    {
        const int rg = tid >> 4, j = tid & 15;
#pragma unroll
        for (int itr = 0; itr < 8; ++itr) {
            const int t = rg + 16 * itr;
            const int r = t / g.tw, cc = t - r * g.tw;
            if (r < qvh && cc < qvw) {
                const int64_t tok = ((int64_t)fq * g.H + by * g.th + r) * g.W + bx * g.tw + cc;
                const uint4 u = *(const uint4 *)(k_lds + t * 256 + ((j ^ (t & 15)) << 4));
                *(uint4 *)(o + tok * o_st + (int64_t)head * o_sh + j * 8) = u;
            }
        }
    }
}

} // namespace

hipError_t launch_attn_mfma(const KGeom &g, const KCache &c, const void *q, int64_t q_st, int64_t q_sh,
                            const int32_t *sel_idx, const int32_t *sel_cnt,
                            void *o, int64_t o_st, int64_t o_sh, float *lse, float scale, hipStream_t stream) {
    const int total = g.heads * g.nb * g.q_frames;
    const int per_xcd = (total + 7) / 8;
    attn_mfma_kernel<<<dim3(per_xcd * 8), 256, 0, stream>>>(g, c, (const __bf16 *)q, q_st, q_sh, sel_idx, sel_cnt,
                                                            (__bf16 *)o, o_st, o_sh, lse, scale * kLog2e,
                                                            total, per_xcd);
    return hipGetLastError();
}

} // namespace lcsa
