// Block-sparse flash attention on the gfx950 matrix cores (bf16, d = 128, 128-token blocks).
//
// Work item = one (head, query block): 128 query rows against its selected key blocks.
// A workgroup has 8 wavefronts = two GROUPS of 4; each group owns one work item (the two
// query blocks of the same spatial tile, which share their window), its own K and V tile
// buffers in LDS, and wavefront w of a group owns query rows 32w .. 32w+31.
//
// Per selected key block a group runs
//     QK   S^T = K Q^T        v_mfma_f32_32x32x16_bf16  (keys on the row axis, queries on lanes)
//     SM   online softmax     VALU, fp32 (eq. 1; scale folded into exp2; lazily updated reference)
//     PV   O^T += V^T P^T     v_mfma_f32_32x32x16_f16   (channels on the row axis, queries on lanes)
// as four phases (two matrix, two vector), every phase ending in a workgroup barrier, and the
// two groups run two phases apart: each SIMD holds one wavefront of either group, so while one
// issues matrix instructions the other issues vector instructions.  Left to themselves two
// independent wavefronts fall into step (both want the matrix pipe, then both want the vector
// pipe); the fixed stagger keeps the two pipes busy together.
//
// A block clipped by the grid border holds its valid tokens first: only the 32-key groups (and
// 32-query wavefronts) that contain valid tokens are computed, and at most one 16-key fragment
// per block needs a mask.
//
// Transposed products put every query column in one lane (and its partner lane^32): the
// softmax statistics need one cross-lane exchange per block, the rescale factor of O is a
// per-lane scalar, and the accumulator of S^T is already in B-operand layout for the second
// product.  K rows fed to MFMA row m are permuted (bits 2 and 3 of m swapped) so that
// accumulator registers 8s..8s+7 of a lane hold 8 consecutive keys: the P fragment for
// k-step s is those registers packed, the matching V^T fragment one 16-byte LDS read.
//
// The second product runs in IEEE half (same matrix-core rate as bf16): probabilities lie in
// [0,1] and need mantissa rather than range, which cuts the kernel's dominant rounding error
// (bf16 P) by 8x; V was converted to half, exactly for all normal-range values, at append time.
//
// K and V tiles are 32 KB byte-for-byte LDS images prepared by the cache append (16-byte
// chunk j of row r at chunk position j ^ (r & 15): conflict-free ds_read_b128 operand reads)
// and are streamed in with direct-to-LDS loads that stay in flight across barriers:
// V(i) arrives during QK(i)+SM(i), K(i+1) during SM(i)+PV(i).
#include "lcsa_kernels.h"

namespace lcsa {

// Built with -DLCSA_TIMERS=1 (only the benchmark's measurement aids do that) the kernel also records, per
// workgroup, the shader-clock counter and the constant 100 MHz counter at entry, before and after the main
// loop and at exit (-DLCSA_TIMERS=2: at entry and exit only; the inner stamps perturb the loop's schedule
// measurably), plus the hardware id of the compute unit: 10 x uint64 per workgroup at *d_attn_timers
// (a device-side pointer variable rather than a kernel argument, which would cost scalar registers for the
// whole kernel; null = no stamps).
#ifdef LCSA_TIMERS
__device__ uint64_t *d_attn_timers;
hipError_t set_attn_timers(uint64_t *device_buffer) {
    return hipMemcpyToSymbol(HIP_SYMBOL(d_attn_timers), &device_buffer, sizeof(device_buffer));
}
#define LCSA_STAMP(slot)                                                                                     \
    if ((LCSA_TIMERS == 1 || (slot) == 0 || (slot) == 3) && threadIdx.x == 0) {                                                                                  \
        uint64_t *timers = d_attn_timers;                                                                    \
        if (timers) {                                                                                        \
            timers[(size_t)blockIdx.x * 10 + 2 * (slot)] = __builtin_readcyclecounter();                     \
            timers[(size_t)blockIdx.x * 10 + 2 * (slot) + 1] = __builtin_amdgcn_s_memrealtime();             \
            if ((slot) == 0)      /* HW_ID (compute unit, shader engine) and, above it, XCC_ID (which of the 8 dies) */ \
                timers[(size_t)blockIdx.x * 10 + 8] = (uint64_t)__builtin_amdgcn_s_getreg(4 | (31 << 11)) |  \
                                                      (uint64_t)__builtin_amdgcn_s_getreg(20 | (31 << 11)) << 32; \
        }                                                                                                    \
    }
#else
#define LCSA_STAMP(slot)
#endif

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kTileBytes = 128 * 256;
constexpr int kAhead = 3;            // operand fragments in flight ahead of the matrix instruction using them
constexpr int kRing = kAhead + 1;
constexpr int kSplit = 4;            // softmax fragments (of 8) done in the first vector phase; the rest in the second
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

#define LCSA_LDS __attribute__((address_space(3)))

// Synchronisation inside the main loop is inline assembly on purpose.  The tile copies are
// direct-to-LDS loads that stay in flight across workgroup barriers; __syncthreads() and the
// compiler's own bookkeeping for LDS-writing loads would drain them (vmcnt(0)) at every
// barrier and before unrelated LDS reads, which serialises copy and compute.  Arrival of a
// tile is established by an explicit vmcnt wait; the barrier itself only orders LDS traffic.
__device__ inline void stage_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
// wait until at most N of this wavefront's vector-memory loads are still in flight
__device__ inline void wait_vm0() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ inline void wait_vm8() { asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); }

// One of the 8 copy instructions of a wavefront's quarter tile: 64 lanes x 16 bytes, lane t lands at
// LDS address dst + 1024*piece + 16*t (M0 + immediate + 16*t).  The source is scalar base (the tile, wavefront-uniform) +
// per-lane byte offset `voff` (wavefront quarter + 16*lane, loop invariant) + an immediate, so the
// copies cost no vector arithmetic.
__device__ inline void copy_piece_to_lds(const char *tile, uint32_t voff, uint32_t dst, int piece) {
    const char *base = tile + (piece >> 2) * 4096;        // immediates reach 4095 bytes
    const uint32_t m0v = dst + (piece >> 2) * 4096;        // the immediate offset is added to the LDS address too
    switch (piece & 3) {
    case 0: asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" :: "v"(voff), "s"(base), "s"(m0v) : "memory", "m0"); break;
    case 1: asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 offset:1024" :: "v"(voff), "s"(base), "s"(m0v) : "memory", "m0"); break;
    case 2: asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 offset:2048" :: "v"(voff), "s"(base), "s"(m0v) : "memory", "m0"); break;
    default: asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 offset:3072" :: "v"(voff), "s"(base), "s"(m0v) : "memory", "m0"); break;
    }
}

// exp2 of 8 scores of one accumulator (registers first..first+7 = 8 consecutive keys), rounded to
// half for the second matrix product; the row sum is kept in float.  (Plain adds on purpose: the
// dot-product instructions v_dot2* run on the matrix pipeline and do not overlap with MFMAs of the
// other wavefront on the SIMD, ordinary vector instructions do.)
__device__ inline void softmax_fragment(const f32x16 &sc, int first, float scale_log2, float m, float &l, f16x8 &out) {
#pragma unroll
    for (int j = 0; j < 8; j += 2) {
        const float p0 = __builtin_amdgcn_exp2f(fmaf(sc[first + j], scale_log2, -m));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(sc[first + j + 1], scale_log2, -m));
        l += p0 + p1;
        out[j] = (_Float16)p0;
        out[j + 1] = (_Float16)p1;
    }
}

// Largest score of each query column over the block's first nf 16-key fragments (both lanes of a
// query agree); nf is wavefront-uniform.
__device__ inline float block_row_max(const f32x16 (&sc)[4], int nf) {
    float mx = -__builtin_inff();
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
        if (ks < nf) {
#pragma unroll
            for (int j = 0; j < 8; ++j) mx = fmaxf(mx, sc[ks >> 1][(ks & 1) * 8 + j]);
        }
    return fmaxf(mx, __shfl_xor(mx, 32));
}

// A selected key block as the loop wants it: ring-slot tile index and its number of valid keys.
//   bits 0..23 tile index (slot*nb + tile), bits 24..30 valid keys - 1
__device__ inline uint32_t pack_block(const KGeom &g, const KCache &c, int start, int head, int kb, int ph, int pw) {
    kb = min(max(kb, 0), c.valid * g.nb - 1);          // ids outside the cache (corrupt input) must not become wild addresses
    const int f = kb / g.nb, kt = kb - f * g.nb;
    const int kby = kt / g.tx, kbx = kt - kby * g.tx;
    const int vh = kby == g.ty - 1 ? ph : g.th, vw = kbx == g.tx - 1 ? pw : g.tw;
    return (uint32_t)(cache_slot(c, g, start, head, f) * g.nb + kt) | (uint32_t)(g.tt * vh * vw - 1) << 24;
}
__device__ inline int block_keys(uint32_t blk) { return (int)(blk >> 24) + 1; }

// SINGLE: one work item per workgroup (group 1 only keeps the barriers company).  A lone group is faster than
// a group that shares its SIMDs, so a launch with no more work items than compute units spreads over twice as
// many units this way.
template <bool SINGLE>
__global__ __launch_bounds__(512, 2) void attn_mfma_kernel(
    KGeom g, KCache c, const __bf16 *__restrict__ q, int64_t q_st, int64_t q_sh,
    const int32_t *__restrict__ sel_idx, const int32_t *__restrict__ sel_cnt,
    __bf16 *__restrict__ o, int64_t o_st, int64_t o_sh, float *__restrict__ lse,
    float scale_log2, int total_items, int pairs_per_xcd) {
    __shared__ __attribute__((aligned(16))) unsigned char lds_all[2][2][kTileBytes];   // [group][K, V]
    LCSA_STAMP(0)

    // Workgroups are dealt to the 8 XCDs round-robin; give each XCD a contiguous run of work
    // items (same head, neighbouring tiles, both query frames) so that K/V tiles shared by
    // neighbouring windows are found in that XCD's L2.
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int total_pairs = SINGLE ? total_items : (total_items + 1) >> 1;
    const int pair = xcd * pairs_per_xcd + idx;
    if (pair >= total_pairs) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int grp8 = __builtin_amdgcn_readfirstlane(tid >> 8);        // which group of 4 wavefronts
    const int wave = __builtin_amdgcn_readfirstlane((tid >> 6) & 3);  // wavefront within the group
    unsigned char *k_lds = lds_all[grp8][0], *v_lds = lds_all[grp8][1];
    const int ql = lane & 31, half = lane >> 5;
    const int n_qb = g.q_groups * g.nb;

    // this group's item, and how many blocks the other group has (the stage clock is shared)
    auto item_row = [&](int item, int &head, int &qb) {
        head = item / n_qb;
        const int rem = item - head * n_qb;
        const int tile = rem / g.q_groups, fq = rem - tile * g.q_groups;   // items ordered (head, tile, group)
        qb = fq * g.nb + tile;
    };
    const int item = SINGLE ? (grp8 == 0 ? pair : total_items) : 2 * pair + grp8;
    const int other = SINGLE ? (grp8 == 0 ? total_items : pair) : 2 * pair + (grp8 ^ 1);
    const bool active = item < total_items;
    int head = 0, qb = 0, cnt = 0, other_cnt = 0;
    const int start = ring_start(c, g);    // requested together with the counts and ids below
    int32_t first_ids = -1;                // selected block `lane` of this row, requested together with the count
    if (active) {
        item_row(item, head, qb);
        cnt = sel_cnt[(int64_t)head * n_qb + qb];
        if (lane < g.topk) first_ids = sel_idx[((int64_t)head * n_qb + qb) * g.topk + lane];
    }
    if (other < total_items) { int h2, q2; item_row(other, h2, q2); other_cnt = sel_cnt[(int64_t)h2 * n_qb + q2]; }
    const int fq = qb / g.nb, tile = qb - fq * g.nb;
    const int by = tile / g.tx, bx = tile - by * g.tx;
    const int qvh = min(g.th, g.H - by * g.th), qvw = min(g.tw, g.W - bx * g.tw);

    // ---- Q fragments (B operand of S^T = K Q^T), requested before the counts are waited for:
    // lane holds query ql of this wavefront, channels 16s+8*half..+8
    const int tq = wave * 32 + ql;
    int qft, qr, qc;
    const bool q_valid = block_token(g, tq, qvh, qvw, qft, qr, qc) && active;
    const int64_t token = q_valid ? raster_token(g, fq, qft, by * g.th + qr, bx * g.tw + qc)
                                  : raster_token(g, fq, 0, by * g.th, bx * g.tw);       // clamp padding rows
    // a wavefront whose 32 query rows are all padding only takes part in the copies and barriers
    const bool wave_on = active && wave * 32 < g.tt * qvh * qvw;
    bf16x8 bq[8];
    {
        const __bf16 *qp = q + token * q_st + (int64_t)head * q_sh + half * 8;
#pragma unroll
        for (int s = 0; s < 8; ++s) bq[s] = *(const bf16x8 *)(qp + s * 16);
    }

    cnt = min(max(__builtin_amdgcn_readfirstlane(cnt), 0), g.topk);            // a row holds at most topk ids
    other_cnt = min(max(__builtin_amdgcn_readfirstlane(other_cnt), 0), g.topk);
    const int n_iter = max(cnt, other_cnt);
    const int64_t row = (int64_t)head * n_qb + qb;
    const int32_t *sel = sel_idx + row * g.topk;

    // ---- the first K tile is requested as soon as its id is known so that its latency overlaps the set-up.
    // Wavefront w copies rows 32w..32w+31 of a K tile, which are only read if they hold valid keys.
    const char *k_head = (const char *)c.k + (int64_t)head * g.cap * g.nb * kTileBytes;
    const char *v_head = (const char *)c.v + (int64_t)head * g.cap * g.nb * kTileBytes;
    auto tile_off = [](uint32_t blk) { return (int64_t)(blk & 0xffffffu) * kTileBytes; };
    auto key_groups = [](uint32_t blk) { return (block_keys(blk) + 31) >> 5; };
    const uint32_t copy_voff = wave * 8192 + lane * 16;     // this lane's byte offset inside any tile image
    const uint32_t kdst = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)((LCSA_LDS unsigned char *)k_lds) + wave * 8192);
    const uint32_t vdst = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)((LCSA_LDS unsigned char *)v_lds) + wave * 8192);
    // selected blocks of this row, 64 at a time, one per lane, already turned into tile indices
    const int ph = g.H - (g.ty - 1) * g.th, pw = g.W - (g.tx - 1) * g.tw;   // extent of clipped edge tiles
    uint32_t blk_chunk = lane < cnt ? pack_block(g, c, start, head, first_ids, ph, pw) : 0u;
    uint32_t blk = __builtin_amdgcn_readfirstlane(blk_chunk);
    if (cnt > 0 && wave < key_groups(blk)) {
#pragma unroll
        for (int piece = 0; piece < 8; ++piece) copy_piece_to_lds(k_head + tile_off(blk), copy_voff, kdst, piece);
    }

    // ---- per-lane LDS offsets
    // K operand: MFMA row m = ql reads key row pi(ql) of each 32-key group (bits 2,3 swapped)
    const int krow = (ql & 0x13) | ((ql & 4) << 1) | ((ql & 8) >> 1);
    // byte offset of the 16-byte chunk (2s + half) of this lane's row: row*256 + (((2s+half) ^ (row&15)) << 4)
    //   = base ^ (s << 5) with base = row*256 + (((half ^ row) & 15) << 4): one XOR per read, two registers
    const int k_base = krow * 256 + (((half ^ krow) & 15) << 4);     // + 8192 * key group
    const int v_base = ql * 256 + (((half ^ ql) & 15) << 4);         // + 8192 * channel group
    auto k_off = [&](int s) { return k_base ^ (s << 5); };
    auto v_off = [&](int s) { return v_base ^ (s << 5); };

    f32x16 oacc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[dt][i] = 0.f;
    float m_run = -__builtin_inff(), l_run = 0.f;

    __builtin_amdgcn_s_waitcnt(0x0F70);    // vmcnt(0), visible to the compiler: Q fragments, ids and the first K tile have arrived
    stage_barrier();                       // first K tiles of both groups are in LDS
    if (grp8 == 1) { stage_barrier(); stage_barrier(); }   // group 1 runs two phases behind group 0

    LCSA_STAMP(1)
    f16x8 pfrag[8];                        // P^T fragments of the previous block: [key group*2 + k-step]
    uint32_t blk_next = 0;
    bool has_next = false;
    float l_before = 0.f;
    int ng = 4, ng_prev = 4;               // 32-key groups of the current / previous block that hold valid keys

    // O^T += V^T P^T over the first `groups` 32-key groups (2 k-steps each) x 4 channel groups.
    // Operand fragments are read kAhead matrix instructions ahead through a register ring; a group
    // without valid keys ends the product (its operands, already requested, are dropped).
    auto pv_phase = [&](int groups) {
        f16x8 va[kRing];
#pragma unroll
        for (int n = 0; n < kAhead; ++n) va[n % kRing] = *(const f16x8 *)(v_lds + (n & 3) * 8192 + v_off(n >> 2));
        __builtin_amdgcn_sched_group_barrier(0x100, kAhead, 0);
#pragma unroll
        for (int kg = 0; kg < 4; ++kg)
            if (kg < groups) {
#pragma unroll
                for (int n = 8 * kg; n < 8 * kg + 8; ++n) {
                    const int ks = n >> 2, dt = n & 3;
                    if (n + kAhead < 32) {
                        va[(n + kAhead) % kRing] = *(const f16x8 *)(v_lds + ((n + kAhead) & 3) * 8192 + v_off((n + kAhead) >> 2));
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    }
                    oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va[n % kRing], pfrag[ks], oacc[dt], 0, 0, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                }
            }
    };

    // Four phases per block, each ending in a workgroup barrier:
    //   P1  PV(i-1)            matrix     P3  softmax(i), first fragments   vector
    //   P2  QK(i)              matrix     P4  softmax(i), the rest + check  vector
    // Group 1 is two phases behind, so every SIMD always holds one wavefront in a matrix phase and
    // one in a vector phase.  Tile copies: V(i) is issued during P2(i) and needed at P1(i+1);
    // K(i+1) is issued during P3(i) and P4(i) and needed at P2(i+1): two to three phases of lead.  The eight
    // copy instructions of a tile are spread through the phase because each one can hold the
    // issuing wavefront while the memory pipeline accepts it.
    for (int it = 0; it <= n_iter; ++it) {
        const bool pv_on = it >= 1 && it - 1 < cnt;   // wavefront-uniform
        const bool on = it < cnt;
        f32x16 sacc[4];                    // S^T of this block: produced in P2, consumed in P3 and P4

        // S^T = K Q^T over the first `groups` key groups x 8 k-steps; the 8 copy instructions of V(i) go along
        auto qk_phase = [&](int groups, const char *vsrc) {
            bf16x8 ka[kRing];
#pragma unroll
            for (int n = 0; n < kAhead; ++n) ka[n % kRing] = *(const bf16x8 *)(k_lds + (n >> 3) * 8192 + k_off(n & 7));
            __builtin_amdgcn_sched_group_barrier(0x100, kAhead, 0);
#pragma unroll
            for (int kg = 0; kg < 4; ++kg) {
                if (kg < groups) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) sacc[kg][i] = 0.f;
#pragma unroll
                    for (int n = 8 * kg; n < 8 * kg + 8; ++n) {
                        const int s = n & 7;
                        if ((n & 3) == 0) copy_piece_to_lds(vsrc, copy_voff, vdst, n >> 2);     // one copy instruction per 4 MFMAs
                        if (n + kAhead < 32) {
                            ka[(n + kAhead) % kRing] = *(const bf16x8 *)(k_lds + ((n + kAhead) >> 3) * 8192 + k_off((n + kAhead) & 7));
                            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                        }
                        sacc[kg] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[n % kRing], bq[s], sacc[kg], 0, 0, 0);
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    }
                } else {
                    copy_piece_to_lds(vsrc, copy_voff, vdst, 2 * kg);
                    copy_piece_to_lds(vsrc, copy_voff, vdst, 2 * kg + 1);
                }
            }
        };

        // ================= P1: O^T += V^T P^T of the previous block ===================================
        if (pv_on && wave_on) {
            __builtin_amdgcn_s_setprio(2);
            pv_phase(ng_prev);
            __builtin_amdgcn_s_setprio(0);
        }
        if (on) wait_vm0();                // K(i) (this wavefront's part) has landed
        __builtin_amdgcn_sched_barrier(0);
        stage_barrier();
        __builtin_amdgcn_sched_barrier(0);

        // ================= P2: S^T = K Q^T; V(i) copy issued alongside ================================
        if (on) {
            blk = it == 0 ? blk : blk_next;
            ng = key_groups(blk);
            const char *vsrc = v_head + tile_off(blk);
            if (wave_on) {
                __builtin_amdgcn_s_setprio(2);
                qk_phase(ng, vsrc);
                __builtin_amdgcn_s_setprio(0);
            } else {
#pragma unroll
                for (int piece = 0; piece < 8; ++piece) copy_piece_to_lds(vsrc, copy_voff, vdst, piece);
            }
            // next block; every 64 iterations the per-lane chunk is refilled (the read of the fresh
            // value sits inside the branch so that the wait for that load does too)
            has_next = it + 1 < cnt;
            if (has_next) {
                if (((it + 1) & 63) == 0) {
                    blk_chunk = (it + 1 + lane) < cnt ? pack_block(g, c, start, head, sel[it + 1 + lane], ph, pw) : 0u;
                    blk_next = __builtin_amdgcn_readlane(blk_chunk, 0);
                } else {
                    blk_next = __builtin_amdgcn_readlane(blk_chunk, (it + 1) & 63);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        stage_barrier();
        __builtin_amdgcn_sched_barrier(0);

        // ================= P3: online softmax, first half; K(i+1) copy issued alongside ===============
        const char *ksrc = k_head + tile_off(blk_next);
        const bool k_copy = on && has_next && wave < key_groups(blk_next);    // this wavefront's rows of K(i+1) hold keys
        const int nv = block_keys(blk);
        const int nf = (nv + 15) >> 4;     // 16-key fragments that hold valid keys
        // everyone in the group is done reading K: the next K tile may overwrite it
        if (k_copy) { copy_piece_to_lds(ksrc, copy_voff, kdst, 0); copy_piece_to_lds(ksrc, copy_voff, kdst, 1); }
        if (on && wave_on) {
            // Padding keys get weight exactly zero.  Valid keys come first in a block, so only the last
            // fragment can be mixed: accumulator register j of fragment ks is key 16*ks + 8*half + j.
            if (nv & 15) {
                const int thr = (nv & 15) - half * 8;      // registers j >= thr of the last fragment are padding
#pragma unroll
                for (int ks = 0; ks < 8; ++ks)
                    if (ks == nf - 1) {
#pragma unroll
                        for (int j = 0; j < 8; ++j)
                            if (j >= thr) sacc[ks >> 1][(ks & 1) * 8 + j] = -__builtin_inff();
                    }
            }
            // Reference point of the exponentials.  Any per-query reference gives the same softmax after
            // the final normalisation; it only has to keep 2^(score - reference) inside half's range.
            // The first block sets it to its exact row maximum; later blocks reuse it without looking
            // for their maximum (which would cost a pass over all scores) and are checked afterwards:
            // see the end of P4.
            if (it == 0) m_run = block_row_max(sacc, nf) * scale_log2;
        }
        if (k_copy) { copy_piece_to_lds(ksrc, copy_voff, kdst, 2); copy_piece_to_lds(ksrc, copy_voff, kdst, 3); }
        if (on && wave_on) {
            l_before = l_run;
            // probabilities -> half for the matrix product; row sum in float
#pragma unroll
            for (int ks = 0; ks < kSplit; ++ks) {
                if (ks < nf) softmax_fragment(sacc[ks >> 1], (ks & 1) * 8, scale_log2, m_run, l_run, pfrag[ks]);
                else pfrag[ks] = f16x8{0, 0, 0, 0, 0, 0, 0, 0};
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        stage_barrier();
        __builtin_amdgcn_sched_barrier(0);

        // ================= P4: online softmax, second half =============================================
        if (k_copy) { copy_piece_to_lds(ksrc, copy_voff, kdst, 4); copy_piece_to_lds(ksrc, copy_voff, kdst, 5); }
        if (on && wave_on) {
#pragma unroll
            for (int ks = kSplit; ks < 8; ++ks) {
                if (ks < nf) softmax_fragment(sacc[ks >> 1], (ks & 1) * 8, scale_log2, m_run, l_run, pfrag[ks]);
                else pfrag[ks] = f16x8{0, 0, 0, 0, 0, 0, 0, 0};
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (k_copy) { copy_piece_to_lds(ksrc, copy_voff, kdst, 6); copy_piece_to_lds(ksrc, copy_voff, kdst, 7); }
        if (on && wave_on) {
            // Check of the reference: this lane's probabilities of the block sum to less than 2^14, hence none
            // of them left half's range.  Otherwise (a block whose scores tower over everything seen before, or
            // non-finite input) redo the block against its exact maximum, rescaling the running sums.
            if (__ballot(!(l_run - l_before < 16384.f))) {
                const float m_new = fmaxf(m_run, block_row_max(sacc, nf) * scale_log2);
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
                l_run = l_before * alpha;
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[dt][i] *= alpha;
                m_run = m_new;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks)
                    if (ks < nf) softmax_fragment(sacc[ks >> 1], (ks & 1) * 8, scale_log2, m_run, l_run, pfrag[ks]);
            }
        }
        if (on) {
            // V(i) has landed (the 8 newer copies in flight are this wavefront's part of the next K tile, if any)
            if (k_copy) wait_vm8(); else wait_vm0();
            ng_prev = ng;
        }
        __builtin_amdgcn_sched_barrier(0);
        stage_barrier();
        __builtin_amdgcn_sched_barrier(0);
    }
    if (grp8 == 0) { stage_barrier(); stage_barrier(); }   // matches group 1's two extra barriers at the start
    LCSA_STAMP(2)

    // ---- epilogue: normalise, transpose through this wavefront's own 8 KB of LDS, store 256-byte rows.
    // No LDS reads of other wavefronts are outstanding: the last stage ended in a barrier.
    if (!active) return;
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    // lane owns query row tq; accumulator register i of channel group dt is channel
    // dt*32 + (i>>2)*8 + half*4 + (i&3): 4 consecutive channels = 8 bytes
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            bf16x4 w;
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = (__bf16)(oacc[dt][i4 * 4 + j] * inv);
            const int chunk = dt * 4 + i4;
            *(bf16x4 *)(k_lds + tq * 256 + ((chunk ^ (tq & 15)) << 4) + half * 8) = w;
        }
    if (lse && half == 0 && q_valid)
        lse[token * g.heads + head] = l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -__builtin_inff();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // rows written by this wavefront are read by it only
    {
        const int rg = lane >> 4, j = lane & 15;            // 4 rows per pass, 16 lanes x 16 bytes per row
#pragma unroll
        for (int itr = 0; itr < 8; ++itr) {
            const int t = wave * 32 + rg + 4 * itr;
            int ft, r, cc;
            if (block_token(g, t, qvh, qvw, ft, r, cc)) {
                const int64_t tok = raster_token(g, fq, ft, by * g.th + r, bx * g.tw + cc);
                const uint4 u = *(const uint4 *)(k_lds + t * 256 + ((j ^ (t & 15)) << 4));
                *(uint4 *)(o + tok * o_st + (int64_t)head * o_sh + j * 8) = u;
            }
        }
    }
    LCSA_STAMP(3)
}

} // namespace

hipError_t launch_attn_mfma(const KGeom &g, const KCache &c, const void *q, int64_t q_st, int64_t q_sh,
                            const int32_t *sel_idx, const int32_t *sel_cnt,
                            void *o, int64_t o_st, int64_t o_sh, float *lse, float scale, hipStream_t stream) {
    const int total = g.heads * g.nb * g.q_groups;
    int n_cu = 0, dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n_cu = 256;
    if (total <= n_cu) {
        const int per_xcd = (total + 7) / 8;
        attn_mfma_kernel<true><<<dim3(per_xcd * 8), 512, 0, stream>>>(g, c, (const __bf16 *)q, q_st, q_sh, sel_idx, sel_cnt,
                                                                      (__bf16 *)o, o_st, o_sh, lse, scale * kLog2e,
                                                                      total, per_xcd);
    } else {
        const int pairs = (total + 1) / 2;
        const int per_xcd = (pairs + 7) / 8;
        attn_mfma_kernel<false><<<dim3(per_xcd * 8), 512, 0, stream>>>(g, c, (const __bf16 *)q, q_st, q_sh, sel_idx, sel_cnt,
                                                                       (__bf16 *)o, o_st, o_sh, lse, scale * kLog2e,
                                                                       total, per_xcd);
    }
    return hipGetLastError();
}

} // namespace lcsa
