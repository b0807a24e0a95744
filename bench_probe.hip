// Measurement aids of bench.py, built into their own shared object (libbench_probe.so); not part of the library.
//
// 1. bench_probe_mfma_bf16: what the matrix cores of this chip sustain on a loop that does nothing else: every
//    wavefront runs back-to-back v_mfma_f32_32x32x16_bf16 on four independent accumulators with operands that
//    stay in registers (pseudo-random bf16 values, so that the data paths toggle as they do on real inputs).
// 2. bench_mock_loop: a loop with the instruction mix of the attention kernel's inner loop and nothing else that
//    could slow it down (no dependences between the pieces, no softmax bookkeeping): per step every one of the 8
//    wavefronts of a workgroup issues 32 matrix instructions whose A operand is a fresh 1 KB ds_read_b128 from a
//    swizzled tile image, a chosen number of vector instructions per matrix instruction (one exp2 among them), a
//    workgroup barrier and 8 direct-to-LDS copy instructions (64 KB per group of 4 wavefronts per two steps...
//    i.e. the K and V tiles of one block).  What it sustains is the ceiling of ANY schedule of that mix on this
//    chip, to be read beside the rate of the real loop.
// 3. bench_attn_timed: lcsa_sparse_attn_fwd's matrix-core kernel compiled with -DLCSA_TIMERS, which stamps the
//    shader-clock and the 100 MHz counters per workgroup (see lcsa_attn_mfma.hip): shader clock under load,
//    cycles per step, length of set-up and epilogue, how the second round of workgroups differs from the first.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "paper_2510_12747_amd/csrc/lcsa_cache_handle.h"

namespace lcsa { hipError_t set_attn_timers(uint64_t *device_buffer); }

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ inline uint32_t mix(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

__global__ __launch_bounds__(512) void probe_mfma_kernel(float *out, int iters) {
    bf16x8 a, b;
    const uint32_t id = blockIdx.x * 512u + threadIdx.x;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        // values in (-1, 1): sign and 7 mantissa bits random, exponent 126 or 125
        const uint32_t ra = mix(id * 16u + j), rb = mix(id * 16u + 8u + j);
        a[j] = __builtin_bit_cast(__bf16, (uint16_t)((ra & 0x807fu) | ((125u + ((ra >> 8) & 1u)) << 7)));
        b[j] = __builtin_bit_cast(__bf16, (uint16_t)((rb & 0x807fu) | ((125u + ((rb >> 8) & 1u)) << 7)));
    }
    f32x16 acc[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 8; ++r)
#pragma unroll
            for (int n = 0; n < 4; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[n], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[n][i];
    out[id] = s;
}

} // namespace

// Runs n_blocks workgroups of 8 wavefronts, every wavefront issuing 32*iters matrix instructions (32768 flop
// each).  out: device float [n_blocks*512], one checksum per thread.  Returns 0, -1 on bad arguments, -3 on a
// launch error.
extern "C" int32_t bench_probe_mfma_bf16(float *out, int32_t n_blocks, int32_t iters, void *stream) {
    if (!out || n_blocks < 1 || n_blocks > 65536 || iters < 1 || iters > (1 << 20)) return -1;
    probe_mfma_kernel<<<dim3(n_blocks), 512, 0, (hipStream_t)stream>>>(out, iters);
    return hipGetLastError() == hipSuccess ? 0 : -3;
}


// ---- 2. mock of the inner loop ------------------------------------------------------------------------------------
namespace {

#define BENCH_LDS __attribute__((address_space(3)))

template <int KV, bool MFMA, bool BARRIER, int NC>
__global__ __launch_bounds__(512, 2) void mock_loop_kernel(float *out, const char *src, int steps) {
    __shared__ __attribute__((aligned(16))) unsigned char lds[128 * 1024];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    unsigned char *tile = lds + (wave >> 2) * 65536;                 // each group of 4 wavefronts has its own K and V image
    const int row = lane & 31, half = lane >> 5;
    const int base = row * 256 + (((half ^ row) & 15) << 4);         // conflict-free operand reads, as in the real kernel
    bf16x8 b;
    for (int j = 0; j < 8; ++j) b[j] = __builtin_bit_cast(__bf16, (uint16_t)((mix(tid * 8 + j) & 0x807fu) | (125u << 7)));
    f32x16 acc[4];
    for (int n = 0; n < 4; ++n) for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;
    float x[8];
    for (int i = 0; i < 8; ++i) x[i] = 0.001f * (tid % 97) + i;
    for (int i = tid; i < 32768; i += 512)                             // pseudo-random bf16 values in (-1, 1)
        ((uint32_t *)lds)[i] = (mix(i) & 0x807f807fu) | 0x3e803e80u;
    __syncthreads();
    const uint32_t voff = (wave & 3) * 8192 + lane * 16;
    const uint32_t dst0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)((BENCH_LDS unsigned char *)tile) + (wave & 3) * 8192);
    for (int s = 0; s < steps; ++s) {
        const char *tsrc = src + (size_t)((s * 7 + blockIdx.x) & 255) * 65536;        // a 16 MB region that stays in L2 / Infinity Cache
#pragma unroll
        for (int n = 0; n < 32; ++n) {
            const bf16x8 a = *(const bf16x8 *)(tile + (n >> 3) * 8192 + ((n & 1) * 32768) + (base ^ ((n & 7) << 5)));
            if (NC > 0 && (n % (32 / NC)) == 0) {
                const uint32_t m0v = dst0 + (n / (32 / NC)) * 1024;
                asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" :: "v"(voff + (n / (32 / NC)) * 1024), "s"(tsrc), "s"(m0v) : "memory", "m0");
            }
            if (MFMA) acc[n & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[n & 3], 0, 0, 0);
            else x[n & 7] += (float)a[n & 7];
#pragma unroll
            for (int k = 0; k < KV; ++k) {
                if (k == 0) x[(n + k) & 7] = __builtin_amdgcn_exp2f(x[(n + k) & 7]);
                else x[(n + k) & 7] = fmaf(x[(n + k) & 7], 0.999f, 0.5f);
            }
        }
        if (BARRIER) {
            if (NC > 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        }
    }
    if (NC > 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    float sum = 0.f;
    for (int n = 0; n < 4; ++n) for (int i = 0; i < 16; ++i) sum += acc[n][i];
    for (int i = 0; i < 8; ++i) sum += x[i];
    out[blockIdx.x * 512 + tid] = sum;
}

} // namespace

// variant: 0 matrix instructions + LDS operand reads only; 1 + 4 vector instructions per matrix instruction;
// 2 + a barrier per step; 3 + 8 copy instructions per step (the full mix); 4 the full mix with 5 vector
// instructions; 5 the full mix without the matrix instructions.  n_blocks workgroups of 512 threads (128 KB of
// LDS each: one per compute unit); out: device float [n_blocks*512]; src: device, 16 MiB.  Per step and
// workgroup: 8 x 32 matrix instructions (32768 flop each).
extern "C" int32_t bench_mock_loop(int32_t variant, float *out, const void *src, int32_t n_blocks, int32_t steps, void *stream) {
    if (!out || !src || n_blocks < 1 || n_blocks > 65536 || steps < 1 || steps > (1 << 20)) return -1;
    hipStream_t st = (hipStream_t)stream;
    const char *s = (const char *)src;
    switch (variant) {
    case 0: mock_loop_kernel<0, true, false, 0><<<n_blocks, 512, 0, st>>>(out, s, steps); break;
    case 1: mock_loop_kernel<4, true, false, 0><<<n_blocks, 512, 0, st>>>(out, s, steps); break;
    case 2: mock_loop_kernel<4, true, true, 0><<<n_blocks, 512, 0, st>>>(out, s, steps); break;
    case 3: mock_loop_kernel<4, true, true, 8><<<n_blocks, 512, 0, st>>>(out, s, steps); break;
    case 4: mock_loop_kernel<5, true, true, 8><<<n_blocks, 512, 0, st>>>(out, s, steps); break;
    case 5: mock_loop_kernel<4, false, true, 8><<<n_blocks, 512, 0, st>>>(out, s, steps); break;
    default: return -1;
    }
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

// ---- 3. the attention kernel with per-workgroup time stamps -------------------------------------------------------
// Arguments as lcsa_sparse_attn_fwd (matrix-core configurations only, else -2); timers: device uint64
// [workgroups][10] (workgroups = 8 * ceil(ceil(heads*n_qb/2)/8)), per workgroup: shader-clock and 100 MHz counter
// at entry, before the main loop, after it, at exit, then HW_ID | XCC_ID << 32, then unused.
extern "C" int32_t bench_attn_timed(const lcsa_geom *geom, const void *q, int64_t q_st, int64_t q_sh, const lcsa_cache *cache,
                                    const int32_t *sel_idx, const int32_t *sel_cnt, void *o, int64_t o_st, int64_t o_sh,
                                    float scale, uint64_t *timers, void *stream) {
    if (!geom || !cache || !q || !o || !sel_idx || !sel_cnt || !timers) return -1;
    if (!cache->kc.mfma_layout) return -2;
    lcsa::KGeom kg = cache->kg;
    kg.topk = geom->topk;
    if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)kg.d);
    if (lcsa::set_attn_timers(timers) != hipSuccess) return -3;      // a synchronous copy to a device variable: fine for a measurement aid
    const hipError_t e = lcsa::launch_attn_mfma(kg, cache->kc, q, q_st, q_sh, sel_idx, sel_cnt, o, o_st, o_sh, nullptr, scale,
                                                (hipStream_t)stream);
    return e == hipSuccess ? 0 : -3;
}
