// Measurement aid of bench.py, built into its own shared object (libbench_probe.so); not part of the library.
//
// What the matrix cores of this chip sustain on a loop that does nothing else: every wavefront runs
// back-to-back v_mfma_f32_32x32x16_bf16 on four independent accumulators with operands that stay in
// registers (pseudo-random bf16 values, so that the data paths toggle as they do on real inputs).  The
// benchmark quotes the rate next to the nominal peak.
#include <hip/hip_runtime.h>
#include <stdint.h>

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
