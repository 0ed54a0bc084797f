// Two reference kernels that say what this machine can do, measured beside the model's kernels:
// a plain streaming read (what a weight-streaming GEMM could reach if it did nothing but read its
// weights) and a register-only loop of the matrix instruction the GEMMs use (what the matrix
// cores sustain when nothing has to be fetched).  Neither is on the model path.
#include "rdlm_internal.h"

namespace rdlm {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Every wave reads a contiguous slice of 1 KiB units (64 lanes x 16 bytes, nontemporal), U units per
// batch, two batches in flight -- the access pattern of gemm_bf16_k without the contraction.
template <int U>
__global__ __launch_bounds__(256) void stream_read_k(const u32x4* __restrict__ p, size_t units_per_wave, uint32_t* sink) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, W = blockDim.x >> 6;
    const size_t wid = (size_t)blockIdx.x * W + wave;
    const u32x4* b = p + wid * units_per_wave * 64 + lane;
    u32x4 acc = {0, 0, 0, 0};
    size_t i = 0;
    for (; i + 2 * U <= units_per_wave; i += 2 * U) {
        u32x4 a[U], c[U];
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = __builtin_nontemporal_load(b + (i + u) * 64);
#pragma unroll
        for (int u = 0; u < U; ++u) c[u] = __builtin_nontemporal_load(b + (i + U + u) * 64);
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= a[u] ^ c[u];
    }
    for (; i < units_per_wave; ++i) acc ^= __builtin_nontemporal_load(b + i * 64);
    // never true for packed bf16 weights of ordinary size; keeps the loads alive
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x7fc1a55au && lane == 63) sink[0] = acc.x;
}

// bytes must be a multiple of workgroups * waves * 1024; the launch reads exactly `bytes`.
void launch_stream_read(const void* p, size_t bytes, int workgroups, int waves, uint32_t* sink, hipStream_t st) {
    const size_t units_per_wave = bytes / 1024 / ((size_t)workgroups * waves);
    hipLaunchKernelGGL(stream_read_k<8>, dim3(workgroups), dim3(waves * 64), 0, st, (const u32x4*)p, units_per_wave, sink);
}

// NACC independent accumulators per wave, `iters` rounds of NACC matrix instructions from registers.
template <int NACC>
__global__ __launch_bounds__(256) void mfma_loop_k(float* out, int iters) {
    f32x16 acc[NACC];
#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[a][i] = 0.f;
    bf16x8 x, w;
#pragma unroll
    for (int i = 0; i < 8; ++i) { x[i] = (__bf16)(float)(threadIdx.x & 3); w[i] = (__bf16)1.0f; }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int a = 0; a < NACC; ++a) acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w, x, acc[a], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[a][i];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// out: workgroups * 256 floats.  Returns the flops of the launch (2 * 32 * 32 * 16 per instruction).
double launch_mfma_loop(float* out, int workgroups, int iters, hipStream_t st) {
    constexpr int NACC = 4;
    hipLaunchKernelGGL(mfma_loop_k<NACC>, dim3(workgroups), dim3(256), 0, st, out, iters);
    return (double)workgroups * 4 * (double)iters * NACC * 32768.0;
}

}  // namespace rdlm
