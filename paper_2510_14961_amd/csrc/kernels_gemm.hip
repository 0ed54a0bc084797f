// Weight-streaming GEMMs  y[rows, N] = x[rows, K] . W[N, K]^T  for the projections of the layer
// (adapter, QKV, output, gate/up, down, LM head).
//
// bf16 path (gfx950 MFMA): at the window sizes of the sampler (tens to a few hundred rows) these
// products are bound by reading W from HBM once, so the kernel is organised around the weight
// stream.  W is stored pre-tiled: a tile is 32 output features x 16 input features, 1 KiB, laid
// out in the lane order of the A operand of v_mfma_f32_32x32x16_bf16, tiles ordered
// [feature block][k tile] -- a wave walking along K reads one contiguous run with 16-byte loads
// per lane.  Activations are stored the same way (32 rows x 16 k per tile, B operand order) by
// the kernels that produce them, so the inner loop is: load NB weight tiles + MT activation
// tiles, NB*MT MFMAs.  The waves of a workgroup split the K range of one feature-block group and
// are summed through LDS in a fixed order; an optional split of K across workgroups writes
// separate partial outputs that the consumer adds in a fixed order (no atomics: results are
// bit-reproducible).
#include "rdlm_internal.h"

namespace rdlm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int UNROLL = 4;   // k tiles fetched ahead per wave

template <int MT, int NB, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void gemm_bf16_k(const bf16x8* __restrict__ xp,
                                                            const bf16x8* __restrict__ wp, float* __restrict__ out,
                                                            int N, int K16, int n_groups, int m_chunks, int ksplit,
                                                            size_t part_stride, const int32_t* n_tiles_p) {
    extern __shared__ float red[];                 // [WAVES][NB*MT*16][64]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int bid = blockIdx.x;
    const int mc = bid % m_chunks; bid /= m_chunks;  // row chunk fastest: neighbours share weights
    const int ks = bid % ksplit;
    const int grp = bid / ksplit;
    const int n_tiles = *n_tiles_p;
    const int t0 = mc * MT;
    if (t0 >= n_tiles) return;
    const int nblk = N >> 5;
    // K range of this wave: K16 tiles split evenly over ksplit * WAVES slices
    const int slices = ksplit * WAVES, sl = ks * WAVES + wave;
    const int kbeg = (int)(((long long)K16 * sl) / slices), kend = (int)(((long long)K16 * (sl + 1)) / slices);

    f32x16 acc[NB][MT];
#pragma unroll
    for (int a = 0; a < NB; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    const bf16x8* wbase[NB];
    const bf16x8* xbase[MT];
#pragma unroll
    for (int a = 0; a < NB; ++a) {
        int nb = min(grp * NB + a, nblk - 1);       // clamp: a ragged last group re-reads a valid block
        wbase[a] = wp + ((size_t)nb * K16) * 64 + lane;
    }
#pragma unroll
    for (int b = 0; b < MT; ++b) {
        int t = min(t0 + b, n_tiles - 1);
        xbase[b] = xp + ((size_t)t * K16) * 64 + lane;
    }

    int kt = kbeg;
    for (; kt + UNROLL <= kend; kt += UNROLL) {
        bf16x8 wv[UNROLL][NB], xv[UNROLL][MT];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
            for (int a = 0; a < NB; ++a) wv[u][a] = __builtin_nontemporal_load(wbase[a] + (size_t)(kt + u) * 64);
#pragma unroll
            for (int b = 0; b < MT; ++b) xv[u][b] = xbase[b][(size_t)(kt + u) * 64];
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
#pragma unroll
            for (int a = 0; a < NB; ++a)
#pragma unroll
                for (int b = 0; b < MT; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv[u][a], xv[u][b], acc[a][b], 0, 0, 0);
    }
    for (; kt < kend; ++kt) {
#pragma unroll
        for (int a = 0; a < NB; ++a) {
            bf16x8 w = __builtin_nontemporal_load(wbase[a] + (size_t)kt * 64);
#pragma unroll
            for (int b = 0; b < MT; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w, xbase[b][(size_t)kt * 64], acc[a][b], 0, 0, 0);
        }
    }

    // cross-wave sum in a fixed order: every wave deposits its accumulators, then wave w adds up
    // and stores the registers r with r % WAVES == w
    constexpr int REGS = NB * MT * 16;
    if (WAVES > 1) {
#pragma unroll
        for (int a = 0; a < NB; ++a)
#pragma unroll
            for (int b = 0; b < MT; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) red[((size_t)wave * REGS + (a * MT + b) * 16 + i) * 64 + lane] = acc[a][b][i];
        __syncthreads();
    }
    float* o = out + (size_t)ks * part_stride;
    const int col = lane & 31, g = lane >> 5;
#pragma unroll
    for (int a = 0; a < NB; ++a) {
        int nb = grp * NB + a;
        if (nb >= nblk) continue;
#pragma unroll
        for (int b = 0; b < MT; ++b) {
            int t = t0 + b;
            if (t >= n_tiles) continue;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (WAVES > 1 && ((a * MT + b) * 4 + q) % WAVES != wave) continue;
                float4 v;
                float* vv = reinterpret_cast<float*>(&v);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    int r = (a * MT + b) * 16 + q * 4 + i;
                    if (WAVES > 1) {
                        float s = 0.f;
#pragma unroll
                        for (int w = 0; w < WAVES; ++w) s += red[((size_t)w * REGS + r) * 64 + lane];
                        vv[i] = s;
                    } else {
                        vv[i] = acc[a][b][q * 4 + i];
                    }
                }
                // accumulator register q*4+i of lane (col, g) is feature 8q + 4g + i of the block, row `col`
                size_t row = (size_t)t * 32 + col;
                *reinterpret_cast<float4*>(o + row * N + nb * 32 + q * 8 + g * 4) = v;
            }
        }
    }
}

template <int MT, int NB, int WAVES>
static void launch_cfg(const void* xp, const void* wp, float* out, int N, int K, size_t part_stride, int ksplit,
                       const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    int nblk = N / 32, groups = (nblk + NB - 1) / NB, m_chunks = (max_tiles + MT - 1) / MT;
    size_t lds = WAVES > 1 ? (size_t)WAVES * NB * MT * 16 * 64 * sizeof(float) : 0;
    hipLaunchKernelGGL((gemm_bf16_k<MT, NB, WAVES>), dim3(groups * ksplit * m_chunks), dim3(WAVES * 64), lds, st,
                       (const bf16x8*)xp, (const bf16x8*)wp, out, N, K / 16, groups, m_chunks, ksplit, part_stride,
                       n_tiles);
}

void launch_gemm_bf16(const void* xp, const void* wp, float* out, int N, int K, size_t part_stride,
                      GemmPlan plan, const int32_t* n_tiles, int max_tiles, hipStream_t st) {
#define RDLM_CASE(MT_, NB_, W_)                                                                        \
    if (plan.mt == MT_ && plan.nb == NB_ && plan.waves == W_) {                                        \
        launch_cfg<MT_, NB_, W_>(xp, wp, out, N, K, part_stride, plan.ksplit, n_tiles, max_tiles, st); \
        return;                                                                                        \
    }
    RDLM_CASE(1, 1, 4) RDLM_CASE(1, 2, 4) RDLM_CASE(1, 4, 4) RDLM_CASE(1, 1, 8) RDLM_CASE(1, 2, 8)
    RDLM_CASE(2, 1, 4) RDLM_CASE(2, 2, 4) RDLM_CASE(4, 1, 4) RDLM_CASE(4, 2, 4)
    RDLM_CASE(1, 2, 2) RDLM_CASE(1, 4, 2) RDLM_CASE(1, 2, 1) RDLM_CASE(1, 4, 1)
#undef RDLM_CASE
    launch_cfg<1, 1, 4>(xp, wp, out, N, K, part_stride, plan.ksplit, n_tiles, max_tiles, st);
}

// canonical bf16 [N][K] -> MFMA-ordered tiles [N/32][K/16][64 lanes][8]
__global__ void pack_weight_k(const uint16_t* w, uint16_t* wp, int N, int K) {
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;       // one lane-vector (8 elements) each
    size_t total = (size_t)(N / 32) * (K / 16) * 64;
    if (idx >= total) return;
    int lane = idx & 63;
    size_t tile = idx >> 6;
    int kt = (int)(tile % (K / 16));
    int nb = (int)(tile / (K / 16));
    const uint16_t* src = w + ((size_t)nb * 32 + (lane & 31)) * K + kt * 16 + (lane >> 5) * 8;
    uint4 v = *reinterpret_cast<const uint4*>(src);
    *reinterpret_cast<uint4*>(wp + idx * 8) = v;
}
void launch_pack_weight(const void* w, void* wp, int N, int K, hipStream_t st) {
    size_t total = (size_t)(N / 32) * (K / 16) * 64;
    hipLaunchKernelGGL(pack_weight_k, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const uint16_t*)w,
                       (uint16_t*)wp, N, K);
}

// f32 rows [rows][K] -> packed bf16 activation tiles (rows rounded up to 32 must be allocated)
__global__ void pack_rows_k(const float* x, uint16_t* xp, int rows, int K) {
    int r = blockIdx.x;
    for (int k = threadIdx.x; k < K; k += blockDim.x)
        xp[packed_off(r, k, K)] = f32_to_bf16(r < rows ? x[(size_t)r * K + k] : 0.f);
}
void launch_pack_rows(const float* x, void* xp, int rows, int K, hipStream_t st) {
    int padded = (rows + 31) / 32 * 32;
    hipLaunchKernelGGL(pack_rows_k, dim3(padded), dim3(256), 0, st, x, (uint16_t*)xp, rows, K);
}

// ---------------------------------------------------------------------------------------------
// f32 path (the small fp32 model): plain FMA kernel.  A wave owns NR weight rows; lanes stride
// over K (coalesced reads of W and x), 32 rows of x per tile; wave reduction at the end.
constexpr int F32_NR = 2;
__global__ __launch_bounds__(256) void gemm_f32_k(const float* __restrict__ x, const float* __restrict__ w,
                                                    float* __restrict__ out, int N, int K, const int32_t* n_tiles_p) {
    int t = blockIdx.y;
    if (t >= *n_tiles_p) return;
    int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int n0 = (blockIdx.x * 4 + wave) * F32_NR;
    if (n0 >= N) return;
    float acc[F32_NR][32];
#pragma unroll
    for (int a = 0; a < F32_NR; ++a)
#pragma unroll
        for (int m = 0; m < 32; ++m) acc[a][m] = 0.f;
    const float* xr = x + (size_t)t * 32 * K;
    for (int k = lane; k < K; k += 64) {
        float wv[F32_NR];
#pragma unroll
        for (int a = 0; a < F32_NR; ++a) wv[a] = (n0 + a < N) ? w[(size_t)(n0 + a) * K + k] : 0.f;
#pragma unroll
        for (int m = 0; m < 32; ++m) {
            float xv = xr[(size_t)m * K + k];
#pragma unroll
            for (int a = 0; a < F32_NR; ++a) acc[a][m] = fmaf(wv[a], xv, acc[a][m]);
        }
    }
#pragma unroll
    for (int a = 0; a < F32_NR; ++a)
#pragma unroll
        for (int m = 0; m < 32; ++m) {
            float v = acc[a][m];
            for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
            if (lane == 0 && n0 + a < N) out[((size_t)t * 32 + m) * N + n0 + a] = v;
        }
}
void launch_gemm_f32(const float* x, const float* w, float* out, int N, int K, const int32_t* n_tiles,
                     int max_tiles, hipStream_t st) {
    dim3 grid((N + 4 * F32_NR - 1) / (4 * F32_NR), max_tiles);
    hipLaunchKernelGGL(gemm_f32_k, grid, dim3(256), 0, st, x, w, out, N, K, n_tiles);
}

}  // namespace rdlm
