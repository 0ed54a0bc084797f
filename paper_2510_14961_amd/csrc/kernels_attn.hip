// Window-vs-cache causal attention: the rows of a tile (one sequence, contiguous positions)
// attend to that sequence's cache positions 0..their own position -- the frozen prefix plus the
// in-flight positions at or before them, all at their latest recurrence (Sec. 3.2, Sec. 3.3).
//
// bf16 path: one workgroup per (head, tile, KV split); its 4 waves take key blocks of 32
// round-robin.  Scores are computed transposed, S^T = K . Q^T (keys on MFMA rows, queries on
// columns), so a lane owns one query column: the running max / sum of the online softmax are
// per-lane scalars (one exchange between the two half-waves), and the probabilities already sit
// in the B-operand layout of the second contraction O^T = V^T . P^T.  V is cached transposed,
// [position block][head][dim][32 positions], with the 32 positions of a block stored in the
// order the score accumulator presents them (vt_slot), so both operands are 16-byte loads.
// Waves are merged through LDS; KV splits write (max, sum, O) partials merged by a second kernel.
#include "rdlm_internal.h"

namespace rdlm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int ATT_WAVES = 4;

// partial record per (tile, head, split): m[32], l[32], O[32][D]
__host__ __device__ inline size_t att_rec_floats(int D) { return 64 + 32 * (size_t)D; }

size_t attention_ws_floats(int max_tiles, int H, int d, int nsplit) {
    return (size_t)max_tiles * H * nsplit * att_rec_floats(d);
}

template <int D>
__global__ __launch_bounds__(ATT_WAVES * 64) void attn_bf16_k(const uint16_t* __restrict__ q,
                                                               const uint16_t* __restrict__ kc,
                                                               const uint16_t* __restrict__ vc, uint16_t* __restrict__ out,
                                                               int H, size_t seq_stride, int nsplit, float* __restrict__ ws,
                                                               const TileDesc* tiles, const int32_t* n_tiles) {
    constexpr int DK = D / 16;      // k steps of the score contraction
    constexpr int DB = D / 32;      // 32-row blocks of O^T
    __shared__ float sm[ATT_WAVES][2][32];
    __shared__ float so[ATT_WAVES][DB * 16][64];
    const int hd = blockIdx.x, t = blockIdx.y, sp = blockIdx.z;
    if (t >= *n_tiles) return;
    const TileDesc td = tiles[t];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int h = H * D;
    const int n_keys = td.pos0 + td.n_valid;                 // keys 0..n_keys-1 are visible to the tile
    const int nkb = (n_keys + 31) >> 5;
    const int kb_lo = (int)(((long long)nkb * sp) / nsplit), kb_hi = (int)(((long long)nkb * (sp + 1)) / nsplit);
    const uint16_t* K = kc + (size_t)td.seq * seq_stride;
    const uint16_t* Vt = vc + (size_t)td.seq * seq_stride;
    const float scale = 1.0f / sqrtf((float)D);
    const int qpos = td.pos0 + col;                           // position of this lane's query

    bf16x8 qv[DK];
    {
        const uint16_t* qr = q + ((size_t)t * 32 + col) * h + hd * D + g * 8;
#pragma unroll
        for (int i = 0; i < DK; ++i) qv[i] = *reinterpret_cast<const bf16x8*>(qr + i * 16);
    }
    f32x16 o[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[b][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;                     // l_run: this half-wave's share of the sum

    for (int kb = kb_lo + wave; kb < kb_hi; kb += ATT_WAVES) {
        f32x16 s;
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = 0.f;
        const uint16_t* kr = K + ((size_t)(kb * 32 + col) * H + hd) * D + g * 8;
#pragma unroll
        for (int i = 0; i < DK; ++i) {
            bf16x8 kv = *reinterpret_cast<const bf16x8*>(kr + i * 16);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kv, qv[i], s, 0, 0, 0);
        }
        // register r of lane (col, g) is key kb*32 + 8*(r/4) + 4g + r%4 against query `col`
        float bm = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int key = kb * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
            float v = (key <= qpos) ? s[r] * scale : -INFINITY;
            s[r] = v;
            bm = fmaxf(bm, v);
        }
        bm = fmaxf(bm, __shfl_xor(bm, 32));
        float m_new = fmaxf(m_run, bm);
        float m_use = (m_new == -INFINITY) ? 0.f : m_new;     // nothing visible yet: all p become 0
        float alpha = __expf(m_run - m_use);                  // m_run = -inf gives 0
        float psum = 0.f;
        bf16x8 p0, p1;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            float a = __expf(s[r] - m_use), b = __expf(s[r + 8] - m_use);
            psum += a + b;
            p0[r] = (__bf16)a;
            p1[r] = (__bf16)b;
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
        const uint16_t* vr = Vt + ((size_t)kb * H + hd) * D * 32 + (size_t)col * 32 + g * 8;
#pragma unroll
        for (int b = 0; b < DB; ++b) {
#pragma unroll
            for (int i = 0; i < 16; ++i) o[b][i] *= alpha;
            bf16x8 v0 = *reinterpret_cast<const bf16x8*>(vr + (size_t)b * 32 * 32);
            bf16x8 v1 = *reinterpret_cast<const bf16x8*>(vr + (size_t)b * 32 * 32 + 16);
            o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v0, p0, o[b], 0, 0, 0);
            o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v1, p1, o[b], 0, 0, 0);
        }
    }
    // merge the waves: common max, rescaled sums
    l_run += __shfl_xor(l_run, 32);
    if (g == 0) { sm[wave][0][col] = m_run; sm[wave][1][col] = l_run; }
    __syncthreads();
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < ATT_WAVES; ++w) M = fmaxf(M, sm[w][0][col]);
    float Muse = (M == -INFINITY) ? 0.f : M;
    float L = 0.f;
#pragma unroll
    for (int w = 0; w < ATT_WAVES; ++w) L += sm[w][1][col] * __expf(sm[w][0][col] - Muse);
    float mine = __expf(m_run - Muse);
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) so[wave][b * 16 + i][lane] = o[b][i] * mine;
    __syncthreads();
    // wave w finishes the registers r with r % ATT_WAVES == w; register (b, i) of lane (col, g) is
    // dim 32b + 8*(i/4) + 4g + i%4 of query `col`; four consecutive i are four consecutive dims
    for (int quad = wave; quad < DB * 4; quad += ATT_WAVES) {
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float acc = 0.f;
#pragma unroll
            for (int w = 0; w < ATT_WAVES; ++w) acc += so[w][quad * 4 + i][lane];
            v[i] = acc;
        }
        int b = quad >> 2, qd = quad & 3;
        int dim = 32 * b + 8 * qd + 4 * g;
        int row = t * 32 + col;
        if (nsplit == 1) {
            float inv = L > 0.f ? 1.0f / L : 0.f;
            ushort4 pk;
            pk.x = f32_to_bf16(v[0] * inv); pk.y = f32_to_bf16(v[1] * inv);
            pk.z = f32_to_bf16(v[2] * inv); pk.w = f32_to_bf16(v[3] * inv);
            *reinterpret_cast<ushort4*>(out + packed_off(row, hd * D + dim, h)) = pk;
        } else {
            float* rec = ws + (((size_t)t * H + hd) * nsplit + sp) * att_rec_floats(D);
            *reinterpret_cast<float4*>(rec + 64 + (size_t)col * D + dim) = make_float4(v[0], v[1], v[2], v[3]);
        }
    }
    if (nsplit > 1 && wave == 0 && g == 0) {
        float* rec = ws + (((size_t)t * H + hd) * nsplit + sp) * att_rec_floats(D);
        rec[col] = M;
        rec[32 + col] = L;
    }
}

template <int D>
__global__ void attn_merge_k(const float* __restrict__ ws, uint16_t* __restrict__ out, int H, int nsplit,
                             const int32_t* n_tiles) {
    const int hd = blockIdx.x, t = blockIdx.y;
    if (t >= *n_tiles) return;
    const float* base = ws + ((size_t)t * H + hd) * nsplit * att_rec_floats(D);
    for (int idx = threadIdx.x; idx < 32 * (D / 4); idx += blockDim.x) {
        int col = idx / (D / 4), dim = (idx % (D / 4)) * 4;
        float M = -INFINITY;
        for (int s = 0; s < nsplit; ++s) M = fmaxf(M, base[s * att_rec_floats(D) + col]);
        float Muse = (M == -INFINITY) ? 0.f : M;
        float L = 0.f;
        float4 acc = make_float4(0, 0, 0, 0);
        for (int s = 0; s < nsplit; ++s) {
            const float* rec = base + s * att_rec_floats(D);
            float w = __expf(rec[col] - Muse);
            L += rec[32 + col] * w;
            float4 v = *reinterpret_cast<const float4*>(rec + 64 + (size_t)col * D + dim);
            acc.x += v.x * w; acc.y += v.y * w; acc.z += v.z * w; acc.w += v.w * w;
        }
        float inv = L > 0.f ? 1.0f / L : 0.f;
        ushort4 pk;
        pk.x = f32_to_bf16(acc.x * inv); pk.y = f32_to_bf16(acc.y * inv);
        pk.z = f32_to_bf16(acc.z * inv); pk.w = f32_to_bf16(acc.w * inv);
        *reinterpret_cast<ushort4*>(out + packed_off(t * 32 + col, hd * D + dim, H * D)) = pk;
    }
}

// f32 path: one workgroup per (row, head); scores kept in LDS.
constexpr int ATT_F32_MAXKEYS = 8192;
__global__ __launch_bounds__(256) void attn_f32_k(const float* __restrict__ q, const float* __restrict__ kc,
                                                    const float* __restrict__ vc, float* __restrict__ out, int H, int d,
                                                    size_t seq_stride, const TileDesc* tiles, const int32_t* n_tiles) {
    __shared__ float sc[ATT_F32_MAXKEYS];
    __shared__ float red[8];
    int r = blockIdx.x, hd = blockIdx.y, t = r >> 5, j = r & 31;
    if (t >= *n_tiles) return;
    TileDesc td = tiles[t];
    int h = H * d;
    float* orow = out + (size_t)r * h + hd * d;
    if (j >= td.n_valid) {
        for (int c = threadIdx.x; c < d; c += blockDim.x) orow[c] = 0.f;
        return;
    }
    int nk = td.pos0 + j + 1;
    const float* K = kc + (size_t)td.seq * seq_stride;
    const float* V = vc + (size_t)td.seq * seq_stride;
    const float* qr = q + (size_t)r * h + hd * d;
    float scale = 1.0f / sqrtf((float)d);
    float mx = -INFINITY;
    for (int k = threadIdx.x; k < nk; k += blockDim.x) {
        const float* kr = K + (size_t)k * h + hd * d;
        float s = 0.f;
        for (int c = 0; c < d; ++c) s = fmaf(qr[c], kr[c], s);
        s *= scale;
        sc[k] = s;
        mx = fmaxf(mx, s);
    }
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float sum = 0.f;
    for (int k = threadIdx.x; k < nk; k += blockDim.x) {
        float p = expf(sc[k] - mx);
        sc[k] = p;
        sum += p;
    }
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[4 + (threadIdx.x >> 6)] = sum;
    __syncthreads();
    sum = red[4] + red[5] + red[6] + red[7];
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
        float acc = 0.f;
        for (int k = 0; k < nk; ++k) acc = fmaf(sc[k], V[(size_t)k * h + hd * d + c], acc);
        orow[c] = acc / sum;
    }
}

void launch_attention(const void* q, const void* kc, const void* vc, void* out, int dtype, int H, int d,
                      size_t seq_stride_elems, int nsplit, float* ws, const TileDesc* tiles,
                      const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    if (dtype == 0) {
        hipLaunchKernelGGL(attn_f32_k, dim3(max_tiles * 32, H), dim3(256), 0, st, (const float*)q, (const float*)kc,
                           (const float*)vc, (float*)out, H, d, seq_stride_elems, tiles, n_tiles);
        return;
    }
    dim3 grid(H, max_tiles, nsplit);
#define RDLM_ATT(D_)                                                                                              \
    if (d == D_) {                                                                                                \
        hipLaunchKernelGGL(attn_bf16_k<D_>, grid, dim3(ATT_WAVES * 64), 0, st, (const uint16_t*)q,                \
                           (const uint16_t*)kc, (const uint16_t*)vc, (uint16_t*)out, H, seq_stride_elems, nsplit, \
                           ws, tiles, n_tiles);                                                                   \
        if (nsplit > 1)                                                                                           \
            hipLaunchKernelGGL(attn_merge_k<D_>, dim3(H, max_tiles), dim3(256), 0, st, ws, (uint16_t*)out, H,     \
                               nsplit, n_tiles);                                                                  \
        return;                                                                                                   \
    }
    RDLM_ATT(32) RDLM_ATT(64) RDLM_ATT(96) RDLM_ATT(128)
#undef RDLM_ATT
}

}  // namespace rdlm
