// Device code shared by the bf16 GEMM kernels (kernels_gemm.hip, kernels_gemm_lds.hip): kernel
// argument block, packed weight block layouts, deferred-RMSNorm row factors and the epilogues.
#pragma once
#include "rdlm_internal.h"

namespace rdlm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct GemmArgs {
    const bf16x8* xp;
    const bf16x8* wp;
    float* out;             // EPI_F32: [ksplit][rows][N] partial sums; EPI_ARGMAX: logits [rows][N] or null
    int N, K16, n_groups, m_chunks, ksplit;
    int max_tiles;          // the host's bound on the tile count (the launch covers that many)
    size_t part_stride;
    const int32_t* n_tiles;
    GemmEpilogue epi;
};

// The GEMM kernels take the fields of GemmArgs that the K loop needs as leading scalar arguments,
// in this order, so that they can be preloaded into scalar registers when the wave starts (the
// first 16 dwords of the argument block); the epilogue's parameters follow as a struct.
#define GEMM_KERNEL_PARAMS                                                                                      \
    const bf16x8 *xp_, const bf16x8 *wp_, const int32_t *n_tiles_, float *out_, int N_, int K16_, int n_groups_, \
        int m_chunks_, int ksplit_, int max_tiles_, size_t part_stride_, GemmEpilogue epi_
#define GEMM_KERNEL_ARGS_STRUCT                                                                                 \
    GemmArgs A;                                                                                                 \
    A.xp = xp_; A.wp = wp_; A.n_tiles = n_tiles_; A.out = out_; A.N = N_; A.K16 = K16_; A.n_groups = n_groups_; \
    A.m_chunks = m_chunks_; A.ksplit = ksplit_; A.max_tiles = max_tiles_; A.part_stride = part_stride_; A.epi = epi_
#define GEMM_LAUNCH_ARGS(a)                                                                                     \
    (a).xp, (a).wp, (a).n_tiles, (a).out, (a).N, (a).K16, (a).n_groups, (a).m_chunks, (a).ksplit, (a).max_tiles, \
        (a).part_stride, (a).epi

// Epilogue helpers ---------------------------------------------------------------------------
__device__ inline float silu_f(float a) { return a / (1.0f + __expf(-a)); }

// Column of the canonical [rows][N] output that row f (0..31) of packed weight block `blk` is.
//   WL_NATURAL: 32 consecutive output features per block.
//   WL_GU16 (gate/up, N = 2F): block j holds gate features [16j, 16j+16) in rows 0..15 and the up
//     features of the same indices in rows 16..31, so a SwiGLU pair sits in one accumulator lane.
//   WL_ROPE (q | k | v, N = 3h): in the q and k sections block j' of a head holds head dims
//     [16j', 16j'+16) and their rotate-half partners [d/2 + 16j', d/2 + 16j' + 16); v is natural.
__host__ __device__ inline int canon_col(int layout, int blk, int f, int N, int n_heads, int head_dim) {
    if (layout == WL_GU16) {
        const int F = N >> 1;
        return (f < 16 ? 0 : F) + 16 * blk + (f & 15);
    }
    if (layout == WL_ROPE) {
        const int h = n_heads * head_dim, hb = h >> 5, sec = blk / hb, r = blk - sec * hb;
        if (sec == 2) return blk * 32 + f;
        const int per = head_dim >> 5, head = r / per, j = r - head * per;
        return sec * h + head * head_dim + (f < 16 ? 0 : (head_dim >> 1)) + 16 * j + (f & 15);
    }
    return blk * 32 + f;
}

// Deferred RMSNorm: 1 / sqrt(mean(x^2) + eps) of the lane's row in each of the workgroup's row tiles,
// from the per-slot sums of squares the producer of the operand left (slot-major, so a wave reads 32
// consecutive floats per slot).  Called before the K loop: the loads overlap the weight stream.
template <int MT>
__device__ __forceinline__ void gemm_row_scales(const GemmArgs& A, int t0, int n_tiles, float (&sc)[MT]) {
    const int col = threadIdx.x & 31;
#pragma unroll
    for (int b = 0; b < MT; ++b) {
        sc[b] = 1.0f;
        if (A.epi.row_ssq) {
            const size_t row = (size_t)min(t0 + b, n_tiles - 1) * 32 + col;
            float ssq = 0.f;
            for (int c = 0; c < A.epi.ssq_chunks; ++c) ssq += A.epi.row_ssq[(size_t)c * A.epi.ssq_stride + row];
            sc[b] = 1.0f / sqrtf(ssq / (float)A.epi.norm_h + A.epi.norm_eps);
        }
    }
}

// Finishing work of a workgroup that holds the sums of NB feature blocks x MT row tiles.
// quad_sum(a, b, q, out[4]) returns accumulator registers 4q..4q+3 of (block a, row tile b) for this
// lane: rows 8q + 4g + i of the weight block against activation row `col`.  The work is cut into
// units of one register quad -- or, for the epilogues that pair row f of a block with row f + 16
// (SwiGLU on WL_GU16 blocks, RoPE on WL_ROPE blocks), of quad q together with quad q + 2 -- and
// wave w of the DEAL waves that share the sums takes the units u with u % DEAL == w.
// OWN_ROWS: the waves of the workgroup hold different row tiles (no other wave has candidates for
// this wave's rows), so the argmax epilogue needs no exchange between waves.
template <int MT, int NB, int WAVES, int DEAL, int EPI, class QuadSum, class CV, class CI, bool OWN_ROWS = false>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& A, const int (&blk)[NB], int t0, int n_tiles, int ks,
                                              int grp, const float (&sc)[MT], QuadSum quad_sum, CV& cand_v,
                                              CI& cand_i, const TileDesc* pre_td = nullptr,
                                              const int* pre_kvblk = nullptr) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nblk = A.N >> 5;
    const int col = lane & 31, g = lane >> 5;
    constexpr bool PAIRED = (EPI == EPI_SWIGLU || EPI == EPI_ROPE_KV);
    constexpr int UQ = PAIRED ? 2 : 4;

    // per row tile: the descriptor of the lane's own row -- the rows of a tile may belong to different
    // sequences (sc: deferred RMSNorm factor of the lane's row)
    TileDesc td[MT];
#pragma unroll
    for (int b = 0; b < MT; ++b) {
        const int t = min(t0 + b, n_tiles - 1);
        // (pre_td / pre_kvblk: the descriptor and the cache block of the lane's row, fetched by the caller
        // before its K loop so that the stores below do not wait for two loads in a row)
        if (EPI == EPI_ARGMAX || EPI == EPI_ROPE_KV) td[b] = pre_td ? pre_td[b] : A.epi.tiles[t * 32 + col];
    }
    float best_v[MT];
    int best_i[MT];
#pragma unroll
    for (int b = 0; b < MT; ++b) { best_v[b] = -INFINITY; best_i[b] = 0x7fffffff; }

#pragma unroll
    for (int unit = 0; unit < NB * MT * UQ; ++unit) {
        const int a = unit / (MT * UQ), b = (unit / UQ) % MT, q = unit % UQ;
        if (DEAL > 1 && unit % DEAL != wave) continue;
        const int t = t0 + b;
        if (t >= n_tiles || blk[a] >= nblk) continue;
        const size_t row = (size_t)t * 32 + col;
        const int f0 = q * 8 + g * 4;
        float lo[4], hi[4];
        quad_sum(a, b, q, lo);
        if (PAIRED) quad_sum(a, b, q + 2, hi);
#pragma unroll
        for (int i = 0; i < 4; ++i) { lo[i] *= sc[b]; if (PAIRED) hi[i] *= sc[b]; }

        if constexpr (EPI == EPI_F32) {
            float* o = A.out + (size_t)ks * A.part_stride;
            const int c0 = canon_col(A.epi.layout, blk[a], f0, A.N, A.epi.n_heads, A.epi.head_dim);
            if (A.epi.fold_counter) {
                // another workgroup reads these: written through to memory, in accumulator order
                // [group][split][register][lane] so that a wave writes 256 contiguous bytes
                float* pf = A.out + (((size_t)grp * A.ksplit + ks) * (NB * 16) + (a * 4 + q) * 4) * 64 + lane;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    __hip_atomic_store(pf + i * 64, lo[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            } else {
                *reinterpret_cast<float4*>(o + row * A.N + c0) = make_float4(lo[0], lo[1], lo[2], lo[3]);
            }
        } else if constexpr (EPI == EPI_SWIGLU) {
            // rows f0.. are gate features 16 blk + f0.., rows 16 + f0.. the up features of the same index
            const int F = A.N >> 1;
            ushort4 pk;
            pk.x = f32_to_bf16(silu_f(lo[0]) * hi[0]);
            pk.y = f32_to_bf16(silu_f(lo[1]) * hi[1]);
            pk.z = f32_to_bf16(silu_f(lo[2]) * hi[2]);
            pk.w = f32_to_bf16(silu_f(lo[3]) * hi[3]);
            *reinterpret_cast<ushort4*>(reinterpret_cast<uint16_t*>(A.epi.act) +
                                        packed_off((int)row, blk[a] * 16 + f0, F)) = pk;
        } else if constexpr (EPI == EPI_ROPE_KV) {
            // q, k: rotate (u, u + d/2) by the row's angle table, q -> bf16 rows for the attention
            // kernel, k -> the layer's cache at the row's position; v -> transposed cache
            const int D = A.epi.head_dim, HALF = D >> 1, H = A.epi.n_heads, h = H * D;
            const int hb = h >> 5, sec = blk[a] / hb, r = blk[a] - sec * hb, per = D >> 5;
            const int head = r / per, j = r - head * per;
            const int pos = td[b].pos0;
            const bool valid = td[b].n_valid > 0;
            if (sec == 2) {
                if (valid) {
                    const int u0 = 32 * j + f0;
                    uint16_t* Vt = reinterpret_cast<uint16_t*>(A.epi.vc) +
                                   (pre_kvblk ? (size_t)pre_kvblk[b] * ((size_t)32 * h)
                                              : kv_block_base(A.epi.kv, td[b].seq, pos >> 5, (size_t)32 * h)) +
                                   ((size_t)head * D + u0) * 32 + vt_slot(pos & 31);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        Vt[(size_t)i * 32] = f32_to_bf16(lo[i]);
                        Vt[(size_t)(16 + i) * 32] = f32_to_bf16(hi[i]);
                    }
                }
            } else {
                const int u0 = 16 * j + f0;                  // < HALF; partner u0 + HALF
                // the lane's four (cos, sin) pairs are 32 contiguous bytes of its row's table (u0 is a
                // multiple of 4, the table 16-byte aligned): two 16-byte loads
                const float4* __restrict__ table4 =
                    reinterpret_cast<const float4*>(A.epi.rope_table + 2 * (row * HALF + u0));
                const float4 t01 = table4[0], t23 = table4[1];
                const float cs_c[4] = {t01.x, t01.z, t23.x, t23.z}, cs_s[4] = {t01.y, t01.w, t23.y, t23.w};
                ushort4 p0, p1;
                uint16_t* p0p = reinterpret_cast<uint16_t*>(&p0);
                uint16_t* p1p = reinterpret_cast<uint16_t*>(&p1);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    p0p[i] = f32_to_bf16(lo[i] * cs_c[i] - hi[i] * cs_s[i]);
                    p1p[i] = f32_to_bf16(hi[i] * cs_c[i] + lo[i] * cs_s[i]);
                }
                if (sec == 0) {
                    uint16_t* dst = reinterpret_cast<uint16_t*>(A.epi.q_out) + row * h + head * D + u0;
                    *reinterpret_cast<ushort4*>(dst) = p0;
                    *reinterpret_cast<ushort4*>(dst + HALF) = p1;
                } else if (valid) {
                    uint16_t* Kc = reinterpret_cast<uint16_t*>(A.epi.kc) +
                                   (pre_kvblk ? (size_t)pre_kvblk[b] * ((size_t)32 * h)
                                              : kv_block_base(A.epi.kv, td[b].seq, pos >> 5, (size_t)32 * h));
                    *reinterpret_cast<ushort4*>(Kc + k_cache_off(pos & 31, head, u0, H, D)) = p0;
                    *reinterpret_cast<ushort4*>(Kc + k_cache_off(pos & 31, head, u0 + HALF, H, D)) = p1;
                }
            }
        } else {   // EPI_ARGMAX
            const int c0 = blk[a] * 32 + f0;
            if (A.out) *reinterpret_cast<float4*>(A.out + row * A.N + c0) = make_float4(lo[0], lo[1], lo[2], lo[3]);
            float gn[4] = {0.f, 0.f, 0.f, 0.f};
            if (A.epi.temperature > 0.f) {
                uint32_t x[4];
                // a sequence counts its sampler steps from the step it joined at
                const int lstep = A.epi.step - (A.epi.seq_step0 ? A.epi.seq_step0[td[b].seq] : 0);
                philox4x32_10(c0 >> 2, td[b].pos0, td[b].rng, ((uint32_t)lstep << 4) | TAG_SAMPLE, A.epi.k0,
                              A.epi.k1, x);
#pragma unroll
                for (int i = 0; i < 4; ++i) gn[i] = -logf(-logf(u24_open(x[i])));
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float s = lo[i];
                if (A.epi.temperature > 0.f) s = s / A.epi.temperature + gn[i];
                if (s > best_v[b] || (s == best_v[b] && c0 + i < best_i[b])) { best_v[b] = s; best_i[b] = c0 + i; }
            }
        }
    }
    if constexpr (EPI == EPI_ARGMAX) {
        // best over the two half-waves, then over the waves; one candidate per (group, row)
#pragma unroll
        for (int b = 0; b < MT; ++b) {
            float ov = __shfl_xor(best_v[b], 32);
            int oi = __shfl_xor(best_i[b], 32);
            if (ov > best_v[b] || (ov == best_v[b] && oi < best_i[b])) { best_v[b] = ov; best_i[b] = oi; }
            if constexpr (OWN_ROWS) {
                if (g == 0 && t0 + b < n_tiles) {
                    const size_t o = (size_t)grp * A.epi.cand_stride + (size_t)(t0 + b) * 32 + col;
                    A.epi.cand_val[o] = best_v[b];
                    A.epi.cand_idx[o] = best_i[b];
                }
            } else {
                if (g == 0) { cand_v[wave][b][col] = best_v[b]; cand_i[wave][b][col] = best_i[b]; }
            }
        }
        if constexpr (OWN_ROWS) return;
        __syncthreads();
        if (wave == 0 && g == 0) {
#pragma unroll
            for (int b = 0; b < MT; ++b) {
                if (t0 + b >= n_tiles) continue;
                float bv = cand_v[0][b][col];
                int bi = cand_i[0][b][col];
#pragma unroll
                for (int w = 1; w < WAVES; ++w) {
                    float ov = cand_v[w][b][col];
                    int oi = cand_i[w][b][col];
                    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
                }
                size_t o = (size_t)grp * A.epi.cand_stride + (size_t)(t0 + b) * 32 + col;
                A.epi.cand_val[o] = bv;
                A.epi.cand_idx[o] = bi;
            }
        }
    }
}

}  // namespace rdlm
