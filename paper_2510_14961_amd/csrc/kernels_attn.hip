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
// Steps with several row tiles per sequence: consecutive tiles of one sequence form groups of up
// to ATT_GROUP (tile descriptor field `group`) served by one workgroup that stages each K / V
// block in LDS once for all of them (attn_group_k).
#include "rdlm_internal.h"

namespace rdlm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int ATT_WAVES = 4;
constexpr int ATT_MAX_SPLIT = 8;

// partial record per (tile, head, split): m[32], l[32], O[32][D]
__host__ __device__ inline size_t att_rec_floats(int D) { return 64 + 32 * (size_t)D; }

size_t attention_ws_floats(int max_tiles, int H, int d, int nsplit) {
    return (size_t)max_tiles * H * nsplit * att_rec_floats(d);
}

// Online-softmax update of one 32-key block for a lane's query: sacc holds the 16 raw scores of
// lane (col, g) (register r = key kb*32 + 8*(r/4) + 4g + r%4 against query `col`).  m_ref is the
// reference the exponentials are taken against: it follows the running maximum lazily -- it only
// moves when a block's maximum exceeds it by more than ATT_LAZY (so every p stays below
// e^ATT_LAZY, far inside the float and bf16 ranges), because moving it costs a rescale of the
// whole output tile, a trip through the accumulator registers for each of its elements.  The
// final result does not depend on the reference: numerator and denominator carry the same factor.
// Returns alpha, the factor for the running output (exactly 1 when the reference stays), and the
// probabilities as the two B operands of O^T += V^T P^T.  `full` (uniform over the wave): every
// key of the block is visible to every query of the tile, so the causal mask is skipped.
constexpr float ATT_LAZY = 8.0f;
__device__ __forceinline__ float att_block_probs(f32x16& sacc, int kb, int g, int qpos, bool full, float scale,
                                                 float& m_ref, float& l_run, bf16x8& p0, bf16x8& p1) {
    float bm = -INFINITY;
    if (full) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            sacc[r] *= scale;
            bm = fmaxf(bm, sacc[r]);
        }
    } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = kb * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
            const float v = (key <= qpos) ? sacc[r] * scale : -INFINITY;
            sacc[r] = v;
            bm = fmaxf(bm, v);
        }
    }
    bm = fmaxf(bm, __shfl_xor(bm, 32));
    const float m_new = (bm > m_ref + ATT_LAZY) ? bm : m_ref; // also the first visible block: m_ref = -inf
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;   // nothing visible yet: all p become 0
    const float alpha = (m_new == m_ref) ? 1.0f : __expf(m_ref - m_use);   // m_ref = -inf gives 0
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const float a = __expf(sacc[r] - m_use), c = __expf(sacc[r + 8] - m_use);
        psum += a + c;
        p0[r] = (__bf16)a;
        p1[r] = (__bf16)c;
    }
    l_run = l_run * alpha + psum;
    m_ref = m_new;
    return alpha;
}

// One row tile per workgroup (MTQ = 1): narrow windows, ragged batches of short windows.
template <int D, int MTQ>
__global__ __launch_bounds__(ATT_WAVES * 64, D <= 96 ? 2 : 1) void attn_bf16_k(const uint16_t* __restrict__ q,
                                                               const uint16_t* __restrict__ kc,
                                                               const uint16_t* __restrict__ vc, uint16_t* __restrict__ out,
                                                               int H, KvPages kvp, int nsplit, float* __restrict__ ws,
                                                               uint32_t* __restrict__ tickets,
                                                               const TileDesc* tiles, const int32_t* n_tiles) {
    constexpr int DK = D / 16;      // k steps of the score contraction
    constexpr int DB = D / 32;      // 32-row blocks of O^T
    __shared__ float sm[ATT_WAVES][2][32];
    __shared__ float so[ATT_WAVES][DB * 16][64];
    const int hd = blockIdx.x, t = blockIdx.y, sp = blockIdx.z;
    // `tiles` are the segments here: up to 32 rows of one sequence at physical rows prow0 .. (several
    // segments may share a physical row tile: only the segment's own rows are read and written)
    const TileDesc td = tiles[t];                             // valid memory for every t of the grid; read
    if (t >= n_tiles[2]) return;                              // together with the count, used only behind it
    int ng = 1;
    if (MTQ > 1) {
        ng = min(td.group, MTQ);
        if (ng <= 0) return;                                  // served by its group leader
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int h = H * D;
    int n_valid_last = td.n_valid;
    if (MTQ > 1 && ng > 1) n_valid_last = tiles[t + ng - 1].n_valid;
    const int n_keys = td.pos0 + 32 * (ng - 1) + n_valid_last;   // keys 0..n_keys-1 are visible to the group
    const int nkb = (n_keys + 31) >> 5;
    const int kb_lo = (int)(((long long)nkb * sp) / nsplit), kb_hi = (int)(((long long)nkb * (sp + 1)) / nsplit);
    const size_t block_elems = (size_t)32 * h;                // one block of 32 positions, all heads
    const float scale = 1.0f / sqrtf((float)D);

    bf16x8 qv[MTQ][DK];
    f32x16 o[MTQ][DB];
    float m_run[MTQ], l_run[MTQ];                             // l_run: this half-wave's share of the sum
#pragma unroll
    for (int b = 0; b < MTQ; ++b) {
        // The queries are asked for before the descriptor is there, at the rows the segment has when no
        // rows are packed (segment t = row tile t: valid memory in any case), and asked for again only if
        // the segment starts elsewhere -- so the usual case does not wait for two loads in a row.
        const uint16_t* qr0 = q + ((size_t)(t + b) * 32 + col) * h + hd * D + g * 8;
#pragma unroll
        for (int i = 0; i < DK; ++i) qv[b][i] = *reinterpret_cast<const bf16x8*>(qr0 + i * 16);
        const TileDesc tb = b == 0 ? td : tiles[t + min(b, ng - 1)];
        if (tb.prow0 != (t + b) * 32) {
            const uint16_t* qr = q + ((size_t)tb.prow0 + min(col, tb.n_valid - 1)) * h + hd * D + g * 8;
#pragma unroll
            for (int i = 0; i < DK; ++i) qv[b][i] = *reinterpret_cast<const bf16x8*>(qr + i * 16);
        }
#pragma unroll
        for (int d = 0; d < DB; ++d)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[b][d][i] = 0.f;
        m_run[b] = -INFINITY; l_run[b] = 0.f;
    }

    // block table entries of the split's first 64 key blocks, one per lane, fetched once (next to the
    // queries): the loads of a key block then do not wait for a table lookup of their own
    int entry = 0;
    if (kb_lo < kb_hi) entry = kvp.table[(size_t)td.seq * kvp.stride + min(kb_lo + lane, kb_hi - 1)];
    auto block_base = [&](int kb) -> size_t {
        const int rel = kb - kb_lo;
        const int id = rel < 64 ? __builtin_amdgcn_readlane(entry, rel) : kvp.table[(size_t)td.seq * kvp.stride + kb];
        return (size_t)id * block_elems;
    };
    bf16x8 kA[DK], vA[2 * DB], kB[DK], vB[2 * DB];
    auto load = [&](bf16x8(&kv)[DK], bf16x8(&vv)[2 * DB], int kb) {
        const size_t base = block_base(kb);
        const uint16_t* kr = kc + base + k_cache_off(col, hd, g * 8, H, D);
#pragma unroll
        for (int i = 0; i < DK; ++i) kv[i] = *reinterpret_cast<const bf16x8*>(kr + i * 512);
        const uint16_t* vr = vc + base + (size_t)hd * D * 32 + (size_t)col * 32 + g * 8;
#pragma unroll
        for (int d = 0; d < DB; ++d) {
            vv[2 * d] = *reinterpret_cast<const bf16x8*>(vr + (size_t)d * 32 * 32);
            vv[2 * d + 1] = *reinterpret_cast<const bf16x8*>(vr + (size_t)d * 32 * 32 + 16);
        }
    };
    auto block = [&](bf16x8(&kv)[DK], bf16x8(&vv)[2 * DB], int kb) {
#pragma unroll
        for (int b = 0; b < MTQ; ++b) {
            if (b >= ng) continue;
            const int qpos = td.pos0 + 32 * b + col;          // position of this lane's query
            if (kb * 32 > td.pos0 + 32 * b + 31) continue;    // the whole block lies after the tile
            f32x16 sacc;
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
            for (int i = 0; i < DK; ++i) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kv[i], qv[b][i], sacc, 0, 0, 0);
            bf16x8 p0, p1;
            const float alpha = att_block_probs(sacc, kb, g, qpos, kb * 32 + 31 <= td.pos0 + 32 * b, scale, m_run[b],
                                                l_run[b], p0, p1);
            const bool rescale = __builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0;   // some lane moved its reference
#pragma unroll
            for (int d = 0; d < DB; ++d) {
                if (rescale) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[b][d][i] *= alpha;
                }
                o[b][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vv[2 * d], p0, o[b][d], 0, 0, 0);
                o[b][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vv[2 * d + 1], p1, o[b][d], 0, 0, 0);
            }
        }
    };
    // the wave's key blocks kb_lo + wave, + ATT_WAVES, ...: the next block's K and V are in flight
    // while the current one is used (loads are issued unconditionally, clamped to the last block)
    {
        const int last = max(kb_hi - 1, 0);
        int kb = kb_lo + wave;
        if (kb < kb_hi) {
            load(kA, vA, kb);
            for (; kb < kb_hi; kb += 2 * ATT_WAVES) {
                load(kB, vB, min(kb + ATT_WAVES, last));
                block(kA, vA, kb);
                load(kA, vA, min(kb + 2 * ATT_WAVES, last));
                if (kb + ATT_WAVES < kb_hi) block(kB, vB, kb + ATT_WAVES);
            }
        }
    }
    // merge the waves, one row tile at a time: common max, rescaled sums
#pragma unroll
    for (int b = 0; b < MTQ; ++b) {
        if (b >= ng) continue;                                // uniform over the workgroup
        if (b > 0) __syncthreads();
        float lr = l_run[b] + __shfl_xor(l_run[b], 32);
        if (g == 0) { sm[wave][0][col] = m_run[b]; sm[wave][1][col] = lr; }
        __syncthreads();
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < ATT_WAVES; ++w) M = fmaxf(M, sm[w][0][col]);
        float Muse = (M == -INFINITY) ? 0.f : M;
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < ATT_WAVES; ++w) L += sm[w][1][col] * __expf(sm[w][0][col] - Muse);
        float mine = __expf(m_run[b] - Muse);
#pragma unroll
        for (int d = 0; d < DB; ++d)
#pragma unroll
            for (int i = 0; i < 16; ++i) so[wave][d * 16 + i][lane] = o[b][d][i] * mine;
        __syncthreads();
        // wave w finishes the register quads with quad % ATT_WAVES == w; register (d, i) of lane
        // (col, g) is dim 32d + 8*(i/4) + 4g + i%4 of query `col`
        const TileDesc tb = b == 0 ? td : tiles[t + b];
        const int row = tb.prow0 + col;
        const bool own = col < tb.n_valid;                    // rows beyond belong to other segments or to nobody
        // split partials: [m[32], l[32], O in accumulator order [quad][i][lane]] (a wave writes 256
        // contiguous bytes), written through to memory when another workgroup will merge them
        float* rec = ws + (((size_t)(t + b) * H + hd) * nsplit + sp) * att_rec_floats(D);
        for (int quad = wave; quad < DB * 4; quad += ATT_WAVES) {
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float acc = 0.f;
#pragma unroll
                for (int w = 0; w < ATT_WAVES; ++w) acc += so[w][quad * 4 + i][lane];
                v[i] = acc;
            }
            int d = quad >> 2, qd = quad & 3;
            int dim = 32 * d + 8 * qd + 4 * g;
            if (nsplit == 1) {
                float inv = L > 0.f ? 1.0f / L : 0.f;
                ushort4 pk;
                pk.x = f32_to_bf16(v[0] * inv); pk.y = f32_to_bf16(v[1] * inv);
                pk.z = f32_to_bf16(v[2] * inv); pk.w = f32_to_bf16(v[3] * inv);
                if (own) *reinterpret_cast<ushort4*>(out + packed_off(row, hd * D + dim, h)) = pk;
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    __hip_atomic_store(rec + 64 + (size_t)(quad * 4 + i) * 64 + lane, v[i], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_SYSTEM);
            }
        }
        if (nsplit > 1 && wave == 0 && g == 0) {
            __hip_atomic_store(rec + col, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            __hip_atomic_store(rec + 32 + col, L, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
    if (nsplit == 1) return;
    // The last split of this (tile, head) to arrive merges all of them.  No device-scope fence:
    // partials are written and read with system-scope accesses, every wave waits for its stores to
    // be acknowledged before the workgroup draws its ticket (a system-scope atomic).
    __shared__ uint32_t ticket;
    uint32_t* tk = tickets + (size_t)t * H + hd;
    if (draw_ticket(tk, &ticket) != (uint32_t)nsplit - 1) return;
    const float* base = ws + ((size_t)t * H + hd) * nsplit * att_rec_floats(D);
    // Thread (wave, lane) merges accumulator quads wave, wave + ATT_WAVES, ... of query column
    // `col`, two quads per round: the loads of a round are all issued before its first use, and
    // the splits' maxima and sums, which depend on the column only, come with the first round.
    constexpr int QPW = DB * 4 / ATT_WAVES;
    static_assert(DB * 4 % ATT_WAVES == 0, "quads must divide over the waves");
    float ms[ATT_MAX_SPLIT], ls[ATT_MAX_SPLIT], w[ATT_MAX_SPLIT], inv = 0.f;
#pragma unroll
    for (int k0 = 0; k0 < QPW; k0 += 2) {
        float v[2][ATT_MAX_SPLIT][4];
#pragma unroll
        for (int s = 0; s < ATT_MAX_SPLIT; ++s) {
            const float* r = base + (size_t)min(s, nsplit - 1) * att_rec_floats(D);
            if (k0 == 0) {
                ms[s] = __hip_atomic_load(r + col, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                ls[s] = __hip_atomic_load(r + 32 + col, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            }
#pragma unroll
            for (int k = 0; k < 2; ++k)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (k0 + k < QPW)
                        v[k][s][i] = __hip_atomic_load(r + 64 + (size_t)((wave + (k0 + k) * ATT_WAVES) * 4 + i) * 64 + lane,
                                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        if (k0 == 0) {
            float Mx = -INFINITY;
#pragma unroll
            for (int s = 0; s < ATT_MAX_SPLIT; ++s)
                if (s < nsplit) Mx = fmaxf(Mx, ms[s]);
            const float Muse = (Mx == -INFINITY) ? 0.f : Mx;
            float Ls = 0.f;
#pragma unroll
            for (int s = 0; s < ATT_MAX_SPLIT; ++s) {
                w[s] = (s < nsplit) ? __expf(ms[s] - Muse) : 0.f;
                Ls += (s < nsplit) ? ls[s] * w[s] : 0.f;
            }
            inv = Ls > 0.f ? 1.0f / Ls : 0.f;
        }
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            if (k0 + k >= QPW) continue;
            float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < ATT_MAX_SPLIT; ++s)
                if (s < nsplit) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[i] += v[k][s][i] * w[s];
                }
            ushort4 pk;
            pk.x = f32_to_bf16(acc[0] * inv); pk.y = f32_to_bf16(acc[1] * inv);
            pk.z = f32_to_bf16(acc[2] * inv); pk.w = f32_to_bf16(acc[3] * inv);
            const int quad = wave + (k0 + k) * ATT_WAVES;
            const int dim = 32 * (quad >> 2) + 8 * (quad & 3) + 4 * g;
            if (col < td.n_valid) *reinterpret_cast<ushort4*>(out + packed_off(td.prow0 + col, hd * D + dim, h)) = pk;
        }
        __builtin_amdgcn_sched_barrier(0);      // keep the next round's loads behind this round
    }
    if (threadIdx.x == 0) __hip_atomic_store(tk, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// Several row tiles per sequence (wide windows, prefill): one workgroup per (head, group of up to
// ATT_GROUP consecutive tiles, KV split).  Every K / V block of the split is fetched once per
// workgroup and staged in LDS in MFMA operand order (double-buffered; the next block's global
// loads are in flight while the current block is used); wave w serves row tile w of the group
// against the staged block, so no cross-wave merge is needed.
template <int D>
__global__ __launch_bounds__(ATT_GROUP * 64) void attn_group_k(const uint16_t* __restrict__ q,
                                                                const uint16_t* __restrict__ kc,
                                                                const uint16_t* __restrict__ vc, uint16_t* __restrict__ out,
                                                                int H, KvPages kvp, int nsplit, float* __restrict__ ws,
                                                                const TileDesc* tiles, const int32_t* n_tiles) {
    constexpr int DK = D / 16, DB = D / 32;
    constexpr int SLOTS = (DK + 2 * DB) * 64;               // 16-byte slots of one staged K + V block
    constexpr int PER = (SLOTS + ATT_GROUP * 64 - 1) / (ATT_GROUP * 64);
    __shared__ bf16x8 stage[2][SLOTS];
    // grid (heads, groups, splits): one workgroup per attention group, found through the leader list
    const int hd = blockIdx.x, sp = blockIdx.z;
    // (groups in reverse order: under the causal mask the later groups of a sequence see the most keys, and
    // the workgroups that take longest should start first)
    const int n_groups = n_tiles[1];
    if ((int)blockIdx.y >= n_groups) return;
    const int t = n_tiles[TILE_LEADERS + n_groups - 1 - (int)blockIdx.y];
    const TileDesc td = tiles[t];
    const int ng = min(td.group, ATT_GROUP);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int h = H * D;
    const int n_keys = td.pos0 + 32 * (ng - 1) + tiles[t + ng - 1].n_valid;
    const int nkb = (n_keys + 31) >> 5;
    const int kb_lo = (int)(((long long)nkb * sp) / nsplit), kb_hi = (int)(((long long)nkb * (sp + 1)) / nsplit);
    const float scale = 1.0f / sqrtf((float)D);
    const bool active = wave < ng;
    const int tq = t + (active ? wave : 0);                   // this wave's segment (they follow each other, also physically)
    const int pos0 = td.pos0 + 32 * (active ? wave : 0);
    const int qpos = pos0 + col;
    const int prow = td.prow0 + 32 * (active ? wave : 0);     // its first physical row
    const int nv = (active && wave == ng - 1) ? tiles[t + ng - 1].n_valid : 32;   // rows of the segment

    bf16x8 qv[DK];
    {
        const uint16_t* qr = q + ((size_t)prow + min(col, nv - 1)) * h + hd * D + g * 8;
#pragma unroll
        for (int i = 0; i < DK; ++i) qv[i] = *reinterpret_cast<const bf16x8*>(qr + i * 16);
    }
    f32x16 o[DB];
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[d][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // slot s < DK*64: K operand (k step s/64, lane s%64); then V operand (j = (s - DK*64)/64).
    // A slot's address is the key block's place in the pool (block table) plus its offset in the block.
    static_assert(SLOTS % (ATT_GROUP * 64) == 0, "every thread stages the same number of slots");
    const size_t kb_stride = (size_t)32 * H * D;
    const uint16_t* fbase[PER];
#pragma unroll
    for (int p = 0; p < PER; ++p) {
        const int s = threadIdx.x + p * ATT_GROUP * 64;
        const int ln = s & 63, c = ln & 31, gg = ln >> 5, i = s >> 6, j = i - DK;
        const uint16_t* sk = kc + k_cache_off(c, hd, gg * 8 + (i < DK ? i : 0) * 16, H, D);
        const uint16_t* sv = vc + (size_t)hd * D * 32 + (size_t)c * 32 + gg * 8 + (size_t)(j >> 1) * 32 * 32 + (j & 1) * 16;
        fbase[p] = i < DK ? sk : sv;
    }
    int entry = 0;                                            // block table entries of the first 64 key blocks, one per lane
    if (kb_lo < kb_hi) entry = kvp.table[(size_t)td.seq * kvp.stride + min(kb_lo + lane, kb_hi - 1)];
    bf16x8 fetch0[PER], fetch1[PER];
    auto load = [&](bf16x8(&fetch)[PER], int kb) {
        const int rel = kb - kb_lo;
        const int id = rel < 64 ? __builtin_amdgcn_readlane(entry, rel) : kvp.table[(size_t)td.seq * kvp.stride + kb];
        const size_t base = (size_t)id * kb_stride;
#pragma unroll
        for (int p = 0; p < PER; ++p) fetch[p] = *reinterpret_cast<const bf16x8*>(fbase[p] + base);
    };
    auto put = [&](bf16x8(&fetch)[PER], int buf) {
#pragma unroll
        for (int p = 0; p < PER; ++p) stage[buf][threadIdx.x + p * ATT_GROUP * 64] = fetch[p];
    };
    auto block = [&](int cur, int kb) {
        // nothing to do past the split's end, or when the whole block lies after the tile
        if (!(active && kb < kb_hi && kb * 32 <= pos0 + 31)) return;
        f32x16 sacc;
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
        for (int i = 0; i < DK; ++i)
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(stage[cur][i * 64 + lane], qv[i], sacc, 0, 0, 0);
        bf16x8 p0, p1;
        const float alpha = att_block_probs(sacc, kb, g, qpos, kb * 32 + 31 <= pos0, scale, m_run, l_run, p0, p1);
        const bool rescale = __builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0;   // some lane moved its reference
#pragma unroll
        for (int d = 0; d < DB; ++d) {
            if (rescale) {
#pragma unroll
                for (int i = 0; i < 16; ++i) o[d][i] *= alpha;
            }
            o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(stage[cur][(DK + 2 * d) * 64 + lane], p0, o[d], 0, 0, 0);
            o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(stage[cur][(DK + 2 * d + 1) * 64 + lane], p1, o[d], 0, 0, 0);
        }
    };
    // Block j of the split (kb = kb_lo + j) is fetched into register set j % 2 two blocks ahead,
    // staged into LDS buffer j % 2 one block ahead (that buffer was last read two blocks ago, before
    // the previous barrier) and used after the barrier that follows.  Every iteration issues the
    // same loads and stores (block indices clamped to the split), so the wait before the staging
    // store covers the older fetch only and the newer one stays in flight.
    auto one = [&](bf16x8(&mine)[PER], bf16x8(&next)[PER], int cur, int kb) {
        load(mine, min(kb + 2, kb_hi - 1));                   // `mine` held block kb, already staged
        block(cur, kb);
        put(next, cur ^ 1);
        __syncthreads();
    };
    if (kb_lo < kb_hi) {
        load(fetch0, kb_lo);
        load(fetch1, min(kb_lo + 1, kb_hi - 1));
        put(fetch0, 0);
        __syncthreads();
        for (int kb = kb_lo; kb < kb_hi; kb += 2) {
            one(fetch0, fetch1, 0, kb);
            one(fetch1, fetch0, 1, kb + 1);
        }
    }
    if (!active) return;
    const float L = l_run + __shfl_xor(l_run, 32);
    const int row = prow + col;
    float* rec = ws + (((size_t)tq * H + hd) * nsplit + sp) * att_rec_floats(D);
    const float inv = L > 0.f ? 1.0f / L : 0.f;
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            const int dim = 32 * d + 8 * qd + 4 * g;
            const float v0 = o[d][qd * 4], v1 = o[d][qd * 4 + 1], v2 = o[d][qd * 4 + 2], v3 = o[d][qd * 4 + 3];
            if (nsplit == 1) {
                ushort4 pk;
                pk.x = f32_to_bf16(v0 * inv); pk.y = f32_to_bf16(v1 * inv);
                pk.z = f32_to_bf16(v2 * inv); pk.w = f32_to_bf16(v3 * inv);
                if (col < nv) *reinterpret_cast<ushort4*>(out + packed_off(row, hd * D + dim, h)) = pk;
            } else {
                *reinterpret_cast<float4*>(rec + 64 + (size_t)col * D + dim) = make_float4(v0, v1, v2, v3);
            }
        }
    if (nsplit > 1 && g == 0) {
        rec[col] = m_run;
        rec[32 + col] = L;
    }
}

// Combine the KV-split partials of a (tile, head): one thread per (query, 4 dims); all loads of
// the thread are issued before the first use.
template <int D>
__global__ __launch_bounds__(256) void attn_merge_k(const float* __restrict__ ws, uint16_t* __restrict__ out, int H,
                                                     int nsplit, const TileDesc* tiles, const int32_t* n_tiles) {
    const int hd = blockIdx.x, t = blockIdx.y;                // t: segment
    if (t >= n_tiles[2]) return;
    const TileDesc td = tiles[t];
    const int idx = blockIdx.z * blockDim.x + threadIdx.x;
    if (idx >= 32 * (D / 4)) return;
    const float* base = ws + ((size_t)t * H + hd) * nsplit * att_rec_floats(D);
    const int col = idx / (D / 4), dim = (idx % (D / 4)) * 4;
    float m[ATT_MAX_SPLIT], l[ATT_MAX_SPLIT];
    float4 v[ATT_MAX_SPLIT];
#pragma unroll
    for (int s = 0; s < ATT_MAX_SPLIT; ++s) {
        if (s < nsplit) {
            const float* rec = base + s * att_rec_floats(D);
            m[s] = rec[col];
            l[s] = rec[32 + col];
            v[s] = *reinterpret_cast<const float4*>(rec + 64 + (size_t)col * D + dim);
        }
    }
    float M = -INFINITY;
#pragma unroll
    for (int s = 0; s < ATT_MAX_SPLIT; ++s)
        if (s < nsplit) M = fmaxf(M, m[s]);
    const float Muse = (M == -INFINITY) ? 0.f : M;
    float L = 0.f;
    float4 acc = make_float4(0, 0, 0, 0);
#pragma unroll
    for (int s = 0; s < ATT_MAX_SPLIT; ++s) {
        if (s < nsplit) {
            const float w = __expf(m[s] - Muse);
            L += l[s] * w;
            acc.x += v[s].x * w; acc.y += v[s].y * w; acc.z += v[s].z * w; acc.w += v[s].w * w;
        }
    }
    const float inv = L > 0.f ? 1.0f / L : 0.f;
    ushort4 pk;
    pk.x = f32_to_bf16(acc.x * inv); pk.y = f32_to_bf16(acc.y * inv);
    pk.z = f32_to_bf16(acc.z * inv); pk.w = f32_to_bf16(acc.w * inv);
    if (col < td.n_valid) *reinterpret_cast<ushort4*>(out + packed_off(td.prow0 + col, hd * D + dim, H * D)) = pk;
}

// f32 path: one workgroup per (row, head); scores kept in LDS.
constexpr int ATT_F32_MAXKEYS = 8192;
__global__ __launch_bounds__(256) void attn_f32_k(const float* __restrict__ q, const float* __restrict__ kc,
                                                    const float* __restrict__ vc, float* __restrict__ out, int H, int d,
                                                    KvPages kvp, const TileDesc* tiles, const int32_t* n_tiles) {
    __shared__ float sc[ATT_F32_MAXKEYS];
    __shared__ float red[8];
    int r = blockIdx.x, hd = blockIdx.y, j = 0;               // (the row's own descriptor)
    if ((r >> 5) >= *n_tiles) return;
    TileDesc td = tiles[r];
    int h = H * d;
    float* orow = out + (size_t)r * h + hd * d;
    if (j >= td.n_valid) {
        for (int c = threadIdx.x; c < d; c += blockDim.x) orow[c] = 0.f;
        return;
    }
    int nk = td.pos0 + j + 1;
    const size_t block_elems = (size_t)32 * h;
    const float* qr = q + (size_t)r * h + hd * d;
    float scale = 1.0f / sqrtf((float)d);
    float mx = -INFINITY;
    for (int k = threadIdx.x; k < nk; k += blockDim.x) {
        const float* kr = kc + kv_block_base(kvp, td.seq, k >> 5, block_elems) + (size_t)(k & 31) * h + hd * d;
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
        for (int k = 0; k < nk; ++k)
            acc = fmaf(sc[k], vc[kv_block_base(kvp, td.seq, k >> 5, block_elems) + (size_t)(k & 31) * h + hd * d + c], acc);
        orow[c] = acc / sum;
    }
}

void launch_attention(const void* q, const void* kc, const void* vc, void* out, int dtype, int H, int d,
                      KvPages kv, int nsplit, bool grouped, float* ws, uint32_t* tickets,
                      const TileDesc* tiles, int rows_pad, const int32_t* n_tiles, int max_tiles, hipStream_t st,
                      int max_groups) {
    const TileDesc* segs = tiles + rows_pad;
    if (dtype == 0) {
        hipLaunchKernelGGL(attn_f32_k, dim3(max_tiles * 32, H), dim3(256), 0, st, (const float*)q, (const float*)kc,
                           (const float*)vc, (float*)out, H, d, kv, tiles, n_tiles);
        return;
    }
    if (nsplit > ATT_MAX_SPLIT) nsplit = ATT_MAX_SPLIT;
    if (nsplit < 1) nsplit = 1;
    if (max_groups <= 0 || max_groups > max_tiles) max_groups = max_tiles;
    dim3 grid(H, grouped ? max_groups : max_tiles, nsplit);
#define RDLM_ATT(D_)                                                                                              \
    if (d == D_) {                                                                                                \
        if (!grouped) {         /* merges its KV splits itself */                                                 \
            hipLaunchKernelGGL((attn_bf16_k<D_, 1>), grid, dim3(ATT_WAVES * 64), 0, st, (const uint16_t*)q,       \
                               (const uint16_t*)kc, (const uint16_t*)vc, (uint16_t*)out, H, kv,                   \
                               nsplit, ws, tickets, segs, n_tiles);                                               \
            return;                                                                                               \
        }                                                                                                         \
        else                                                                                                      \
            hipLaunchKernelGGL(attn_group_k<D_>, grid, dim3(ATT_GROUP * 64), 0, st, (const uint16_t*)q,           \
                               (const uint16_t*)kc, (const uint16_t*)vc, (uint16_t*)out, H, kv,                   \
                               nsplit, ws, segs, n_tiles);                                                        \
        if (nsplit > 1)                                                                                           \
            hipLaunchKernelGGL(attn_merge_k<D_>, dim3(H, max_tiles, (32 * (D_ / 4) + 255) / 256), dim3(256), 0,   \
                               st, ws, (uint16_t*)out, H, nsplit, segs, n_tiles);                                 \
        return;                                                                                                   \
    }
    RDLM_ATT(32) RDLM_ATT(64) RDLM_ATT(96) RDLM_ATT(128)
#undef RDLM_ATT
}

}  // namespace rdlm
