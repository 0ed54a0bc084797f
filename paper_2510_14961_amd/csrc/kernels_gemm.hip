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
#include "gemm_common.h"

namespace rdlm {

// Fold of the split-K partial sums by the last workgroup of a feature group to arrive (see
// GemmEpilogue::fold_counter).  No device-scope fence: the partial sums are written and read with
// system-scope accesses (write-through stores, cache-bypassing loads), every wave waits for its
// stores to be acknowledged before the workgroup takes its ticket, and the ticket is a
// system-scope atomic -- so whoever draws the last ticket finds all partial sums in memory.
// Which workgroup that is does not matter: it adds the S partial sums in split order.
template <int NB, int THREADS>
__device__ __forceinline__ void gemm_fold_tail(const GemmArgs& A, int grp, int t0) {
    static_assert(NB == 1 || NB == 2 || NB == 4, "a row's columns of the group sit in 8, 16 or 32 adjacent lanes");
    __shared__ uint32_t ticket;
    if (draw_ticket(A.epi.fold_counter + grp, &ticket) != (uint32_t)A.ksplit - 1) return;
    // one thread per (register quad u of the group, lane): 4 consecutive columns of one row, read
    // back in the order they were written (coalesced)
    constexpr int UNITS = NB * 4;
    __shared__ float unit_ss[UNITS][64];
    const int N = A.N;
    for (int slot = threadIdx.x; slot < UNITS * 64; slot += THREADS) {
        const int u = slot >> 6, ln = slot & 63;
        const int col = grp * NB * 32 + (u >> 2) * 32 + (u & 3) * 8 + (ln >> 5) * 4;
        const size_t row = (size_t)t0 * 32 + (ln & 31);
        float ss = 0.f;
        if (col < N) {
            const size_t off = row * N + col;
            float4 v = A.epi.fold_xin ? *reinterpret_cast<const float4*>(A.epi.fold_xin + off) : make_float4(0, 0, 0, 0);
            // all loads of a batch of up to 4 splits are issued before the first add
            for (int s0 = 0; s0 < A.ksplit; s0 += 4) {
                float p[4][4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float* pp = A.out + (((size_t)grp * A.ksplit + min(s0 + j, A.ksplit - 1)) * (NB * 16) + u * 4) * 64 + ln;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        p[j][i] = __hip_atomic_load(pp + i * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (s0 + j < A.ksplit) { v.x += p[j][0]; v.y += p[j][1]; v.z += p[j][2]; v.w += p[j][3]; }
                }
            }
            ss = v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
            *reinterpret_cast<float4*>(A.epi.fold_xout + off) = v;
            const float4 g = *reinterpret_cast<const float4*>(A.epi.fold_gain + col);
            ushort4 pk;
            pk.x = f32_to_bf16(v.x * g.x); pk.y = f32_to_bf16(v.y * g.y);
            pk.z = f32_to_bf16(v.z * g.z); pk.w = f32_to_bf16(v.w * g.w);
            *reinterpret_cast<ushort4*>(reinterpret_cast<uint16_t*>(A.epi.fold_xg) + packed_off((int)row, col, N)) = pk;
        }
        unit_ss[u][ln] = ss;
    }
    __syncthreads();
    if (threadIdx.x < 32) {                        // the group's share of each row's sum of squares
        float ss = 0.f;
#pragma unroll
        for (int u = 0; u < UNITS; ++u) ss += unit_ss[u][threadIdx.x] + unit_ss[u][threadIdx.x + 32];
        __hip_atomic_store(A.epi.fold_ssq + (size_t)grp * A.epi.ssq_stride + (size_t)t0 * 32 + threadIdx.x, ss,
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    if (threadIdx.x == 0) __hip_atomic_store(A.epi.fold_counter + grp, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    // second level, same protocol: the last group to finish adds the groups' shares of every row's
    // sum of squares (in group order) and leaves one value per row for the consumer
    uint32_t* total = A.epi.fold_counter + SSQ_MAX_CHUNKS;
    if (draw_ticket(total, &ticket) != (uint32_t)A.n_groups - 1) return;
    __shared__ float part_ss[THREADS / 32][32];
    {
        constexpr int PARTS = THREADS / 32;
        const int rt = threadIdx.x & 31, pt = threadIdx.x >> 5;
        const size_t row = (size_t)t0 * 32 + rt;
        float acc = 0.f;
        for (int c0 = pt; c0 < A.n_groups; c0 += 8 * PARTS) {           // batches of 8 loads in flight
            float v8[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                v8[j] = __hip_atomic_load(A.epi.fold_ssq + (size_t)min(c0 + j * PARTS, A.n_groups - 1) * A.epi.ssq_stride + row,
                                          __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (c0 + j * PARTS < A.n_groups) acc += v8[j];
        }
        part_ss[pt][rt] = acc;
        __syncthreads();
        if (pt == 0) {
            float tot = 0.f;
#pragma unroll
            for (int q = 0; q < PARTS; ++q) tot += part_ss[q][rt];
            A.epi.fold_ssq[(size_t)SSQ_MAX_CHUNKS * A.epi.ssq_stride + row] = tot;
        }
    }
    if (threadIdx.x == 0) __hip_atomic_store(total, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

template <int MT, int NB, int WAVES, int U, int EPI>
__global__ __launch_bounds__(WAVES * 64) void gemm_bf16_k(GEMM_KERNEL_PARAMS) {
    GEMM_KERNEL_ARGS_STRUCT;
    // cross-wave sums: [WAVES][NB*MT*16][64] for one row tile; with several row tiles the waves
    // finish one row tile at a time through [WAVES][NB*16][64]
    extern __shared__ float red[];
    constexpr bool PER_TILE = WAVES > 1 && MT > 1;
    constexpr int CW = (EPI == EPI_ARGMAX && WAVES > 1) ? WAVES : 1;
    constexpr int CM = PER_TILE ? 1 : MT;
    __shared__ float cand_v[CW][CM][32];
    __shared__ int cand_i[CW][CM][32];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int bid = blockIdx.x;
    const int mc = bid % A.m_chunks; bid /= A.m_chunks;   // row chunk fastest: neighbours share weights
    const int ks = bid % A.ksplit;
    const int grp = bid / A.ksplit;
    const int t0 = mc * MT;
    // The tile count lives in device memory.  A launch over a single row tile does not wait for
    // it before its first weights are on their way: tile 0's operand is valid memory whatever
    // the count is, and the count is looked at when the contraction is done.
    const bool late_count = A.max_tiles == 1;
    int n_tiles = 1;
    if (!late_count) {
        n_tiles = *A.n_tiles;
        if (t0 >= n_tiles) return;
    }
    const int nblk = A.N >> 5, K16 = A.K16;
    // K range of this wave: K16 tiles split evenly over ksplit * WAVES slices
    const int slices = A.ksplit * WAVES, sl = ks * WAVES + wave;
    const int kbeg = (int)(((long long)K16 * sl) / slices), kend = (int)(((long long)K16 * (sl + 1)) / slices);
    float sc[MT];
    gemm_row_scales<MT>(A, t0, n_tiles, sc);        // late_count: tile 0, as n_tiles = 1 stands in
    // RoPE / cache epilogue over one row tile: the lane's row descriptor and, once it is there, the cache block
    // of the row's position are asked for up front, so the epilogue's stores do not wait for two dependent
    // loads.  The descriptor is valid memory for every row of tile t0; when the tile count is only looked at
    // after the K loop it may be a stale one, so the table index is clamped to the table (the epilogue, which
    // runs only for tiles of this step, then finds the entry of its own row).
    constexpr bool PRE = (EPI == EPI_ROPE_KV && MT == 1);
    TileDesc pre_td[1];
    int pre_kvblk[1] = {0};
    if constexpr (PRE) pre_td[0] = A.epi.tiles[(size_t)t0 * 32 + (lane & 31)];
    auto pre_lookup = [&]() {
        if constexpr (PRE)
            pre_kvblk[0] = A.epi.kv.table[(size_t)min(max(pre_td[0].seq, 0), A.epi.kv.slots - 1) * A.epi.kv.stride +
                                          min(max(pre_td[0].pos0 >> 5, 0), A.epi.kv.stride - 1)];
    };

    f32x16 acc[NB][MT];
#pragma unroll
    for (int a = 0; a < NB; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    int blk[NB];
    const bf16x8* wbase[NB];
    const bf16x8* xbase[MT];
#pragma unroll
    for (int a = 0; a < NB; ++a) {
        blk[a] = grp * NB + a;
        int nb = min(blk[a], nblk - 1);             // a ragged last group re-reads a valid block
        wbase[a] = A.wp + ((size_t)nb * K16) * 64 + lane;
    }
#pragma unroll
    for (int b = 0; b < MT; ++b) {
        int t = min(t0 + b, n_tiles - 1);
        xbase[b] = A.xp + ((size_t)t * K16) * 64 + lane;
    }

    bf16x8 wa[U][NB], xa[U][MT], wb[U][NB], xb[U][MT];
    auto load = [&](bf16x8(&wv)[U][NB], bf16x8(&xv)[U][MT], int kt) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int a = 0; a < NB; ++a) wv[u][a] = __builtin_nontemporal_load(wbase[a] + (size_t)(kt + u) * 64);
#pragma unroll
            for (int b = 0; b < MT; ++b) xv[u][b] = xbase[b][(size_t)(kt + u) * 64];
        }
        __builtin_amdgcn_sched_barrier(0);          // all loads of the batch are issued before any MFMA
    };
    auto compute = [&](bf16x8(&wv)[U][NB], bf16x8(&xv)[U][MT]) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int a = 0; a < NB; ++a)
#pragma unroll
                for (int b = 0; b < MT; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv[u][a], xv[u][b], acc[a][b], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    };
    int kt = kbeg;
    int batches = (kend - kbeg) / U;
    if (batches > 0) {                              // double-buffered: one batch in flight while one is consumed
        load(wa, xa, kt); kt += U;
        pre_lookup();
        int rem = batches - 1;
        while (rem >= 2) {
            load(wb, xb, kt); kt += U;
            compute(wa, xa);
            load(wa, xa, kt); kt += U;
            compute(wb, xb);
            rem -= 2;
        }
        if (rem == 1) {
            load(wb, xb, kt); kt += U;
            compute(wa, xa);
            compute(wb, xb);
        } else {
            compute(wa, xa);
        }
    }
    if (batches <= 0) pre_lookup();
    for (; kt < kend; ++kt) {
#pragma unroll
        for (int a = 0; a < NB; ++a) {
            bf16x8 w = __builtin_nontemporal_load(wbase[a] + (size_t)kt * 64);
#pragma unroll
            for (int b = 0; b < MT; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w, xbase[b][(size_t)kt * 64], acc[a][b], 0, 0, 0);
        }
    }

    if (late_count) {
        n_tiles = *A.n_tiles;
        if (n_tiles <= 0) return;
    }

    // Cross-wave sum in a fixed order: every wave deposits its accumulators; the finishing work is
    // dealt to the waves in units of one register quad (see gemm_epilogue).
    if constexpr (PER_TILE) {
        constexpr int REGS = NB * 16;
#pragma unroll
        for (int b = 0; b < MT; ++b) {
            if (b > 0) __syncthreads();            // the previous row tile's sums have been read
#pragma unroll
            for (int a = 0; a < NB; ++a)
#pragma unroll
                for (int i = 0; i < 16; ++i) red[((size_t)wave * REGS + a * 16 + i) * 64 + lane] = acc[a][b][i];
            __syncthreads();
            auto quad_sum = [&](int a, int, int q, float (&o)[4]) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float sum = 0.f;
#pragma unroll
                    for (int w = 0; w < WAVES; ++w) sum += red[((size_t)w * REGS + a * 16 + q * 4 + i) * 64 + lane];
                    o[i] = sum;
                }
            };
            const float sc1[1] = {sc[b]};
            gemm_epilogue<1, NB, WAVES, WAVES, EPI>(A, blk, t0 + b, n_tiles, ks, grp, sc1, quad_sum, cand_v, cand_i);
        }
    } else {
        constexpr int REGS = NB * MT * 16;
        if (WAVES > 1) {
#pragma unroll
            for (int a = 0; a < NB; ++a)
#pragma unroll
                for (int b = 0; b < MT; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        red[((size_t)wave * REGS + (a * MT + b) * 16 + i) * 64 + lane] = acc[a][b][i];
            __syncthreads();
        }
        auto quad_sum = [&](int a, int b, int q, float (&o)[4]) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = (a * MT + b) * 16 + q * 4 + i;
                if (WAVES > 1) {
                    float sum = 0.f;
#pragma unroll
                    for (int w = 0; w < WAVES; ++w) sum += red[((size_t)w * REGS + r) * 64 + lane];
                    o[i] = sum;
                } else {
                    o[i] = acc[a][b][q * 4 + i];
                }
            }
        };
        gemm_epilogue<MT, NB, WAVES, WAVES, EPI>(A, blk, t0, n_tiles, ks, grp, sc, quad_sum, cand_v, cand_i,
                                                 PRE ? pre_td : nullptr, PRE ? pre_kvblk : nullptr);
    }
    if constexpr (EPI == EPI_F32 && MT == 1 && (NB == 1 || NB == 2 || NB == 4))
        if (A.epi.fold_counter) gemm_fold_tail<NB, WAVES * 64>(A, grp, t0);
}

// Row-tile-sharing variant for steps with several row tiles (wide windows, ragged batches,
// prefill).  The waves of a workgroup own different feature blocks (NB each) over the same K range
// and the same MT row tiles; the activation tiles of a K step are staged once per workgroup in
// LDS (three stages, 1 KiB per tile, read back with conflict-free 16-byte reads), so the
// activation traffic per weight byte drops by the number of waves, and every wave streams its own
// weights straight into registers.  No cross-wave reduction: a wave finishes its own blocks.
// Workgroups of one (feature group, K split) that cover different row chunks get ids that land on
// the same XCD one after the other, so the weights they share are served by that XCD's L2.
template <int MT, int NB, int WAVES, int KU, int EPI>
__global__ __launch_bounds__(WAVES * 64) void gemm_bf16_rows_k(GEMM_KERNEL_PARAMS) {
    GEMM_KERNEL_ARGS_STRUCT;
    extern __shared__ float red[];                 // activation stages: [3][KU * MT][64] x 16 bytes
    bf16x8* xs = reinterpret_cast<bf16x8*>(red);
    constexpr int CW = EPI == EPI_ARGMAX ? WAVES : 1;
    __shared__ float cand_v[CW][MT][32];
    __shared__ int cand_i[CW][MT][32];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // id = xcd + 8 * (row chunk + m_chunks * j): (group, split) index gk = 8 j + xcd
    const int xcd = blockIdx.x & 7, rest = blockIdx.x >> 3;
    const int mc = rest % A.m_chunks, gk = (rest / A.m_chunks) * 8 + xcd;
    if (gk >= A.n_groups * A.ksplit) return;
    const int ks = gk % A.ksplit, grp = gk / A.ksplit;
    const int t0 = mc * MT;
    const bool late_count = A.max_tiles == 1;      // as in gemm_bf16_k: look at the count afterwards
    int n_tiles = 1;
    if (!late_count) {
        n_tiles = *A.n_tiles;
        if (t0 >= n_tiles) return;
    }
    const int nblk = A.N >> 5, K16 = A.K16;
    const int kbeg = (int)(((long long)K16 * ks) / A.ksplit), kend = (int)(((long long)K16 * (ks + 1)) / A.ksplit);
    float sc[MT];
    gemm_row_scales<MT>(A, t0, n_tiles, sc);

    f32x16 acc[NB][MT];
#pragma unroll
    for (int a = 0; a < NB; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    int blk[NB];
    const bf16x8* wbase[NB];
#pragma unroll
    for (int a = 0; a < NB; ++a) {
        blk[a] = (grp * WAVES + wave) * NB + a;
        wbase[a] = A.wp + ((size_t)min(blk[a], nblk - 1) * K16) * 64 + lane;
    }
    // staging: tile ti = u * MT + b of a K step; thread slot i covers tile wave + i * WAVES
    constexpr int XL = (KU * MT + WAVES - 1) / WAVES;
    const bf16x8* xsrc[XL];
#pragma unroll
    for (int i = 0; i < XL; ++i) {
        const int ti = wave + i * WAVES, u = ti / MT, b = ti - u * MT;
        const int t = min(t0 + b, n_tiles - 1);
        xsrc[i] = A.xp + ((size_t)t * K16 + u) * 64 + lane;
    }
    const bool stream_w = A.m_chunks == 1;          // weights used once: keep them out of the caches

    bf16x8 w0[KU][NB], w1[KU][NB], w2[KU][NB], xr[XL];
    uint32_t xok = 0;                               // bit i: staged tile i of the loaded step lies inside the K range
    // Every K step issues the same loads, stores and matrix instructions (k indices clamped to the
    // range; activation tiles beyond it are staged as zeros), so the loop body is one straight
    // path and the compiler can count the memory operations: activations first -- the staging
    // store then waits for them only, and the weight loads issued after them stay in flight (the
    // memory counter retires in issue order).
    static_assert((KU * MT) % WAVES == 0, "every wave stages the same number of tiles");
    auto load = [&](bf16x8(&wv)[KU][NB], int kt) {  // activations and weights of the K step at kt
        xok = 0;
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            const int u = (wave + i * WAVES) / MT;
            xr[i] = xsrc[i][(size_t)(min(kt + u, kend - 1) - u) * 64];
            xok |= (kt + u < kend ? 1u : 0u) << i;
        }
#pragma unroll
        for (int u = 0; u < KU; ++u) {
            const size_t k = (size_t)min(kt + u, kend - 1);
#pragma unroll
            for (int a = 0; a < NB; ++a)
                wv[u][a] = stream_w ? __builtin_nontemporal_load(wbase[a] + k * 64) : wbase[a][k * 64];
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    // the same loads for a K step that lies inside the range as a whole: no clamping, no masks
    auto load_in = [&](bf16x8(&wv)[KU][NB], int kt) {
        const size_t off = (size_t)kt * 64;
        xok = (1u << XL) - 1u;
#pragma unroll
        for (int i = 0; i < XL; ++i) xr[i] = xsrc[i][off];
#pragma unroll
        for (int u = 0; u < KU; ++u)
#pragma unroll
            for (int a = 0; a < NB; ++a)
                wv[u][a] = stream_w ? __builtin_nontemporal_load(wbase[a] + off + (size_t)u * 64) : wbase[a][off + (size_t)u * 64];
        __builtin_amdgcn_sched_barrier(0);
    };
    auto stage_in = [&](int buf) {
#pragma unroll
        for (int i = 0; i < XL; ++i) xs[((size_t)buf * KU * MT + wave + i * WAVES) * 64 + lane] = xr[i];
    };
    auto stage = [&](int buf) {
        const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < XL; ++i)
            xs[((size_t)buf * KU * MT + wave + i * WAVES) * 64 + lane] = ((xok >> i) & 1u) ? xr[i] : zero;
    };
    // The activation tiles of K tile u + 1 are read from LDS while the matrix instructions of
    // K tile u run (two register sets), so the wave does not sit out the LDS latency per tile.
    auto compute = [&](bf16x8(&wv)[KU][NB], int buf) {
        bf16x8 xv[2][MT];
#pragma unroll
        for (int b = 0; b < MT; ++b) xv[0][b] = xs[((size_t)buf * KU * MT + b) * 64 + lane];
#pragma unroll
        for (int u = 0; u < KU; ++u) {
            if (u + 1 < KU) {
#pragma unroll
                for (int b = 0; b < MT; ++b)
                    xv[(u + 1) & 1][b] = xs[((size_t)buf * KU * MT + (u + 1) * MT + b) * 64 + lane];
            }
#pragma unroll
            for (int b = 0; b < MT; ++b)
#pragma unroll
                for (int a = 0; a < NB; ++a)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv[u][a], xv[u & 1][b], acc[a][b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // K step s uses weight registers s % 3 and stage buffer s % 3.  Its loads are issued at the top
    // of step s - 2; its activation tiles go from registers to LDS at the top of step s - 1 (that
    // buffer was last read in step s - 3, which every wave has left two barriers ago) and are read
    // after the barrier that ends step s - 1.
    auto step = [&](bf16x8(&wcur)[KU][NB], bf16x8(&wnext)[KU][NB], int bcur, int kt) {
        stage(bcur == 2 ? 0 : bcur + 1);
        load(wnext, min(kt + 2 * KU, kend - 1));
        compute(wcur, bcur);
        __syncthreads();
    };
    // a step whose staged tiles (K step s + 1) and loads (K step s + 2) all lie inside the range
    auto step_in = [&](bf16x8(&wcur)[KU][NB], bf16x8(&wnext)[KU][NB], int bcur, int kt) {
        stage_in(bcur == 2 ? 0 : bcur + 1);
        load_in(wnext, kt + 2 * KU);
        compute(wcur, bcur);
        __syncthreads();
    };
    // The loop body is three steps (one turn of the register ring) without exits in between; the
    // one or two steps left over run after it.
    const int nsteps = (kend - kbeg + KU - 1) / KU;
    int kt = kbeg;
    if (nsteps > 0) {
        load(w0, kt);
        stage(0);
        load(w1, min(kt + KU, kend - 1));
        __syncthreads();
        // turns of the ring in which every step is an inside step: step s qualifies while K steps
        // s + 1 and s + 2 are whole, i.e. s + 3 <= (kend - kbeg) / KU
        int s3 = nsteps / 3;
        int in3 = min(s3, max(0, ((kend - kbeg) / KU - 2) / 3));
        s3 -= in3;
        for (; in3 > 0; --in3) {
            step_in(w0, w2, 0, kt); kt += KU;
            step_in(w1, w0, 1, kt); kt += KU;
            step_in(w2, w1, 2, kt); kt += KU;
        }
        for (; s3 > 0; --s3) {
            step(w0, w2, 0, kt); kt += KU;
            step(w1, w0, 1, kt); kt += KU;
            step(w2, w1, 2, kt); kt += KU;
        }
        const int rem = nsteps % 3;
        if (rem >= 1) {
            if (rem == 2) stage(1);
            compute(w0, 0);
            if (rem == 2) {
                __syncthreads();
                compute(w1, 1);
            }
        }
    }
    if (late_count) {
        n_tiles = *A.n_tiles;
        if (n_tiles <= 0) return;
    }
    auto quad_sum = [&](int a, int b, int q, float (&o)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = acc[a][b][q * 4 + i];
    };
    gemm_epilogue<MT, NB, WAVES, 1, EPI>(A, blk, t0, n_tiles, ks, grp, sc, quad_sum, cand_v, cand_i);
}

// one candidate (score, token) per (feature group, row) -> the row's token; lowest id wins ties
__global__ void argmax_final_k(const float* cand_val, const int32_t* cand_idx, int n_groups, size_t cand_stride,
                               int32_t* tok_out, const int32_t* n_tiles) {
    __shared__ float sv[256];
    __shared__ int si[256];
    const int r = blockIdx.x;
    if ((r >> 5) >= *n_tiles) return;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int gq = threadIdx.x; gq < n_groups; gq += blockDim.x) {
        float ov = cand_val[(size_t)gq * cand_stride + r];
        int oi = cand_idx[(size_t)gq * cand_stride + r];
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    sv[threadIdx.x] = bv; si[threadIdx.x] = bi;
    __syncthreads();
    for (int o = blockDim.x >> 1; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) {
            float ov = sv[threadIdx.x + o]; int oi = si[threadIdx.x + o];
            if (ov > sv[threadIdx.x] || (ov == sv[threadIdx.x] && oi < si[threadIdx.x])) {
                sv[threadIdx.x] = ov; si[threadIdx.x] = oi;
            }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) tok_out[r] = (si[0] == 0x7fffffff) ? 0 : si[0];
}

void launch_argmax_final(const float* cand_val, const int32_t* cand_idx, int n_groups, size_t cand_stride,
                         int32_t* tok_out, const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    hipLaunchKernelGGL(argmax_final_k, dim3(max_tiles * 32), dim3(256), 0, st, cand_val, cand_idx, n_groups,
                       cand_stride, tok_out, n_tiles);
}

template <int MT, int NB, int WAVES, int U, int EPI>
static bool launch_cfg(const void* xp, const void* wp, float* out, int N, int K, size_t part_stride, int ksplit,
                       const GemmEpilogue& epi, const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    const int nblk = N / 32;
    const int groups = (nblk + NB - 1) / NB;
    const int m_chunks = (max_tiles + MT - 1) / MT;
    const size_t lds = WAVES > 1 ? (size_t)WAVES * NB * 16 * 64 * sizeof(float) : 0;   // one row tile at a time
    auto kern = gemm_bf16_k<MT, NB, WAVES, U, EPI>;
    if (lds > 64 * 1024) {
        static bool raised = false, ok = false;
        if (!raised) {
            raised = true;
            ok = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)lds) == hipSuccess;
            if (!ok) (void)hipGetLastError();
        }
        if (!ok) return false;
    }
    GemmArgs a;
    a.xp = (const bf16x8*)xp; a.wp = (const bf16x8*)wp; a.out = out; a.N = N; a.K16 = K / 16; a.n_groups = groups;
    a.m_chunks = m_chunks; a.max_tiles = max_tiles; a.ksplit = ksplit; a.part_stride = part_stride; a.n_tiles = n_tiles; a.epi = epi;
    hipLaunchKernelGGL(kern, dim3(groups * ksplit * m_chunks), dim3(WAVES * 64), lds, st, GEMM_LAUNCH_ARGS(a));
    return true;
}

template <int MT, int NB, int WAVES, int KU, int EPI>
static bool launch_rows_cfg(const void* xp, const void* wp, float* out, int N, int K, size_t part_stride, int ksplit,
                            const GemmEpilogue& epi, const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    const int nblk = N / 32;
    const int groups = (nblk + NB * WAVES - 1) / (NB * WAVES);
    const int m_chunks = (max_tiles + MT - 1) / MT;
    const size_t lds = (size_t)3 * KU * MT * 1024;
    auto kern = gemm_bf16_rows_k<MT, NB, WAVES, KU, EPI>;
    if (lds > 64 * 1024) {
        static bool raised = false, ok = false;
        if (!raised) {
            raised = true;
            ok = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)lds) == hipSuccess;
            if (!ok) (void)hipGetLastError();
        }
        if (!ok) return false;
    }
    GemmArgs a;
    a.xp = (const bf16x8*)xp; a.wp = (const bf16x8*)wp; a.out = out; a.N = N; a.K16 = K / 16; a.n_groups = groups;
    a.m_chunks = m_chunks; a.max_tiles = max_tiles; a.ksplit = ksplit; a.part_stride = part_stride; a.n_tiles = n_tiles; a.epi = epi;
    const int gk8 = (groups * ksplit + 7) / 8 * 8;
    hipLaunchKernelGGL(kern, dim3(gk8 * m_chunks), dim3(WAVES * 64), lds, st, GEMM_LAUNCH_ARGS(a));
    return true;
}

int gemm_groups(int N, const GemmPlan& plan, int epi_kind) {
    const int nblk = N / 32;
    (void)epi_kind;
    const int per = plan.kind == GEMM_ROWS ? plan.nb * plan.waves : plan.nb;     // (GEMM_LDS: nb blocks per workgroup)
    return (nblk + per - 1) / per;
}

static bool launch_gemm_rows(const void* xp, const void* wp, float* out, int N, int K, size_t part_stride,
                             GemmPlan plan, const GemmEpilogue& epi, const int32_t* n_tiles, int max_tiles,
                             hipStream_t st) {
#define RDLM_RCASE(MT_, NB_, W_, U_)                                                                             \
    if (plan.mt == MT_ && plan.nb == NB_ && plan.waves == W_ && plan.unroll == U_) {                             \
        if (epi.kind == EPI_F32)                                                                                 \
            return launch_rows_cfg<MT_, NB_, W_, U_, EPI_F32>(xp, wp, out, N, K, part_stride, plan.ksplit, epi,  \
                                                              n_tiles, max_tiles, st);                           \
        if (epi.kind == EPI_ARGMAX)                                                                              \
            return launch_rows_cfg<MT_, NB_, W_, U_, EPI_ARGMAX>(xp, wp, out, N, K, part_stride, 1, epi,         \
                                                                 n_tiles, max_tiles, st);                        \
        if (epi.kind == EPI_SWIGLU)                                                                              \
            return launch_rows_cfg<MT_, NB_, W_, U_, EPI_SWIGLU>(xp, wp, out, N, K, part_stride, 1, epi,         \
                                                                 n_tiles, max_tiles, st);                        \
        if (epi.kind == EPI_ROPE_KV)                                                                             \
            return launch_rows_cfg<MT_, NB_, W_, U_, EPI_ROPE_KV>(xp, wp, out, N, K, part_stride, 1, epi,        \
                                                                  n_tiles, max_tiles, st);                       \
        return false;                                                                                            \
    }
    RDLM_RCASE(2, 1, 4, 8) RDLM_RCASE(2, 1, 4, 4) RDLM_RCASE(2, 2, 4, 4) RDLM_RCASE(2, 2, 4, 2) RDLM_RCASE(2, 1, 8, 4)
    RDLM_RCASE(4, 1, 4, 4) RDLM_RCASE(4, 1, 4, 2) RDLM_RCASE(4, 2, 4, 4) RDLM_RCASE(4, 2, 4, 2) RDLM_RCASE(4, 1, 8, 4)
    RDLM_RCASE(8, 1, 4, 4) RDLM_RCASE(8, 1, 4, 2) RDLM_RCASE(8, 2, 4, 4) RDLM_RCASE(8, 2, 4, 2) RDLM_RCASE(8, 1, 8, 2)
    // five waves: 1120 and 165 feature blocks (widths 35840 and 5280) split into equal workgroups
    RDLM_RCASE(2, 1, 5, 5) RDLM_RCASE(4, 1, 5, 5)
#undef RDLM_RCASE
    return false;
}

bool launch_gemm_bf16(const void* xp, const void* wp, float* out, int N, int K, size_t part_stride,
                      GemmPlan plan, const GemmEpilogue& epi, const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    if (plan.kind == GEMM_ROWS)
        return launch_gemm_rows(xp, wp, out, N, K, part_stride, plan, epi, n_tiles, max_tiles, st);
    if (plan.kind == GEMM_LDS)
        return launch_gemm_lds(xp, wp, out, N, K, part_stride, plan, epi, n_tiles, max_tiles, st);
#define RDLM_CASE(MT_, NB_, W_, U_)                                                                              \
    if (plan.mt == MT_ && plan.nb == NB_ && plan.waves == W_ && plan.unroll == U_) {                             \
        if (epi.kind == EPI_F32)                                                                                 \
            return launch_cfg<MT_, NB_, W_, U_, EPI_F32>(xp, wp, out, N, K, part_stride, plan.ksplit, epi,       \
                                                         n_tiles, max_tiles, st);                                \
        if (epi.kind == EPI_ARGMAX)                                                                              \
            return launch_cfg<MT_, NB_, W_, U_, EPI_ARGMAX>(xp, wp, out, N, K, part_stride, 1, epi, n_tiles,     \
                                                            max_tiles, st);                                      \
        if (epi.kind == EPI_SWIGLU)                                                                              \
            return launch_cfg<MT_, NB_, W_, U_, EPI_SWIGLU>(xp, wp, out, N, K, part_stride, 1, epi, n_tiles,     \
                                                            max_tiles, st);                                      \
        if (epi.kind == EPI_ROPE_KV)                                                                             \
            return launch_cfg<MT_, NB_, W_, U_, EPI_ROPE_KV>(xp, wp, out, N, K, part_stride, 1, epi, n_tiles,    \
                                                             max_tiles, st);                                     \
        return false;                                                                                            \
    }
#define RDLM_ROW(NB_)                                                                                            \
    RDLM_CASE(1, NB_, 2, 4) RDLM_CASE(1, NB_, 2, 8) RDLM_CASE(1, NB_, 4, 2) RDLM_CASE(1, NB_, 4, 4)              \
    RDLM_CASE(1, NB_, 8, 1) RDLM_CASE(1, NB_, 8, 2)
    RDLM_ROW(1) RDLM_ROW(2) RDLM_ROW(3) RDLM_ROW(4) RDLM_ROW(5)
    // two and four row tiles per workgroup (windows of 33..128 rows): the same shapes as above
    RDLM_CASE(2, 2, 2, 4) RDLM_CASE(2, 2, 2, 2) RDLM_CASE(2, 2, 8, 1) RDLM_CASE(2, 2, 8, 2) RDLM_CASE(2, 5, 4, 2)
    RDLM_CASE(2, 4, 4, 2)
    RDLM_CASE(4, 2, 8, 1) RDLM_CASE(4, 2, 8, 2)
#undef RDLM_ROW
#undef RDLM_CASE
    return false;
}

// canonical bf16 rows -> MFMA-ordered tiles [N/32][K/16][64 lanes][8].  Row f of packed block b is
// canonical row canon_col(layout, b, f); canonical rows below `split` come from w0, the others
// from w1 (the gate and up matrices are separate tensors).
__global__ void pack_weight_k(const uint16_t* w0, const uint16_t* w1, int split, uint16_t* wp, int N, int K,
                              int layout, int n_heads, int head_dim, int ld) {
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;       // one lane-vector (8 elements) each
    size_t total = (size_t)(N / 32) * (K / 16) * 64;
    if (idx >= total) return;
    int lane = idx & 63;
    size_t tile = idx >> 6;
    int kt = (int)(tile % (K / 16));
    int nb = (int)(tile / (K / 16));
    int n = canon_col(layout, nb, lane & 31, N, n_heads, head_dim);
    const uint16_t* src = (n < split ? w0 + (size_t)n * ld : w1 + (size_t)(n - split) * ld) + kt * 16 + (lane >> 5) * 8;
    uint4 v = *reinterpret_cast<const uint4*>(src);
    *reinterpret_cast<uint4*>(wp + idx * 8) = v;
}
void launch_pack_weight(const void* w0, const void* w1, int split, void* wp, int N, int K, int layout, int n_heads,
                        int head_dim, hipStream_t st, int ld) {
    size_t total = (size_t)(N / 32) * (K / 16) * 64;
    hipLaunchKernelGGL(pack_weight_k, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const uint16_t*)w0,
                       (const uint16_t*)w1, split, (uint16_t*)wp, N, K, layout, n_heads, head_dim, ld ? ld : K);
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
