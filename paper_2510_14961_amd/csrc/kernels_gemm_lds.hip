// GEMM for steps with several row tiles (wide windows, ragged batches, prefill), third data flow:
// every operand tile goes from global memory straight into LDS (global_load_lds_dwordx4: no
// registers in between, so the prefetch can run several stages ahead), the weight tiles of a
// stage are shared by all waves of the workgroup, and wave w owns row tiles w*MTW .. w*MTW+MTW-1
// against all FB feature blocks of the workgroup -- the mirror image of gemm_bf16_rows_k, whose
// waves own feature blocks and share the row tiles.  One weight tile read from LDS feeds MTW
// matrix instructions.
//
// Ring of D stages of KU k tiles.  All loads of a wave are direct-to-LDS loads, so one in-order
// counter (vmcnt) tells which stages have landed; a wave waits until its own loads of stage s+1
// are done, the barrier that follows makes that true for every wave, and only then is the slot of
// stage s-1 (which every wave has finished reading: its LDS reads are waited for before the barrier)
// refilled.  While the matrix instructions of one k tile run, the operands of the next one -- the
// next stage's first, at the end of a stage -- are read from LDS.  (Ordinary register loads in the
// same loop would share the counter but not the return order of the direct-to-LDS loads: measured,
// a mix gave wrong sums at shallow ring depths.)
#include "gemm_common.h"

#include <type_traits>

// instances: (feature blocks, row tiles per wave, waves, k tiles per stage, ring depth)
#define RDLM_LDS_INSTANCES                                                                                    \
    RDLM_LCASE(5, 1, 4, 2, 6) RDLM_LCASE(5, 1, 4, 3, 4) RDLM_LCASE(5, 1, 8, 1, 8) RDLM_LCASE(5, 2, 4, 2, 4)   \
    RDLM_LCASE(5, 2, 8, 1, 6) RDLM_LCASE(8, 1, 4, 2, 6) RDLM_LCASE(8, 1, 8, 1, 6) RDLM_LCASE(4, 2, 8, 1, 6)   \
    RDLM_LCASE(2, 1, 4, 2, 6) RDLM_LCASE(2, 2, 8, 1, 6) RDLM_LCASE(4, 1, 4, 2, 6) RDLM_LCASE(4, 1, 8, 1, 8)   \
    RDLM_LCASE(3, 1, 4, 2, 6) RDLM_LCASE(3, 2, 8, 1, 6) RDLM_LCASE(2, 1, 8, 2, 6) RDLM_LCASE(2, 4, 4, 1, 6)

namespace rdlm {

typedef const void __attribute__((address_space(1)))* lds_gptr_t;
typedef void __attribute__((address_space(3)))* lds_lptr_t;

constexpr int lds_slot_tiles(int FB, int MTW, int WM, int KU) { return KU * FB + 1 + WM * KU * MTW; }

template <int FB, int MTW, int WM, int KU, int D, int NT, int EPI>
__global__ __launch_bounds__(WM * 64) void gemm_bf16_lds_k(GEMM_KERNEL_PARAMS) {
    GEMM_KERNEL_ARGS_STRUCT;
    static_assert((D * KU) % 2 == 0 && D >= 4, "operand double buffer parity, ring depth");
    constexpr int WT = KU * FB;                     // weight tiles per stage
    constexpr int PERW = (WT + WM - 1) / WM;        // weight loads per wave per stage (padded with loads into a spare tile)
    constexpr int XT = KU * MTW;                    // activation tiles per wave per stage
    constexpr int VM = PERW + XT;                   // loads per wave per stage
    constexpr int INFL = (D - 3) * VM;              // loads outstanding once stage s+1 has landed
    static_assert((D - 1) * VM <= 63, "the counter holds 63");
    constexpr int SLOT = lds_slot_tiles(FB, MTW, WM, KU);   // tiles per ring slot: weights, spare, activations [wave][k][tile]
    extern __shared__ float red[];
    bf16x8* lds = reinterpret_cast<bf16x8*>(red);
    __shared__ float cand_v[1][MTW][32];            // (the argmax epilogue of this kernel needs no exchange)
    __shared__ int cand_i[1][MTW][32];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nblk = A.N >> 5, K16 = A.K16;
    // id = xcd + 8 * (row chunk + m_chunks * j): the row chunks of one (group, split) run back to back on one XCD
    const int xcd = blockIdx.x & 7, rest = blockIdx.x >> 3;
    const int mc = rest % A.m_chunks, gk = (rest / A.m_chunks) * 8 + xcd;
    if (gk >= A.n_groups * A.ksplit) return;
    const int ks = gk % A.ksplit, grp = gk / A.ksplit;
    const int n_tiles = *A.n_tiles;
    if (mc * WM * MTW >= n_tiles) return;
    const int t0 = (mc * WM + wave) * MTW;          // this wave's first row tile (may lie beyond the count: nothing stored)
    const int kbeg = (int)(((long long)K16 * ks) / A.ksplit), kend = (int)(((long long)K16 * (ks + 1)) / A.ksplit);
    const int nsteps = (kend - kbeg + KU - 1) / KU;
    float sc[MTW];
    gemm_row_scales<MTW>(A, t0, n_tiles, sc);

    int blk[FB];
#pragma unroll
    for (int a = 0; a < FB; ++a) blk[a] = grp * FB + a;
    const bf16x8* wsrc[PERW];
    int wdst[PERW], wu[PERW];
#pragma unroll
    for (int i = 0; i < PERW; ++i) {
        int idx = wave + i * WM;
        const bool real = idx < WT;
        if (!real) idx = 0;
        wu[i] = idx / FB;
        wsrc[i] = A.wp + ((size_t)min(grp * FB + idx % FB, nblk - 1) * K16) * 64 + lane;   // a ragged last group re-reads a valid block
        wdst[i] = real ? idx : WT;
    }
    const bf16x8* xsrc[MTW];
#pragma unroll
    for (int b = 0; b < MTW; ++b) xsrc[b] = A.xp + ((size_t)min(t0 + b, n_tiles - 1) * K16) * 64 + lane;
    const int xoff = WT + 1 + wave * XT;

    f32x16 acc[FB][MTW];
#pragma unroll
    for (int a = 0; a < FB; ++a)
#pragma unroll
        for (int b = 0; b < MTW; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    // loads of stage `st` (clamped to the k range: every stage issues the same loads) into ring slot `pos`
    auto issue = [&](int pos, int st) {
        const int kt = kbeg + min(st, nsteps - 1) * KU;
#pragma unroll
        for (int i = 0; i < PERW; ++i)
            __builtin_amdgcn_global_load_lds((lds_gptr_t)(wsrc[i] + (size_t)min(kt + wu[i], kend - 1) * 64),
                                             (lds_lptr_t)(lds + ((size_t)pos * SLOT + wdst[i]) * 64), 16, 0, NT ? 2 : 0);
#pragma unroll
        for (int u = 0; u < KU; ++u)
#pragma unroll
            for (int b = 0; b < MTW; ++b)
                __builtin_amdgcn_global_load_lds((lds_gptr_t)(xsrc[b] + (size_t)min(kt + u, kend - 1) * 64),
                                                 (lds_lptr_t)(lds + ((size_t)pos * SLOT + xoff + u * MTW + b) * 64), 16, 0, 0);
    };
    bf16x8 wv[2][FB], xv[2][MTW];
    auto read_ops = [&](int par, int pos, int u) {
        const bf16x8* st = lds + (size_t)pos * SLOT * 64 + lane;
#pragma unroll
        for (int a = 0; a < FB; ++a) wv[par][a] = st[(u * FB + a) * 64];
#pragma unroll
        for (int b = 0; b < MTW; ++b) xv[par][b] = st[(xoff + u * MTW + b) * 64];
    };
    auto wait_loads = [](auto n) {                  // vmcnt(n) lgkmcnt(0)
        constexpr int N = decltype(n)::value;
        __builtin_amdgcn_s_waitcnt(0x0070 | (N & 0xF) | ((N >> 4) << 14));
    };
#pragma unroll
    for (int p = 0; p < D - 1; ++p) issue(p, p);
    wait_loads(std::integral_constant<int, (D - 2) * VM>{});    // stage 0
    __builtin_amdgcn_s_barrier();
    read_ops(0, 0, 0);
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int s0 = 0; s0 < nsteps; s0 += D) {        // ring turns; steps beyond the range add zeros
#pragma unroll
        for (int p = 0; p < D; ++p) {
            const int s = s0 + p;
            wait_loads(std::integral_constant<int, INFL>{});     // own loads of stage s+1 landed; operands of this step arrived
            __builtin_amdgcn_s_barrier();
            issue((p + D - 1) % D, s + D - 1);
#pragma unroll
            for (int u = 0; u < KU; ++u) {
                const int par = (p * KU + u) & 1;
                if (u + 1 < KU) read_ops(par ^ 1, p, u + 1);
                else read_ops(par ^ 1, (p + 1) % D, 0);
                const bool live = s < nsteps && kbeg + s * KU + u < kend;
#pragma unroll
                for (int b = 0; b < MTW; ++b) {
                    const bf16x8 x = live ? xv[par][b] : zero;
#pragma unroll
                    for (int a = 0; a < FB; ++a)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv[par][a], x, acc[a][b], 0, 0, 0);
                }
                // schedule: one LDS read between matrix instructions while there are reads left
#pragma unroll
                for (int i = 0; i < FB + MTW; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                if (FB * MTW > FB + MTW) __builtin_amdgcn_sched_group_barrier(0x008, FB * MTW - FB - MTW, 0);
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(0);                  // the clamped loads of the last turns must land before the workgroup ends
    auto quad_sum = [&](int a, int b, int q, float (&o)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = acc[a][b][q * 4 + i];
    };
    gemm_epilogue<MTW, FB, 1, 1, EPI, decltype(quad_sum), decltype(cand_v), decltype(cand_i), true>(
        A, blk, t0, n_tiles, ks, grp, sc, quad_sum, cand_v, cand_i);
}

template <int FB, int MTW, int WM, int KU, int D, int NT, int EPI>
static bool launch_lds_cfg(const void* xp, const void* wp, float* out, int N, int K, size_t part_stride, int ksplit,
                           const GemmEpilogue& epi, const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    const int nblk = N / 32;
    const int groups = (nblk + FB - 1) / FB;
    const int m_chunks = (max_tiles + WM * MTW - 1) / (WM * MTW);
    const size_t lds = (size_t)D * lds_slot_tiles(FB, MTW, WM, KU) * 1024;
    if (lds > 158 * 1024) return false;
    auto kern = gemm_bf16_lds_k<FB, MTW, WM, KU, D, NT, EPI>;
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
    hipLaunchKernelGGL(kern, dim3(gk8 * m_chunks), dim3(WM * 64), lds, st, GEMM_LAUNCH_ARGS(a));
    return true;
}

// plan: nb = FB (feature blocks per workgroup), waves = WM, mt = WM * MTW (row tiles per workgroup),
// unroll = KU, depth = D.  Weights are read with the non-temporal hint when no other workgroup
// re-reads them (one row chunk).
bool launch_gemm_lds(const void* xp, const void* wp, float* out, int N, int K, size_t part_stride, GemmPlan plan,
                     const GemmEpilogue& epi, const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    if (plan.waves < 1 || plan.mt % plan.waves) return false;
    const int mtw = plan.mt / plan.waves;
    const bool nt = (max_tiles + plan.mt - 1) / plan.mt == 1;
#define RDLM_LCASE2(FB_, MTW_, WM_, KU_, D_, NT_)                                                                  \
    {                                                                                                              \
        if (epi.kind == EPI_F32)                                                                                   \
            return launch_lds_cfg<FB_, MTW_, WM_, KU_, D_, NT_, EPI_F32>(xp, wp, out, N, K, part_stride, plan.ksplit, \
                                                                         epi, n_tiles, max_tiles, st);             \
        if (epi.kind == EPI_ARGMAX)                                                                                \
            return launch_lds_cfg<FB_, MTW_, WM_, KU_, D_, NT_, EPI_ARGMAX>(xp, wp, out, N, K, part_stride, 1, epi, \
                                                                            n_tiles, max_tiles, st);               \
        if (epi.kind == EPI_SWIGLU)                                                                                \
            return launch_lds_cfg<FB_, MTW_, WM_, KU_, D_, NT_, EPI_SWIGLU>(xp, wp, out, N, K, part_stride, 1, epi, \
                                                                            n_tiles, max_tiles, st);               \
        if (epi.kind == EPI_ROPE_KV)                                                                               \
            return launch_lds_cfg<FB_, MTW_, WM_, KU_, D_, NT_, EPI_ROPE_KV>(xp, wp, out, N, K, part_stride, 1, epi, \
                                                                             n_tiles, max_tiles, st);              \
        return false;                                                                                              \
    }
#define RDLM_LCASE(FB_, MTW_, WM_, KU_, D_)                                                                        \
    if (plan.nb == FB_ && mtw == MTW_ && plan.waves == WM_ && plan.unroll == KU_ && plan.depth == D_) {            \
        if (nt) RDLM_LCASE2(FB_, MTW_, WM_, KU_, D_, 1)                                                            \
        else RDLM_LCASE2(FB_, MTW_, WM_, KU_, D_, 0)                                                               \
    }
    RDLM_LDS_INSTANCES
#undef RDLM_LCASE
#undef RDLM_LCASE2
    return false;
}

}  // namespace rdlm
