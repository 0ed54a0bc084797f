// Host side of librdlm: context, weight re-tiling, the block forwards (P, R, C), the sampler
// driver of Alg. 1 / Alg. 2 on one stream, and the C ABI declared in include/rdlm.h.
#include "../../include/rdlm.h"
#include "rdlm_internal.h"

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cctype>
#include <cstring>
#include <strings.h>
#include <utility>
#include <vector>

using namespace rdlm;

struct Layer {
    float* g1 = nullptr;
    float* g2 = nullptr;
    void* wqkv = nullptr;
    void* wo = nullptr;
    void* wgu = nullptr;     // gate rows then up rows: [2F, h]
    void* wd = nullptr;
    void* kc = nullptr;      // K pool: [kv_pool_blocks] blocks of 32 positions; f32 [32][H][d], bf16 in operand order (k_cache_off)
    void* vc = nullptr;      // V pool: f32 same layout; bf16 transposed per block
};

enum Proj { PROJ_QKV = 0, PROJ_O, PROJ_GU, PROJ_D, PROJ_A, PROJ_HEAD, PROJ_COUNT };

// Tuning knobs (launch shapes, fusion switches).  Read from the environment once, in rdlm_create
// (RDLM_<NAME> with NAME in upper case), or set on a context with rdlm_set_tuning; never looked up
// inside a step.
struct Knobs {
    int att_split = 0;               // > 0: forced number of KV splits of the attention kernels
    long long att_group_keys = -1;   // >= 0: segments x visible keys from which the grouped attention kernel is used
    bool no_rope_fusion = false;     // RoPE + cache writes in a kernel of their own instead of the QKV epilogue
    bool no_fold_fusion = false;     // split-K folds in fold_k launches instead of the producing GEMM
    bool no_fold = false;            // full RMSNorm kernels instead of the deferred 1/rms factor
    bool no_lds_gemm = false;        // steps with three row tiles and more: the row-sharing kernel everywhere
    bool no_pack = false;            // every sequence's rows start a row tile of their own (short windows are not packed)
    bool no_hoist = false;           // several recurrences per call: W_a . [e; z] in one product every time
    bool has_plan[PROJ_COUNT] = {}, has_plan_rows[PROJ_COUNT] = {};
    GemmPlan plan[PROJ_COUNT], plan_rows[PROJ_COUNT];
};

// Scratch memory of a step: everything the kernels of one call write and read back, nothing that has
// to survive the call except that the ticket words are zero between launches.  One slab, cut up by
// carve_workspace: the context's own (allocated by rdlm_create or handed in by the caller) or, for
// rdlm_core_step_static, the file-scope device array below.
struct Workspace {
    int max_tiles = 0, rows_pad = 0;
    TileDesc* tiles = nullptr;
    int32_t* n_tiles = nullptr;
    TileDesc* tiles_samp = nullptr;      // the sampler's own tile list (built at the end of each step for the next)
    int32_t* n_tiles_samp = nullptr;
    float *x = nullptr, *e = nullptr, *qkv = nullptr, *gu = nullptr, *part = nullptr, *logits = nullptr;
    float *delta = nullptr, *zp_api = nullptr, *att_ws = nullptr;
    float* xe = nullptr;            // bf16: W_e . e of the current rows, kept over the recurrences of a call
    void *xn = nullptr, *abuf = nullptr, *q = nullptr, *att = nullptr;
    int32_t* drafts = nullptr;
    float* ssq = nullptr;           // [SSQ_MAX_CHUNKS + 1][rows_pad] partial sums of squares of the folded rows
    uint32_t* fold_counter = nullptr;   // tickets of the folding GEMMs, one per feature group, zero between launches
    float* rope_tab = nullptr;      // [rows_pad][d/2] (cos, sin) of the current step's rows
    float* cand_val = nullptr;
    int32_t* cand_idx = nullptr;
    uint32_t* att_tickets = nullptr;     // [max_tiles][heads], zero between launches
    uint32_t* step_ticket = nullptr;     // step_end_k's arrival counter, zero between launches
    // the ticket words, for clearing: [ticket_lo, ticket_lo + ticket_bytes)
    void* ticket_lo = nullptr;
    size_t ticket_bytes = 0;
};

struct rdlm_ctx : Workspace {
    rdlm_model m;
    int max_seqs = 0, max_positions = 0, ctx_pad = 0, max_rows = 0;
    hipStream_t st = nullptr;
    int fmt = ACT_F32;
    size_t esz = 4;
    std::vector<Layer> layers;
    void* emb_canon = nullptr;
    void* emb_w = nullptr;
    void* wa = nullptr;
    void* wa_e = nullptr;                // bf16: the two [h, h] halves of W_a packed on their own (the e half's
    void* wa_z = nullptr;                // product is computed once for all recurrences of a call)
    int seg_tiles = 0;                   // bound on the segments (runs of up to 32 rows of one sequence) of the current tile list
    int att_groups = 0;                  // bound on the attention groups of the current tile list (0: the tile count)
    bool hoist_split = false;            // this step's prelude leaves e and z as separate adapter operands
    float* gf = nullptr;
    float* gout = nullptr;
    float* theta = nullptr;
    int ssq_count = 0;              // slots per row the last producer of the normalised operand filled
    int att_max_split = 8;
    // paged KV cache: block table (device and host copy), free list, blocks held per slot
    int32_t* blk_table = nullptr;        // [max_seqs][blocks_per_seq] physical block of each logical block
    int blocks_per_seq = 0, kv_pool_blocks = 0;
    std::vector<int32_t> tbl_host;
    std::vector<int> free_blocks, seq_blocks;
    std::vector<int> pos_bound;          // sampler: positions a sequence may have reached before the next step
    int32_t* seq_ident = nullptr;        // [max_seqs] identity of the slot's sequence in the random generator's counters
    std::vector<int32_t> ident_host;
    // sampler state
    SeqState* seqs = nullptr;
    int32_t* y = nullptr;
    int32_t* counts = nullptr;
    int32_t* seq_step0 = nullptr;    // [max_seqs] sampler step each sequence joined at
    float *z_store = nullptr, *z_prev = nullptr, *e_store = nullptr;
    int32_t* n_active = nullptr;     // [0] unfinished sequences, [1] step the last one finished at, [2] non-finite deltas seen
    int32_t* n_active_host = nullptr;    // pinned
    SamplerParams sp;
    rdlm_sampler sampler;
    int samp_seqs = 0;
    int step = 0;
    bool sampler_on = false;
    bool joined = false;             // a sequence joined the running sampler (windows no longer grow in lockstep)
    std::vector<int> prompt_len;
    int last_hip = 0;
    size_t bytes = 0;
    std::vector<void*> allocs;
    bool coda_ready = false;        // the closing norm of the recurrence left the coda's first operand in xn
    bool grouped = false;           // current step: some sequence has several row tiles (grouped attention)
    int seq_tiles_max = 1;          // current step: most row tiles of one sequence
    Knobs knobs;
    // per-launch GEMM timing
    int prof_n = 0, prof_k = 0, prof_used = 0;
    std::vector<hipEvent_t> prof_ev;
};

#define HIPCHK(call)                                                                          \
    do {                                                                                      \
        hipError_t e__ = (call);                                                              \
        if (e__ != hipSuccess) {                                                              \
            fprintf(stderr, "rdlm: %s failed: %s (%s:%d)\n", #call, hipGetErrorString(e__),   \
                    __FILE__, __LINE__);                                                      \
            ctx->last_hip = (int)e__;                                                         \
            return RDLM_EHIP;                                                                 \
        }                                                                                     \
    } while (0)

static int dalloc(rdlm_ctx* ctx, void** p, size_t bytes, bool zero) {
    if (bytes == 0) bytes = 256;
    hipError_t e = hipMalloc(p, bytes);
    if (e != hipSuccess) {
        fprintf(stderr, "rdlm: hipMalloc(%zu bytes) failed: %s (total so far %zu)\n", bytes, hipGetErrorString(e),
                ctx->bytes);
        ctx->last_hip = (int)e; *p = nullptr; return RDLM_ENOMEM;
    }
    ctx->allocs.push_back(*p);
    ctx->bytes += bytes;
    if (zero) {
        e = hipMemsetAsync(*p, 0, bytes, ctx->st);
        if (e != hipSuccess) { ctx->last_hip = (int)e; return RDLM_EHIP; }
    }
    return RDLM_OK;
}
#define DALLOC(ptr, bytes, zero)                                              \
    do {                                                                      \
        int rc__ = dalloc(ctx, reinterpret_cast<void**>(&(ptr)), (bytes), (zero)); \
        if (rc__ != RDLM_OK) return rc__;                                     \
    } while (0)

static int check_launch(rdlm_ctx* ctx) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        fprintf(stderr, "rdlm: kernel launch failed: %s\n", hipGetErrorString(e));
        ctx->last_hip = (int)e;
        return RDLM_EHIP;
    }
    return RDLM_OK;
}

extern "C" const char* rdlm_strerror(int s) {
    switch (s) {
        case RDLM_OK: return "ok";
        case RDLM_EINVAL: return "invalid argument";
        case RDLM_ECAPACITY: return "exceeds the capacity the context was created with";
        case RDLM_ENOMEM: return "device allocation failed";
        case RDLM_EHIP: return "HIP call failed";
        case RDLM_ESTATE: return "call out of order";
        case RDLM_ENUMERIC: return "a non-finite latent reached the exit rule";
        default: return "unknown status";
    }
}
extern "C" int rdlm_last_hip_error(const rdlm_ctx* ctx) { return ctx ? ctx->last_hip : 0; }
extern "C" size_t rdlm_device_bytes(const rdlm_ctx* ctx) { return ctx ? ctx->bytes : 0; }

static bool model_ok(const rdlm_model* m) {
    if (!m) return false;
    if (m->hidden > 8192) return false;                 // row kernels keep a row in registers
    if (m->vocab <= 0 || m->hidden <= 0 || m->n_heads <= 0 || m->head_dim <= 0 || m->mlp <= 0) return false;
    if (m->n_prelude < 0 || m->n_core < 1 || m->n_coda < 0) return false;
    if ((long long)m->n_heads * m->head_dim != m->hidden) return false;
    if (m->head_dim % 2) return false;
    if (!(m->rope_base > 0.f) || !(m->rms_eps >= 0.f)) return false;
    if (m->dtype == RDLM_F32) {
        if (m->hidden % 4 || m->mlp % 4) return false;
    } else if (m->dtype == RDLM_BF16) {
        if (m->hidden % 32 || m->mlp % 32 || m->vocab % 32) return false;
        if (m->head_dim != 32 && m->head_dim != 64 && m->head_dim != 96 && m->head_dim != 128) return false;
    } else {
        return false;
    }
    if (m->mlp < m->hidden) return false;               // staging buffers assume h <= F
    return true;
}

extern "C" int32_t rdlm_num_weights(const rdlm_model* m) {
    if (!m) return 0;
    return 1 + 7 * (m->n_prelude + m->n_core + m->n_coda) + 3;
}

extern "C" int rdlm_destroy(rdlm_ctx* ctx) {
    if (!ctx) return RDLM_EINVAL;
    (void)hipStreamSynchronize(ctx->st);
    for (void* p : ctx->allocs) (void)hipFree(p);
    for (hipEvent_t ev : ctx->prof_ev) (void)hipEventDestroy(ev);
    if (ctx->n_active_host) (void)hipHostFree(ctx->n_active_host);
    delete ctx;
    return RDLM_OK;
}

// copy (f32) or re-tile (bf16) a matrix [N,K] into library memory
static int take_matrix(rdlm_ctx* ctx, const void* src, int N, int K, void** dst, int layout = WL_NATURAL) {
    size_t bytes = (size_t)N * K * ctx->esz;
    DALLOC(*dst, bytes, false);
    if (ctx->m.dtype == RDLM_F32) HIPCHK(hipMemcpyAsync(*dst, src, bytes, hipMemcpyDeviceToDevice, ctx->st));
    else launch_pack_weight(src, src, N, *dst, N, K, layout, ctx->m.n_heads, ctx->m.head_dim, ctx->st);
    return check_launch(ctx);
}
static int take_gain(rdlm_ctx* ctx, const void* src, int h, float** dst) {
    DALLOC(*dst, (size_t)h * 4, false);
    HIPCHK(hipMemcpyAsync(*dst, src, (size_t)h * 4, hipMemcpyDeviceToDevice, ctx->st));
    return RDLM_OK;
}

// Cut a workspace for steps of up to max_tiles row tiles out of the slab at `base` (null: only
// count).  Returns the bytes needed.  `full`: also what the prelude, the coda and the sampler use
// (conditioning rows, logits, argmax candidates, drafts, the sampler's second tile list); without
// it only what rdlm_core_step touches.
static size_t carve_workspace(Workspace* ws, void* base, const rdlm_model& m, int max_tiles, int att_max_split,
                              bool full) {
    const int h = m.hidden, F = m.mlp, V = m.vocab;
    const size_t esz = m.dtype == RDLM_F32 ? 4 : 2;
    const size_t R = (size_t)max_tiles * 32;
    const size_t wide = (size_t)std::max(2 * h, F);
    size_t off = 0;
    auto take = [&](size_t bytes) -> void* {
        void* p = base ? static_cast<char*>(base) + off : nullptr;
        off += (std::max<size_t>(bytes, 1) + 255) / 256 * 256;
        return p;
    };
    Workspace w;
    w.max_tiles = max_tiles; w.rows_pad = (int)R;
    // ticket words first, contiguous: they are the only part that must read zero when a call starts
    w.ticket_lo = take(0);
    w.fold_counter = (uint32_t*)take((SSQ_MAX_CHUNKS + 1) * 4);
    w.att_tickets = (uint32_t*)take((size_t)max_tiles * m.n_heads * 4);
    w.step_ticket = (uint32_t*)take(64);
    w.ticket_bytes = off;
    w.tiles = (TileDesc*)take(sizeof(TileDesc) * (R + max_tiles));     // row descriptors, then the segments
    w.n_tiles = (int32_t*)take(tile_count_bytes(max_tiles));
    w.x = (float*)take(R * h * 4);
    w.qkv = (float*)take(R * 3 * h * 4);
    // f32 gate/up sums: the f32 path's GEMM output, rdlm_linear's, and the staging area of rdlm_read_kv
    if (full || m.dtype == RDLM_F32) w.gu = (float*)take(R * 2 * F * 4);
    w.part = (float*)take(8 * R * h * 4);
    w.delta = (float*)take(R * 4);
    w.zp_api = (float*)take(R * h * 4);
    if (m.dtype == RDLM_BF16) w.xe = (float*)take(R * h * 4);
    w.xn = take(R * h * esz);
    w.abuf = take(R * wide * esz);
    w.q = take(R * h * esz);
    w.att = take(R * h * esz);
    w.ssq = (float*)take(R * (SSQ_MAX_CHUNKS + 1) * 4);       // + one slot: row totals left by a folding GEMM
    w.rope_tab = (float*)take(R * (m.head_dim / 2) * 8);
    if (m.dtype == RDLM_BF16) w.att_ws = (float*)take(attention_ws_floats(max_tiles, m.n_heads, m.head_dim, att_max_split) * 4);
    if (full) {
        w.tiles_samp = (TileDesc*)take(sizeof(TileDesc) * (R + max_tiles));
        w.n_tiles_samp = (int32_t*)take(tile_count_bytes(max_tiles));
        w.e = (float*)take(R * h * 4);
        w.logits = (float*)take(R * V * 4);
        w.drafts = (int32_t*)take(R * 4);
        w.cand_val = (float*)take((size_t)(V / 32 + 1) * R * 4);
        w.cand_idx = (int32_t*)take((size_t)(V / 32 + 1) * R * 4);
    }
    if (ws) *ws = w;
    return off;
}

static int tiles_for(int max_seqs, int max_rows) { return (max_rows + 31) / 32 + max_seqs; }

static int create_impl(rdlm_ctx* ctx, const void* const* wp, void* workspace) {
    const rdlm_model& m = ctx->m;
    const int h = m.hidden, F = m.mlp, V = m.vocab;
    const size_t esz = ctx->esz;
    int wi = 0, rc;
    // embedding: canonical copy for the gather, tiled copy as the tied LM head
    DALLOC(ctx->emb_canon, (size_t)V * h * esz, false);
    HIPCHK(hipMemcpyAsync(ctx->emb_canon, wp[wi], (size_t)V * h * esz, hipMemcpyDeviceToDevice, ctx->st));
    if (m.dtype == RDLM_F32) ctx->emb_w = ctx->emb_canon;
    else if ((rc = take_matrix(ctx, wp[wi], V, h, &ctx->emb_w))) return rc;
    ++wi;
    const int nl = m.n_prelude + m.n_core + m.n_coda;
    ctx->layers.resize(nl);
    const size_t cache_elems = (size_t)ctx->kv_pool_blocks * 32 * h;
    for (int l = 0; l < nl; ++l) {
        Layer& L = ctx->layers[l];
        if ((rc = take_gain(ctx, wp[wi++], h, &L.g1))) return rc;
        if ((rc = take_matrix(ctx, wp[wi++], 3 * h, h, &L.wqkv, WL_ROPE))) return rc;
        if ((rc = take_matrix(ctx, wp[wi++], h, h, &L.wo))) return rc;
        if ((rc = take_gain(ctx, wp[wi++], h, &L.g2))) return rc;
        // gate and up as one [2F, h] matrix (bf16: 16 gate rows and their 16 up rows per block)
        DALLOC(L.wgu, (size_t)2 * F * h * esz, false);
        if (m.dtype == RDLM_F32) {
            for (int part = 0; part < 2; ++part)
                HIPCHK(hipMemcpyAsync(reinterpret_cast<char*>(L.wgu) + (size_t)part * F * h * esz, wp[wi + part],
                                      (size_t)F * h * esz, hipMemcpyDeviceToDevice, ctx->st));
        } else {
            launch_pack_weight(wp[wi], wp[wi + 1], F, L.wgu, 2 * F, h, WL_GU16, m.n_heads, m.head_dim, ctx->st);
        }
        wi += 2;
        if ((rc = take_matrix(ctx, wp[wi++], h, F, &L.wd))) return rc;
        DALLOC(L.kc, cache_elems * esz, true);
        DALLOC(L.vc, cache_elems * esz, true);
    }
    if (m.dtype == RDLM_BF16) {
        const uint16_t* src = static_cast<const uint16_t*>(wp[wi]);
        const size_t half = (size_t)h * h * 2;
        DALLOC(ctx->wa_e, half, false);
        DALLOC(ctx->wa_z, half, false);
        launch_pack_weight(src, src, h, ctx->wa_e, h, h, WL_NATURAL, m.n_heads, m.head_dim, ctx->st, 2 * h);
        launch_pack_weight(src + h, src + h, h, ctx->wa_z, h, h, WL_NATURAL, m.n_heads, m.head_dim, ctx->st, 2 * h);
    }
    if ((rc = take_matrix(ctx, wp[wi++], h, 2 * h, &ctx->wa))) return rc;
    if ((rc = take_gain(ctx, wp[wi++], h, &ctx->gf))) return rc;
    if ((rc = take_gain(ctx, wp[wi++], h, &ctx->gout))) return rc;
    if ((rc = check_launch(ctx))) return rc;

    // RoPE angles theta_i = base^(-2i/d), rounded once from double
    {
        std::vector<float> th(m.head_dim / 2);
        for (int i = 0; i < m.head_dim / 2; ++i)
            th[i] = (float)std::pow((double)m.rope_base, -2.0 * i / (double)m.head_dim);
        DALLOC(ctx->theta, th.size() * 4, false);
        HIPCHK(hipMemcpy(ctx->theta, th.data(), th.size() * 4, hipMemcpyHostToDevice));
    }
    // workspace: one slab (the caller's, or allocated here), cleared once with a fill kernel
    {
        const size_t need = carve_workspace(nullptr, nullptr, m, ctx->max_tiles, ctx->att_max_split, true);
        void* slab = workspace;
        if (!slab) DALLOC(slab, need, false);
        carve_workspace(ctx, slab, m, ctx->max_tiles, ctx->att_max_split, true);
        launch_fill_i32(reinterpret_cast<int32_t*>(slab), 0, need / 4, ctx->st);
    }
    // block table: every entry names a valid block (0) until a block is assigned, so that a clamped read
    // of an entry that no sequence owns yet stays inside the pool
    DALLOC(ctx->blk_table, (size_t)ctx->max_seqs * ctx->blocks_per_seq * 4, true);
    ctx->tbl_host.assign((size_t)ctx->max_seqs * ctx->blocks_per_seq, 0);
    ctx->seq_blocks.assign(ctx->max_seqs, 0);
    ctx->pos_bound.assign(ctx->max_seqs, 0);
    ctx->free_blocks.resize(ctx->kv_pool_blocks);
    for (int i = 0; i < ctx->kv_pool_blocks; ++i) ctx->free_blocks[i] = ctx->kv_pool_blocks - 1 - i;   // block 0 goes out first
    DALLOC(ctx->seq_ident, 4 * ctx->max_seqs + 64, true);
    ctx->ident_host.resize(ctx->max_seqs);
    for (int q = 0; q < ctx->max_seqs; ++q) ctx->ident_host[q] = q;
    HIPCHK(hipMemcpy(ctx->seq_ident, ctx->ident_host.data(), 4 * ctx->max_seqs, hipMemcpyHostToDevice));
    // sampler state
    const size_t SP = (size_t)ctx->max_seqs * ctx->max_positions;
    DALLOC(ctx->seqs, sizeof(SeqState) * ctx->max_seqs, true);
    DALLOC(ctx->seq_step0, 4 * ctx->max_seqs + 64, true);
    DALLOC(ctx->y, (SP + 64) * 4, true);
    DALLOC(ctx->counts, (SP + 64) * 4, true);
    DALLOC(ctx->z_store, SP * h * 4, true);
    DALLOC(ctx->z_prev, SP * h * 4, true);
    DALLOC(ctx->e_store, SP * h * 4, true);
    DALLOC(ctx->n_active, 64, true);
    HIPCHK(hipHostMalloc(reinterpret_cast<void**>(&ctx->n_active_host), 64, hipHostMallocDefault));
    memset(ctx->n_active_host, 0, 64);
    ctx->prompt_len.assign(ctx->max_seqs, 0);
    HIPCHK(hipStreamSynchronize(ctx->st));
    return RDLM_OK;
}

// ---------------------------------------------------------------------------------------------
// tuning knobs

static const char* kProjName[PROJ_COUNT] = {"qkv", "o", "gu", "d", "a", "head"};

static int set_knob(Knobs* k, const char* name, const char* value) {
    if (!name || !value) return RDLM_EINVAL;
    auto is = [&](const char* n) { return strcasecmp(name, n) == 0; };
    if (is("att_split")) { k->att_split = atoi(value); return RDLM_OK; }
    if (is("att_group_keys")) { k->att_group_keys = *value ? atoll(value) : -1; return RDLM_OK; }
    if (is("no_rope_fusion")) { k->no_rope_fusion = atoi(value) != 0; return RDLM_OK; }
    if (is("no_fold_fusion")) { k->no_fold_fusion = atoi(value) != 0; return RDLM_OK; }
    if (is("no_fold")) { k->no_fold = atoi(value) != 0; return RDLM_OK; }
    if (is("no_lds_gemm")) { k->no_lds_gemm = atoi(value) != 0; return RDLM_OK; }
    if (is("no_hoist")) { k->no_hoist = atoi(value) != 0; return RDLM_OK; }
    if (is("no_pack")) { k->no_pack = atoi(value) != 0; return RDLM_OK; }      // (refused while a sampler runs, see rdlm_set_tuning)
    for (int pj = 0; pj < PROJ_COUNT; ++pj) {
        char nm[32];
        // plan_<proj> = "nb,waves,unroll,ksplit": the one-tile launch shape ("" = default again)
        snprintf(nm, sizeof nm, "plan_%s", kProjName[pj]);
        if (is(nm)) {
            GemmPlan o = {1, 0, 0, 0, 0};
            k->has_plan[pj] = sscanf(value, "%d,%d,%d,%d", &o.nb, &o.waves, &o.unroll, &o.ksplit) == 4;
            if (k->has_plan[pj]) k->plan[pj] = o;
            return (k->has_plan[pj] || !value[0]) ? RDLM_OK : RDLM_EINVAL;
        }
        // planr_<proj> = "mt,nb,waves,unroll,ksplit" (row-sharing kernel) or "s<the same>" (streaming
        // kernel): the launch shape for several row tiles
        snprintf(nm, sizeof nm, "planr_%s", kProjName[pj]);
        if (is(nm)) {
            GemmPlan o = {0, 0, 0, 0, 1, GEMM_ROWS};
            const bool stream = value[0] == 's';
            if (value[0] == 'l') {      // "l<blocks>,<row tiles per wave>,<waves>,<k tiles per stage>,<ring depth>,<ksplit>"
                int mtw = 0;
                o.kind = GEMM_LDS;
                k->has_plan_rows[pj] =
                    sscanf(value + 1, "%d,%d,%d,%d,%d,%d", &o.nb, &mtw, &o.waves, &o.unroll, &o.depth, &o.ksplit) == 6;
                o.mt = mtw * o.waves;
                if (k->has_plan_rows[pj]) k->plan_rows[pj] = o;
                return k->has_plan_rows[pj] ? RDLM_OK : RDLM_EINVAL;
            }
            k->has_plan_rows[pj] =
                sscanf(value + (stream ? 1 : 0), "%d,%d,%d,%d,%d", &o.mt, &o.nb, &o.waves, &o.unroll, &o.ksplit) == 5;
            if (stream) o.kind = GEMM_STREAM;
            if (k->has_plan_rows[pj]) k->plan_rows[pj] = o;
            return (k->has_plan_rows[pj] || !value[0]) ? RDLM_OK : RDLM_EINVAL;
        }
    }
    return RDLM_EINVAL;
}

static void knobs_from_env(Knobs* k) {
    static const char* names[] = {"att_split", "att_group_keys", "no_rope_fusion", "no_fold_fusion", "no_fold", "no_lds_gemm", "no_hoist", "no_pack"};
    auto env_of = [](const char* name) {
        char buf[48] = "RDLM_";
        size_t n = strlen(buf);
        for (const char* c = name; *c && n + 1 < sizeof buf; ++c) buf[n++] = (char)toupper((unsigned char)*c);
        buf[n] = 0;
        return getenv(buf);
    };
    for (const char* nm : names)
        if (const char* v = env_of(nm)) (void)set_knob(k, nm, v);
    for (int pj = 0; pj < PROJ_COUNT; ++pj)
        for (const char* pre : {"plan_", "planr_"}) {
            char nm[32];
            snprintf(nm, sizeof nm, "%s%s", pre, kProjName[pj]);
            if (const char* v = env_of(nm)) (void)set_knob(k, nm, v);
        }
}

extern "C" int rdlm_set_tuning(rdlm_ctx* ctx, const char* name, const char* value) {
    if (!ctx) return RDLM_EINVAL;
    // the running sampler's tile list was laid out with the current setting
    if (name && !strcmp(name, "no_pack") && ctx->sampler_on) return RDLM_ESTATE;
    return set_knob(&ctx->knobs, name, value);
}

// ---------------------------------------------------------------------------------------------
// Scratch for callers that cannot allocate (rdlm_core_step_static): a file-scope device array.  Its
// name is a host-side stand-in, not a device address: the address is asked for once per device
// (static_scratch_for) and only that pointer is ever handed to kernels or copies.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)RDLM_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static void* g_scratch_ptr[MAX_DEVICES] = {};

// address of the current device's copy of `scratch`; looked up at most once per device
static int static_scratch_for(int* dev_out, void** ptr_out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return RDLM_EHIP;
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            fprintf(stderr, "rdlm: hipGetSymbolAddress(scratch) failed on device %d: %s\n", dev, hipGetErrorString(e));
            return RDLM_EHIP;
        }
        g_scratch_ptr[dev] = p;
    }
    if (dev_out) *dev_out = dev;
    if (ptr_out) *ptr_out = g_scratch_ptr[dev];
    return RDLM_OK;
}

extern "C" size_t rdlm_workspace_bytes(const rdlm_model* m, int32_t max_seqs, int32_t max_rows) {
    if (!model_ok(m) || max_seqs < 1 || max_seqs > MAX_API_SEQS || max_rows < 1) return 0;
    return carve_workspace(nullptr, nullptr, *m, tiles_for(max_seqs, max_rows), 8, true);
}

static int create_any(const rdlm_model* m, const void* const* weight_ptrs, int32_t max_seqs, int32_t max_positions,
                      int32_t max_rows, int32_t kv_pool_positions, void* hip_stream, void* workspace,
                      size_t workspace_bytes, rdlm_ctx** out) {
    if (!out) return RDLM_EINVAL;
    *out = nullptr;
    if (!model_ok(m) || !weight_ptrs) return RDLM_EINVAL;
    if (max_seqs < 1 || max_seqs > MAX_API_SEQS || max_positions < 2 || max_rows < 1) return RDLM_EINVAL;
    if (m->dtype == RDLM_F32 && max_positions > 8192) return RDLM_EINVAL;   // f32 attention keeps scores in LDS
    for (int i = 0; i < rdlm_num_weights(m); ++i)
        if (!weight_ptrs[i]) return RDLM_EINVAL;
    if (workspace) {
        if (reinterpret_cast<uintptr_t>(workspace) % 256) return RDLM_EINVAL;
        if (workspace_bytes < rdlm_workspace_bytes(m, max_seqs, max_rows)) return RDLM_ECAPACITY;
    }
    rdlm_ctx* ctx = new rdlm_ctx();
    ctx->m = *m;
    ctx->max_seqs = max_seqs;
    ctx->max_positions = max_positions;
    ctx->ctx_pad = (max_positions + 31) / 32 * 32;
    ctx->blocks_per_seq = ctx->ctx_pad / 32;
    // pool: by default every slot can reach max_positions at once; a smaller pool is shared by need
    ctx->kv_pool_blocks = kv_pool_positions > 0 ? (kv_pool_positions + 31) / 32 : max_seqs * ctx->blocks_per_seq;
    ctx->max_rows = max_rows;
    ctx->max_tiles = tiles_for(max_seqs, max_rows);
    ctx->rows_pad = ctx->max_tiles * 32;
    ctx->st = reinterpret_cast<hipStream_t>(hip_stream);
    ctx->fmt = m->dtype == RDLM_F32 ? ACT_F32 : ACT_BF16P;
    ctx->esz = m->dtype == RDLM_F32 ? 4 : 2;
    knobs_from_env(&ctx->knobs);
    int rc = static_scratch_for(nullptr, nullptr);     // this device's static scratch, for rdlm_core_step_static
    if (rc == RDLM_OK) rc = create_impl(ctx, weight_ptrs, workspace);
    if (rc != RDLM_OK) {
        for (void* p : ctx->allocs) (void)hipFree(p);
        if (ctx->n_active_host) (void)hipHostFree(ctx->n_active_host);
        delete ctx;
        return rc;
    }
    *out = ctx;
    return RDLM_OK;
}

extern "C" int rdlm_create_ws(const rdlm_model* m, const void* const* weight_ptrs, int32_t max_seqs,
                              int32_t max_positions, int32_t max_rows, void* hip_stream, void* workspace,
                              size_t workspace_bytes, rdlm_ctx** out) {
    return create_any(m, weight_ptrs, max_seqs, max_positions, max_rows, 0, hip_stream, workspace, workspace_bytes, out);
}

extern "C" int rdlm_create(const rdlm_model* m, const void* const* weight_ptrs, int32_t max_seqs,
                           int32_t max_positions, int32_t max_rows, void* hip_stream, rdlm_ctx** out) {
    return create_any(m, weight_ptrs, max_seqs, max_positions, max_rows, 0, hip_stream, nullptr, 0, out);
}

extern "C" int rdlm_create_paged(const rdlm_model* m, const void* const* weight_ptrs, int32_t max_seqs,
                                 int32_t max_positions, int32_t max_rows, int32_t kv_pool_positions, void* hip_stream,
                                 rdlm_ctx** out) {
    if (kv_pool_positions < 32) return RDLM_EINVAL;
    return create_any(m, weight_ptrs, max_seqs, max_positions, max_rows, kv_pool_positions, hip_stream, nullptr, 0, out);
}

// ---------------------------------------------------------------------------------------------
// paged KV cache: host-side block bookkeeping

static KvPages kv_pages(const rdlm_ctx* ctx) {
    KvPages kv;
    kv.table = ctx->blk_table;
    kv.stride = ctx->blocks_per_seq;
    kv.slots = ctx->max_seqs;
    return kv;
}

// Make sure the slot owns blocks for positions [0, n_positions).  New table entries are enqueued on the
// stream (a small kernel, entries by value), i.e. ordered before the kernels that use them.
static int ensure_blocks(rdlm_ctx* ctx, int seq, int n_positions) {
    const int need = (std::min(n_positions, ctx->ctx_pad) + 31) / 32;
    int have = ctx->seq_blocks[seq];
    if (need <= have) return RDLM_OK;
    if (need - have > (int)ctx->free_blocks.size()) return RDLM_ECAPACITY;     // pool exhausted: nothing taken
    while (have < need) {
        BlockIds ids;
        ids.n = 0;
        ids.first = seq * ctx->blocks_per_seq + have;
        while (have < need && ids.n < 16) {
            const int id = ctx->free_blocks.back();
            ctx->free_blocks.pop_back();
            ctx->tbl_host[(size_t)seq * ctx->blocks_per_seq + have] = id;
            ids.id[ids.n++] = id;
            ++have;
        }
        launch_table_set(ctx->blk_table, ids, ctx->st);
    }
    ctx->seq_blocks[seq] = have;
    return RDLM_OK;
}

static void release_blocks(rdlm_ctx* ctx, int seq) {
    for (int b = ctx->seq_blocks[seq] - 1; b >= 0; --b)
        ctx->free_blocks.push_back(ctx->tbl_host[(size_t)seq * ctx->blocks_per_seq + b]);
    ctx->seq_blocks[seq] = 0;
}

extern "C" int rdlm_kv_blocks(const rdlm_ctx* ctx, int32_t* total_out, int32_t* free_out) {
    if (!ctx) return RDLM_EINVAL;
    if (total_out) *total_out = ctx->kv_pool_blocks;
    if (free_out) *free_out = (int32_t)ctx->free_blocks.size();
    return RDLM_OK;
}

extern "C" int rdlm_seq_release(rdlm_ctx* ctx, int32_t seq) {
    if (!ctx || seq < 0) return RDLM_EINVAL;
    if (seq >= ctx->max_seqs) return RDLM_ECAPACITY;
    HIPCHK(hipStreamSynchronize(ctx->st));          // nothing in flight may still read the blocks
    if (ctx->sampler_on) {
        launch_seq_retire(ctx->seqs, seq, -1, ctx->st);         // frozen text stays readable
        launch_build_tiles_sampler(ctx->seqs, ctx->seq_ident, ctx->samp_seqs, ctx->max_positions, ctx->tiles_samp,
                                   ctx->n_tiles_samp, ctx->rows_pad, !ctx->knobs.no_pack, ctx->st);
    }
    release_blocks(ctx, seq);
    ctx->pos_bound[seq] = 0;
    return check_launch(ctx);
}

// ---------------------------------------------------------------------------------------------
// GEMM dispatch

// Launch shape of a projection for T row tiles: {row tiles per workgroup, feature blocks per
// workgroup (per wave for the row-sharing kernel), waves, k tiles fetched per batch, split of K
// across workgroups, kernel kind}.  The defaults come from sweeps on MI355X at the 3.5B shape;
// the knobs plan_<proj> and planr_<proj> override the one-tile and the several-tile case (tuning aids).
static GemmPlan plan_for(const rdlm_ctx* ctx, int proj, int N, int K, int T) {
    GemmPlan g;
    const bool split_ok = proj == PROJ_O || proj == PROJ_D || proj == PROJ_A;
    if (T == 1) {
        switch (proj) {
            // (alternating runs inside the sampler step, 3.5B shape: eight waves with one k tile per batch
            // beat four waves with two for gate/up by 0.7 us per launch, two waves with four for QKV by 0.8)
            case PROJ_GU: g = {1, 5, 8, 1, 1}; break;
            case PROJ_HEAD: g = {1, 4, 4, 2, 1}; break;
            case PROJ_QKV: g = {1, 2, 8, 1, 1}; break;
            default: g = {1, 2, 8, 1, 3}; break;       // O, D, A
        }
        if (ctx->knobs.has_plan[proj]) g = ctx->knobs.plan[proj];
    } else {
        // several row tiles: the row-sharing kernel.  Shapes from sweeps at 64..4096 rows.  While the
        // step is bound by weight streaming, small row chunks with many workgroups in flight win
        // (chunks of one feature group run back to back on one XCD and share the weights in its
        // L2); from a few hundred rows on, 256-row chunks feed the matrix cores.
        const bool wide = proj == PROJ_GU || proj == PROJ_HEAD;       // many feature blocks, no K split
        const bool deep = proj == PROJ_D || proj == PROJ_A;           // long K, few feature blocks
        // waves per workgroup of a projection without K split: the count (4, 5 or 8 feature blocks
        // per workgroup) that fills the 256 compute units most evenly, e.g. 5 for 1120 blocks
        auto even_waves = [&](int mt) {
            const int nblk = N / 32, chunks = (T + mt - 1) / mt;
            int best = 8;
            double best_u = 0.0;
            for (int w : {8, 5, 4}) {
                const int wgs = (nblk + w - 1) / w * chunks;
                const double u = (double)nblk * chunks / ((double)((wgs + 255) / 256 * 256) * w);
                if (u > best_u + 1e-9) { best_u = u; best = w; }
            }
            return best;
        };
        auto wide_plan = [&](int mt) {
            const int w = even_waves(mt);
            return GemmPlan{mt, 1, w, w == 5 ? 5 : 4, 1, GEMM_ROWS};
        };
        // Up to two row tiles (and four, where the accumulators still fit) the streaming kernel of
        // the one-tile step carries over: no barrier in its K loop, and a weight tile in registers
        // meets every row tile.
        if (T <= 2) {
            switch (proj) {
                case PROJ_GU: g = {2, 5, 4, 2, 1}; break;
                case PROJ_HEAD: g = {2, 4, 4, 2, 1}; break;
                case PROJ_QKV: g = {2, 2, 8, 1, 1}; break;
                case PROJ_A: g = GemmPlan{2, 1, 8, 4, 8, GEMM_ROWS}; break;
                default: g = {2, 2, 8, 1, 3}; break;       // O, D
            }
        } else if (T <= 4) {
            g = wide             ? wide_plan(4)
                : proj == PROJ_D ? GemmPlan{4, 2, 8, 1, 3}
                                 : GemmPlan{2, 1, 4, 4, deep ? 8 : 3, GEMM_ROWS};
        }
        else if (T <= 8)
            g = wide             ? GemmPlan{8, 1, 8, 2, 1, GEMM_ROWS}
                : proj == PROJ_A ? GemmPlan{4, 1, 4, 2, 8, GEMM_ROWS}
                                 : GemmPlan{2, 1, 8, 4, 3, GEMM_ROWS};
        else if (T <= 24)
            g = proj == PROJ_HEAD ? GemmPlan{8, 1, 8, 2, 1, GEMM_ROWS}
                : proj == PROJ_GU ? GemmPlan{4, 1, 4, 4, 1, GEMM_ROWS}
                : proj == PROJ_A  ? GemmPlan{4, 1, 4, 2, 4, GEMM_ROWS}
                                  : GemmPlan{4, 1, 8, 4, 3, GEMM_ROWS};
        else g = GemmPlan{8, 1, 8, 2, deep ? 3 : 2, GEMM_ROWS};
        // Three row tiles and more: where it measured faster (3.5B shape, 96 .. 4095 rows), the kernel
        // whose operands all go straight from global memory into an LDS ring (kernels_gemm_lds.hip):
        // {row tiles per workgroup, feature blocks per workgroup, waves, k tiles per stage, K split, kind, ring depth}.
        // Five blocks per workgroup give the gate/up projection 224 equal workgroups, eight the LM head 256.
        if (T >= 3 && !ctx->knobs.no_lds_gemm) {
            auto lds = [](int fb, int mtw, int wm, int ku, int d, int ks) { return GemmPlan{mtw * wm, fb, wm, ku, ks, GEMM_LDS, d}; };
            const int tier = T <= 4 ? 0 : T <= 8 ? 1 : T <= 16 ? 2 : T <= 32 ? 3 : 4;
            switch (proj) {
                case PROJ_GU:
                    g = tier == 0 ? lds(5, 1, 4, 2, 6, 1) : tier == 1 ? (T <= 6 ? lds(5, 2, 4, 2, 4, 1) : lds(5, 1, 8, 1, 8, 1))
                                                                      : lds(5, 2, 8, 1, 6, 1);
                    break;
                case PROJ_D:
                    if (tier == 0) g = lds(5, 1, 4, 2, 6, 7);
                    else if (tier == 1) g = lds(5, 2, 4, 2, 4, 7);
                    break;
                case PROJ_HEAD:
                    if (tier == 0) g = lds(8, 1, 4, 2, 6, 1);
                    else if (tier == 1 || tier == 3) g = lds(8, 1, 8, 1, 6, 1);
                    else if (tier == 2) g = lds(4, 2, 8, 1, 6, 1);
                    else if (tier == 4) g = lds(5, 2, 8, 1, 6, 1);
                    break;
                case PROJ_O:
                    if (tier == 3) g = lds(8, 1, 8, 1, 6, 3);
                    else if (tier == 4) g = lds(4, 2, 8, 1, 6, 2);
                    break;
                case PROJ_A:
                    if (tier == 1) g = lds(4, 1, 4, 2, 6, 3);
                    else if (tier == 2) g = lds(4, 1, 8, 1, 8, 3);
                    break;
                case PROJ_QKV:
                    if (tier == 0) g = lds(2, 1, 4, 2, 6, 1);
                    else if (tier == 1) g = lds(4, 1, 4, 2, 6, 1);
                    break;
                default: break;
            }
        }
        if (ctx->knobs.has_plan_rows[proj]) g = ctx->knobs.plan_rows[proj];
    }
    if (!split_ok) g.ksplit = 1;
    if (split_ok) {     // at least 4 k tiles per wave, at most 8 partial outputs
        int kmax = std::max(1, (K / 16) / ((g.kind == GEMM_STREAM ? g.waves : 1) * 4));
        g.ksplit = std::max(1, std::min(std::min(g.ksplit, 8), kmax));
    }
    return g;
}

struct SampleArgs {
    float temperature;
    uint32_t k0, k1;
    int step;
    bool want_logits;
    const int32_t* seq_step0 = nullptr;   // sampler: per-sequence step offsets (device)
    float top_p = 0.f;                    // in (0, 1): nucleus filter (needs temperature > 0)
};
static bool top_p_on(const SampleArgs* sa) { return sa && sa->temperature > 0.f && sa->top_p > 0.f && sa->top_p < 1.f; }

// One projection of the model path.  Output by projection:
//   QKV -> ctx->qkv (f32), O / D / A -> ctx->part ([S] partial sums, *S_out = S),
//   GU -> ctx->abuf (SwiGLU applied; bf16 path fuses it into the GEMM), HEAD -> ctx->drafts
//   (sampled tokens; logits in ctx->logits when asked for, always on the f32 path).
// fold (O, D, A on the one-tile bf16 path): the GEMM itself folds its split-K partial sums into
// the residual rows and prepares the next normalised operand (see GemmEpilogue::fold_counter);
// *folded tells whether it did, in which case no partial sums are pending (*S_out = 0).
struct FoldSpec {
    const float* xin;     // residual rows before the projection (null: none)
    float* xout;
    const float* gain;    // gain of the RMSNorm that follows
};
static int run_proj(rdlm_ctx* ctx, int proj, const void* xin, const void* W, int T, int* S_out,
                    const SampleArgs* sa = nullptr, bool plain = false, bool deferred_norm = false,
                    const Layer* rope_layer = nullptr, bool* rope_fused = nullptr, const FoldSpec* fold = nullptr,
                    bool* folded = nullptr) {
    const rdlm_model& m = ctx->m;
    const int h = m.hidden, F = m.mlp;
    int N, K;
    float* out;
    switch (proj) {
        case PROJ_QKV: N = 3 * h; K = h; out = ctx->qkv; break;
        case PROJ_O: N = h; K = h; out = ctx->part; break;
        case PROJ_GU: N = 2 * F; K = h; out = ctx->gu; break;
        case PROJ_D: N = h; K = F; out = ctx->part; break;
        case PROJ_A: N = h; K = 2 * h; out = ctx->part; break;
        default: N = m.vocab; K = h; out = ctx->logits; break;
    }
    if (S_out) *S_out = 1;
    if (m.dtype == RDLM_F32) {
        launch_gemm_f32(reinterpret_cast<const float*>(xin), reinterpret_cast<const float*>(W), out, N, K,
                        ctx->n_tiles, T, ctx->st);
        if (plain) return RDLM_OK;
        if (proj == PROJ_GU) launch_swiglu(ctx->gu, 1, 0, ctx->abuf, ctx->fmt, F, ctx->n_tiles, T, ctx->st);
        if (proj == PROJ_HEAD && top_p_on(sa))
            launch_sample_top_p(ctx->logits, m.vocab, sa->temperature, sa->top_p, sa->k0, sa->k1, sa->step,
                                sa->seq_step0, ctx->drafts, ctx->tiles, ctx->n_tiles, T, ctx->st);
        else if (proj == PROJ_HEAD && sa)
            launch_sample(ctx->logits, m.vocab, sa->temperature, sa->k0, sa->k1, sa->step, sa->seq_step0, ctx->drafts, ctx->tiles,
                          ctx->n_tiles, T, ctx->st);
        return RDLM_OK;
    }
    GemmPlan g = plan_for(ctx, proj, N, K, T);
    GemmEpilogue epi;
    epi.ssq_stride = ctx->rows_pad;
    epi.n_heads = m.n_heads; epi.head_dim = m.head_dim;
    if (proj == PROJ_GU) epi.layout = WL_GU16;
    if (proj == PROJ_QKV) epi.layout = WL_ROPE;
    if (!plain && proj == PROJ_GU) {
        epi.kind = EPI_SWIGLU;
        epi.act = ctx->abuf;
    } else if (!plain && proj == PROJ_QKV && rope_layer && !ctx->knobs.no_rope_fusion) {
        // RoPE and the cache writes happen in the GEMM epilogue
        epi.kind = EPI_ROPE_KV;
        epi.q_out = ctx->q; epi.kc = rope_layer->kc; epi.vc = rope_layer->vc; epi.rope_table = ctx->rope_tab;
        epi.kv = kv_pages(ctx);
        epi.tiles = ctx->tiles;
    } else if (!plain && proj == PROJ_HEAD && sa) {
        epi.kind = EPI_ARGMAX;
        epi.cand_val = ctx->cand_val; epi.cand_idx = ctx->cand_idx; epi.cand_stride = ctx->rows_pad;
        epi.temperature = sa->temperature; epi.k0 = sa->k0; epi.k1 = sa->k1; epi.step = sa->step;
        epi.seq_step0 = sa->seq_step0;
        epi.tiles = ctx->tiles;
        if (!sa->want_logits && !top_p_on(sa)) out = nullptr;      // the nucleus filter reads full logits
    }
    if (deferred_norm) {
        // ssq_count 0: a folding GEMM left the row totals in the last slot
        epi.row_ssq = ctx->ssq_count ? ctx->ssq : ctx->ssq + (size_t)SSQ_MAX_CHUNKS * ctx->rows_pad;
        epi.ssq_chunks = ctx->ssq_count ? ctx->ssq_count : 1; epi.norm_h = h; epi.norm_eps = m.rms_eps;
    }
    if (folded) *folded = false;
    // (one row tile only: folding two to four tiles of one workgroup tile after tile in the same
    // tail was measured -- 1115 -> 1123 tokens/s at a 64-row window, nothing at 128 rows -- and left out)
    const bool do_fold = fold && !plain && T == 1 && epi.kind == EPI_F32 && g.kind == GEMM_STREAM && g.mt == 1 &&
                         (g.nb == 1 || g.nb == 2 || g.nb == 4) && gemm_groups(N, g, EPI_F32) <= SSQ_MAX_CHUNKS &&
                         // partial sums in accumulator order cover whole feature groups: they must fit
                         (size_t)g.ksplit * T * 32 * gemm_groups(N, g, EPI_F32) * g.nb * 32 <=
                             (size_t)8 * ctx->rows_pad * h &&
                         !ctx->knobs.no_fold_fusion;
    if (do_fold) {
        epi.fold_counter = ctx->fold_counter; epi.fold_xin = fold->xin; epi.fold_xout = fold->xout;
        epi.fold_gain = fold->gain; epi.fold_xg = ctx->xn; epi.fold_ssq = ctx->ssq;
    }
    const bool prof = ctx->prof_n == N && ctx->prof_k == K && (size_t)ctx->prof_used + 2 <= ctx->prof_ev.size();
    if (prof) (void)hipEventRecord(ctx->prof_ev[ctx->prof_used++], ctx->st);
    bool ok = launch_gemm_bf16(xin, W, out, N, K, (size_t)ctx->rows_pad * N, g, epi, ctx->n_tiles, T, ctx->st);
    if (rope_fused) *rope_fused = ok && epi.kind == EPI_ROPE_KV;
    if (!ok && epi.kind == EPI_ROPE_KV) {      // no fused instance: plain projection, the caller runs the RoPE kernel
        epi.kind = EPI_F32;
        g = plan_for(ctx, proj, N, K, T);
        ok = launch_gemm_bf16(xin, W, out, N, K, (size_t)ctx->rows_pad * N, g, epi, ctx->n_tiles, T, ctx->st);
    }
    if (!ok) {      // no instance for this plan: the plain one-block kernel always exists
        if (g.kind == GEMM_LDS) g = {4, 1, 4, 4, 1, GEMM_ROWS};     // (the row-sharing kernel's plain instance)
        else if (g.mt > 1) {
            g = {g.mt, 1, 4, g.mt == 2 ? 8 : 4, 1, GEMM_ROWS};
            epi.fold_counter = nullptr;         // the row-sharing kernel leaves plain partial sums
        }
        else g = {1, 1, 4, 4, g.ksplit};
        ok = launch_gemm_bf16(xin, W, out, N, K, (size_t)ctx->rows_pad * N, g, epi, ctx->n_tiles, T, ctx->st);
        if (!ok) {
            fprintf(stderr, "rdlm: no GEMM kernel instance for plan {%d,%d,%d,%d} epilogue %d\n", g.mt, g.nb, g.waves,
                    g.unroll, epi.kind);
            return RDLM_EINVAL;
        }
    }
    if (prof) (void)hipEventRecord(ctx->prof_ev[ctx->prof_used++], ctx->st);
    if (epi.kind == EPI_ARGMAX && top_p_on(sa))
        launch_sample_top_p(ctx->logits, m.vocab, sa->temperature, sa->top_p, sa->k0, sa->k1, sa->step, sa->seq_step0,
                            ctx->drafts, ctx->tiles, ctx->n_tiles, T, ctx->st);
    else if (epi.kind == EPI_ARGMAX)
        launch_argmax_final(ctx->cand_val, ctx->cand_idx, gemm_groups(N, g, EPI_ARGMAX), ctx->rows_pad, ctx->drafts,
                            ctx->n_tiles, T, ctx->st);
    if (S_out) *S_out = g.ksplit;
    if (do_fold && epi.fold_counter) {      // (a fallback plan above would have dropped the fold with the epilogue)
        ctx->ssq_count = 0;
        if (S_out) *S_out = 0;
        if (folded) *folded = true;
    }
    return RDLM_OK;
}

// Sequences with several row tiles: the grouped kernel reads every K/V block once for up to four row tiles,
// but its workgroups walk their key blocks one after the other; the one-tile kernel, launched per segment,
// reads the blocks once per tile with four waves on different blocks.  Below about ATT_GROUP_KEYS
// (row tiles of a sequence x visible keys, i.e. the K/V traffic the per-segment launch spends on one
// sequence) the second is faster, whatever the number of sequences in the step.
constexpr long long ATT_GROUP_KEYS = 7000;
static bool att_grouped_for(const rdlm_ctx* ctx, int max_keys) {
    if (!ctx->grouped || ctx->m.dtype == RDLM_F32) return ctx->grouped;
    const long long lim = ctx->knobs.att_group_keys >= 0 ? ctx->knobs.att_group_keys : ATT_GROUP_KEYS;
    return (long long)ctx->seq_tiles_max * max_keys > lim;
}

static int att_split_for(const rdlm_ctx* ctx, int T, int max_keys, bool grouped) {
    if (ctx->m.dtype == RDLM_F32) return 1;
    if (ctx->knobs.att_split > 0) return std::min(ctx->knobs.att_split, ctx->att_max_split);
    int wgs = ctx->m.n_heads * (grouped ? (T + ATT_GROUP - 1) / ATT_GROUP : T);
    int kb = (max_keys + 31) / 32;
    if (T == 1) {
        // one tile: n_heads workgroups per split.  Measured at 55 heads x 96: four splits pay from
        // about 1500 keys on, eight not before 6000
        int s1 = kb >= 512 ? 8 : kb >= 48 ? 4 : kb >= 32 ? 2 : 1;
        return std::min(s1, ctx->att_max_split);
    }
    int s = 1;
    while (s < ctx->att_max_split && wgs * s < 512 && kb / (s * 2) >= 16) s *= 2;
    return s;
}

// x_out = x_in + pending partial sums, and the normalised GEMM operand of it.  bf16 path: the
// 1/rms factor is left to the consuming GEMM's epilogue (returns true); f32 path: full RMSNorm.
static bool norm_operand(rdlm_ctx* ctx, const float* xin, float* xout, int S, const float* gain, void* xn, int T) {
    const rdlm_model& m = ctx->m;
    const size_t pst = (size_t)ctx->rows_pad * m.hidden;
    if (m.dtype == RDLM_BF16 && fold_chunks(m.hidden) > 0 && !ctx->knobs.no_fold) {
        launch_fold(xin, xout, ctx->part, S, pst, gain, xn, ctx->ssq, ctx->rows_pad, m.hidden, ctx->n_tiles, T, ctx->st);
        ctx->ssq_count = fold_chunks(m.hidden);
        return true;
    }
    launch_addnorm(xin, xout, ctx->part, S, pst, gain, xn, ctx->fmt, m.hidden, m.rms_eps, ctx->n_tiles, T, ctx->st);
    return false;
}

// One transformer layer over the current tiles.  On entry the residual stream is
// x (+ the S_in partial sums in part, if any) -- or, with xn_ready, x is complete and its
// normalised operand (gain g1) is already in xn.  On exit it is x + the *S_out partials in part;
// with next_gain the down projection may fold them itself and prepare the operand of the norm with
// that gain (*next_ready).
#define PROPAGATE(call)                 \
    do {                                \
        int rc__ = (call);              \
        if (rc__ != RDLM_OK) return rc__; \
    } while (0)

static int layer_forward(rdlm_ctx* ctx, const Layer& L, int T, int max_keys, bool x_valid, int S_in, int* S_out,
                         bool xn_ready = false, const float* next_gain = nullptr, bool* next_ready = nullptr) {
    const rdlm_model& m = ctx->m;
    const int h = m.hidden;
    hipStream_t st = ctx->st;
    int S;
    bool dn = true;
    if (!xn_ready) dn = norm_operand(ctx, x_valid ? ctx->x : nullptr, ctx->x, S_in, L.g1, ctx->xn, T);
    bool rope_done = false;
    PROPAGATE(run_proj(ctx, PROJ_QKV, ctx->xn, L.wqkv, T, &S, nullptr, false, dn, &L, &rope_done));
    if (!rope_done)
        launch_rope_kv(ctx->qkv, 1, 0, ctx->q, L.kc, L.vc, m.dtype, m.n_heads, m.head_dim, ctx->rope_tab,
                       kv_pages(ctx), ctx->tiles, ctx->n_tiles, T, st);
    const int segs = ctx->seg_tiles > 0 ? ctx->seg_tiles : T;      // attention works on segments, not on row tiles
    const bool grouped = att_grouped_for(ctx, max_keys);
    launch_attention(ctx->q, L.kc, L.vc, ctx->att, m.dtype, m.n_heads, m.head_dim, kv_pages(ctx),
                     att_split_for(ctx, segs, max_keys, grouped), grouped, ctx->att_ws, ctx->att_tickets, ctx->tiles,
                     ctx->rows_pad, ctx->n_tiles, segs, st, ctx->att_groups);
    const FoldSpec fo = {ctx->x, ctx->x, L.g2};
    bool folded = false;
    PROPAGATE(run_proj(ctx, PROJ_O, ctx->att, L.wo, T, &S, nullptr, false, false, nullptr, nullptr, &fo, &folded));
    dn = folded ? true : norm_operand(ctx, ctx->x, ctx->x, S, L.g2, ctx->xn, T);
    PROPAGATE(run_proj(ctx, PROJ_GU, ctx->xn, L.wgu, T, &S, nullptr, false, dn));   // leaves silu(gate) * up in abuf
    const FoldSpec fd = {ctx->x, ctx->x, next_gain};
    folded = false;
    PROPAGATE(run_proj(ctx, PROJ_D, ctx->abuf, L.wd, T, S_out, nullptr, false, false, nullptr, nullptr,
                       next_gain ? &fd : nullptr, &folded));
    if (next_ready) *next_ready = folded;
    return RDLM_OK;
}

// e = P(tokens): embedding gather (scaled) and the prelude layers; result in e_out rows (erow0).
// With z_cat (bf16 path, internal e buffer): the closing pass also writes the adapter operand
// concat(e, z) for the recurrence that follows, and the function returns true.
static int prelude_forward(rdlm_ctx* ctx, const int32_t* tokens, float* e_out, int e_which, int T, int max_keys,
                           const float* z_cat = nullptr, bool* cat_ready = nullptr) {
    if (cat_ready) *cat_ready = false;
    const rdlm_model& m = ctx->m;
    // the gather also writes the RoPE table of the step's rows and, on the bf16 path, the operand
    // of the first layer's norm
    const bool prep = m.dtype == RDLM_BF16 && m.n_prelude > 0 && fold_chunks(m.hidden) > 0 && !ctx->knobs.no_fold;
    launch_embed(ctx->emb_canon, m.dtype, tokens, m.emb_scale, ctx->x, m.hidden, m.vocab, ctx->rope_tab, ctx->theta,
                 m.head_dim / 2, prep ? ctx->layers[0].g1 : nullptr, prep ? ctx->xn : nullptr, ctx->ssq, ctx->rows_pad,
                 ctx->tiles, ctx->n_tiles, T, ctx->st);
    int S = 0;
    bool ready = prep;
    if (prep) ctx->ssq_count = fold_chunks(m.hidden);
    for (int l = 0; l < m.n_prelude; ++l)
        PROPAGATE(layer_forward(ctx, ctx->layers[l], T, max_keys, true, S, &S, ready,
                                l + 1 < m.n_prelude ? ctx->layers[l + 1].g1 : nullptr, &ready));
    const size_t pst = (size_t)ctx->rows_pad * m.hidden;
    if (z_cat && e_which < 0 && m.dtype == RDLM_BF16 && fold_chunks(m.hidden) > 0 && !ctx->knobs.no_fold) {
        launch_prelude_end(ctx->x, ctx->part, S, pst, e_out, z_cat, ctx->abuf, ctx->hoist_split ? ctx->att : nullptr,
                           m.hidden, ctx->tiles, ctx->n_tiles, T, ctx->st);
        if (cat_ready) *cat_ready = true;
        return RDLM_OK;
    }
    // fold the pending partial sums: x <- x + sum part (no norm output needed)
    launch_addnorm(ctx->x, ctx->x, ctx->part, S, pst, ctx->gf, nullptr, ctx->fmt, m.hidden, m.rms_eps, ctx->n_tiles, T,
                   ctx->st);
    if (e_out != ctx->x) {
        if (e_which < 0)   // internal e buffer is indexed by padded row: plain copy
            (void)hipMemcpyAsync(e_out, ctx->x, (size_t)T * 32 * m.hidden * 4, hipMemcpyDeviceToDevice, ctx->st);
        else
            launch_copy_rows_out(ctx->x, e_out, m.hidden, e_which, ctx->tiles, ctx->n_tiles, T, ctx->st);
    }
    return RDLM_OK;
}

// z <- R(z, e): adapter on concat(e, z), the core layers, closing norm; optional delta vs z_prev.
// cat_ready: the adapter operand was already written (by the prelude's closing pass); x_for_coda:
// also leave z' in the residual buffer, where the coda starts from.
//
// hoist (several recurrences on the same e; Sec. 3.2: e is computed once, only s changes between
// recurrences): W_a . [e; z] = W_e . e + W_z . z, and the first term is the same every time.
// 1 = first recurrence: compute W_e . e into ctx->xe, then add W_z . z; 2 = a later one: reuse ctx->xe.
// Both halves are [h, h] products, i.e. they run with the output projection's launch shapes.
static bool hoist_ok(const rdlm_ctx* ctx, int n_recurrences) {
    return n_recurrences > 1 && ctx->m.dtype == RDLM_BF16 && !ctx->knobs.no_hoist;
}
static int core_forward(rdlm_ctx* ctx, const float* e, float* z, float* z_prev, int update_prev, float* delta,
                        int T, int max_keys, bool cat_ready = false, bool x_for_coda = false, int hoist = 0) {
    const rdlm_model& m = ctx->m;
    const int h = m.hidden;
    const float* g1 = ctx->layers[m.n_prelude].g1;
    int S;
    bool ready = false;
    bool x_valid;
    if (hoist) {
        if (hoist == 1) {
            if (!cat_ready) launch_concat(e, nullptr, ctx->att, ctx->fmt, h, ctx->tiles, ctx->n_tiles, T, ctx->st);
            const FoldSpec fe = {nullptr, ctx->xe, g1};
            PROPAGATE(run_proj(ctx, PROJ_O, ctx->att, ctx->wa_e, T, &S, nullptr, false, false, nullptr, nullptr, &fe, &ready));
            if (!ready) norm_operand(ctx, nullptr, ctx->xe, S, g1, ctx->xn, T);
        }
        if (!(cat_ready && hoist == 1)) launch_concat(nullptr, z, ctx->abuf, ctx->fmt, h, ctx->tiles, ctx->n_tiles, T, ctx->st);
        const FoldSpec fz = {ctx->xe, ctx->x, g1};
        ready = false;
        PROPAGATE(run_proj(ctx, PROJ_O, ctx->abuf, ctx->wa_z, T, &S, nullptr, false, false, nullptr, nullptr, &fz, &ready));
        if (!ready) {        // partial sums pending: x = xe + their sum; the first layer's operand is ready
            ready = norm_operand(ctx, ctx->xe, ctx->x, S, g1, ctx->xn, T);   // only on the deferred-norm path
            S = 0;
        }
        x_valid = true;
    } else {
        if (!cat_ready) launch_concat(e, z, ctx->abuf, ctx->fmt, h, ctx->tiles, ctx->n_tiles, T, ctx->st);
        const FoldSpec fa = {nullptr, ctx->x, g1};
        PROPAGATE(run_proj(ctx, PROJ_A, ctx->abuf, ctx->wa, T, &S, nullptr, false, false, nullptr, nullptr, &fa, &ready));
        x_valid = ready;
    }
    for (int l = 0; l < m.n_core; ++l) {
        PROPAGATE(layer_forward(ctx, ctx->layers[m.n_prelude + l], T, max_keys, x_valid, S, &S, ready,
                                l + 1 < m.n_core ? ctx->layers[m.n_prelude + l + 1].g1 : nullptr, &ready));
        x_valid = true;
    }
    // before the coda: also leave z' in the residual buffer and, on the bf16 path, the operand of the
    // coda's first norm with the row totals of z'^2
    const bool prep = x_for_coda && m.dtype == RDLM_BF16 && m.n_coda > 0 && !ctx->knobs.no_fold;
    launch_final_norm(ctx->x, ctx->part, S, (size_t)ctx->rows_pad * h, ctx->gf, h, m.rms_eps, z, z_prev, update_prev,
                      delta, x_for_coda ? ctx->x : nullptr, prep ? ctx->layers[m.n_prelude + m.n_core].g1 : nullptr,
                      prep ? ctx->xn : nullptr, ctx->ssq + (size_t)SSQ_MAX_CHUNKS * ctx->rows_pad, ctx->tiles,
                      ctx->n_tiles, T, ctx->st);
    if (prep) ctx->ssq_count = 0;
    ctx->coda_ready = prep;
    return RDLM_OK;
}

// C: coda layers on z; with sa: final norm, tied LM head and Sample -> ctx->drafts (+ logits).
static int coda_forward(rdlm_ctx* ctx, const float* z, const SampleArgs* sa, int T, int max_keys,
                        bool x_ready = false) {
    const rdlm_model& m = ctx->m;
    const int h = m.hidden;
    if (!x_ready) launch_copy_rows_in(z, ctx->x, h, 0, ctx->tiles, ctx->n_tiles, T, ctx->st);
    int S = 0;
    bool ready = x_ready && ctx->coda_ready;
    ctx->coda_ready = false;
    const int l0 = m.n_prelude + m.n_core;
    for (int l = 0; l < m.n_coda; ++l)
        PROPAGATE(layer_forward(ctx, ctx->layers[l0 + l], T, max_keys, true, S, &S, ready,
                                l + 1 < m.n_coda ? ctx->layers[l0 + l + 1].g1 : (sa ? ctx->gout : nullptr), &ready));
    if (!sa) return RDLM_OK;
    bool dn = ready ? true : norm_operand(ctx, ctx->x, nullptr, S, ctx->gout, ctx->xn, T);
    return run_proj(ctx, PROJ_HEAD, ctx->xn, ctx->emb_w, T, nullptr, sa, false, dn);
}

// ---------------------------------------------------------------------------------------------
// argument checking shared by the row-based calls

// Row tiles that windows of the given sizes take, laid out in order: a window of more than 32 rows gets
// whole tiles; shorter ones are packed into the tile that is open as long as they fit.
static int phys_tiles(const int32_t* rows, int n, bool pack) {
    int np = 0, cap = 0;
    for (int i = 0; i < n; ++i) {
        const int r = rows[i];
        if (r <= 0) continue;
        const bool small = pack && r <= TILE_ROWS;
        if (small && cap >= r) { cap -= r; continue; }
        np += (r + TILE_ROWS - 1) / TILE_ROWS;
        cap = small ? TILE_ROWS - r : 0;
    }
    return np;
}

static int check_rows(rdlm_ctx* ctx, int n_seqs, const int32_t* seq_ids, const int32_t* pos0,
                      const int32_t* n_rows, SeqWindows* w, int* T, int* M, int* max_keys) {
    if (!ctx || !seq_ids || !pos0 || !n_rows || n_seqs < 1) return RDLM_EINVAL;
    if (n_seqs > MAX_API_SEQS) return RDLM_ECAPACITY;
    int tiles = 0, rows = 0, mk = 0;
    w->n = n_seqs;
    for (int i = 0; i < n_seqs; ++i) {
        if (seq_ids[i] < 0 || pos0[i] < 0 || n_rows[i] < 1) return RDLM_EINVAL;
        if (seq_ids[i] >= ctx->max_seqs) return RDLM_ECAPACITY;
        if ((long long)pos0[i] + n_rows[i] > ctx->max_positions) return RDLM_ECAPACITY;
        for (int j = 0; j < i; ++j)
            if (seq_ids[j] == seq_ids[i]) return RDLM_EINVAL;      // one window per sequence per step
        w->seq[i] = seq_ids[i]; w->pos0[i] = pos0[i]; w->rows[i] = n_rows[i];
        tiles += (n_rows[i] + 31) / 32;
        rows += n_rows[i];
        mk = std::max(mk, pos0[i] + n_rows[i]);
    }
    if (rows > ctx->max_rows || tiles > ctx->max_tiles) return RDLM_ECAPACITY;
    // row tiles of the step: windows of up to 32 rows share row tiles (the layout of TileLayout::add)
    *T = phys_tiles(n_rows, n_seqs, !ctx->knobs.no_pack);
    ctx->seg_tiles = tiles;
    *M = rows; *max_keys = mk;
    bool grouped = false;
    ctx->seq_tiles_max = 1;
    for (int i = 0; i < n_seqs; ++i) {
        grouped = grouped || n_rows[i] > TILE_ROWS;
        ctx->seq_tiles_max = std::max(ctx->seq_tiles_max, (n_rows[i] + 31) / 32);
    }
    ctx->grouped = grouped;
    ctx->att_groups = 0;
    for (int i = 0; i < n_seqs; ++i) ctx->att_groups += ((n_rows[i] + 31) / 32 + ATT_GROUP - 1) / ATT_GROUP;
    // cache blocks for the rows' positions (the rows attend to everything before them: blocks from 0 on)
    int need = 0;
    for (int i = 0; i < n_seqs; ++i)
        need += std::max(0, (pos0[i] + n_rows[i] + 31) / 32 - ctx->seq_blocks[seq_ids[i]]);
    if (need > (int)ctx->free_blocks.size()) return RDLM_ECAPACITY;
    for (int i = 0; i < n_seqs; ++i) {
        int rc = ensure_blocks(ctx, seq_ids[i], pos0[i] + n_rows[i]);
        if (rc) return rc;
    }
    return RDLM_OK;
}

extern "C" int rdlm_set_tokens(rdlm_ctx* ctx, int32_t seq, const int32_t* tokens_host, int32_t n) {
    if (!ctx || !tokens_host || n < 1 || seq < 0) return RDLM_EINVAL;
    if (seq >= ctx->max_seqs || n >= ctx->max_positions) return RDLM_ECAPACITY;
    for (int i = 0; i < n; ++i)
        if (tokens_host[i] < 0 || tokens_host[i] >= ctx->m.vocab) return RDLM_EINVAL;
    HIPCHK(hipStreamSynchronize(ctx->st));
    size_t base = (size_t)seq * ctx->max_positions;
    launch_fill_i32(ctx->y + base, 0, ctx->max_positions, ctx->st);
    launch_fill_i32(ctx->counts + base, 0, ctx->max_positions, ctx->st);
    HIPCHK(hipStreamSynchronize(ctx->st));
    HIPCHK(hipMemcpy(ctx->y + base, tokens_host, (size_t)n * 4, hipMemcpyHostToDevice));
    ctx->prompt_len[seq] = n;
    ctx->pos_bound[seq] = 0;
    ctx->ident_host[seq] = seq;         // a slot that starts over is its own sequence again
    launch_fill_i32(ctx->seq_ident + seq, seq, 1, ctx->st);
    if (ctx->sampler_on) {          // the slot leaves the running sampler until it joins again
        launch_seq_retire(ctx->seqs, seq, n, ctx->st);
        launch_build_tiles_sampler(ctx->seqs, ctx->seq_ident, ctx->samp_seqs, ctx->max_positions, ctx->tiles_samp, ctx->n_tiles_samp, ctx->rows_pad, !ctx->knobs.no_pack,
                                   ctx->st);
    }
    return check_launch(ctx);
}

extern "C" int rdlm_prefill(rdlm_ctx* ctx, int32_t seq, int32_t n, int32_t r, float alpha, uint64_t seed) {
    if (!ctx || seq < 0 || n < 0 || r < 0) return RDLM_EINVAL;
    if (seq >= ctx->max_seqs || n > ctx->max_rows || n > ctx->max_positions) return RDLM_ECAPACITY;
    if (n == 0) return RDLM_OK;
    PROPAGATE(ensure_blocks(ctx, seq, n));
    SeqWindows w;
    w.n = 1; w.seq[0] = seq; w.pos0[0] = 0; w.rows[0] = n;
    const int T = (n + 31) / 32;
    ctx->grouped = T > 1;
    ctx->seq_tiles_max = T;
    ctx->seg_tiles = T;
    ctx->att_groups = (T + ATT_GROUP - 1) / ATT_GROUP;
    launch_build_tiles_store(w, ctx->seq_ident, ctx->max_positions, ctx->tiles, ctx->n_tiles, ctx->rows_pad, !ctx->knobs.no_pack, ctx->st);
    launch_init_state_rows(ctx->z_store, nullptr, ctx->m.hidden, ctx->ident_host[seq], 0, n,
                           (size_t)seq * ctx->max_positions, alpha, (uint32_t)seed, (uint32_t)(seed >> 32), ctx->st);
    PROPAGATE(prelude_forward(ctx, ctx->y, ctx->e, -1, T, n));
    for (int i = 0; i < r; ++i)
        PROPAGATE(core_forward(ctx, ctx->e, ctx->z_store, nullptr, 0, nullptr, T, n, false, false,
                               hoist_ok(ctx, r) ? (i == 0 ? 1 : 2) : 0));
    PROPAGATE(coda_forward(ctx, ctx->z_store, nullptr, T, n));
    return check_launch(ctx);
}

extern "C" int rdlm_init_state(rdlm_ctx* ctx, int32_t seq, int32_t pos0, int32_t n, float alpha, uint64_t seed,
                               float* z_out) {
    if (!ctx || !z_out || seq < 0 || pos0 < 0 || n < 0) return RDLM_EINVAL;
    launch_init_state_rows(z_out, nullptr, ctx->m.hidden, seq, pos0, n, 0, alpha, (uint32_t)seed,
                           (uint32_t)(seed >> 32), ctx->st);
    return check_launch(ctx);
}

extern "C" int rdlm_prelude(rdlm_ctx* ctx, int32_t n_seqs, const int32_t* seq_ids, const int32_t* pos0,
                            const int32_t* n_rows, const int32_t* tokens_dev, float* e_out) {
    SeqWindows w;
    int T, M, mk;
    if (!tokens_dev || !e_out) return RDLM_EINVAL;
    int rc = check_rows(ctx, n_seqs, seq_ids, pos0, n_rows, &w, &T, &M, &mk);
    if (rc) return rc;
    launch_build_tiles_api(w, ctx->seq_ident, ctx->tiles, ctx->n_tiles, ctx->rows_pad, !ctx->knobs.no_pack, ctx->st);
    PROPAGATE(prelude_forward(ctx, tokens_dev, e_out, 1, T, mk));
    return check_launch(ctx);
}

// the body of rdlm_core_step over whatever workspace the context currently points at
static int core_step_run(rdlm_ctx* ctx, const SeqWindows& w, int T, int M, int mk, const float* e, float* z_inout,
                         int r_inner, float* delta_out) {
    launch_build_tiles_api(w, ctx->seq_ident, ctx->tiles, ctx->n_tiles, ctx->rows_pad, !ctx->knobs.no_pack, ctx->st);
    launch_rope_table(ctx->rope_tab, ctx->theta, ctx->m.head_dim / 2, ctx->tiles, ctx->n_tiles, T, ctx->st);
    if (delta_out)
        HIPCHK(hipMemcpyAsync(ctx->zp_api, z_inout, (size_t)M * ctx->m.hidden * 4, hipMemcpyDeviceToDevice, ctx->st));
    for (int i = 0; i < r_inner; ++i) {
        bool last = i == r_inner - 1;
        PROPAGATE(core_forward(ctx, e, z_inout, (last && delta_out) ? ctx->zp_api : nullptr, 0,
                               (last && delta_out) ? ctx->delta : nullptr, T, mk, false, false,
                               hoist_ok(ctx, r_inner) ? (i == 0 ? 1 : 2) : 0));
    }
    if (delta_out) launch_copy_rows_out(ctx->delta, delta_out, 1, 2, ctx->tiles, ctx->n_tiles, T, ctx->st);
    return check_launch(ctx);
}

extern "C" int rdlm_core_step(rdlm_ctx* ctx, int32_t n_seqs, const int32_t* seq_ids, const int32_t* pos0,
                              const int32_t* n_rows, const float* e, float* z_inout, int32_t r_inner,
                              float* delta_out) {
    SeqWindows w;
    int T, M, mk;
    if (!e || !z_inout || r_inner < 1) return RDLM_EINVAL;
    int rc = check_rows(ctx, n_seqs, seq_ids, pos0, n_rows, &w, &T, &M, &mk);
    if (rc) return rc;
    return core_step_run(ctx, w, T, M, mk, e, z_inout, r_inner, delta_out);
}

extern "C" size_t rdlm_core_step_static_bytes(const rdlm_ctx* ctx, int32_t n_tiles) {
    if (!ctx || n_tiles < 1) return 0;
    return carve_workspace(nullptr, nullptr, ctx->m, n_tiles, ctx->att_max_split, false);
}

extern "C" int rdlm_core_step_static(rdlm_ctx* ctx, int32_t n_seqs, const int32_t* seq_ids, const int32_t* pos0,
                                     const int32_t* n_rows, const float* e, float* z_inout, int32_t r_inner,
                                     float* delta_out) {
    if (!ctx || !e || !z_inout || r_inner < 1 || !seq_ids || !pos0 || !n_rows || n_seqs < 1) return RDLM_EINVAL;
    if (n_seqs > MAX_API_SEQS) return RDLM_ECAPACITY;
    // capacity is what fits the static array, not what the context was created for
    int tiles = 0;
    for (int i = 0; i < n_seqs; ++i) {
        if (n_rows[i] < 1) return RDLM_EINVAL;
        tiles += (n_rows[i] + 31) / 32;
    }
    const size_t need = carve_workspace(nullptr, nullptr, ctx->m, tiles, ctx->att_max_split, false);
    if (need > STATIC_SCRATCH_BYTES) {
        fprintf(stderr, "rdlm_core_step_static: %d row tiles of this model need %zu bytes of scratch, the static "
                        "array holds %zu\n", tiles, need, STATIC_SCRATCH_BYTES);
        return RDLM_ECAPACITY;
    }
    void* sp = nullptr;
    int rc = static_scratch_for(nullptr, &sp);      // looked up by rdlm_create on this device; a table read here
    if (rc) return rc;
    // the context's workspace steps aside for the length of this call
    const Workspace own = *ctx;
    const int own_rows = ctx->max_rows;
    carve_workspace(ctx, sp, ctx->m, tiles, ctx->att_max_split, false);
    ctx->max_rows = tiles * 32;
    SeqWindows w;
    int T, M, mk;
    rc = check_rows(ctx, n_seqs, seq_ids, pos0, n_rows, &w, &T, &M, &mk);
    if (rc == RDLM_OK) {
        // the array keeps whatever the last call (of any context) left: the ticket words must read zero
        launch_fill_i32(reinterpret_cast<int32_t*>(ctx->ticket_lo), 0, ctx->ticket_bytes / 4, ctx->st);
        rc = core_step_run(ctx, w, T, M, mk, e, z_inout, r_inner, delta_out);
    }
    static_cast<Workspace&>(*ctx) = own;
    ctx->max_rows = own_rows;
    return rc;
}

extern "C" int rdlm_coda_decode(rdlm_ctx* ctx, int32_t n_seqs, const int32_t* seq_ids, const int32_t* pos0,
                                const int32_t* n_rows, const float* z, float temperature, uint64_t seed,
                                int32_t step, int32_t* tokens_out, float* logits_out, float top_p) {
    SeqWindows w;
    int T, M, mk;
    if (!z || !tokens_out || !(temperature >= 0.f) || step < 0 || !(top_p >= 0.f)) return RDLM_EINVAL;
    if (ctx && top_p > 0.f && top_p < 1.f && (ctx->m.vocab > TOPP_MAX_VOCAB || ctx->m.vocab % 4)) return RDLM_EINVAL;
    int rc = check_rows(ctx, n_seqs, seq_ids, pos0, n_rows, &w, &T, &M, &mk);
    if (rc) return rc;
    launch_build_tiles_api(w, ctx->seq_ident, ctx->tiles, ctx->n_tiles, ctx->rows_pad, !ctx->knobs.no_pack, ctx->st);
    launch_rope_table(ctx->rope_tab, ctx->theta, ctx->m.head_dim / 2, ctx->tiles, ctx->n_tiles, T, ctx->st);
    SampleArgs sa = {temperature, (uint32_t)seed, (uint32_t)(seed >> 32), step, logits_out != nullptr, nullptr, top_p};
    PROPAGATE(coda_forward(ctx, z, &sa, T, mk));
    launch_copy_i32_out(ctx->drafts, tokens_out, ctx->tiles, ctx->n_tiles, T, ctx->st);
    if (logits_out) launch_copy_rows_out(ctx->logits, logits_out, ctx->m.vocab, 2, ctx->tiles, ctx->n_tiles, T, ctx->st);
    return check_launch(ctx);
}

// ---------------------------------------------------------------------------------------------
// sampler driver

extern "C" int rdlm_sampler_begin(rdlm_ctx* ctx, const rdlm_sampler* s, int32_t n_seqs) {
    if (!ctx || !s || n_seqs < 1) return RDLM_EINVAL;
    if (n_seqs > ctx->max_seqs) return RDLM_ECAPACITY;
    if (s->n_new < 1 || s->r_inner < 1 || s->r_total < 1 || s->headway < 1 || !(s->temperature >= 0.f) ||
        !(s->eps >= 0.f) || s->pad_token < 0 || s->pad_token >= ctx->m.vocab || !(s->beta >= 0.f && s->beta <= 1.f) ||
        !(s->eta >= 0.f && s->eta < 1.f) || !(s->top_p >= 0.f) || (s->init_mode != 0 && s->init_mode != 1))
        return RDLM_EINVAL;
    if (s->top_p > 0.f && s->top_p < 1.f && (ctx->m.vocab > TOPP_MAX_VOCAB || ctx->m.vocab % 4)) return RDLM_EINVAL;
    rdlm_sampler sp = *s;
    const int wave = (sp.r_total + sp.r_inner - 1) / sp.r_inner;
    if (sp.w_max <= 0 || !sp.adaptive) sp.w_max = wave * sp.headway;
    int tiles = n_seqs * ((sp.w_max + 31) / 32);
    if (tiles > ctx->max_tiles || n_seqs * sp.w_max > ctx->max_rows) return RDLM_ECAPACITY;
    for (int q = 0; q < n_seqs; ++q) {
        if (ctx->prompt_len[q] < 1) return RDLM_ESTATE;
        if ((long long)ctx->prompt_len[q] + sp.n_new + sp.w_max + sp.headway + 1 > ctx->max_positions) return RDLM_ECAPACITY;
    }
    for (int q = 0; q < n_seqs; ++q) {                  // the first state sits at position L - 1
        PROPAGATE(ensure_blocks(ctx, q, ctx->prompt_len[q]));
        ctx->pos_bound[q] = ctx->prompt_len[q];
    }
    HIPCHK(hipStreamSynchronize(ctx->st));
    std::vector<SeqState> hs(ctx->max_seqs);            // slots beyond n_seqs: finished, no rows
    memset(hs.data(), 0, sizeof(SeqState) * ctx->max_seqs);
    for (int q = n_seqs; q < ctx->max_seqs; ++q) { hs[q].done = 1; ctx->pos_bound[q] = 0; }
    for (int q = 0; q < n_seqs; ++q) {
        const int L = ctx->prompt_len[q];
        hs[q].prompt_len = L; hs[q].n_frozen = L; hs[q].win_pos0 = L - 1; hs[q].win_n = 1;
        size_t base = (size_t)q * ctx->max_positions;
        launch_fill_i32(ctx->y + base + L, sp.pad_token, ctx->max_positions - L, ctx->st);
        launch_fill_i32(ctx->counts + base, 0, ctx->max_positions, ctx->st);
        launch_init_state_rows(ctx->z_store, ctx->z_prev, ctx->m.hidden, ctx->ident_host[q], L - 1, 1, base + L - 1,
                               sp.alpha, (uint32_t)sp.seed, (uint32_t)(sp.seed >> 32), ctx->st);
    }
    launch_fill_i32(ctx->seq_step0, 0, ctx->max_seqs, ctx->st);
    HIPCHK(hipMemcpy(ctx->seqs, hs.data(), sizeof(SeqState) * ctx->max_seqs, hipMemcpyHostToDevice));
    launch_build_tiles_sampler(ctx->seqs, ctx->seq_ident, n_seqs, ctx->max_positions, ctx->tiles_samp, ctx->n_tiles_samp, ctx->rows_pad, !ctx->knobs.no_pack, ctx->st);
    int32_t act[3] = {n_seqs, 0, 0};
    HIPCHK(hipMemcpy(ctx->n_active, act, sizeof(act), hipMemcpyHostToDevice));
    ctx->sampler = sp;
    ctx->sp.n_new = sp.n_new; ctx->sp.r_inner = sp.r_inner; ctx->sp.r_total = sp.r_total; ctx->sp.w_max = sp.w_max;
    ctx->sp.headway = sp.headway; ctx->sp.adaptive = sp.adaptive; ctx->sp.eps = sp.eps; ctx->sp.alpha = sp.alpha;
    ctx->sp.temperature = sp.temperature; ctx->sp.pad_token = sp.pad_token;
    ctx->sp.seed_lo = (uint32_t)sp.seed; ctx->sp.seed_hi = (uint32_t)(sp.seed >> 32);
    ctx->sp.beta = sp.beta; ctx->sp.eta = sp.eta; ctx->sp.init_mode = sp.init_mode;
    ctx->samp_seqs = n_seqs;
    ctx->step = 0;
    ctx->joined = false;
    ctx->sampler_on = true;
    HIPCHK(hipStreamSynchronize(ctx->st));
    return check_launch(ctx);
}

extern "C" int rdlm_sampler_join(rdlm_ctx* ctx, int32_t seq) {
    if (!ctx || seq < 0) return RDLM_EINVAL;
    if (!ctx->sampler_on) return RDLM_ESTATE;
    if (seq >= ctx->max_seqs) return RDLM_ECAPACITY;
    const rdlm_sampler& sp = ctx->sampler;
    const int L = ctx->prompt_len[seq];
    if (L < 1) return RDLM_ESTATE;
    if ((long long)L + sp.n_new + sp.w_max + sp.headway + 1 > ctx->max_positions) return RDLM_ECAPACITY;
    const int n = std::max(ctx->samp_seqs, seq + 1);
    if (n * ((sp.w_max + 31) / 32) > ctx->max_tiles || n * sp.w_max > ctx->max_rows) return RDLM_ECAPACITY;
    PROPAGATE(ensure_blocks(ctx, seq, L));
    ctx->pos_bound[seq] = L;
    const size_t base = (size_t)seq * ctx->max_positions;
    launch_fill_i32(ctx->y + base + L, sp.pad_token, ctx->max_positions - L, ctx->st);
    launch_fill_i32(ctx->counts + base, 0, ctx->max_positions, ctx->st);
    launch_init_state_rows(ctx->z_store, ctx->z_prev, ctx->m.hidden, ctx->ident_host[seq], L - 1, 1, base + L - 1,
                           sp.alpha, (uint32_t)sp.seed, (uint32_t)(sp.seed >> 32), ctx->st);
    launch_seq_join(ctx->seqs, ctx->seq_step0, seq, L, ctx->step, ctx->st);
    ctx->samp_seqs = n;
    ctx->joined = true;
    launch_build_tiles_sampler(ctx->seqs, ctx->seq_ident, n, ctx->max_positions, ctx->tiles_samp, ctx->n_tiles_samp, ctx->rows_pad, !ctx->knobs.no_pack, ctx->st);
    return check_launch(ctx);
}

// ---------------------------------------------------------------------------------------------
// Eviction and re-admission of a sequence (App. "Larger batch sizes": hidden-state slots are fungible,
// can be evicted from a device and bundled into a later forward call, possibly elsewhere).  What makes
// up a sequence is copied to host memory as it is -- its cache blocks of every layer, its latents,
// z_prev, conditioning, tokens, step counters and window record -- and its blocks go back to the pool;
// re-admission puts the same bytes into whatever blocks and slot are free, so the sequence goes on
// exactly as if it had never left (its random draws are keyed by its identity, not by the slot).

struct EvictHeader {
    uint32_t magic, version;
    rdlm_model model;
    int32_t n_pos, n_blocks, prompt_len, ident, in_sampler, local_steps, pos_bound, pad;
    SeqState st;
    rdlm_sampler sampler;
};
constexpr uint32_t EVICT_MAGIC = 0x4d4c4452u;   // "RDLM"

static size_t evict_bytes(const rdlm_ctx* ctx, int n_pos, int n_blocks) {
    const size_t h = ctx->m.hidden;
    return sizeof(EvictHeader) + (size_t)n_pos * 4 * 2 + (size_t)3 * n_pos * h * 4 +
           (size_t)ctx->layers.size() * 2 * n_blocks * 32 * h * ctx->esz;
}

// Rows of the per-position stores worth keeping: every cached position, the prompt, and the window, which
// may already reach one step beyond the cached positions (plus the draft of its last position).
static int evict_rows(const rdlm_ctx* ctx, int seq) {
    const int reach = ctx->pos_bound[seq] > 0 ? ctx->pos_bound[seq] + 1 : 0;
    return std::min(ctx->max_positions, std::max({ctx->seq_blocks[seq] * 32, ctx->prompt_len[seq], reach}));
}

extern "C" size_t rdlm_seq_evict_bytes(const rdlm_ctx* ctx, int32_t seq) {
    if (!ctx || seq < 0 || seq >= ctx->max_seqs) return 0;
    return evict_bytes(ctx, evict_rows(ctx, seq), ctx->seq_blocks[seq]);
}

extern "C" int rdlm_seq_evict(rdlm_ctx* ctx, int32_t seq, void* host_buf, size_t cap) {
    if (!ctx || !host_buf || seq < 0) return RDLM_EINVAL;
    if (seq >= ctx->max_seqs) return RDLM_ECAPACITY;
    const int nb = ctx->seq_blocks[seq];
    const int n_pos = evict_rows(ctx, seq);
    if (cap < evict_bytes(ctx, n_pos, nb)) return RDLM_ECAPACITY;
    HIPCHK(hipStreamSynchronize(ctx->st));
    EvictHeader hd;
    memset(&hd, 0, sizeof hd);
    hd.magic = EVICT_MAGIC; hd.version = 1; hd.model = ctx->m;
    hd.n_pos = n_pos; hd.n_blocks = nb; hd.prompt_len = ctx->prompt_len[seq]; hd.ident = ctx->ident_host[seq];
    hd.pos_bound = ctx->pos_bound[seq];
    hd.in_sampler = ctx->sampler_on && seq < ctx->samp_seqs && ctx->pos_bound[seq] > 0;
    if (hd.in_sampler) {
        int32_t step0 = 0;
        HIPCHK(hipMemcpy(&hd.st, ctx->seqs + seq, sizeof(SeqState), hipMemcpyDeviceToHost));
        HIPCHK(hipMemcpy(&step0, ctx->seq_step0 + seq, 4, hipMemcpyDeviceToHost));
        hd.local_steps = ctx->step - step0;
        hd.sampler = ctx->sampler;
    }
    char* out = static_cast<char*>(host_buf);
    memcpy(out, &hd, sizeof hd); out += sizeof hd;
    const size_t h = ctx->m.hidden, row0 = (size_t)seq * ctx->max_positions;
    auto take = [&](const void* dev, size_t bytes) -> int {
        if (bytes) HIPCHK(hipMemcpy(out, dev, bytes, hipMemcpyDeviceToHost));
        out += bytes;
        return RDLM_OK;
    };
    PROPAGATE(take(ctx->y + row0, (size_t)n_pos * 4));
    PROPAGATE(take(ctx->counts + row0, (size_t)n_pos * 4));
    PROPAGATE(take(ctx->z_store + row0 * h, (size_t)n_pos * h * 4));
    PROPAGATE(take(ctx->z_prev + row0 * h, (size_t)n_pos * h * 4));
    PROPAGATE(take(ctx->e_store + row0 * h, (size_t)n_pos * h * 4));
    const size_t blk_bytes = (size_t)32 * h * ctx->esz;
    for (const Layer& L : ctx->layers)
        for (const void* pool : {L.kc, L.vc})
            for (int b = 0; b < nb; ++b)
                PROPAGATE(take(static_cast<const char*>(pool) + (size_t)ctx->tbl_host[(size_t)seq * ctx->blocks_per_seq + b] * blk_bytes,
                               blk_bytes));
    // the slot is empty from here on
    if (ctx->sampler_on) {
        launch_seq_retire(ctx->seqs, seq, 0, ctx->st);
        launch_build_tiles_sampler(ctx->seqs, ctx->seq_ident, ctx->samp_seqs, ctx->max_positions, ctx->tiles_samp,
                                   ctx->n_tiles_samp, ctx->rows_pad, !ctx->knobs.no_pack, ctx->st);
    }
    release_blocks(ctx, seq);
    ctx->pos_bound[seq] = 0;
    ctx->prompt_len[seq] = 0;
    return check_launch(ctx);
}

extern "C" int rdlm_seq_admit(rdlm_ctx* ctx, int32_t seq, const void* host_buf, size_t bytes) {
    if (!ctx || !host_buf || seq < 0 || bytes < sizeof(EvictHeader)) return RDLM_EINVAL;
    if (seq >= ctx->max_seqs) return RDLM_ECAPACITY;
    EvictHeader hd;
    memcpy(&hd, host_buf, sizeof hd);
    if (hd.magic != EVICT_MAGIC || hd.version != 1 || memcmp(&hd.model, &ctx->m, sizeof(rdlm_model)) != 0) return RDLM_EINVAL;
    if (hd.n_pos < 0 || hd.n_blocks < 0 || bytes < evict_bytes(ctx, hd.n_pos, hd.n_blocks))
        return RDLM_EINVAL;
    if (hd.n_pos > ctx->max_positions || hd.n_blocks > ctx->blocks_per_seq) return RDLM_ECAPACITY;
    // what the record says about itself must hang together before any of it reaches the device
    if (hd.prompt_len < 0 || hd.prompt_len > hd.n_pos || hd.pos_bound < 0 || hd.pos_bound > ctx->max_positions ||
        hd.local_steps < 0)
        return RDLM_EINVAL;
    if (ctx->seq_blocks[seq] != 0 || ctx->pos_bound[seq] > 0) return RDLM_ESTATE;       // the slot must be empty (released)
    if (hd.in_sampler) {
        const SeqState& q = hd.st;
        if (q.prompt_len != hd.prompt_len || q.n_frozen < q.prompt_len || q.win_pos0 < 0 || q.win_n < 0 ||
            q.win_n > std::max(hd.sampler.w_max, 1) || q.new_pos0 < 0 || q.new_n < 0 ||
            (long long)q.win_pos0 + q.win_n > hd.pos_bound || (long long)q.new_pos0 + q.new_n > hd.pos_bound ||
            q.n_frozen > hd.pos_bound || hd.pos_bound > hd.n_pos)
            return RDLM_EINVAL;
        if (!ctx->sampler_on || memcmp(&hd.sampler, &ctx->sampler, sizeof(rdlm_sampler)) != 0) return RDLM_ESTATE;
        const rdlm_sampler& sp = ctx->sampler;
        const int n = std::max(ctx->samp_seqs, seq + 1);
        if (n * ((sp.w_max + 31) / 32) > ctx->max_tiles || n * sp.w_max > ctx->max_rows) return RDLM_ECAPACITY;
        if ((long long)hd.prompt_len + sp.n_new + sp.w_max + sp.headway + 1 > ctx->max_positions) return RDLM_ECAPACITY;
    }
    if (hd.n_blocks > (int)ctx->free_blocks.size()) return RDLM_ECAPACITY;
    PROPAGATE(ensure_blocks(ctx, seq, hd.n_blocks * 32));
    HIPCHK(hipStreamSynchronize(ctx->st));
    const char* in = static_cast<const char*>(host_buf) + sizeof hd;
    const size_t h = ctx->m.hidden, row0 = (size_t)seq * ctx->max_positions;
    auto put = [&](void* dev, size_t nbytes) -> int {
        if (nbytes) HIPCHK(hipMemcpy(dev, in, nbytes, hipMemcpyHostToDevice));
        in += nbytes;
        return RDLM_OK;
    };
    const int pad = ctx->sampler_on ? ctx->sampler.pad_token : 0;
    launch_fill_i32(ctx->y + row0, pad, ctx->max_positions, ctx->st);
    launch_fill_i32(ctx->counts + row0, 0, ctx->max_positions, ctx->st);
    HIPCHK(hipStreamSynchronize(ctx->st));
    PROPAGATE(put(ctx->y + row0, (size_t)hd.n_pos * 4));
    PROPAGATE(put(ctx->counts + row0, (size_t)hd.n_pos * 4));
    PROPAGATE(put(ctx->z_store + row0 * h, (size_t)hd.n_pos * h * 4));
    PROPAGATE(put(ctx->z_prev + row0 * h, (size_t)hd.n_pos * h * 4));
    PROPAGATE(put(ctx->e_store + row0 * h, (size_t)hd.n_pos * h * 4));
    const size_t blk_bytes = (size_t)32 * h * ctx->esz;
    for (const Layer& L : ctx->layers)
        for (void* pool : {L.kc, L.vc})
            for (int b = 0; b < hd.n_blocks; ++b)
                PROPAGATE(put(static_cast<char*>(pool) + (size_t)ctx->tbl_host[(size_t)seq * ctx->blocks_per_seq + b] * blk_bytes,
                              blk_bytes));
    ctx->prompt_len[seq] = hd.prompt_len;
    ctx->ident_host[seq] = hd.ident;
    launch_fill_i32(ctx->seq_ident + seq, hd.ident, 1, ctx->st);
    if (hd.in_sampler) {
        HIPCHK(hipMemcpy(ctx->seqs + seq, &hd.st, sizeof(SeqState), hipMemcpyHostToDevice));
        launch_fill_i32(ctx->seq_step0 + seq, ctx->step - hd.local_steps, 1, ctx->st);
        ctx->pos_bound[seq] = hd.pos_bound;
        ctx->samp_seqs = std::max(ctx->samp_seqs, seq + 1);
        ctx->joined = true;
        // (the device's count of unfinished sequences is brought up to date by the next step's bookkeeping)
        launch_build_tiles_sampler(ctx->seqs, ctx->seq_ident, ctx->samp_seqs, ctx->max_positions, ctx->tiles_samp,
                                   ctx->n_tiles_samp, ctx->rows_pad, !ctx->knobs.no_pack, ctx->st);
    }
    HIPCHK(hipStreamSynchronize(ctx->st));
    return check_launch(ctx);
}

extern "C" int rdlm_sample_step(rdlm_ctx* ctx) {
    if (!ctx) return RDLM_EINVAL;
    if (!ctx->sampler_on) return RDLM_ESTATE;
    const rdlm_sampler& s = ctx->sampler;
    const rdlm_model& m = ctx->m;
    const int n = ctx->samp_seqs;
    // cache blocks for the positions the windows may cover in this step (a window ends at most `headway`
    // positions further on after every step); a pool that cannot supply them refuses the step before
    // anything is enqueued -- release or evict a sequence and call again
    {
        int need = 0;
        for (int q = 0; q < n; ++q)
            if (ctx->pos_bound[q] > 0) need += std::max(0, (ctx->pos_bound[q] + 31) / 32 - ctx->seq_blocks[q]);
        if (need > (int)ctx->free_blocks.size()) return RDLM_ECAPACITY;
        for (int q = 0; q < n; ++q) {
            if (ctx->pos_bound[q] <= 0) continue;       // slot not in the sampler
            PROPAGATE(ensure_blocks(ctx, q, ctx->pos_bound[q]));
            const int cap = std::min(ctx->max_positions, ctx->prompt_len[q] + s.n_new + s.w_max + s.headway);
            ctx->pos_bound[q] = std::min(cap, ctx->pos_bound[q] + s.headway);
        }
    }
    const int t = ++ctx->step;
    // upper bound of the wave size at this step: it grows by at most `headway` per step, and a
    // state stays at most ceil(r / r') steps (then it and every older state are freezable), so no
    // more than that many generations of `headway` states are in flight -- also under the
    // adaptive exit rule, whatever the wavefront limit
    long long grow = 1 + (long long)(t - 1) * s.headway;
    const long long in_flight = (long long)((s.r_total + s.r_inner - 1) / s.r_inner) * s.headway;
    int wmax_now = (int)std::min<long long>(std::min<long long>(s.w_max, in_flight), grow);   // (a joined sequence restarts at 1: still a bound)
    const int segs = n * ((wmax_now + 31) / 32);
    // row tiles: windows of up to 32 rows are packed in sequence order into the tile that is open, so a tile
    // that is closed holds at least floor(32 / wmax_now) of them
    const int T = (!ctx->knobs.no_pack && wmax_now <= TILE_ROWS) ? (n + TILE_ROWS / wmax_now - 1) / (TILE_ROWS / wmax_now) : segs;
    ctx->seg_tiles = segs;
    ctx->grouped = wmax_now > TILE_ROWS;
    ctx->seq_tiles_max = (wmax_now + TILE_ROWS - 1) / TILE_ROWS;
    ctx->att_groups = n * (((wmax_now + 31) / 32 + ATT_GROUP - 1) / ATT_GROUP);
    // keys a window can see in this step (only the launch shape of the attention kernels depends on it):
    // the host's bound on where the windows end, which follows the step count
    int max_keys = 1;
    for (int q = 0; q < n; ++q)
        if (ctx->pos_bound[q] > 0) max_keys = std::max(max_keys, ctx->pos_bound[q]);
    // the tile list of this step was built by sampler_begin or by the end of the previous step
    std::swap(ctx->tiles, ctx->tiles_samp);
    std::swap(ctx->n_tiles, ctx->n_tiles_samp);
    // e <- P(y_current); without momentum or noise the closing pass of P also writes concat(e, z)
    const bool plain = !(s.eta > 0.f) && !(s.beta > 0.f);
    bool cat_ready = false;
    const bool hoist = hoist_ok(ctx, s.r_inner);
    ctx->hoist_split = hoist;
    int rc = prelude_forward(ctx, ctx->y, ctx->e, -1, T, max_keys, plain ? ctx->z_store : nullptr, &cat_ready);
    ctx->hoist_split = false;
    if (s.eta > 0.f)                                                             // Eq. 1
        launch_momentum(ctx->e, ctx->e_store, ctx->counts, s.eta, m.hidden, ctx->tiles, ctx->n_tiles, T, ctx->st);
    if (s.beta > 0.f)                                                            // Eq. 2
        launch_noise_mix(ctx->z_store, ctx->counts, s.beta, (s.r_total + s.r_inner - 1) / s.r_inner, s.alpha,
                         ctx->sp.seed_lo, ctx->sp.seed_hi, t, ctx->seq_step0, m.hidden, ctx->tiles, ctx->n_tiles, T,
                         ctx->st);
    for (int i = 0; i < s.r_inner; ++i) {                                        // inner recurrence
        bool last = i == s.r_inner - 1;
        if (rc == RDLM_OK)
            rc = core_forward(ctx, ctx->e, ctx->z_store, last ? ctx->z_prev : nullptr, last ? 1 : 0,
                              last ? ctx->delta : nullptr, T, max_keys, cat_ready && i == 0, last,
                              hoist ? (i == 0 ? 1 : 2) : 0);
    }
    SampleArgs sa = {s.temperature, ctx->sp.seed_lo, ctx->sp.seed_hi, t, false, ctx->seq_step0, s.top_p};
    if (rc == RDLM_OK) rc = coda_forward(ctx, ctx->z_store, &sa, T, max_keys, true);   // p <- C(z); y_hat <- Sample(p)
    if (rc != RDLM_OK) {
        // a projection could not be launched (no kernel instance for a launch shape set through
        // rdlm_set_tuning): part of the step has run, so the sampler cannot go on from here
        std::swap(ctx->tiles, ctx->tiles_samp);
        std::swap(ctx->n_tiles, ctx->n_tiles_samp);
        ctx->sampler_on = false;
        return rc;
    }
    // freeze, append, InitState of the appended positions, tile list of the next step
    launch_step_end(ctx->seqs, ctx->seq_ident, n, ctx->sp, ctx->y, ctx->counts, ctx->max_positions, ctx->drafts, ctx->delta,
                    ctx->z_store, ctx->z_prev, m.hidden, ctx->tiles, ctx->n_tiles, ctx->n_active, t, ctx->step_ticket, ctx->rows_pad, !ctx->knobs.no_pack,
                    ctx->st);
    std::swap(ctx->tiles, ctx->tiles_samp);
    std::swap(ctx->n_tiles, ctx->n_tiles_samp);
    return check_launch(ctx);
}

extern "C" int rdlm_generate(rdlm_ctx* ctx, int32_t max_steps, int32_t* steps_out) {
    if (!ctx || max_steps < 1) return RDLM_EINVAL;
    if (!ctx->sampler_on) return RDLM_ESTATE;
    const rdlm_sampler& s = ctx->sampler;
    const int wave = (s.r_total + s.r_inner - 1) / s.r_inner;
    const int step0 = ctx->step;                 // sampler steps taken before this call
    // fixed exit: the step count is known; adaptive: look at the device every few steps
    int next_poll = s.adaptive ? 8 : std::max(1, wave + (s.n_new - 1 + s.headway - 1) / s.headway - step0);
    int done_steps = 0;
    bool nonfinite = false;
    for (int i = 1; i <= max_steps; ++i) {
        int rc = rdlm_sample_step(ctx);
        if (rc) return rc;
        done_steps = i;
        if (i >= next_poll || i == max_steps) {
            HIPCHK(hipMemcpyAsync(ctx->n_active_host, ctx->n_active, 12, hipMemcpyDeviceToHost, ctx->st));
            HIPCHK(hipStreamSynchronize(ctx->st));
            nonfinite = ctx->n_active_host[2] != 0;
            if (ctx->n_active_host[0] == 0) {            // steps after the finishing one were no-ops
                done_steps = std::max(0, ctx->n_active_host[1] - step0);
                break;
            }
            if (nonfinite) break;
            next_poll = i + (s.adaptive ? 8 : 1);
        }
    }
    HIPCHK(hipStreamSynchronize(ctx->st));
    if (steps_out) *steps_out = done_steps;
    return nonfinite ? RDLM_ENUMERIC : RDLM_OK;
}

// ---------------------------------------------------------------------------------------------
// read-back

extern "C" int rdlm_sampler_status(rdlm_ctx* ctx, int32_t* n_active_out, int32_t* nonfinite_out) {
    if (!ctx) return RDLM_EINVAL;
    if (!ctx->sampler_on) return RDLM_ESTATE;
    HIPCHK(hipStreamSynchronize(ctx->st));
    int32_t a[3] = {0, 0, 0};
    HIPCHK(hipMemcpy(a, ctx->n_active, sizeof a, hipMemcpyDeviceToHost));
    if (n_active_out) *n_active_out = a[0];
    if (nonfinite_out) *nonfinite_out = a[2] != 0;
    return RDLM_OK;
}

extern "C" int rdlm_read_tokens(rdlm_ctx* ctx, int32_t seq, int32_t* tokens_host, int32_t cap,
                                int32_t* n_frozen_out) {
    if (!ctx || !tokens_host || cap < 0 || seq < 0) return RDLM_EINVAL;
    if (seq >= ctx->max_seqs) return RDLM_ECAPACITY;
    HIPCHK(hipStreamSynchronize(ctx->st));
    int n = std::min(cap, ctx->max_positions);
    HIPCHK(hipMemcpy(tokens_host, ctx->y + (size_t)seq * ctx->max_positions, (size_t)n * 4, hipMemcpyDeviceToHost));
    if (n_frozen_out) {
        SeqState q;
        HIPCHK(hipMemcpy(&q, ctx->seqs + seq, sizeof(q), hipMemcpyDeviceToHost));
        *n_frozen_out = ctx->sampler_on ? q.n_frozen : ctx->prompt_len[seq];
    }
    return RDLM_OK;
}

// The frozen text only (y_frozen of Alg. 1 / Alg. 2): prompt and the tokens made final so far.
extern "C" int rdlm_read_frozen(rdlm_ctx* ctx, int32_t seq, int32_t* tokens_host, int32_t cap, int32_t* n_out) {
    if (!ctx || !tokens_host || !n_out || cap < 0 || seq < 0) return RDLM_EINVAL;
    if (seq >= ctx->max_seqs) return RDLM_ECAPACITY;
    HIPCHK(hipStreamSynchronize(ctx->st));
    int nf = ctx->prompt_len[seq];
    if (ctx->sampler_on) {
        SeqState q;
        HIPCHK(hipMemcpy(&q, ctx->seqs + seq, sizeof(q), hipMemcpyDeviceToHost));
        nf = q.n_frozen;
    }
    *n_out = nf;
    const int n = std::min(std::min(cap, nf), ctx->max_positions);
    if (n > 0) HIPCHK(hipMemcpy(tokens_host, ctx->y + (size_t)seq * ctx->max_positions, (size_t)n * 4, hipMemcpyDeviceToHost));
    return RDLM_OK;
}

extern "C" int rdlm_read_states(rdlm_ctx* ctx, int32_t seq, int32_t pos0, int32_t n, float* z_host) {
    if (!ctx || !z_host || seq < 0 || pos0 < 0 || n < 0) return RDLM_EINVAL;
    if (seq >= ctx->max_seqs || (long long)pos0 + n > ctx->max_positions) return RDLM_ECAPACITY;
    HIPCHK(hipStreamSynchronize(ctx->st));
    HIPCHK(hipMemcpy(z_host, ctx->z_store + ((size_t)seq * ctx->max_positions + pos0) * ctx->m.hidden,
                     (size_t)n * ctx->m.hidden * 4, hipMemcpyDeviceToHost));
    return RDLM_OK;
}

extern "C" int rdlm_read_prev_states(rdlm_ctx* ctx, int32_t seq, int32_t pos0, int32_t n, float* z_host) {
    if (!ctx || !z_host || seq < 0 || pos0 < 0 || n < 0) return RDLM_EINVAL;
    if (seq >= ctx->max_seqs || (long long)pos0 + n > ctx->max_positions) return RDLM_ECAPACITY;
    HIPCHK(hipStreamSynchronize(ctx->st));
    HIPCHK(hipMemcpy(z_host, ctx->z_prev + ((size_t)seq * ctx->max_positions + pos0) * ctx->m.hidden,
                     (size_t)n * ctx->m.hidden * 4, hipMemcpyDeviceToHost));
    return RDLM_OK;
}

extern "C" int rdlm_read_window(rdlm_ctx* ctx, int32_t seq, int32_t* pos0_out, int32_t* n_out, int32_t* done_out) {
    if (!ctx || seq < 0) return RDLM_EINVAL;
    if (seq >= ctx->max_seqs) return RDLM_ECAPACITY;
    if (!ctx->sampler_on) return RDLM_ESTATE;
    HIPCHK(hipStreamSynchronize(ctx->st));
    SeqState q;
    HIPCHK(hipMemcpy(&q, ctx->seqs + seq, sizeof(q), hipMemcpyDeviceToHost));
    if (pos0_out) *pos0_out = q.win_pos0;
    if (n_out) *n_out = q.done ? 0 : q.win_n;
    if (done_out) *done_out = q.done;
    return RDLM_OK;
}

extern "C" int rdlm_read_counts(rdlm_ctx* ctx, int32_t seq, int32_t pos0, int32_t n, int32_t* counts_host) {
    if (!ctx || !counts_host || seq < 0 || pos0 < 0 || n < 0) return RDLM_EINVAL;
    if (seq >= ctx->max_seqs || (long long)pos0 + n > ctx->max_positions) return RDLM_ECAPACITY;
    HIPCHK(hipStreamSynchronize(ctx->st));
    HIPCHK(hipMemcpy(counts_host, ctx->counts + (size_t)seq * ctx->max_positions + pos0, (size_t)n * 4,
                     hipMemcpyDeviceToHost));
    return RDLM_OK;
}

extern "C" int rdlm_read_deltas(rdlm_ctx* ctx, int32_t seq, float* delta_host, int32_t cap, int32_t* n_out) {
    if (!ctx || !delta_host || !n_out || seq < 0 || cap < 0) return RDLM_EINVAL;
    if (seq >= ctx->max_seqs) return RDLM_ECAPACITY;
    if (!ctx->sampler_on) return RDLM_ESTATE;
    HIPCHK(hipStreamSynchronize(ctx->st));
    SeqState q;
    HIPCHK(hipMemcpy(&q, ctx->seqs + seq, sizeof(q), hipMemcpyDeviceToHost));
    int n = std::min(cap, q.last_rows);
    if (n > 0)
        HIPCHK(hipMemcpy(delta_host, ctx->delta + (size_t)q.last_row0, (size_t)n * 4, hipMemcpyDeviceToHost));
    *n_out = q.last_rows;
    return RDLM_OK;
}

extern "C" int rdlm_read_kv(rdlm_ctx* ctx, int32_t layer, int32_t seq, int32_t pos0, int32_t n, float* k_host,
                            float* v_host) {
    if (!ctx || !k_host || !v_host || layer < 0 || seq < 0 || pos0 < 0 || n < 0) return RDLM_EINVAL;
    if (layer >= (int)ctx->layers.size()) return RDLM_EINVAL;
    if (seq >= ctx->max_seqs || (long long)pos0 + n > ctx->max_positions) return RDLM_ECAPACITY;
    if (n == 0) return RDLM_OK;
    const int h = ctx->m.hidden;
    if ((size_t)n * h * 2 > (size_t)ctx->rows_pad * 2 * ctx->m.mlp) return RDLM_ECAPACITY;   // staged in gu
    HIPCHK(hipStreamSynchronize(ctx->st));
    const Layer& L = ctx->layers[layer];
    // positions beyond the slot's blocks have no entries yet (a window's newest positions get theirs in the
    // step that computes them): they read as zeros; a slot without any block has no cache at all
    const int owned = ctx->seq_blocks[seq] * 32;
    if (owned == 0) return RDLM_ESTATE;
    const int n_dev = std::max(0, std::min(n, owned - pos0));
    float* kd = ctx->gu;
    float* vd = ctx->gu + (size_t)n * h;
    launch_read_kv(L.kc, L.vc, kv_pages(ctx), seq, ctx->m.dtype, ctx->m.n_heads, ctx->m.head_dim, pos0, n_dev, kd, vd, ctx->st);
    HIPCHK(hipStreamSynchronize(ctx->st));
    if (n_dev) {
        HIPCHK(hipMemcpy(k_host, kd, (size_t)n_dev * h * 4, hipMemcpyDeviceToHost));
        HIPCHK(hipMemcpy(v_host, vd, (size_t)n_dev * h * 4, hipMemcpyDeviceToHost));
    }
    memset(k_host + (size_t)n_dev * h, 0, (size_t)(n - n_dev) * h * 4);
    memset(v_host + (size_t)n_dev * h, 0, (size_t)(n - n_dev) * h * 4);
    return RDLM_OK;
}

// ---------------------------------------------------------------------------------------------
// kernel-level entry points

static int weight_by_index(const rdlm_ctx* ctx, int idx, const void** W, int* proj, int* N, int* K) {
    const rdlm_model& m = ctx->m;
    const int h = m.hidden, F = m.mlp;
    const int nl = m.n_prelude + m.n_core + m.n_coda;
    if (idx == 0) { *W = ctx->emb_w; *proj = PROJ_HEAD; *N = m.vocab; *K = h; return RDLM_OK; }
    if (idx >= 1 && idx < 1 + 7 * nl) {
        const Layer& L = ctx->layers[(idx - 1) / 7];
        switch ((idx - 1) % 7) {
            case 1: *W = L.wqkv; *proj = PROJ_QKV; *N = 3 * h; *K = h; return RDLM_OK;
            case 2: *W = L.wo; *proj = PROJ_O; *N = h; *K = h; return RDLM_OK;
            case 4: *W = L.wgu; *proj = PROJ_GU; *N = 2 * F; *K = h; return RDLM_OK;
            case 6: *W = L.wd; *proj = PROJ_D; *N = h; *K = F; return RDLM_OK;
            default: return RDLM_EINVAL;
        }
    }
    if (idx == 1 + 7 * nl) { *W = ctx->wa; *proj = PROJ_A; *N = h; *K = 2 * h; return RDLM_OK; }
    return RDLM_EINVAL;
}

static int linear_setup(rdlm_ctx* ctx, int m_rows, int* T) {
    if (m_rows < 1) return RDLM_EINVAL;
    if (m_rows > ctx->max_rows) return RDLM_ECAPACITY;
    SeqWindows w;
    w.n = 1; w.seq[0] = 0; w.pos0[0] = 0; w.rows[0] = m_rows;
    *T = (m_rows + 31) / 32;
    ctx->seg_tiles = *T;
    launch_build_tiles_api(w, ctx->seq_ident, ctx->tiles, ctx->n_tiles, ctx->rows_pad, !ctx->knobs.no_pack, ctx->st);
    return RDLM_OK;
}

// input operand buffer of a projection with K input features (the one the model path uses)
static void* proj_input(rdlm_ctx* ctx, int K) { return K == ctx->m.hidden ? ctx->xn : ctx->abuf; }

extern "C" int rdlm_linear(rdlm_ctx* ctx, int32_t w_index, const float* x, int32_t m_rows, float* y) {
    if (!ctx || !x || !y) return RDLM_EINVAL;
    const void* W; int proj, N, K, T;
    int rc = weight_by_index(ctx, w_index, &W, &proj, &N, &K);
    if (rc) return rc;
    if ((rc = linear_setup(ctx, m_rows, &T))) return rc;
    void* xin = proj_input(ctx, K);
    if (ctx->m.dtype == RDLM_F32) {       // rows beyond m_rows of the last tile are zero
        HIPCHK(hipMemsetAsync(xin, 0, (size_t)T * 32 * K * 4, ctx->st));
        HIPCHK(hipMemcpyAsync(xin, x, (size_t)m_rows * K * 4, hipMemcpyDeviceToDevice, ctx->st));
    } else {
        launch_pack_rows(x, xin, m_rows, K, ctx->st);
    }
    int S;
    if ((rc = run_proj(ctx, proj, xin, W, T, &S, nullptr, true))) return rc;
    const float* res = proj == PROJ_QKV ? ctx->qkv : proj == PROJ_GU ? ctx->gu : proj == PROJ_HEAD ? ctx->logits : nullptr;
    if (!res) {     // fold split-K partials exactly as the model path's consumer does
        launch_addnorm(nullptr, ctx->x, ctx->part, S, (size_t)ctx->rows_pad * N, ctx->gf, nullptr, ctx->fmt, N,
                       ctx->m.rms_eps, ctx->n_tiles, T, ctx->st);
        res = ctx->x;
    }
    launch_copy_rows_out(res, y, N, 2, ctx->tiles, ctx->n_tiles, T, ctx->st);
    return check_launch(ctx);
}

extern "C" int rdlm_time_linear(rdlm_ctx* ctx, int32_t w_index, int32_t m_rows, int32_t iters, float* ms_out) {
    if (!ctx || !ms_out || iters < 1) return RDLM_EINVAL;
    const void* W; int proj, N, K, T;
    int rc = weight_by_index(ctx, w_index, &W, &proj, &N, &K);
    if (rc) return rc;
    if ((rc = linear_setup(ctx, m_rows, &T))) return rc;
    if ((rc = ensure_blocks(ctx, 0, m_rows))) return rc;       // the QKV projection writes these positions of slot 0
    // Gaussian rows as input (values do not affect timing; keeps everything finite)
    void* xin = proj_input(ctx, K);
    float* stage = (size_t)K <= (size_t)3 * ctx->m.hidden ? ctx->qkv : ctx->gu;   // both idle here
    if (stage == ctx->gu && (proj == PROJ_GU || K > 2 * ctx->m.mlp)) return RDLM_EINVAL;
    launch_init_state_rows(stage, nullptr, K, 0, 0, T * 32, 0, 1.0f, 1u, 0u, ctx->st);
    if (ctx->m.dtype == RDLM_BF16) launch_pack_rows(stage, xin, T * 32, K, ctx->st);
    else HIPCHK(hipMemcpyAsync(xin, stage, (size_t)T * 32 * K * 4, hipMemcpyDeviceToDevice, ctx->st));
    SampleArgs sa = {0.f, 1u, 0u, 1, false};
    hipEvent_t a, b;
    HIPCHK(hipEventCreate(&a));
    HIPCHK(hipEventCreate(&b));
    int S;
    // the QKV projection is timed as the model runs it: RoPE and the cache writes in its epilogue
    // (rows land at positions 0.. of sequence 0 in the first layer's cache)
    const Layer* rl = proj == PROJ_QKV ? &ctx->layers[0] : nullptr;
    bool fused = false;
    launch_rope_table(ctx->rope_tab, ctx->theta, ctx->m.head_dim / 2, ctx->tiles, ctx->n_tiles, T, ctx->st);
    for (int i = 0; i < 3; ++i)
        if ((rc = run_proj(ctx, proj, xin, W, T, &S, &sa, false, false, rl, &fused))) return rc;
    // the timed launches go round the same projection of every layer, as a model pass does, so
    // that no launch finds its weights in a cache left by the one before
    std::vector<const void*> ring;
    if (w_index >= 1 && w_index < 1 + 7 * (int)ctx->layers.size())
        for (int l = 0; l < (int)ctx->layers.size(); ++l) {
            const void* Wl; int pj, n2, k2;
            if (weight_by_index(ctx, 1 + 7 * l + (w_index - 1) % 7, &Wl, &pj, &n2, &k2) == RDLM_OK) ring.push_back(Wl);
        }
    if (ring.empty()) ring.push_back(W);
    HIPCHK(hipEventRecord(a, ctx->st));
    for (int i = 0; i < iters; ++i)
        run_proj(ctx, proj, xin, ring[i % ring.size()], T, &S, &sa, false, false, rl, &fused);
    HIPCHK(hipEventRecord(b, ctx->st));
    HIPCHK(hipEventSynchronize(b));
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, a, b));
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    *ms_out = ms / iters;
    return check_launch(ctx);
}

// What the machine does with nothing but the reads: the packed weights of projection w_index of
// every layer in turn (so that no launch finds its bytes in a cache), `workgroups` x `waves` waves,
// each reading one contiguous slice.
extern "C" int rdlm_time_stream_read(rdlm_ctx* ctx, int32_t w_index, int32_t workgroups, int32_t waves, int32_t iters,
                                     float* ms_out, size_t* bytes_out) {
    if (!ctx || !ms_out || iters < 1 || workgroups < 1 || waves < 1 || waves > 4) return RDLM_EINVAL;
    if (ctx->m.dtype != RDLM_BF16) return RDLM_EINVAL;
    const void* W; int proj, N, K;
    int rc = weight_by_index(ctx, w_index, &W, &proj, &N, &K);
    if (rc) return rc;
    const size_t unit = (size_t)workgroups * waves * 1024;
    const size_t bytes = (size_t)N * K * 2 / unit * unit;       // whole 1 KiB units per wave, inside the tensor
    if (bytes == 0) return RDLM_EINVAL;
    std::vector<const void*> ring;
    if (w_index >= 1 && w_index < 1 + 7 * (int)ctx->layers.size())
        for (int l = 0; l < (int)ctx->layers.size(); ++l) {
            const void* Wl; int pj, n2, k2;
            if (weight_by_index(ctx, 1 + 7 * l + (w_index - 1) % 7, &Wl, &pj, &n2, &k2) == RDLM_OK) ring.push_back(Wl);
        }
    if (ring.empty()) ring.push_back(W);
    uint32_t* sink = reinterpret_cast<uint32_t*>(ctx->delta);
    hipEvent_t a, b;
    HIPCHK(hipEventCreate(&a));
    HIPCHK(hipEventCreate(&b));
    for (int i = 0; i < 2; ++i) launch_stream_read(ring[i % ring.size()], bytes, workgroups, waves, sink, ctx->st);
    HIPCHK(hipEventRecord(a, ctx->st));
    for (int i = 0; i < iters; ++i) launch_stream_read(ring[i % ring.size()], bytes, workgroups, waves, sink, ctx->st);
    HIPCHK(hipEventRecord(b, ctx->st));
    HIPCHK(hipEventSynchronize(b));
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, a, b));
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    *ms_out = ms / iters;
    if (bytes_out) *bytes_out = bytes;
    return check_launch(ctx);
}

// What the matrix cores do from registers alone: `workgroups` x 4 waves, each `inner_iters` rounds of
// four independent v_mfma_f32_32x32x16_bf16.  Long launches also show the clock the chip sustains
// under matrix load.
extern "C" int rdlm_time_mfma_loop(rdlm_ctx* ctx, int32_t workgroups, int32_t inner_iters, int32_t launches,
                                   float* ms_out, double* flops_out) {
    if (!ctx || !ms_out || workgroups < 1 || inner_iters < 1 || launches < 1) return RDLM_EINVAL;
    if ((size_t)workgroups * 256 > (size_t)8 * ctx->rows_pad * ctx->m.hidden) return RDLM_ECAPACITY;   // written to `part`
    hipEvent_t a, b;
    HIPCHK(hipEventCreate(&a));
    HIPCHK(hipEventCreate(&b));
    double flops = launch_mfma_loop(ctx->part, workgroups, 16, ctx->st);
    HIPCHK(hipEventRecord(a, ctx->st));
    for (int i = 0; i < launches; ++i) flops = launch_mfma_loop(ctx->part, workgroups, inner_iters, ctx->st);
    HIPCHK(hipEventRecord(b, ctx->st));
    HIPCHK(hipEventSynchronize(b));
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, a, b));
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    *ms_out = ms / launches;
    if (flops_out) *flops_out = flops;
    return check_launch(ctx);
}

extern "C" int rdlm_profile_gemm_begin(rdlm_ctx* ctx, int32_t n_out, int32_t k_in, int32_t max_launches) {
    if (!ctx || n_out < 1 || k_in < 1 || max_launches < 1 || max_launches > (1 << 20)) return RDLM_EINVAL;
    while ((int)ctx->prof_ev.size() < 2 * max_launches) {
        hipEvent_t ev;
        HIPCHK(hipEventCreate(&ev));
        ctx->prof_ev.push_back(ev);
    }
    ctx->prof_n = n_out; ctx->prof_k = k_in; ctx->prof_used = 0;
    return RDLM_OK;
}

extern "C" int rdlm_profile_gemm_read(rdlm_ctx* ctx, float* avg_ms_out, int32_t* launches_out) {
    if (!ctx || !avg_ms_out || !launches_out) return RDLM_EINVAL;
    HIPCHK(hipStreamSynchronize(ctx->st));
    double tot = 0.0;
    int n = ctx->prof_used / 2;
    for (int i = 0; i < n; ++i) {
        float ms = 0.f;
        HIPCHK(hipEventElapsedTime(&ms, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]));
        tot += ms;
    }
    *avg_ms_out = n ? (float)(tot / n) : 0.f;
    *launches_out = n;
    ctx->prof_n = ctx->prof_k = 0; ctx->prof_used = 0;
    return RDLM_OK;
}

extern "C" int rdlm_time_core_step(rdlm_ctx* ctx, int32_t seq, int32_t pos0, int32_t n, int32_t iters,
                                   float* ms_out) {
    if (!ctx || !ms_out || iters < 1 || seq < 0 || pos0 < 0 || n < 1) return RDLM_EINVAL;
    if (seq >= ctx->max_seqs || n > ctx->max_rows || (long long)pos0 + n > ctx->max_positions) return RDLM_ECAPACITY;
    PROPAGATE(ensure_blocks(ctx, seq, pos0 + n));
    SeqWindows w;
    w.n = 1; w.seq[0] = seq; w.pos0[0] = pos0; w.rows[0] = n;
    const int T = (n + 31) / 32;
    ctx->grouped = T > 1;
    ctx->seq_tiles_max = T;
    ctx->seg_tiles = T;
    ctx->att_groups = (T + ATT_GROUP - 1) / ATT_GROUP;
    launch_build_tiles_store(w, ctx->seq_ident, ctx->max_positions, ctx->tiles, ctx->n_tiles, ctx->rows_pad, !ctx->knobs.no_pack, ctx->st);
    launch_rope_table(ctx->rope_tab, ctx->theta, ctx->m.head_dim / 2, ctx->tiles, ctx->n_tiles, T, ctx->st);
    const size_t zrow0 = (size_t)seq * ctx->max_positions + pos0;
    launch_init_state_rows(ctx->z_store, nullptr, ctx->m.hidden, seq, pos0, n, zrow0, 1.0f, 7u, 0u, ctx->st);
    launch_init_state_rows(ctx->e, nullptr, ctx->m.hidden, seq, pos0, T * 32, 0, 1.0f, 9u, 0u, ctx->st);
    hipEvent_t a, b;
    HIPCHK(hipEventCreate(&a));
    HIPCHK(hipEventCreate(&b));
    for (int i = 0; i < 2; ++i) core_forward(ctx, ctx->e, ctx->z_store, nullptr, 0, nullptr, T, pos0 + n);
    HIPCHK(hipEventRecord(a, ctx->st));
    for (int i = 0; i < iters; ++i) core_forward(ctx, ctx->e, ctx->z_store, nullptr, 0, nullptr, T, pos0 + n);
    HIPCHK(hipEventRecord(b, ctx->st));
    HIPCHK(hipEventSynchronize(b));
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, a, b));
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    *ms_out = ms / iters;
    return check_launch(ctx);
}
