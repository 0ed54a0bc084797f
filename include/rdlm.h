/*
 * rdlm.h -- C ABI of the diffusion-forcing sampler hot path for recurrent-depth language models
 * on AMD MI355X (gfx950).
 *
 * Model (Sec. 3.1 of the paper):  e = P(x),  s_0 ~ N(0, sigma^2 I),  s_i = R(e, s_{i-1}),
 * p = C(s_r), with prelude P, recurrent block R and coda C made of transformer layers, input
 * injection through an adapter Linear(2h -> h) on concat(e, s), and a KV cache shared across
 * recurrence depth (Sec. 3.2: one K/V entry per layer and position, overwritten in place).
 * Samplers: Alg. 1 (fixed exit) and Alg. 2 (exit on the latent's relative change, Eq. 3, with a
 * wavefront limit).
 *
 * Conventions
 *   - Every function returns RDLM_OK (0) or a negative rdlm_status.  Arguments are validated on
 *     the host before anything is enqueued; a failed call enqueues nothing.
 *   - "device" pointers are HIP device memory owned by the caller unless stated otherwise;
 *     "host" pointers are ordinary host memory.  No torch types cross this boundary.
 *   - All work is enqueued on the stream given to rdlm_create and is asynchronous, except the
 *     rdlm_read_* functions and rdlm_generate, which synchronise that stream.
 *   - After rdlm_create the library allocates no further memory.  The step workspace is one slab:
 *     the library's own, or the caller's (rdlm_workspace_bytes + rdlm_create_ws).  Weights (re-tiled
 *     copies), the KV cache and the per-position sampler stores (latents, tokens, counters) are
 *     always the library's: their layouts are internal (MFMA operand order).
 *   - Rows of a step are given per sequence as (seq id, first position, row count): row j of
 *     sequence entry i sits at absolute position pos0[i] + j; rows of all entries are
 *     concatenated in the order given ("M rows").  Row-major float32 [M, hidden] everywhere.
 *   - Calls on one context must not overlap in time (one stream, one workspace).
 */
#ifndef RDLM_H
#define RDLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rdlm_ctx rdlm_ctx;

typedef enum {
    RDLM_OK = 0,
    RDLM_EINVAL = -1,     /* null pointer, non-positive size, shape the kernels do not support   */
    RDLM_ECAPACITY = -2,  /* more sequences, rows or positions than the context was created for   */
    RDLM_ENOMEM = -3,     /* device allocation failed in rdlm_create                              */
    RDLM_EHIP = -4,       /* a HIP call failed; see rdlm_last_hip_error                           */
    RDLM_ESTATE = -5,     /* call out of order (e.g. sample_step before sampler_begin)            */
    RDLM_ENUMERIC = -6    /* a non-finite delta_i (NaN / infinite latent, or ||z|| = 0) reached the  */
                          /* exit rule of Eq. 3; such a state is never frozen by it                  */
} rdlm_status;

enum { RDLM_F32 = 0, RDLM_BF16 = 1 };

/* Shape of the model.  dtype is the storage type of the matrices (and of the KV cache and GEMM
 * operands); accumulation, norms, softmax and the latent state are always float32.
 * RDLM_BF16 needs hidden % 32 == 0, mlp % 32 == 0, vocab % 32 == 0 and head_dim 32, 64, 96 or 128.
 * Both types need hidden <= 8192 (row kernels keep a row in registers), mlp >= hidden (staging
 * buffers are sized by mlp) and an even head_dim; anything else is RDLM_EINVAL from rdlm_create. */
typedef struct {
    int32_t vocab, hidden, n_heads, head_dim, mlp;
    int32_t n_prelude, n_core, n_coda;
    float rope_base;      /* RoPE base, rotate-half pairing (i, i + head_dim/2), absolute positions */
    float rms_eps;        /* x * g / sqrt(mean(x^2) + rms_eps)                                     */
    float emb_scale;      /* factor applied to gathered embedding rows                             */
    int32_t dtype;        /* RDLM_F32 or RDLM_BF16                                                 */
} rdlm_model;

/* Hyper-parameters of Alg. 1 / Alg. 2.  adaptive = 0: a state is frozen after r_total
 * recurrences (Alg. 1).  adaptive = 1: the longest prefix of states with delta_i < eps, or with
 * r_total recurrences, is frozen, and states are appended only while fewer than w_max are in
 * flight (Alg. 2, Eq. 3).  headway states are appended per step (Sec. 4.2); those beyond the
 * first read pad_token until a draft exists.  temperature 0 = greedy (lowest id wins ties),
 * otherwise Gumbel-max sampling from softmax(logits / temperature).
 * Stabilising components (Sec. 3.4), both off at 0:
 *   eta  -- momentum on the conditioning, e = eta e_prev + (1 - eta) P(y_current) (Eq. 1), per
 *           position; a position's first step takes P(y_current) as it is.
 *   beta -- state noise before the inner recurrences, z <- (1 - b) z + b z_noise (Eq. 2) with
 *           z_noise = InitState(1, alpha) drawn afresh each step (generator tag 3, counter
 *           includes the step) and b = beta * max(0, 1 - c / ceil(r_total / r_inner)) for a
 *           position that has had c sampler steps (linear schedule, later steps less noisy). */
typedef struct {
    int32_t n_new;        /* N: tokens to generate per sequence                                   */
    int32_t r_inner;      /* r'                                                                   */
    int32_t r_total;      /* r (fixed exit) or the recurrence cap (adaptive)                      */
    int32_t w_max;        /* wavefront limit; <= 0 means ceil(r_total / r_inner) * headway        */
    int32_t headway;
    int32_t adaptive;
    float eps;
    float alpha;          /* init scale of InitState                                              */
    float temperature;
    int32_t pad_token;
    float beta;           /* state-noise level of a position's first step, in [0, 1]              */
    float eta;            /* momentum of the conditioning, in [0, 1)                              */
    float top_p;          /* in (0, 1) with temperature > 0: sample from the smallest set of most */
                          /* probable tokens whose mass reaches top_p; 0 or >= 1: off.  Needs      */
                          /* vocab <= 65536 and vocab % 4 == 0                                     */
    int32_t init_mode;    /* states of appended positions: 0 = InitState draws (Alg. 1); 1 = copies  */
                          /* of the latest state of the position to the left (App., "continuous    */
                          /* compute"); the first state of a sequence is always a draw              */
    uint64_t seed;        /* key of the counter-based generator (state init, Gumbel, state noise) */
} rdlm_sampler;

/* Number of weight tensors rdlm_create expects, and their order:
 *   emb [V,h];  then for each layer of P, then R, then C:
 *   g1 [h] (f32), wqkv [3h,h] (rows: all q heads, all k heads, all v heads), wo [h,h], g2 [h] (f32),
 *   wg [F,h], wu [F,h], wd [h,F];  then wa [h,2h] (columns: e first, then s), gf [h] (f32),
 *   gout [h] (f32).   Matrices are row-major [out_features, in_features] in the model dtype
 *   (bf16 = upper 16 bits of the float32 pattern); gains are float32.  The LM head is emb (tied). */
int32_t rdlm_num_weights(const rdlm_model* m);

/* Create a context for up to max_seqs sequences of up to max_positions positions each and up to
 * max_rows rows per step (window rows of all sequences, or prefill rows).  weight_ptrs: host
 * array of rdlm_num_weights() device pointers; the library copies (and re-tiles) what it needs,
 * so the caller may free them afterwards.  hip_stream: a hipStream_t (NULL = default stream). */
int rdlm_create(const rdlm_model* m, const void* const* weight_ptrs, int32_t max_seqs,
                int32_t max_positions, int32_t max_rows, void* hip_stream, rdlm_ctx** out);
int rdlm_destroy(rdlm_ctx* ctx);

/* The same with the step workspace in caller-owned device memory: `workspace` (256-byte aligned)
 * of at least rdlm_workspace_bytes(m, max_seqs, max_rows) bytes, which must stay valid until
 * rdlm_destroy and is used by this context only.  workspace = NULL: the library allocates it.
 * rdlm_workspace_bytes returns 0 for a model or sizes rdlm_create would refuse. */
size_t rdlm_workspace_bytes(const rdlm_model* m, int32_t max_seqs, int32_t max_rows);
int rdlm_create_ws(const rdlm_model* m, const void* const* weight_ptrs, int32_t max_seqs,
                   int32_t max_positions, int32_t max_rows, void* hip_stream, void* workspace,
                   size_t workspace_bytes, rdlm_ctx** out);

/* ---- paged KV cache, eviction and re-admission --------------------------------------------- */
/* App. "Larger batch sizes" observes that with diffusion forcing the slots of a batch are
 * fungible: a sequence's states can be taken off the device and bundled into a later forward
 * call.  For that the KV cache of every layer is a pool of blocks of 32 positions, and a sequence
 * slot owns just the blocks its positions so far need: a per-slot block table (device memory,
 * max_seqs x ceil(max_positions / 32) entries) maps (slot, position / 32) to a pool block.  Blocks
 * are handed out lazily by the calls that write new positions (prefill, sampler steps, the building
 * blocks) and go back to the pool on rdlm_seq_release / rdlm_seq_evict / rdlm_destroy.
 *
 * rdlm_create sizes the pool so that every slot can reach max_positions (it can never run dry);
 * rdlm_create_paged sizes it to kv_pool_positions (>= 32, rounded up to whole blocks) positions in
 * total, shared by all slots.  A call that needs more blocks than the pool has left returns
 * RDLM_ECAPACITY and changes nothing; release or evict a sequence and call it again. */
int rdlm_create_paged(const rdlm_model* m, const void* const* weight_ptrs, int32_t max_seqs,
                      int32_t max_positions, int32_t max_rows, int32_t kv_pool_positions,
                      void* hip_stream, rdlm_ctx** out);
/* Blocks in the pool and blocks not owned by any slot right now (either pointer may be NULL). */
int rdlm_kv_blocks(const rdlm_ctx* ctx, int32_t* total_out, int32_t* free_out);
/* Give the blocks of slot seq back to the pool and, in a running sampler, take the slot out of it
 * (it contributes no rows until a sequence is joined or admitted there).  Tokens already read stay
 * readable; cache, states and window of the sequence are gone.  Synchronises the stream. */
int rdlm_seq_release(rdlm_ctx* ctx, int32_t seq);
/* Evict: copy everything that makes up the sequence in slot seq -- its cache blocks of all layers,
 * latents s, previous-step latents, conditioning e, tokens, per-position step counts, and (inside
 * a running sampler) its window record, step count and the sampler's parameters -- into host_buf
 * (host memory, cap >= rdlm_seq_evict_bytes(ctx, seq) bytes, else RDLM_ECAPACITY), then release the
 * slot as rdlm_seq_release does.  The buffer is self-contained and position-independent: it names
 * no slot and no block.  Synchronises the stream. */
size_t rdlm_seq_evict_bytes(const rdlm_ctx* ctx, int32_t seq);
int rdlm_seq_evict(rdlm_ctx* ctx, int32_t seq, void* host_buf, size_t cap);
/* Re-admit an evicted sequence into slot seq, which must be empty (never used, or released /
 * evicted; RDLM_ESTATE otherwise), of this context or of another one created for the same model.
 * If the sequence was evicted out of a running sampler, a sampler with the same parameters must
 * be running here (RDLM_ESTATE otherwise); the sequence then goes on from the step it had reached,
 * and since its generator counters are keyed by its own step count and by the slot number it
 * started in (kept in the buffer), its tokens and states are those of a run that was never
 * interrupted, whichever slot and blocks it now occupies.  RDLM_ECAPACITY if the pool has too few
 * free blocks or the slot table / row budget of the running sampler is exceeded (nothing changes),
 * RDLM_EINVAL for a buffer that is not an eviction record of this model.  Synchronises the stream. */
int rdlm_seq_admit(rdlm_ctx* ctx, int32_t seq, const void* host_buf, size_t bytes);

const char* rdlm_strerror(int status);
int rdlm_last_hip_error(const rdlm_ctx* ctx);   /* hipError_t of the last failed HIP call, or 0 */

/* Bytes of device memory the context holds (weights re-tiled, KV cache, workspace, sampler state). */
size_t rdlm_device_bytes(const rdlm_ctx* ctx);

/* ---- sequence text ------------------------------------------------------------------------ */
/* Set the known tokens of a sequence (y_frozen = y_current = x, Alg. 1, initialisation); tokens_host
 * [n] int32 in [0, vocab).  Synchronises the stream.  If a sampler is running, the sequence leaves
 * it (its slot contributes no rows) until rdlm_sampler_join puts it back. */
int rdlm_set_tokens(rdlm_ctx* ctx, int32_t seq, const int32_t* tokens_host, int32_t n);

/* Parallel prefill (Sec. 3.3): positions 0..n-1 of the sequence at once: e = P(x), fresh states
 * InitState(n, alpha), r recurrences of R, then the coda layers, so that every layer's cache holds
 * these positions.  n may be 0 (no-op).  Needs n <= max_rows. */
int rdlm_prefill(rdlm_ctx* ctx, int32_t seq, int32_t n, int32_t r, float alpha, uint64_t seed);

/* ---- the four calls of the sampler (Alg. 1: InitState, R, C + Sample, one whole iteration) --- */

/* InitState(n, alpha): z_out[j, :] ~ alpha * N(0, I) for positions pos0..pos0+n-1 of sequence
 * seq (device float32 [n, hidden]).  Counter-based: Philox4x32-10 keyed by seed, counter
 * (element/4, position, seq, tag), Box-Muller on uniforms u = (x>>9 + 1/2) * 2^-23. */
int rdlm_init_state(rdlm_ctx* ctx, int32_t seq, int32_t pos0, int32_t n, float alpha,
                    uint64_t seed, float* z_out);

/* e = P(tokens) for the given rows (prelude caches at those positions are overwritten).
 * tokens_dev: device int32 [M]; e_out: device float32 [M, hidden]. */
int rdlm_prelude(rdlm_ctx* ctx, int32_t n_seqs, const int32_t* seq_ids, const int32_t* pos0,
                 const int32_t* n_rows, const int32_t* tokens_dev, float* e_out);

/* r_inner recurrences z <- R(z, e) over all given rows at once (Alg. 1, inner recurrence), each row
 * attending to the cache prefix plus the rows before it in this step; core caches at those
 * positions are overwritten.  delta_out (device float32 [M], may be NULL) receives
 * ||z_new - z_in|| / ||z_new|| per row (Eq. 3 with z_prev = the z passed in).
 * seq_ids / pos0 / n_rows: host int32 [n_seqs].  e, z_inout: device float32 [M, hidden]. */
int rdlm_core_step(rdlm_ctx* ctx, int32_t n_seqs, const int32_t* seq_ids, const int32_t* pos0,
                   const int32_t* n_rows, const float* e, float* z_inout, int32_t r_inner,
                   float* delta_out);

/* rdlm_core_step for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments, same kernels, same
 * result, but every scratch buffer of the step (tile list, packed operands, split-K partial sums,
 * fold and attention tickets, KV-split partials) lives in one file-scope device array of
 * RDLM_STATIC_SCRATCH_BYTES bytes that each GPU the library runs on holds until the process ends;
 * the call performs no hipMalloc / hipFree.  The caller still owns e, z_inout and delta_out; weights
 * and the KV cache are the context's.  A call whose row tiles (sum over the windows of
 * ceil(n_rows / 32)) need more than the array holds -- rdlm_core_step_static_bytes(ctx, tiles)
 * tells -- is refused with RDLM_ECAPACITY and a message on stderr (3.5B shape: 2 tiles = 64 rows).
 * All calls on one GPU share that GPU's array, whatever their context: the array keeps the last
 * call's contents (the call clears the ticket words it needs at zero with a fill kernel, nothing
 * else is read before it is written), and calls that overlap in time on one GPU race. */
#define RDLM_STATIC_SCRATCH_BYTES (40u << 20)
size_t rdlm_core_step_static_bytes(const rdlm_ctx* ctx, int32_t n_tiles);
int rdlm_core_step_static(rdlm_ctx* ctx, int32_t n_seqs, const int32_t* seq_ids, const int32_t* pos0,
                          const int32_t* n_rows, const float* e, float* z_inout, int32_t r_inner,
                          float* delta_out);

/* C + Sample on every given row (Alg. 1, decode and sample): coda layers (caches overwritten), final
 * norm, tied LM head, then greedy or Gumbel-max at (seed, step), restricted to the top-p set when
 * 0 < top_p < 1 (App. "Dataset details": the paper samples at temperature 0.2, top-p 0.95).
 * tokens_out: device int32 [M]; logits_out: device float32 [M, vocab] or NULL. */
int rdlm_coda_decode(rdlm_ctx* ctx, int32_t n_seqs, const int32_t* seq_ids, const int32_t* pos0,
                     const int32_t* n_rows, const float* z, float temperature, uint64_t seed,
                     int32_t step, int32_t* tokens_out, float* logits_out, float top_p);

/* Start the sampler on sequences 0..n_seqs-1: each needs rdlm_set_tokens (L >= 1 tokens) and
 * rdlm_prefill of its first L-1 positions before.  Creates one fresh state at position L-1
 * (Alg. 1, initial state).  Needs L + n_new + w_max + headway <= max_positions and
 * n_seqs * roundup32(w_max) <= max_rows. */
int rdlm_sampler_begin(rdlm_ctx* ctx, const rdlm_sampler* s, int32_t n_seqs);

/* Continuous batching (App. "Larger batch sizes": slots whose occupants come and go while the
 * sampler runs).  Put sequence slot seq -- tokens set with rdlm_set_tokens, first L-1 positions
 * prefilled, in a slot that never ran or whose sequence has finished -- into the sampler started by
 * rdlm_sampler_begin, with one fresh state at position L-1 and the running sampler's
 * hyper-parameters.  The sequence counts its sampler steps (generator counters of Sample and of
 * the state noise) from the step it joins at, so its tokens and states are those of a run of its
 * own.  Enqueued on the stream, no synchronisation.  Same capacity rules as rdlm_sampler_begin,
 * with n_seqs = the highest slot in use + 1. */
int rdlm_sampler_join(rdlm_ctx* ctx, int32_t seq);

/* One iteration of Alg. 1 / Alg. 2 for all sequences that are not finished, entirely on the
 * device (no host synchronisation): P on the in-flight tokens, r' x R, C, Sample, drafts written
 * back, delta_i and k*, freeze, append. */
int rdlm_sample_step(rdlm_ctx* ctx);

/* Iterate rdlm_sample_step until every sequence has n_new frozen tokens or max_steps steps were
 * taken; synchronises.  The device is looked at only every few iterations (at the predicted last
 * one for the fixed exit rule); iterations enqueued after the finishing one do nothing.
 * steps_out (host, may be NULL) receives the number of iterations of this call up to the finishing
 * one.  Returns RDLM_ENUMERIC (after stopping at the next look) if a non-finite delta_i was seen. */
int rdlm_generate(rdlm_ctx* ctx, int32_t max_steps, int32_t* steps_out);

/* ---- read-back (synchronise the stream) ------------------------------------------------- */
/* State of the running sampler: sequences not yet finished, and whether any step since
 * rdlm_sampler_begin saw a non-finite delta_i (either may be NULL). */
int rdlm_sampler_status(rdlm_ctx* ctx, int32_t* n_active_out, int32_t* nonfinite_out);
/* Tokens of a sequence: frozen ones first (prompt + generated); n_frozen_out = |y_frozen|.
 * Copies min(cap, max_positions) entries of y_current (frozen, then current drafts, then pad). */
int rdlm_read_tokens(rdlm_ctx* ctx, int32_t seq, int32_t* tokens_host, int32_t cap,
                     int32_t* n_frozen_out);
/* The frozen text alone (y_frozen of Alg. 1 / Alg. 2: the prompt and the tokens made final so far):
 * *n_out = |y_frozen|, of which min(cap, |y_frozen|) tokens are copied. */
int rdlm_read_frozen(rdlm_ctx* ctx, int32_t seq, int32_t* tokens_host, int32_t cap, int32_t* n_out);
/* Latent states kept per position by the sampler (the state a position had when last updated). */
int rdlm_read_states(rdlm_ctx* ctx, int32_t seq, int32_t pos0, int32_t n, float* z_host);
/* z_prev of Alg. 2 per position: the state the position had at the end of the step before the last
 * one that touched it (what delta_i of the last step compared against); same layout. */
int rdlm_read_prev_states(rdlm_ctx* ctx, int32_t seq, int32_t pos0, int32_t n, float* z_host);
/* The in-flight window of a sequence as the next rdlm_sample_step will see it: position of its
 * oldest state, number of states (0 once the sequence is finished), finished flag (each may be NULL). */
int rdlm_read_window(rdlm_ctx* ctx, int32_t seq, int32_t* pos0_out, int32_t* n_out, int32_t* done_out);
/* Sampler steps each position spent in flight (its recurrence count is this times r_inner). */
int rdlm_read_counts(rdlm_ctx* ctx, int32_t seq, int32_t pos0, int32_t n, int32_t* counts_host);
/* delta_i of the rows of the last sample_step, in row order of sequence seq's window at that
 * step; n_out = number of rows it had. */
int rdlm_read_deltas(rdlm_ctx* ctx, int32_t seq, float* delta_host, int32_t cap, int32_t* n_out);
/* K and V rows of one layer (0-based over P, R, C layers in order) in natural order:
 * float32 [n, n_heads, head_dim] each (host).  Positions beyond the cache blocks the slot owns
 * (the newest window positions before the step that computes them) read as zeros; a slot that
 * owns no block at all (never used, released, evicted) is RDLM_ESTATE. */
int rdlm_read_kv(rdlm_ctx* ctx, int32_t layer, int32_t seq, int32_t pos0, int32_t n,
                 float* k_host, float* v_host);

/* ---- kernel-level entry points (measurement and unit tests) ------------------------------- */
/* Tuning knobs of a context (launch shapes, fusion switches); the same names in upper case with
 * the prefix RDLM_ are read from the environment once, by rdlm_create.  Names: "att_split" (forced
 * number of KV splits, 0 = automatic), "att_group_keys" (row tiles of a sequence x visible keys from which sequences with
 * several row tiles go through the grouped attention kernel; "" = default), "no_rope_fusion", "no_fold_fusion", "no_fold", "no_lds_gemm",
 * "no_hoist" (several recurrences per call: the e half of the adapter product is recomputed every
 * time instead of once), "no_pack" (every sequence's rows start a row tile of their own instead of short
 * windows sharing row tiles; RDLM_ESTATE while a sampler runs) ("1" / "0"), "plan_<p>" = "nb,waves,unroll,ksplit" and "planr_<p>" = "[s]mt,nb,waves,unroll,ksplit" or
 * "l<blocks>,<row tiles per wave>,<waves>,<k tiles per stage>,<ring depth>,<ksplit>" with <p> in
 * qkv, o, gu, d, a, head ("" = default).  A launch shape without a kernel instance makes the calls
 * that would use it return RDLM_EINVAL (and ends a running sampler: part of the step has run). */
int rdlm_set_tuning(rdlm_ctx* ctx, const char* name, const char* value);
/* y[M,N] = x[M,K] . W^T for weight tensor index w_index (as in the rdlm_create order; wg and wu
 * are one fused [2F,h] matrix reachable through wg's index).  x, y: device float32 row-major.
 * Runs the same tiled kernel the model path uses (including its split-K reduction). */
int rdlm_linear(rdlm_ctx* ctx, int32_t w_index, const float* x, int32_t m, float* y);
/* Time `iters` launches of that GEMM alone with HIP events on the context's stream, inputs
 * resident; the launches go round the same projection of every layer (same shape, different
 * weights), so that none finds its weights cached by the one before.  Returns the average
 * milliseconds per launch in ms_out (host). Synchronises. */
int rdlm_time_linear(rdlm_ctx* ctx, int32_t w_index, int32_t m, int32_t iters, float* ms_out);
/* Time `iters` core steps (r_inner = 1) over one sequence window [pos0, pos0+n) with HIP events;
 * the cache content at those positions is overwritten.  Synchronises. */
int rdlm_time_core_step(rdlm_ctx* ctx, int32_t seq, int32_t pos0, int32_t n, int32_t iters,
                        float* ms_out);

/* The machine beside the kernels ("achievable" next to the published peaks):
 * rdlm_time_stream_read -- a plain streaming read (nontemporal 16-byte loads, `workgroups` x `waves`
 *   waves, waves <= 4, one contiguous slice each) over the packed weights of projection w_index,
 *   going round the layers like rdlm_time_linear; average ms per launch and the bytes one launch
 *   reads.  bf16 models only.
 * rdlm_time_mfma_loop -- `workgroups` x 4 waves, each `inner_iters` rounds of four independent
 *   v_mfma_f32_32x32x16_bf16 on registers; average ms per launch and the flops of one launch.
 * Both synchronise. */
int rdlm_time_stream_read(rdlm_ctx* ctx, int32_t w_index, int32_t workgroups, int32_t waves, int32_t iters,
                          float* ms_out, size_t* bytes_out);
int rdlm_time_mfma_loop(rdlm_ctx* ctx, int32_t workgroups, int32_t inner_iters, int32_t launches, float* ms_out,
                        double* flops_out);

/* Per-launch timing of one GEMM shape inside the model path: while enabled, every launch of the
 * projection with n_out output and k_in input features (e.g. 2*mlp x hidden = gate/up) is
 * bracketed by HIP events on the context's stream, up to max_launches launches.
 * rdlm_profile_gemm_read synchronises, returns the average milliseconds per launch and the
 * number of launches recorded, and disables the recording. */
int rdlm_profile_gemm_begin(rdlm_ctx* ctx, int32_t n_out, int32_t k_in, int32_t max_launches);
int rdlm_profile_gemm_read(rdlm_ctx* ctx, float* avg_ms_out, int32_t* launches_out);

#ifdef __cplusplus
}
#endif
#endif /* RDLM_H */
