// Internal declarations shared by the HIP sources of librdlm (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace rdlm {

// A step works on "tiles" of up to 32 rows.  Every tile belongs to one sequence and covers
// contiguous positions; rows of a tile beyond n_valid are padding (computed, never stored into
// caches or states).  Internal activations use the padded ("physical") row index.
//
// Two kinds of descriptor share this struct and one device array (`tiles`):
//   tiles[r], r < rows_pad: the descriptor of physical row r alone -- pos0 is the row's position, the
//     *row0 fields its own rows in the arrays it reads and writes, n_valid 1 (0: padding row);
//   tiles[rows_pad + s]: segment s, up to 32 rows of one sequence at consecutive positions, at physical
//     rows prow0 .. prow0 + n_valid - 1.
// The matrix products and the row-wise kernels work on physical rows in tiles of 32 (descriptor by row);
// attention works on segments.  A sequence with more than 32 rows owns whole physical tiles, one segment
// each; sequences with fewer rows are packed, several segments to a physical tile (a batch of short
// windows then costs the products one row tile, not one per sequence).
struct TileDesc {
    int32_t seq;      // sequence (selects the KV-cache slab)
    int32_t pos0;     // absolute position of row 0 of the tile
    int32_t n_valid;  // 1..32
    int32_t zrow0;    // row of the tile's first state in the latent array it is read from / written to
    int32_t erow0;    // row of the tile's first conditioning vector e
    int32_t yrow0;    // index of the tile's first input token in the token array it reads
    int32_t crow0;    // compact row index (rows of all tiles concatenated without padding)
    int32_t group;    // attention: tiles t..t+group-1 (same sequence, consecutive positions) are served
                      // together by the workgroup of tile t; 0 = served by an earlier tile's workgroup
    int32_t rng;      // identity of the sequence in the counters of the random generator (its slot number
                      // unless the sequence moved in from another slot)
    int32_t prow0;    // physical row of the segment's first row (of the row itself in a row descriptor)
};

// Paged KV cache (App. "Larger batch sizes": state slots are fungible): a layer's K and V entries live in
// a pool of blocks of 32 positions x hidden elements; logical block b of the sequence in slot s is
// physical block table[s * stride + b].  Inside a block the layouts are those of k_cache_off / vt_slot.
struct KvPages {
    const int32_t* table = nullptr;   // device [slots][stride]
    int32_t stride = 0;               // logical blocks per slot
    int32_t slots = 0;                // rows of the table
};
__device__ inline size_t kv_block_base(const KvPages& kv, int seq, int block, size_t block_elems) {
    return (size_t)kv.table[(size_t)seq * kv.stride + block] * block_elems;
}
constexpr int ATT_GROUP = 4;

constexpr int TILE_ROWS = 32;
// The word block behind a tile list: [0] number of physical row tiles, [1] number of attention groups,
// [2] number of segments, and from TILE_LEADERS on the segment index of each group's first segment (so
// that the grouped attention kernels launch one workgroup per group and split, none for the segments a
// group serves).
constexpr int TILE_LEADERS = 16;
inline size_t tile_count_bytes(int max_tiles) { return (size_t)(TILE_LEADERS + max_tiles) * 4; }
constexpr int MAX_API_SEQS = 64;      // sequences per API call (descriptor passed as a kernel argument)

struct SeqWindows {                   // by-value kernel argument of build_tiles
    int32_t n;
    int32_t seq[MAX_API_SEQS];
    int32_t pos0[MAX_API_SEQS];
    int32_t rows[MAX_API_SEQS];
};

// Per-sequence sampler state kept on the device (Alg. 1 / Alg. 2 bookkeeping).
struct SeqState {
    int32_t prompt_len;   // |x|
    int32_t n_frozen;     // |y_frozen|
    int32_t win_pos0;     // position of the oldest in-flight state
    int32_t win_n;        // number of in-flight states
    int32_t done;         // n_frozen - prompt_len >= n_new
    int32_t last_rows;    // rows the sequence had in the last step (for read_deltas)
    int32_t last_pos0;
    int32_t new_pos0;     // states appended by the last bookkeeping pass: [new_pos0, new_pos0+new_n)
    int32_t new_n;
    int32_t last_row0;    // first physical row the sequence had in the last step
    int32_t cur_rows;     // rows / first physical row of the sequence in the tile list built for the next step
    int32_t cur_row0;
};

struct SamplerParams {
    int32_t n_new, r_inner, r_total, w_max, headway, adaptive;
    float eps, alpha, temperature;
    int32_t pad_token;
    uint32_t seed_lo, seed_hi;
    float beta, eta;
    int32_t init_mode;      // 0: appended states are InitState draws; 1: copies of the left neighbour's latest state
};

enum ActFmt { ACT_F32 = 0, ACT_BF16P = 1 };

// ---------------------------------------------------------------------------------------------
// bf16 <-> f32 (bit patterns; round to nearest even)
__host__ __device__ inline uint16_t f32_to_bf16(float f) {
    union { float f; uint32_t u; } v; v.f = f;
    uint32_t lsb = (v.u >> 16) & 1u;
    return (uint16_t)((v.u + 0x7FFFu + lsb) >> 16);
}
__host__ __device__ inline float bf16_to_f32(uint16_t b) {
    union { float f; uint32_t u; } v; v.u = ((uint32_t)b) << 16; return v.f;
}

// Offset (in bf16 elements) of element (row, k) of a packed activation with K columns:
// tiles of 32 rows x 16 columns, 1 KiB each, stored in MFMA operand order: lane = (row%32) +
// 32*((k%16)/8) holds 8 consecutive k.  Tiles are ordered [row tile][k tile].
__host__ __device__ inline size_t packed_off(int row, int k, int K) {
    int t = row >> 5, m = row & 31, kt = k >> 4, kk = k & 15;
    return (((size_t)t * (K >> 4) + kt) * 64 + m + 32 * (kk >> 3)) * 8 + (kk & 7);
}

// Offset of (position, head, dim) inside one sequence's bf16 K cache.  Keys are stored in blocks of
// 32 positions per head, each block as the A operands of the score contraction S^T = K.Q^T:
// [pos / 32][head][dim / 16][lane = 32 * (dim % 16 / 8) + pos % 32][dim % 8].  A wave's load of one
// k step is 1 KiB contiguous and a (block, head) is 64 * D contiguous bytes, as in the V cache.
__host__ __device__ inline size_t k_cache_off(int pos, int hd, int dim, int H, int D) {
    return ((((size_t)(pos >> 5) * H + hd) * (D >> 4) + (dim >> 4)) * 64 + 32 * ((dim >> 3) & 1) + (pos & 31)) * 8 +
           (dim & 7);
}

// Position of key `kappa` (0..31) inside a 32-position block of the transposed V cache.  The
// order is the one in which the 32x32 score accumulator of the attention kernel hands its keys to
// the P.V contraction, so that both operands of that contraction are plain 16-byte loads.
__host__ __device__ inline int vt_slot(int kappa) {
    int m = kappa >> 4, w = kappa & 15;
    return m * 16 + ((w & 7) >> 2) * 8 + (w >> 3) * 4 + (w & 3);
}

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  counter = (block, position, seq, step*16 + tag).
constexpr uint32_t TAG_INIT_STATE = 1, TAG_SAMPLE = 2, TAG_NOISE = 3;

__host__ __device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4]) {
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}
// 23 random bits plus one half: u in (0,1), never 0 or 1, exactly representable in float32
__host__ __device__ inline float u24_open(uint32_t x) {
    return ((float)(x >> 9) + 0.5f) * (1.0f / 8388608.0f);
}

// ---------------------------------------------------------------------------------------------
// Arrival ticket of a workgroup at a hand-over point: data that another workgroup will read has
// been written with system-scope (write-through) stores; the workgroup then draws a ticket from a
// system-scope counter, and whoever draws the last one reads the others' data back with
// system-scope (cache-bypassing) loads.  Ordering, hardware side: s_waitcnt(0) holds every wave
// until its stores have been acknowledged by memory, and the barrier holds thread 0's atomic until
// every wave got there.  Compiler side: __syncthreads() carries workgroup-scope release and acquire
// fences, which no store before it may sink below and no load after it may rise above, and the two
// single-thread fences pin the wait itself between the stores and the barrier.  (A device-scope
// release on the atomic would order the same accesses by the memory model's letter, but on this
// multi-die part it is an L2 write-back per workgroup -- tens of microseconds per launch.)
// Must be called by every thread of the workgroup.  The caller resets the counter to zero.
#ifdef __HIPCC__
__device__ __forceinline__ uint32_t draw_ticket(uint32_t* counter, uint32_t* shared_slot) {
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __builtin_amdgcn_s_waitcnt(0);
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __syncthreads();
    if (threadIdx.x == 0)
        *shared_slot = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    __syncthreads();
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    return *shared_slot;
}
#endif

// ---------------------------------------------------------------------------------------------
// Launchers (defined in the kernel sources).  All enqueue on `st`; none synchronises.

// kind GEMM_STREAM: the waves of a workgroup split K (one row-tile group, weights streamed once);
// kind GEMM_ROWS: the waves own different feature blocks and share the activation tiles through LDS.
// kind GEMM_LDS: every operand tile goes straight from global memory into LDS, the waves own different
// row tiles and share the weight tiles (see kernels_gemm_lds.hip); `depth` = stages of its LDS ring.
enum { GEMM_STREAM = 0, GEMM_ROWS = 1, GEMM_LDS = 2 };
struct GemmPlan { int mt, nb, waves, unroll, ksplit, kind = GEMM_STREAM, depth = 0; };

// What the GEMM does with a finished output tile.
enum { EPI_F32 = 0, EPI_SWIGLU = 1, EPI_ARGMAX = 2, EPI_ROPE_KV = 3 };
// Order of the output features inside the packed weight blocks (see canon_col in kernels_gemm.hip).
enum { WL_NATURAL = 0, WL_GU16 = 1, WL_ROPE = 2 };
struct GemmEpilogue {
    int kind = EPI_F32;
    int layout = WL_NATURAL;          // weight block layout; EPI_F32 writes canonical columns
    void* act = nullptr;              // EPI_SWIGLU: packed bf16 activation [rows][F]
    float* cand_val = nullptr;        // EPI_ARGMAX: best score / token per (feature group, row)
    int32_t* cand_idx = nullptr;
    size_t cand_stride = 0;           // rows per group in the candidate arrays
    float temperature = 0.f;          // > 0: Gumbel-max on logits / temperature
    uint32_t k0 = 0, k1 = 0;
    int step = 0;
    const int32_t* seq_step0 = nullptr;   // per sequence: sampler step it joined at (its own steps count from there)
    const TileDesc* tiles = nullptr;
    // EPI_ROPE_KV (QKV projection, WL_ROPE blocks): rotate q and k, store q (bf16 rows), k and v
    // into the layer's cache at the rows' positions
    void* q_out = nullptr;
    void* kc = nullptr;
    void* vc = nullptr;
    const float* rope_table = nullptr;   // [rows][d/2] (cos, sin)
    int n_heads = 0, head_dim = 0;
    KvPages kv;
    // Deferred RMSNorm: when row_ssq is set, the input rows were stored as x * gain without the
    // 1/rms factor; every output row is multiplied by 1/sqrt(sum_c row_ssq[row][c] / h + eps).
    const float* row_ssq = nullptr;      // [slot][ssq_stride rows]
    int ssq_chunks = 0;
    size_t ssq_stride = 0;
    // EPI_F32 with fold_counter set (one row tile, WL_NATURAL, 1, 2 or 4 blocks per workgroup): the
    // split-K partial sums are written through to memory; the last workgroup of a feature group to
    // arrive (ticket in fold_counter[group], left at zero again) adds them in split order to the
    // residual rows, and writes x_out, bf16(x_out * gain) as packed operand and the group's share
    // of each row's sum of squares (slot = group) -- what fold_k would do in a launch of its own.
    uint32_t* fold_counter = nullptr;
    const float* fold_xin = nullptr;
    float* fold_xout = nullptr;
    const float* fold_gain = nullptr;
    void* fold_xg = nullptr;
    float* fold_ssq = nullptr;
    int norm_h = 0;
    float norm_eps = 0.f;
};
constexpr int SSQ_MAX_CHUNKS = 256;   // slots per row: chunks of fold_k, or feature groups of a folding GEMM

// elementwise / row kernels ------------------------------------------------------------------
// ident: per slot, the sequence's identity in the random generator's counters
// tiles: [rows_pad] row descriptors followed by the segments; pack: short windows share row tiles
void launch_build_tiles_api(const SeqWindows& w, const int32_t* ident, TileDesc* tiles, int32_t* n_tiles, int rows_pad,
                            bool pack, hipStream_t st);
// same, but rows map to the library's per-(sequence, position) stores instead of compact arrays
void launch_build_tiles_store(const SeqWindows& w, const int32_t* ident, int max_positions, TileDesc* tiles,
                              int32_t* n_tiles, int rows_pad, bool pack, hipStream_t st);
void launch_build_tiles_sampler(const SeqState* seqs, const int32_t* ident, int n_seqs, int max_positions,
                                TileDesc* tiles, int32_t* n_tiles, int rows_pad, bool pack, hipStream_t st);
// block table entries table[first + i] = ids[i], i < n <= 16 (new blocks of a growing sequence)
struct BlockIds { int32_t n; int32_t first; int32_t id[16]; };
void launch_table_set(int32_t* table, BlockIds ids, hipStream_t st);
// x[row] = scale * emb[token of the row]; with rope_table: also the (cos, sin) table of the rows;
// with xg (bf16 path): also bf16(x * gain) as packed operand and the fold_chunks(h) per-chunk sums of
// squares of each row (what fold_k would leave for the first layer's norm)
void launch_embed(const void* emb, int dtype, const int32_t* tokens, float scale, float* x, int h, int V,
                  float* rope_table, const float* theta, int half, const float* gain, void* xg, float* ssq,
                  size_t ssq_stride, const TileDesc* tiles, const int32_t* n_tiles, int max_tiles, hipStream_t st);
void launch_copy_rows_in(const float* src, float* x, int h, int which /*0=z,1=e*/,
                         const TileDesc* tiles, const int32_t* n_tiles, int max_tiles, hipStream_t st);
void launch_copy_rows_out(const float* x, float* dst, int width, int which /*0=z,1=e,2=compact*/,
                          const TileDesc* tiles, const int32_t* n_tiles, int max_tiles, hipStream_t st);
void launch_copy_i32_out(const int32_t* src, int32_t* dst, const TileDesc* tiles,
                         const int32_t* n_tiles, int max_tiles, hipStream_t st);
// adapter operand concat(e, z) of width 2h; with e or z null: the other one alone, width h
void launch_concat(const float* e, const float* z, void* cat, int fmt, int h, const TileDesc* tiles,
                   const int32_t* n_tiles, int max_tiles, hipStream_t st);
void launch_addnorm(const float* xin, float* xout, const float* part, int S, size_t part_stride,
                    const float* gain, void* xn, int fmt, int h, float eps, const int32_t* n_tiles,
                    int max_tiles, hipStream_t st);
// bf16 path: x_out = x_in + sum_s part[s];  xg = bf16(x_out * gain) (packed, NOT divided by the rms);
// ssq[row][c] = sum of x_out^2 over chunk c of the row (SSQ_MAX_CHUNKS slots per row).  The
// row is split over `chunks` workgroups, so a 32-row step still fills the chip.
int fold_chunks(int h);
void launch_fold(const float* xin, float* xout, const float* part, int S, size_t part_stride,
                 const float* gain, void* xg, float* ssq, size_t ssq_stride, int h, const int32_t* n_tiles,
                 int max_tiles, hipStream_t st);
void launch_final_norm(const float* xin, const float* part, int S, size_t part_stride,
                       const float* gain, int h, float eps, float* z, float* z_prev, int update_prev,
                       float* delta, float* xcopy /* padded-row copy of z for the coda, or null */,
                       const float* gain2, void* xg /* with xcopy: packed bf16(z' * gain2), or null */,
                       float* ssq_tot /* with xg: sum of z'^2 per row */,
                       const TileDesc* tiles, const int32_t* n_tiles, int max_tiles, hipStream_t st);
// bf16 path, end of the prelude: e_out (f32, padded rows) = xin + sum part, and the packed adapter
// operand cat = concat(e, z) with z read from the latent store rows of the tiles; with cat_e the two
// halves become operands of width h of their own (e in cat_e, z in cat)
void launch_prelude_end(const float* xin, const float* part, int S, size_t part_stride, float* e_out, const float* z,
                        void* cat, void* cat_e, int h, const TileDesc* tiles, const int32_t* n_tiles, int max_tiles,
                        hipStream_t st);
// table: [rows][d/2] (cos, sin) pairs written by launch_rope_table for the current tiles
void launch_rope_table(float* table, const float* theta, int half, const TileDesc* tiles,
                       const int32_t* n_tiles, int max_tiles, hipStream_t st);
void launch_rope_kv(const float* qkv, int S, size_t part_stride, void* q, void* kc, void* vc,
                    int dtype, int H, int d, const float* table, KvPages kv,
                    const TileDesc* tiles, const int32_t* n_tiles, int max_tiles, hipStream_t st);
void launch_swiglu(const float* gu, int S, size_t part_stride, void* act, int fmt, int F,
                   const int32_t* n_tiles, int max_tiles, hipStream_t st);
void launch_init_state_rows(float* z, float* z_prev, int h, int seq, int pos0, int n, size_t zrow0,
                            float alpha, uint32_t k0, uint32_t k1, hipStream_t st);
// Eq. 1 on the rows of the step: e <- eta e_prev + (1 - eta) e for positions that have been in
// flight before (counts > 0); e_store keeps the result per (sequence, position).
void launch_momentum(float* e, float* e_store, const int32_t* counts, float eta, int h, const TileDesc* tiles,
                     const int32_t* n_tiles, int max_tiles, hipStream_t st);
// Eq. 2 on the rows of the step, in place on the latent store: z <- (1 - b) z + b z_noise with
// b = beta * max(0, 1 - counts / n_steps) and z_noise drawn at (position, seq, step).
void launch_noise_mix(float* z, const int32_t* counts, float beta, int n_steps, float alpha, uint32_t k0,
                      uint32_t k1, int step, const int32_t* seq_step0, int h, const TileDesc* tiles,
                      const int32_t* n_tiles, int max_tiles, hipStream_t st);
void launch_sample(const float* logits, int V, float temperature, uint32_t k0, uint32_t k1, int step,
                   const int32_t* seq_step0, int32_t* tok_out, const TileDesc* tiles, const int32_t* n_tiles,
                   int max_tiles, hipStream_t st);
// Sample with a top-p filter from full logits [rows][V]; V % 4 == 0, V <= TOPP_MAX_VOCAB.
constexpr int TOPP_MAX_VOCAB = 65536;
void launch_sample_top_p(const float* logits, int V, float temperature, float top_p, uint32_t k0, uint32_t k1,
                         int step, const int32_t* seq_step0, int32_t* tok_out, const TileDesc* tiles,
                         const int32_t* n_tiles, int max_tiles, hipStream_t st);
// Continuous batching: put a sequence into (join) or take it out of (retire) a running sampler.
void launch_seq_join(SeqState* seqs, int32_t* seq_step0, int seq, int prompt_len, int step, hipStream_t st);
void launch_seq_retire(SeqState* seqs, int seq, int prompt_len, hipStream_t st);
// End of a sampler step in one launch (one workgroup per sequence): drafts -> y_current, step
// counters, k*, freeze, append (Alg. 1 assign / freeze / append, Alg. 2), Gaussian states of the appended
// positions, and the tile list of the next step.  ticket: one device word, zero between launches.
void launch_step_end(SeqState* seqs, const int32_t* ident, int n_seqs, SamplerParams p, int32_t* y, int32_t* counts,
                     int max_positions, const int32_t* drafts, const float* delta, float* z, float* z_prev, int h,
                     TileDesc* tiles, int32_t* n_tiles, int32_t* n_active, int step, uint32_t* ticket, int rows_pad,
                     bool pack, hipStream_t st);
void launch_fill_i32(int32_t* p, int32_t v, size_t n, hipStream_t st);
void launch_read_kv(const void* kc, const void* vc, KvPages kv, int seq, int dtype, int H, int d, int pos0, int n,
                    float* k_out, float* v_out, hipStream_t st);

// GEMMs ---------------------------------------------------------------------------------------
// bf16: x packed [tiles][K/16][512], w packed [N/32][K/16][512]; EPI_F32 writes f32
// [ksplit][rows_total][N].  Returns false if no kernel instance exists for (plan, epilogue).
bool launch_gemm_bf16(const void* xp, const void* wp, float* out, int N, int K, size_t part_stride,
                      GemmPlan plan, const GemmEpilogue& epi, const int32_t* n_tiles, int max_tiles,
                      hipStream_t st);
bool launch_gemm_lds(const void* xp, const void* wp, float* out, int N, int K, size_t part_stride, GemmPlan plan,
                     const GemmEpilogue& epi, const int32_t* n_tiles, int max_tiles, hipStream_t st);
int gemm_groups(int N, const GemmPlan& plan, int epi_kind);
void launch_argmax_final(const float* cand_val, const int32_t* cand_idx, int n_groups, size_t cand_stride,
                         int32_t* tok_out, const int32_t* n_tiles, int max_tiles, hipStream_t st);
// f32: x [rows][K], w [N][K], out [rows][N]
void launch_gemm_f32(const float* x, const float* w, float* out, int N, int K,
                     const int32_t* n_tiles, int max_tiles, hipStream_t st);
// canonical bf16 rows [N][K] (rows < split from w0, the rest from w1) -> packed blocks in `layout`;
// ld: elements between consecutive source rows (0 = K; larger: K columns out of a wider matrix)
void launch_pack_weight(const void* w0, const void* w1, int split, void* w_packed, int N, int K, int layout,
                        int n_heads, int head_dim, hipStream_t st, int ld = 0);
void launch_pack_rows(const float* x, void* xp, int rows, int K, hipStream_t st);   // f32 rows -> packed bf16

// reference kernels (measurement only) -------------------------------------------------------
void launch_stream_read(const void* p, size_t bytes, int workgroups, int waves, uint32_t* sink, hipStream_t st);
double launch_mfma_loop(float* out, int workgroups, int iters, hipStream_t st);

// attention -----------------------------------------------------------------------------------
// q: f32 [rows][H*d] (RDLM_F32) or bf16 [rows][H*d]; caches per the model dtype; out: activation
// format of the model dtype, width H*d.  ws: split-KV partials.
void launch_attention(const void* q, const void* kc, const void* vc, void* out, int dtype, int H, int d,
                      KvPages kv, int nsplit, bool grouped, float* ws,
                      uint32_t* tickets /* [max_tiles][H], zero between launches */,
                      const TileDesc* tiles /* row descriptors, then the segments */, int rows_pad,
                      const int32_t* n_tiles, int max_tiles /* bound on the segments */, hipStream_t st,
                      int max_groups = 0 /* grouped: the host's bound on the number of attention groups (0: max_tiles) */);
size_t attention_ws_floats(int max_tiles, int H, int d, int nsplit);

}  // namespace rdlm
