// Row-wise kernels of the recurrent-depth LM step: tile descriptors, embedding gather, adapter
// concat, residual-add + RMSNorm (which also folds the split-K partial sums of the preceding
// GEMM), end-of-recurrence norm + convergence reduction (Eq. 3), RoPE + KV-cache write
// (Sec. 3.2: in-place overwrite), SwiGLU, Gaussian state init, sampling, and the sampler's
// device-side bookkeeping (Alg. 1 assign / freeze / append, Alg. 2).
#include "rdlm_internal.h"

namespace rdlm {

// ---------------------------------------------------------------------------------------------
__device__ inline float block_sum(float v, float* sh) {          // up to 1024 threads, sh[16]
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[w] = v;
    __syncthreads();
    float t = 0.f;
    for (int i = 0; i < (int)(blockDim.x >> 6); ++i) t += sh[i];
    return t;
}

template <int FMT>
__device__ inline void act_store4(void* base, int K, int row, int k, float a, float b, float c, float d) {
    if (FMT == ACT_F32) {
        float4 v = make_float4(a, b, c, d);
        *reinterpret_cast<float4*>(reinterpret_cast<float*>(base) + (size_t)row * K + k) = v;
    } else {
        ushort4 v;
        v.x = f32_to_bf16(a); v.y = f32_to_bf16(b); v.z = f32_to_bf16(c); v.w = f32_to_bf16(d);
        *reinterpret_cast<ushort4*>(reinterpret_cast<uint16_t*>(base) + packed_off(row, k, K)) = v;
    }
}

__device__ inline float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }

// ---------------------------------------------------------------------------------------------
// tile descriptors
//
// Lays the windows of a step out on physical rows.  Thread 0 of one workgroup calls add() for every
// window in sequence order and then counts(); after a barrier all threads of the workgroup call rows().
// A window of more than 32 rows gets whole row tiles (one segment per tile, groups of up to ATT_GROUP
// segments for the attention kernels); shorter windows are packed one after the other into the row
// tile that is open, as long as they fit (`pack`), so a batch of short windows shares row tiles.
constexpr int TILE_LDS_SEGS = 64;
struct TileLayout {
    TileDesc* tiles;        // [rows_pad] row descriptors, then the segments
    TileDesc* sh_segs = nullptr;   // LDS copy of the first TILE_LDS_SEGS segments
    int32_t* n_tiles;
    int rows_pad, pack;
    int n_seg = 0, n_phys = 0, n_lead = 0, c = 0, open_row = 0, open_cap = 0;
    // store_base < 0: caller-owned compact arrays; else row of position 0 of the sequence in the library's stores
    __device__ int add(int seq, int rng, int pos0, int nrows, long long store_base) {
        if (nrows <= 0) return n_phys * TILE_ROWS;
        int first;
        const bool small = pack && nrows <= TILE_ROWS;
        if (small && open_cap >= nrows) {
            first = open_row; open_row += nrows; open_cap -= nrows;
        } else {
            first = n_phys * TILE_ROWS;
            n_phys += (nrows + TILE_ROWS - 1) / TILE_ROWS;
            open_row = first + nrows;
            open_cap = small ? TILE_ROWS - nrows : 0;
        }
        TileDesc* segs = tiles + rows_pad;
        for (int off = 0; off < nrows; off += TILE_ROWS) {
            TileDesc d;
            d.seq = seq; d.rng = rng;
            d.pos0 = pos0 + off;
            d.n_valid = min(TILE_ROWS, nrows - off);
            d.prow0 = first + off;
            if (store_base < 0) {
                d.zrow0 = d.erow0 = d.yrow0 = c + off;
            } else {
                d.zrow0 = d.yrow0 = (int)(store_base + d.pos0);
                d.erow0 = d.prow0;
            }
            d.crow0 = c + off;
            const int k = off / TILE_ROWS, left = (nrows - off + TILE_ROWS - 1) / TILE_ROWS;
            d.group = (k % ATT_GROUP == 0) ? min(ATT_GROUP, left) : 0;
            if (d.group > 0) n_tiles[TILE_LEADERS + n_lead++] = n_seg;
            if (n_seg < TILE_LDS_SEGS) sh_segs[n_seg] = d;
            segs[n_seg++] = d;
        }
        c += nrows;
        return first;
    }
    // counts and (up to TILE_LDS_SEGS) segments also go to LDS, so that the other threads of the workgroup
    // need no trip through memory to write the row descriptors
    __device__ void counts(int* sh_counts) {
        n_tiles[0] = n_phys; n_tiles[1] = n_lead; n_tiles[2] = n_seg;
        sh_counts[0] = n_phys; sh_counts[1] = n_seg;
    }
    // all threads, after a barrier behind counts(): the descriptor of every physical row
    __device__ void rows(const int* sh_counts, const TileDesc* sh_segs) {
        const int np = sh_counts[0], ns = sh_counts[1];
        TileDesc pad;
        pad.seq = 0; pad.pos0 = 0; pad.n_valid = 0; pad.zrow0 = pad.erow0 = pad.yrow0 = pad.crow0 = 0; pad.group = 0; pad.rng = 0;
        if (ns <= TILE_LDS_SEGS) {
            // one pass: every row looks its segment up in LDS (segments are in ascending row order)
            for (int r = threadIdx.x; r < np * TILE_ROWS; r += blockDim.x) {
                int found = -1;
                for (int sg = 0; sg < ns; ++sg) {
                    const int p0 = sh_segs[sg].prow0;
                    if (r >= p0 && r < p0 + sh_segs[sg].n_valid) found = sg;
                }
                const int sg = max(found, 0);
                const int j = r - sh_segs[sg].prow0;
                const bool ok = found >= 0;
                TileDesc rd;
                rd.seq = ok ? sh_segs[sg].seq : 0;
                rd.pos0 = ok ? sh_segs[sg].pos0 + j : 0;
                rd.n_valid = ok ? 1 : 0;
                rd.zrow0 = ok ? sh_segs[sg].zrow0 + j : 0;
                rd.erow0 = ok ? sh_segs[sg].erow0 + j : 0;
                rd.yrow0 = ok ? sh_segs[sg].yrow0 + j : 0;
                rd.crow0 = ok ? sh_segs[sg].crow0 + j : 0;
                rd.group = 0;
                rd.rng = ok ? sh_segs[sg].rng : 0;
                rd.prow0 = r;
                tiles[r] = rd;
            }
            return;
        }
        for (int r = threadIdx.x; r < np * TILE_ROWS; r += blockDim.x) { pad.prow0 = r; tiles[r] = pad; }
        __syncthreads();
        const TileDesc* segs = tiles + rows_pad;
        for (int sg = 0; sg < ns; ++sg) {
            const TileDesc d = segs[sg];
            for (int j = threadIdx.x; j < d.n_valid; j += blockDim.x) {
                TileDesc rd = d;
                rd.pos0 += j; rd.zrow0 += j; rd.erow0 += j; rd.yrow0 += j; rd.crow0 += j; rd.prow0 += j;
                rd.n_valid = 1; rd.group = 0;
                tiles[d.prow0 + j] = rd;
            }
        }
    }
};

__global__ void build_tiles_api_k(SeqWindows w, const int32_t* ident, int mode, int max_positions, TileDesc* tiles,
                                  int32_t* n_tiles, int rows_pad, int pack) {
    __shared__ int sh_counts[2];
    __shared__ TileDesc sh_segs[TILE_LDS_SEGS];
    TileLayout lay;
    lay.tiles = tiles; lay.n_tiles = n_tiles; lay.rows_pad = rows_pad; lay.pack = pack; lay.sh_segs = sh_segs;
    if (threadIdx.x == 0) {
        for (int i = 0; i < w.n; ++i)
            lay.add(w.seq[i], ident[w.seq[i]], w.pos0[i], w.rows[i], mode == 0 ? -1LL : (long long)w.seq[i] * max_positions);
        lay.counts(sh_counts);
    }
    __syncthreads();
    lay.rows(sh_counts, sh_segs);
}

__global__ void build_tiles_sampler_k(SeqState* seqs, const int32_t* ident, int n_seqs, int max_positions,
                                      TileDesc* tiles, int32_t* n_tiles, int rows_pad, int pack) {
    __shared__ int sh_counts[2];
    __shared__ TileDesc sh_segs[TILE_LDS_SEGS];
    TileLayout lay;
    lay.tiles = tiles; lay.n_tiles = n_tiles; lay.rows_pad = rows_pad; lay.pack = pack; lay.sh_segs = sh_segs;
    if (threadIdx.x == 0) {
        for (int s = 0; s < n_seqs; ++s) {
            SeqState& q = seqs[s];
            const int rows = q.done ? 0 : q.win_n;
            q.cur_rows = rows;
            q.cur_row0 = lay.add(s, ident[s], q.win_pos0, rows, (long long)s * max_positions);
        }
        lay.counts(sh_counts);
    }
    __syncthreads();
    lay.rows(sh_counts, sh_segs);
}

// ---------------------------------------------------------------------------------------------
// Embedding gather, a row cut into `chunks` workgroups; chunk 0 also writes the row's RoPE table.
template <typename T>
__global__ void embed_k(const T* emb, const int32_t* tokens, float scale, float* x, int h, int V, int chunks,
                        float2* rope_table, const float* theta, int half, const float* gain, void* xg, float* ssq,
                        size_t ssq_stride, const TileDesc* tiles, const int32_t* n_tiles) {
    __shared__ float sh[16];
    int r = blockIdx.y, c = blockIdx.x, j = 0;          // (the row's own descriptor: offsets within it are 0)
    if ((r >> 5) >= *n_tiles) return;
    TileDesc d = tiles[r];
    bool valid = j < d.n_valid;
    int tok = valid ? tokens[d.yrow0 + j] : 0;
    tok = min(max(tok, 0), V - 1);
    const int cw = (h + chunks - 1) / chunks;
    float ss = 0.f;
    for (int k = c * cw + threadIdx.x; k < min(h, (c + 1) * cw); k += blockDim.x) {
        float v = 0.f;
        if (valid) {
            if (sizeof(T) == 2) v = bf16_to_f32(reinterpret_cast<const uint16_t*>(emb)[(size_t)tok * h + k]);
            else v = reinterpret_cast<const float*>(emb)[(size_t)tok * h + k];
        }
        v *= scale;
        x[(size_t)r * h + k] = v;
        if (xg) {                 // operand of the first layer's norm, 1/rms left to the consuming GEMM
            reinterpret_cast<uint16_t*>(xg)[packed_off(r, k, h)] = f32_to_bf16(v * gain[k]);
            ss += v * v;
        }
    }
    if (xg) {
        ss = block_sum(ss, sh);
        if (threadIdx.x == 0) ssq[(size_t)c * ssq_stride + r] = ss;
    }
    if (rope_table && c == 0) {
        const int pos = d.pos0 + j;
        for (int i = threadIdx.x; i < half; i += blockDim.x) {
            float sn, cs;
            sincosf((float)pos * theta[i], &sn, &cs);
            rope_table[(size_t)r * half + i] = make_float2(cs, sn);
        }
    }
}

__global__ void copy_rows_in_k(const float* src, float* x, int h, int which, const TileDesc* tiles,
                               const int32_t* n_tiles) {
    int r = blockIdx.x, j = 0;          // (the row's own descriptor: offsets within it are 0)
    if ((r >> 5) >= *n_tiles) return;
    TileDesc d = tiles[r];
    bool valid = j < d.n_valid;
    size_t srow = (size_t)(which == 0 ? d.zrow0 : d.erow0) + j;
    for (int k = threadIdx.x * 4; k < h; k += blockDim.x * 4) {
        float4 v = valid ? ld4(src + srow * h + k) : make_float4(0, 0, 0, 0);
        *reinterpret_cast<float4*>(x + (size_t)r * h + k) = v;
    }
}

__global__ void copy_rows_out_k(const float* x, float* dst, int width, int which, const TileDesc* tiles,
                                const int32_t* n_tiles) {
    int r = blockIdx.x, j = 0;          // (the row's own descriptor: offsets within it are 0)
    if ((r >> 5) >= *n_tiles) return;
    TileDesc d = tiles[r];
    if (j >= d.n_valid) return;
    size_t drow = (size_t)(which == 0 ? d.zrow0 : which == 1 ? d.erow0 : d.crow0) + j;
    for (int k = threadIdx.x; k < width; k += blockDim.x)
        dst[drow * width + k] = x[(size_t)r * width + k];
}

__global__ void copy_i32_out_k(const int32_t* src, int32_t* dst, const TileDesc* tiles, const int32_t* n_tiles) {
    int r = blockIdx.x * blockDim.x + threadIdx.x, j = 0;          // (the row's own descriptor: offsets within it are 0)
    if ((r >> 5) >= *n_tiles) return;
    TileDesc d = tiles[r];
    if (j < d.n_valid) dst[d.crow0 + j] = src[r];
}

template <int FMT>
__global__ void concat_k(const float* e, const float* z, void* cat, int h, const TileDesc* tiles,
                         const int32_t* n_tiles) {
    int r = blockIdx.x, j = 0;          // (the row's own descriptor: offsets within it are 0)
    if ((r >> 5) >= *n_tiles) return;
    TileDesc d = tiles[r];
    bool valid = j < d.n_valid;
    if (!e || !z) {      // one half alone, as an operand of width h (adapter product cut in two)
        const float* sr = e ? e + ((size_t)d.erow0 + j) * h : z + ((size_t)d.zrow0 + j) * h;
        for (int k = threadIdx.x * 4; k < h; k += blockDim.x * 4) {
            float4 v = make_float4(0, 0, 0, 0);
            if (valid) v = ld4(sr + k);
            act_store4<FMT>(cat, h, r, k, v.x, v.y, v.z, v.w);
        }
        return;
    }
    const float* er = e + ((size_t)d.erow0 + j) * h;
    const float* zr = z + ((size_t)d.zrow0 + j) * h;
    for (int k = threadIdx.x * 4; k < 2 * h; k += blockDim.x * 4) {
        float4 v = make_float4(0, 0, 0, 0);
        if (valid) v = (k < h) ? ld4(er + k) : ld4(zr + (k - h));
        act_store4<FMT>(cat, 2 * h, r, k, v.x, v.y, v.z, v.w);
    }
}

// x_out = x_in + sum_s part[s];  xn = x_out * gain / sqrt(mean(x_out^2) + eps).
// One workgroup per row; the row stays in registers between the reduction and the stores
// (up to ROW_VEC float4 per thread, i.e. h <= 256*4*ROW_VEC).
constexpr int ROW_VEC = 8;

__device__ inline float4 row_value(const float* xin, const float* part, int S, size_t part_stride, size_t off) {
    float4 v = xin ? ld4(xin + off) : make_float4(0, 0, 0, 0);
    for (int s = 0; s < S; ++s) {
        float4 p = ld4(part + s * part_stride + off);
        v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    return v;
}

template <int FMT>
__global__ __launch_bounds__(256) void addnorm_k(const float* xin, float* xout, const float* part, int S,
                                                  size_t part_stride, const float* gain, void* xn, int h, float eps,
                                                  const int32_t* n_tiles) {
    __shared__ float sh[16];
    int r = blockIdx.x;
    if ((r >> 5) >= *n_tiles) return;
    float4 v[ROW_VEC];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < ROW_VEC; ++i) {
        int k = (threadIdx.x + i * 256) * 4;
        if (k < h) {
            v[i] = row_value(xin, part, S, part_stride, (size_t)r * h + k);
            ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
        }
    }
    ss = block_sum(ss, sh);
    float inv = 1.0f / sqrtf(ss / (float)h + eps);
#pragma unroll
    for (int i = 0; i < ROW_VEC; ++i) {
        int k = (threadIdx.x + i * 256) * 4;
        if (k < h) {
            if (xout) *reinterpret_cast<float4*>(xout + (size_t)r * h + k) = v[i];
            if (xn) {
                float4 g = ld4(gain + k);
                act_store4<FMT>(xn, h, r, k, v[i].x * inv * g.x, v[i].y * inv * g.y, v[i].z * inv * g.z,
                                v[i].w * inv * g.w);
            }
        }
    }
}

// End of the prelude on the bf16 path: e = x + sum part (f32, padded rows) and the adapter operand
// concat(e, z) as packed bf16 in one pass; a row is cut into `chunks` pieces like fold_k.
__global__ __launch_bounds__(256) void prelude_end_k(const float* xin, const float* part, int S, size_t part_stride,
                                                      float* e_out, const float* z, void* cat, void* cat_e, int h,
                                                      int chunks, const TileDesc* tiles, const int32_t* n_tiles) {
    const int r = blockIdx.y, c = blockIdx.x, j = 0;   // (the row's own descriptor: offsets within it are 0)
    if ((r >> 5) >= *n_tiles) return;
    const TileDesc d = tiles[r];
    const bool valid = j < d.n_valid;
    const int cw = h / chunks;
    const int k = c * cw + threadIdx.x * 4;
    if ((int)threadIdx.x * 4 >= cw) return;
    float4 v = row_value(xin, part, S, part_stride, (size_t)r * h + k);
    *reinterpret_cast<float4*>(e_out + (size_t)r * h + k) = v;
    float4 zz = make_float4(0, 0, 0, 0);
    if (valid) zz = ld4(z + ((size_t)d.zrow0 + j) * h + k);
    else v = make_float4(0, 0, 0, 0);
    if (cat_e) {         // the two halves as operands of their own (adapter product cut in two)
        act_store4<ACT_BF16P>(cat_e, h, r, k, v.x, v.y, v.z, v.w);
        act_store4<ACT_BF16P>(cat, h, r, k, zz.x, zz.y, zz.z, zz.w);
        return;
    }
    act_store4<ACT_BF16P>(cat, 2 * h, r, k, v.x, v.y, v.z, v.w);
    act_store4<ACT_BF16P>(cat, 2 * h, r, h + k, zz.x, zz.y, zz.z, zz.w);
}

// Residual add + split-K fold with the RMS factor left to the consumer: a row is cut into
// `chunks` pieces handled by different workgroups; each writes x_out, bf16(x_out * gain) in the
// packed operand layout and its piece of the row's sum of squares.
__global__ __launch_bounds__(256) void fold_k(const float* xin, float* xout, const float* part, int S,
                                               size_t part_stride, const float* gain, void* xg, float* ssq,
                                               size_t ssq_stride, int h, int chunks, const int32_t* n_tiles) {
    __shared__ float sh[16];
    const int r = blockIdx.y, c = blockIdx.x;
    if ((r >> 5) >= *n_tiles) return;
    const int cw = h / chunks;
    const int k = c * cw + threadIdx.x * 4;
    float ss = 0.f;
    if ((int)threadIdx.x * 4 < cw) {
        float4 v = row_value(xin, part, S, part_stride, (size_t)r * h + k);
        ss = v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
        if (xout) *reinterpret_cast<float4*>(xout + (size_t)r * h + k) = v;
        if (xg) {
            float4 g = ld4(gain + k);
            act_store4<ACT_BF16P>(xg, h, r, k, v.x * g.x, v.y * g.y, v.z * g.z, v.w * g.w);
        }
    }
    ss = block_sum(ss, sh);
    if (threadIdx.x == 0 && ssq) ssq[(size_t)c * ssq_stride + r] = ss;
}

// End of a recurrence: z' = RMSNorm(x + sum part) * gain, stored to the latent array; optionally
// delta = ||z' - z_prev|| / ||z'|| (Eq. 3) and z_prev <- z'.
template <int NT>
__global__ __launch_bounds__(NT) void final_norm_k(const float* xin, const float* part, int S, size_t part_stride,
                                                     const float* gain, int h, float eps, float* z, float* z_prev,
                                                     int update_prev, float* delta, float* xcopy, const float* gain2,
                                                     void* xg, float* ssq_tot, const TileDesc* tiles,
                                                     const int32_t* n_tiles) {
    __shared__ float sh[16];
    int r = blockIdx.x, j = 0;          // (the row's own descriptor: offsets within it are 0)
    if ((r >> 5) >= *n_tiles) return;
    TileDesc d = tiles[r];
    bool valid = j < d.n_valid;
    constexpr int RV = ROW_VEC * 256 / NT;          // float4 per thread: h <= 8192
    float4 v[RV];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < RV; ++i) {
        int k = (threadIdx.x + i * NT) * 4;
        if (k < h) {
            v[i] = row_value(xin, part, S, part_stride, (size_t)r * h + k);
            ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
        }
    }
    ss = block_sum(ss, sh);
    float inv = 1.0f / sqrtf(ss / (float)h + eps);
    float num = 0.f, den = 0.f;
    size_t zr = (size_t)d.zrow0 + j;
#pragma unroll
    for (int i = 0; i < RV; ++i) {
        int k = (threadIdx.x + i * NT) * 4;
        if (k < h && !valid && xcopy) {
            *reinterpret_cast<float4*>(xcopy + (size_t)r * h + k) = make_float4(0, 0, 0, 0);
            if (xg) act_store4<ACT_BF16P>(xg, h, r, k, 0.f, 0.f, 0.f, 0.f);
        }
        if (k < h && valid) {
            float4 g = ld4(gain + k);
            float4 o = make_float4(v[i].x * inv * g.x, v[i].y * inv * g.y, v[i].z * inv * g.z, v[i].w * inv * g.w);
            if (z_prev) {
                float4 p = ld4(z_prev + zr * h + k);
                num += (o.x - p.x) * (o.x - p.x) + (o.y - p.y) * (o.y - p.y) + (o.z - p.z) * (o.z - p.z) +
                       (o.w - p.w) * (o.w - p.w);
                if (update_prev) *reinterpret_cast<float4*>(z_prev + zr * h + k) = o;
            }
            den += o.x * o.x + o.y * o.y + o.z * o.z + o.w * o.w;
            *reinterpret_cast<float4*>(z + zr * h + k) = o;
            if (xcopy) *reinterpret_cast<float4*>(xcopy + (size_t)r * h + k) = o;
            if (xg) {             // operand of the coda's first norm (gain2), 1/rms left to the consuming GEMM
                float4 g2 = ld4(gain2 + k);
                act_store4<ACT_BF16P>(xg, h, r, k, o.x * g2.x, o.y * g2.y, o.z * g2.z, o.w * g2.w);
            }
        }
    }
    if (delta || xg) {
        num = block_sum(num, sh);
        den = block_sum(den, sh);
        if (threadIdx.x == 0) {
            if (delta) delta[r] = valid ? sqrtf(num) / sqrtf(den) : 0.f;
            if (xg) ssq_tot[r] = den;                       // sum of z'^2 over the row (0 for padding rows)
        }
    }
}

// cos / sin of pos * theta_i for every row of the step, computed once per step.
__global__ void rope_table_k(float2* table, const float* theta, int half, const TileDesc* tiles,
                             const int32_t* n_tiles) {
    int r = blockIdx.x;
    if ((r >> 5) >= *n_tiles) return;
    int pos = tiles[r].pos0;
    for (int i = threadIdx.x; i < half; i += blockDim.x) {
        float sn, cs;
        sincosf((float)pos * theta[i], &sn, &cs);
        table[(size_t)r * half + i] = make_float2(cs, sn);
    }
}

// RoPE (rotate-half pairs (i, i+d/2), angle pos * theta_i) on q and k; q is written for the
// attention kernel, k and v are written into the layer's cache at the row's position,
// replacing what an earlier recurrence or sampler step left there.  One workgroup per
// (head, tile); v goes through LDS so that the writes into the transposed bf16 V cache walk the
// 32 positions of a block together.
template <int DT>
__global__ __launch_bounds__(256) void rope_kv_k(const float* qkv, int S, size_t part_stride, void* qout, void* kc,
                                                  void* vc, int H, int d, const float2* table, KvPages kv,
                                                  const TileDesc* tiles, const int32_t* n_tiles) {
    extern __shared__ float sv[];                       // [32][d + 1]
    const int hd = blockIdx.x, t = blockIdx.y;          // physical row tile: its rows may belong to several sequences
    if (t >= *n_tiles) return;
    const TileDesc* rowd = tiles + (size_t)t * 32;
    const int h = H * d, half = d >> 1;
    auto at = [&](int row, int colidx) {
        float v = 0.f;
        for (int s = 0; s < S; ++s) v += qkv[s * part_stride + (size_t)row * 3 * h + colidx];
        return v;
    };
    for (int idx = threadIdx.x; idx < 32 * half; idx += blockDim.x) {
        const int j = idx / half, i = idx - j * half;
        const TileDesc ds = rowd[j];
        const int r = t * 32 + j, pos = ds.pos0;
        const bool valid = ds.n_valid > 0;
        const float2 cssn = table[(size_t)r * half + i];
        const int c0 = hd * d + i, c1 = c0 + half;
        const float q0 = at(r, c0), q1 = at(r, c1), k0 = at(r, h + c0), k1 = at(r, h + c1);
        const float qa = q0 * cssn.x - q1 * cssn.y, qb = q1 * cssn.x + q0 * cssn.y;
        const float ka = k0 * cssn.x - k1 * cssn.y, kb = k1 * cssn.x + k0 * cssn.y;
        sv[j * (d + 1) + i] = at(r, 2 * h + c0);
        sv[j * (d + 1) + i + half] = at(r, 2 * h + c1);
        if (DT == 0) {
            float* q = reinterpret_cast<float*>(qout);
            q[(size_t)r * h + c0] = qa; q[(size_t)r * h + c1] = qb;
            if (valid) {
                float* K = reinterpret_cast<float*>(kc) + kv_block_base(kv, ds.seq, pos >> 5, (size_t)32 * h) +
                           (size_t)(pos & 31) * h;
                K[c0] = ka; K[c1] = kb;
            }
        } else {
            uint16_t* q = reinterpret_cast<uint16_t*>(qout);
            q[(size_t)r * h + c0] = f32_to_bf16(qa); q[(size_t)r * h + c1] = f32_to_bf16(qb);
            if (valid) {
                uint16_t* K = reinterpret_cast<uint16_t*>(kc) + kv_block_base(kv, ds.seq, pos >> 5, (size_t)32 * h);
                K[k_cache_off(pos & 31, hd, i, H, d)] = f32_to_bf16(ka);
                K[k_cache_off(pos & 31, hd, i + half, H, d)] = f32_to_bf16(kb);
            }
        }
    }
    __syncthreads();
    if (DT == 0) {
        for (int idx = threadIdx.x; idx < 32 * d; idx += blockDim.x) {
            const int j = idx / d, dd = idx - j * d;
            const TileDesc ds = rowd[j];
            if (ds.n_valid > 0) {
                const int pos = ds.pos0;
                reinterpret_cast<float*>(vc)[kv_block_base(kv, ds.seq, pos >> 5, (size_t)32 * h) + (size_t)(pos & 31) * h +
                                             hd * d + dd] = sv[j * (d + 1) + dd];
            }
        }
    } else {
        // transposed V: [position block][head][dim][32 slots]; lanes run over the rows of the tile
        for (int idx = threadIdx.x; idx < 32 * d; idx += blockDim.x) {
            const int dd = idx >> 5, j = idx & 31;
            const TileDesc ds = rowd[j];
            const int pos = ds.pos0;
            if (ds.n_valid > 0)
                reinterpret_cast<uint16_t*>(vc)[kv_block_base(kv, ds.seq, pos >> 5, (size_t)32 * h) +
                                                ((size_t)hd * d + dd) * 32 + vt_slot(pos & 31)] =
                    f32_to_bf16(sv[j * (d + 1) + dd]);
        }
    }
}

template <int FMT>
__global__ void swiglu_k(const float* gu, int S, size_t part_stride, void* act, int F, const int32_t* n_tiles) {
    int r = blockIdx.y;
    if ((r >> 5) >= *n_tiles) return;
    int k = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (k >= F) return;
    float4 g = make_float4(0, 0, 0, 0), u = g;
    for (int s = 0; s < S; ++s) {
        float4 a = ld4(gu + s * part_stride + (size_t)r * 2 * F + k);
        float4 b = ld4(gu + s * part_stride + (size_t)r * 2 * F + F + k);
        g.x += a.x; g.y += a.y; g.z += a.z; g.w += a.w;
        u.x += b.x; u.y += b.y; u.z += b.z; u.w += b.w;
    }
    auto f = [](float a, float b) { return a / (1.0f + expf(-a)) * b; };
    act_store4<FMT>(act, F, r, k, f(g.x, u.x), f(g.y, u.y), f(g.z, u.z), f(g.w, u.w));
}

// ---------------------------------------------------------------------------------------------
// InitState: four normals per Philox block through two Box-Muller pairs.
__device__ inline void gauss4(uint32_t blk, uint32_t pos, uint32_t seq, uint32_t k0, uint32_t k1, float alpha,
                              float out[4], uint32_t c3 = TAG_INIT_STATE) {
    uint32_t x[4];
    philox4x32_10(blk, pos, seq, c3, k0, k1, x);
    for (int p = 0; p < 2; ++p) {
        float ua = u24_open(x[2 * p]), ub = u24_open(x[2 * p + 1]);
        float rad = sqrtf(-2.0f * logf(ua));
        float sn, cs;
        sincospif(2.0f * ub, &sn, &cs);
        out[2 * p] = alpha * rad * cs;
        out[2 * p + 1] = alpha * rad * sn;
    }
}

__global__ void init_state_rows_k(float* z, float* z_prev, int h, int seq, int pos0, int n, size_t zrow0,
                                  float alpha, uint32_t k0, uint32_t k1) {
    int row = blockIdx.y;
    int blk = blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= n || blk * 4 >= h) return;
    float g[4];
    gauss4(blk, pos0 + row, seq, k0, k1, alpha, g);
    for (int i = 0; i < 4 && blk * 4 + i < h; ++i) {
        size_t o = (zrow0 + row) * h + blk * 4 + i;
        z[o] = g[i];
        if (z_prev) z_prev[o] = g[i];
    }
}

// Momentum on the conditioning (Eq. 1), one workgroup per row.
__global__ void momentum_k(float* e, float* e_store, const int32_t* counts, float eta, int h, const TileDesc* tiles,
                           const int32_t* n_tiles) {
    int r = blockIdx.x, j = 0;          // (the row's own descriptor: offsets within it are 0)
    if ((r >> 5) >= *n_tiles) return;
    TileDesc d = tiles[r];
    if (j >= d.n_valid) return;
    const size_t srow = (size_t)d.zrow0 + j;               // (sequence, position) row of the stores
    const bool first = counts[srow] == 0;                   // no previous conditioning yet
    float* er = e + ((size_t)d.erow0 + j) * h;
    float* pr = e_store + srow * h;
    for (int k = threadIdx.x * 4; k < h; k += blockDim.x * 4) {
        float4 v = ld4(er + k);
        if (!first) {
            float4 p = ld4(pr + k);
            v.x = eta * p.x + (1.0f - eta) * v.x; v.y = eta * p.y + (1.0f - eta) * v.y;
            v.z = eta * p.z + (1.0f - eta) * v.z; v.w = eta * p.w + (1.0f - eta) * v.w;
            *reinterpret_cast<float4*>(er + k) = v;
        }
        *reinterpret_cast<float4*>(pr + k) = v;
    }
}

// Scheduled state noise (Eq. 2), one workgroup per row, in place on the latent store.
__global__ void noise_mix_k(float* z, const int32_t* counts, float beta, int n_steps, float alpha, uint32_t k0,
                            uint32_t k1, int step, const int32_t* seq_step0, int h, const TileDesc* tiles,
                            const int32_t* n_tiles) {
    int r = blockIdx.x, j = 0;          // (the row's own descriptor: offsets within it are 0)
    if ((r >> 5) >= *n_tiles) return;
    TileDesc d = tiles[r];
    if (j >= d.n_valid) return;
    const size_t srow = (size_t)d.zrow0 + j;
    const float b = beta * fmaxf(0.0f, 1.0f - (float)counts[srow] / (float)n_steps);
    if (b == 0.0f) return;
    const int lstep = step - (seq_step0 ? seq_step0[d.seq] : 0);
    float* zr = z + srow * h;
    for (int blk = threadIdx.x; blk * 4 < h; blk += blockDim.x) {
        float g[4];
        gauss4(blk, d.pos0 + j, d.rng, k0, k1, alpha, g, ((uint32_t)lstep << 4) | TAG_NOISE);
        for (int i = 0; i < 4 && blk * 4 + i < h; ++i) zr[blk * 4 + i] = (1.0f - b) * zr[blk * 4 + i] + b * g[i];
    }
}

// Sample: greedy or Gumbel-max, one workgroup per row; lowest token id wins ties.
__global__ void sample_k(const float* logits, int V, float temperature, uint32_t k0, uint32_t k1, int step,
                         const int32_t* seq_step0, int32_t* tok_out, const TileDesc* tiles, const int32_t* n_tiles) {
    __shared__ float sv[256];
    __shared__ int si[256];
    int r = blockIdx.x, j = 0;          // (the row's own descriptor: offsets within it are 0)
    if ((r >> 5) >= *n_tiles) return;
    TileDesc d = tiles[r];
    int pos = d.pos0 + j;
    const float* lg = logits + (size_t)r * V;
    float best = -INFINITY;
    int bi = 0x7fffffff;
    for (int b = threadIdx.x; b * 4 < V; b += blockDim.x) {
        float g[4] = {0.f, 0.f, 0.f, 0.f};
        if (temperature > 0.f) {
            uint32_t x[4];
            philox4x32_10(b, pos, d.rng, ((uint32_t)(step - (seq_step0 ? seq_step0[d.seq] : 0)) << 4) | TAG_SAMPLE, k0, k1, x);
            for (int i = 0; i < 4; ++i) g[i] = -logf(-logf(u24_open(x[i])));
        }
        for (int i = 0; i < 4 && b * 4 + i < V; ++i) {
            float sc = lg[b * 4 + i];
            if (temperature > 0.f) sc = sc / temperature + g[i];
            if (sc > best) { best = sc; bi = b * 4 + i; }      // ascending ids: first maximum kept
        }
    }
    sv[threadIdx.x] = best; si[threadIdx.x] = bi;
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

// Sample with a top-p filter (the paper's runs: temperature 0.2, top-p 0.95), one workgroup of
// 1024 threads per row, up to 65536 classes held in registers as e_v = exp(logit_v / T - max).
// The kept set is {v : e_v >= thr} with thr the largest value whose tail mass
// sum_{e_v >= thr} e_v reaches top_p * sum_v e_v -- found by bisection on the bit pattern of thr
// (the mass is a step function of thr that only changes at the e_v), every mass summed in a
// fixed order.  The Gumbel race among the kept classes draws from the renormalised nucleus.
constexpr int TOPP_THREADS = 1024, TOPP_VEC = 16, TOPP_CAND = 1024;
__device__ inline float block_max(float v, float* sh) {
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[w] = v;
    __syncthreads();
    float t = -INFINITY;
    for (int i = 0; i < (int)(blockDim.x >> 6); ++i) t = fmaxf(t, sh[i]);
    return t;
}
__global__ __launch_bounds__(TOPP_THREADS) void sample_top_p_k(const float* logits, int V, float temperature,
                                                                float top_p, uint32_t k0, uint32_t k1, int step,
                                                                const int32_t* seq_step0, int32_t* tok_out,
                                                                const TileDesc* tiles, const int32_t* n_tiles) {
    __shared__ float sh[16];
    __shared__ float sv[16];
    __shared__ int si[16];
    __shared__ int wtot[TOPP_THREADS / 64];
    __shared__ float cand[TOPP_CAND];
    __shared__ uint32_t thr_sh;
    const int r = blockIdx.x, j = 0;          // (the row's own descriptor: offsets within it are 0)
    if ((r >> 5) >= *n_tiles) return;
    const TileDesc d = tiles[r];
    const int pos = d.pos0 + j;
    const float* lg = logits + (size_t)r * V;
    const float invT = 1.0f / temperature;
    float e[TOPP_VEC][4];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < TOPP_VEC; ++i) {
        const int v0 = (i * TOPP_THREADS + threadIdx.x) * 4;
        if (v0 < V) {
            const float4 l = ld4(lg + v0);
            e[i][0] = l.x * invT; e[i][1] = l.y * invT; e[i][2] = l.z * invT; e[i][3] = l.w * invT;
        } else {
            e[i][0] = e[i][1] = e[i][2] = e[i][3] = -INFINITY;
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) mx = fmaxf(mx, e[i][c]);
    }
    mx = block_max(mx, sh);
    float part = 0.f;
#pragma unroll
    for (int i = 0; i < TOPP_VEC; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) { e[i][c] = __expf(e[i][c] - mx); part += e[i][c]; }
    const float total = block_sum(part, sh);
    const float target = top_p * total;
    // The classes below floor = (1 - top_p) total / V hold less than (1 - top_p) total together,
    // so the cut lies at or above it (half of it is used, to stay clear of rounding).  Usually only
    // a few classes reach that: when no more than TOPP_CAND do, they are compacted (in a fixed
    // order) into LDS and one wave runs the bisection over them with wave-level sums; otherwise
    // the whole workgroup bisects over the values in registers.
    const float floor_e = 0.5f * (1.0f - top_p) * total / (float)V;
    int mine = 0;
#pragma unroll
    for (int i = 0; i < TOPP_VEC; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) mine += e[i][c] >= floor_e ? 1 : 0;
    // exclusive prefix sum of the per-thread counts (wave scan, then the waves' totals)
    int incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o);
        if ((int)(threadIdx.x & 63) >= o) incl += up;
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 63) wtot[threadIdx.x >> 6] = incl;
    __syncthreads();
    int before = 0, n_cand = 0;
#pragma unroll
    for (int w = 0; w < TOPP_THREADS / 64; ++w) {
        if (w < (int)(threadIdx.x >> 6)) before += wtot[w];
        n_cand += wtot[w];
    }
    uint32_t lo = __float_as_uint(floor_e) & 0x7fffffffu, hi = 0x3f800001u;   // mass(floor) >= target; e_v <= 1
    if (n_cand > 0 && n_cand <= TOPP_CAND) {
        int at = before + incl - mine;
#pragma unroll
        for (int i = 0; i < TOPP_VEC; ++i)
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (e[i][c] >= floor_e) cand[at++] = e[i][c];
        for (int q = n_cand + threadIdx.x; q < TOPP_CAND; q += TOPP_THREADS) cand[q] = 0.f;
        __syncthreads();
        if (threadIdx.x < 64) {
            float v[TOPP_CAND / 64];
#pragma unroll
            for (int q = 0; q < TOPP_CAND / 64; ++q) v[q] = cand[q * 64 + threadIdx.x];
            while (hi - lo > 1u) {
                const uint32_t mid = lo + ((hi - lo) >> 1);
                const float thr = __uint_as_float(mid);
                float m = 0.f;
#pragma unroll
                for (int q = 0; q < TOPP_CAND / 64; ++q) m += v[q] >= thr ? v[q] : 0.f;
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) m += __shfl_xor(m, o);    // every lane ends with the same sum
                if (m >= target) lo = mid; else hi = mid;
            }
            if (threadIdx.x == 0) thr_sh = lo;
        }
        __syncthreads();
        lo = thr_sh;
    } else {
        lo = n_cand > 0 ? lo : 0u;                         // nothing reached the floor (not finite): search from +0
        while (hi - lo > 1u) {
            const uint32_t mid = lo + ((hi - lo) >> 1);
            const float thr = __uint_as_float(mid);
            float m = 0.f;
#pragma unroll
            for (int i = 0; i < TOPP_VEC; ++i)
#pragma unroll
                for (int c = 0; c < 4; ++c) m += e[i][c] >= thr ? e[i][c] : 0.f;
            m = block_sum(m, sh);
            if (m >= target) lo = mid; else hi = mid;
        }
    }
    const float thr = __uint_as_float(lo);
    const int lstep = step - (seq_step0 ? seq_step0[d.seq] : 0);
    float best = -INFINITY;
    int bi = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < TOPP_VEC; ++i) {
        const int v0 = (i * TOPP_THREADS + threadIdx.x) * 4;
        if (v0 >= V) continue;
        bool any = false;
#pragma unroll
        for (int c = 0; c < 4; ++c) any = any || e[i][c] >= thr;
        if (!any) continue;
        uint32_t x[4];
        philox4x32_10(v0 >> 2, pos, d.rng, ((uint32_t)lstep << 4) | TAG_SAMPLE, k0, k1, x);
        const float4 l = ld4(lg + v0);
        const float lv[4] = {l.x, l.y, l.z, l.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (e[i][c] >= thr) {
                const float sc = lv[c] / temperature + (-logf(-logf(u24_open(x[c]))));
                if (sc > best) { best = sc; bi = v0 + c; }     // ascending ids: first maximum kept
            }
        }
    }
    // lowest id wins ties: reduce (value, id) over the workgroup
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(best, o);
        const int oi = __shfl_xor(bi, o);
        if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = best; si[threadIdx.x >> 6] = bi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < TOPP_THREADS / 64; ++w)
            if (sv[w] > best || (sv[w] == best && si[w] < bi)) { best = sv[w]; bi = si[w]; }
        tok_out[r] = bi == 0x7fffffff ? 0 : bi;
    }
}

// End of a sampler step, one workgroup per sequence (its rows in parallel): the drafts become
// y_current and the step counters advance (Alg. 1, assign), the longest freezable prefix k* is
// frozen (Alg. 1 freeze / Eq. 3), new states are appended unless the wavefront is full (Alg. 1
// append, Alg. 2) and drawn (InitState).  The last workgroup to finish then builds the tile list
// of the next step from all updated windows: the sequence records are handed over with
// system-scope stores and loads around a ticket (no device-scope fence), as the GEMM folds are.
__global__ __launch_bounds__(1024) void step_end_k(SeqState* seqs, const int32_t* ident, int n_seqs, SamplerParams p, int32_t* y,
                                                   int32_t* counts, int max_positions, const int32_t* drafts,
                                                   const float* delta, float* z, float* z_prev, int h,
                                                   TileDesc* tiles, int32_t* n_tiles, int32_t* n_active, int step,
                                                   uint32_t* ticket_ctr, int rows_pad, int pack) {
    __shared__ int first_open;                       // first row of the window that is not freezable
    __shared__ SeqState cur;
    __shared__ uint32_t ticket;
    constexpr int NF = sizeof(SeqState) / sizeof(int32_t);
    const int tid = threadIdx.x;
    const int s = blockIdx.x;
    if (s < n_seqs) {
        if (tid == 0) { cur = seqs[s]; first_open = 0x7fffffff; }
        __syncthreads();
        SeqState q = cur;
        const int rows = q.cur_rows;                 // rows this sequence had in the step just run
        const size_t base = (size_t)s * max_positions;
        if (!q.done && rows > 0) {
            const int row0 = q.cur_row0;                // its rows are contiguous in physical row space
            for (int i = tid; i < rows; i += blockDim.x) {
                const int pos = q.win_pos0 + i;
                y[base + pos + 1] = drafts[row0 + i];                    // y_current <- [y_frozen, y_hat]
                const int c = counts[base + pos] + 1;
                counts[base + pos] = c;
                const float dl = delta[row0 + i];
                const bool finite = (dl == dl) && fabsf(dl) != INFINITY;
                // a non-finite delta_i (NaN or infinite latent, or ||z|| = 0) never freezes a state; it is
                // also reported: n_active[2] counts as "seen", every writer stores the same value
                if (!finite) n_active[2] = 1;
                const bool conv = p.adaptive && finite && dl < p.eps;
                const bool cap = c * p.r_inner >= p.r_total;
                if (!(conv || cap)) atomicMin(&first_open, i);
            }
            __syncthreads();
            if (tid == 0) {
                const int k = min(first_open, rows);                     // longest freezable prefix
                q.last_rows = rows; q.last_pos0 = q.win_pos0; q.last_row0 = q.cur_row0;
                q.n_frozen += k; q.win_pos0 += k; q.win_n -= k;
                q.new_n = 0;
                if (q.n_frozen - q.prompt_len >= p.n_new) {
                    q.done = 1; q.win_n = 0;
                } else {
                    const int n_app = min(p.headway, p.w_max - q.win_n);
                    if (n_app > 0) {
                        const int start = q.win_n > 0 ? q.win_pos0 + q.win_n : q.n_frozen - 1;
                        if (q.win_n == 0) q.win_pos0 = start;
                        q.new_pos0 = start; q.new_n = n_app;
                        for (int a = 0; a < n_app; ++a) counts[base + start + a] = 0;
                        q.win_n += n_app;
                    }
                }
                cur = q;
                // the record goes to memory for the workgroup that builds the tile list
                const int32_t* src = reinterpret_cast<const int32_t*>(&q);
                int32_t* dst = reinterpret_cast<int32_t*>(&seqs[s]);
                for (int f = 0; f < NF; ++f) __hip_atomic_store(dst + f, src[f], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            }
            __syncthreads();
            q = cur;
            // InitState for the appended positions: a random draw, or ("continuous compute", App.,
            // additional hyperparameter sweeps) the latest state of the position one step to the
            // left, which is the last row of the window this step ran on
            // (the draws are the bulk of this kernel's time -- a counter-based generator and a Box-Muller
            // transform per four values -- which is why the workgroup has 1024 threads)
            const int nb = (h + 3) / 4;
            const size_t left = (base + q.new_pos0 - 1) * h;
            const int id = ident[s];
            for (int idx = tid; idx < q.new_n * nb; idx += blockDim.x) {
                const int a = idx / nb, blk = idx - a * nb, pos = q.new_pos0 + a;
                float g[4];
                if (p.init_mode == 1) {
                    for (int i = 0; i < 4 && blk * 4 + i < h; ++i) g[i] = z[left + blk * 4 + i];
                } else {
                    gauss4(blk, pos, id, p.seed_lo, p.seed_hi, p.alpha, g);
                }
                for (int i = 0; i < 4 && blk * 4 + i < h; ++i) {
                    const size_t o = (base + pos) * h + blk * 4 + i;
                    z[o] = g[i];
                    z_prev[o] = g[i];
                }
            }
        }
    }
    if (gridDim.x > 1) {
        if (draw_ticket(ticket_ctr, &ticket) != gridDim.x - 1) return;
    } else {
        __syncthreads();
    }
    // tile list of the next step: the records of up to 256 sequences at a time are fetched in
    // parallel, one thread lays the windows out in sequence order, all write the row descriptors
    __shared__ int32_t s_done[256], s_win_n[256], s_pos0[256];
    __shared__ int sh_counts[2];
    __shared__ TileDesc sh_segs[TILE_LDS_SEGS];
    TileLayout lay;
    lay.tiles = tiles; lay.n_tiles = n_tiles; lay.rows_pad = rows_pad; lay.pack = pack; lay.sh_segs = sh_segs;
    int active = 0;
    for (int s0 = 0; s0 < n_seqs; s0 += 256) {
        const int i = s0 + tid;
        if (tid < 256 && i < n_seqs) {
            s_done[tid] = __hip_atomic_load(&seqs[i].done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            s_win_n[tid] = __hip_atomic_load(&seqs[i].win_n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            s_pos0[tid] = __hip_atomic_load(&seqs[i].win_pos0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        __syncthreads();
        if (tid == 0) {
            for (int j = 0; j < min(256, n_seqs - s0); ++j) {
                const int sq = s0 + j;
                if (!s_done[j]) active++;
                const int rows = s_done[j] ? 0 : s_win_n[j];
                seqs[sq].cur_rows = rows;
                seqs[sq].cur_row0 = lay.add(sq, ident[sq], s_pos0[j], rows, (long long)sq * max_positions);
            }
        }
        __syncthreads();
    }
    if (tid == 0) {
        // n_active[1] remembers the step at which the last sequence finished (0 = still running)
        if (active == 0 && n_active[0] != 0) n_active[1] = step;
        n_active[0] = active;
        lay.counts(sh_counts);
    }
    __syncthreads();
    lay.rows(sh_counts, sh_segs);
    if (tid == 0 && gridDim.x > 1) __hip_atomic_store(ticket_ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// Continuous batching: a sequence (tokens set, first L-1 positions prefilled) enters a running
// sampler with one fresh state at position L-1 and counts its steps from `step`; a retired slot
// contributes no rows.
__global__ void seq_join_k(SeqState* seqs, int32_t* seq_step0, int seq, int prompt_len, int step) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    SeqState q;
    q.prompt_len = prompt_len; q.n_frozen = prompt_len; q.win_pos0 = prompt_len - 1; q.win_n = 1; q.done = 0;
    q.last_rows = 0; q.last_pos0 = 0; q.new_pos0 = 0; q.new_n = 0; q.last_row0 = 0; q.cur_rows = 0; q.cur_row0 = 0;
    seqs[seq] = q;
    seq_step0[seq] = step;
}
__global__ void seq_retire_k(SeqState* seqs, int seq, int prompt_len) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    SeqState& q = seqs[seq];
    q.done = 1; q.win_n = 0; q.cur_rows = 0; q.last_rows = 0;
    if (prompt_len >= 0) { q.prompt_len = prompt_len; q.n_frozen = prompt_len; }   // < 0: the text stays readable
}

__global__ void fill_i32_k(int32_t* p, int32_t v, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

template <int DT>
__global__ void read_kv_k(const void* kc, const void* vc, KvPages kv, int seq, int H, int d, int pos0, int n, float* k_out,
                          float* v_out) {
    int i = blockIdx.x, pos = pos0 + i, h = H * d;
    const size_t base = kv_block_base(kv, seq, pos >> 5, (size_t)32 * h);
    for (int c = threadIdx.x; c < h; c += blockDim.x) {
        if (DT == 0) {
            k_out[(size_t)i * h + c] = reinterpret_cast<const float*>(kc)[base + (size_t)(pos & 31) * h + c];
            v_out[(size_t)i * h + c] = reinterpret_cast<const float*>(vc)[base + (size_t)(pos & 31) * h + c];
        } else {
            int hd = c / d, dd = c - hd * d;
            k_out[(size_t)i * h + c] =
                bf16_to_f32(reinterpret_cast<const uint16_t*>(kc)[base + k_cache_off(pos & 31, hd, dd, H, d)]);
            v_out[(size_t)i * h + c] = bf16_to_f32(reinterpret_cast<const uint16_t*>(vc)[
                base + ((size_t)hd * d + dd) * 32 + vt_slot(pos & 31)]);
        }
    }
}

__global__ void table_set_k(int32_t* table, BlockIds ids) {
    if ((int)threadIdx.x < ids.n) table[ids.first + threadIdx.x] = ids.id[threadIdx.x];
}

// ---------------------------------------------------------------------------------------------
// launchers

void launch_build_tiles_api(const SeqWindows& w, const int32_t* ident, TileDesc* tiles, int32_t* n_tiles, int rows_pad,
                            bool pack, hipStream_t st) {
    hipLaunchKernelGGL(build_tiles_api_k, dim3(1), dim3(256), 0, st, w, ident, 0, 0, tiles, n_tiles, rows_pad, pack ? 1 : 0);
}
void launch_build_tiles_store(const SeqWindows& w, const int32_t* ident, int max_positions, TileDesc* tiles,
                              int32_t* n_tiles, int rows_pad, bool pack, hipStream_t st) {
    hipLaunchKernelGGL(build_tiles_api_k, dim3(1), dim3(256), 0, st, w, ident, 1, max_positions, tiles, n_tiles, rows_pad,
                       pack ? 1 : 0);
}
void launch_build_tiles_sampler(const SeqState* seqs, const int32_t* ident, int n_seqs, int max_positions, TileDesc* tiles,
                                int32_t* n_tiles, int rows_pad, bool pack, hipStream_t st) {
    hipLaunchKernelGGL(build_tiles_sampler_k, dim3(1), dim3(256), 0, st, const_cast<SeqState*>(seqs), ident, n_seqs,
                       max_positions, tiles, n_tiles, rows_pad, pack ? 1 : 0);
}
void launch_table_set(int32_t* table, BlockIds ids, hipStream_t st) {
    if (ids.n <= 0) return;
    hipLaunchKernelGGL(table_set_k, dim3(1), dim3(64), 0, st, table, ids);
}
void launch_embed(const void* emb, int dtype, const int32_t* tokens, float scale, float* x, int h, int V,
                  float* rope_table, const float* theta, int half, const float* gain, void* xg, float* ssq,
                  size_t ssq_stride, const TileDesc* tiles, const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    const int chunks = xg ? fold_chunks(h) : (h >= 2048 ? 8 : 1);
    dim3 grid(chunks, max_tiles * 32);
    float2* tab = reinterpret_cast<float2*>(rope_table);
    if (dtype == 0)
        hipLaunchKernelGGL(embed_k<float>, grid, dim3(256), 0, st, (const float*)emb, tokens, scale, x, h, V, chunks,
                           tab, theta, half, gain, xg, ssq, ssq_stride, tiles, n_tiles);
    else
        hipLaunchKernelGGL(embed_k<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)emb, tokens, scale, x, h, V,
                           chunks, tab, theta, half, gain, xg, ssq, ssq_stride, tiles, n_tiles);
}
void launch_copy_rows_in(const float* src, float* x, int h, int which, const TileDesc* tiles,
                         const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    hipLaunchKernelGGL(copy_rows_in_k, dim3(max_tiles * 32), dim3(256), 0, st, src, x, h, which, tiles, n_tiles);
}
void launch_copy_rows_out(const float* x, float* dst, int width, int which, const TileDesc* tiles,
                          const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    hipLaunchKernelGGL(copy_rows_out_k, dim3(max_tiles * 32), dim3(256), 0, st, x, dst, width, which, tiles, n_tiles);
}
void launch_copy_i32_out(const int32_t* src, int32_t* dst, const TileDesc* tiles, const int32_t* n_tiles,
                         int max_tiles, hipStream_t st) {
    hipLaunchKernelGGL(copy_i32_out_k, dim3((max_tiles * 32 + 255) / 256), dim3(256), 0, st, src, dst, tiles, n_tiles);
}
void launch_concat(const float* e, const float* z, void* cat, int fmt, int h, const TileDesc* tiles,
                   const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    if (fmt == ACT_F32)
        hipLaunchKernelGGL(concat_k<ACT_F32>, dim3(max_tiles * 32), dim3(256), 0, st, e, z, cat, h, tiles, n_tiles);
    else
        hipLaunchKernelGGL(concat_k<ACT_BF16P>, dim3(max_tiles * 32), dim3(256), 0, st, e, z, cat, h, tiles, n_tiles);
}
void launch_addnorm(const float* xin, float* xout, const float* part, int S, size_t part_stride,
                    const float* gain, void* xn, int fmt, int h, float eps, const int32_t* n_tiles,
                    int max_tiles, hipStream_t st) {
    if (fmt == ACT_F32)
        hipLaunchKernelGGL(addnorm_k<ACT_F32>, dim3(max_tiles * 32), dim3(256), 0, st, xin, xout, part, S,
                           part_stride, gain, xn, h, eps, n_tiles);
    else
        hipLaunchKernelGGL(addnorm_k<ACT_BF16P>, dim3(max_tiles * 32), dim3(256), 0, st, xin, xout, part, S,
                           part_stride, gain, xn, h, eps, n_tiles);
}
int fold_chunks(int h) {
    for (int c : {8, 4, 2})
        if (h % (4 * c) == 0 && h / c <= 1024 * 1 && h / c >= 64) return c;
    for (int c : {8, 4, 2})
        if (h % (4 * c) == 0 && h / c <= 1024) return c;
    return h <= 1024 ? 1 : 0;
}
void launch_fold(const float* xin, float* xout, const float* part, int S, size_t part_stride, const float* gain,
                 void* xg, float* ssq, size_t ssq_stride, int h, const int32_t* n_tiles, int max_tiles,
                 hipStream_t st) {
    const int c = fold_chunks(h);
    hipLaunchKernelGGL(fold_k, dim3(c, max_tiles * 32), dim3(256), 0, st, xin, xout, part, S, part_stride, gain, xg,
                       ssq, ssq_stride, h, c, n_tiles);
}
void launch_prelude_end(const float* xin, const float* part, int S, size_t part_stride, float* e_out, const float* z,
                        void* cat, void* cat_e, int h, const TileDesc* tiles, const int32_t* n_tiles, int max_tiles,
                        hipStream_t st) {
    const int c = fold_chunks(h);
    hipLaunchKernelGGL(prelude_end_k, dim3(c, max_tiles * 32), dim3(256), 0, st, xin, part, S, part_stride, e_out, z,
                       cat, cat_e, h, c, tiles, n_tiles);
}
void launch_final_norm(const float* xin, const float* part, int S, size_t part_stride, const float* gain,
                       int h, float eps, float* z, float* z_prev, int update_prev, float* delta, float* xcopy,
                       const float* gain2, void* xg, float* ssq_tot, const TileDesc* tiles, const int32_t* n_tiles,
                       int max_tiles, hipStream_t st) {
    if (h > 2048)     // long rows: more loads in flight per row
        hipLaunchKernelGGL(final_norm_k<1024>, dim3(max_tiles * 32), dim3(1024), 0, st, xin, part, S, part_stride,
                           gain, h, eps, z, z_prev, update_prev, delta, xcopy, gain2, xg, ssq_tot, tiles, n_tiles);
    else
        hipLaunchKernelGGL(final_norm_k<256>, dim3(max_tiles * 32), dim3(256), 0, st, xin, part, S, part_stride, gain,
                           h, eps, z, z_prev, update_prev, delta, xcopy, gain2, xg, ssq_tot, tiles, n_tiles);
}
void launch_rope_table(float* table, const float* theta, int half, const TileDesc* tiles, const int32_t* n_tiles,
                       int max_tiles, hipStream_t st) {
    hipLaunchKernelGGL(rope_table_k, dim3(max_tiles * 32), dim3(64), 0, st, reinterpret_cast<float2*>(table), theta,
                       half, tiles, n_tiles);
}
void launch_rope_kv(const float* qkv, int S, size_t part_stride, void* q, void* kc, void* vc, int dtype,
                    int H, int d, const float* table, KvPages kv, const TileDesc* tiles,
                    const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    const size_t lds = (size_t)32 * (d + 1) * sizeof(float);
    const float2* tb = reinterpret_cast<const float2*>(table);
    if (dtype == 0)
        hipLaunchKernelGGL(rope_kv_k<0>, dim3(H, max_tiles), dim3(256), lds, st, qkv, S, part_stride, q, kc, vc, H, d,
                           tb, kv, tiles, n_tiles);
    else
        hipLaunchKernelGGL(rope_kv_k<1>, dim3(H, max_tiles), dim3(256), lds, st, qkv, S, part_stride, q, kc, vc, H, d,
                           tb, kv, tiles, n_tiles);
}
void launch_swiglu(const float* gu, int S, size_t part_stride, void* act, int fmt, int F,
                   const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    dim3 grid((F / 4 + 255) / 256, max_tiles * 32);
    if (fmt == ACT_F32)
        hipLaunchKernelGGL(swiglu_k<ACT_F32>, grid, dim3(256), 0, st, gu, S, part_stride, act, F, n_tiles);
    else
        hipLaunchKernelGGL(swiglu_k<ACT_BF16P>, grid, dim3(256), 0, st, gu, S, part_stride, act, F, n_tiles);
}
void launch_init_state_rows(float* z, float* z_prev, int h, int seq, int pos0, int n, size_t zrow0,
                            float alpha, uint32_t k0, uint32_t k1, hipStream_t st) {
    if (n <= 0) return;
    int nb = (h + 3) / 4;
    hipLaunchKernelGGL(init_state_rows_k, dim3((nb + 255) / 256, n), dim3(256), 0, st, z, z_prev, h, seq, pos0, n,
                       zrow0, alpha, k0, k1);
}
void launch_momentum(float* e, float* e_store, const int32_t* counts, float eta, int h, const TileDesc* tiles,
                     const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    hipLaunchKernelGGL(momentum_k, dim3(max_tiles * 32), dim3(256), 0, st, e, e_store, counts, eta, h, tiles, n_tiles);
}
void launch_noise_mix(float* z, const int32_t* counts, float beta, int n_steps, float alpha, uint32_t k0,
                      uint32_t k1, int step, const int32_t* seq_step0, int h, const TileDesc* tiles,
                      const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    hipLaunchKernelGGL(noise_mix_k, dim3(max_tiles * 32), dim3(256), 0, st, z, counts, beta, n_steps, alpha, k0, k1,
                       step, seq_step0, h, tiles, n_tiles);
}
void launch_sample(const float* logits, int V, float temperature, uint32_t k0, uint32_t k1, int step,
                   const int32_t* seq_step0, int32_t* tok_out, const TileDesc* tiles, const int32_t* n_tiles,
                   int max_tiles, hipStream_t st) {
    hipLaunchKernelGGL(sample_k, dim3(max_tiles * 32), dim3(256), 0, st, logits, V, temperature, k0, k1, step,
                       seq_step0, tok_out, tiles, n_tiles);
}
void launch_sample_top_p(const float* logits, int V, float temperature, float top_p, uint32_t k0, uint32_t k1,
                         int step, const int32_t* seq_step0, int32_t* tok_out, const TileDesc* tiles,
                         const int32_t* n_tiles, int max_tiles, hipStream_t st) {
    hipLaunchKernelGGL(sample_top_p_k, dim3(max_tiles * 32), dim3(TOPP_THREADS), 0, st, logits, V, temperature, top_p,
                       k0, k1, step, seq_step0, tok_out, tiles, n_tiles);
}
void launch_step_end(SeqState* seqs, const int32_t* ident, int n_seqs, SamplerParams p, int32_t* y, int32_t* counts,
                     int max_positions, const int32_t* drafts, const float* delta, float* z, float* z_prev, int h,
                     TileDesc* tiles, int32_t* n_tiles, int32_t* n_active, int step, uint32_t* ticket, int rows_pad,
                     bool pack, hipStream_t st) {
    hipLaunchKernelGGL(step_end_k, dim3(n_seqs), dim3(1024), 0, st, seqs, ident, n_seqs, p, y, counts, max_positions, drafts,
                       delta, z, z_prev, h, tiles, n_tiles, n_active, step, ticket, rows_pad, pack ? 1 : 0);
}
void launch_seq_join(SeqState* seqs, int32_t* seq_step0, int seq, int prompt_len, int step, hipStream_t st) {
    hipLaunchKernelGGL(seq_join_k, dim3(1), dim3(64), 0, st, seqs, seq_step0, seq, prompt_len, step);
}
void launch_seq_retire(SeqState* seqs, int seq, int prompt_len, hipStream_t st) {
    hipLaunchKernelGGL(seq_retire_k, dim3(1), dim3(64), 0, st, seqs, seq, prompt_len);
}
void launch_fill_i32(int32_t* p, int32_t v, size_t n, hipStream_t st) {
    if (!n) return;
    hipLaunchKernelGGL(fill_i32_k, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, v, n);
}
void launch_read_kv(const void* kc, const void* vc, KvPages kv, int seq, int dtype, int H, int d, int pos0, int n,
                    float* k_out, float* v_out, hipStream_t st) {
    if (n <= 0) return;
    if (dtype == 0)
        hipLaunchKernelGGL(read_kv_k<0>, dim3(n), dim3(256), 0, st, kc, vc, kv, seq, H, d, pos0, n, k_out, v_out);
    else
        hipLaunchKernelGGL(read_kv_k<1>, dim3(n), dim3(256), 0, st, kc, vc, kv, seq, H, d, pos0, n, k_out, v_out);
}

}  // namespace rdlm
