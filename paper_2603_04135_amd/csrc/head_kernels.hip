// HBM-bound kernels around the vocabulary GEMMs of the LM-head path: row gather and
// transposes, target logits, combination of per-tile softmax partials, the per-token
// surrogate + KL terms of Eq. 1 and their derivative, the row scales that turn a chunk of stored
// exponentials into softmax gradients (bf16 path) or the softmax-gradient pass over a stored logits
// chunk (float32 path), and the segmented (per packed sequence) loss reduction.
// All global accesses are coalesced 16-byte (or full-wave contiguous) transactions; the
// transposes go through padded LDS tiles.
#include "dppo_internal.h"

namespace dppo {
namespace {

typedef float f32x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float bf16_to_f32(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }
__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(uint16_t x) { return bf16_to_f32(x); }

// ------------------------------------------------------------------------------------
__global__ void fill_zero_kernel(uint4* p, size_t n16, unsigned char* tail, size_t ntail) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
    if (blockIdx.x == 0 && threadIdx.x < ntail) tail[threadIdx.x] = 0;
}

// ------------------------------------------------------------------------------------
// Tiled gather + transpose. Source rows come from `src` (row stride ld_src) through an
// optional row index; rows >= n_valid read as zero. Writes dst[r, c] (optional) and
// dstT[c, r] (optional) for r < n_rows_out, c < n_cols_out where columns >= n_cols read as 0.
template <typename E>
__global__ __launch_bounds__(256) void gather_transpose_kernel(
    const E* __restrict__ src, int64_t ld_src, const int32_t* __restrict__ row_index, int64_t row_index_base,
    int64_t src_row0, int64_t src_rows_total, int32_t n_valid, int32_t n_cols, int32_t n_rows_out,
    int32_t n_cols_out, E* __restrict__ dst, int64_t ld_dst, E* __restrict__ dstT, int64_t ld_dstT) {
    __shared__ E tile[64][65];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int rr = ty; rr < 64; rr += 4) {
        const int r = r0 + rr, c = c0 + tx;
        E v = (E)0;
        if (r < n_valid && c < n_cols) {
            int64_t sr = row_index ? (int64_t)row_index[row_index_base + r] : src_row0 + r;
            sr = sr < 0 ? 0 : (sr >= src_rows_total ? src_rows_total - 1 : sr);
            v = src[sr * ld_src + c];
        }
        tile[rr][tx] = v;
        if (dst && r < n_rows_out && c < n_cols_out) dst[(int64_t)r * ld_dst + c] = v;
    }
    __syncthreads();
    if (dstT) {
        for (int cc = ty; cc < 64; cc += 4) {
            const int c = c0 + cc, r = r0 + tx;
            if (c < n_cols_out && r < n_rows_out) dstT[(int64_t)c * ld_dstT + r] = tile[tx][cc];
        }
    }
}

// Target id and (clamped) row of H of every loss token of the chunk. An id outside [0, V) or a
// position outside [0, T) is clamped into the range and reported in *status, so that every later
// gather and scatter of the call stays in bounds.
__global__ void targets_kernel(const int32_t* __restrict__ ids, const int32_t* __restrict__ loss_pos, int64_t T,
                               int32_t V, int64_t n0, int32_t n_c, int32_t n_cp, int32_t* __restrict__ y,
                               int32_t* __restrict__ rowc, int32_t* status) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= n_cp) return;
    int32_t t = 0, row = 0;
    int flags = 0;
    if (n < n_c) {
        int64_t r = loss_pos ? (int64_t)loss_pos[n0 + n] : n0 + n;
        int64_t pos = loss_pos ? r + 1 : r;
        if (r < 0 || pos >= T) flags |= DPPO_HEAD_BAD_POSITION;
        r = r < 0 ? 0 : (r >= T ? T - 1 : r);
        pos = pos < 0 ? 0 : (pos >= T ? T - 1 : pos);
        t = ids[pos];
        if (t < 0 || t >= V) flags |= DPPO_HEAD_BAD_TARGET;
        t = t < 0 ? 0 : (t >= V ? V - 1 : t);
        row = (int32_t)r;
    }
    y[n] = t;
    rowc[n] = row;
    if (flags != 0 && status != nullptr) atomicOr(status, flags);
}

// ------------------------------------------------------------------------------------
// One wavefront per token: zy[n] = Hc[n] . W[y[n]], copied to bref[n] if bref is not NULL;
// clears *flag if flag is not NULL.
template <typename E>
__global__ __launch_bounds__(256) void target_logit_kernel(const E* __restrict__ Hc, const E* __restrict__ W,
                                                           const int32_t* __restrict__ y, int32_t n_cp, int32_t D,
                                                           float* __restrict__ zy, float* __restrict__ bref,
                                                           int32_t* __restrict__ flag) {
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (flag && blockIdx.x == 0 && threadIdx.x == 0) *flag = 0;
    if (n >= n_cp) return;
    const E* h = Hc + (size_t)n * D;
    const E* w = W + (size_t)y[n] * D;
    float s = 0.0f;
    if (sizeof(E) == 2 && D % 8 == 0) {          // bf16 rows (16-byte aligned): 8 elements per lane and step
        const uint4* h8 = reinterpret_cast<const uint4*>(h);
        const uint4* w8 = reinterpret_cast<const uint4*>(w);
        for (int c = lane; c < D / 8; c += 64) {
            const uint4 a = h8[c], b = w8[c];
            const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                s = fmaf(__uint_as_float(aw[k] << 16), __uint_as_float(bw[k] << 16), s);
                s = fmaf(__uint_as_float(aw[k] & 0xffff0000u), __uint_as_float(bw[k] & 0xffff0000u), s);
            }
        }
    } else {
        for (int d = lane; d < D; d += 64) s = fmaf(to_f32(h[d]), to_f32(w[d]), s);
    }
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0) {
        zy[n] = s;
        if (bref) bref[n] = s;
    }
}

// ------------------------------------------------------------------------------------
// 64 tokens per workgroup, the vocabulary tiles split over 4 wavefronts; each thread folds its
// tiles into a running (max, sum) pair in one pass, the four pairs of a token meet in LDS.
__global__ __launch_bounds__(256) void combine_logprob_kernel(const float2* __restrict__ part, int32_t n_tiles,
                                                              const float* __restrict__ zy, int64_t n0, int32_t n_c,
                                                              int32_t n_cp, float* __restrict__ lse_chunk,
                                                              float* __restrict__ logp_out,
                                                              float* __restrict__ lse_out) {
    __shared__ float2 red[4][64];
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int n = blockIdx.x * 64 + lane;
    const float NEG_INF = -__builtin_inff();
    float m = NEG_INF, s = 0.0f;
    if (n < n_c) {
        for (int t = q; t < n_tiles; t += 4) {
            const float2 p = part[(size_t)t * n_cp + n];
            if (p.x > m) { s = s * expf(m - p.x) + p.y; m = p.x; }      // exp(-inf) = 0 on the first tile
            else if (p.x > NEG_INF) s += p.y * expf(p.x - m);
        }
    }
    red[q][lane] = make_float2(m, s);
    __syncthreads();
    if (q != 0 || n >= n_cp) return;
    if (n >= n_c) { lse_chunk[n] = 0.0f; return; }
    float mm = NEG_INF;
#pragma unroll
    for (int i = 0; i < 4; ++i) mm = fmaxf(mm, red[i][lane].x);
    float ss = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float2 r = red[i][lane];
        ss += (r.x == NEG_INF) ? 0.0f : r.y * expf(r.x - mm);
    }
    const float lse = mm + logf(ss);
    lse_chunk[n] = lse;
    logp_out[n0 + n] = zy[n] - lse;
    if (lse_out) lse_out[n0 + n] = lse;
}

// Same split of the work for the GEMM that stores exponentials: part[tile][n] = (max z, sum of
// exp(z - bref[n])) with one reference per token, so the sums of the tiles add up and
// lse = bref + log(sum). With the target logit as reference the sum is 1 / p(target), the stored
// exponentials reach that size and the row scale c p(target) shrinks by it; beyond 1e15 (a target
// token with log-prob below about -34.5) the scaled hidden-state rows of the dW operand would
// approach the bottom of the bf16 range for small loss weights, so the token goes on the redo
// list instead and is redone against its row maximum.
constexpr float EXP_SUM_LIMIT = 1e15f;
__global__ __launch_bounds__(256) void combine_exp_kernel(const float2* __restrict__ part, int32_t n_tiles,
                                                          const float* __restrict__ zy,
                                                          const float* __restrict__ bref, int64_t n0, int32_t n_c,
                                                          int32_t n_cp, float* __restrict__ lse_chunk,
                                                          float* __restrict__ logp_out, float* __restrict__ mx,
                                                          int32_t* redo_count, int32_t* __restrict__ redo_list,
                                                          float* __restrict__ redo_sum) {
    __shared__ float2 red[4][64];
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int n = blockIdx.x * 64 + lane;
    float m = -__builtin_inff(), s = 0.0f;
    if (n < n_cp) {
#pragma unroll 8
        for (int t = q; t < n_tiles; t += 4) {
            const float2 p = part[(size_t)t * n_cp + n];
            m = fmaxf(m, p.x);
            s += p.y;
        }
    }
    red[q][lane] = make_float2(m, s);
    __syncthreads();
    if (q != 0 || n >= n_cp) return;
#pragma unroll
    for (int i = 1; i < 4; ++i) {
        m = fmaxf(m, red[i][lane].x);
        s += red[i][lane].y;
    }
    mx[n] = m;
    if (n >= n_c) { lse_chunk[n] = 0.0f; return; }
    if (!(s < EXP_SUM_LIMIT)) {
        redo_list[atomicAdd(redo_count, 1)] = n;
        redo_sum[n] = 0.0f;
        return;
    }
    const float lse = bref[n] + logf(s);
    lse_chunk[n] = lse;
    logp_out[n0 + n] = zy[n] - lse;
}

// Slow exact path for the tokens on the redo list: E[n, v] = exp(Hc[n] . W[v] - mx[n]) with fp32
// dot products, 8 listed tokens x 256 vocabulary entries per workgroup pass (one thread per
// vocabulary entry, the token rows in LDS in slabs of REDO_SLAB columns), row sums by atomic adds.
constexpr int REDO_TOK = 8, REDO_SLAB = 2048;
__global__ __launch_bounds__(256) void exp_redo_rows_kernel(const int32_t* redo_count,
                                                            const int32_t* __restrict__ redo_list,
                                                            const uint16_t* __restrict__ Hc,
                                                            const uint16_t* __restrict__ W, int32_t V, int32_t D,
                                                            const float* __restrict__ mx, uint16_t* __restrict__ E,
                                                            int64_t lde, float* redo_sum) {
    __shared__ uint4 hs[REDO_TOK][REDO_SLAB / 8];
    const int cnt = *reinterpret_cast<const volatile int32_t*>(redo_count);
    const int v = blockIdx.x * 256 + threadIdx.x;
    const int lane = threadIdx.x & 63;
    const int vr = v < V ? v : V - 1;
    for (int g = blockIdx.y; g * REDO_TOK < cnt; g += gridDim.y) {
        const int nt = (cnt - g * REDO_TOK) < REDO_TOK ? (cnt - g * REDO_TOK) : REDO_TOK;
        float acc[REDO_TOK];
#pragma unroll
        for (int t = 0; t < REDO_TOK; ++t) acc[t] = 0.0f;
        for (int d0 = 0; d0 < D; d0 += REDO_SLAB) {
            const int dw = ((D - d0) < REDO_SLAB ? (D - d0) : REDO_SLAB) / 8;   // 16-byte pieces of the slab
            __syncthreads();
            for (int i = threadIdx.x; i < REDO_TOK * dw; i += 256) {
                const int t = i / dw, c = i % dw;
                uint4 x = make_uint4(0, 0, 0, 0);
                if (t < nt) x = *reinterpret_cast<const uint4*>(Hc + (size_t)redo_list[g * REDO_TOK + t] * D + d0 + c * 8);
                hs[t][c] = x;
            }
            __syncthreads();
            const uint4* wr = reinterpret_cast<const uint4*>(W + (size_t)vr * D + d0);
            for (int c = 0; c < dw; ++c) {
                const uint4 w8 = wr[c];
                const uint32_t ww[4] = {w8.x, w8.y, w8.z, w8.w};
#pragma unroll
                for (int t = 0; t < REDO_TOK; ++t) {
                    const uint4 h8 = hs[t][c];
                    const uint32_t hh[4] = {h8.x, h8.y, h8.z, h8.w};
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        acc[t] = fmaf(__uint_as_float(ww[k] << 16), __uint_as_float(hh[k] << 16), acc[t]);
                        acc[t] = fmaf(__uint_as_float(ww[k] & 0xffff0000u), __uint_as_float(hh[k] & 0xffff0000u), acc[t]);
                    }
                }
            }
        }
#pragma unroll
        for (int t = 0; t < REDO_TOK; ++t) {
            if (t >= nt) break;                                  // uniform over the workgroup
            const int64_t n = redo_list[g * REDO_TOK + t];
            float e = v < V ? expf(acc[t] - mx[n]) : 0.0f;
            const __bf16 eb = (__bf16)e;
            constexpr int64_t BR = 64, BC = 256;                 // blocked chunk layout; v < lde by the grid
            E[(size_t)(n / BR) * BR * lde + (size_t)(v / BC) * (BR * BC) + (n % BR) * BC + v % BC] =
                __builtin_bit_cast(uint16_t, eb);
            for (int off = 32; off > 0; off >>= 1) e += __shfl_xor(e, off, 64);
            if (lane == 0) atomicAdd(redo_sum + n, e);
        }
    }
}

__global__ void exp_redo_finish_kernel(const int32_t* redo_count, const int32_t* __restrict__ redo_list,
                                       const float* __restrict__ redo_sum, const float* __restrict__ zy,
                                       const float* __restrict__ mx, int64_t n0, float* __restrict__ bref,
                                       float* __restrict__ lse_chunk, float* __restrict__ logp_out) {
    const int cnt = *reinterpret_cast<const volatile int32_t*>(redo_count);
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < cnt; i += gridDim.x * blockDim.x) {
        const int n = redo_list[i];
        const float lse = mx[n] + logf(redo_sum[n]);
        bref[n] = mx[n];
        lse_chunk[n] = lse;
        logp_out[n0 + n] = zy[n] - lse;
    }
}

// Row scale of the stored exponentials and their entry at the target: with E[n, v] = exp(z - b[n]),
// c[n] (1[v = y] - p[n, v]) = s[n] E'[n, v] for s[n] = -c[n] exp(b[n] - lse[n]) and E' = E except
// E'[n, y[n]] = exp(zy[n] - b[n]) - exp(lse[n] - b[n]). Rows beyond n_c get s = 0.
__global__ void softmax_scale_kernel(const int32_t* __restrict__ y, const float* __restrict__ zy,
                                     const float* __restrict__ bref, const float* __restrict__ lse,
                                     const float* __restrict__ cvec, int32_t n_c, int32_t n_cp,
                                     uint16_t* __restrict__ E, int64_t lde, float* __restrict__ scale) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= n_cp) return;
    if (n >= n_c) { scale[n] = 0.0f; return; }
    const float b = bref[n], l = lse[n];
    scale[n] = -cvec[n] * expf(b - l);
    const __bf16 e = (__bf16)(expf(zy[n] - b) - expf(l - b));
    const int64_t v = y[n];
    constexpr int64_t BR = 64, BC = 256;   // blocked chunk layout
    E[(size_t)(n / BR) * BR * lde + (size_t)(v / BC) * (BR * BC) + (n % BR) * BC + v % BC] =
        __builtin_bit_cast(uint16_t, e);
}

// bf16 transpose by 16-byte accesses: dstT[c, r] = scale[r] * src[r, c] (scale NULL = 1) for
// r < rows_out, c < cols; source rows >= rows_valid read as zero. cols and rows_out are
// multiples of 64, all pointers and pitches multiples of 8 elements. A 64 x 64 tile goes through
// LDS; every thread loads and stores whole 8-element vectors. dstT is row-major with pitch
// ld_dstT, or (blocked != 0) the blocked B-operand layout of the MFMA GEMMs with ld_dstT = rows_out
// columns in all: blocks of GEMM_B_BLOCK_ROWS rows x GEMM_B_BLOCK_K columns, block (i, j) at
// (i * ld_dstT / GEMM_B_BLOCK_K + j) blocks from the start (a 64 x 64 tile is then one contiguous 8 KB run).
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const uint16_t* __restrict__ src, int64_t ld_src,
                                                             int32_t rows_valid, const float* __restrict__ scale,
                                                             uint16_t* __restrict__ dstT, int64_t ld_dstT, int blocked) {
    __shared__ uint16_t tile[64][64 + 2];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    const int vec = threadIdx.x & 7, line = threadIdx.x >> 3;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int rr = line + pass * 32, r = r0 + rr;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (r < rows_valid) v = *reinterpret_cast<const uint4*>(src + (int64_t)r * ld_src + c0 + vec * 8);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        if (scale && r < rows_valid) {
            const float sc = scale[r];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const __bf16 lo = (__bf16)(sc * __uint_as_float(w[k] << 16));
                const __bf16 hi = (__bf16)(sc * __uint_as_float(w[k] & 0xffff0000u));
                tile[rr][vec * 8 + 2 * k] = __builtin_bit_cast(uint16_t, lo);
                tile[rr][vec * 8 + 2 * k + 1] = __builtin_bit_cast(uint16_t, hi);
            }
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                tile[rr][vec * 8 + 2 * k] = (uint16_t)(w[k] & 0xffffu);
                tile[rr][vec * 8 + 2 * k + 1] = (uint16_t)(w[k] >> 16);
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int cc = line + pass * 32;
        uint32_t w[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            w[k] = (uint32_t)tile[vec * 8 + 2 * k][cc] | ((uint32_t)tile[vec * 8 + 2 * k + 1][cc] << 16);
        static_assert(GEMM_B_BLOCK_K == 64, "a 64-column tile = one block column");
        const int64_t drow = c0 + cc;
        const int64_t off = blocked ? ((drow / GEMM_B_BLOCK_ROWS) * (ld_dstT / GEMM_B_BLOCK_K) + r0 / GEMM_B_BLOCK_K) *
                                              (int64_t)(GEMM_B_BLOCK_ROWS * GEMM_B_BLOCK_K) +
                                          (drow % GEMM_B_BLOCK_ROWS) * GEMM_B_BLOCK_K + vec * 8
                                    : drow * ld_dstT + r0 + vec * 8;
        *reinterpret_cast<uint4*>(dstT + off) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// bf16 row gather by 16-byte vectors: dst[r] = src[row(r)] for r < n_valid (row through the
// optional index, clamped), zero rows up to n_rows_out. vec_per_row = D / 8.
__global__ __launch_bounds__(256) void gather_rows_bf16_kernel(const uint4* __restrict__ src, int32_t vec_per_row,
                                                               const int32_t* __restrict__ row_index,
                                                               int64_t row_index_base, int64_t src_row0,
                                                               int64_t src_rows_total, int32_t n_valid,
                                                               int32_t n_rows_out, uint4* __restrict__ dst) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)n_rows_out * vec_per_row) return;
    const int32_t r = (int32_t)(i / vec_per_row), c = (int32_t)(i % vec_per_row);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r < n_valid) {
        int64_t sr = row_index ? (int64_t)row_index[row_index_base + r] : src_row0 + r;
        sr = sr < 0 ? 0 : (sr >= src_rows_total ? src_rows_total - 1 : sr);
        v = src[sr * vec_per_row + c];
    }
    dst[i] = v;
}

// fp32 path: one workgroup per token over the stored logits row.
__global__ __launch_bounds__(256) void row_stats_kernel(const float* __restrict__ Z, int64_t ldz, int32_t V,
                                                        const int32_t* __restrict__ y, int64_t n0, int32_t n_c,
                                                        float* __restrict__ lse_chunk, float* __restrict__ logp_out,
                                                        float* __restrict__ lse_out) {
    __shared__ float red[256];
    const int n = blockIdx.x;
    if (n >= n_c) { if (threadIdx.x == 0) lse_chunk[n] = 0.0f; return; }
    const float* z = Z + (size_t)n * ldz;
    float m = -__builtin_inff();
    for (int v = threadIdx.x; v < V; v += 256) m = fmaxf(m, z[v]);
    red[threadIdx.x] = m;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + s]);
        __syncthreads();
    }
    m = red[0];
    __syncthreads();
    float sum = 0.0f;
    for (int v = threadIdx.x; v < V; v += 256) sum += expf(z[v] - m);
    red[threadIdx.x] = sum;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const float lse = m + logf(red[0]);
        lse_chunk[n] = lse;
        logp_out[n0 + n] = z[y[n]] - lse;
        if (lse_out) lse_out[n0 + n] = lse;
    }
}

// ------------------------------------------------------------------------------------
// Per-token terms of Eq. 1 and d(loss)/d(logp), weighted by seq_coef / C_s (token-sum aggregation:
// by seq_coef). With a sequence-level ratio every token of a sequence uses the same rho.
__global__ void token_loss_kernel(TokenLossArgs a, int64_t n0, int32_t n_c, int32_t n_cp) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= n_cp) return;
    if (n >= n_c) { a.c_chunk[n] = 0.0f; return; }
    const int64_t gi = n0 + n;
    int lo = 0, hi = a.S;          // largest s with loss_cu[s] <= gi
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((int64_t)a.loss_cu[mid] <= gi) lo = mid; else hi = mid;
    }
    const int s = lo;
    const float A = a.seq_adv[s];
    const float w = a.aggregation == DPPO_AGG_TOKEN_SUM ? a.seq_coef[s]
                                                       : a.seq_coef[s] / (float)(a.loss_cu[s + 1] - a.loss_cu[s]);
    const float lp = a.logp[gi];
    const float d_old = lp - a.logp_old[gi];
    const float d_ref = a.logp_ref[gi] - lp;
    const float rho = a.ratio_level == DPPO_RATIO_SEQUENCE ? a.seq_ratio[s] : expf(d_old);
    const float unclipped = rho * A;
    const float clipped = fminf(fmaxf(rho, a.lo), a.hi) * A;
    const float sur = fminf(unclipped, clipped);
    const float em1 = expm1f(d_ref);             // rho_hat - 1
    const float kl = em1 - d_ref;                // rho_hat - log rho_hat - 1
    const bool away = (A > 0.0f && rho > a.hi) || (A < 0.0f && rho < a.lo);
    const float g = (away ? 0.0f : -A * rho) - a.beta * em1;
    a.ell[gi] = -sur + a.beta * kl;
    a.kl[gi] = kl;
    a.clipped[gi] = away ? 1.0f : 0.0f;
    a.c_chunk[n] = w * g;
}

// ------------------------------------------------------------------------------------
// Softmax-gradient pass over a stored logits chunk, 64 tokens x 64 vocabulary entries per
// workgroup: in place Z[n,v] -> G[n,v], and the transposed copy GT[v,n] through LDS.
template <typename ZT, typename GT_, typename ZV, typename GV>
__global__ __launch_bounds__(256) void grad_logits_kernel(void* ZG, GT_* __restrict__ GTp, int32_t V, int64_t ld,
                                                          const int32_t* __restrict__ y, const float* __restrict__ lse,
                                                          const float* __restrict__ cvec, int64_t n_cp) {
    __shared__ GT_ tile[64][64 + 8];   // [v][n]
    const int v0 = blockIdx.x * 64, nb = blockIdx.y * 64;
    const int t = threadIdx.x;
    const int kc = t & 7;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int r = (t >> 3) + pass * 32;
        const int64_t n = nb + r;
        const float l = lse[n], cn = cvec[n];
        const int yt = y[n];
        char* p = reinterpret_cast<char*>(ZG) + ((size_t)n * ld + v0 + kc * 8) * sizeof(ZT);
        const ZV z = *reinterpret_cast<const ZV*>(p);
        GV g;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int v = v0 + kc * 8 + q;
            const float pr = expf((float)z[q] - l);
            float gv = cn * ((v == yt ? 1.0f : 0.0f) - pr);
            gv = v < V ? gv : 0.0f;
            const GT_ b = (GT_)gv;   // keep the scalar: reading g[q] back right after writing it miscompiles
            g[q] = b;
            tile[kc * 8 + q][r] = b;
        }
        *reinterpret_cast<GV*>(p) = g;
    }
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int v = (t >> 3) + pass * 32;
        GV g;
#pragma unroll
        for (int q = 0; q < 8; ++q) g[q] = tile[v][kc * 8 + q];
        *reinterpret_cast<GV*>(GTp + (size_t)(v0 + v) * n_cp + nb + kc * 8) = g;
    }
}

// One workgroup per packed sequence: exp of the mean log-ratio over its tokens, for the sequences
// that end in the token range (n_lo, n_hi] (all their log-probs are known once the tokens below
// n_hi are). A sequence that starts below n_lo and ends beyond n_hi is longer than the caller
// promised: it is flagged in `status` (its ratio is not written by this launch).
__global__ __launch_bounds__(256) void seq_ratio_kernel(const int32_t* __restrict__ loss_cu, int32_t S,
                                                        const float* __restrict__ logp,
                                                        const float* __restrict__ logp_old,
                                                        float* __restrict__ seq_ratio, int64_t n_lo, int64_t n_hi,
                                                        int32_t* __restrict__ status) {
    __shared__ float r0[256];
    for (int s = blockIdx.x; s < S; s += gridDim.x) {
        const int b = loss_cu[s], e = loss_cu[s + 1];
        if (e > n_hi) {
            if (b < n_lo && status && threadIdx.x == 0) atomicOr(status, DPPO_HEAD_SEQ_TOO_LONG);
            continue;
        }
        if (e <= n_lo) continue;
        float x = 0.0f;
        for (int i = b + threadIdx.x; i < e; i += 256) x += logp[i] - logp_old[i];
        r0[threadIdx.x] = x;
        __syncthreads();
        for (int st = 128; st > 0; st >>= 1) {
            if (threadIdx.x < st) r0[threadIdx.x] += r0[threadIdx.x + st];
            __syncthreads();
        }
        if (threadIdx.x == 0) seq_ratio[s] = e > b ? expf(r0[0] / (float)(e - b)) : 1.0f;
        __syncthreads();
    }
}

// One thread per prompt group: coef * G / (completion tokens of the whole group).
__global__ void token_norm_coef_kernel(int32_t Q, int32_t G, const int32_t* __restrict__ comp_len,
                                       const float* coef, float* coef_out) {
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= Q) return;
    int64_t tot = 0;
    for (int i = 0; i < G; ++i) tot += comp_len[(size_t)q * G + i];
    const float f = tot > 0 ? (float)((double)G / (double)tot) : 0.0f;
    for (int i = 0; i < G; ++i) coef_out[(size_t)q * G + i] = coef[(size_t)q * G + i] * f;
}

// ------------------------------------------------------------------------------------
// One workgroup per packed sequence: token-mean (or token-sum) loss, KL sum, clipped count.
__global__ __launch_bounds__(256) void seq_reduce_kernel(SeqReduceArgs a) {
    __shared__ float r0[256], r1[256], r2[256];
    for (int s = blockIdx.x; s < a.S; s += gridDim.x) {
        const int b = a.loss_cu[s], e = a.loss_cu[s + 1];
        float x0 = 0.0f, x1 = 0.0f, x2 = 0.0f;
        for (int i = b + threadIdx.x; i < e; i += 256) { x0 += a.ell[i]; x1 += a.kl[i]; x2 += a.clipped[i]; }
        r0[threadIdx.x] = x0; r1[threadIdx.x] = x1; r2[threadIdx.x] = x2;
        __syncthreads();
        for (int st = 128; st > 0; st >>= 1) {
            if (threadIdx.x < st) {
                r0[threadIdx.x] += r0[threadIdx.x + st];
                r1[threadIdx.x] += r1[threadIdx.x + st];
                r2[threadIdx.x] += r2[threadIdx.x + st];
            }
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            // an empty segment contributes nothing (its sums are 0)
            const float mean = (a.aggregation == DPPO_AGG_TOKEN_SUM || e <= b) ? r0[0] : r0[0] / (float)(e - b);
            a.seq_mean[s] = mean;
            a.seq_kl[s] = r1[0];
            a.seq_clip[s] = r2[0];
            if (a.seq_loss_out) a.seq_loss_out[s] = mean;
        }
        __syncthreads();
    }
}

// One workgroup: weighted sum over sequences in fp64, fixed order.
__global__ __launch_bounds__(256) void final_reduce_kernel(SeqReduceArgs a) {
    __shared__ double r0[256], r1[256], r2[256];
    double x0 = 0.0, x1 = 0.0, x2 = 0.0;
    for (int s = threadIdx.x; s < a.S; s += 256) {
        x0 += (double)a.seq_coef[s] * (double)a.seq_mean[s];
        x1 += (double)a.seq_kl[s];
        x2 += (double)a.seq_clip[s];
    }
    r0[threadIdx.x] = x0; r1[threadIdx.x] = x1; r2[threadIdx.x] = x2;
    __syncthreads();
    for (int st = 128; st > 0; st >>= 1) {
        if (threadIdx.x < st) {
            r0[threadIdx.x] += r0[threadIdx.x + st];
            r1[threadIdx.x] += r1[threadIdx.x + st];
            r2[threadIdx.x] += r2[threadIdx.x + st];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        a.loss_out[0] = (float)r0[0];
        if (a.stats_out) {
            const double n = a.N > 0 ? (double)a.N : 1.0;
            a.stats_out[0] = (float)(r1[0] / n);
            a.stats_out[1] = (float)(r2[0] / n);
            a.stats_out[2] = (float)a.N;
            a.stats_out[3] = 0.0f;
        }
    }
}

}  // namespace

// ======================================================================================
void launch_fill_zero(void* p, size_t bytes, hipStream_t st) {
    if (bytes == 0) return;
    const size_t n16 = bytes / 16, ntail = bytes % 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    if (blocks == 0) blocks = 1;
    fill_zero_kernel<<<(unsigned)blocks, 256, 0, st>>>(reinterpret_cast<uint4*>(p), n16,
                                                       reinterpret_cast<unsigned char*>(p) + n16 * 16, ntail);
}

void launch_gather_rows(int dtype, const void* H, const int32_t* ids, const int32_t* loss_pos, int64_t T,
                        int32_t D, int32_t V, ChunkView cv, void* Hc, void* HcT, int32_t* y, int32_t* rowc,
                        int32_t* status, hipStream_t st) {
    targets_kernel<<<(unsigned)ceil_div(cv.n_cp, 256), 256, 0, st>>>(ids, loss_pos, T, V, cv.n0, cv.n_c, cv.n_cp, y,
                                                                     rowc, status);
    dim3 grid((unsigned)ceil_div(D, 64), (unsigned)(cv.n_cp / 64));
    if (dtype == 1 && HcT == nullptr && D % 8 == 0) {
        const int64_t n_vec = (int64_t)cv.n_cp * (D / 8);
        gather_rows_bf16_kernel<<<(unsigned)ceil_div(n_vec, 256), 256, 0, st>>>(
            reinterpret_cast<const uint4*>(H), D / 8, rowc, 0, 0, T, cv.n_c, cv.n_cp, reinterpret_cast<uint4*>(Hc));
    } else if (dtype == 1) {
        gather_transpose_kernel<uint16_t><<<grid, 256, 0, st>>>(
            reinterpret_cast<const uint16_t*>(H), D, rowc, 0, 0, T, cv.n_c, D, cv.n_cp, D,
            reinterpret_cast<uint16_t*>(Hc), D, reinterpret_cast<uint16_t*>(HcT), cv.n_cp);
    } else {
        gather_transpose_kernel<float><<<grid, 256, 0, st>>>(
            reinterpret_cast<const float*>(H), D, rowc, 0, 0, T, cv.n_c, D, cv.n_cp, D,
            reinterpret_cast<float*>(Hc), D, reinterpret_cast<float*>(HcT), cv.n_cp);
    }
}

void launch_transpose_w(int dtype, const void* W, int32_t V, int32_t D, int32_t Vp, void* WT, hipStream_t st) {
    dim3 grid((unsigned)ceil_div(D, 64), (unsigned)ceil_div(Vp, 64));
    if (dtype == 1) {      // D and Vp are multiples of 64 on the bf16 path
        transpose_bf16_kernel<<<grid, 256, 0, st>>>(reinterpret_cast<const uint16_t*>(W), D, V, nullptr,
                                                    reinterpret_cast<uint16_t*>(WT), Vp, 1);
    } else {
        gather_transpose_kernel<float><<<grid, 256, 0, st>>>(reinterpret_cast<const float*>(W), D, nullptr, 0, 0, V,
                                                             V, D, Vp, D, nullptr, 0, reinterpret_cast<float*>(WT),
                                                             Vp);
    }
}

void launch_target_logit(int dtype, const void* Hc, const void* W, const int32_t* y, int32_t n_cp, int32_t D,
                         float* zy, float* bref, int32_t* flag, hipStream_t st) {
    const unsigned blocks = (unsigned)ceil_div(n_cp, 4);
    if (dtype == 1)
        target_logit_kernel<uint16_t><<<blocks, 256, 0, st>>>(reinterpret_cast<const uint16_t*>(Hc),
                                                              reinterpret_cast<const uint16_t*>(W), y, n_cp, D, zy,
                                                              bref, flag);
    else
        target_logit_kernel<float><<<blocks, 256, 0, st>>>(reinterpret_cast<const float*>(Hc),
                                                           reinterpret_cast<const float*>(W), y, n_cp, D, zy, bref,
                                                           flag);
}

void launch_combine_exp(const float2* part, int32_t n_tiles, const float* zy, const float* bref, ChunkView cv,
                        float* lse_chunk, float* logp_out, float* mx, int32_t* redo_count, int32_t* redo_list,
                        float* redo_sum, hipStream_t st) {
    combine_exp_kernel<<<(unsigned)ceil_div(cv.n_cp, 64), 256, 0, st>>>(part, n_tiles, zy, bref, cv.n0, cv.n_c, cv.n_cp,
                                                                        lse_chunk, logp_out, mx, redo_count, redo_list,
                                                                        redo_sum);
}

void launch_exp_redo_rows(const int32_t* redo_count, const int32_t* redo_list, float* redo_sum, const void* Hc,
                          const void* W, int32_t V, int32_t Vp, int32_t D, const float* zy, const float* mx,
                          ChunkView cv, void* E, int64_t lde, float* bref, float* lse_chunk, float* logp_out,
                          hipStream_t st) {
    dim3 grid((unsigned)(Vp / 256), 4);
    exp_redo_rows_kernel<<<grid, 256, 0, st>>>(redo_count, redo_list, reinterpret_cast<const uint16_t*>(Hc),
                                               reinterpret_cast<const uint16_t*>(W), V, D, mx,
                                               reinterpret_cast<uint16_t*>(E), lde, redo_sum);
    exp_redo_finish_kernel<<<4, 256, 0, st>>>(redo_count, redo_list, redo_sum, zy, mx, cv.n0, bref, lse_chunk,
                                              logp_out);
}

void launch_softmax_scale(const int32_t* y, const float* zy, const float* bref, const float* lse, const float* c,
                          ChunkView cv, void* E, int64_t lde, float* scale, hipStream_t st) {
    softmax_scale_kernel<<<(unsigned)ceil_div(cv.n_cp, 256), 256, 0, st>>>(y, zy, bref, lse, c, cv.n_c, cv.n_cp,
                                                                           reinterpret_cast<uint16_t*>(E), lde, scale);
}

void launch_scale_transpose_bf16(const void* Hc, const float* scale, int32_t n_cp, int32_t D, void* HcT, hipStream_t st) {
    dim3 grid((unsigned)(D / 64), (unsigned)(n_cp / 64));
    transpose_bf16_kernel<<<grid, 256, 0, st>>>(reinterpret_cast<const uint16_t*>(Hc), D, n_cp, scale,
                                                reinterpret_cast<uint16_t*>(HcT), n_cp, 1);
}

void launch_combine_logprob(const float2* part, int32_t n_tiles, const float* zy, ChunkView cv, float* lse_chunk,
                            float* logp_out, float* lse_out, hipStream_t st) {
    combine_logprob_kernel<<<(unsigned)ceil_div(cv.n_cp, 64), 256, 0, st>>>(part, n_tiles, zy, cv.n0, cv.n_c, cv.n_cp,
                                                                            lse_chunk, logp_out, lse_out);
}

void launch_row_stats_f32(const float* Z, int64_t ldz, int32_t V, const int32_t* y, ChunkView cv, float* lse_chunk,
                          float* logp_out, float* lse_out, hipStream_t st) {
    row_stats_kernel<<<(unsigned)cv.n_cp, 256, 0, st>>>(Z, ldz, V, y, cv.n0, cv.n_c, lse_chunk, logp_out, lse_out);
}

void launch_token_loss(const TokenLossArgs& a, ChunkView cv, hipStream_t st) {
    token_loss_kernel<<<(unsigned)ceil_div(cv.n_cp, 256), 256, 0, st>>>(a, cv.n0, cv.n_c, cv.n_cp);
}

void launch_seq_ratio(const int32_t* loss_cu, int32_t S, const float* logp, const float* logp_old,
                      float* seq_ratio, int64_t n_lo, int64_t n_hi, int32_t* status, hipStream_t st) {
    if (S <= 0) return;
    const unsigned blocks = S < 4096 ? (unsigned)S : 4096u;
    seq_ratio_kernel<<<blocks, 256, 0, st>>>(loss_cu, S, logp, logp_old, seq_ratio, n_lo, n_hi, status);
}

void launch_token_norm_coef(int32_t Q, int32_t G, const int32_t* comp_len, const float* coef, float* coef_out,
                            hipStream_t st) {
    token_norm_coef_kernel<<<(unsigned)ceil_div(Q, 64), 64, 0, st>>>(Q, G, comp_len, coef, coef_out);
}

void launch_grad_logits_f32(float* ZG, float* GT, int32_t V, int32_t Vp, const int32_t* y, const float* lse,
                            const float* c, int32_t n_cp, hipStream_t st) {
    dim3 grid((unsigned)(Vp / 64), (unsigned)(n_cp / 64));
    grad_logits_kernel<float, float, f32x8, f32x8><<<grid, 256, 0, st>>>(ZG, GT, V, Vp, y, lse, c, n_cp);
}

void launch_seq_reduce(const SeqReduceArgs& a, hipStream_t st) {
    if (a.S > 0) {
        const unsigned blocks = a.S < 4096 ? (unsigned)a.S : 4096u;
        seq_reduce_kernel<<<blocks, 256, 0, st>>>(a);
    }
    final_reduce_kernel<<<1, 256, 0, st>>>(a);
}

}  // namespace dppo
