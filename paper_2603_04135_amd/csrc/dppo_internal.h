// Internal declarations shared by the translation units of the DPPO HIP library.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "dppo.h"

namespace dppo {

// Records a formatted message for dppo_last_error() and returns `code`.
int fail(int code, const char* fmt, ...);
// Turns the status of the last launch on this thread into a dppo status.
int check_launch(const char* what);

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- selection (select.hip) -------------------------------------------------
void launch_select(const dppo_select_params& p, int n_bottom, const float* rewards, const float* hist,
                   const float* u_prompt, const float* u_comp, float* adv, float* mean_abs_adv,
                   uint8_t* keep_prompt, uint8_t* keep_comp, float* gamma_q, float* gamma_o,
                   float* coef, int32_t* counts, float* prune_q, float* prune_o, hipStream_t st);
void launch_variance_terms(int32_t Q, int32_t G, const float* g, const float* prune_q, const float* prune_o,
                           double* group_out, double* total_out, hipStream_t st);

void launch_history_update(int32_t n, const int32_t* prompt_index, const uint8_t* keep_prompt,
                           const float* mean_abs_adv, float* hist_table, int64_t table_size, hipStream_t st);

// ---- packing (pack.hip) -----------------------------------------------------
void launch_pack(const dppo_pack_params& p, const int32_t* prompt_len, const int32_t* comp_len,
                 const uint8_t* keep, int32_t* order, int32_t* row_ptr, int32_t* cu, int32_t* lcu,
                 int32_t* loss_pos, int64_t loss_pos_capacity, int32_t* meta, hipStream_t st);
void launch_gather_f32(int64_t n, const int32_t* idx, const float* src, float* dst, hipStream_t st);

// ---- layout / elementwise kernels (head_kernels.hip) -------------------------
// E = element type of H and W (float or bf16 stored as uint16_t).
struct ChunkView {
    int64_t n0;    // first loss token of the chunk
    int32_t n_c;   // loss tokens in the chunk
    int32_t n_cp;  // padded chunk rows (multiple of 256)
};

void launch_fill_zero(void* p, size_t bytes, hipStream_t st);
// y[n] = target id of loss token n0+n and rowc[n] = its row of H, both clamped into range (a clamp
// that changed something is OR-ed into *status, see DPPO_HEAD_BAD_*; status may be NULL);
// Hc[n_cp, D] = H[rowc[n]] (zero rows beyond n_c); HcT[D, n_cp] its transpose (may be NULL).
void launch_gather_rows(int dtype, const void* H, const int32_t* ids, const int32_t* loss_pos,
                        int64_t T, int32_t D, int32_t V, ChunkView cv, void* Hc, void* HcT,
                        int32_t* y, int32_t* rowc, int32_t* status, hipStream_t st);
// Blocked layout of the B operand of the dH and dW GEMMs (WT, HcT): blocks of GEMM_B_BLOCK_ROWS rows x
// GEMM_B_BLOCK_K columns of a [rows, K] matrix, block (i, j) at (i * K / GEMM_B_BLOCK_K + j) blocks from
// the start, row-major inside; the rows are padded to whole blocks (the pad rows are never written and only
// reach output columns that are not stored).
constexpr int GEMM_B_BLOCK_ROWS = 256, GEMM_B_BLOCK_K = 64;
inline size_t gemm_b_blocked_elems(int64_t rows, int64_t K) {
    return (size_t)((rows + GEMM_B_BLOCK_ROWS - 1) / GEMM_B_BLOCK_ROWS * GEMM_B_BLOCK_ROWS) * (size_t)K;
}
// WT = transpose of W[V, D], columns v >= V zero: row-major [D, Vp] (float32) or blocked (bfloat16, K = Vp).
void launch_transpose_w(int dtype, const void* W, int32_t V, int32_t D, int32_t Vp, void* WT,
                        hipStream_t st);
// zy[n] = Hc[n] . W[y[n]] in fp32; also copied to bref[n] and *flag cleared where not NULL.
void launch_target_logit(int dtype, const void* Hc, const void* W, const int32_t* y, int32_t n_cp,
                         int32_t D, float* zy, float* bref, int32_t* flag, hipStream_t st);
// lse from per-tile partial (max, sumexp) pairs part[tile][n_cp]; logp = zy - lse.
void launch_combine_logprob(const float2* part, int32_t n_tiles, const float* zy, ChunkView cv,
                            float* lse_chunk, float* logp_out, float* lse_out, hipStream_t st);
// Statistics of the GEMM that stores exponentials against the per-token reference bref[n]:
// part[tile][n] = (max z, sum exp(z - bref[n])); lse = bref + log(sum), logp = zy - lse, mx[n] = row
// maximum. Tokens whose sum is out of the safe range are appended to redo_list (count in
// *redo_count, cleared beforehand by launch_target_logit) instead.
void launch_combine_exp(const float2* part, int32_t n_tiles, const float* zy, const float* bref, ChunkView cv,
                        float* lse_chunk, float* logp_out, float* mx, int32_t* redo_count, int32_t* redo_list,
                        float* redo_sum, hipStream_t st);
// Redoes the listed tokens against their row maximum, with plain fp32 dot products: E rows,
// lse, logp, and bref[n] = mx[n]. Costs one pass over W per 8 listed tokens; nothing when the list
// is empty.
void launch_exp_redo_rows(const int32_t* redo_count, const int32_t* redo_list, float* redo_sum, const void* Hc,
                          const void* W, int32_t V, int32_t Vp, int32_t D, const float* zy, const float* mx,
                          ChunkView cv, void* E, int64_t lde, float* bref, float* lse_chunk, float* logp_out,
                          hipStream_t st);
// scale[n] = -c[n] exp(bref[n] - lse[n]) (0 beyond n_c) and the target entry of the stored
// exponentials E (blocked chunk, pitch lde) replaced by exp(zy - bref) - exp(lse - bref), so that
// scale[n] E[n, v] = c[n] (1[v == y[n]] - softmax[n, v]).
void launch_softmax_scale(const int32_t* y, const float* zy, const float* bref, const float* lse, const float* c,
                          ChunkView cv, void* E, int64_t lde, float* scale, hipStream_t st);
// HcT = transpose of diag(scale) Hc[n_cp, D] in bf16 (scale NULL = 1), in the blocked B-operand layout (K = n_cp).
void launch_scale_transpose_bf16(const void* Hc, const float* scale, int32_t n_cp, int32_t D, void* HcT, hipStream_t st);
// fp32 path: row statistics straight from stored logits Z[n_cp, ldz].
void launch_row_stats_f32(const float* Z, int64_t ldz, int32_t V, const int32_t* y, ChunkView cv,
                          float* lse_chunk, float* logp_out, float* lse_out, hipStream_t st);

struct TokenLossArgs {
    const int32_t* loss_cu; int32_t S;
    const float* seq_adv; const float* seq_coef;
    const float* logp_old; const float* logp_ref;
    const float* logp;      // [N] current-policy log-probs (written by the combine step)
    float lo, hi, beta;     // ratio bounds 1-clip_lo, 1+clip_hi and KL weight
    int32_t ratio_level, aggregation;
    const float* seq_ratio; // [S] sequence-level ratio (ratio_level 1), else unused
    float* c_chunk;         // [n_cp] dL/dlogp of the chunk's tokens (0 beyond n_c)
    float* ell; float* kl; float* clipped;   // [N] per-token loss, KL, clipped-away flag
};
void launch_token_loss(const TokenLossArgs& a, ChunkView cv, hipStream_t st);
// seq_ratio[s] = exp(mean over the sequence's tokens of logp - logp_old) for the sequences that end
// in the token range (n_lo, n_hi]; sequences that start below n_lo and end beyond n_hi are flagged
// in `status` (may be NULL) as DPPO_HEAD_SEQ_TOO_LONG.
void launch_seq_ratio(const int32_t* loss_cu, int32_t S, const float* logp, const float* logp_old,
                      float* seq_ratio, int64_t n_lo, int64_t n_hi, int32_t* status, hipStream_t st);
void launch_token_norm_coef(int32_t Q, int32_t G, const int32_t* comp_len, const float* coef, float* coef_out,
                            hipStream_t st);

// float32 path, in place over the chunk's stored logits: G[n,v] = c[n] (1[v==y[n]] - exp(z - lse[n]))
// for v < V, 0 for V <= v < Vp; row-major [n_cp, Vp], also written transposed to GT[Vp, n_cp].
void launch_grad_logits_f32(float* ZG, float* GT, int32_t V, int32_t Vp, const int32_t* y, const float* lse,
                            const float* c, int32_t n_cp, hipStream_t st);

struct SeqReduceArgs {
    const int32_t* loss_cu; int32_t S; int64_t N;
    const float* seq_coef;
    int32_t aggregation;    // 0: per-sequence mean of ell, 1: sum
    const float* ell; const float* kl; const float* clipped;
    float* seq_mean; float* seq_kl; float* seq_clip;   // [S] scratch
    float* seq_loss_out;                                // [S] or NULL
    float* loss_out; float* stats_out;                  // [1], [4] or NULL
};
void launch_seq_reduce(const SeqReduceArgs& a, hipStream_t st);

// ---- GEMMs -------------------------------------------------------------------
// Output description of C[M,N] = A[M,K] B[N,K]^T.
struct StoreSpec {
    void* C; int64_t ldc;
    int32_t out_bf16;          // 0: float output, 1: bf16 output
    int32_t accumulate;        // add to existing contents (float output only)
    const int32_t* row_map;    // output row = row_map[row_base + m] if not NULL
    int64_t row_base;
};
// fp32 reference-grade GEMM (any sizes), gemm_plain.hip.
void launch_gemm_plain_f32(const float* A, int64_t lda, const float* B, int64_t ldb, int32_t M,
                           int32_t N, int32_t K, const StoreSpec& out, hipStream_t st);

// bf16 MFMA GEMMs (gemm_mfma.hip). K must be a multiple of 64; A and B rows may be read up
// to the next multiple of the tile size, so operands are padded scratch buffers or clamped.
// Kernel attribute setup for the current device (once per device) and its compute-unit count;
// returns a dppo status.
int mfma_setup(int* compute_units);
// Vocabulary GEMM: rows = vocabulary entries (A = W[V,D]), columns = tokens (B = Hc[n_cp,D]).
// Writes per-(row tile, token) partial (max, sum exp(z - max)) to part[tile*n_cp + n].
int32_t mfma_logits_row_tiles(int32_t V);
int32_t mfma_vocab_tile();
void launch_mfma_logits(const void* W, int32_t V, int32_t D, const void* Hc, int32_t n_cp, float2* part,
                        hipStream_t st);
// Same GEMM; stores E[n, v] = exp(z[n, v] - bref[n]) as bf16 (0 for V <= v < Vp) to E, a [n_cp, lde]
// matrix in the blocked chunk layout (blocks of 64 tokens x 256 vocabulary entries, each
// contiguous; block (i, j) at element i * 64 * lde + j * 16384); lde = Vp must be a multiple of
// mfma_vocab_tile() (whole tiles are stored). part[tile*n_cp + n] = (max z, sum exp(z - bref[n]))
// over the tile's rows. Returns a dppo status.
int launch_mfma_logits_exp(const void* W, int32_t V, int32_t D, const void* Hc, int32_t n_cp, float2* part,
                           const float* bref, void* E, int64_t lde, int32_t Vp, hipStream_t st);
// Same GEMM, but the epilogue turns logits straight into gradient entries
// G[n,v] = c[n] (1[v==y[n]] - exp(z - lse[n])) written as bf16 to the blocked chunk G (pitch ldg = Vp).
int launch_mfma_logits_grad(const void* W, int32_t V, int32_t D, const void* Hc, int32_t n_cp,
                            const int32_t* y, const float* lse, const float* c, void* G, int64_t ldg,
                            int32_t Vp, hipStream_t st);
// dH rows of a chunk: C[n_c, D] = diag(row_scale) G[n_c, Vp] WT[D, Vp]^T with G in the blocked chunk
// layout (pitch Vp) and WT in the blocked B-operand layout; row_scale may be NULL (= 1). `partial`: as for
// launch_mfma_dw.
void launch_mfma_dh(int cus, const void* G, int32_t Vp, const void* WT, int32_t n_c, int32_t D, const float* row_scale,
                    const StoreSpec& out, float* partial, hipStream_t st);
// dW of a chunk: C[V, D] (+)= G^T HcT^T = sum_n G[n, v] HcT[d, n] (HcT in the blocked B-operand layout, K = n_cp),
// G read k-major from the same blocks.
// `partial` is scratch of mfma_dw_partial_bytes() bytes (or NULL): with it, the tiles of a
// sparsely filled last round are split along K over the idle compute units (cus = compute units
// of the device).
size_t mfma_dw_partial_bytes();
void launch_mfma_dw(int cus, const void* G, int32_t Vp, const void* HcT, int32_t n_cp, int32_t V, int32_t D,
                    const StoreSpec& out, float* partial, hipStream_t st);

// Benchmark aid: device array of 12 counters (3 GEMM stages x {prologue, main loop, epilogue cycles, tiles})
// that the whole-tile launches of the vocabulary, dH and dW GEMMs add to; NULL switches it off.
void mfma_set_phase_counters(unsigned long long* counters);
// Register-only MFMA loop on `cus` workgroups (benchmark aid); returns the flop it enqueues. out: cus floats.
double launch_mfma_rate_probe(int cus, int iters, int random_values, float* out, hipStream_t st);

}  // namespace dppo
