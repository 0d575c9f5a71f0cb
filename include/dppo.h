/*
 * dppo.h -- C ABI of the MI355X (gfx950) library for the DPPO policy-loss hot path:
 * selection (advantages, prune masks, importance-rescaling weights), dense packing,
 * fused LM-head token log-probabilities, and the reweighted GRPO loss forward+backward.
 *
 * Conventions that hold for every call unless an argument says otherwise
 *   - every array pointer is a DEVICE pointer owned by the caller; the library never
 *     allocates or frees device memory (scratch is the caller's `ws`);
 *   - parameter structs and the returned status live on the host;
 *   - calls are asynchronous on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and never synchronise it (the one exception is the benchmark aid
 *     dppo_timing_read, which waits for its events on the host);
 *   - arguments that can be checked on the host (NULL pointers, non-positive sizes,
 *     rates outside [0,1), too small a workspace) are checked before anything is
 *     launched: the call returns an error status and launches nothing;
 *   - conditions only the device can see are reported through a device-side status
 *     word (dppo_pack: meta[3]; the LM-head calls: `status`) and leave the outputs defined;
 *   - the library keeps no state between calls except: the message of the last error
 *     (per thread), per-device kernel attributes and compute-unit count (looked up on the
 *     first bfloat16 LM-head call on each device), and the optional stage timing below;
 *   - no C++ exception crosses this boundary.
 */
#ifndef DPPO_H_
#define DPPO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DPPO_OK = 0,
    DPPO_ERR_INVALID_ARG = 1, /* NULL pointer, value out of range                      */
    DPPO_ERR_SHAPE = 2,       /* non-positive or inconsistent sizes                    */
    DPPO_ERR_CAPACITY = 3,    /* an item longer than the packing window                */
    DPPO_ERR_WORKSPACE = 4,   /* workspace missing, misaligned or too small            */
    DPPO_ERR_UNSUPPORTED = 5, /* shape or dtype outside what the kernels are built for */
    DPPO_ERR_DEVICE = 6       /* a HIP runtime call failed                             */
} dppo_status;

/* Static description of a status code (never NULL). */
const char* dppo_status_str(int status);
/* Detail of the last error raised on the calling thread ("" if none; never NULL). */
const char* dppo_last_error(void);

/* --------------------------------------------------------------------------------
 * dppo_select -- Sec. 3 Eq. 2 and Sec. 4.2 Eq. 14-18 of the paper.
 *
 * For a batch of Q prompts with G completions each:
 *   adv[k,i]        group-relative advantage (r - mean_k) / (std_k + adv_eps), from the
 *                   full group, std with divisor G - std_ddof                     (Eq. 2)
 *   mean_abs_adv[k] the prompt's threshold / next-epoch history score            (Eq. 14)
 *   completion candidates: |adv[k,i]| <= mean_abs_adv[k], decided exactly in fp64 on the
 *                   equivalent form G|G r_i - S| <= sum_j |G r_j - S|            (Eq. 15)
 *   prompt candidates: the floor(bottom_frac*Q) prompts with the lowest hist[k], ties to
 *                   the lower index; none if hist or u_prompt is NULL (first epoch)(Eq. 17)
 *   masks: a candidate prompt is pruned iff u_prompt[k] < r_q, a candidate completion iff
 *                   u_comp[k,i] < r_o (float32 compares); completions of a pruned prompt
 *                   are dropped; u_comp NULL = no completion pruning. With fixed_count the
 *                   floor(r n) candidates with the smallest uniforms are pruned instead
 *                   (App. A, Alg. 1; floor taken after scaling r n by 1 + 1e-6 because r is float32)
 *   gamma_q[k]   = (|S^q|/Q) / (1 - P^q_k),  gamma_o[k,i] = (|S^o_k|/G) / (1 - P^o_{k,i})
 *                   with the realised retained counts; 0 for pruned entries      (Eq. 18)
 *   coef[k,i]    = gamma_q gamma_o / (|S^q| |S^o_k|): weight of sequence (k,i) in the batch
 *                   loss (mean over retained prompts of the mean over retained completions)
 *   counts[0] = |S^q|, counts[1+k] = |S^o_k| (0 for a pruned prompt)
 *   prune_q[k], prune_o[k,i] (optional): the prune probability P^q_k, P^o_{k,i} that entered
 *                   Eq. 18 (0 for non-candidates), whether or not the item was pruned
 *
 * Layout: rewards, u_comp, adv, keep_comp, gamma_o, coef are [Q*G] row-major (prompt
 * major); hist, u_prompt, mean_abs_adv, keep_prompt, gamma_q are [Q]; counts is [1+Q].
 * Masks are bit-exact functions of the inputs. Requires Q <= 16384, G <= 1024,
 * G - std_ddof >= 1, r_q and r_o in [0,1), 0 <= bottom_frac <= 1, adv_eps > 0 (a group of
 * equal rewards has standard deviation 0; with adv_eps > 0 its advantages are 0).
 */
typedef struct {
    int32_t Q, G;
    float r_q, r_o;     /* prune probabilities of candidate prompts / completions */
    float adv_eps;      /* added to the standard deviation (1e-6 customary)       */
    int32_t std_ddof;   /* 0 = population, 1 = sample standard deviation          */
    float bottom_frac;  /* fraction of prompts that are candidates (paper: 0.5)   */
    int32_t fixed_count;    /* 0: Bernoulli pruning (u < r); 1: exactly floor(r n) of each
                               candidate set of n are pruned (App. A, Alg. 1): those with the
                               smallest (uniform, index); one candidate always survives      */
    int32_t realised_rate;  /* fixed_count only. 1: Eq. 18 uses the realised rate floor(r n)/n
                               (exactly unbiased); 0: the nominal r, as the equation is printed */
} dppo_select_params;

int dppo_select(const dppo_select_params* p,
                const float* rewards, const float* hist /* or NULL */,
                const float* u_prompt /* or NULL */, const float* u_comp /* or NULL */,
                float* adv, float* mean_abs_adv,
                uint8_t* keep_prompt, uint8_t* keep_comp,
                float* gamma_q, float* gamma_o, float* coef,
                int32_t* counts, float* prune_q /* or NULL */, float* prune_o /* or NULL */, void* stream);

/* dppo_history_update -- Sec. 4.2 Eq. 16 (carry-forward history score).
 * For the n prompts of a batch, prompt b being entry prompt_index[b] of the dataset-wide
 * score table hist_table[table_size]: a prompt retained in this epoch (keep_prompt[b] != 0)
 * takes its fresh score mean_abs_adv[b]; a pruned prompt keeps its last score. Indices
 * outside the table are ignored; indices must be distinct within a call.
 */
int dppo_history_update(int32_t n, const int32_t* prompt_index, const uint8_t* keep_prompt,
                        const float* mean_abs_adv, float* hist_table, int64_t table_size, void* stream);

/* --------------------------------------------------------------------------------
 * dppo_pack -- Sec. 4.3 (Dense Prompt Packing), applied to the retained sequences.
 *
 * Items are the n_items sequences in index order, item j having prompt_len[j] +
 * comp_len[j] tokens; items with keep[j] == 0 are skipped (keep NULL = all kept).
 * A pool of up to n_win items in arrival order is refilled from the stream after every
 * placement. The paper leaves the greedy choice inside the pool open; `policy` picks a reading:
 *   DPPO_PACK_FIRST_FIT  for each row of `capacity` tokens the pool is scanned from oldest to
 *                        newest (items fetched meanwhile included) and every item that still
 *                        fits is placed;
 *   DPPO_PACK_BEST_FIT   the longest pool item that fits is placed (the oldest among equals),
 *                        repeatedly, refilled items included, until no pool item fits.
 * comp_len NULL packs prompts alone, the paper's own use before any rollout: loss_cu is then
 * all zero, N = 0, and loss_pos is not touched (it may be NULL). capacity 0 stands for
 * L_max = the longest kept item, the paper's definition.
 *
 * Outputs (all int32):
 *   order[s]       original index of the s-th packed sequence           [n_items], S valid
 *   row_ptr[r]     first packed sequence of row r                       [n_items+1], n_rows+1 valid
 *   cu_seqlens[s]  first token of packed sequence s; [S] = T            [n_items+1]
 *   loss_cu[s]     first loss token of packed sequence s; [S] = N       [n_items+1]
 *   loss_pos[n]    packed position whose hidden state predicts the n-th completion token:
 *                  sequence s contributes cu[s]+P-1 ... cu[s]+P+C-2     [loss_pos_capacity]
 *   meta[8]        {n_rows, T, N, device_status, S, capacity used, d_lo, d_hi}; d_lo, d_hi are the
 *                  low and high 32 bits of a double: the fill density T / (n_rows * capacity
 *                  used), the share of row slots that hold a real token (0 if nothing is packed)
 * device_status: 0 ok; 1 = a kept item has prompt_len < 1, comp_len < 1 or does not fit
 * `capacity`; 2 = N exceeds loss_pos_capacity; 3 = T does not fit int32. On a non-zero
 * status n_rows = T = N = S = 0 and no other output is meaningful.
 * cu_seqlens and loss_cu are also used as scratch while packing.
 * The result is a bit-exact function of the inputs (one deterministic wavefront).
 */
enum { DPPO_PACK_FIRST_FIT = 0, DPPO_PACK_BEST_FIT = 1 };

typedef struct {
    int32_t n_items, capacity, n_win;
    int32_t policy;   /* DPPO_PACK_FIRST_FIT or DPPO_PACK_BEST_FIT */
} dppo_pack_params;

int dppo_pack(const dppo_pack_params* p,
              const int32_t* prompt_len, const int32_t* comp_len /* or NULL */, const uint8_t* keep /* or NULL */,
              int32_t* order, int32_t* row_ptr, int32_t* cu_seqlens, int32_t* loss_cu,
              int32_t* loss_pos, int64_t loss_pos_capacity, int32_t* meta, void* stream);

/* dst[i] = src[idx[i]], i < n: puts per-item adv / coef into packed order (idx = order). */
int dppo_gather_f32(int64_t n, const int32_t* idx, const float* src, float* dst, void* stream);

/* --------------------------------------------------------------------------------
 * LM head: pi_theta(o_t | q, o_<t) of Sec. 3 as log-softmax of H W^T gathered at the
 * target token, and the loss of Eq. 1 reweighted by Eq. 18, forward and backward.
 *
 * H[T,D] row-major hidden states of the packed tokens, W[V,D] row-major vocabulary
 * matrix (logits z = H W^T, no bias, temperature 1), ids[T] token ids in [0,V).
 * loss_pos[N] lists the rows of H that predict a completion token; the target of loss
 * token n is ids[loss_pos[n]+1]. loss_pos NULL means identity: N <= T rows of H are
 * loss rows and ids[n] is the target of row n.
 * dtype 0: H, W float32, fp32 arithmetic. dtype 1: H, W bfloat16, bf16 MFMA with fp32
 * accumulation (needs D % 64 == 0). Statistics (max, sum-exp, log-probs, loss terms) are
 * fp32; logits are never written out in full (at most one token chunk at a time, in the
 * workspace).
 * status (device int32, or NULL): cleared at the start of the call, then OR-ed with
 *   DPPO_HEAD_BAD_TARGET    a target id outside [0,V): the id is clamped into the range;
 *   DPPO_HEAD_BAD_POSITION  a loss_pos entry p with p < 0 or p + 1 >= T: the row and its target
 *                           position are clamped into [0,T).
 *   DPPO_HEAD_SEQ_TOO_LONG  (dppo_loss_fwd_bwd with the sequence-level ratio) a sequence has more
 *                           loss tokens than dppo_loss_params.max_seq_tokens promised and its
 *                           ratio was not complete when its first tokens' gradients were formed.
 * Every kernel still runs to the end and every output is defined; what the outputs mean for the
 * offending tokens is up to the caller. Entries of loss_pos must be distinct (not checked).
 */
enum { DPPO_HEAD_BAD_TARGET = 1, DPPO_HEAD_BAD_POSITION = 2, DPPO_HEAD_SEQ_TOO_LONG = 4 };

typedef struct {
    int64_t T, N;
    int32_t D, V;
    int32_t dtype; /* 0 = float32, 1 = bfloat16 */
} dppo_head_shape;

/* Recommended workspace size in bytes (0 if the shape is invalid). Any size of at least
 * dppo_workspace_min_bytes works: a smaller workspace means smaller token chunks.
 * want_backward (both calls): 0 = dppo_token_logprob, 1 = dppo_loss_fwd_bwd, 2 = dppo_loss_fwd_bwd
 * with the sequence-level ratio and max_seq_tokens given (two sets of per-chunk regions). */
size_t dppo_workspace_bytes(const dppo_head_shape* shape, int want_backward);
size_t dppo_workspace_min_bytes(const dppo_head_shape* shape, int want_backward);

/* logp[n] = z[n,y_n] - lse[n], lse[n] = log sum_v exp z[n,v]; lse may be NULL.
 * ws must be 256-byte aligned. */
int dppo_token_logprob(const dppo_head_shape* shape,
                       const void* H, const void* W, const int32_t* ids,
                       const int32_t* loss_pos /* or NULL */,
                       float* logp, float* lse /* or NULL */, int32_t* status /* or NULL */,
                       void* ws, size_t ws_bytes, void* stream);

/* dppo_token_logprob_noalloc -- for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): dppo_token_logprob with
 * the workspace replaced by a fixed device array inside the library, DPPO_STATIC_SCRATCH_MIB MiB
 * per GPU the library runs on, held until the process ends (dppo_static_scratch_bytes() returns
 * the size in bytes). Same arguments, kernels and results otherwise; the token chunks are as
 * large as that array allows (about 6 000 tokens at D = 2560, V = 151936), so large batches run
 * slower than with a recommended-size workspace. The call itself allocates and frees nothing and
 * calls no allocating routine (keep stage timing off: it creates events).
 * A shape whose smallest chunk (256 tokens: 256 rows of H, the per-tile softmax statistics and
 * a few vectors) does not fit the array is refused with DPPO_ERR_WORKSPACE and nothing is launched.
 * All calls on one GPU share that GPU's array, whose contents are whatever the last call left
 * (no part of it needs to start at zero: every region is written before it is read): calls that
 * overlap in time on one GPU, on different streams or threads, race on it. */
#define DPPO_STATIC_SCRATCH_MIB 64
size_t dppo_static_scratch_bytes(void);
int dppo_token_logprob_noalloc(const dppo_head_shape* shape,
                               const void* H, const void* W, const int32_t* ids,
                               const int32_t* loss_pos /* or NULL */,
                               float* logp, float* lse /* or NULL */, int32_t* status /* or NULL */,
                               void* stream);

/* Loss L = sum_s seq_coef[s] * (1/C_s) * sum_{n in s} l_n over the S packed sequences
 * (segments loss_cu[s]..loss_cu[s+1] of the loss tokens, C_s their length; loss_cu must be
 * non-decreasing from 0 to N, and an empty segment contributes 0, with seq_loss[s] = 0), with
 *   rho = exp(logp - logp_old),  l = -min(rho A, clip(rho, 1-clip_lo, 1+clip_hi) A)
 *   + beta (rho_hat - log rho_hat - 1),  rho_hat = exp(logp_ref - logp),  A = seq_adv[s]
 * (Eq. 1; the weight multiplies surrogate and KL alike), and its gradients
 *   dH[T,D] (dtype of H; rows not in loss_pos are zero) and dW[V,D] (float32; added to
 *   the buffer's contents if accumulate_dW != 0, otherwise overwritten).
 * Optional outputs: logp[N]; seq_loss[S] (token-mean loss of each sequence);
 * stats[4] = {mean KL over loss tokens, fraction of tokens whose surrogate gradient is
 * clipped away, N, 0}. loss is one float on the device.
 * recompute_logits = 0 (bfloat16) keeps, per chunk of tokens, exp(z - target logit) as bfloat16 in
 * the workspace, which the backward GEMMs turn into softmax gradients by a row scale (tokens whose
 * target has a log-prob below about -34 take a slower exact path); 1 runs the vocabulary GEMM a
 * second time in the backward instead and keeps the gradient entries themselves.
 * The call is asynchronous on `stream` and deterministic, except that the log-probs of tokens on
 * that exact path are summed with atomic adds (last bits may vary between runs).
 *
 * Variants for the other objectives the method is plugged into (Sec. 5, robustness across RL
 * algorithms; the paper names them without formulas, these are this library's readings):
 *   ratio_level = DPPO_RATIO_SEQUENCE: one ratio per sequence, exp(mean_n (logp - logp_old)), takes
 *     the place of rho in every token of the sequence (clip and min as above; KL stays per token).
 *     It needs the log-probs of a whole sequence before any of its gradients. With
 *     max_seq_tokens > 0 (the caller's upper bound on the loss tokens of one sequence; loss_cu
 *     lives on the device and the call never reads it back) and a workspace that holds two sets
 *     of per-chunk regions with chunks of at least max_seq_tokens tokens, the forward of chunk
 *     c + 1 runs ahead of the backward of chunk c and the work stays three GEMMs per token; a
 *     sequence that breaks the promise sets DPPO_HEAD_SEQ_TOO_LONG. With max_seq_tokens = 0, or a
 *     workspace too small for that, the vocabulary GEMM runs one extra forward pass over all
 *     tokens first (unless a single chunk holds the batch).
 *   aggregation = DPPO_AGG_TOKEN_SUM: the per-sequence term is sum_n l_n instead of the mean; with
 *     weights from dppo_token_norm_coef this is the token-level normalisation of the decoupled-clip
 *     objective (clip_lo != clip_hi is the decoupled clip itself). seq_loss then holds the sums.
 */
enum { DPPO_RATIO_TOKEN = 0, DPPO_RATIO_SEQUENCE = 1 };
enum { DPPO_AGG_SEQ_MEAN = 0, DPPO_AGG_TOKEN_SUM = 1 };

typedef struct {
    float clip_lo, clip_hi;
    float beta;
    int32_t accumulate_dW;
    int32_t recompute_logits;
    int32_t ratio_level;   /* DPPO_RATIO_TOKEN (Eq. 1) or DPPO_RATIO_SEQUENCE */
    int32_t aggregation;   /* DPPO_AGG_SEQ_MEAN (Eq. 1) or DPPO_AGG_TOKEN_SUM */
    int32_t max_seq_tokens; /* sequence-level ratio only: upper bound on C_s, or 0 = unknown */
} dppo_loss_params;

int dppo_loss_fwd_bwd(const dppo_head_shape* shape, const dppo_loss_params* p, int32_t S,
                      const void* H, const void* W, const int32_t* ids,
                      const int32_t* loss_pos /* or NULL */, const int32_t* loss_cu,
                      const float* seq_adv, const float* seq_coef,
                      const float* logp_old, const float* logp_ref,
                      float* loss, float* logp /* or NULL */, float* seq_loss /* or NULL */,
                      float* stats /* or NULL */, int32_t* status /* or NULL */,
                      void* dH, float* dW,
                      void* ws, size_t ws_bytes, void* stream);

/* dppo_variance_terms -- App. D (variance of the rescaled single-sample estimator
 * gamma(q) gamma(o,q) g(q,o), q and o drawn from the pruned densities) for one scalar component
 * g[Q*G] of the gradient term and the prune probabilities reported by dppo_select.
 *   group_out[4k..4k+3] = { G(q_k) = mean_o g,  Var_O[g],  Var[gamma g] under the pruned completion
 *                           density (App. D.1),  1.0 if the completion-level condition of the
 *                           bound holds for the group else 0.0 }
 *   total_out[10] = { mean of G(q), Var_Q[G(q)], Var[gamma(q) G(q)] (term I), prompt-level
 *                     condition (1/0), E[gamma(q)^2], mean_q Var_O, term II, term I + term II,
 *                     Theorem D.1 bound = Var_Q + E[gamma(q)^2] mean_q Var_O, 0 }
 * All outputs double, computed in float64 in a fixed order (a diagnostic, one workgroup). */
int dppo_variance_terms(int32_t Q, int32_t G, const float* g, const float* prune_q, const float* prune_o,
                        double* group_out, double* total_out, void* stream);

/* coef_out[q*G+i] = coef[q*G+i] * G / sum_j comp_len[q*G+j]: weights for DPPO_AGG_TOKEN_SUM. The sum runs
 * over all G completions of the prompt, pruned ones included (their lengths are known before
 * pruning). Device arrays; coef_out may alias coef. A group whose lengths sum to <= 0 gets 0. */
int dppo_token_norm_coef(int32_t Q, int32_t G, const int32_t* comp_len, const float* coef, float* coef_out,
                         void* stream);

/* --------------------------------------------------------------------------------
 * Optional stage timing, for benchmarks. While enabled, dppo_token_logprob and
 * dppo_loss_fwd_bwd record a pair of HIP events around each launch of the stages below, on
 * the caller's stream (the kernels themselves are unchanged). dppo_timing_read waits for the
 * recorded events (a host-side wait), returns the summed milliseconds and the launch count
 * of every stage since the last reset, and with reset != 0 forgets them. Host arrays.
 * The switch and the recorded events are process-wide state (guarded by a mutex). Events
 * cannot be recorded on a stream that is being captured into a graph: keep timing off then.
 */
enum {
    DPPO_STAGE_LOGITS_GEMM = 0, /* vocabulary GEMM with the online max / sum-exp epilogue */
    DPPO_STAGE_GRAD_LOGITS = 1, /* softmax-gradient pass over the stored chunk (float32), row scales (bfloat16) */
    DPPO_STAGE_DH_GEMM = 2,     /* dH = G W                                               */
    DPPO_STAGE_DW_GEMM = 3,     /* dW += G^T H                                            */
    DPPO_STAGE_ELEMENTWISE = 4, /* every other kernel of the two LM-head calls: row gather, transposes,
                                   target logits, combination of the per-tile statistics, token loss
                                   terms, zero fill of dH, the segmented reduction (HBM-bound)  */
    DPPO_N_STAGES = 5
};
int dppo_timing_enable(int on);
int dppo_timing_read(double* ms /* [DPPO_N_STAGES] */, int64_t* launches /* [DPPO_N_STAGES] */, int reset);

/* Benchmark aid: where the workgroups of the three big GEMMs spend their time. counters: device array of
 * 12 uint64 the caller has zeroed, {vocabulary GEMM, dH GEMM, dW GEMM} x {shader cycles from the start of a
 * workgroup until its first operand slice is in LDS, cycles in the main loop, cycles in the epilogue, number of
 * workgroups}; while set, every whole-tile launch of the bfloat16 LM-head calls adds to it (4 atomic
 * adds per workgroup; the launches that split K are left out). NULL switches it off. Process-wide state,
 * like the stage timing; the array must outlive the launches that write it. */
int dppo_timing_tile_phases(uint64_t* counters);

/* Benchmark aid: enqueues a loop of `iters` x 32 bf16 MFMA instructions (the GEMMs' own, 16x16x32)
 * per wavefront, 8 wavefronts on every compute unit, operands in registers only (random_operands 0:
 * all ones, 1: pseudo-random values in [-1, 1]: the chip's power limit makes the sustained rate depend
 * on the data). *flop (host) receives the floating-point operations enqueued; the caller times the
 * stream and divides: that rate is the ceiling the GEMM stages can be compared with. out (device):
 * at least one float per compute unit of the device (out_floats says how many it holds). */
int dppo_mfma_rate_probe(int random_operands, int iters, float* out, int32_t out_floats, double* flop, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DPPO_H_ */
