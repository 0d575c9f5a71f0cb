// Selection kernels: group-relative advantages (Eq. 2), completion and prompt candidate
// sets (Eq. 14-17), Bernoulli or fixed-count prune masks from caller-supplied uniforms, the discrete
// importance-rescaling weights (Eq. 18) and the history carry-forward (Eq. 16). Tiny, latency-bound
// work: one thread per group,
// fp64 in a fixed order so that the masks are a bit-exact function of the inputs.
// This file is compiled with floating-point contraction off.
#include "dppo_internal.h"

namespace dppo {
namespace {

// One thread per prompt group: advantages, mean |A|, candidate flag (bit 1 of keep_comp).
__global__ void select_group_kernel(int Q, int G, double eps, int ddof, const float* __restrict__ rewards,
                                    float* __restrict__ adv, float* __restrict__ mean_abs_adv,
                                    uint8_t* __restrict__ cand) {
    int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= Q) return;
    const float* r = rewards + (size_t)k * G;
    double S = 0.0;
    for (int i = 0; i < G; ++i) S = S + (double)r[i];
    double mu = S / (double)G;
    double ss = 0.0;
    for (int i = 0; i < G; ++i) {
        double d = (double)r[i] - mu;
        ss = ss + d * d;
    }
    double sd = sqrt(ss / (double)(G - ddof));
    double sum_abs = 0.0;
    for (int i = 0; i < G; ++i) {
        double a = ((double)r[i] - mu) / (sd + eps);
        adv[(size_t)k * G + i] = (float)a;
        sum_abs = sum_abs + fabs(a);
    }
    mean_abs_adv[k] = (float)(sum_abs / (double)G);
    // |A_i| <= mean_j |A_j|  <=>  G |G r_i - S| <= sum_j |G r_j - S|   (Eq. 15, exact on integers)
    double tot = 0.0;
    for (int i = 0; i < G; ++i) tot = tot + fabs((double)G * (double)r[i] - S);
    for (int i = 0; i < G; ++i) {
        double e = fabs((double)G * (double)r[i] - S);
        cand[(size_t)k * G + i] = ((double)G * e <= tot) ? 2 : 0;   // bit 1 = candidate
    }
}

// Number pruned from a candidate set of n in the fixed-count form: floor(r n), with the float32
// rate's rounding absorbed (0.9f * 10 -> 9) and at least one candidate left.
__device__ __forceinline__ int fixed_prune_count(float r, int n) {
    if (n <= 0) return 0;
    int m = (int)floor((double)r * (double)n * (1.0 + 1e-6));
    m = m < 0 ? 0 : m;
    return m < n - 1 ? m : n - 1;
}

// One workgroup: rank prompts by (hist, index), mark the n_bottom lowest as candidates (bit 1 of
// keep_prompt), prune them (Bernoulli: u < r_q; fixed count: the floor(r_q n_bottom) smallest
// (u, index)), set bit 0 of keep_prompt for the retained ones and count them.
__global__ void select_prompt_kernel(int Q, int n_bottom, float r_q, int fixed_count,
                                     const float* __restrict__ hist, const float* __restrict__ u_prompt,
                                     uint8_t* keep_prompt, int32_t* __restrict__ counts) {
    __shared__ int s_count;
    if (threadIdx.x == 0) s_count = 0;
    const bool active = hist != nullptr && u_prompt != nullptr && n_bottom > 0;
    for (int k = threadIdx.x; k < Q; k += blockDim.x) {
        bool inB = false;
        if (active) {
            const float hk = hist[k];
            int rank = 0;
            for (int j = 0; j < Q; ++j) {
                const float hj = hist[j];
                rank += (hj < hk || (hj == hk && j < k)) ? 1 : 0;
            }
            inB = rank < n_bottom;
        }
        keep_prompt[k] = inB ? 2 : 0;
    }
    __syncthreads();
    const int m_q = fixed_count ? fixed_prune_count(r_q, active ? n_bottom : 0) : 0;
    int local = 0;
    for (int k = threadIdx.x; k < Q; k += blockDim.x) {
        const bool inB = (keep_prompt[k] & 2) != 0;
        bool pruned = false;
        if (inB) {
            if (!fixed_count) {
                pruned = u_prompt[k] < r_q;
            } else {
                const float uk = u_prompt[k];
                int rank = 0;       // candidates ordered by (u, index); bit 1 never changes in this pass
                for (int j = 0; j < Q; ++j) {
                    if ((keep_prompt[j] & 2) == 0) continue;
                    const float uj = u_prompt[j];
                    rank += (uj < uk || (uj == uk && j < k)) ? 1 : 0;
                }
                pruned = rank < m_q;
            }
        }
        keep_prompt[k] = (uint8_t)((inB ? 2 : 0) | (pruned ? 0 : 1));
        local += pruned ? 0 : 1;
    }
    atomicAdd(&s_count, local);   // integer: exact in any order
    __syncthreads();
    if (threadIdx.x == 0) counts[0] = s_count;
}

// One thread per prompt group: completion masks, retained counts, gamma_q, gamma_o, coef. While it
// runs, bit 1 of a flag byte means "candidate" and bit 0 "retained"; the bytes leave as 0 / 1.
// The rate P that enters Eq. 18 is r for candidates (Bernoulli, or fixed count with nominal
// weights) or the realised m/n of the candidate set, 0 for non-candidates.
__global__ void select_weight_kernel(int Q, int G, int n_bottom, float r_q, float r_o, int fixed_count,
                                     int realised_rate, const float* __restrict__ u_comp, uint8_t* keep_prompt,
                                     uint8_t* keep_comp, float* __restrict__ gamma_q,
                                     float* __restrict__ gamma_o, float* __restrict__ coef,
                                     int32_t* __restrict__ counts, float* __restrict__ prune_q,
                                     float* __restrict__ prune_o) {
    int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= Q) return;
    const int n_q = counts[0];
    const uint8_t fp = keep_prompt[k];
    const bool kp = (fp & 1) != 0;
    double Pq = 0.0;
    if ((fp & 2) != 0)
        Pq = (fixed_count && realised_rate) ? (double)fixed_prune_count(r_q, n_bottom) / (double)n_bottom : (double)r_q;
    uint8_t* flags = keep_comp + (size_t)k * G;
    const float* u = u_comp ? u_comp + (size_t)k * G : nullptr;
    int n_cand = 0;
    for (int i = 0; i < G; ++i) n_cand += (flags[i] & 2) != 0 ? 1 : 0;
    const int m_o = (fixed_count && u != nullptr) ? fixed_prune_count(r_o, n_cand) : 0;
    double Po_cand = 0.0;
    if (u != nullptr) Po_cand = (fixed_count && realised_rate) ? (double)m_o / (double)(n_cand > 0 ? n_cand : 1) : (double)r_o;
    int n_o = 0;
    for (int i = 0; i < G; ++i) {
        const bool is_cand = (flags[i] & 2) != 0;
        bool pruned = false;
        if (u != nullptr && is_cand) {
            if (!fixed_count) {
                pruned = u[i] < r_o;
            } else {
                int rank = 0;       // candidates of the group ordered by (u, index)
                for (int j = 0; j < G; ++j) {
                    if ((flags[j] & 2) == 0) continue;
                    rank += (u[j] < u[i] || (u[j] == u[i] && j < i)) ? 1 : 0;
                }
                pruned = rank < m_o;
            }
        }
        const bool keep = kp && !pruned;
        flags[i] = (uint8_t)((keep ? 1 : 0) | (is_cand ? 2 : 0));
        n_o += keep ? 1 : 0;
    }
    counts[1 + k] = n_o;
    const double gq = kp ? ((double)n_q / (double)Q) / (1.0 - Pq) : 0.0;
    gamma_q[k] = (float)gq;
    if (prune_q) prune_q[k] = (float)Pq;
    keep_prompt[k] = kp ? 1 : 0;
    for (int i = 0; i < G; ++i) {
        const size_t idx = (size_t)k * G + i;
        const bool keep = (flags[i] & 1) != 0;
        const double Po = (flags[i] & 2) != 0 ? Po_cand : 0.0;
        double go = 0.0, cf = 0.0;
        if (keep) {
            go = ((double)n_o / (double)G) / (1.0 - Po);
            cf = gq * go / (double)((int64_t)n_q * (int64_t)n_o);
        }
        gamma_o[idx] = (float)go;
        coef[idx] = (float)cf;
        if (prune_o) prune_o[idx] = (float)Po;
        flags[i] = keep ? 1 : 0;
    }
}

// Carry-forward history score (Eq. 16): selected prompts take their fresh mean |A|.
__global__ void history_update_kernel(int n, const int32_t* __restrict__ prompt_index,
                                      const uint8_t* __restrict__ keep_prompt,
                                      const float* __restrict__ mean_abs_adv, float* __restrict__ hist_table,
                                      int64_t table_size) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= n) return;
    const int64_t q = prompt_index[b];
    if (keep_prompt[b] != 0 && q >= 0 && q < table_size) hist_table[q] = mean_abs_adv[b];
}

// App. D in float64, fixed order: threads take prompt groups, thread 0 sums over the groups.
__global__ __launch_bounds__(256) void variance_terms_kernel(int Q, int G, const float* __restrict__ g,
                                                             const float* __restrict__ prune_q,
                                                             const float* __restrict__ prune_o,
                                                             double* __restrict__ group_out,
                                                             double* __restrict__ total_out) {
    for (int k = threadIdx.x; k < Q; k += blockDim.x) {
        const float* gk = g + (size_t)k * G;
        const float* pk = prune_o + (size_t)k * G;
        double s1 = 0.0, s2 = 0.0, keep = 0.0, w2 = 0.0, c2 = 0.0;
        int nc = 0;
        for (int i = 0; i < G; ++i) {
            const double x = (double)gk[i], P = (double)pk[i];
            s1 = s1 + x;
            s2 = s2 + x * x;
            keep = keep + (1.0 - P);
            w2 = w2 + x * x / (1.0 - P);
            if (P > 0.0) { c2 = c2 + x * x / (1.0 - P); nc += 1; }
        }
        const double Gq = s1 / G, m2 = s2 / G, Co = keep / G;
        group_out[4 * k + 0] = Gq;
        group_out[4 * k + 1] = m2 - Gq * Gq;
        group_out[4 * k + 2] = (Co / G) * w2 - Gq * Gq;
        group_out[4 * k + 3] = (nc == 0 || c2 / nc <= m2) ? 1.0 : 0.0;
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    double sG = 0.0, sG2 = 0.0, keep = 0.0, wG2 = 0.0, inv = 0.0, sVarO = 0.0, wVar = 0.0, c2 = 0.0;
    int nc = 0;
    for (int k = 0; k < Q; ++k) {
        const double Gq = group_out[4 * k], P = (double)prune_q[k];
        sG = sG + Gq;
        sG2 = sG2 + Gq * Gq;
        keep = keep + (1.0 - P);
        wG2 = wG2 + Gq * Gq / (1.0 - P);
        inv = inv + 1.0 / (1.0 - P);
        sVarO = sVarO + group_out[4 * k + 1];
        wVar = wVar + group_out[4 * k + 2] / (1.0 - P);
        if (P > 0.0) { c2 = c2 + Gq * Gq / (1.0 - P); nc += 1; }
    }
    const double Gbar = sG / Q, varQ = sG2 / Q - Gbar * Gbar, Cq = keep / Q;
    const double term1 = (Cq / Q) * wG2 - Gbar * Gbar, eg2 = (Cq / Q) * inv, term2 = (Cq / Q) * wVar;
    total_out[0] = Gbar; total_out[1] = varQ; total_out[2] = term1;
    total_out[3] = (nc == 0 || c2 / nc <= sG2 / Q) ? 1.0 : 0.0;
    total_out[4] = eg2; total_out[5] = sVarO / Q; total_out[6] = term2; total_out[7] = term1 + term2;
    total_out[8] = varQ + eg2 * (sVarO / Q); total_out[9] = 0.0;
}

}  // namespace

void launch_variance_terms(int32_t Q, int32_t G, const float* g, const float* prune_q, const float* prune_o,
                           double* group_out, double* total_out, hipStream_t st) {
    variance_terms_kernel<<<1, 256, 0, st>>>(Q, G, g, prune_q, prune_o, group_out, total_out);
}

void launch_select(const dppo_select_params& p, int n_bottom, const float* rewards, const float* hist,
                   const float* u_prompt, const float* u_comp, float* adv, float* mean_abs_adv,
                   uint8_t* keep_prompt, uint8_t* keep_comp, float* gamma_q, float* gamma_o,
                   float* coef, int32_t* counts, float* prune_q, float* prune_o, hipStream_t st) {
    const int threads = 64;
    const int blocks = (p.Q + threads - 1) / threads;
    select_group_kernel<<<blocks, threads, 0, st>>>(p.Q, p.G, (double)p.adv_eps, p.std_ddof, rewards, adv,
                                                    mean_abs_adv, keep_comp);
    select_prompt_kernel<<<1, 1024, 0, st>>>(p.Q, n_bottom, p.r_q, p.fixed_count, hist, u_prompt, keep_prompt,
                                             counts);
    select_weight_kernel<<<blocks, threads, 0, st>>>(p.Q, p.G, n_bottom, p.r_q, p.r_o, p.fixed_count,
                                                     p.realised_rate, u_comp, keep_prompt, keep_comp, gamma_q,
                                                     gamma_o, coef, counts, prune_q, prune_o);
}

void launch_history_update(int32_t n, const int32_t* prompt_index, const uint8_t* keep_prompt,
                           const float* mean_abs_adv, float* hist_table, int64_t table_size, hipStream_t st) {
    if (n <= 0) return;
    history_update_kernel<<<(n + 255) / 256, 256, 0, st>>>(n, prompt_index, keep_prompt, mean_abs_adv, hist_table,
                                                          table_size);
}

}  // namespace dppo
