// Selection kernels: group-relative advantages (Eq. 2), completion and prompt candidate
// sets (Eq. 14-17), Bernoulli prune masks from caller-supplied uniforms, and the discrete
// importance-rescaling weights (Eq. 18). Tiny, latency-bound work: one thread per group,
// fp64 in a fixed order so that the masks are a bit-exact function of the inputs.
// This file is compiled with floating-point contraction off.
#include "dppo_internal.h"

namespace dppo {
namespace {

// One thread per prompt group: advantages, mean |A|, candidate bits (left in keep_comp).
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
        cand[(size_t)k * G + i] = ((double)G * e <= tot) ? 1 : 0;
    }
}

// One workgroup: rank prompts by (hist, index), mark the n_bottom lowest as candidates, apply
// the uniforms, count the retained prompts. in_bottom is left in gamma_q as 0/1 for the next kernel.
__global__ void select_prompt_kernel(int Q, int n_bottom, float r_q, const float* __restrict__ hist,
                                     const float* __restrict__ u_prompt, uint8_t* __restrict__ keep_prompt,
                                     float* __restrict__ in_bottom, int32_t* __restrict__ counts) {
    __shared__ int s_count;
    if (threadIdx.x == 0) s_count = 0;
    __syncthreads();
    int local = 0;
    for (int k = threadIdx.x; k < Q; k += blockDim.x) {
        bool inB = false;
        if (hist != nullptr && u_prompt != nullptr && n_bottom > 0) {
            float hk = hist[k];
            int rank = 0;
            for (int j = 0; j < Q; ++j) {
                float hj = hist[j];
                rank += (hj < hk || (hj == hk && j < k)) ? 1 : 0;
            }
            inB = rank < n_bottom;
        }
        bool pruned = inB && (u_prompt[k] < r_q);
        keep_prompt[k] = pruned ? 0 : 1;
        in_bottom[k] = inB ? 1.0f : 0.0f;
        local += pruned ? 0 : 1;
    }
    atomicAdd(&s_count, local);   // integer: exact in any order
    __syncthreads();
    if (threadIdx.x == 0) counts[0] = s_count;
}

// One thread per prompt group: completion masks, retained counts, gamma_q, gamma_o, coef.
__global__ void select_weight_kernel(int Q, int G, float r_q, float r_o, const float* __restrict__ u_comp,
                                     const uint8_t* __restrict__ keep_prompt, uint8_t* __restrict__ keep_comp,
                                     float* __restrict__ gamma_q, float* __restrict__ gamma_o,
                                     float* __restrict__ coef, int32_t* __restrict__ counts) {
    int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= Q) return;
    const int n_q = counts[0];
    const bool kp = keep_prompt[k] != 0;
    const double Pq = (gamma_q[k] != 0.0f) ? (double)r_q : 0.0;   // in_bottom flag from the prompt kernel
    int n_o = 0;
    for (int i = 0; i < G; ++i) {
        size_t idx = (size_t)k * G + i;
        bool is_cand = keep_comp[idx] != 0;
        bool pruned = (u_comp != nullptr) && is_cand && (u_comp[idx] < r_o);
        bool keep = kp && !pruned;
        // bit 0: kept, bit 1: candidate (needed for the weight below)
        keep_comp[idx] = (uint8_t)((keep ? 1 : 0) | (is_cand ? 2 : 0));
        n_o += keep ? 1 : 0;
    }
    counts[1 + k] = n_o;
    double gq = kp ? ((double)n_q / (double)Q) / (1.0 - Pq) : 0.0;
    gamma_q[k] = (float)gq;
    for (int i = 0; i < G; ++i) {
        size_t idx = (size_t)k * G + i;
        uint8_t f = keep_comp[idx];
        bool keep = (f & 1) != 0;
        double Po = ((f & 2) != 0 && u_comp != nullptr) ? (double)r_o : 0.0;
        double go = 0.0, cf = 0.0;
        if (keep) {
            go = ((double)n_o / (double)G) / (1.0 - Po);
            cf = gq * go / (double)((int64_t)n_q * (int64_t)n_o);
        }
        gamma_o[idx] = (float)go;
        coef[idx] = (float)cf;
        keep_comp[idx] = keep ? 1 : 0;
    }
}

}  // namespace

void launch_select(const dppo_select_params& p, int n_bottom, const float* rewards, const float* hist,
                   const float* u_prompt, const float* u_comp, float* adv, float* mean_abs_adv,
                   uint8_t* keep_prompt, uint8_t* keep_comp, float* gamma_q, float* gamma_o,
                   float* coef, int32_t* counts, hipStream_t st) {
    const int threads = 64;
    const int blocks = (p.Q + threads - 1) / threads;
    select_group_kernel<<<blocks, threads, 0, st>>>(p.Q, p.G, (double)p.adv_eps, p.std_ddof, rewards, adv,
                                                    mean_abs_adv, keep_comp);
    select_prompt_kernel<<<1, 1024, 0, st>>>(p.Q, n_bottom, p.r_q, hist, u_prompt, keep_prompt, gamma_q, counts);
    select_weight_kernel<<<blocks, threads, 0, st>>>(p.Q, p.G, p.r_q, p.r_o, u_comp, keep_prompt, keep_comp,
                                                     gamma_q, gamma_o, coef, counts);
}

}  // namespace dppo
