// Dense packing (Sec. 4.3): window-based greedy selection of the retained sequences into
// rows of `capacity` tokens. The algorithm is sequential by definition (each placement
// changes the remaining space and refills the pool), so it runs in ONE wavefront: the pool
// is the set of not-yet-placed items among the first `next` stream items, 64 of them are
// examined per step (one per lane), a ballot finds the oldest item that fits (first-fit
// reading) or a wave-wide max finds the longest one (best-fit reading), and the
// wave-uniform state (remaining space, pool end, output position) lives in scalars.
// Integer work only; the result is a bit-exact function of the inputs.
#include "dppo_internal.h"

namespace dppo {
namespace {

constexpr int WAVE = 64;

__device__ __forceinline__ int64_t wave_sum64(int64_t v) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, WAVE);
    return v;
}

__device__ __forceinline__ int64_t wave_max64(int64_t v) {
    for (int off = 32; off > 0; off >>= 1) {
        int64_t o = __shfl_xor(v, off, WAVE);
        v = o > v ? o : v;
    }
    return v;
}

__global__ __launch_bounds__(WAVE) void pack_kernel(
    int n_items, int capacity, int n_win, int policy, const int32_t* __restrict__ prompt_len,
    const int32_t* __restrict__ comp_len, const uint8_t* __restrict__ keep, int32_t* order,
    int32_t* row_ptr, int32_t* cu /* scratch: stream item length, -1 once placed */,
    int32_t* lcu /* scratch: stream item -> original index */, int64_t loss_pos_capacity, int32_t* meta) {
    const int lane = threadIdx.x;
    const uint64_t lanes_below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));

    // ---- compact the kept items into the stream, validate, total T and N -------------
    int S = 0;
    int bad = 0;
    int64_t T = 0, N = 0, longest = 1;
    const int min_c = comp_len != nullptr ? 1 : 0;   // prompts alone: no completion part
    for (int j0 = 0; j0 < n_items; j0 += WAVE) {
        int j = j0 + lane;
        bool kept = j < n_items && (keep == nullptr || keep[j] != 0);
        int P = kept ? prompt_len[j] : 1;
        int C = (kept && comp_len != nullptr) ? comp_len[j] : min_c;
        int64_t len = (int64_t)P + (int64_t)C;
        if (kept && (P < 1 || C < min_c || len > 0x7fffffffLL)) bad = 1;
        if (kept && len > longest) longest = len;
        uint64_t m = __ballot(kept);
        if (kept) {
            int pos = S + __popcll(m & lanes_below);
            cu[pos] = (int32_t)(len > 0x7fffffffLL ? 0x7fffffff : len);
            lcu[pos] = j;
        }
        S += __popcll(m);
        T += wave_sum64(kept ? len : 0);
        N += wave_sum64(kept ? (int64_t)C : 0);
    }
    longest = wave_max64(longest);
    if (capacity == 0) capacity = (int)(longest > 0x7fffffffLL ? 0x7fffffff : longest);   // L_max = longest item
    int status = 0;
    if (__any(bad) || longest > (int64_t)capacity) status = 1;
    else if (N > loss_pos_capacity) status = 2;
    else if (T > 0x7fffffffLL) status = 3;
    if (status != 0) {
        if (lane == 0) {
            meta[0] = 0; meta[1] = 0; meta[2] = 0; meta[3] = status;
            meta[4] = 0; meta[5] = capacity; meta[6] = 0; meta[7] = 0;
            row_ptr[0] = 0; cu[0] = 0; lcu[0] = 0;
        }
        return;
    }
    __syncthreads();   // stream arrays written above are read by other lanes below

    // ---- window-based greedy placement -------------------------------------------------
    int next = n_win < S ? n_win : S;   // pool = unplaced stream items with index < next
    int lo = 0;                         // every stream item below lo is placed
    int pos = 0;                        // sequences placed so far
    int rows = 0;
    if (lane == 0) row_ptr[0] = 0;
    while (pos < S) {
        int rem = capacity;
        if (policy == DPPO_PACK_BEST_FIT) {
            // longest pool item that fits, oldest among equals; repeat until none fits
            while (true) {
                int64_t best = -1;
                for (int i0 = lo; i0 < next; i0 += WAVE) {
                    int i = i0 + lane;
                    int len = (i < next) ? ((volatile const int32_t*)cu)[i] : -1;
                    if (len > 0 && len <= rem) {
                        int64_t key = ((int64_t)len << 32) | (int64_t)(0x7fffffff - i);
                        best = key > best ? key : best;
                    }
                }
                best = wave_max64(best);
                if (best < 0) break;
                const int sel = 0x7fffffff - (int)(best & 0xffffffffLL);
                if (lane == 0) {
                    order[pos] = lcu[sel];
                    cu[sel] = -1;
                }
                __syncthreads();   // the mark must be visible to the next scan
                rem -= (int)(best >> 32);
                pos += 1;
                if (next < S) next += 1;
            }
        } else
        for (int i0 = lo; i0 < next; i0 += WAVE) {
            int i = i0 + lane;
            int len = (i < S) ? ((volatile const int32_t*)cu)[i] : -1;   // -1: placed or past the end
            int orig = (i < S) ? lcu[i] : 0;
            uint64_t done = 0;                        // lanes already passed by the scan
            while (true) {
                bool fits = len > 0 && len <= rem && i < next;
                uint64_t m = __ballot(fits) & ~done;
                if (m == 0) break;
                int f = __ffsll((unsigned long long)m) - 1;
                int lf = __shfl(len, f, WAVE);
                if (lane == f) {
                    order[pos] = orig;
                    cu[i] = -1;
                    len = -1;
                }
                rem -= lf;
                pos += 1;
                if (next < S) next += 1;             // refill the pool from the stream
                done = (f == 63) ? ~0ull : ((1ull << (f + 1)) - 1ull);
            }
        }
        rows += 1;
        if (lane == 0) row_ptr[rows] = pos;
        __syncthreads();   // placed marks must be visible to the reloads below
        // advance lo past the placed prefix
        while (lo < S) {
            int i = lo + lane;
            bool unplaced = (i < S) && ((volatile const int32_t*)cu)[i] > 0;
            uint64_t m = __ballot(unplaced);
            if (m != 0) { lo += __ffsll((unsigned long long)m) - 1; break; }
            lo += WAVE;
        }
        if (lo > S) lo = S;
    }
    __syncthreads();

    // ---- offsets of the packed sequences ---------------------------------------------
    int64_t tok = 0, ltok = 0;
    if (lane == 0) { cu[0] = 0; lcu[0] = 0; }
    for (int s0 = 0; s0 < S; s0 += WAVE) {
        int s = s0 + lane;
        int j = (s < S) ? order[s] : 0;
        int P = (s < S) ? prompt_len[j] : 0;
        int C = (s < S && comp_len != nullptr) ? comp_len[j] : 0;
        int64_t a = (int64_t)P + C, b = C;
        for (int off = 1; off < WAVE; off <<= 1) {   // inclusive scan over the wave
            int64_t ta = __shfl_up(a, off, WAVE), tb = __shfl_up(b, off, WAVE);
            if (lane >= off) { a += ta; b += tb; }
        }
        if (s < S) {
            cu[s + 1] = (int32_t)(tok + a);
            lcu[s + 1] = (int32_t)(ltok + b);
        }
        tok += __shfl(a, WAVE - 1, WAVE);
        ltok += __shfl(b, WAVE - 1, WAVE);
    }
    if (lane == 0) {
        meta[0] = rows; meta[1] = (int32_t)T; meta[2] = (int32_t)N; meta[3] = 0;
        meta[4] = S; meta[5] = capacity;
        // fill density T / (rows * capacity) as the two halves of a double (low word first)
        const double dens = rows > 0 ? (double)T / ((double)rows * (double)capacity) : 0.0;
        const uint64_t bits = (uint64_t)__double_as_longlong(dens);
        meta[6] = (int32_t)(uint32_t)(bits & 0xffffffffull); meta[7] = (int32_t)(uint32_t)(bits >> 32);
    }
}

// loss_pos of every packed sequence: one workgroup per sequence (grid-strided).
__global__ void loss_pos_kernel(const int32_t* __restrict__ meta, const int32_t* __restrict__ order,
                                const int32_t* __restrict__ prompt_len, const int32_t* __restrict__ cu,
                                const int32_t* __restrict__ lcu, int32_t* __restrict__ loss_pos) {
    const int S = meta[4];
    for (int s = blockIdx.x; s < S; s += gridDim.x) {
        const int P = prompt_len[order[s]];
        const int first = cu[s] + P - 1;
        const int a = lcu[s], b = lcu[s + 1];
        for (int t = a + threadIdx.x; t < b; t += blockDim.x) loss_pos[t] = first + (t - a);
    }
}

__global__ void gather_f32_kernel(int64_t n, const int32_t* __restrict__ idx, const float* __restrict__ src,
                                  float* __restrict__ dst) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[idx[i]];
}

}  // namespace

void launch_pack(const dppo_pack_params& p, const int32_t* prompt_len, const int32_t* comp_len,
                 const uint8_t* keep, int32_t* order, int32_t* row_ptr, int32_t* cu, int32_t* lcu,
                 int32_t* loss_pos, int64_t loss_pos_capacity, int32_t* meta, hipStream_t st) {
    pack_kernel<<<1, WAVE, 0, st>>>(p.n_items, p.capacity, p.n_win, p.policy, prompt_len, comp_len, keep, order,
                                    row_ptr, cu, lcu, loss_pos_capacity, meta);
    if (comp_len == nullptr) return;   // prompts alone: no loss positions
    int blocks = p.n_items < 2048 ? p.n_items : 2048;
    loss_pos_kernel<<<blocks, 256, 0, st>>>(meta, order, prompt_len, cu, lcu, loss_pos);
}

void launch_gather_f32(int64_t n, const int32_t* idx, const float* src, float* dst, hipStream_t st) {
    if (n <= 0) return;
    gather_f32_kernel<<<(unsigned)ceil_div(n, 256), 256, 0, st>>>(n, idx, src, dst);
}

}  // namespace dppo
