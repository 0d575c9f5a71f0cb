// C ABI of the DPPO HIP library: argument validation, workspace planning and the
// orchestration of the kernels on the caller's stream. No device memory is allocated here.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "dppo_internal.h"

namespace dppo {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(DPPO_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
    return DPPO_OK;
}

namespace {

// ---- optional stage timing (benchmarks): HIP events around the launches of each stage, on the
// caller's stream; read back with dppo_timing_read ---------------------------------------------
struct TimingState {
    std::mutex mu;
    bool on = false;
    struct Span { int stage; hipEvent_t a, b; };
    std::vector<Span> spans;
    std::vector<hipEvent_t> pool;
    hipEvent_t get() {
        if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
};
TimingState g_timing;

struct StageTimer {
    int stage; hipStream_t st; hipEvent_t a = nullptr, b = nullptr;
    StageTimer(int stage_, hipStream_t st_) : stage(stage_), st(st_) {
        std::lock_guard<std::mutex> lk(g_timing.mu);
        if (!g_timing.on || g_timing.spans.size() >= (1u << 16)) return;
        a = g_timing.get(); b = g_timing.get();
        if (a && b) (void)hipEventRecord(a, st); else a = b = nullptr;
    }
    ~StageTimer() {
        if (!a) return;
        (void)hipEventRecord(b, st);
        std::lock_guard<std::mutex> lk(g_timing.mu);
        g_timing.spans.push_back({stage, a, b});
    }
};

constexpr int32_t CHUNK_ALIGN = 256;      // token-chunk granularity (= GEMM tile edge)
constexpr int32_t CHUNK_MAX = 32768;      // largest token chunk
// The chunk's gathered hidden states [n_cp, D] are the operand that every tile row of the vocabulary GEMM
// (and, transposed, of the dW GEMM) reads again; they must stay resident in the 256 MB Infinity Cache next
// to the W panels streaming through it (a 268 MB chunk, 32768 tokens of D = 4096, runs 7 % slower per token).
constexpr size_t CHUNK_CACHE_BYTES = (size_t)192 << 20;
int32_t chunk_max_for(int32_t D, size_t es) {
    const int64_t fit = (int64_t)(CHUNK_CACHE_BYTES / ((size_t)D * es)) / CHUNK_ALIGN * CHUNK_ALIGN;
    return (int32_t)(fit < CHUNK_ALIGN ? CHUNK_ALIGN : (fit > CHUNK_MAX ? CHUNK_MAX : fit));
}
constexpr size_t REGION_ALIGN = 256;

struct WsPlan {
    int32_t Vp, n_tiles, n_cp;     // padded vocabulary, row tiles of the vocabulary GEMM, chunk rows
    int64_t n_chunks;
    size_t es, zs;                 // element sizes of H/W and of the stored logits / gradient entries
    size_t fixed_bytes, chunk_bytes; // bytes of the per-call regions / of one set of per-chunk regions
    int sets;                      // sets of per-chunk regions (2: the forward of chunk c + 1 runs ahead of the backward of chunk c)
    // region offsets
    size_t o_wt, o_logp, o_ell, o_kl, o_clip, o_seq, o_sratio, o_hc, o_hct, o_part, o_zg, o_gt, o_y, o_rowc, o_zy, o_lse, o_c;
    size_t o_bref, o_mx, o_scale, o_redo_list, o_redo_sum, o_redo_count, o_dwpart;   // bf16 backward only
    size_t total;
};

int32_t round_up32(int64_t x, int32_t a) { return (int32_t)((x + a - 1) / a * a); }

// Lays the workspace out for chunk size n_cp (multiple of CHUNK_ALIGN): the per-call regions, then `sets`
// copies of the per-chunk regions (the offsets are those of set 0; set i lies i * chunk_bytes further on).
void layout(const dppo_head_shape& s, bool bwd, int32_t n_cp, WsPlan& p, int sets = 1) {
    p.es = s.dtype == 1 ? 2 : 4;
    p.zs = p.es;
    p.Vp = round_up32(s.V, mfma_vocab_tile());   // whole vocabulary tiles: the logits epilogue stores unconditionally
    p.n_tiles = s.dtype == 1 ? mfma_logits_row_tiles(s.V) : 0;
    p.n_cp = n_cp;
    const bool need_z = bwd || s.dtype == 0;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, REGION_ALIGN); return o; };
    const size_t N = (size_t)s.N;
    p.o_wt = take(!bwd ? 0 : s.dtype == 1 ? gemm_b_blocked_elems(s.D, p.Vp) * p.es : (size_t)s.D * p.Vp * p.es);
    p.o_logp = take(bwd ? N * 4 : 0);   // log-probs of the batch when the caller wants none back
    p.o_ell = take(bwd ? N * 4 : 0);
    p.o_kl = take(bwd ? N * 4 : 0);
    p.o_clip = take(bwd ? N * 4 : 0);
    p.o_seq = take(bwd ? 3 * N * 4 : 0);
    p.o_sratio = take(bwd ? N * 4 : 0);
    p.o_dwpart = take(bwd && s.dtype == 1 ? mfma_dw_partial_bytes() : 0);
    p.fixed_bytes = off;
    p.o_hc = take((size_t)n_cp * s.D * p.es);
    p.o_hct = take(!bwd ? 0 : s.dtype == 1 ? gemm_b_blocked_elems(s.D, n_cp) * p.es : (size_t)n_cp * s.D * p.es);
    p.o_part = take((size_t)p.n_tiles * n_cp * 8);
    p.o_zg = take(need_z ? (size_t)n_cp * p.Vp * p.zs : 0);
    p.o_gt = take(bwd && s.dtype == 0 ? (size_t)n_cp * p.Vp * p.zs : 0);   // transposed copy: float32 path only
    p.o_y = take((size_t)n_cp * 4);
    p.o_rowc = take((size_t)n_cp * 4);
    p.o_zy = take((size_t)n_cp * 4);
    p.o_lse = take((size_t)n_cp * 4);
    p.o_c = take((size_t)n_cp * 4);
    const size_t per_tok = bwd && s.dtype == 1 ? (size_t)n_cp * 4 : 0;
    p.o_bref = take(per_tok);
    p.o_mx = take(per_tok);
    p.o_scale = take(per_tok);
    p.o_redo_list = take(per_tok);
    p.o_redo_sum = take(per_tok);
    p.o_redo_count = take(per_tok ? 4 : 0);
    p.chunk_bytes = off - p.fixed_bytes;
    p.sets = sets;
    p.total = p.fixed_bytes + (size_t)sets * p.chunk_bytes;
}

// Chunk size for N loss tokens: balanced chunks of at most CHUNK_MAX tokens, their number chosen so
// that the dH GEMM (tiles of 256 tokens x 256 columns, one workgroup per compute unit, so it runs in
// rounds of one tile per compute unit) wastes little of its last round. Cost of a chunk in dH rounds: whole
// rounds, plus the last one (a fraction if it is at most half full, since its tiles are then cut
// along K), plus what every chunk costs regardless of its size (the dW read-modify-write, the
// small kernels, ramps).
constexpr int DEFAULT_CUS = 256;          // MI355X; used where no device is at hand (size queries)
constexpr double CHUNK_OVERHEAD_ROUNDS = 0.35;
int32_t target_chunk(int64_t N, int32_t D, size_t es, int cus) {
    if (N <= 0) return CHUNK_ALIGN;
    const int64_t CHIP_CUS = cus > 0 ? cus : DEFAULT_CUS;
    const int64_t tiles_n = ceil_div(D, 256);
    const int64_t c0 = ceil_div(N, chunk_max_for(D, es));
    double best = 0.0;
    int64_t best_c = c0;
    for (int64_t c = c0; c <= c0 + 6; ++c) {
        const int64_t tiles = ceil_div(ceil_div(N, c), 256) * tiles_n;
        const int64_t full = tiles / CHIP_CUS, tail = tiles % CHIP_CUS;
        double rounds = (double)full;
        if (tail > 0) {
            int64_t parts = 2 * tail <= CHIP_CUS ? CHIP_CUS / tail : 1;
            if (parts > 8) parts = 8;
            rounds += 1.0 / (double)parts;
        }
        const double cost = (double)c * (rounds + CHUNK_OVERHEAD_ROUNDS);
        if (c == c0 || cost < best) { best = cost; best_c = c; }
    }
    return round_up32(ceil_div(N, best_c), CHUNK_ALIGN);
}

int validate_shape(const dppo_head_shape* s) {
    if (!s) return fail(DPPO_ERR_INVALID_ARG, "shape is NULL");
    if (s->dtype != 0 && s->dtype != 1) return fail(DPPO_ERR_UNSUPPORTED, "dtype %d (0 = float32, 1 = bfloat16)", s->dtype);
    if (s->T < 0 || s->N < 0 || s->N > s->T) return fail(DPPO_ERR_SHAPE, "need 0 <= N <= T (T=%lld N=%lld)", (long long)s->T, (long long)s->N);
    if (s->D <= 0 || s->V <= 0) return fail(DPPO_ERR_SHAPE, "need D > 0 and V > 0 (D=%d V=%d)", s->D, s->V);
    if (s->T > 0x7fffffffLL) return fail(DPPO_ERR_UNSUPPORTED, "T above 2^31-1 packed tokens");
    if (s->dtype == 1 && s->D % 64 != 0) return fail(DPPO_ERR_UNSUPPORTED, "bfloat16 path needs D %% 64 == 0 (D=%d)", s->D);
    return DPPO_OK;
}

// Host-checkable part of the workspace test (needs no device): the smallest chunk must fit.
int check_min_workspace(const dppo_head_shape& s, bool bwd, size_t ws_bytes) {
    WsPlan q;
    layout(s, bwd, CHUNK_ALIGN, q);
    if (q.total > ws_bytes)
        return fail(DPPO_ERR_WORKSPACE, "workspace of %zu bytes is below the minimum of %zu", ws_bytes, q.total);
    return DPPO_OK;
}

// Picks the largest chunk that fits `ws_bytes` (at most the balanced target chunk).
int plan_for(const dppo_head_shape& s, bool bwd, size_t ws_bytes, int cus, WsPlan& p, int sets = 1) {
    const int32_t target = target_chunk(s.N, s.D, s.dtype == 1 ? 2 : 4, cus);
    layout(s, bwd, target, p, sets);
    if (p.total > ws_bytes) {
        WsPlan q;
        layout(s, bwd, CHUNK_ALIGN, q, sets);
        if (q.total > ws_bytes) {
            if (sets > 1) return DPPO_ERR_WORKSPACE;   // the caller falls back to one set: no message
            return fail(DPPO_ERR_WORKSPACE, "workspace of %zu bytes is below the minimum of %zu", ws_bytes, q.total);
        }
        int32_t lo = 1, hi = target / CHUNK_ALIGN;   // in units of CHUNK_ALIGN: lo fits, hi does not
        while (hi - lo > 1) {
            const int32_t mid = (lo + hi) / 2;
            layout(s, bwd, mid * CHUNK_ALIGN, q, sets);
            if (q.total <= ws_bytes) lo = mid; else hi = mid;
        }
        layout(s, bwd, lo * CHUNK_ALIGN, p, sets);
    }
    p.n_chunks = s.N > 0 ? ceil_div(s.N, p.n_cp) : 0;
    return DPPO_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct Regions {
    char* base;
    const WsPlan& p;
    template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(base + off); }
};

// Forward statistics of one chunk: Hc, targets, log-probs, lse. `ws` is the base of the set of
// per-chunk regions to use (the workspace itself for set 0); no per-call region is touched. With keep_z the chunk's logits
// stay in the workspace for the backward pass: as float32 logits (float32 path, which also gets
// HcT), or as bf16 exponentials against the per-token reference left in the bref region (bf16 path).
int chunk_forward(const dppo_head_shape& s, const WsPlan& p, char* ws, const void* H, const void* W,
                   const int32_t* ids, const int32_t* loss_pos, ChunkView cv, bool keep_z,
                   float* logp_all, float* lse_all, int32_t* status, hipStream_t st) {
    void* Hc = ws + p.o_hc;
    int32_t* y = reinterpret_cast<int32_t*>(ws + p.o_y);
    float* zy = reinterpret_cast<float*>(ws + p.o_zy);
    float* lse_c = reinterpret_cast<float*>(ws + p.o_lse);
    {
        StageTimer tm(DPPO_STAGE_ELEMENTWISE, st);
        launch_gather_rows(s.dtype, H, ids, loss_pos, s.T, s.D, s.V, cv, Hc, keep_z && s.dtype == 0 ? ws + p.o_hct : nullptr,
                           y, reinterpret_cast<int32_t*>(ws + p.o_rowc), status, st);
    }
    if (s.dtype == 1 && keep_z) {
        float2* part = reinterpret_cast<float2*>(ws + p.o_part);
        float* bref = reinterpret_cast<float*>(ws + p.o_bref);
        float* mx = reinterpret_cast<float*>(ws + p.o_mx);
        int32_t* redo_count = reinterpret_cast<int32_t*>(ws + p.o_redo_count);
        int32_t* redo_list = reinterpret_cast<int32_t*>(ws + p.o_redo_list);
        float* redo_sum = reinterpret_cast<float*>(ws + p.o_redo_sum);
        // reference of the stored exponentials = the target logit: lse - reference = -logp of a
        // token that was sampled from (nearly) this policy, a few units in any sane batch
        {
            StageTimer tm(DPPO_STAGE_ELEMENTWISE, st);
            launch_target_logit(1, Hc, W, y, cv.n_cp, s.D, zy, bref, redo_count, st);
        }
        {
            StageTimer tm(DPPO_STAGE_LOGITS_GEMM, st);
            const int rc = launch_mfma_logits_exp(W, s.V, s.D, Hc, cv.n_cp, part, bref, ws + p.o_zg, p.Vp, p.Vp, st);
            if (rc != DPPO_OK) return rc;
        }
        StageTimer tm(DPPO_STAGE_ELEMENTWISE, st);
        launch_combine_exp(part, p.n_tiles, zy, bref, cv, lse_c, logp_all, mx, redo_count, redo_list, redo_sum, st);
        launch_exp_redo_rows(redo_count, redo_list, redo_sum, Hc, W, s.V, p.Vp, s.D, zy, mx, cv, ws + p.o_zg, p.Vp,
                             bref, lse_c, logp_all, st);
    } else if (s.dtype == 1) {
        float2* part = reinterpret_cast<float2*>(ws + p.o_part);
        {
            StageTimer tm(DPPO_STAGE_LOGITS_GEMM, st);
            launch_mfma_logits(W, s.V, s.D, Hc, cv.n_cp, part, st);
        }
        StageTimer tm(DPPO_STAGE_ELEMENTWISE, st);
        launch_target_logit(1, Hc, W, y, cv.n_cp, s.D, zy, nullptr, nullptr, st);
        launch_combine_logprob(part, p.n_tiles, zy, cv, lse_c, logp_all, lse_all, st);
    } else {
        StoreSpec out{ws + p.o_zg, p.Vp, 0, 0, nullptr, 0};
        launch_gemm_plain_f32(reinterpret_cast<const float*>(Hc), s.D, reinterpret_cast<const float*>(W), s.D,
                              cv.n_cp, s.V, s.D, out, st);
        launch_row_stats_f32(reinterpret_cast<const float*>(ws + p.o_zg), p.Vp, s.V, y, cv, lse_c, logp_all,
                             lse_all, st);
    }
    return DPPO_OK;
}

// ---- scratch of the entry point that allocates nothing ---------------------------------------
// A device array of fixed size takes the place of the caller's workspace. In host code the
// array's name is only a stand-in for the symbol: the device address is looked up once per
// device (each device holds its own copy at its own address) and only that pointer is ever
// handed to kernels.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)DPPO_STATIC_SCRATCH_MIB << 20;
__device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int MAX_SCRATCH_DEVICES = 64;
void* g_scratch_ptr[MAX_SCRATCH_DEVICES] = {};
std::mutex g_scratch_mu;

// Device address of `scratch` on the current device (looked up on the first call on each device).
int static_scratch(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(DPPO_ERR_DEVICE, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_SCRATCH_DEVICES) return fail(DPPO_ERR_UNSUPPORTED, "device index %d", dev);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(DPPO_ERR_DEVICE, "hipGetSymbolAddress(static scratch) on device %d: %s", dev, hipGetErrorString(e));
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return DPPO_OK;
}

}  // namespace
}  // namespace dppo

using namespace dppo;

extern "C" {

const char* dppo_status_str(int status) {
    switch (status) {
        case DPPO_OK: return "ok";
        case DPPO_ERR_INVALID_ARG: return "invalid argument";
        case DPPO_ERR_SHAPE: return "invalid shape";
        case DPPO_ERR_CAPACITY: return "item exceeds packing capacity";
        case DPPO_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case DPPO_ERR_UNSUPPORTED: return "unsupported shape or dtype";
        case DPPO_ERR_DEVICE: return "HIP runtime error";
        default: return "unknown status";
    }
}

const char* dppo_last_error(void) { return g_err; }

int dppo_select(const dppo_select_params* p, const float* rewards, const float* hist, const float* u_prompt,
                const float* u_comp, float* adv, float* mean_abs_adv, uint8_t* keep_prompt, uint8_t* keep_comp,
                float* gamma_q, float* gamma_o, float* coef, int32_t* counts, float* prune_q, float* prune_o,
                void* stream) {
    if (!p) return fail(DPPO_ERR_INVALID_ARG, "params is NULL");
    if (!rewards || !adv || !mean_abs_adv || !keep_prompt || !keep_comp || !gamma_q || !gamma_o || !coef || !counts)
        return fail(DPPO_ERR_INVALID_ARG, "a required array pointer is NULL");
    if (p->Q <= 0 || p->G <= 0) return fail(DPPO_ERR_SHAPE, "need Q > 0 and G > 0 (Q=%d G=%d)", p->Q, p->G);
    if (p->Q > 16384 || p->G > 1024) return fail(DPPO_ERR_UNSUPPORTED, "Q <= 16384 and G <= 1024 supported (Q=%d G=%d)", p->Q, p->G);
    if (p->std_ddof != 0 && p->std_ddof != 1) return fail(DPPO_ERR_INVALID_ARG, "std_ddof must be 0 or 1");
    if (p->G - p->std_ddof < 1) return fail(DPPO_ERR_SHAPE, "G - std_ddof must be at least 1");
    if (!(p->r_q >= 0.0f && p->r_q < 1.0f) || !(p->r_o >= 0.0f && p->r_o < 1.0f))
        return fail(DPPO_ERR_INVALID_ARG, "prune probabilities must lie in [0,1) (r_q=%g r_o=%g)", p->r_q, p->r_o);
    if (!(p->adv_eps > 0.0f)) return fail(DPPO_ERR_INVALID_ARG, "adv_eps must be > 0 (a constant group has standard deviation 0)");
    if (!(p->bottom_frac >= 0.0f && p->bottom_frac <= 1.0f)) return fail(DPPO_ERR_INVALID_ARG, "bottom_frac must lie in [0,1]");
    if ((p->fixed_count != 0 && p->fixed_count != 1) || (p->realised_rate != 0 && p->realised_rate != 1))
        return fail(DPPO_ERR_INVALID_ARG, "fixed_count and realised_rate must be 0 or 1");
    const int n_bottom = (int)std::floor((double)p->bottom_frac * (double)p->Q);
    launch_select(*p, n_bottom, rewards, hist, u_prompt, u_comp, adv, mean_abs_adv, keep_prompt, keep_comp, gamma_q,
                  gamma_o, coef, counts, prune_q, prune_o, (hipStream_t)stream);
    return check_launch("dppo_select");
}

int dppo_variance_terms(int32_t Q, int32_t G, const float* g, const float* prune_q, const float* prune_o,
                        double* group_out, double* total_out, void* stream) {
    if (Q <= 0 || G <= 0) return fail(DPPO_ERR_SHAPE, "Q and G must be positive (Q=%d G=%d)", Q, G);
    if (!g || !prune_q || !prune_o || !group_out || !total_out)
        return fail(DPPO_ERR_INVALID_ARG, "a required array pointer is NULL");
    launch_variance_terms(Q, G, g, prune_q, prune_o, group_out, total_out, (hipStream_t)stream);
    return check_launch("dppo_variance_terms");
}

int dppo_history_update(int32_t n, const int32_t* prompt_index, const uint8_t* keep_prompt,
                        const float* mean_abs_adv, float* hist_table, int64_t table_size, void* stream) {
    if (n < 0 || table_size < 0) return fail(DPPO_ERR_SHAPE, "n and table_size must be >= 0");
    if (n == 0) return DPPO_OK;
    if (!prompt_index || !keep_prompt || !mean_abs_adv || !hist_table)
        return fail(DPPO_ERR_INVALID_ARG, "a required array pointer is NULL");
    launch_history_update(n, prompt_index, keep_prompt, mean_abs_adv, hist_table, table_size, (hipStream_t)stream);
    return check_launch("dppo_history_update");
}

int dppo_pack(const dppo_pack_params* p, const int32_t* prompt_len, const int32_t* comp_len, const uint8_t* keep,
              int32_t* order, int32_t* row_ptr, int32_t* cu_seqlens, int32_t* loss_cu, int32_t* loss_pos,
              int64_t loss_pos_capacity, int32_t* meta, void* stream) {
    if (!p) return fail(DPPO_ERR_INVALID_ARG, "params is NULL");
    if (!prompt_len || !order || !row_ptr || !cu_seqlens || !loss_cu || !meta)
        return fail(DPPO_ERR_INVALID_ARG, "a required array pointer is NULL");
    if (comp_len && !loss_pos) return fail(DPPO_ERR_INVALID_ARG, "loss_pos is NULL although completions are packed");
    if (p->n_items <= 0) return fail(DPPO_ERR_SHAPE, "n_items must be positive (%d)", p->n_items);
    if (p->capacity < 0 || (p->capacity != 0 && p->capacity < (comp_len ? 2 : 1)))
        return fail(DPPO_ERR_CAPACITY, "capacity must be 0 (longest item) or hold the shortest possible item (%d)",
                    p->capacity);
    if (p->n_win < 1) return fail(DPPO_ERR_INVALID_ARG, "n_win must be at least 1 (%d)", p->n_win);
    if (p->policy != DPPO_PACK_FIRST_FIT && p->policy != DPPO_PACK_BEST_FIT)
        return fail(DPPO_ERR_INVALID_ARG, "unknown packing policy %d", p->policy);
    if (loss_pos_capacity < 0) return fail(DPPO_ERR_SHAPE, "loss_pos_capacity is negative");
    launch_pack(*p, prompt_len, comp_len, keep, order, row_ptr, cu_seqlens, loss_cu, loss_pos, loss_pos_capacity,
                meta, (hipStream_t)stream);
    return check_launch("dppo_pack");
}

int dppo_token_norm_coef(int32_t Q, int32_t G, const int32_t* comp_len, const float* coef, float* coef_out,
                         void* stream) {
    if (Q <= 0 || G <= 0) return fail(DPPO_ERR_SHAPE, "Q and G must be positive (Q=%d G=%d)", Q, G);
    if (!comp_len || !coef || !coef_out) return fail(DPPO_ERR_INVALID_ARG, "a required array pointer is NULL");
    launch_token_norm_coef(Q, G, comp_len, coef, coef_out, (hipStream_t)stream);
    return check_launch("dppo_token_norm_coef");
}

int dppo_gather_f32(int64_t n, const int32_t* idx, const float* src, float* dst, void* stream) {
    if (n < 0) return fail(DPPO_ERR_SHAPE, "n is negative");
    if (n == 0) return DPPO_OK;
    if (!idx || !src || !dst) return fail(DPPO_ERR_INVALID_ARG, "a required array pointer is NULL");
    launch_gather_f32(n, idx, src, dst, (hipStream_t)stream);
    return check_launch("dppo_gather_f32");
}

int dppo_timing_enable(int on) {
    std::lock_guard<std::mutex> lk(g_timing.mu);
    g_timing.on = on != 0;
    return DPPO_OK;
}

int dppo_timing_read(double* ms, int64_t* launches, int reset) {
    if (!ms || !launches) return fail(DPPO_ERR_INVALID_ARG, "ms and launches must not be NULL");
    std::lock_guard<std::mutex> lk(g_timing.mu);
    for (int i = 0; i < DPPO_N_STAGES; ++i) { ms[i] = 0.0; launches[i] = 0; }
    for (const auto& sp : g_timing.spans) {
        float t = 0.0f;
        hipError_t e = hipEventSynchronize(sp.b);
        if (e == hipSuccess) e = hipEventElapsedTime(&t, sp.a, sp.b);
        if (e != hipSuccess) return fail(DPPO_ERR_DEVICE, "stage timing: %s", hipGetErrorString(e));
        if (sp.stage >= 0 && sp.stage < DPPO_N_STAGES) { ms[sp.stage] += (double)t; launches[sp.stage] += 1; }
    }
    if (reset) {
        for (const auto& sp : g_timing.spans) { g_timing.pool.push_back(sp.a); g_timing.pool.push_back(sp.b); }
        g_timing.spans.clear();
    }
    return DPPO_OK;
}

int dppo_timing_tile_phases(uint64_t* counters) {
    mfma_set_phase_counters(reinterpret_cast<unsigned long long*>(counters));
    return DPPO_OK;
}

int dppo_mfma_rate_probe(int random_operands, int iters, float* out, int32_t out_floats, double* flop, void* stream) {
    if (iters <= 0 || !out || !flop) return fail(DPPO_ERR_INVALID_ARG, "iters must be positive, out and flop not NULL");
    int cus = 0;
    const int rc = mfma_setup(&cus);
    if (rc != DPPO_OK) return rc;
    if (out_floats < cus) return fail(DPPO_ERR_SHAPE, "out holds %d floats, the device has %d compute units", out_floats, cus);
    *flop = launch_mfma_rate_probe(cus, iters, random_operands != 0, out, (hipStream_t)stream);
    return check_launch("dppo_mfma_rate_probe");
}

size_t dppo_workspace_bytes(const dppo_head_shape* shape, int want_backward) {
    if (validate_shape(shape) != DPPO_OK) return 0;
    WsPlan p;
    layout(*shape, want_backward != 0, target_chunk(shape->N, shape->D, shape->dtype == 1 ? 2 : 4, DEFAULT_CUS), p,
           want_backward == 2 ? 2 : 1);
    return p.total;
}

size_t dppo_workspace_min_bytes(const dppo_head_shape* shape, int want_backward) {
    if (validate_shape(shape) != DPPO_OK) return 0;
    WsPlan p;
    layout(*shape, want_backward != 0, CHUNK_ALIGN, p, want_backward == 2 ? 2 : 1);
    return p.total;
}

int dppo_token_logprob(const dppo_head_shape* shape, const void* H, const void* W, const int32_t* ids,
                       const int32_t* loss_pos, float* logp, float* lse, int32_t* status, void* ws, size_t ws_bytes,
                       void* stream) {
    int rc = validate_shape(shape);
    if (rc != DPPO_OK) return rc;
    const dppo_head_shape& s = *shape;
    if (s.N == 0) return DPPO_OK;
    if (!H || !W || !ids || !logp) return fail(DPPO_ERR_INVALID_ARG, "a required array pointer is NULL");
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return fail(DPPO_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
    if (s.dtype == 1 && (!aligned16(H) || !aligned16(W))) return fail(DPPO_ERR_INVALID_ARG, "H and W must be 16-byte aligned");
    if ((rc = check_min_workspace(s, false, ws_bytes)) != DPPO_OK) return rc;
    int cus = DEFAULT_CUS;
    if (s.dtype == 1 && (rc = mfma_setup(&cus)) != DPPO_OK) return rc;
    WsPlan p;
    rc = plan_for(s, false, ws_bytes, cus, p);
    if (rc != DPPO_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    char* w = reinterpret_cast<char*>(ws);
    if (status) launch_fill_zero(status, 4, st);
    for (int64_t n0 = 0; n0 < s.N; n0 += p.n_cp) {
        ChunkView cv;
        cv.n0 = n0;
        cv.n_c = (int32_t)((s.N - n0) < p.n_cp ? (s.N - n0) : p.n_cp);
        cv.n_cp = round_up32(cv.n_c, CHUNK_ALIGN);
        if (int rc = chunk_forward(s, p, w, H, W, ids, loss_pos, cv, false, logp, lse, status, st)) return rc;
    }
    return check_launch("dppo_token_logprob");
}

size_t dppo_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

int dppo_token_logprob_noalloc(const dppo_head_shape* shape, const void* H, const void* W, const int32_t* ids,
                               const int32_t* loss_pos, float* logp, float* lse, int32_t* status, void* stream) {
    int rc = validate_shape(shape);
    if (rc != DPPO_OK) return rc;
    // sizes beyond what the fixed scratch can serve are refused before anything else happens
    WsPlan q;
    layout(*shape, false, CHUNK_ALIGN, q);
    if (q.total > STATIC_SCRATCH_BYTES)
        return fail(DPPO_ERR_WORKSPACE,
                    "shape needs at least %zu bytes of scratch (one 256-token chunk of D=%d, V=%d), above the fixed %zu bytes "
                    "of dppo_token_logprob_noalloc; use dppo_token_logprob with a workspace",
                    q.total, shape->D, shape->V, STATIC_SCRATCH_BYTES);
    if (shape->N == 0) return DPPO_OK;
    void* ws = nullptr;
    if ((rc = static_scratch(&ws)) != DPPO_OK) return rc;
    return dppo_token_logprob(shape, H, W, ids, loss_pos, logp, lse, status, ws, STATIC_SCRATCH_BYTES, stream);
}

int dppo_loss_fwd_bwd(const dppo_head_shape* shape, const dppo_loss_params* lp, int32_t S, const void* H,
                      const void* W, const int32_t* ids, const int32_t* loss_pos, const int32_t* loss_cu,
                      const float* seq_adv, const float* seq_coef, const float* logp_old, const float* logp_ref,
                      float* loss, float* logp, float* seq_loss, float* stats, int32_t* status, void* dH, float* dW,
                      void* ws, size_t ws_bytes, void* stream) {
    int rc = validate_shape(shape);
    if (rc != DPPO_OK) return rc;
    const dppo_head_shape& s = *shape;
    if (!lp) return fail(DPPO_ERR_INVALID_ARG, "loss params is NULL");
    if (!(lp->clip_lo >= 0.0f && lp->clip_lo < 1.0f) || !(lp->clip_hi >= 0.0f))
        return fail(DPPO_ERR_INVALID_ARG, "need 0 <= clip_lo < 1 and clip_hi >= 0");
    if (!(lp->beta >= 0.0f)) return fail(DPPO_ERR_INVALID_ARG, "beta must be >= 0");
    if ((lp->ratio_level != DPPO_RATIO_TOKEN && lp->ratio_level != DPPO_RATIO_SEQUENCE) ||
        (lp->aggregation != DPPO_AGG_SEQ_MEAN && lp->aggregation != DPPO_AGG_TOKEN_SUM))
        return fail(DPPO_ERR_INVALID_ARG, "unknown ratio_level %d or aggregation %d", lp->ratio_level, lp->aggregation);
    if (S < 0 || (s.N > 0 && S < 1) || (int64_t)S > s.N) return fail(DPPO_ERR_SHAPE, "need 1 <= S <= N when N > 0 (S=%d N=%lld)", S, (long long)s.N);
    if (!loss || !dH || !dW || !W) return fail(DPPO_ERR_INVALID_ARG, "loss, dH, dW and W must not be NULL");
    if (s.N > 0 && (!H || !ids || !loss_cu || !seq_adv || !seq_coef || !logp_old || !logp_ref))
        return fail(DPPO_ERR_INVALID_ARG, "a required array pointer is NULL");
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return fail(DPPO_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
    if (s.dtype == 1 && (!aligned16(H) || !aligned16(W) || !aligned16(dH) || !aligned16(dW)))
        return fail(DPPO_ERR_INVALID_ARG, "H, W, dH and dW must be 16-byte aligned");
    if (lp->recompute_logits != 0 && s.dtype != 1)
        return fail(DPPO_ERR_UNSUPPORTED, "recompute_logits is a bfloat16-path option");
    if ((rc = check_min_workspace(s, true, ws_bytes)) != DPPO_OK) return rc;
    int cus = DEFAULT_CUS;
    if (s.dtype == 1 && (rc = mfma_setup(&cus)) != DPPO_OK) return rc;
    WsPlan p;
    // Sequence-level ratio: a sequence's ratio needs all its log-probs before any of its gradients.
    // With two sets of per-chunk regions the forward of chunk c + 1 runs ahead of the backward of
    // chunk c, which is enough when no sequence is longer than a chunk (it then ends inside the
    // chunk after the one it starts in). Otherwise: one forward-only pass over every chunk first.
    bool ahead = false;
    if (lp->ratio_level == DPPO_RATIO_SEQUENCE && s.N > 0 && lp->max_seq_tokens > 0) {
        WsPlan p2;
        if (plan_for(s, true, ws_bytes, cus, p2, 2) == DPPO_OK && lp->max_seq_tokens <= p2.n_cp) {
            p = p2;
            ahead = true;
        }
    }
    if (!ahead) {
        rc = plan_for(s, true, ws_bytes, cus, p);
        if (rc != DPPO_OK) return rc;
        // a single chunk holds every sequence whole: its own forward serves
        ahead = lp->ratio_level == DPPO_RATIO_SEQUENCE && p.n_chunks == 1;
    }

    hipStream_t st = (hipStream_t)stream;
    char* w = reinterpret_cast<char*>(ws);
    float* logp_all = logp ? logp : reinterpret_cast<float*>(w + p.o_logp);
    float* ell = reinterpret_cast<float*>(w + p.o_ell);
    float* kl = reinterpret_cast<float*>(w + p.o_kl);
    float* clipf = reinterpret_cast<float*>(w + p.o_clip);
    float* seq_tmp = reinterpret_cast<float*>(w + p.o_seq);

    if (status) launch_fill_zero(status, 4, st);
    {
        StageTimer tm(DPPO_STAGE_ELEMENTWISE, st);
        launch_fill_zero(dH, (size_t)s.T * s.D * p.es, st);
        if (!lp->accumulate_dW && s.N == 0) launch_fill_zero(dW, (size_t)s.V * s.D * 4, st);
        if (s.N > 0) launch_transpose_w(s.dtype, W, s.V, s.D, p.Vp, w + p.o_wt, st);
    }

    const bool recompute = lp->recompute_logits != 0;
    const bool seq_level = lp->ratio_level == DPPO_RATIO_SEQUENCE && s.N > 0;
    float* seq_ratio = reinterpret_cast<float*>(w + p.o_sratio);
    auto view = [&](int64_t c) {
        ChunkView cv;
        cv.n0 = c * p.n_cp;
        cv.n_c = (int32_t)((s.N - cv.n0) < p.n_cp ? (s.N - cv.n0) : p.n_cp);
        cv.n_cp = round_up32(cv.n_c, CHUNK_ALIGN);
        return cv;
    };
    // per-chunk regions of chunk c: set c & 1 when the forward runs ahead, else the only set
    auto regions = [&](int64_t c) { return w + (p.sets == 2 ? (size_t)(c & 1) * p.chunk_bytes : 0); };

    if (seq_level && !ahead) {
        for (int64_t c = 0; c < p.n_chunks; ++c)
            if (int rc2 = chunk_forward(s, p, w, H, W, ids, loss_pos, view(c), false, logp_all, nullptr, status, st)) return rc2;
        launch_seq_ratio(loss_cu, S, logp_all, logp_old, seq_ratio, 0, s.N, nullptr, st);
    }

    // forward of chunk c: statistics and log-probs, and what the backward needs of its logits;
    // with the forward running ahead, also the ratios of the sequences that end in it
    auto forward = [&](int64_t c) -> int {
        const ChunkView cv = view(c);
        if (int rc2 = chunk_forward(s, p, regions(c), H, W, ids, loss_pos, cv, s.dtype == 0 || !recompute, logp_all, nullptr, status, st))
            return rc2;
        if (ahead) launch_seq_ratio(loss_cu, S, logp_all, logp_old, seq_ratio, cv.n0, cv.n0 + cv.n_c, status, st);
        return DPPO_OK;
    };

    auto backward = [&](int64_t c, bool first) -> int {
        const ChunkView cv = view(c);
        char* wc = regions(c);
        TokenLossArgs ta;
        ta.loss_cu = loss_cu; ta.S = S; ta.seq_adv = seq_adv; ta.seq_coef = seq_coef;
        ta.logp_old = logp_old; ta.logp_ref = logp_ref; ta.logp = logp_all;
        ta.lo = (float)(1.0 - (double)lp->clip_lo); ta.hi = (float)(1.0 + (double)lp->clip_hi); ta.beta = lp->beta;
        ta.ratio_level = lp->ratio_level; ta.aggregation = lp->aggregation; ta.seq_ratio = seq_ratio;
        ta.c_chunk = reinterpret_cast<float*>(wc + p.o_c);
        ta.ell = ell; ta.kl = kl; ta.clipped = clipf;
        {
            StageTimer tm(DPPO_STAGE_ELEMENTWISE, st);
            launch_token_loss(ta, cv, st);
        }

        const int32_t* y = reinterpret_cast<const int32_t*>(wc + p.o_y);
        const float* lse_c = reinterpret_cast<const float*>(wc + p.o_lse);
        // bf16: the chunk region holds either gradient entries (recompute) or exponentials whose
        // row scale goes to the dH epilogue and into the HcT operand of dW; in the blocked layout it
        // serves both GEMMs. float32: row-major G and its transposed copy GT.
        void* G = wc + p.o_zg;
        const float* row_scale = nullptr;
        if (s.dtype == 0) {
            StageTimer tm(DPPO_STAGE_GRAD_LOGITS, st);
            launch_grad_logits_f32(reinterpret_cast<float*>(G), reinterpret_cast<float*>(wc + p.o_gt), s.V, p.Vp, y, lse_c,
                                   ta.c_chunk, cv.n_cp, st);
        } else if (recompute) {
            StageTimer tm(DPPO_STAGE_LOGITS_GEMM, st);
            const int rc2 = launch_mfma_logits_grad(W, s.V, s.D, wc + p.o_hc, cv.n_cp, y, lse_c, ta.c_chunk, G, p.Vp,
                                                    p.Vp, st);
            if (rc2 != DPPO_OK) return rc2;
        } else {
            StageTimer tm(DPPO_STAGE_GRAD_LOGITS, st);
            float* scale = reinterpret_cast<float*>(wc + p.o_scale);
            launch_softmax_scale(y, reinterpret_cast<const float*>(wc + p.o_zy), reinterpret_cast<const float*>(wc + p.o_bref),
                                 lse_c, ta.c_chunk, cv, G, p.Vp, scale, st);
            row_scale = scale;
        }
        if (s.dtype == 1) {
            StageTimer tm(DPPO_STAGE_ELEMENTWISE, st);
            launch_scale_transpose_bf16(wc + p.o_hc, row_scale, cv.n_cp, s.D, wc + p.o_hct, st);
        }

        // dH rows of the chunk: diag(row_scale) G[n_c, Vp] * WT[D, Vp]^T, scattered to the loss rows of dH
        StoreSpec oh;
        oh.out_bf16 = s.dtype == 1; oh.accumulate = 0; oh.ldc = s.D;
        // the scatter goes through the chunk's clamped rows, so it stays inside dH whatever loss_pos holds
        if (loss_pos) { oh.C = dH; oh.row_map = reinterpret_cast<const int32_t*>(wc + p.o_rowc); oh.row_base = 0; }
        else { oh.C = reinterpret_cast<char*>(dH) + (size_t)cv.n0 * s.D * p.es; oh.row_map = nullptr; oh.row_base = 0; }
        // dW[v, d] (+)= sum_n G[n, v] HcT[d, n]
        StoreSpec ow;
        ow.C = dW; ow.ldc = s.D; ow.out_bf16 = 0; ow.accumulate = (first && !lp->accumulate_dW) ? 0 : 1;
        ow.row_map = nullptr; ow.row_base = 0;
        if (s.dtype == 1) {
            {
                StageTimer tm(DPPO_STAGE_DH_GEMM, st);
                launch_mfma_dh(cus, G, p.Vp, w + p.o_wt, cv.n_c, s.D, row_scale, oh, reinterpret_cast<float*>(w + p.o_dwpart), st);
            }
            {
                StageTimer tm(DPPO_STAGE_DW_GEMM, st);
                launch_mfma_dw(cus, G, p.Vp, wc + p.o_hct, cv.n_cp, s.V, s.D, ow,
                               reinterpret_cast<float*>(w + p.o_dwpart), st);
            }
        } else {
            launch_gemm_plain_f32(reinterpret_cast<const float*>(G), p.Vp, reinterpret_cast<const float*>(w + p.o_wt),
                                  p.Vp, cv.n_c, s.D, p.Vp, oh, st);
            launch_gemm_plain_f32(reinterpret_cast<const float*>(wc + p.o_gt), cv.n_cp,
                                  reinterpret_cast<const float*>(wc + p.o_hct), cv.n_cp, s.V, s.D, cv.n_cp, ow, st);
        }
        return DPPO_OK;
    };

    if (ahead) {
        if (int rc2 = forward(0)) return rc2;
        for (int64_t c = 0; c < p.n_chunks; ++c) {
            if (c + 1 < p.n_chunks)
                if (int rc2 = forward(c + 1)) return rc2;
            if (int rc2 = backward(c, c == 0)) return rc2;
        }
    } else {
        for (int64_t c = 0; c < p.n_chunks; ++c) {
            if (int rc2 = forward(c)) return rc2;
            if (int rc2 = backward(c, c == 0)) return rc2;
        }
    }

    SeqReduceArgs ra;
    ra.loss_cu = loss_cu; ra.S = s.N > 0 ? S : 0; ra.N = s.N; ra.seq_coef = seq_coef;
    ra.aggregation = lp->aggregation;
    ra.ell = ell; ra.kl = kl; ra.clipped = clipf;
    ra.seq_mean = seq_tmp; ra.seq_kl = seq_tmp + s.N; ra.seq_clip = seq_tmp + 2 * s.N;
    ra.seq_loss_out = seq_loss; ra.loss_out = loss; ra.stats_out = stats;
    {
        StageTimer tm(DPPO_STAGE_ELEMENTWISE, st);
        launch_seq_reduce(ra, st);
    }
    return check_launch("dppo_loss_fwd_bwd");
}

}  // extern "C"
