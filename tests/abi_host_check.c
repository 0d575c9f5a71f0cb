/* Host-side check of the C ABI, meant to be built with the host sanitizers (address, undefined) and
 * run without a GPU: it includes the header as plain C, drives every entry point through its
 * argument validation with real (small, host) arrays behind every pointer, and sweeps the workspace
 * arithmetic over ordinary and extreme shapes. No call here may reach a kernel with valid
 * arguments AND a device: where the arguments are valid the call is expected to stop at the first
 * device query (DPPO_ERR_DEVICE) on a host without a GPU, or to succeed on one that has it.
 * Exit status 0 and "abi_host_check: ok" on stdout mean every expectation held; the sanitizers
 * report on stderr and abort by themselves. */
#include "dppo.h"

#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static int failures = 0;

static void expect(int got, int want, const char* what) {
    if (got != want) {
        fprintf(stderr, "abi_host_check: %s: status %d (%s), expected %d; last error: %s\n", what, got,
                dppo_status_str(got), want, dppo_last_error());
        ++failures;
    }
}

/* valid arguments: either the device query fails (no GPU) or the call goes through */
static void expect_ok_or_device(int got, const char* what) {
    if (got != DPPO_OK && got != DPPO_ERR_DEVICE) expect(got, DPPO_OK, what);
}

int main(void) {
    enum { NBUF = 4096 };
    float* f = (float*)calloc(NBUF, sizeof(float));
    int32_t* i32 = (int32_t*)calloc(NBUF, sizeof(int32_t));
    uint8_t* u8 = (uint8_t*)calloc(NBUF, 1);
    double* f64 = (double*)calloc(NBUF, sizeof(double));
    void* ws = aligned_alloc(256, 1 << 20);   /* C11 */
    if (!f || !i32 || !u8 || !f64 || !ws) return 2;

    /* status strings for every code and a few that are not codes */
    for (int code = -2; code < 12; ++code)
        if (!dppo_status_str(code) || !strlen(dppo_status_str(code))) { fprintf(stderr, "empty status string %d\n", code); ++failures; }
    if (!dppo_last_error()) ++failures;

    /* ---- dppo_select ---- */
    dppo_select_params sp = {4, 4, 0.5f, 0.5f, 1e-6f, 1, 0.5f, 0, 1};
    dppo_select_params bad = sp;
    expect(dppo_select(NULL, f, f, f, f, f, f, u8, u8, f, f, f, i32, f, f, NULL), DPPO_ERR_INVALID_ARG, "select: NULL params");
    expect(dppo_select(&sp, NULL, f, f, f, f, f, u8, u8, f, f, f, i32, f, f, NULL), DPPO_ERR_INVALID_ARG, "select: NULL rewards");
    bad = sp; bad.r_q = 1.0f;
    expect(dppo_select(&bad, f, f, f, f, f, f, u8, u8, f, f, f, i32, f, f, NULL), DPPO_ERR_INVALID_ARG, "select: r_q = 1");
    bad = sp; bad.r_o = -0.1f;
    expect(dppo_select(&bad, f, f, f, f, f, f, u8, u8, f, f, f, i32, f, f, NULL), DPPO_ERR_INVALID_ARG, "select: r_o < 0");
    bad = sp; bad.G = 1;
    expect(dppo_select(&bad, f, f, f, f, f, f, u8, u8, f, f, f, i32, f, f, NULL), DPPO_ERR_SHAPE, "select: G - ddof < 1");
    bad = sp; bad.Q = 0;
    expect(dppo_select(&bad, f, f, f, f, f, f, u8, u8, f, f, f, i32, f, f, NULL), DPPO_ERR_SHAPE, "select: Q = 0");
    bad = sp; bad.Q = 1 << 20;
    expect(dppo_select(&bad, f, f, f, f, f, f, u8, u8, f, f, f, i32, f, f, NULL), DPPO_ERR_UNSUPPORTED, "select: Q too large");
    bad = sp; bad.adv_eps = 0.0f;
    expect(dppo_select(&bad, f, f, f, f, f, f, u8, u8, f, f, f, i32, f, f, NULL), DPPO_ERR_INVALID_ARG, "select: adv_eps = 0");
    bad = sp; bad.bottom_frac = 1.5f;
    expect(dppo_select(&bad, f, f, f, f, f, f, u8, u8, f, f, f, i32, f, f, NULL), DPPO_ERR_INVALID_ARG, "select: bottom_frac > 1");
    bad = sp; bad.std_ddof = 2;
    expect(dppo_select(&bad, f, f, f, f, f, f, u8, u8, f, f, f, i32, f, f, NULL), DPPO_ERR_INVALID_ARG, "select: ddof = 2");

    /* ---- dppo_history_update, dppo_token_norm_coef, dppo_variance_terms, dppo_gather_f32 ---- */
    expect(dppo_history_update(-1, i32, u8, f, f, 10, NULL), DPPO_ERR_SHAPE, "history_update: n < 0");
    expect(dppo_history_update(0, NULL, NULL, NULL, NULL, 0, NULL), DPPO_OK, "history_update: n = 0");
    expect(dppo_history_update(4, NULL, u8, f, f, 10, NULL), DPPO_ERR_INVALID_ARG, "history_update: NULL index");
    expect(dppo_token_norm_coef(0, 4, i32, f, f, NULL), DPPO_ERR_SHAPE, "token_norm_coef: Q = 0");
    expect(dppo_variance_terms(4, 0, f, f, f, f64, f64, NULL), DPPO_ERR_SHAPE, "variance_terms: G = 0");
    expect(dppo_variance_terms(4, 4, f, NULL, f, f64, f64, NULL), DPPO_ERR_INVALID_ARG, "variance_terms: NULL prune_q");

    /* ---- dppo_pack ---- */
    dppo_pack_params pp = {4, 16, 4, 0};
    dppo_pack_params pbad = pp;
    pbad.n_items = 0;
    expect(dppo_pack(&pbad, i32, i32, u8, i32, i32, i32, i32, i32, 10, i32, NULL), DPPO_ERR_SHAPE, "pack: no items");
    pbad = pp; pbad.n_win = 0;
    expect(dppo_pack(&pbad, i32, i32, u8, i32, i32, i32, i32, i32, 10, i32, NULL), DPPO_ERR_INVALID_ARG, "pack: window 0");
    pbad = pp; pbad.policy = 7;
    expect(dppo_pack(&pbad, i32, i32, u8, i32, i32, i32, i32, i32, 10, i32, NULL), DPPO_ERR_INVALID_ARG, "pack: unknown policy");
    pbad = pp; pbad.capacity = 1;
    expect(dppo_pack(&pbad, i32, i32, u8, i32, i32, i32, i32, i32, 10, i32, NULL), DPPO_ERR_CAPACITY, "pack: capacity 1");
    expect(dppo_pack(NULL, i32, i32, u8, i32, i32, i32, i32, i32, 10, i32, NULL), DPPO_ERR_INVALID_ARG, "pack: NULL params");

    /* ---- workspace arithmetic over a grid of shapes (the sanitizer watches the integer work) ---- */
    const int64_t Ts[] = {0, 1, 255, 256, 257, 100000, 370000, 5000000, 0x7fffffffLL};
    const int32_t Ds[] = {64, 1024, 2560, 4096, 8192, 65536};
    const int32_t Vs[] = {1, 255, 256, 32000, 151936, 1 << 20, 0x7fffff00};
    for (unsigned a = 0; a < sizeof Ts / sizeof *Ts; ++a)
        for (unsigned b = 0; b < sizeof Ds / sizeof *Ds; ++b)
            for (unsigned c = 0; c < sizeof Vs / sizeof *Vs; ++c)
                for (int dtype = 0; dtype < 2; ++dtype) {
                    dppo_head_shape s = {Ts[a], Ts[a] - Ts[a] / 5, Ds[b], Vs[c], dtype};
                    size_t prev = 0;
                    for (int bw = 0; bw < 3; ++bw) {
                        const size_t rec = dppo_workspace_bytes(&s, bw), mn = dppo_workspace_min_bytes(&s, bw);
                        if (rec == 0 || mn == 0 || mn > rec || rec < prev) {
                            fprintf(stderr, "workspace sizes T=%lld D=%d V=%d dtype=%d bw=%d: rec %zu min %zu prev %zu\n",
                                    (long long)Ts[a], Ds[b], Vs[c], dtype, bw, rec, mn, prev);
                            ++failures;
                        }
                        prev = rec;
                    }
                }
    dppo_head_shape hs = {100, 50, 72, 1000, 1};
    if (dppo_workspace_bytes(&hs, 1) != 0 || dppo_workspace_bytes(NULL, 1) != 0) { fprintf(stderr, "invalid shape got a size\n"); ++failures; }
    if (dppo_static_scratch_bytes() != ((size_t)DPPO_STATIC_SCRATCH_MIB << 20)) ++failures;

    /* ---- dppo_token_logprob and its variant on the fixed scratch ---- */
    expect(dppo_token_logprob(&hs, f, f, i32, i32, f, f, i32, ws, 1 << 20, NULL), DPPO_ERR_UNSUPPORTED, "token_logprob: D % 64");
    expect(dppo_token_logprob_noalloc(&hs, f, f, i32, i32, f, f, i32, NULL), DPPO_ERR_UNSUPPORTED, "token_logprob_noalloc: D % 64");
    hs.D = 64; hs.N = 200;
    expect(dppo_token_logprob(&hs, f, f, i32, i32, f, f, i32, ws, 1 << 20, NULL), DPPO_ERR_SHAPE, "token_logprob: N > T");
    hs.N = 0;
    expect(dppo_token_logprob(&hs, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL), DPPO_OK, "token_logprob: N = 0");
    hs.N = 50;
    expect(dppo_token_logprob(&hs, NULL, f, i32, i32, f, f, i32, ws, 1 << 20, NULL), DPPO_ERR_INVALID_ARG, "token_logprob: NULL H");
    expect(dppo_token_logprob(&hs, f, f, i32, i32, f, f, i32, NULL, 1 << 20, NULL), DPPO_ERR_WORKSPACE, "token_logprob: NULL workspace");
    expect(dppo_token_logprob(&hs, f, f, i32, i32, f, f, i32, (char*)ws + 16, 1 << 19, NULL), DPPO_ERR_WORKSPACE, "token_logprob: misaligned workspace");
    expect(dppo_token_logprob(&hs, f, f, i32, i32, f, f, i32, ws, 1024, NULL), DPPO_ERR_WORKSPACE, "token_logprob: tiny workspace");
    expect(dppo_token_logprob(&hs, (char*)f + 4, f, i32, i32, f, f, i32, ws, 1 << 20, NULL), DPPO_ERR_INVALID_ARG, "token_logprob: misaligned H");
    dppo_head_shape big = {4096, 4096, 128 * 1024, 151936, 1};
    expect(dppo_token_logprob_noalloc(&big, f, f, i32, i32, f, f, i32, NULL), DPPO_ERR_WORKSPACE, "token_logprob_noalloc: too large");
    expect(dppo_token_logprob_noalloc(NULL, f, f, i32, i32, f, f, i32, NULL), DPPO_ERR_INVALID_ARG, "token_logprob_noalloc: NULL shape");

    /* ---- dppo_loss_fwd_bwd ---- */
    dppo_loss_params lp = {0.2f, 0.2f, 0.04f, 0, 0, DPPO_RATIO_TOKEN, DPPO_AGG_SEQ_MEAN, 0};
    dppo_loss_params lbad = lp;
#define LOSS(shape, params, S, wsp, wsb) \
    dppo_loss_fwd_bwd(shape, params, S, f, f, i32, i32, i32, f, f, f, f, f, f, f, f, i32, f, f, wsp, wsb, NULL)
    expect(LOSS(&hs, NULL, 3, ws, 1 << 20), DPPO_ERR_INVALID_ARG, "loss: NULL params");
    lbad = lp; lbad.clip_lo = 1.0f;
    expect(LOSS(&hs, &lbad, 3, ws, 1 << 20), DPPO_ERR_INVALID_ARG, "loss: clip_lo = 1");
    lbad = lp; lbad.beta = -1.0f;
    expect(LOSS(&hs, &lbad, 3, ws, 1 << 20), DPPO_ERR_INVALID_ARG, "loss: beta < 0");
    lbad = lp; lbad.ratio_level = 2;
    expect(LOSS(&hs, &lbad, 3, ws, 1 << 20), DPPO_ERR_INVALID_ARG, "loss: unknown ratio level");
    lbad = lp; lbad.aggregation = -1;
    expect(LOSS(&hs, &lbad, 3, ws, 1 << 20), DPPO_ERR_INVALID_ARG, "loss: unknown aggregation");
    expect(LOSS(&hs, &lp, 0, ws, 1 << 20), DPPO_ERR_SHAPE, "loss: S = 0 with N > 0");
    expect(LOSS(&hs, &lp, 51, ws, 1 << 20), DPPO_ERR_SHAPE, "loss: S > N");
    expect(LOSS(&hs, &lp, 3, ws, 1024), DPPO_ERR_WORKSPACE, "loss: tiny workspace");
    expect(LOSS(&hs, &lp, 3, NULL, 1 << 20), DPPO_ERR_WORKSPACE, "loss: NULL workspace");
    dppo_head_shape hs32 = {100, 50, 64, 1000, 0};
    lbad = lp; lbad.recompute_logits = 1;
    expect(LOSS(&hs32, &lbad, 3, ws, 1 << 20), DPPO_ERR_UNSUPPORTED, "loss: recompute on float32");
    lbad = lp; lbad.ratio_level = DPPO_RATIO_SEQUENCE; lbad.max_seq_tokens = 1 << 30;
    expect(LOSS(&hs, &lbad, 3, ws, 1024), DPPO_ERR_WORKSPACE, "loss: sequence level, tiny workspace");

    /* ---- timing and probes: valid calls that need a device ---- */
    expect(dppo_timing_enable(0), DPPO_OK, "timing_enable(0)");
    {
        double ms[DPPO_N_STAGES];
        int64_t cnt[DPPO_N_STAGES];
        expect(dppo_timing_read(ms, cnt, 1), DPPO_OK, "timing_read with nothing recorded");
        expect(dppo_timing_read(NULL, cnt, 1), DPPO_ERR_INVALID_ARG, "timing_read: NULL");
    }
    expect(dppo_timing_tile_phases(NULL), DPPO_OK, "tile_phases off");
    {
        double flop = 0.0;
        expect(dppo_mfma_rate_probe(0, 0, f, 1024, &flop, NULL), DPPO_ERR_INVALID_ARG, "mfma_rate_probe: iters = 0");
        expect(dppo_mfma_rate_probe(0, 10, NULL, 1024, &flop, NULL), DPPO_ERR_INVALID_ARG, "mfma_rate_probe: NULL out");
    }
    /* valid arguments with host pointers would be a fault on a GPU: only try them where there is none */
    {
        const char* no_gpu = getenv("DPPO_ABI_CHECK_NO_GPU");
        if (no_gpu && no_gpu[0] == '1') {
            expect(dppo_select(&sp, f, f, f, f, f, f, u8, u8, f, f, f, i32, f, f, NULL), DPPO_ERR_DEVICE, "select without a device");
            expect(dppo_token_logprob(&hs, f, f, i32, i32, f, f, i32, ws, 1 << 20, NULL), DPPO_ERR_DEVICE, "token_logprob without a device");
            const size_t need = dppo_workspace_bytes(&hs, 1);
            void* ws_loss = aligned_alloc(256, (need + 255) / 256 * 256);
            if (!ws_loss) return 2;
            expect(LOSS(&hs, &lp, 3, ws_loss, need), DPPO_ERR_DEVICE, "loss without a device");
            free(ws_loss);
            expect_ok_or_device(dppo_token_logprob_noalloc(&hs, f, f, i32, i32, f, f, i32, NULL), "token_logprob_noalloc without a device");
        }
    }

    free(f); free(i32); free(u8); free(f64); free(ws);
    if (failures) { fprintf(stderr, "abi_host_check: %d expectation(s) failed\n", failures); return 1; }
    printf("abi_host_check: ok\n");
    return 0;
}
