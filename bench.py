#!/usr/bin/env python3
"""Benchmark of the DPPO policy-loss hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch that is already resident in
HBM: dppo_select -> dppo_pack -> dppo_gather_f32 (adv, coef) -> dppo_loss_fwd_bwd (fused
LM-head log-probs, reweighted surrogate + KL, dH and dW). Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload qwen3_4b] [--vendor-gemm]

What the line holds besides the contract fields:
  ms_per_step / value            wall time of K whole steps (host clock, synchronised on both sides);
  loss_fwd_bwd_ms                HIP-event time of the dppo_loss_fwd_bwd call alone, per step: median, min, max;
  stage_ms_per_step              HIP-event time of the GEMM stages and of all other kernels inside that call;
  stages                         dppo_select, dppo_pack, dppo_gather_f32, dppo_token_logprob and the
                                 elementwise kernels timed on their own, with algorithmic bytes and GB/s;
  roofline                       the slowest GEMM stage against the bf16 MFMA peak, and against the rate a
                                 register-only loop of the same MFMA sustains in this run (achievable);
  tile_phases                    shader cycles the GEMM workgroups spend before their first slice is in LDS, in the
                                 main loop and in the epilogue, against the cycles their MFMAs alone need;
  cpu_baseline                   the NumPy oracle on a bounded sample, on all host cores and on one.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E peak
# L2 <-> fabric bytes per launch, NOT measured by this run: taken from the FETCH_SIZE / WRITE_SIZE counter
# runs summarised in profiles/bench_qwen3_4b_hbm_traffic.txt (fetch scaled by the factor a plain copy
# gives). Keyed by (workload, kernel, recompute); an entry is deleted when that kernel changes, until
# the counters are taken again.
MEASURED_TRAFFIC_BYTES = {
    ("qwen3_4b", "logits_gemm", False): 2.0 * 19078238 * 1024 + 9734993 * 1024,
    ("qwen3_4b", "dh_gemm", False): 2.0 * 21319216 * 1024 + 161247 * 1024,
    ("qwen3_4b", "dw_gemm", False): 2.0 * 22005603 * 1024 + 1560944 * 1024,   # both dispatches
}


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(rb, H, W, ids_np, n_sample, n_sample_1t, seed):
    """The CPU oracle, as it stands, on the first loss tokens of the same batch: once with the BLAS
    thread pool as the host gives it (n_sample tokens), once limited to one thread (n_sample_1t tokens)."""
    import numpy as np
    import torch
    from threadpoolctl import threadpool_info, threadpool_limits

    import workloads as WL
    from oracle import dppo_oracle as O

    wl = rb.wl
    t0 = time.perf_counter()
    sel = O.select(rb.rewards, rb.hist, rb.u_prompt, rb.u_comp, wl.r_q, wl.r_o)
    pk = O.pack(rb.item_prompt_len, rb.item_comp_len, sel["keep_comp"].reshape(-1), wl.capacity, wl.n_win)
    t_sel_pack = time.perf_counter() - t0          # plain Python loops: one thread whatever the pool says
    W64 = W.to("cpu").to(torch.float64).numpy()

    def leg(n):
        n = min(n, pk["N"])
        S = 0
        while pk["loss_cu"][S] < n:
            S += 1
        loss_cu = pk["loss_cu"][:S + 1].copy()
        loss_cu[S] = n
        loss_pos = pk["loss_pos"][:n]
        T = int(loss_pos[-1]) + 2
        H64 = H[:T].to("cpu").to(torch.float64).numpy()
        adv = sel["adv"].reshape(-1)[pk["order"][:S]]
        coef = sel["coef"].reshape(-1)[pk["order"][:S]]
        base, _ = O.token_logprob(H64, W64, ids_np[:T], loss_pos)
        old = WL.perturb_logp(base, wl.logp_noise, seed, 0)
        ref = WL.perturb_logp(base, wl.logp_noise, seed, 1)
        t0 = time.perf_counter()
        O.loss_fwd_bwd(H64, W64, ids_np[:T], loss_pos, loss_cu, adv, coef, old, ref, wl.clip_eps, wl.clip_eps,
                       wl.kl_beta)
        t_loss = time.perf_counter() - t0
        return n, t_loss, t_loss + t_sel_pack * (n / max(pk["N"], 1))

    pools = threadpool_info()
    threads = max([p.get("num_threads", 1) for p in pools] or [1])
    blas = ", ".join(sorted({"%s %s" % (p.get("internal_api", "?"), p.get("version", "")) for p in pools})) or "none"
    n_all, t_all, tot_all = leg(n_sample)
    with threadpool_limits(limits=1):
        n_one, t_one, tot_one = leg(n_sample_1t)
    return {"value": n_all / tot_all, "unit": "packed tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": "fp64 NumPy oracle: select+pack of the whole batch (%.3f s, one thread, charged pro rata) and "
                      "loss fwd+bwd on the first %d of %d loss tokens at full D and V (%.2f s on %d BLAS threads)"
                      % (t_sel_pack, n_all, pk["N"], t_all, threads),
            "single_thread": {"value": n_one / tot_one, "cores": 1,
                              "sample": "the same on the first %d loss tokens with the BLAS pool limited to one thread "
                                        "(%.2f s)" % (n_one, t_one)},
            "cpu_model": cpu_model(), "host_cpus_visible": os.cpu_count(), "blas": blas}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="qwen3_4b")
    ap.add_argument("--cpu-sample", type=int, default=2048, help="loss tokens the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--cpu-sample-1t", type=int, default=256, help="loss tokens of the single-thread oracle leg")
    ap.add_argument("--recompute", action="store_true", help="recompute the logits in the backward")
    ap.add_argument("--ratio-level", choices=("token", "sequence"), default="token",
                    help="token = Eq. 1 (the benchmark); sequence = the sequence-level ratio variant, with the longest "
                         "sequence promised to the library so that its forward runs one chunk ahead (context only)")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="also time the vendor BLAS (torch.mm) on the three GEMM shapes of one chunk, same value distributions")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (reference point for HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on ONE GPU; --gpus %d is not supported (no sharding, no collectives)"
              % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2603_04135_amd as P
    import workloads as WL

    P.load()          # raises if the HIP library has not been built: there is no fallback
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda:0"
    rb = WL.make_rollout(args.workload)
    wl = rb.wl
    seed = rb.seed
    QG = wl.Q * wl.G

    # ---- inputs resident in HBM before the timed region ---------------------------------
    d = lambda a, dt: torch.as_tensor(a, device=dev).to(dt).contiguous()
    rewards, hist = d(rb.rewards, torch.float32), d(rb.hist, torch.float32)
    u_prompt, u_comp = d(rb.u_prompt, torch.float32), d(rb.u_comp, torch.float32)
    item_pl, item_cl = d(rb.item_prompt_len, torch.int32), d(rb.item_comp_len, torch.int32)
    lp_cap = int(rb.item_comp_len.sum())

    def select_pack():
        sel = P.dppo_select(rewards, hist, u_prompt, u_comp, wl.r_q, wl.r_o, device=dev)
        pk = P.dppo_pack(item_pl, item_cl, sel["keep_comp"].reshape(-1), wl.capacity, wl.n_win,
                         loss_pos_capacity=lp_cap, device=dev)
        return sel, pk

    sel, pk = select_pack()
    assert pk["device_status"] == 0
    T, N, S = pk["T"], pk["N"], pk["S"]
    H = WL.make_hidden(wl, T, seed, dev)
    W = WL.make_vocab_matrix(wl, seed, dev)
    ids_np = WL.make_ids(wl, T, seed)
    ids = torch.as_tensor(ids_np, device=dev)
    dtype_code = 0 if wl.dtype == "f32" else 1
    es = 4 if dtype_code == 0 else 2
    seq_level = args.ratio_level == "sequence"
    max_seq = int(rb.comp_len.max()) if seq_level else 0
    ws = P.alloc_workspace(P.dppo_workspace_bytes(T, N, wl.D, wl.V, dtype_code, 2 if seq_level else 1), dev)
    base, _ = P.dppo_token_logprob(H, W, ids, pk["loss_pos"], want_lse=False, ws=ws)
    base_np = base.cpu().numpy()
    logp_old = torch.as_tensor(WL.perturb_logp(base_np, wl.logp_noise, seed, 0), device=dev)
    logp_ref = torch.as_tensor(WL.perturb_logp(base_np, wl.logp_noise, seed, 1), device=dev)
    dH = torch.empty_like(H)
    dW = torch.empty((wl.V, wl.D), dtype=torch.float32, device=dev)
    f32 = dict(dtype=torch.float32, device=dev)
    outbuf = dict(loss=torch.empty(1, **f32), logp=torch.empty(N, **f32), seq_loss=torch.empty(QG, **f32),
                  stats=torch.empty(4, **f32))
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    loss_events = []

    def step(record=False):
        sel, pk = select_pack()
        seq_adv = P.dppo_gather_f32(pk["order"], sel["adv"])
        seq_coef = P.dppo_gather_f32(pk["order"], sel["coef"])
        if record:
            a, b = ev(), ev()
            a.record()
        out = P.dppo_loss_fwd_bwd(H, W, ids, pk["loss_pos"], pk["loss_cu"], seq_adv, seq_coef, logp_old, logp_ref,
                                  wl.clip_eps, wl.clip_eps, wl.kl_beta, dW=dW, dH=dH, ws=ws, out=outbuf,
                                  recompute_logits=args.recompute, status=status, ratio_level=args.ratio_level,
                                  max_seq_tokens=max_seq)
        if record:
            b.record()
            loss_events.append((a, b))
        return out

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    P.dppo_timing_enable(True)
    P.dppo_timing_read(reset=True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out = step(record=True)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stages = P.dppo_timing_read(reset=True)
    P.dppo_timing_enable(False)
    ms_per_step = dt * 1e3 / args.steps
    loss = float(out["loss"].item())
    if not np.isfinite(loss) or int(status.item()) != 0:
        print("bench.py: non-finite loss or non-zero device status", file=sys.stderr)
        return 1
    call_ms = [a.elapsed_time(b) for a, b in loss_events]

    def timed(fn, reps):
        """Median HIP-event milliseconds of fn() over reps runs on the current stream."""
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            a, b = ev(), ev()
            a.record()
            fn()
            b.record()
            b.synchronize()
            ts.append(a.elapsed_time(b))
        return statistics.median(ts)

    def stage(ms, nbytes, note, flop=None):
        e = {"ms": ms, "bytes": int(nbytes), "GB/s": nbytes / (ms * 1e-3) / 1e9,
             "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "note": note}
        if flop is not None:
            e["TFLOP/s"] = flop / (ms * 1e-3) / 1e12
            e["frac_of_bf16_peak"] = e["TFLOP/s"] / PEAK_BF16_TFLOPS
        return e

    # ---- the other calls of the path, each on its own (HIP events, median of 10) -----------
    Q, G = wl.Q, wl.G
    sel_bytes = QG * (4 + 4) + Q * 8 + QG * (4 + 1 + 4 + 4 + 4) + Q * (4 + 1 + 4 + 4 + 4) + 4
    pack_bytes = QG * 9 + QG * 16 + 2 * S * 4 + N * 4
    gather_bytes = 2 * S * 12
    keep_flat = sel["keep_comp"].reshape(-1)
    other = {
        "dppo_select": stage(timed(lambda: P.dppo_select(rewards, hist, u_prompt, u_comp, wl.r_q, wl.r_o, device=dev), 10),
                             sel_bytes, "3 small kernels, latency-bound (one thread per group)"),
        "dppo_pack": stage(timed(lambda: P.dppo_pack(item_pl, item_cl, keep_flat, wl.capacity, wl.n_win,
                                                     loss_pos_capacity=lp_cap, device=dev), 10),
                           pack_bytes, "one deterministic wavefront + loss_pos fill; the binding's host read-back of "
                                       "the 8-int meta is inside the time"),
        "dppo_gather_f32": stage(timed(lambda: (P.dppo_gather_f32(pk["order"], sel["adv"]),
                                                P.dppo_gather_f32(pk["order"], sel["coef"])), 10),
                                 gather_bytes, "two launches (adv, coef)"),
    }
    if dtype_code == 1:
        t_lp = timed(lambda: P.dppo_token_logprob(H, W, ids, pk["loss_pos"], want_lse=False, ws=ws), 3)
        other["dppo_token_logprob"] = stage(t_lp, N * wl.D * es + wl.V * wl.D * es + N * 12,
                                            "forward only; bound by the vocabulary GEMM, not by HBM",
                                            flop=2.0 * wl.D * wl.V * N)
    n_chunks = max(1.0, stages["logits_gemm"][1] / args.steps / (2.0 if args.recompute else 1.0))
    ew_ms, _ = stages.get("elementwise", (0.0, 0))
    if ew_ms > 0:
        n_tiles = -(-wl.V // 256)
        ew_bytes = (N * wl.D * es * 2          # row gather: read H rows, write the chunk copy
                    + N * wl.D * es * 2        # target logits: chunk rows and W[y] rows
                    + N * n_tiles * 8          # per-tile (max, sum) pairs
                    + N * wl.D * es * 2        # scaled transpose of the chunk copy
                    + 2 * wl.V * wl.D * es     # W -> W^T, once per call
                    + T * wl.D * es            # zero fill of dH
                    + N * 60)                  # per-token vectors
        other["elementwise_in_loss_fwd_bwd"] = stage(ew_ms / args.steps, ew_bytes,
                                                     "all non-GEMM kernels of one dppo_loss_fwd_bwd call (%d chunks), "
                                                     "HIP events around each group of launches" % round(n_chunks))

    # ---- roofline of the dominant kernel (one of the three vocabulary-sized MFMA GEMMs) -----
    gemm_stages = {k: v for k, v in stages.items() if k.endswith("_gemm") and v[1] > 0}
    roofline = None
    if dtype_code == 1 and gemm_stages:
        name = max(gemm_stages, key=lambda k: gemm_stages[k][0])
        ms_tot, launches = gemm_stages[name]
        launches_per_step = launches / args.steps
        passes = 2.0 if (name == "logits_gemm" and args.recompute) else 1.0
        tokens_per_launch = N * passes / launches_per_step
        flop_per_launch = 2.0 * wl.D * wl.V * tokens_per_launch     # 2 D V flop per loss token and GEMM
        avg_ms = ms_tot / launches
        achieved = flop_per_launch / (avg_ms * 1e-3) / 1e12
        traffic = MEASURED_TRAFFIC_BYTES.get((args.workload, name, bool(args.recompute)))
        roofline = {"bound": "mfma", "kernel": name, "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
                    "traffic_source": "profiles/ (rocprofv3 counters of an earlier run of the same kernel), not this run"
                                      if traffic is not None else None,
                    "avg_launch_ms": avg_ms, "launches_per_step": launches_per_step}
        # what the matrix pipes sustain with operands in registers, measured now: the achievable ceiling
        probe_out = torch.empty(1024, **f32)
        rates = {}
        for label, rnd in (("random_operands", True), ("constant_operands", False)):
            P.dppo_mfma_rate_probe(rnd, 2000, probe_out)
            torch.cuda.synchronize()
            a, b = ev(), ev()
            a.record()
            flop = P.dppo_mfma_rate_probe(rnd, 40000, probe_out)
            b.record()
            b.synchronize()
            rates[label] = flop / (a.elapsed_time(b) * 1e-3) / 1e12
        roofline["achievable"] = rates["random_operands"]
        roofline["frac_of_achievable"] = achieved / rates["random_operands"]
        roofline["register_only_mfma_tflops"] = rates
    # ---- where the GEMM workgroups spend their cycles: one more step with the tile-phase counters on ----
    tile_phases = None
    if dtype_code == 1:
        counters = torch.zeros(12, dtype=torch.int64, device=dev)
        P.dppo_timing_tile_phases(counters)
        step()
        torch.cuda.synchronize()
        P.dppo_timing_tile_phases(None)
        c = counters.cpu().tolist()
        Vp = -(-wl.V // 256) * 256
        n_cp = -(-int(round(N / n_chunks)) // 256) * 256
        slices = {"logits_gemm": wl.D / 64.0, "dh_gemm": Vp / 64.0, "dw_gemm": n_cp / 64.0}
        tile_phases = {}
        for i, name in enumerate(("logits_gemm", "dh_gemm", "dw_gemm")):
            pro, loop, epi, n = c[4 * i:4 * i + 4]
            if n == 0:
                continue
            ideal = slices[name] * 2 * 64 * 16      # 2 wavefronts per SIMD x 64 MFMAs per slice x 16 cycles
            tot = (pro + loop + epi) / n
            tile_phases[name] = {"workgroups": n, "cycles_prologue": pro / n, "cycles_main_loop": loop / n,
                                 "cycles_epilogue": epi / n, "mfma_cycles_of_a_tile": ideal,
                                 "main_loop_mfma_share": ideal / (loop / n), "tile_mfma_share": ideal / tot}
    stage_ms = {k: v[0] / args.steps for k, v in stages.items()}
    mfu = 6.0 * wl.D * wl.V * N / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS

    vendor = None
    if args.vendor_gemm and dtype_code == 1:
        # the three GEMMs of one chunk on the vendor BLAS, operands laid out as it likes them ([M,K] x [N,K]^T),
        # values distributed like the path's own (N(0, 0.02) weights, N(0, 1) hidden states, exponentials)
        n_c = int(round(N / n_chunks))
        bf = torch.bfloat16
        Hc = torch.randn((n_c, wl.D), device=dev).to(bf)
        Wm = (torch.randn((wl.V, wl.D), device=dev) * 0.02).to(bf)
        E = torch.exp(torch.randn((n_c, wl.V), device=dev, dtype=bf).float() - 12.0).to(bf)
        WT, HcT, ET = Wm.t().contiguous(), Hc.t().contiguous(), E.t().contiguous()
        shapes = {"logits (W Hc^T)": (Wm, Hc.t()), "dH (E W)": (E, Wm), "dW (E^T Hc)": (E.t(), Hc),
                  # the same two with every operand as a K-contiguous copy (the layout BLAS kernels like best;
                  # the library makes the W^T and Hc^T copies itself but never a transposed copy of the chunk)
                  "dH, W^T copy given": (E, WT.t()), "dW, E^T and Hc^T copies given": (ET, HcT.t())}
        vendor = {}
        for k, (a_, b_) in shapes.items():
            ms = timed(lambda: torch.mm(a_, b_), 5)
            vendor[k] = {"ms": ms, "TFLOP/s": 2.0 * n_c * wl.V * wl.D / (ms * 1e-3) / 1e12}
        del Hc, Wm, E, WT, HcT, ET

    if args.calibrate_copy:
        src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cpu = None
    if args.cpu_sample > 0:
        cpu = cpu_baseline(rb, H, W, ids_np, args.cpu_sample, args.cpu_sample_1t, seed)

    med_call = statistics.median(call_ms)
    line = {
        "metric": "packed tokens/s, fused logprob+GRPO loss fwd+bwd; % bf16 MFMA peak",
        "value": N / (ms_per_step * 1e-3), "unit": "packed tokens/s",
        "value_counts": "loss tokens N (completion tokens of the surviving sequences) per second of the whole step; "
                        "all packed tokens T per second in packed_tokens_T_per_s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": args.workload, "Q": wl.Q, "G": wl.G, "D": wl.D, "V": wl.V,
                   "loss_tokens_N": N, "packed_tokens_T": T, "sequences_S": S,
                   "recompute_logits": bool(args.recompute), "ratio_level": args.ratio_level},
        "mfu_6dv_frac_of_bf16_peak": mfu,
        "packed_tokens_T_per_s": T / (ms_per_step * 1e-3),
        "loss_fwd_bwd_ms": {"median": med_call, "min": min(call_ms), "max": max(call_ms),
                            "loss_tokens_per_s_at_median": N / (med_call * 1e-3),
                            "mfu_6dv_at_median": 6.0 * wl.D * wl.V * N / (med_call * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
        "stage_ms_per_step": stage_ms,
        "stages": other,
        "loss": loss,
        "roofline": roofline,
        "tile_phases": tile_phases,
        "vendor_blas": vendor,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
