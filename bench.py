#!/usr/bin/env python3
"""Benchmark of the DPPO policy-loss hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch that is already resident in
HBM: dppo_select -> dppo_pack -> dppo_gather_f32 (adv, coef) -> dppo_loss_fwd_bwd (fused
LM-head log-probs, reweighted surrogate + KL, dH and dW). Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload qwen3_4b]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA peak
# L2 <-> fabric bytes per launch from the FETCH_SIZE / WRITE_SIZE counter runs summarised in
# profiles/bench_qwen3_4b_hbm_traffic.txt (fetch scaled by the factor a plain copy gives). Keyed by
# (workload, kernel, recompute); an entry is deleted when that kernel changes, until the counters
# are taken again.
MEASURED_TRAFFIC_BYTES = {
    ("qwen3_4b", "logits_gemm", False): 2.0 * 18858430 * 1024 + 9730179 * 1024,
    ("qwen3_4b", "dh_gemm", False): 2.0 * 21368820 * 1024 + 161168 * 1024,
    ("qwen3_4b", "dw_gemm", False): 2.0 * (21963849 + 29430) * 1024 + (1560576 + 12032) * 1024,   # both dispatches + the sum
}


def cpu_baseline(rb, pk_host, sel_host, H, W, ids_np, n_sample, seed):
    """The CPU oracle, as it stands, on the first n_sample loss tokens of the same batch."""
    import numpy as np
    import torch
    import workloads as WL
    from oracle import dppo_oracle as O

    wl = rb.wl
    t0 = time.perf_counter()
    sel = O.select(rb.rewards, rb.hist, rb.u_prompt, rb.u_comp, wl.r_q, wl.r_o)
    pk = O.pack(rb.item_prompt_len, rb.item_comp_len, sel["keep_comp"].reshape(-1), wl.capacity, wl.n_win)
    t_sel_pack = time.perf_counter() - t0
    n = min(n_sample, pk["N"])
    S = 0
    while pk["loss_cu"][S] < n:
        S += 1
    loss_cu = pk["loss_cu"][:S + 1].copy()
    loss_cu[S] = n
    loss_pos = pk["loss_pos"][:n]
    T = int(loss_pos[-1]) + 2
    H64 = H[:T].to("cpu").to(torch.float64).numpy()
    W64 = W.to("cpu").to(torch.float64).numpy()
    adv = sel["adv"].reshape(-1)[pk["order"][:S]]
    coef = sel["coef"].reshape(-1)[pk["order"][:S]]
    t0 = time.perf_counter()
    base, _ = O.token_logprob(H64, W64, ids_np[:T], loss_pos)
    t_logp = time.perf_counter() - t0
    old = WL.perturb_logp(base, wl.logp_noise, seed, 0)
    ref = WL.perturb_logp(base, wl.logp_noise, seed, 1)
    t0 = time.perf_counter()
    O.loss_fwd_bwd(H64, W64, ids_np[:T], loss_pos, loss_cu, adv, coef, old, ref, wl.clip_eps, wl.clip_eps, wl.kl_beta)
    t_loss = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    t_total = t_loss + t_sel_pack * (n / max(pk["N"], 1))
    return {"value": n / t_total, "unit": "packed tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "fp64 NumPy oracle: select+pack of the whole batch (%.3f s, charged pro rata) and "
                      "loss fwd+bwd on the first %d of %d loss tokens at full D and V (%.2f s)"
                      % (t_sel_pack, n, pk["N"], t_loss)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="qwen3_4b")
    ap.add_argument("--cpu-sample", type=int, default=2048, help="loss tokens the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--recompute", action="store_true", help="recompute the logits in the backward")
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
    ws = P.alloc_workspace(P.dppo_workspace_bytes(T, N, wl.D, wl.V, dtype_code, True), dev)
    base, _ = P.dppo_token_logprob(H, W, ids, pk["loss_pos"], want_lse=False, ws=ws)
    base_np = base.cpu().numpy()
    logp_old = torch.as_tensor(WL.perturb_logp(base_np, wl.logp_noise, seed, 0), device=dev)
    logp_ref = torch.as_tensor(WL.perturb_logp(base_np, wl.logp_noise, seed, 1), device=dev)
    dH = torch.empty_like(H)
    dW = torch.empty((wl.V, wl.D), dtype=torch.float32, device=dev)
    f32 = dict(dtype=torch.float32, device=dev)
    outbuf = dict(loss=torch.empty(1, **f32), logp=torch.empty(N, **f32), seq_loss=torch.empty(QG, **f32),
                  stats=torch.empty(4, **f32))

    def step():
        sel, pk = select_pack()
        seq_adv = P.dppo_gather_f32(pk["order"], sel["adv"])
        seq_coef = P.dppo_gather_f32(pk["order"], sel["coef"])
        return P.dppo_loss_fwd_bwd(H, W, ids, pk["loss_pos"], pk["loss_cu"], seq_adv, seq_coef, logp_old, logp_ref,
                                   wl.clip_eps, wl.clip_eps, wl.kl_beta, dW=dW, dH=dH, ws=ws, out=outbuf,
                                   recompute_logits=args.recompute)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    P.dppo_timing_enable(True)
    P.dppo_timing_read(reset=True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out = step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stages = P.dppo_timing_read(reset=True)
    P.dppo_timing_enable(False)
    ms_per_step = dt * 1e3 / args.steps
    loss = float(out["loss"].item())
    if not np.isfinite(loss):
        print("bench.py: non-finite loss", file=sys.stderr)
        return 1

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
                    "avg_launch_ms": avg_ms, "launches_per_step": launches_per_step}
    stage_ms = {k: v[0] / args.steps for k, v in stages.items()}
    mfu = 6.0 * wl.D * wl.V * N / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS

    if args.calibrate_copy:
        src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cpu = None
    if args.cpu_sample > 0:
        cpu = cpu_baseline(rb, pk, sel, H, W, ids_np, args.cpu_sample, seed)

    line = {
        "metric": "packed tokens/s, fused logprob+GRPO loss fwd+bwd; % bf16 MFMA peak",
        "value": N / (ms_per_step * 1e-3), "unit": "packed tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": args.workload, "Q": wl.Q, "G": wl.G, "D": wl.D, "V": wl.V,
                   "loss_tokens_N": N, "packed_tokens_T": T, "sequences_S": S,
                   "recompute_logits": bool(args.recompute)},
        "mfu_6dv_frac_of_bf16_peak": mfu,
        "packed_tokens_T_per_s": T / (ms_per_step * 1e-3),
        "stage_ms_per_step": stage_ms,
        "loss": loss,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
