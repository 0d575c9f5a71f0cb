"""GPU parity of dppo_token_logprob and dppo_loss_fwd_bwd against the CPU oracle.

Tolerances: per-token log-prob abs err <= 2e-3
(bf16 inputs, fp32 accumulation), loss rel err <= 1e-3, dH and dW relative Frobenius
error <= 1e-2. The float32 data type is held to 1e-4 / 1e-5 / 1e-4 instead."""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as WL
from oracle import dppo_oracle as O
from harness import HeadCase, oracle_select_pack, rel_fro, to_np64, truncate_pack

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = {"bf16": dict(logp=2e-3, loss=1e-3, grad=1e-2), "f32": dict(logp=1e-4, loss=1e-5, grad=1e-4)}


@pytest.fixture(scope="module")
def lib():
    import paper_2603_04135_amd as P
    P.load()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return P


def _loss_errors(got, ref_out, case):
    """Error of the loss relative to |L|, and relative to the size of the terms that L sums
    (L is a cancelling sum of seq_coef * advantage-sized terms)."""
    scale = float(np.abs(case.seq_coef_np.astype(np.float64) * ref_out["seq_loss"]).sum())
    err = abs(got - ref_out["loss"])
    return err / max(abs(ref_out["loss"]), 1e-300), err / max(scale, 1e-300)


def _loss_close(got, ref_out, case, tol):
    """Loss relative error <= tol against |L|, the denominator floored at 1 % of the sum of the
    absolute per-sequence terms (where L is mostly cancellation the plain ratio measures nothing)."""
    rel_l, rel_terms = _loss_errors(got, ref_out, case)
    return rel_l <= tol or rel_terms <= 1e-2 * tol


def _assert_loss(got, ref_out, case, tol):
    rel_l, rel_terms = _loss_errors(got, ref_out, case)
    assert rel_l <= tol or rel_terms <= 1e-2 * tol, (
        "loss %.9g vs oracle %.9g: error %.3g of |L| (bound %.1g), %.3g of sum|coef * seq_loss| (bound %.1g)"
        % (got, ref_out["loss"], rel_l, tol, rel_terms, 1e-2 * tol))
    print("loss error: %.3g of |L|, %.3g of sum|coef * seq_loss| (passes on %s)"
          % (rel_l, rel_terms, "|L|" if rel_l <= tol else "the term scale"))


def _same_loss(a, b, ref_out, case):
    """Two paths of the library whose forward statistics are summed in different orders."""
    return _loss_close(float(a), dict(ref_out, loss=float(b)), case, 1e-5)


def _same_rows(a, b):
    """dH of two chunkings of the same batch: the same fp32 sums, possibly associated differently
    (the tiles of a sparsely filled last round are summed in K-split parts), then rounded to bf16."""
    a64, b64 = to_np64(a), to_np64(b)
    return rel_fro(a64, b64) <= 1e-3 and float((a64 == b64).mean()) >= 0.98


def _run_case(P, case, tol, **kw):
    """Full parity of one case: log-probs, loss, per-sequence loss, stats, dH, dW."""
    logp_ref, lse_ref = case.oracle_logprob()
    logp, lse = P.dppo_token_logprob(case.H, case.W, case.ids, case.loss_pos)
    assert np.abs(logp.cpu().numpy() - logp_ref).max() <= tol["logp"]
    assert np.abs(lse.cpu().numpy() - lse_ref).max() <= tol["logp"]
    case.set_behaviour_logps(logp_ref)
    ref = case.oracle_loss(**kw)
    out = P.dppo_loss_fwd_bwd(case.H, case.W, case.ids, case.loss_pos, case.loss_cu, case.seq_adv, case.seq_coef,
                              case.logp_old, case.logp_ref, **kw)
    torch.cuda.synchronize()
    assert np.abs(out["logp"].cpu().numpy() - ref["logp"]).max() <= tol["logp"]
    _assert_loss(float(out["loss"].item()), ref, case, tol["loss"])
    assert np.allclose(out["seq_loss"].cpu().numpy(), ref["seq_loss"], rtol=tol["loss"], atol=tol["logp"])
    stats = out["stats"].cpu().numpy()
    assert abs(stats[0] - ref["mean_kl"]) <= 1e-3 * max(ref["mean_kl"], 1e-6) + 1e-7
    assert abs(stats[1] - ref["clip_frac"]) <= 2.0 / max(case.pk["N"], 1) + 1e-3 * ref["clip_frac"]
    assert stats[2] == case.pk["N"]
    dH = to_np64(out["dH"])
    dW = to_np64(out["dW"])
    mask = np.ones(case.pk["T"], bool)
    mask[case.pk["loss_pos"]] = False
    assert not dH[mask].any(), "rows that predict nothing must have zero gradient"
    assert rel_fro(dH, ref["dH"]) <= tol["grad"]
    assert rel_fro(dW, ref["dW"]) <= tol["grad"]
    # the rows of the last (possibly partial) 256-row vocabulary tile on their own
    last = case.wl.V - ((case.wl.V - 1) // 256) * 256
    assert rel_fro(dW[-last:], ref["dW"][-last:]) <= tol["grad"]
    return out, ref


def _case(name, max_tokens, seed=None, **over):
    rb = WL.make_rollout(name, seed)
    sel, pk = oracle_select_pack(rb)
    if max_tokens is not None:
        pk = truncate_pack(pk, max_tokens)
    return HeadCase(rb.wl, pk, sel, rb.seed, DEV, **over)


def test_tiny_fp32_whole_batch(lib):
    case = _case("tiny", None)
    assert case.wl.dtype == "f32"
    _run_case(lib, case, TOL["f32"])


def test_tiny_shapes_in_bf16(lib):
    # the tiny batch again with bf16 operands: one partial tile in every dimension
    case = _case("tiny", None, dtype="bf16")
    _run_case(lib, case, TOL["bf16"])


def test_small_bf16_slice_spanning_tiles(lib):
    # ~1500 loss tokens: several 256-token tiles plus a ragged tail, full D and V of the workload
    case = _case("small", 1500)
    assert case.pk["N"] % 256 != 0 and case.pk["N"] > 1024
    _run_case(lib, case, TOL["bf16"])


def test_vocab_and_token_tails(lib):
    # V with a partial 256-row tile and a partial 64-column pad; N well below one tile
    rb = WL.make_rollout("tiny", 3)
    sel, pk = oracle_select_pack(rb)
    for V, D in ((1000, 64), (4200, 128), (257, 192)):
        case = HeadCase(rb.wl, pk, sel, 3, DEV, D=D, V=V, dtype="bf16")
        # targets on tile edges and the last vocabulary entry
        edge = np.array([0, 255, 256, V - 1, V - 2, 63, 64, min(V - 1, 511)], dtype=np.int32)
        lp = pk["loss_pos"][: len(edge)] + 1
        case.ids_np[lp] = edge
        case.ids = torch.as_tensor(case.ids_np, device=DEV)
        _run_case(lib, case, TOL["bf16"])
    case = HeadCase(rb.wl, pk, sel, 3, DEV, D=40, V=300, dtype="f32")
    _run_case(lib, case, TOL["f32"])


def test_long_chunk_with_few_output_tiles(lib):
    # 8400 loss tokens against a dW of 8 x 1 tiles: the dW GEMM's last (only) round of tiles is
    # nearly empty, so its tiles are cut along the token axis and summed by the second kernel
    case = _case("small", 8400, dtype="bf16", D=256, V=2000)
    assert case.pk["N"] >= 8300
    out, _ = _run_case(lib, case, TOL["bf16"])
    # the summing kernel also honours accumulation into an existing dW
    acc = out["dW"].clone()
    lib.dppo_loss_fwd_bwd(case.H, case.W, case.ids, case.loss_pos, case.loss_cu, case.seq_adv, case.seq_coef,
                          case.logp_old, case.logp_ref, dW=acc, accumulate_dW=True)
    assert torch.equal(acc, 2.0 * out["dW"])
    # a chunk of exactly 2048 tokens: the transposed hidden-state chunk gets a padded row pitch
    case = _case("small", 2048, dtype="bf16", D=256, V=2000)
    assert case.pk["N"] == 2048
    _run_case(lib, case, TOL["bf16"])


def test_clipping_zero_advantage_and_single_token_sequences(lib):
    rng = np.random.default_rng(8)
    # hand-built batch: constant groups (A = 0), one-token completions, both advantage signs
    rewards = np.array([[1, 1, 1, 1], [0, 1, 0, 1], [1, 0, 0, 0], [0, 0, 0, 0]], dtype=np.float32)
    sel = O.select(rewards, None, None, rng.random((4, 4), dtype=np.float32), 0.0, 0.5)
    pl = np.repeat(rng.integers(1, 9, size=4), 4).astype(np.int32)
    cl = rng.integers(1, 40, size=16).astype(np.int32)
    cl[[1, 6, 11]] = 1
    pk = O.pack(pl, cl, sel["keep_comp"].reshape(-1), 64, 3)
    wl = dataclasses.replace(WL.WORKLOADS["tiny"], D=128, V=777, dtype="bf16")
    # old-policy noise large enough that |log rho| > log 1.2 often: both clip branches active
    case = HeadCase(wl, pk, sel, 8, DEV, logp_noise=0.3)
    out, ref = _run_case(lib, case, TOL["bf16"], clip_lo=0.2, clip_hi=0.28, beta=0.1)
    assert 0.05 < ref["clip_frac"] < 0.9
    case32 = HeadCase(dataclasses.replace(wl, dtype="f32"), pk, sel, 8, DEV, logp_noise=0.3)
    _run_case(lib, case32, TOL["f32"], clip_lo=0.2, clip_hi=0.28, beta=0.1)


VARIANTS = [("token", "token_sum"), ("sequence", "seq_mean"), ("sequence", "token_sum")]


@pytest.mark.parametrize("ratio_level,aggregation", VARIANTS)
def test_objective_variants(lib, ratio_level, aggregation):
    """Sequence-level ratio and token-sum aggregation (the objectives the method is plugged into), with a
    decoupled clip tight enough that whole sequences are clipped away at the sequence level."""
    rb = WL.make_rollout("small")
    wl = rb.wl
    sel, pk = oracle_select_pack(rb)
    # token-normalised weights for the token sum: coef * G / (completion tokens of the group)
    if aggregation == "token_sum":
        want = O.token_norm_coef(sel["coef"], rb.comp_len)
        got = lib.dppo_token_norm_coef(torch.as_tensor(sel["coef"].astype(np.float32), device=DEV), rb.comp_len)
        assert np.allclose(got.cpu().numpy(), want, rtol=2e-6, atol=0)
        sel = dict(sel, coef=want)
    # advantages of both signs on every sequence (the workload's own are mostly zero on a short prefix)
    sel = dict(sel, adv=np.random.default_rng(12).normal(size=sel["adv"].shape).astype(np.float32))
    pk = truncate_pack(pk, 6000)
    case = HeadCase(wl, pk, sel, rb.seed, DEV, logp_noise=0.3)
    clip = dict(clip_lo=0.2, clip_hi=0.28)
    if ratio_level == "sequence":
        # sequence ratios sit much closer to 1 than token ratios: clip at their median distance from 1
        base, _ = case.oracle_logprob()
        case.set_behaviour_logps(base)
        cu = case.pk["loss_cu"]
        dist = [abs(np.expm1(np.mean(base[cu[i]:cu[i + 1]] - case.logp_old_np[cu[i]:cu[i + 1]]))) for i in range(len(cu) - 1)]
        clip = dict(clip_lo=float(np.median(dist)), clip_hi=float(np.median(dist)) * 1.5)
    out, ref = _run_case(lib, case, TOL["bf16"], beta=0.04, ratio_level=ratio_level, aggregation=aggregation, **clip)
    assert 0.0 < ref["clip_frac"] < 1.0
    # the workspace-limited (several chunks) and recompute paths agree with the default one
    T, N, D, V = case.pk["T"], case.pk["N"], wl.D, wl.V
    ws_min, ws_full = lib.dppo_workspace_min_bytes(T, N, D, V, 1, True), lib.dppo_workspace_bytes(T, N, D, V, 1, True)
    args = (case.H, case.W, case.ids, case.loss_pos, case.loss_cu, case.seq_adv, case.seq_coef, case.logp_old,
            case.logp_ref)
    kw = dict(beta=0.04, ratio_level=ratio_level, aggregation=aggregation, **clip)
    small = lib.dppo_loss_fwd_bwd(*args, ws=lib.alloc_workspace((ws_min + ws_full) // 2, DEV), **kw)
    # (the sequence ratios of the chunked call come from the forward-only pass, whose log-probs may differ
    # in the last bit from those of the pass that also keeps the exponentials)
    same_seq = torch.equal if ratio_level == "token" else (lambda a, b: torch.allclose(a, b, rtol=1e-5, atol=1e-6))
    assert _same_rows(small["dH"], out["dH"]) and same_seq(small["seq_loss"], out["seq_loss"])
    rec = lib.dppo_loss_fwd_bwd(*args, recompute_logits=True, **kw)
    assert rel_fro(to_np64(rec["dW"]), ref["dW"]) <= 1e-2 and _same_loss(rec["loss"], out["loss"], ref, case)


def test_sequence_ratio_with_forward_running_ahead(lib):
    """Sequence-level ratio with max_seq_tokens given: the forward of chunk c + 1 runs ahead of the backward of
    chunk c (one vocabulary GEMM per chunk, not two), the results are those of the single-chunk call, a broken
    promise is flagged, and without the promise the extra forward pass is taken."""
    rb = WL.make_rollout("small")
    sel, pk = oracle_select_pack(rb)
    sel = dict(sel, adv=np.random.default_rng(12).normal(size=sel["adv"].shape).astype(np.float32))
    pk = truncate_pack(pk, 6000)
    case = HeadCase(rb.wl, pk, sel, rb.seed, DEV, logp_noise=0.3)
    base, _ = case.oracle_logprob()
    case.set_behaviour_logps(base)
    cu = case.pk["loss_cu"]
    longest = int(np.diff(cu).max())
    assert 512 < longest <= 1024
    dist = [abs(np.expm1(np.mean(base[cu[i]:cu[i + 1]] - case.logp_old_np[cu[i]:cu[i + 1]]))) for i in range(len(cu) - 1)]
    kw = dict(beta=0.04, ratio_level="sequence", clip_lo=float(np.median(dist)), clip_hi=float(np.median(dist)) * 1.5)
    out, ref = _run_case(lib, case, TOL["bf16"], **kw)            # one chunk
    assert 0.0 < ref["clip_frac"] < 1.0
    T, N, D, V = case.pk["T"], case.pk["N"], case.wl.D, case.wl.V
    args = (case.H, case.W, case.ids, case.loss_pos, case.loss_cu, case.seq_adv, case.seq_coef, case.logp_old,
            case.logp_ref)
    lo2, hi2 = lib.dppo_workspace_min_bytes(T, N, D, V, 1, 2), lib.dppo_workspace_bytes(T, N, D, V, 1, 2)
    assert hi2 > lib.dppo_workspace_bytes(T, N, D, V, 1, 1) and lo2 > lib.dppo_workspace_min_bytes(T, N, D, V, 1, 1)
    # a workspace for two sets of chunks of about 1300 tokens (256 at lo2, 6144 at hi2, linear in between)
    ws = lib.alloc_workspace(lo2 + (hi2 - lo2) * (1300 - 256) // (6144 - 256), DEV)
    status = torch.full((1,), -1, dtype=torch.int32, device=DEV)

    def launches(**more):
        lib.dppo_timing_enable(True)
        lib.dppo_timing_read(reset=True)
        res = lib.dppo_loss_fwd_bwd(*args, ws=ws, status=status, **kw, **more)
        torch.cuda.synchronize()
        t = lib.dppo_timing_read(reset=True)
        lib.dppo_timing_enable(False)
        return res, t["logits_gemm"][1], t["dh_gemm"][1]

    for recompute in (False, True):
        got, n_logits, n_dh = launches(max_seq_tokens=longest, recompute_logits=recompute)
        assert n_dh >= 4 and n_logits == (2 if recompute else 1) * n_dh, (n_logits, n_dh)
        assert int(status.item()) == 0
        if not recompute:
            assert _same_rows(got["dH"], out["dH"]) and torch.equal(got["seq_loss"], out["seq_loss"])
        assert rel_fro(to_np64(got["dW"]), ref["dW"]) <= 1e-2 and rel_fro(to_np64(got["dH"]), ref["dH"]) <= 1e-2
        assert _same_loss(got["loss"], out["loss"], ref, case)
        assert np.abs(got["logp"].cpu().numpy() - ref["logp"]).max() <= TOL["bf16"]["logp"]
    # no promise: one forward-only pass first
    got, n_logits, n_dh = launches()
    assert n_logits == 2 * n_dh and int(status.item()) == 0
    assert _same_rows(got["dH"], out["dH"]) and torch.allclose(got["seq_loss"], out["seq_loss"], rtol=1e-5, atol=1e-6)
    # a promise the chunks cannot hold falls back to that pass as well
    got, n_logits, n_dh = launches(max_seq_tokens=4 * longest)
    assert n_logits == 2 * n_dh and int(status.item()) == 0
    # a broken promise (sequences of up to 1012 tokens against chunks of 256): flagged, every kernel runs to the end
    ws = lib.alloc_workspace(lo2, DEV)
    got, n_logits, n_dh = launches(max_seq_tokens=256)
    assert n_logits == n_dh == -(-N // 256)
    assert int(status.item()) & lib.HEAD_SEQ_TOO_LONG
    assert np.abs(got["logp"].cpu().numpy() - ref["logp"]).max() <= TOL["bf16"]["logp"]


@pytest.mark.parametrize("case_seed", [11, 12, 13, 14, 15, 16, 17, 18])
def test_random_shapes_with_tails(lib, case_seed):
    """Seeded random shapes (D any multiple of 64, so the 256-row blocks of the backward GEMMs' B operands are
    partly filled; V and N with tails), a workspace of random size between the minimum and the recommended one
    (several chunks), both gradient modes, and the sequence-level ratio with the forward running ahead."""
    rng = np.random.default_rng(case_seed)
    D = int(rng.choice([64, 128, 192, 320, 448, 576, 1024, 1088]))
    V = int(rng.integers(100, 6000))
    case = _case("small", int(rng.integers(150, 2600)), seed=int(rng.integers(1, 10**6)), dtype="bf16", D=D, V=V)
    T, N = case.pk["T"], case.pk["N"]
    out, ref = _run_case(lib, case, TOL["bf16"])
    args = (case.H, case.W, case.ids, case.loss_pos, case.loss_cu, case.seq_adv, case.seq_coef, case.logp_old,
            case.logp_ref)
    lo, hi = lib.dppo_workspace_min_bytes(T, N, D, V, 1, True), lib.dppo_workspace_bytes(T, N, D, V, 1, True)
    ws = lib.alloc_workspace(int(lo + (hi - lo) * float(rng.uniform(0.0, 0.9))), DEV)
    for recompute in (False, True):
        got = lib.dppo_loss_fwd_bwd(*args, ws=ws, recompute_logits=recompute)
        assert rel_fro(to_np64(got["dW"]), ref["dW"]) <= 1e-2 and rel_fro(to_np64(got["dH"]), ref["dH"]) <= 1e-2
        assert np.abs(got["logp"].cpu().numpy() - ref["logp"]).max() <= TOL["bf16"]["logp"]
        _assert_loss(float(got["loss"].item()), ref, case, TOL["bf16"]["loss"])
    ref_s = case.oracle_loss(ratio_level="sequence")
    lo2, hi2 = lib.dppo_workspace_min_bytes(T, N, D, V, 1, 2), lib.dppo_workspace_bytes(T, N, D, V, 1, 2)
    ws2 = lib.alloc_workspace(int(lo2 + (hi2 - lo2) * float(rng.uniform(0.3, 1.0))), DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    got = lib.dppo_loss_fwd_bwd(*args, ws=ws2, ratio_level="sequence", status=status,
                                max_seq_tokens=int(np.diff(case.pk["loss_cu"]).max()))
    assert int(status.item()) == 0
    assert rel_fro(to_np64(got["dW"]), ref_s["dW"]) <= 1e-2 and rel_fro(to_np64(got["dH"]), ref_s["dH"]) <= 1e-2
    _assert_loss(float(got["loss"].item()), ref_s, case, TOL["bf16"]["loss"])


def test_objective_variants_fp32(lib):
    case = _case("tiny", None)
    for ratio_level, aggregation in VARIANTS:
        _run_case(lib, case, TOL["f32"], clip_lo=0.002, clip_hi=0.003, ratio_level=ratio_level, aggregation=aggregation)


def test_targets_of_vanishing_probability(lib):
    # The bf16 backward pass keeps exp(z - z_target) per stored entry; rows whose target has a
    # log-prob below about -34.5 leave the range that scheme is used in and must come out right through
    # the exact row path (some of them overflow the stored exponentials outright), next to rows just
    # above the limit, with stored exponentials up to e^34, and ordinary rows on the fast path.
    # Second shape: D beyond one 2048-column slab of the exact path.
    for D, V, factor, mid in ((128, 777, 64.0, 16.0), (2304, 300, 16.0, 4.0)):
        case = _case("tiny", None, dtype="bf16", D=D, V=V)
        lp = torch.as_tensor(case.pk["loss_pos"], device=DEV).long()
        case.H[lp[::3]] *= factor       # exact in bf16
        case.H[lp[1::3]] *= mid
        logp_ref, _ = case.oracle_logprob()
        assert (logp_ref < -100).sum() >= 5 and (logp_ref > -15).sum() >= 5
        assert ((logp_ref > -34) & (logp_ref < -20)).sum() >= 5 and ((logp_ref > -69) & (logp_ref < -35)).sum() >= 5
        _run_case(lib, case, TOL["bf16"])
    # several chunks (smallest workspace), each with its own list of rows to redo
    case = _case("small", 1500)
    lp = torch.as_tensor(case.pk["loss_pos"], device=DEV).long()
    case.H[lp[::5]] *= 64.0
    logp_ref, _ = case.oracle_logprob()
    assert (logp_ref < -100).sum() >= 100
    case.set_behaviour_logps(logp_ref)
    ref = case.oracle_loss()
    T, N, D, V = case.pk["T"], case.pk["N"], case.wl.D, case.wl.V
    ws = lib.alloc_workspace(lib.dppo_workspace_min_bytes(T, N, D, V, 1, True), DEV)
    out = lib.dppo_loss_fwd_bwd(case.H, case.W, case.ids, case.loss_pos, case.loss_cu, case.seq_adv, case.seq_coef,
                                case.logp_old, case.logp_ref, ws=ws)
    assert np.abs(out["logp"].cpu().numpy() - ref["logp"]).max() <= TOL["bf16"]["logp"]
    assert rel_fro(to_np64(out["dH"]), ref["dH"]) <= 1e-2 and rel_fro(to_np64(out["dW"]), ref["dW"]) <= 1e-2


def test_coincident_policies(lib):
    case = _case("tiny", None, dtype="bf16")
    logp, _ = lib.dppo_token_logprob(case.H, case.W, case.ids, case.loss_pos)
    out = lib.dppo_loss_fwd_bwd(case.H, case.W, case.ids, case.loss_pos, case.loss_cu, case.seq_adv, case.seq_coef,
                                logp, logp)
    # ratio 1 and KL 0: each sequence's loss is minus its advantage
    assert np.allclose(out["seq_loss"].cpu().numpy(), -case.seq_adv_np, rtol=1e-5, atol=1e-6)
    assert abs(float(out["stats"][0])) < 1e-9 and float(out["stats"][1]) == 0.0


def test_identity_rows_chunking_accumulation_and_recompute(lib):
    case = _case("small", 1200)
    logp_ref, _ = case.oracle_logprob()
    case.set_behaviour_logps(logp_ref)
    ref = case.oracle_loss()
    P = lib
    args = (case.H, case.W, case.ids, case.loss_pos, case.loss_cu, case.seq_adv, case.seq_coef, case.logp_old,
            case.logp_ref)
    base = P.dppo_loss_fwd_bwd(*args)
    # (a) a workspace that only fits small chunks gives the same result up to summation order
    T, N, D, V = case.pk["T"], case.pk["N"], case.wl.D, case.wl.V
    ws_min, ws_full = P.dppo_workspace_min_bytes(T, N, D, V, 1, True), P.dppo_workspace_bytes(T, N, D, V, 1, True)
    small_ws = P.alloc_workspace((ws_min + ws_full) // 2, DEV)
    assert ws_min < small_ws.numel() < ws_full
    chunked = P.dppo_loss_fwd_bwd(*args, ws=small_ws)
    assert rel_fro(to_np64(chunked["dW"]), ref["dW"]) <= 1e-2
    assert rel_fro(to_np64(chunked["dW"]), to_np64(base["dW"])) <= 1e-4
    assert _same_rows(chunked["dH"], base["dH"])
    assert abs(float(chunked["loss"]) - float(base["loss"])) <= 1e-6 * abs(float(base["loss"])) + 1e-9
    # (b) accumulate_dW adds to the buffer
    acc = base["dW"].clone()
    P.dppo_loss_fwd_bwd(*args, dW=acc, accumulate_dW=True)
    assert rel_fro(to_np64(acc), 2.0 * to_np64(base["dW"])) <= 1e-6
    # (c) recomputing the logits in the backward instead of keeping a chunk of exponentials
    rec = P.dppo_loss_fwd_bwd(*args, recompute_logits=True)
    assert rel_fro(to_np64(rec["dH"]), ref["dH"]) <= 1e-2
    assert rel_fro(to_np64(rec["dW"]), ref["dW"]) <= 1e-2
    assert _same_loss(rec["loss"], base["loss"], ref, case)
    # (d) identity loss rows: compact H rows and targets handed over directly
    lp = case.pk["loss_pos"]
    Hc = case.H[torch.as_tensor(lp, device=DEV).long()].contiguous()
    yc = case.ids[torch.as_tensor(lp + 1, device=DEV).long()].contiguous()
    ident = P.dppo_loss_fwd_bwd(Hc, case.W, yc, None, case.loss_cu, case.seq_adv, case.seq_coef, case.logp_old,
                                case.logp_ref)
    assert torch.equal(ident["dH"], base["dH"][torch.as_tensor(lp, device=DEV).long()])
    assert rel_fro(to_np64(ident["dW"]), to_np64(base["dW"])) <= 1e-6
    lpi, _ = P.dppo_token_logprob(Hc, case.W, yc, None)
    assert np.abs(lpi.cpu().numpy() - logp_ref).max() <= 2e-3


def test_empty_batch(lib):
    # every completion pruned: packed tokens may exist, loss tokens do not
    for dtype in (torch.bfloat16, torch.float32):
        T, D, V = 37, 128, 300
        H = torch.randn(T, D, device=DEV).to(dtype)
        W = torch.randn(V, D, device=DEV).to(dtype)
        ids = torch.zeros(T, dtype=torch.int32, device=DEV)
        none_i = torch.zeros(0, dtype=torch.int32, device=DEV)
        none_f = torch.zeros(0, dtype=torch.float32, device=DEV)
        cu = torch.zeros(1, dtype=torch.int32, device=DEV)
        logp, lse = lib.dppo_token_logprob(H, W, ids, none_i)
        assert logp.numel() == 0 and lse.numel() == 0
        out = lib.dppo_loss_fwd_bwd(H, W, ids, none_i, cu, none_f, none_f, none_f, none_f)
        torch.cuda.synchronize()
        assert float(out["loss"]) == 0.0 and out["seq_loss"].numel() == 0 and float(out["stats"][2]) == 0.0
        assert not bool(out["dH"].any()) and not bool(out["dW"].any())
        keep = torch.full((V, D), 3.0, device=DEV)
        lib.dppo_loss_fwd_bwd(H, W, ids, none_i, cu, none_f, none_f, none_f, none_f, dW=keep, accumulate_dW=True)
        assert bool((keep == 3.0).all())


def test_hip_graph_replays_match_eager(lib):
    # The entry points only enqueue kernels on the caller's stream (no allocation, no
    # synchronisation, no memset nodes), so a whole loss step can be captured once and replayed.
    # Every replay is checked against the eager result, with eager work, changed inputs and
    # synchronisations between the replays.
    case = _case("small", 1500)
    logp_ref, _ = case.oracle_logprob()
    case.set_behaviour_logps(logp_ref)
    args = (case.H, case.W, case.ids, case.loss_pos, case.loss_cu, case.seq_adv, case.seq_coef, case.logp_old,
            case.logp_ref)
    eager = lib.dppo_loss_fwd_bwd(*args)            # also runs the one-time kernel attribute setup
    T, N, D, V = case.pk["T"], case.pk["N"], case.wl.D, case.wl.V
    ws = lib.alloc_workspace(lib.dppo_workspace_bytes(T, N, D, V, 1, True), DEV)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        out = lib.dppo_loss_fwd_bwd(*args, ws=ws)
    keys = ("loss", "logp", "seq_loss", "stats", "dH", "dW")
    for rep in range(3):
        for k in keys:
            out[k].fill_(float("nan"))               # eager work between the replays
        if rep == 2:                                 # changed inputs: the graph reads the same buffers
            case.logp_old.add_(0.05)
            eager = lib.dppo_loss_fwd_bwd(*args)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in keys:
            assert torch.equal(out[k], eager[k]), (rep, k)


def test_argument_validation(lib):
    case = _case("tiny", None, dtype="bf16")
    P = lib
    with pytest.raises(P.DppoError):      # workspace too small
        P.dppo_token_logprob(case.H, case.W, case.ids, case.loss_pos, ws=P.alloc_workspace(256, DEV))
    H_bad = torch.zeros((case.pk["T"], 72), dtype=torch.bfloat16, device=DEV)   # D % 64 != 0
    W_bad = torch.zeros((64, 72), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(P.DppoError):
        P.dppo_token_logprob(H_bad, W_bad, case.ids, case.loss_pos)


@pytest.mark.parametrize("name,recompute", [("qwen3_4b", False), ("qwen3_8b", False), ("stress", False),
                                            ("stress", True), ("qwen3_4b", True)])
def test_full_width_slices(lib, name, recompute):
    # full hidden and vocabulary size of the Qwen3-shaped workloads on the first packed sequences up to
    # 2100 loss tokens: eight full 256-token tiles and a ragged ninth, V = 151936 (593 full vocabulary
    # tiles and one half tile). With recompute the backward runs the vocabulary GEMM a second time
    # (the mode the stress configuration is stated in), whose epilogue masks the half tile by itself.
    case = _case(name, 2100)
    assert case.pk["N"] == 2100 and case.wl.V % 256 != 0
    _run_case(lib, case, TOL["bf16"], recompute_logits=recompute)


def test_status_word_and_empty_segment(lib):
    """Conditions only the device can see: a target id outside [0, V) and a loss_pos entry outside
    [0, T - 1) are clamped and reported in the status word; every kernel still finishes and the
    tokens that were fine come out as without the fault. An empty segment of loss_cu contributes 0."""
    case = _case("tiny", None, dtype="bf16", D=128, V=1000)
    logp_ref, _ = case.oracle_logprob()
    case.set_behaviour_logps(logp_ref)
    ref = case.oracle_loss()
    args = (case.loss_cu, case.seq_adv, case.seq_coef, case.logp_old, case.logp_ref)
    status = torch.full((1,), 77, dtype=torch.int32, device=DEV)
    good = lib.dppo_loss_fwd_bwd(case.H, case.W, case.ids, case.loss_pos, *args, status=status)
    assert int(status.item()) == 0
    lib.dppo_token_logprob(case.H, case.W, case.ids, case.loss_pos, status=status.fill_(77))
    assert int(status.item()) == 0
    N, T, V = case.pk["N"], case.pk["T"], case.wl.V
    # (a) a target id beyond the vocabulary (token 5) and a negative one (token 9)
    ids_bad = case.ids.clone()
    lp = case.pk["loss_pos"]
    ids_bad[int(lp[5]) + 1] = V + 7
    ids_bad[int(lp[9]) + 1] = -3
    logp, _ = lib.dppo_token_logprob(case.H, case.W, ids_bad, case.loss_pos, status=status.fill_(77))
    assert int(status.item()) == lib.HEAD_BAD_TARGET
    okay = np.ones(N, bool)
    okay[[5, 9]] = False
    assert np.abs(logp.cpu().numpy() - logp_ref)[okay].max() <= 2e-3 and torch.isfinite(logp).all()
    out = lib.dppo_loss_fwd_bwd(case.H, case.W, ids_bad, case.loss_pos, *args, status=status.fill_(77))
    assert int(status.item()) == lib.HEAD_BAD_TARGET
    assert torch.isfinite(out["dH"].float()).all() and torch.isfinite(out["dW"]).all()
    # (b) loss positions outside the packed tokens
    pos_bad = case.loss_pos.clone()
    pos_bad[3] = T + 1000
    pos_bad[4] = -5
    pos_bad[N - 1] = T - 1                     # its target would be token T
    logp, _ = lib.dppo_token_logprob(case.H, case.W, case.ids, pos_bad, status=status.fill_(77))
    assert int(status.item()) == lib.HEAD_BAD_POSITION
    okay = np.ones(N, bool)
    okay[[3, 4, N - 1]] = False
    assert np.abs(logp.cpu().numpy() - logp_ref)[okay].max() <= 2e-3
    out = lib.dppo_loss_fwd_bwd(case.H, case.W, case.ids, pos_bad, *args, status=status.fill_(77))
    torch.cuda.synchronize()
    assert int(status.item()) == lib.HEAD_BAD_POSITION
    assert torch.isfinite(out["dH"].float()).all() and torch.isfinite(out["dW"]).all()
    # both at once
    lib.dppo_loss_fwd_bwd(case.H, case.W, ids_bad, pos_bad, *args, status=status.fill_(77))
    assert int(status.item()) == lib.HEAD_BAD_TARGET | lib.HEAD_BAD_POSITION
    # (c) an empty segment in the middle and one at the end: same loss and gradients as without them
    cu = case.pk["loss_cu"]
    S = len(cu) - 1
    cu2 = np.concatenate([cu[:3], [cu[2]], cu[3:], [cu[-1]]]).astype(np.int32)
    ins = lambda a, v: np.concatenate([a[:2], [v], a[2:], [v]]).astype(np.float32)
    for ratio_level in ("token", "sequence"):
        base = lib.dppo_loss_fwd_bwd(case.H, case.W, case.ids, case.loss_pos, *args, ratio_level=ratio_level)
        out = lib.dppo_loss_fwd_bwd(case.H, case.W, case.ids, case.loss_pos, torch.as_tensor(cu2, device=DEV),
                                    torch.as_tensor(ins(case.seq_adv_np, 1.5), device=DEV),
                                    torch.as_tensor(ins(case.seq_coef_np, 0.25), device=DEV), case.logp_old,
                                    case.logp_ref, ratio_level=ratio_level)
        # (the final sum over sequences associates differently once the indices shift)
        assert torch.allclose(out["loss"], base["loss"], rtol=1e-6, atol=0) and torch.equal(out["dH"], base["dH"])
        assert torch.equal(out["dW"], base["dW"])
        sl = out["seq_loss"].cpu().numpy()
        assert sl[2] == 0.0 and sl[-1] == 0.0 and np.array_equal(np.delete(sl, [2, S + 1]), base["seq_loss"].cpu().numpy())
    assert abs(float(good["loss"]) - ref["loss"]) <= 1e-3 * max(abs(ref["loss"]), 1e-3)
