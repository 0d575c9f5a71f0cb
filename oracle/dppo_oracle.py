"""CPU oracle for the DPPO loss hot path -- TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 NumPy statement of what the path computes, written from the
paper's definitions (Sec. 3 Eq. 1-2; Sec. 4.2 Eq. 14-18; Sec. 4.3; Alg. 1). It
shares no code with the HIP library, imports nothing from it, and must never be
called by it: only tests, the smoke check and the benchmark's CPU-baseline leg
use it. NumPy's matmul / exp / log are the only library steps; nothing is
blocked, fused or reordered beyond what the definitions say.

Every function here is pinned by tests that do not go through this module's own
formulas (closed forms, brute-force enumeration, invariants, finite differences,
library log-softmax and autograd); none is "parity unpinned". Readings of the
paper where it is silent (sample std, realised-count constants, first-fit scan,
weights on the KL term, ...) are listed with each function.
"""
from __future__ import annotations

import math
from typing import Optional

import numpy as np


# ----------------------------------------------------------------------------
# Sec. 3, Eq. 2: group-relative advantages
# ----------------------------------------------------------------------------
def group_advantages(rewards, ddof: int = 1, eps: float = 1e-6) -> np.ndarray:
    """A[k,i] = (r[k,i] - mean_k) / (std_k + eps), one group per row (Eq. 2).

    Reading: the paper says only "std"; ddof selects population (0) or sample (1)
    and eps is added to the standard deviation so constant groups give A = 0.
    """
    r = np.asarray(rewards, dtype=np.float64)
    Q, G = r.shape
    if G - ddof <= 0:
        raise ValueError("G - ddof must be positive")
    A = np.empty_like(r)
    for k in range(Q):
        mu = sum(float(x) for x in r[k]) / G
        var = sum((float(x) - mu) ** 2 for x in r[k]) / (G - ddof)
        sd = math.sqrt(var)
        for i in range(G):
            A[k, i] = (float(r[k, i]) - mu) / (sd + eps)
    return A


def completion_candidates(rewards) -> np.ndarray:
    """Candidate test of Eq. 15: |A_i| <= mean_j |A_j| within a group (inclusive).

    Both sides of the inequality carry the same positive factor 1/(std+eps) and the
    same 1/G, so it is decided on the scaled integers-friendly form
        G * |G r_i - S|  <=  sum_j |G r_j - S| ,   S = sum_j r_j ,
    in fp64, left to right, without fused multiply-add. With binary or small
    integer rewards every quantity is an exact integer, so ties (balanced groups,
    constant groups) come out as the real-number inequality says.
    """
    r = np.asarray(rewards, dtype=np.float64)
    Q, G = r.shape
    cand = np.zeros((Q, G), dtype=bool)
    for k in range(Q):
        S = 0.0
        for i in range(G):
            S = S + float(r[k, i])
        e = [abs(float(G) * float(r[k, i]) - S) for i in range(G)]
        tot = 0.0
        for i in range(G):
            tot = tot + e[i]
        for i in range(G):
            cand[k, i] = (float(G) * e[i]) <= tot
    return cand


def prompt_candidates(hist, bottom_frac: float = 0.5) -> np.ndarray:
    """B_t of Eq. 17: the floor(bottom_frac*Q) prompts with the lowest history score.

    Reading: ties are broken by the lower prompt index; for odd Q the count is
    rounded down.
    """
    h = np.asarray(hist, dtype=np.float32)
    Q = h.shape[0]
    n_b = int(math.floor(float(np.float32(bottom_frac)) * Q))
    idx = sorted(range(Q), key=lambda k: (float(h[k]), k))
    inB = np.zeros(Q, dtype=bool)
    for k in idx[:n_b]:
        inB[k] = True
    return inB


# ----------------------------------------------------------------------------
# Sec. 4.2: pruning policies (Eq. 14-17), realised masks, rescaling (Eq. 18)
# ----------------------------------------------------------------------------
def fixed_prune_count(r: float, n: int) -> int:
    """Number pruned from a candidate set of n in the fixed-count form (App. A; Alg. 1:
    floor(r * n)). r arrives as float32 (relative error 6e-8), so the product is scaled by
    1 + 1e-6 before the floor: 0.9f * 10 gives 9 and 0.7f * 100 gives 70. At least one
    candidate always survives."""
    if n <= 0:
        return 0
    m = int(math.floor(float(np.float32(r)) * n * (1.0 + 1e-6)))
    return max(0, min(m, n - 1))


def select(rewards, hist, u_prompt, u_comp, r_q: float, r_o: float,
           ddof: int = 1, eps: float = 1e-6, bottom_frac: float = 0.5,
           fixed_count: bool = False, realised_rate: bool = True) -> dict:
    """Advantages, prune masks and importance-rescaling weights for one batch.

    Pruning is the Bernoulli form of Eq. 15 / Eq. 17 with caller-supplied uniforms:
    a candidate is pruned iff its uniform is < r (float32 comparison). hist=None
    skips prompt-level pruning (first epoch), u_*=None skips that level.
    A pruned prompt drops all its completions. Advantages always come from the
    full group (Alg. 1 computes them before pruning).

    fixed_count=True is the form of App. A / Alg. 1: exactly floor(r * |candidates|) of each
    candidate set are pruned. Reading: the paper does not say which ones; here they are the
    candidates with the smallest uniforms (ties to the lower index), i.e. a uniformly random
    subset of fixed size, so every candidate is pruned with probability m/n. With
    realised_rate=True that realised rate m/n replaces r in Eq. 18, which keeps the estimator
    exactly unbiased; realised_rate=False uses the nominal r as Eq. 18 is printed (unbiased
    only when r * n is an integer).

    Weights follow Eq. 18 with the realised counts:
        gamma_q[k]   = (|S^q| / Q) / (1 - P^q[k])
        gamma_o[k,i] = (|S^o_k| / G) / (1 - P^o[k,i])
    and coef[k,i] = gamma_q*gamma_o / (|S^q| * |S^o_k|) is the weight of sequence
    (k,i) in the batch loss (mean over retained prompts of the mean over retained
    completions), 0 for pruned sequences.
    """
    r = np.asarray(rewards, dtype=np.float32)
    Q, G = r.shape
    rq = float(np.float32(r_q))
    ro = float(np.float32(r_o))
    A = group_advantages(r, ddof, eps)
    mean_abs = np.array([sum(abs(float(a)) for a in A[k]) / G for k in range(Q)])
    cand = completion_candidates(r)
    inB = prompt_candidates(hist, bottom_frac) if hist is not None else np.zeros(Q, dtype=bool)
    if u_prompt is None:
        inB_eff = np.zeros(Q, dtype=bool)
    else:
        inB_eff = inB
    uc = None if u_comp is None else np.asarray(u_comp, dtype=np.float32).reshape(Q, G)
    keep_prompt = np.ones(Q, dtype=np.uint8)
    keep_comp = np.zeros((Q, G), dtype=np.uint8)
    Pq = np.zeros(Q)
    Po = np.zeros((Q, G))
    if not fixed_count:
        Pq = np.where(inB_eff, rq, 0.0)
        Po = np.where(cand, ro, 0.0) if uc is not None else np.zeros((Q, G))
        if u_prompt is not None:
            up = np.asarray(u_prompt, dtype=np.float32)
            for k in range(Q):
                if inB_eff[k] and up[k] < np.float32(r_q):
                    keep_prompt[k] = 0
        for k in range(Q):
            for i in range(G):
                pruned = (uc is not None) and bool(cand[k, i]) and (uc[k, i] < np.float32(r_o))
                keep_comp[k, i] = 1 if (keep_prompt[k] and not pruned) else 0
    else:
        if u_prompt is not None:
            up = np.asarray(u_prompt, dtype=np.float32)
            B = [k for k in range(Q) if inB_eff[k]]
            m_q = fixed_prune_count(r_q, len(B))
            for k in sorted(B, key=lambda k: (float(up[k]), k))[:m_q]:
                keep_prompt[k] = 0
            for k in B:
                Pq[k] = (m_q / len(B)) if realised_rate else rq
        for k in range(Q):
            pruned_set = set()
            if uc is not None:
                Ck = [i for i in range(G) if cand[k, i]]
                m_o = fixed_prune_count(r_o, len(Ck))
                pruned_set = set(sorted(Ck, key=lambda i: (float(uc[k, i]), i))[:m_o])
                for i in Ck:
                    Po[k, i] = (m_o / len(Ck)) if realised_rate else ro
            for i in range(G):
                keep_comp[k, i] = 1 if (keep_prompt[k] and i not in pruned_set) else 0

    n_q = int(keep_prompt.sum())
    n_o = keep_comp.sum(axis=1).astype(np.int64)
    gamma_q = np.zeros(Q)
    gamma_o = np.zeros((Q, G))
    coef = np.zeros((Q, G))
    for k in range(Q):
        if not keep_prompt[k]:
            continue
        gamma_q[k] = (n_q / Q) / (1.0 - Pq[k])
        for i in range(G):
            if keep_comp[k, i]:
                gamma_o[k, i] = (int(n_o[k]) / G) / (1.0 - Po[k, i])
                coef[k, i] = gamma_q[k] * gamma_o[k, i] / (n_q * int(n_o[k]))
    return dict(adv=A, mean_abs_adv=mean_abs, cand=cand, in_bottom=inB_eff,
                keep_prompt=keep_prompt, keep_comp=keep_comp,
                gamma_q=gamma_q, gamma_o=gamma_o, coef=coef,
                counts=np.concatenate([[n_q], n_o]).astype(np.int32),
                P_q=Pq, P_o=Po)


def history_update(hist_table, prompt_index, keep_prompt, mean_abs_adv) -> np.ndarray:
    """Carry-forward history score of Eq. 16: a prompt selected in this epoch gets its fresh
    mean |A|; a prompt that was pruned (no rollout, no new statistics) keeps its last score.
    hist_table is the score of every prompt of the dataset, prompt_index the dataset index of
    each prompt of the batch. Returns the updated table (float32)."""
    out = np.array(hist_table, dtype=np.float32, copy=True)
    for b, q in enumerate(np.asarray(prompt_index, dtype=np.int64)):
        if keep_prompt[b]:
            out[q] = np.float32(mean_abs_adv[b])
    return out


# ----------------------------------------------------------------------------
# Sec. 4.3: Dense Prompt Packing (window-based greedy selection)
# ----------------------------------------------------------------------------
def pack(prompt_len, comp_len, keep, capacity, n_win: int, policy: str = "first_fit") -> dict:
    """Window-based greedy packing of the kept sequences into rows of `capacity` tokens (Sec. 4.3).

    Items are the kept sequences in index order, length = prompt + completion.
    A pool holds up to n_win items in arrival order and is refilled from the stream
    after every placement. The paper only says that samples of the pool that fit the
    remaining space are selected greedily; two readings are offered:
      "first_fit": the pool is scanned from its oldest item to its newest (items fetched
                   during the scan included) and every item that still fits is placed;
      "best_fit":  the longest pool item that fits is placed (oldest among equals), and
                   this repeats, refilled items included, until no pool item fits.

    comp_len=None packs prompts alone, the paper's own use at dataset initialisation:
    no loss positions exist then. capacity=None or 0 takes L_max = the longest kept item.

    Returns order (original item indices in packed order), row_ptr (row boundaries
    in sequences), cu_seqlens (token offsets of the packed sequences), loss_cu
    (offsets into the compact loss-token index), loss_pos (packed positions
    whose hidden state predicts a completion token: for a sequence starting at c
    with prompt P and completion C these are c+P-1 ... c+P+C-2), the capacity used and
    density = T / (n_rows * capacity), the share of row slots that hold a real token.
    """
    pl = np.asarray(prompt_len, dtype=np.int64)
    prompts_only = comp_len is None
    cl = np.zeros_like(pl) if prompts_only else np.asarray(comp_len, dtype=np.int64)
    n_all = pl.shape[0]
    kept = [j for j in range(n_all) if keep is None or keep[j]]
    if not capacity:
        capacity = max([int(pl[j] + cl[j]) for j in kept], default=1)
    for j in kept:
        if pl[j] < 1 or (cl[j] < 1 and not prompts_only) or pl[j] + cl[j] > capacity:
            raise ValueError("item %d does not fit a row or has an empty part" % j)
    if n_win < 1:
        raise ValueError("n_win must be >= 1")
    if policy not in ("first_fit", "best_fit"):
        raise ValueError("unknown policy %r" % (policy,))
    n = len(kept)
    stream = list(kept)
    pool = stream[:min(n_win, n)]
    nxt = len(pool)
    order, row_ptr = [], [0]
    while pool:
        rem = capacity
        if policy == "first_fit":
            pos = 0
            while pos < len(pool):
                j = pool[pos]
                ell = int(pl[j] + cl[j])
                if ell <= rem:
                    order.append(j)
                    rem -= ell
                    del pool[pos]
                    if nxt < n:
                        pool.append(stream[nxt])
                        nxt += 1
                else:
                    pos += 1
        else:
            while True:
                best = -1
                for pos, j in enumerate(pool):
                    ell = int(pl[j] + cl[j])
                    if ell <= rem and (best < 0 or ell > int(pl[pool[best]] + cl[pool[best]])):
                        best = pos
                if best < 0:
                    break
                j = pool.pop(best)
                order.append(j)
                rem -= int(pl[j] + cl[j])
                if nxt < n:
                    pool.append(stream[nxt])
                    nxt += 1
        row_ptr.append(len(order))
    cu = [0]
    lcu = [0]
    loss_pos = []
    for j in order:
        c0 = cu[-1]
        P, C = int(pl[j]), int(cl[j])
        loss_pos.extend(range(c0 + P - 1, c0 + P + C - 1))
        cu.append(c0 + P + C)
        lcu.append(lcu[-1] + C)
    return dict(order=np.array(order, dtype=np.int32), row_ptr=np.array(row_ptr, dtype=np.int32),
                cu_seqlens=np.array(cu, dtype=np.int32), loss_cu=np.array(lcu, dtype=np.int32),
                loss_pos=np.array(loss_pos, dtype=np.int32),
                n_rows=len(row_ptr) - 1, T=cu[-1], N=lcu[-1], S=n, capacity=int(capacity),
                density=(cu[-1] / ((len(row_ptr) - 1) * capacity)) if n else 0.0)


# ----------------------------------------------------------------------------
# Variance of the rescaled single-sample estimator (App. D)
# ----------------------------------------------------------------------------
def variance_terms(g, P_q, P_o) -> dict:
    """Quantities of App. D for a scalar component g[Q,G] of Psi(q, o) and prune probabilities
    P_q[Q], P_o[Q,G] (the ones select() reports).

    The estimator is  G_hat = gamma(q) gamma(o,q) g(q,o)  with q drawn from the pruned prompt
    density P~(q) ~ (1 - P_q) / |Q|, o from pi~(o|q) ~ (1 - P_o) / |O|, and the weights of
    Eq. 9 / Eq. 12: gamma(o,q) = C_o(q) / (1 - P_o), C_o(q) = mean_o (1 - P_o), likewise for q.

    Per group (App. D.1):  G(q) = mean_o g,  Var_O = mean_o g^2 - G(q)^2,
        var_o[q] = (C_o / |O|) sum_o g^2 / (1 - P_o) - G(q)^2          (variance of gamma g under pi~)
        cond_o[q] = mean over pruned-with-positive-probability o of g^2/(1-P_o)  <=  mean_o g^2
    Prompt level (App. D.2) the same with G(q) in place of g.
    Total (App. D.3):  term1 = var of gamma(q) G(q);  term2 = E_{q~P~}[gamma(q)^2 var_o[q]]
        = (C_q / |Q|) sum_q var_o[q] / (1 - P_q);  total = term1 + term2;
        egamma2 = E_{q~P~}[gamma(q)^2] = (C_q / |Q|) sum_q 1 / (1 - P_q);
        bound = Var_Q[G(q)] + egamma2 * mean_q Var_O   (Theorem D.1; holds under both conditions).
    """
    g = np.asarray(g, dtype=np.float64)
    Pq = np.asarray(P_q, dtype=np.float64)
    Po = np.asarray(P_o, dtype=np.float64)
    Q, G = g.shape
    Gq = g.mean(axis=1)
    mean_g2 = (g * g).mean(axis=1)
    var_O = mean_g2 - Gq * Gq
    C_o = (1.0 - Po).mean(axis=1)
    var_o = (C_o / G) * (g * g / (1.0 - Po)).sum(axis=1) - Gq * Gq
    cond_o = np.ones(Q, dtype=bool)
    for k in range(Q):
        sel = Po[k] > 0
        if sel.any():
            cond_o[k] = (g[k, sel] ** 2 / (1.0 - Po[k, sel])).mean() <= mean_g2[k]
    Gbar = Gq.mean()
    var_Q = (Gq * Gq).mean() - Gbar * Gbar
    C_q = (1.0 - Pq).mean()
    term1 = (C_q / Q) * (Gq * Gq / (1.0 - Pq)).sum() - Gbar * Gbar
    selq = Pq > 0
    cond_q = bool((Gq[selq] ** 2 / (1.0 - Pq[selq])).mean() <= (Gq * Gq).mean()) if selq.any() else True
    egamma2 = (C_q / Q) * (1.0 / (1.0 - Pq)).sum()
    term2 = (C_q / Q) * (var_o / (1.0 - Pq)).sum()
    return dict(G_q=Gq, var_O=var_O, var_o=var_o, cond_o=cond_o, G_bar=float(Gbar), var_Q=float(var_Q),
                term1=float(term1), cond_q=cond_q, egamma2=float(egamma2), mean_var_O=float(var_O.mean()),
                term2=float(term2), total=float(term1 + term2),
                bound=float(var_Q + egamma2 * var_O.mean()))


# ----------------------------------------------------------------------------
# pi_theta(o_t | q, o_<t): LM-head projection, log-softmax, target gather
# ----------------------------------------------------------------------------
def _targets(ids, loss_pos, N):
    ids = np.asarray(ids)
    if loss_pos is None:
        return np.arange(N), ids[:N].astype(np.int64)
    lp = np.asarray(loss_pos, dtype=np.int64)
    return lp, ids[lp + 1].astype(np.int64)


def token_logprob(H, W, ids, loss_pos):
    """logp[n] = z[n, y_n] - log sum_v exp z[n, v],  z = H[loss_pos] W^T  (no bias, T=1).

    y_n = ids[loss_pos[n] + 1]: the hidden state at a position predicts the next
    token. loss_pos=None means rows of H are the loss rows and ids[n] the targets.
    """
    H = np.asarray(H, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    N = H.shape[0] if loss_pos is None else len(loss_pos)
    rows, y = _targets(ids, loss_pos, N)
    Z = H[rows] @ W.T
    m = Z.max(axis=1)
    lse = m + np.log(np.exp(Z - m[:, None]).sum(axis=1))
    logp = Z[np.arange(N), y] - lse
    return logp, lse


# ----------------------------------------------------------------------------
# Sec. 3 Eq. 1 with the rescaling of Eq. 18: loss and gradients
# ----------------------------------------------------------------------------
def token_terms(logp, logp_old, logp_ref, A, clip_lo: float, clip_hi: float, beta: float):
    """Per-token loss and its derivative w.r.t. logp (Eq. 1, one token).

    rho = pi/pi_old; surrogate = min(rho*A, clip(rho, 1-lo, 1+hi)*A);
    KL = rho_hat - log rho_hat - 1 with rho_hat = pi_ref/pi;  loss = -surrogate + beta*KL.
    The derivative of the min/clip takes the unclipped branch on ties.
    """
    logp = np.asarray(logp, dtype=np.float64)
    d_old = logp - np.asarray(logp_old, dtype=np.float64)
    d_ref = np.asarray(logp_ref, dtype=np.float64) - logp
    rho = np.exp(d_old)
    lo, hi = 1.0 - clip_lo, 1.0 + clip_hi
    unclipped = rho * A
    clipped = np.clip(rho, lo, hi) * A
    surrogate = np.minimum(unclipped, clipped)
    rho_hat = np.exp(d_ref)
    kl = rho_hat - d_ref - 1.0
    ell = -surrogate + beta * kl
    clipped_away = ((A > 0) & (rho > hi)) | ((A < 0) & (rho < lo))
    g = np.where(clipped_away, 0.0, -A * rho) + beta * (1.0 - rho_hat)
    return ell, g, kl, clipped_away


def sequence_terms(logp, logp_old, logp_ref, loss_cu, seq_adv, clip_lo: float, clip_hi: float, beta: float,
                   ratio_level: str = "token", aggregation: str = "seq_mean"):
    """Per-sequence loss term (what the rescaling weight multiplies) and its derivative w.r.t. every
    token log-prob, for the objectives DPPO is plugged into (Sec. 5, robustness across RL algorithms).
    The paper names the algorithms but prints no formulas for them; the readings taken here:

    ratio_level "token" (GRPO, DAPO): every token has its own ratio, token_terms() above.
    ratio_level "sequence" (sequence-level likelihood-ratio optimisation): one ratio per sequence,
        s = (pi(o|q) / pi_old(o|q)) ** (1/|o|) = exp(mean_t (logp_t - logp_old_t)), and every token of the
        sequence carries  loss_t = -min(s A, clip(s, 1-lo, 1+hi) A) + beta KL_t  (unclipped branch on ties).
    aggregation "seq_mean" (Eq. 1): term_s = (1/|o|) sum_t loss_t.
    aggregation "token_sum" (token-level normalisation of the decoupled-clip objective): term_s = sum_t loss_t;
        the 1 / (tokens of the group) factor belongs to the weight, see token_norm_coef().

    Returns (term[S], dterm_dlogp[N], ell[N], kl[N], clipped_away[N]).
    """
    if ratio_level not in ("token", "sequence") or aggregation not in ("seq_mean", "token_sum"):
        raise ValueError("unknown objective variant")
    logp = np.asarray(logp, dtype=np.float64)
    logp_old = np.asarray(logp_old, dtype=np.float64)
    loss_cu = np.asarray(loss_cu, dtype=np.int64)
    S = len(loss_cu) - 1
    N = int(loss_cu[-1])
    A_tok = np.empty(N)
    C_tok = np.empty(N)
    for s in range(S):
        a, b = int(loss_cu[s]), int(loss_cu[s + 1])
        A_tok[a:b] = float(seq_adv[s])
        C_tok[a:b] = b - a
    ell, g, kl, away = token_terms(logp, logp_old, logp_ref, A_tok, clip_lo, clip_hi, beta)
    if ratio_level == "sequence":
        lo, hi = 1.0 - clip_lo, 1.0 + clip_hi
        rho_hat = np.exp(np.asarray(logp_ref, dtype=np.float64) - logp)
        for s in range(S):
            a, b = int(loss_cu[s]), int(loss_cu[s + 1])
            A = float(seq_adv[s])
            ratio = np.exp(np.mean(logp[a:b] - logp_old[a:b]))
            surrogate = min(ratio * A, min(max(ratio, lo), hi) * A)
            gone = (A > 0 and ratio > hi) or (A < 0 and ratio < lo)
            ell[a:b] = -surrogate + beta * kl[a:b]
            away[a:b] = gone
            # d loss_t' / d logp_t = -(A ratio / |o|) 1[not clipped away] for every pair (t', t) of the
            # sequence; summed over t' (all |o| tokens carry the term) this is -A ratio per token t
            g[a:b] = (0.0 if gone else -A * ratio) + beta * (1.0 - rho_hat[a:b])
    term = np.zeros(S)
    for s in range(S):
        a, b = int(loss_cu[s]), int(loss_cu[s + 1])
        term[s] = ell[a:b].mean() if aggregation == "seq_mean" else ell[a:b].sum()
    dterm = g / C_tok if aggregation == "seq_mean" else g
    return term, dterm, ell, kl, away


def token_norm_coef(coef, comp_len):
    """Weights for the token-level normalisation: the group's term is (1 / sum_j |o_j|) sum_i sum_t loss
    instead of (1/G) sum_i (1/|o_i|) sum_t loss, so coef_i is multiplied by G / sum_j |o_j|, the sum running
    over ALL G completions of the prompt (their lengths are known before pruning), kept or not.
    """
    coef = np.asarray(coef, dtype=np.float64)
    cl = np.asarray(comp_len, dtype=np.float64).reshape(coef.shape)
    G = coef.shape[1]
    return coef * (G / cl.sum(axis=1, keepdims=True))


def loss_fwd_bwd(H, W, ids, loss_pos, loss_cu, seq_adv, seq_coef, logp_old, logp_ref,
                 clip_lo: float = 0.2, clip_hi: float = 0.2, beta: float = 0.04,
                 ratio_level: str = "token", aggregation: str = "seq_mean") -> dict:
    """Loss L = sum_s coef_s * term_s, term_s = (1/C_s) sum_{n in s} loss_n  (= -J of Eq. 1, reweighted)
    or one of the variants of sequence_terms(), and its gradients w.r.t. H (rows at loss_pos; all
    other rows zero) and W.

    Reading: the rescaling weight multiplies the whole per-sequence term (surrogate
    and KL), and |o_i| is the number of completion tokens C_s.
    """
    H = np.asarray(H, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    loss_cu = np.asarray(loss_cu, dtype=np.int64)
    S = len(loss_cu) - 1
    N = int(loss_cu[-1])
    rows, y = _targets(ids, loss_pos, N)
    Hn = H[rows]
    Z = Hn @ W.T
    m = Z.max(axis=1)
    lse = m + np.log(np.exp(Z - m[:, None]).sum(axis=1))
    logp = Z[np.arange(N), y] - lse

    seq_loss, dterm, ell, kl, clipped = sequence_terms(logp, logp_old, logp_ref, loss_cu, seq_adv, clip_lo, clip_hi,
                                                       beta, ratio_level, aggregation)
    coef_tok = np.empty(N)
    for s in range(S):
        coef_tok[int(loss_cu[s]):int(loss_cu[s + 1])] = float(seq_coef[s])
    loss = float(np.sum(np.asarray(seq_coef, dtype=np.float64) * seq_loss))

    c = coef_tok * dterm                           # dL/dlogp[n]
    dZ = -np.exp(Z - lse[:, None]) * c[:, None]    # -c_n p[n,v]
    dZ[np.arange(N), y] += c                       # + c_n 1[v = y_n]
    dH = np.zeros_like(H)
    np.add.at(dH, rows, dZ @ W)
    dW = dZ.T @ Hn
    return dict(loss=loss, logp=logp, lse=lse, seq_loss=seq_loss, dH=dH, dW=dW, c=c,
                mean_kl=float(kl.mean()) if N else 0.0,
                clip_frac=float(clipped.mean()) if N else 0.0)
