"""Shared helpers of the GPU parity tests: build one workload's inputs once, hand the same
arrays to the HIP library (through the binding) and to the CPU oracle."""
from __future__ import annotations

import numpy as np
import torch

import workloads as WL
from oracle import dppo_oracle as O


def to_np64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a float32 / bfloat16 tensor to float64 on the host."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def oracle_select_pack(rb: WL.RolloutBatch, n_win=None, first_epoch=False):
    wl = rb.wl
    sel = O.select(rb.rewards, None if first_epoch else rb.hist, None if first_epoch else rb.u_prompt,
                   rb.u_comp, wl.r_q, wl.r_o)
    pk = O.pack(rb.item_prompt_len, rb.item_comp_len, sel["keep_comp"].reshape(-1), wl.capacity,
                wl.n_win if n_win is None else n_win)
    return sel, pk


def truncate_pack(pk: dict, max_loss_tokens: int) -> dict:
    """A smaller batch: the first packed sequences up to exactly max_loss_tokens loss tokens
    (the last sequence's completion is cut short if needed, which is just another valid batch)."""
    if pk["N"] <= max_loss_tokens:
        return pk
    S = 0
    while pk["loss_cu"][S] < max_loss_tokens:
        S += 1
    N = int(max_loss_tokens)
    loss_cu = pk["loss_cu"][:S + 1].copy()
    loss_cu[S] = N
    loss_pos = pk["loss_pos"][:N]
    T = int(loss_pos[-1]) + 2                      # the last loss row needs its target token
    cu = pk["cu_seqlens"][:S + 1].copy()
    cu[S] = T
    return dict(order=pk["order"][:S], cu_seqlens=cu, loss_cu=loss_cu, loss_pos=loss_pos, T=T, N=N, S=S)


class HeadCase:
    """Inputs of the LM-head path for a (possibly truncated) packed batch, on host and device."""

    def __init__(self, wl: WL.Workload, pk: dict, sel: dict, seed: int, device="cuda:0", D=None, V=None,
                 logp_noise=None, dtype=None):
        import dataclasses
        if D is not None or V is not None or dtype is not None:
            wl = dataclasses.replace(wl, D=D or wl.D, V=V or wl.V, dtype=dtype or wl.dtype)
        self.wl, self.pk, self.device = wl, pk, device
        T = pk["T"]
        self.H = WL.make_hidden(wl, T, seed, device)
        self.W = WL.make_vocab_matrix(wl, seed, device)
        self.ids_np = WL.make_ids(wl, T, seed)
        self.ids = torch.as_tensor(self.ids_np, device=device)
        self.loss_pos = torch.as_tensor(pk["loss_pos"], device=device)
        self.loss_cu = torch.as_tensor(pk["loss_cu"], device=device)
        od = pk["order"]
        self.seq_adv_np = sel["adv"].reshape(-1)[od].astype(np.float32)
        self.seq_coef_np = sel["coef"].reshape(-1)[od].astype(np.float32)
        self.seq_adv = torch.as_tensor(self.seq_adv_np, device=device)
        self.seq_coef = torch.as_tensor(self.seq_coef_np, device=device)
        self.noise = wl.logp_noise if logp_noise is None else logp_noise
        self.seed = seed
        self._H64 = self._W64 = None

    def host64(self):
        if self._H64 is None:
            self._H64, self._W64 = to_np64(self.H), to_np64(self.W)
        return self._H64, self._W64

    def set_behaviour_logps(self, base: np.ndarray):
        """logp_old / logp_ref = base + noise, the same arrays for both sides."""
        self.logp_old_np = WL.perturb_logp(base, self.noise, self.seed, 0)
        self.logp_ref_np = WL.perturb_logp(base, self.noise, self.seed, 1)
        self.logp_old = torch.as_tensor(self.logp_old_np, device=self.device)
        self.logp_ref = torch.as_tensor(self.logp_ref_np, device=self.device)

    def oracle_logprob(self):
        H64, W64 = self.host64()
        return O.token_logprob(H64, W64, self.ids_np, self.pk["loss_pos"])

    def oracle_loss(self, **kw):
        H64, W64 = self.host64()
        wl = self.wl
        return O.loss_fwd_bwd(H64, W64, self.ids_np, self.pk["loss_pos"], self.pk["loss_cu"],
                              self.seq_adv_np, self.seq_coef_np, self.logp_old_np, self.logp_ref_np,
                              kw.get("clip_lo", wl.clip_eps), kw.get("clip_hi", wl.clip_eps),
                              kw.get("beta", wl.kl_beta), ratio_level=kw.get("ratio_level", "token"),
                              aggregation=kw.get("aggregation", "seq_mean"))


def rel_fro(a: np.ndarray, b: np.ndarray) -> float:
    """||a - b||_F / ||b||_F"""
    den = float(np.linalg.norm(b))
    return float(np.linalg.norm(a - b)) / (den if den > 0 else 1.0)
