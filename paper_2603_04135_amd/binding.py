"""ctypes binding of libdppo_hip.so: argument marshalling only.

Every function has the name and argument meaning of the C entry point it calls
(see include/dppo.h). PyTorch is used to hold device memory and to name the
current HIP stream; all arithmetic happens in the library's kernels. There is
no fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p
from typing import Optional

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdppo_hip.so")
_lib = None

EXPORTS = ["dppo_status_str", "dppo_last_error", "dppo_select", "dppo_pack", "dppo_gather_f32", "dppo_token_norm_coef", "dppo_variance_terms",
           "dppo_workspace_bytes", "dppo_workspace_min_bytes", "dppo_token_logprob", "dppo_loss_fwd_bwd",
           "dppo_timing_enable", "dppo_timing_read", "dppo_history_update", "dppo_token_logprob_noalloc",
           "dppo_static_scratch_bytes", "dppo_mfma_rate_probe", "dppo_timing_tile_phases"]
STAGES = ["logits_gemm", "grad_logits", "dh_gemm", "dw_gemm", "elementwise"]


class DppoError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str):
        super().__init__("%s failed: status %d (%s)" % (where, status, detail))
        self.status = status


class SelectParams(ctypes.Structure):
    _fields_ = [("Q", c_int32), ("G", c_int32), ("r_q", c_float), ("r_o", c_float),
                ("adv_eps", c_float), ("std_ddof", c_int32), ("bottom_frac", c_float),
                ("fixed_count", c_int32), ("realised_rate", c_int32)]


class PackParams(ctypes.Structure):
    _fields_ = [("n_items", c_int32), ("capacity", c_int32), ("n_win", c_int32), ("policy", c_int32)]


PACK_POLICIES = {"first_fit": 0, "best_fit": 1}


class HeadShape(ctypes.Structure):
    _fields_ = [("T", c_int64), ("N", c_int64), ("D", c_int32), ("V", c_int32), ("dtype", c_int32)]


class LossParams(ctypes.Structure):
    _fields_ = [("clip_lo", c_float), ("clip_hi", c_float), ("beta", c_float),
                ("accumulate_dW", c_int32), ("recompute_logits", c_int32),
                ("ratio_level", c_int32), ("aggregation", c_int32), ("max_seq_tokens", c_int32)]


HEAD_BAD_TARGET, HEAD_BAD_POSITION, HEAD_SEQ_TOO_LONG = 1, 2, 4     # bits of the LM-head calls' device status word
RATIO_LEVELS = {"token": 0, "sequence": 1}
AGGREGATIONS = {"seq_mean": 0, "token_sum": 1}


def library_path() -> str:
    return _LIB_PATH


def load():
    """Loads the shared library (raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("%s is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                           "(or paper_2603_04135_amd/build.py) first" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    lib.dppo_status_str.restype = c_char_p
    lib.dppo_status_str.argtypes = [c_int]
    lib.dppo_last_error.restype = c_char_p
    lib.dppo_last_error.argtypes = []
    lib.dppo_select.restype = c_int
    lib.dppo_select.argtypes = [POINTER(SelectParams)] + [c_void_p] * 15
    lib.dppo_variance_terms.restype = c_int
    lib.dppo_variance_terms.argtypes = [c_int32, c_int32] + [c_void_p] * 6
    lib.dppo_pack.restype = c_int
    lib.dppo_pack.argtypes = [POINTER(PackParams)] + [c_void_p] * 8 + [c_int64, c_void_p, c_void_p]
    lib.dppo_token_norm_coef.restype = c_int
    lib.dppo_token_norm_coef.argtypes = [c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.dppo_gather_f32.restype = c_int
    lib.dppo_gather_f32.argtypes = [c_int64, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.dppo_workspace_bytes.restype = c_size_t
    lib.dppo_workspace_bytes.argtypes = [POINTER(HeadShape), c_int]
    lib.dppo_workspace_min_bytes.restype = c_size_t
    lib.dppo_workspace_min_bytes.argtypes = [POINTER(HeadShape), c_int]
    lib.dppo_token_logprob.restype = c_int
    lib.dppo_token_logprob.argtypes = [POINTER(HeadShape)] + [c_void_p] * 8 + [c_size_t, c_void_p]
    lib.dppo_token_logprob_noalloc.restype = c_int
    lib.dppo_token_logprob_noalloc.argtypes = [POINTER(HeadShape)] + [c_void_p] * 8
    lib.dppo_static_scratch_bytes.restype = c_size_t
    lib.dppo_static_scratch_bytes.argtypes = []
    lib.dppo_timing_tile_phases.restype = c_int
    lib.dppo_timing_tile_phases.argtypes = [c_void_p]
    lib.dppo_mfma_rate_probe.restype = c_int
    lib.dppo_mfma_rate_probe.argtypes = [c_int, c_int, c_void_p, c_int32, POINTER(ctypes.c_double), c_void_p]
    lib.dppo_loss_fwd_bwd.restype = c_int
    lib.dppo_loss_fwd_bwd.argtypes = ([POINTER(HeadShape), POINTER(LossParams), c_int32] + [c_void_p] * 17
                                      + [c_size_t, c_void_p])
    lib.dppo_history_update.restype = c_int
    lib.dppo_history_update.argtypes = [c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_void_p]
    lib.dppo_timing_enable.restype = c_int
    lib.dppo_timing_enable.argtypes = [c_int]
    lib.dppo_timing_read.restype = c_int
    lib.dppo_timing_read.argtypes = [POINTER(ctypes.c_double), POINTER(c_int64), c_int]
    _lib = lib
    return lib


def _check(status: int, where: str):
    if status != 0:
        lib = load()
        raise DppoError(status, where, "%s: %s" % (lib.dppo_status_str(status).decode(),
                                                    lib.dppo_last_error().decode()))


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("the DPPO library takes device tensors only")
    if not t.is_contiguous():
        raise ValueError("tensors handed to the DPPO library must be contiguous")
    return c_void_p(t.data_ptr())


def _stream(device) -> c_void_p:
    return c_void_p(torch.cuda.current_stream(device).cuda_stream)


def _as(t, dtype, device):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor):
        t = torch.as_tensor(t)
    return t.to(device=device, dtype=dtype).contiguous()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return 0
    if t.dtype == torch.bfloat16:
        return 1
    raise ValueError("H and W must be float32 or bfloat16")


# --------------------------------------------------------------------------------------
def dppo_select(rewards, hist, u_prompt, u_comp, r_q: float, r_o: float, adv_eps: float = 1e-6,
                std_ddof: int = 1, bottom_frac: float = 0.5, fixed_count: bool = False,
                realised_rate: bool = True, device="cuda:0") -> dict:
    """rewards [Q,G]; hist/u_prompt [Q] or None; u_comp [Q,G] or None. Returns device tensors."""
    lib = load()
    rewards = _as(rewards, torch.float32, device)
    Q, G = rewards.shape
    hist = _as(hist, torch.float32, device)
    u_prompt = _as(u_prompt, torch.float32, device)
    u_comp = _as(u_comp, torch.float32, device)
    f32 = dict(dtype=torch.float32, device=device)
    out = dict(adv=torch.empty((Q, G), **f32), mean_abs_adv=torch.empty(Q, **f32),
               keep_prompt=torch.empty(Q, dtype=torch.uint8, device=device),
               keep_comp=torch.empty((Q, G), dtype=torch.uint8, device=device),
               gamma_q=torch.empty(Q, **f32), gamma_o=torch.empty((Q, G), **f32),
               coef=torch.empty((Q, G), **f32), counts=torch.empty(1 + Q, dtype=torch.int32, device=device),
               prune_q=torch.empty(Q, **f32), prune_o=torch.empty((Q, G), **f32))
    p = SelectParams(Q, G, r_q, r_o, adv_eps, std_ddof, bottom_frac, 1 if fixed_count else 0,
                     1 if realised_rate else 0)
    st = lib.dppo_select(ctypes.byref(p), _ptr(rewards), _ptr(hist), _ptr(u_prompt), _ptr(u_comp),
                         _ptr(out["adv"]), _ptr(out["mean_abs_adv"]), _ptr(out["keep_prompt"]),
                         _ptr(out["keep_comp"]), _ptr(out["gamma_q"]), _ptr(out["gamma_o"]), _ptr(out["coef"]),
                         _ptr(out["counts"]), _ptr(out["prune_q"]), _ptr(out["prune_o"]), _stream(device))
    _check(st, "dppo_select")
    return out


def dppo_variance_terms(g, prune_q, prune_o, device="cuda:0") -> dict:
    """g [Q,G], prune_q [Q], prune_o [Q,G] -> dict(group[Q,4], total[10]) of float64 device tensors (App. D)."""
    lib = load()
    g = _as(g, torch.float32, device)
    Q, G = g.shape
    prune_q = _as(prune_q, torch.float32, device)
    prune_o = _as(prune_o, torch.float32, device)
    group = torch.empty((Q, 4), dtype=torch.float64, device=device)
    total = torch.empty(10, dtype=torch.float64, device=device)
    _check(lib.dppo_variance_terms(Q, G, _ptr(g), _ptr(prune_q), _ptr(prune_o), _ptr(group), _ptr(total),
                                   _stream(device)), "dppo_variance_terms")
    return dict(group=group, total=total)


def dppo_history_update(hist_table: torch.Tensor, prompt_index, keep_prompt, mean_abs_adv) -> torch.Tensor:
    """Updates hist_table (float32 device tensor) in place and returns it."""
    lib = load()
    device = hist_table.device
    if hist_table.dtype != torch.float32:
        raise ValueError("hist_table must be float32")
    prompt_index = _as(prompt_index, torch.int32, device)
    keep_prompt = _as(keep_prompt, torch.uint8, device)
    mean_abs_adv = _as(mean_abs_adv, torch.float32, device)
    st = lib.dppo_history_update(prompt_index.numel(), _ptr(prompt_index), _ptr(keep_prompt), _ptr(mean_abs_adv),
                                 _ptr(hist_table), hist_table.numel(), _stream(device))
    _check(st, "dppo_history_update")
    return hist_table


def dppo_pack(prompt_len, comp_len, keep, capacity: int, n_win: int, loss_pos_capacity: Optional[int] = None,
              device="cuda:0", policy: str = "first_fit") -> dict:
    """prompt_len, comp_len [n_items] int32 (comp_len None: prompts alone); keep [n_items] uint8 or None;
    capacity 0 or None: the longest kept item.

    Returns device tensors sized for the worst case plus the host copy of meta
    (this is the one place the path synchronises: the caller needs T and N to size H)."""
    lib = load()
    prompt_len = _as(prompt_len, torch.int32, device)
    comp_len = _as(comp_len, torch.int32, device)
    keep = _as(keep, torch.uint8, device)
    n = prompt_len.numel()
    if loss_pos_capacity is None:
        loss_pos_capacity = 0 if comp_len is None else int(comp_len.clamp(min=0).sum().item())
    i32 = dict(dtype=torch.int32, device=device)
    order = torch.empty(n, **i32)
    row_ptr = torch.empty(n + 1, **i32)
    cu = torch.empty(n + 1, **i32)
    lcu = torch.empty(n + 1, **i32)
    loss_pos = torch.empty(max(1, loss_pos_capacity), **i32)
    meta = torch.zeros(8, **i32)
    p = PackParams(n, int(capacity or 0), n_win, PACK_POLICIES[policy])
    st = lib.dppo_pack(ctypes.byref(p), _ptr(prompt_len), _ptr(comp_len), _ptr(keep), _ptr(order), _ptr(row_ptr),
                       _ptr(cu), _ptr(lcu), _ptr(loss_pos), loss_pos_capacity, _ptr(meta), _stream(device))
    _check(st, "dppo_pack")
    meta_host = meta.cpu()
    m = meta_host.tolist()
    n_rows, T, N, dev_status, S, cap = m[0], m[1], m[2], m[3], m[4], m[5]
    density = float(meta_host[6:8].view(torch.float64)[0])     # the library's own number (a double in two words)
    return dict(order=order[:S], row_ptr=row_ptr[:n_rows + 1], cu_seqlens=cu[:S + 1], loss_cu=lcu[:S + 1],
                loss_pos=loss_pos[:N], n_rows=n_rows, T=T, N=N, S=S, device_status=dev_status, capacity=cap,
                density=density)


def dppo_token_norm_coef(coef: torch.Tensor, comp_len) -> torch.Tensor:
    """coef [Q,G] float32, comp_len [Q,G] int32 -> coef * G / (completion tokens of the group)."""
    lib = load()
    device = coef.device
    Q, G = coef.shape
    coef = _as(coef, torch.float32, device)
    comp_len = _as(comp_len, torch.int32, device)
    out = torch.empty_like(coef)
    _check(lib.dppo_token_norm_coef(Q, G, _ptr(comp_len), _ptr(coef), _ptr(out), _stream(device)),
           "dppo_token_norm_coef")
    return out


def dppo_gather_f32(idx: torch.Tensor, src: torch.Tensor) -> torch.Tensor:
    lib = load()
    device = src.device
    idx = _as(idx, torch.int32, device)
    src = _as(src.reshape(-1), torch.float32, device)
    dst = torch.empty(idx.numel(), dtype=torch.float32, device=device)
    _check(lib.dppo_gather_f32(idx.numel(), _ptr(idx), _ptr(src), _ptr(dst), _stream(device)), "dppo_gather_f32")
    return dst


def _shape(H, W, N) -> HeadShape:
    T, D = H.shape
    V, D2 = W.shape
    if D != D2 or H.dtype != W.dtype:
        raise ValueError("H [T,D] and W [V,D] must agree in D and dtype")
    return HeadShape(T, N, D, V, _dtype_code(H))


def dppo_workspace_bytes(T: int, N: int, D: int, V: int, dtype_code: int, want_backward) -> int:
    """want_backward: False / 0, True / 1, or 2 (backward with the sequence-level ratio and max_seq_tokens)."""
    shape = HeadShape(T, N, D, V, dtype_code)
    return int(load().dppo_workspace_bytes(ctypes.byref(shape), int(want_backward)))


def dppo_workspace_min_bytes(T: int, N: int, D: int, V: int, dtype_code: int, want_backward) -> int:
    shape = HeadShape(T, N, D, V, dtype_code)
    return int(load().dppo_workspace_min_bytes(ctypes.byref(shape), int(want_backward)))


def alloc_workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(256, nbytes), dtype=torch.uint8, device=device)


def dppo_token_logprob(H, W, ids, loss_pos=None, want_lse: bool = True, ws: Optional[torch.Tensor] = None,
                       status: Optional[torch.Tensor] = None):
    """Returns (logp[N], lse[N] or None) as float32 device tensors. status: optional int32[1] device
    tensor that receives the device-side status word (DPPO_HEAD_BAD_*)."""
    lib = load()
    device = H.device
    N = H.shape[0] if loss_pos is None else loss_pos.numel()
    shape = _shape(H, W, N)
    if ws is None:
        ws = alloc_workspace(lib.dppo_workspace_bytes(ctypes.byref(shape), 0), device)
    logp = torch.empty(N, dtype=torch.float32, device=device)
    lse = torch.empty(N, dtype=torch.float32, device=device) if want_lse else None
    st = lib.dppo_token_logprob(ctypes.byref(shape), _ptr(H), _ptr(W), _ptr(ids), _ptr(loss_pos), _ptr(logp),
                                _ptr(lse), _ptr(status), _ptr(ws), ws.numel(), _stream(device))
    _check(st, "dppo_token_logprob")
    return logp, lse


def dppo_token_logprob_noalloc(H, W, ids, loss_pos, logp: torch.Tensor, lse: Optional[torch.Tensor] = None,
                               status: Optional[torch.Tensor] = None) -> None:
    """dppo_token_logprob on the library's fixed scratch array: fills the caller's logp[N] (and lse[N]);
    this wrapper allocates nothing either."""
    lib = load()
    N = H.shape[0] if loss_pos is None else loss_pos.numel()
    shape = _shape(H, W, N)
    st = lib.dppo_token_logprob_noalloc(ctypes.byref(shape), _ptr(H), _ptr(W), _ptr(ids), _ptr(loss_pos), _ptr(logp),
                                        _ptr(lse), _ptr(status), _stream(H.device))
    _check(st, "dppo_token_logprob_noalloc")


def dppo_static_scratch_bytes() -> int:
    return int(load().dppo_static_scratch_bytes())


def dppo_loss_fwd_bwd(H, W, ids, loss_pos, loss_cu, seq_adv, seq_coef, logp_old, logp_ref,
                      clip_lo: float = 0.2, clip_hi: float = 0.2, beta: float = 0.04,
                      dW: Optional[torch.Tensor] = None, accumulate_dW: bool = False,
                      recompute_logits: bool = False, ws: Optional[torch.Tensor] = None,
                      dH: Optional[torch.Tensor] = None, out: Optional[dict] = None,
                      ratio_level: str = "token", aggregation: str = "seq_mean",
                      status: Optional[torch.Tensor] = None, max_seq_tokens: int = 0) -> dict:
    """Returns dict(loss[1], logp[N], seq_loss[S], stats[4], dH[T,D], dW[V,D]) of device tensors.
    status: optional int32[1] device tensor for the device-side status word (DPPO_HEAD_BAD_*)."""
    lib = load()
    device = H.device
    N = H.shape[0] if loss_pos is None else loss_pos.numel()
    S = loss_cu.numel() - 1
    shape = _shape(H, W, N)
    if ws is None:
        ws = alloc_workspace(lib.dppo_workspace_bytes(ctypes.byref(shape), 2 if max_seq_tokens > 0 else 1), device)
    f32 = dict(dtype=torch.float32, device=device)
    if out is None:
        out = dict(loss=torch.empty(1, **f32), logp=torch.empty(N, **f32), seq_loss=torch.empty(max(S, 1), **f32),
                   stats=torch.empty(4, **f32))
    if dH is None:
        dH = torch.empty_like(H)
    if dW is None:
        if accumulate_dW:
            raise ValueError("accumulate_dW needs the dW buffer to accumulate into")
        dW = torch.empty(W.shape, **f32)
    p = LossParams(clip_lo, clip_hi, beta, 1 if accumulate_dW else 0, 1 if recompute_logits else 0,
                   RATIO_LEVELS[ratio_level], AGGREGATIONS[aggregation], int(max_seq_tokens))
    st = lib.dppo_loss_fwd_bwd(ctypes.byref(shape), ctypes.byref(p), S, _ptr(H), _ptr(W), _ptr(ids), _ptr(loss_pos),
                               _ptr(loss_cu), _ptr(seq_adv), _ptr(seq_coef), _ptr(logp_old), _ptr(logp_ref),
                               _ptr(out["loss"]), _ptr(out["logp"]), _ptr(out["seq_loss"]), _ptr(out["stats"]),
                               _ptr(status), _ptr(dH), _ptr(dW), _ptr(ws), ws.numel(), _stream(device))
    _check(st, "dppo_loss_fwd_bwd")
    res = dict(out)
    res["seq_loss"] = out["seq_loss"][:S]
    res["dH"] = dH
    res["dW"] = dW
    return res


def dppo_mfma_rate_probe(random_operands: bool, iters: int, out: torch.Tensor) -> float:
    """Enqueues the register-only MFMA loop on the current stream; returns the flop enqueued (the caller times it)."""
    flop = ctypes.c_double(0.0)
    _check(load().dppo_mfma_rate_probe(1 if random_operands else 0, iters, _ptr(out), out.numel(), ctypes.byref(flop),
                                       _stream(out.device)), "dppo_mfma_rate_probe")
    return float(flop.value)


def dppo_timing_tile_phases(counters: Optional[torch.Tensor]) -> None:
    """counters: zeroed int64[12] device tensor (3 GEMM stages x {prologue, loop, epilogue cycles, workgroups}) or None."""
    if counters is not None and (counters.dtype != torch.int64 or counters.numel() < 12):
        raise ValueError("counters must be an int64 device tensor of at least 12 elements")
    _check(load().dppo_timing_tile_phases(_ptr(counters)), "dppo_timing_tile_phases")


def dppo_timing_enable(on: bool) -> None:
    _check(load().dppo_timing_enable(1 if on else 0), "dppo_timing_enable")


def dppo_timing_read(reset: bool = True) -> dict:
    """{stage: (milliseconds, launches)} summed since the last reset."""
    n = len(STAGES)
    ms = (ctypes.c_double * n)()
    cnt = (c_int64 * n)()
    _check(load().dppo_timing_read(ms, cnt, 1 if reset else 0), "dppo_timing_read")
    return {name: (float(ms[i]), int(cnt[i])) for i, name in enumerate(STAGES)}
