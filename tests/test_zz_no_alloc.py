"""The entry point that allocates nothing (dppo_token_logprob_noalloc, through the C ABI) against
dppo_token_logprob with a caller workspace: two calls in a row on the same fixed scratch array, the
second with a smaller input, then a shape the array cannot serve."""
import numpy as np
import pytest
import torch

import workloads as WL
from harness import HeadCase, oracle_select_pack, truncate_pack

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(name, tokens, **over):
    rb = WL.make_rollout(name)
    sel, pk = oracle_select_pack(rb)
    return HeadCase(rb.wl, truncate_pack(pk, tokens), sel, rb.seed, DEV, **over)


def test_noalloc_entry_matches_workspace_entry():
    import paper_2603_04135_amd as P
    P.load()
    assert torch.cuda.is_available(), "this test needs the GPU"
    assert P.dppo_static_scratch_bytes() == 64 << 20
    # first call: 20 000 tokens of the small workload (the fixed array serves them in several chunks,
    # the recommended workspace in one); second call: a smaller batch of another shape, which
    # reuses the array as the first call left it
    for name, tokens, over in (("small", 20000, {}), ("tiny", None, dict(dtype="bf16", D=128, V=1000))):
        case = _case(name, tokens if tokens else 10 ** 9, **over)
        N = case.pk["N"]
        ref_logp, ref_lse = P.dppo_token_logprob(case.H, case.W, case.ids, case.loss_pos)
        logp = torch.full((N,), float("nan"), device=DEV)
        lse = torch.full((N,), float("nan"), device=DEV)
        status = torch.full((1,), 9, dtype=torch.int32, device=DEV)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated(DEV)
        P.dppo_token_logprob_noalloc(case.H, case.W, case.ids, case.loss_pos, logp, lse, status)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated(DEV) == before
        assert int(status.item()) == 0
        # same kernels on the same token columns: the chunking does not enter a token's arithmetic
        assert torch.equal(logp, ref_logp) and torch.equal(lse, ref_lse)
        o_logp, o_lse = case.oracle_logprob()
        assert np.abs(logp.cpu().numpy() - o_logp).max() <= 2e-3 and np.abs(lse.cpu().numpy() - o_lse).max() <= 2e-3
    # a shape whose smallest chunk exceeds the array is refused, nothing is launched
    D, V = 128 * 1024, 300000
    H = torch.zeros((4, D), dtype=torch.bfloat16, device=DEV)
    W = torch.zeros((8, D), dtype=torch.bfloat16, device=DEV)     # never read: the shape below claims V rows
    ids = torch.zeros(4, dtype=torch.int32, device=DEV)
    import ctypes
    from paper_2603_04135_amd.binding import HeadShape
    lib = P.load()
    hs = HeadShape(4, 4, D, V, 1)
    out = torch.zeros(4, device=DEV)
    rc = lib.dppo_token_logprob_noalloc(ctypes.byref(hs), ctypes.c_void_p(H.data_ptr()), ctypes.c_void_p(W.data_ptr()),
                                        ctypes.c_void_p(ids.data_ptr()), None, ctypes.c_void_p(out.data_ptr()), None,
                                        None, None)
    assert rc == 4 and b"fixed" in lib.dppo_last_error()
