"""The entry point that allocates nothing (probsparse_attn_fwd_static: scratch in the library's own
static device array) against probsparse_attn_fwd on a caller-owned workspace, through the C ABI.

Two calls in a row on the one array, the second on a smaller input: the array keeps the first
call's contents, and the second call must not be disturbed by them.  The two entry points run the
same kernels in the same fixed merge order, so their outputs must agree bit for bit (the bar for
the floating-point outputs is the parity tolerance; equality is what is checked and expected).
"""
import numpy as np
import pytest
import torch

from paper_2106_09236_amd import binding as psa
from paper_2106_09236_amd import workloads as W
from tests import parity

pytestmark = pytest.mark.gpu


def _device(w):
    def t(a):
        x = torch.from_numpy(a)
        if w.cfg.dtype == "bf16":
            x = x.view(torch.int16).view(torch.bfloat16)
        return x.cuda()
    lengths = None if w.lengths is None else torch.from_numpy(w.lengths).cuda()
    return t(w.Q), t(w.K), t(w.V), lengths, torch.from_numpy(w.sample_idx).cuda()


def _both(w):
    Q, K, V, lengths, idx = _device(w)
    ref = psa.probsparse_attn_fwd(Q, K, V, lengths, idx, w.cfg.c)
    out = torch.full_like(Q, float("nan"))
    before = torch.cuda.memory_allocated()
    psa.probsparse_attn_fwd_static(Q, K, V, lengths, idx, w.cfg.c, out)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), ref.float().cpu().numpy()


@pytest.mark.parametrize("first,second", [
    (W.CONFIGS["conformer_s"], W.CONFIGS["tiny"]),                                        # float32, ticket hand-over
    (W.small_config("a", 3, 4, 2300, 40, 5.0, "bf16", "mixture", True, 1100, 2300),     # select kernel, merge kernel
     W.small_config("b", 2, 2, 333, 30, 5.0, "bf16", "peaky", True, 20, 333)),
])
def test_static_scratch_matches_workspace_call(first, second):
    assert psa.load().probsparse_static_workspace_bytes() == 16 << 20
    for cfg in (first, second):                      # the second, smaller call finds the first one's leftovers
        w = W.make_workload(cfg, seed=4242 + cfg.L)
        got, ref = _both(w)
        assert not np.isnan(got).any()
        err = parity.output_error(got, ref)
        assert err <= parity.OUT_TOL[cfg.dtype], f"{cfg.name}: {err}"
        assert np.array_equal(got, ref), f"{cfg.name}: not bit-identical (error {err})"


def test_static_scratch_rejects_large_shapes():
    # needs more than the 16 MiB array: refused before anything is enqueued
    Q = torch.zeros((1, 1, 8, 64), device="cuda")
    idx = torch.zeros((1, 1, 8, 4), dtype=torch.int32, device="cuda")
    big = psa.make_shape(512, 8, 4096, 40, psa.PSA_BF16)
    assert psa.workspace_bytes(big, 5.0) > (16 << 20)
    rc = psa.load().probsparse_attn_fwd_static(Q.data_ptr(), Q.data_ptr(), Q.data_ptr(), None, idx.data_ptr(), 5.0,
                                               Q.data_ptr(), __import__("ctypes").byref(big), None)
    assert rc == -5
