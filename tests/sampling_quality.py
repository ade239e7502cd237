"""How well does the sampled sparsity measure pick the queries the exact one would?

    python -m tests.sampling_quality [--workload conformer_s] [--c 1 5]

For each sampling factor c the keys of every query are re-drawn (U = ceil(c ln L)
uniform samples with replacement, seeded), the forward is run with u fixed by
--u-factor, and its index sets (step a2, from the sampled measure of Eq. 11) are
compared with the top-u of the exact measure of Eq. 10 computed by
`probsparse_exact_measure`.  Reported: mean and minimum over (batch, head) of
|I_sampled & I_exact| / u.  The paper lowers r_sample from 5 to 1 together with
index sharing (Sec. 4.4) without loss of accuracy; this shows what that costs
in selection quality on a given input.

A diagnostic that lives with the tests, not in the product package: both measures
come from the library's kernels, while the reference top-u of the exact measure is
taken here with a library sort (stable, ties to the lower index).
"""
from __future__ import annotations

import argparse
import json
import math

import torch

from paper_2106_09236_amd import binding as psa
from paper_2106_09236_amd import workloads as W


def exact_top_u(M_exact: torch.Tensor, lengths, u: torch.Tensor) -> list:
    """Index sets of the u_b largest exact measures per (b, h), ties to the lower index."""
    B, H, L = M_exact.shape
    out = []
    for b in range(B):
        n = L if lengths is None else int(lengths[b])
        order = torch.sort(M_exact[b, :, :n], dim=-1, descending=True, stable=True).indices
        out.append([set(order[h, :int(u[b])].tolist()) for h in range(H)])
    return out


def overlap_report(Q, K, V, lengths, c_values, u_factor: float = 5.0, seed: int = 0) -> dict:
    B, H, L, _ = Q.shape
    M_exact = psa.probsparse_exact_measure(Q, K, lengths)
    gen = torch.Generator(device="cpu").manual_seed(seed)
    n_of_b = torch.full((B,), L, dtype=torch.int64) if lengths is None else lengths.cpu().to(torch.int64)
    report = {}
    for c in c_values:
        U = max(1, min(L, math.ceil(c * math.log(L))))
        r = torch.rand((B, H, L, U), generator=gen)
        idx = (r * n_of_b.view(B, 1, 1, 1).clamp(min=1)).to(torch.int32).cuda()
        _, _, sel, u = psa.probsparse_attn_fwd_debug(Q, K, V, lengths, idx, u_factor)
        torch.cuda.synchronize()
        best = exact_top_u(M_exact, None if lengths is None else lengths.cpu(), u.cpu())
        sel, u = sel.cpu(), u.cpu()
        fr = []
        for b in range(B):
            ub = int(u[b])
            for h in range(H):
                if ub > 0:
                    fr.append(len(best[b][h] & set(sel[b, h, :ub].tolist())) / ub)
        report[f"c={c:g}"] = {"U": U, "mean_overlap": round(sum(fr) / max(1, len(fr)), 4),
                              "min_overlap": round(min(fr, default=1.0), 4)}
    return report


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="conformer_s")
    ap.add_argument("--c", type=float, nargs="+", default=[1.0, 5.0])
    ap.add_argument("--u-factor", type=float, default=5.0, help="c of u = ceil(c ln n), kept fixed")
    args = ap.parse_args()
    cfg = W.CONFIGS[args.workload]
    w = W.make_workload(cfg)

    def dev(a):
        x = torch.from_numpy(a)
        if cfg.dtype == "bf16":
            x = x.view(torch.int16).view(torch.bfloat16)
        return x.cuda()

    lengths = None if w.lengths is None else torch.from_numpy(w.lengths).cuda()
    rep = overlap_report(dev(w.Q), dev(w.K), dev(w.V), lengths, args.c, args.u_factor)
    print(json.dumps({"workload": cfg.name, "u_factor": args.u_factor, "overlap_with_exact_top_u": rep}))


if __name__ == "__main__":
    main()
