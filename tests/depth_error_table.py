"""Logit error of the HIP library against BOTH K/V storage modes of the CPU oracle, by depth and cached positions.

Not a test (pytest does not collect it): a measurement script for the tolerance section of the design notes.
    python tests/depth_error_table.py llama7b:8,16,32 llama13b:40 --positions 12,48,192
For every cell: weights of the named workload cut to the given depth, a random prompt of the given length, one
cycle (k = 4 drafts with every second layer skipped, verify of 5 rows).  The library is driven with the tokens of
the oracle whose K/V storage parameter equals the library's cache type; the "exact" oracle (fp64 cache) is teacher-forced with
the same tokens.  Printed per cell and mode: the largest |logit error| over prompt, draft and verify rows, the
largest error in units of the bound 2e-2 + 1e-2 |ref|, and the number of elements over the bound.
"""
import argparse
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

from oracle import argmax_lowest  # noqa: E402
from synth import WORKLOADS, make_prompt, reduced_depth  # noqa: E402
from tests._parity import TOL, make_pair_gpu_generated  # noqa: E402


def cell(ctx, orcs, shape, prompt, k, mask):
    tol_a, tol_r = TOL[shape.dtype]
    P = len(prompt)
    res = {m: {"err": 0.0, "units": 0.0, "over": 0, "worst": ""} for m in orcs}

    def cmp(mode, got, ref, what):
        err = np.abs(np.asarray(got, np.float64) - ref)
        units = err / (tol_a + tol_r * np.abs(ref))
        r = res[mode]
        if units.max() > r["units"]:
            r["units"], r["worst"] = float(units.max()), what
        r["err"] = max(r["err"], float(err.max()))
        r["over"] += int((units > 1.0).sum())

    print("  [cell: prompt %d ...]" % len(prompt), file=sys.stderr, flush=True)
    ctx.ssd_reset()
    g_first = ctx.ssd_prefill(prompt)
    zp = ctx.ssd_copy_logits(0, 1)[0]
    pend = {}
    for m, orc in orcs.items():
        for a in range(0, P, 16):     # the prompt in pieces (the cache makes this the same computation): progress lines
            z = orc.forward(prompt[a:a + 16], a)["logits"][-1]
            print("  [oracle %s: prompt rows %d/%d]" % (m, min(a + 16, P), P), file=sys.stderr, flush=True)
        cmp(m, zp, z, "prompt")
        pend[m] = argmax_lowest(z)
    drive = "cache" if "cache" in orcs else "exact"
    if g_first != pend[drive]:        # near-tie at the prompt's last row: the two sides would decode different tokens
        for m in res:
            res[m]["worst"] += " (first token differs: prompt row only)"
        return res
    # drafts: tokens of the driving oracle, every mode fed the same ones
    toks = [pend[drive]]
    zd = {m: [] for m in orcs}
    for i in range(k):
        for m, orc in orcs.items():
            zd[m].append(orc.forward([toks[i]], P + i, skip_mask=mask)["logits"][0])
        toks.append(argmax_lowest(zd[drive][i]))
    dg = ctx.ssd_draft_step(mask, k)
    zg = ctx.ssd_copy_logits(0, k)
    ok_rows = 1
    while ok_rows < k and dg[ok_rows - 1] == toks[ok_rows]:
        ok_rows += 1                          # later rows saw the same inputs only while the tokens agree
    for m in orcs:
        for i in range(ok_rows):
            cmp(m, zg[i], zd[m][i], "draft %d" % i)
    ctx.ssd_verify(toks[1:])
    zv = ctx.ssd_copy_logits(0, k + 1)
    for m, orc in orcs.items():
        ref = orc.forward(toks, P)["logits"]
        for j in range(k + 1):
            cmp(m, zv[j], ref[j], "verify %d" % j)
    ctx.ssd_force_commit(toks[1:], 0, toks[1])
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("cells", nargs="+", help="workload:depth[,depth...]")
    ap.add_argument("--positions", default="12,48,192")
    ap.add_argument("--kv", default=None, help="cache type of the library context: bf16, fp16 or fp32 (default: the binding's)")
    ap.add_argument("--modes", default="cache,exact", help="oracle K/V storage modes to compare with (cache = the context's type)")
    args = ap.parse_args()
    positions = [int(x) for x in args.positions.split(",")]
    print("cache type:", args.kv or "default", flush=True)
    print("| shape | layers | positions | max err vs same-storage oracle (units of bound, over) | max err vs exact-cache oracle "
          "(units of bound, over) | worst row (same storage / exact) | s |", flush=True)
    print("|---|---|---|---|---|---|---|", flush=True)
    for spec in args.cells:
        name, depths = spec.split(":")
        wl = WORKLOADS[name]
        for L in (int(x) for x in depths.split(",")):
            shape = wl.shape if L == wl.shape.n_layers else reduced_depth(wl.shape, L)
            orcs, ctx = make_pair_gpu_generated(shape, wl.seed, max(positions) + 16, max_k=4, kv_storage=tuple(args.modes.split(",")),
                                                 **({"kv_dtype": args.kv} if args.kv else {}))
            mask = np.zeros(L, np.uint8)
            mask[1:L - 1:2] = 1
            for P in positions:
                t0 = time.time()
                prompt = make_prompt(shape.vocab, P, wl.seed).tolist()
                r = cell(ctx, orcs, shape, prompt, 4, mask)
                na = {"err": float("nan"), "units": float("nan"), "over": -1, "worst": "-"}
                rc, re_ = r.get("cache", na), r.get("exact", na)
                print("| %s | %d | %d | %.2e (%.2f, %d) | %.2e (%.2f, %d) | %s / %s | %.0f |" % (
                    name, L, P, rc["err"], rc["units"], rc["over"], re_["err"], re_["units"], re_["over"], rc["worst"],
                    re_["worst"], time.time() - t0), flush=True)
            ctx.close()
            for o in orcs.values():
                o.close()
            del ctx, orcs
            import torch
            torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
