"""The experiment behind the paper's Table 1, on the GPU path: the mean squared error of
m / (sqrt(v) + eps) when the two moments are stored in each of the sixteen (format, expansion)
combinations -- E4M3 or E5M2, with or without the dynamic range expansion, per moment.

The paper measures real optimizer states of a training run; those are not available, so the
moments here are synthetic (synth_inputs.torch_moments: widely different scales across groups,
small dynamic range inside a group).  The VALUES therefore differ from the paper's; what carries
over is the structure: expansion lowers the error for either format and either moment, the best
cells have E4M3+Expand for the first moment and an expanded second moment (whose format then
hardly matters, in the paper too), and plain E5M2 for the first moment is the worst row.  Every quantize / dequantize runs in the HIP kernels
through the C ABI (coat_quant_group, coat_dequant_group); torch only forms the ratio and the mean.

    python table1_experiment.py [--n 16777216] [--group-size 128] [--seed 0]
"""
from __future__ import annotations

import argparse
import json
import os
import sys

CELLS = (("E4M3", False, False), ("E4M3+Expand", False, True), ("E5M2", True, False), ("E5M2+Expand", True, True))


def table1(n: int, G: int, seed: int, eps: float = 1e-8):
    """-> (labels, 4 x 4 list of MSE values: rows = first moment, columns = second moment)."""
    import torch
    import paper_2410_19313_amd as C
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    import synth_inputs as S

    dev = torch.device("cuda:0")
    gen = S.torch_generator(dev, seed)
    m, v = S.torch_moments(n, dev, gen, G=G)
    exact = m.double() / (v.double().sqrt() + eps)

    def through_fp8(x, e5m2, expand):
        q, scale, k = C.coat_quant_group(x, G, expand=expand, e5m2=e5m2)
        return C.coat_dequant_group(q, scale, k, G, e5m2=e5m2)

    m_hat = [through_fp8(m, e5, ex) for _, e5, ex in CELLS]
    v_hat = [through_fp8(v, e5, ex) for _, e5, ex in CELLS]
    rows = []
    for mh in m_hat:
        rows.append([float(((mh.double() / (vh.double().sqrt() + eps) - exact) ** 2).mean().item()) for vh in v_hat])
    return [c[0] for c in CELLS], rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=1 << 24)
    ap.add_argument("--group-size", type=int, default=128)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    labels, rows = table1(args.n, args.group_size, args.seed)
    scale = 1.0 / min(min(r) for r in rows)
    print("MSE of m/(sqrt(v)+eps), synthetic moments, n=%d, G=%d (relative to the best cell)" % (args.n, args.group_size))
    print("%-14s" % "first \\ second" + "".join("%14s" % l for l in labels))
    for l, r in zip(labels, rows):
        print("%-14s" % l + "".join("%14.3f" % (x * scale) for x in r))
    print(json.dumps({"labels": labels, "mse": rows}))


if __name__ == "__main__":
    main()
