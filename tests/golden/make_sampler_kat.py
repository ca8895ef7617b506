"""Writes tests/golden/sampler_kat.json: a few kernels drawn by the oracle's
sampler, stored as integers and fp32 bit patterns.  Calls only oracle/."""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
import oracle  # noqa: E402

CASES = [(0, 4, 1, 512), (1, 4, 20, 50000), (2004, 3, 20, 200000), (2**63 + 5, 3, 3, 11)]


def main():
    cases = []
    for seed, K, C, L in CASES:
        kr = oracle.sample_kernels(seed, K, C, L)
        case = {"seed": seed, "K": K, "C": C, "L": L}
        for name in ("length", "dilation", "padding", "n_ch", "channels"):
            case[name] = kr[name].tolist()
        case["bias_bits"] = kr["bias"].view(np.uint32).tolist()
        case["weight_bits"] = kr["weights"].view(np.uint32).tolist()
        cases.append(case)
    with open(os.path.join(HERE, "sampler_kat.json"), "w") as f:
        json.dump({"cases": cases}, f, indent=0)
        f.write("\n")


if __name__ == "__main__":
    main()
