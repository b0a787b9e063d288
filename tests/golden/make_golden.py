"""Writes tests/golden/c1_decode_oracle.txt: the oracle's fp64 output for the smallest workload
(batch 1, context 128, Hq 8, Hkv 2, head_dim 64, block_size 16, fp16, seed 0).

Calls only the input generator and the CPU oracle.  The stored numbers are a regression
anchor for the oracle and the generator together (a change to either shows up as a diff);
they are not taken from the paper, which prints no worked example.
Run from the repository root:  python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle as O          # noqa: E402
import workloads as W       # noqa: E402


def main():
    case = W.make_case(W.CONFIGS["C1"])
    kc, vc = case.k_cache.copy(), case.v_cache.copy()
    O.reshape_and_cache(case.k_new, case.v_new, kc, vc, case.slot_mapping)
    out = O.paged_attention(case.q, kc, vc, case.block_tables, case.context_lens, case.slopes,
                            case.scale, case.dtype)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_decode_oracle.txt")
    with open(path, "w") as f:
        f.write("# oracle fp64 output, workload C1 (seed 0): rows = query head, cols = first 8 dims\n")
        f.write("# block_table: " + " ".join(str(int(x)) for x in case.block_tables[0]) + "\n")
        for h in range(out.shape[1]):
            f.write(" ".join(f"{x:.17e}" for x in out[0, h, :8]) + "\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
