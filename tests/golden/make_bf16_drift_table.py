#!/usr/bin/env python3
"""Writes tests/golden/bf16_drift_7b.json: the deviation between correct bf16 evaluations of the 7B-width decoder
as a function of depth, from which the parity tests of deep bf16 models take their tolerances
(tests/bf16_drift.py: what is measured and why).  CPU only; calls the oracle and the fp32 evaluation in
tests/bf16_drift.py, never the HIP library.  About a quarter of an hour on 8 cores.

    python tests/golden/make_bf16_drift_table.py [--layers 32] [--envs 4] [--seed 0]
"""
import argparse
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(HERE))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import bf16_drift as bd  # noqa: E402


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--envs", type=int, default=4)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    rows = bd.drift_by_depth(args.layers, args.envs, seed=args.seed,
                             progress=lambda r: print(f"depth {r['depth']:2d}: logits rms ops {r['ops']['logits_rms']:.4f} "
                                                      f"exact {r['exact']['logits_rms']:.4f} impl {r['impl']['logits_rms']:.4f}",
                                                      flush=True))
    out = {"what": "deviation between bf16 evaluations of the 7B-width decoder (hidden 4096, 32 heads, ffn 11008) on the "
                   "recompute workload's rows (288-row prefix + 6 stored tokens), by depth; see tests/bf16_drift.py",
           "made_by": "tests/golden/make_bf16_drift_table.py", "envs": args.envs, "seed": args.seed,
           "k_chunks_of_second_fp32_evaluation": 4, "depths": rows}
    with open(bd.TABLE, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", bd.TABLE)


if __name__ == "__main__":
    main()
