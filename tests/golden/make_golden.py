"""Writes tests/golden/config1_oracle.json: loss, lse, argmax and a few gradient entries of the
tiny DPR-style workload (config 1), computed by the fp64 oracle ONLY (never by the HIP path).

The paper prints no worked numerical example, so this fixture is not a pin of the oracle; it
freezes the oracle's output on the seeded config-1 inputs so that a later change of the oracle
or of the input generator shows up as a diff.

    python tests/golden/make_golden.py
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import gc_oracle as O  # noqa: E402
from paper_2101_06983_amd import synth  # noqa: E402


def main():
    q, p, r = (synth.widen(t) for t in synth.config1())
    out = O.loss_and_rep_grad(q, p, r)
    rec = {
        "source": "oracle/gc_oracle.py on paper_2101_06983_amd.synth.config1() (Eq. 1, 4-7); written by tests/golden/make_golden.py",
        "loss": out["loss"],
        "lse": out["lse"].tolist(),
        "argmax": out["argmax"].tolist(),
        "dq_row0": out["dq"][0].tolist(),
        "dp_row0": out["dp"][0].tolist(),
        "dp_row1": out["dp"][1].tolist(),
    }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config1_oracle.json")
    with open(path, "w") as f:
        json.dump(rec, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
