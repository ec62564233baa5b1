"""Writes tests/golden/nf_tables.txt from the CPU oracle only (no GPU code is involved).

The paper gives the NormalFloat recipe (Section 4.2) but prints no table values, so
these stored bit patterns are a regression guard for the oracle, not an external pin;
the external pins (forward Gaussian CDF, invariants) live in tests/test_oracle_pins.py.

Run:  python tests/golden/make_golden.py
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import lutq_oracle as orc  # noqa: E402


def main():
    lines = ["# NormalFloat-b tables (Section 4.2 recipe) as 16-bit patterns, written by make_golden.py",
             "# name dtype entries..."]
    for bits in (2, 3, 4):
        for dtype in ("f16", "bf16"):
            vals = orc.from_f64(orc.nf_table(bits), dtype)
            lines.append(" ".join([f"NF{bits}", dtype] + [f"{int(v):04x}" for v in vals]))
    with open(os.path.join(HERE, "nf_tables.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
