#!/usr/bin/env python3
"""What one MI355X sustains on the inner loop of a 256 x 256 x 64 bf16 GEMM tile as the loop's
ingredients are added one at a time (registers only; + LDS fragment reads; + global->LDS tile
loads from the L2; + the GEMM's real address pattern), for the two bf16 MFMA shapes.

Runs the stand-alone program built from paper_2312_02515_amd/csrc/bench/mfma_ceiling.hip (built
by `python -c 'import __graft_entry__ as g; g.build()'`) and prints its markdown table: the
ceiling against which the base-product kernel's rate is read.  Hardware characterisation, no
part of the operator; bench.py is the benchmark proper.
"""
import argparse
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
BIN = os.path.join(ROOT, "paper_2312_02515_amd", "mfma_ceiling.bin")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--tiles", type=int, default=8000, help="contraction tiles per block and launch")
    ap.add_argument("--reps", type=int, default=4, help="launches per variant; the first is a warm-up")
    ap.add_argument("--verbose", action="store_true", help="also print every launch's rate")
    args = ap.parse_args()
    if not os.path.exists(BIN):
        sys.exit(f"{BIN} is missing: build first (python -c 'import __graft_entry__ as g; g.build()')")
    r = subprocess.run([BIN, str(args.tiles), str(max(args.reps, 2))], capture_output=True, text=True, timeout=600)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        sys.exit(r.returncode)
    for line in r.stdout.splitlines():
        if args.verbose or line.startswith("|"):
            print(line)


if __name__ == "__main__":
    main()
