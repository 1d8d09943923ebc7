#!/usr/bin/env python3
"""Writes tests/golden/uniform24.txt: a few hundred 24-bit rounding draws of the oracle
(the counter hash behind Eq. 4's "with probability"), over seeds, streams, wire rows and
columns.  Calls only oracle/.  The paper fixes no generator, so these values pin nothing
to the paper; they freeze the build's own choice, so that the draws cannot change again
without this file (and therefore a reviewed commit) changing with them.

    python tests/golden/make_uniform24.py
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402

SEEDS = [0, 1, 20230301, 0xABCDEF0123456789, 2**64 - 1, 2**32, 2**32 + 1]
STREAMS = [0, 1, 2, 7, 2**31, 2**32 - 1]
ROWS = [0, 1, 63, 64, 2_883_366, 2**31 - 1]
COLS = [0, 1, 63, 64, 255, 601, 65_535]


def cases():
    for si, seed in enumerate(SEEDS):
        for ti, stream in enumerate(STREAMS):
            for ri, row in enumerate(ROWS):
                for ci, col in enumerate(COLS):
                    # a thinned grid: every key varies against every other somewhere
                    if (si + 2 * ti + 3 * ri + 5 * ci) % 5 == 0:
                        yield seed, stream, row, col


def main():
    path = os.path.join(HERE, "uniform24.txt")
    with open(path, "w") as f:
        f.write("# 24-bit rounding draws of oracle.uniform24(seed, stream, wire row, column).\n")
        f.write("# Written by tests/golden/make_uniform24.py from oracle/ alone; not values of the paper\n")
        f.write("# (it names no generator): a freeze of this build's counter hash.\n")
        f.write("# seed stream row col draw\n")
        n = 0
        for seed, stream, row, col in cases():
            f.write(f"{seed} {stream} {row} {col} {oracle.uniform24(seed, stream, row, col)}\n")
            n += 1
    print(f"wrote {n} draws to {path}")


if __name__ == "__main__":
    main()
