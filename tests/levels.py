"""Reader for the hand-built level fixtures under tests/golden/."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
CHARS = {
    "binary": {".": 0, "#": 1},
    "maze": {".": 0, "#": 1, "P": 2, "D": 3},
    "dungeon": {".": 0, "#": 1, "P": 2, "K": 3, "D": 4, "E": 5, "C": 6},
}
PROBLEM_ID = {"binary": 0, "maze": 1, "dungeon": 2}


def load(name):
    """-> (problem name, tiles int8 [h, w], {metric name: expected value})."""
    problem, expect, rows, in_level = None, {}, [], False
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.rstrip("\n")
            if in_level:
                if line.strip():
                    rows.append(line.strip())
                continue
            if line.startswith("#") or not line.strip():
                continue
            key, _, val = line.partition(":")
            if key == "problem":
                problem = val.strip()
            elif key == "expect":
                for kv in val.split():
                    k, _, v = kv.partition("=")
                    expect[k] = int(v)
            elif key == "level":
                in_level = True
    tiles = np.array([[CHARS[problem][c] for c in r] for r in rows], np.int8)
    return problem, tiles, expect


def all_fixtures():
    return sorted(f for f in os.listdir(GOLDEN) if f.endswith(".txt"))
