"""Writes tests/golden/plan_vectors.json from the CPU oracle only.

The paper does not fix the pseudo-random generator (Sec. 3.1 only asks for the same seed
on every worker), so these vectors pin this build's hash convention, not the paper: they
guard the oracle against accidental change and give the GPU generator exact targets.
Run:  python tests/golden/make_plan_vectors.py
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402

CASES = [
    # (seed, n, m, iter)
    (0, 4, 2, 0), (0, 4, 2, 1), (0, 4, 2, 2), (0, 4, 2, 3), (0, 4, 2, 4),
    (0, 16, 4, 0), (0, 16, 4, 1), (0, 16, 4, 7), (0, 16, 4, 2 ** 32 - 1), (0, 16, 4, 2 ** 32),
    (0, 16, 4, 2 ** 40 + 3), (1, 16, 4, 0), (2 ** 63 + 5, 16, 4, 9),
    (0, 8, 2, 0), (0, 8, 4, 5), (0, 32, 4, 3), (0, 64, 8, 0), (0, 64, 64, 1), (0, 64, 1, 2),
    (7, 63, 9, 11), (0, 1, 1, 0),
]


def main():
    out = []
    for seed, n, m, it in CASES:
        p = oracle.plan(n, m, it, seed=seed)
        out.append({"seed": seed, "n": n, "group_size": m, "iter": it,
                    "keys": [int(k) for k in p["keys"]],
                    "rank": [int(r) for r in p["rank"]],
                    "group_of": [int(g) for g in p["group_of"]],
                    "members": [[int(w) for w in row] for row in p["members"]]})
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "plan_vectors.json")
    with open(path, "w") as f:
        json.dump({"_source": "written by make_plan_vectors.py from oracle/ only", "cases": out},
                  f, indent=0)
    print("wrote", path, len(out), "cases")


if __name__ == "__main__":
    main()
