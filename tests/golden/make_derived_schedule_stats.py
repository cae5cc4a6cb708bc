"""Rewrites derived_schedule_stats.json from the CPU oracle alone.
Run from the repository root: python tests/golden/make_derived_schedule_stats.py"""
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
from oracle import schedule as S  # noqa: E402

CASES = [(4, 2, 1, 4), (6, 3, 3, 8), (4, 2, 1, 8), (8, 3, 7, 8), (16, 4, 8, 16)]
KEYS = ("max_mismatch", "max_inflight", "max_inflight_per_pipeline", "max_live_versions", "mismatched")

path = os.path.join(HERE, "derived_schedule_stats.json")
doc = json.load(open(path))
doc["cases"] = []
for d, P, i, T in CASES:
    st = S.stats(S.generate(d, P, i, T, 3 * T), T)
    doc["cases"].append({"d": d, "P": P, "i": i, "T": T, "M": 3 * T, **{k: st[k] for k in KEYS}})
json.dump(doc, open(path, "w"), indent=1)
print("wrote", path)
