"""Writes tests/golden/depth_mask_seeded.json: for a few (T, n_drop, seed) the generator words of
the steps and the set of dropped steps, the latter listed from the words by the rule of the
seeded depth subset (Sec. 3.4 depth pruning with a seeded set of depths): the n_drop steps with
the smallest (word, step).  Calls only the oracle's generator, not its mask function; the
selection below is a plain repeated minimum so that it shares nothing with the function it pins.

Run from the repository root: python tests/golden/make_depth_mask_golden.py
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import philox  # noqa: E402

cases = []
for T, n_drop, seed in ((20, 4, 42), (16, 4, 42), (8, 2, 42), (20, 7, 1223627), (5, 5, 1), (6, 0, 9)):
    words = [int(philox.words(seed, 0, i, philox.TAG_DEPTH, 1)[0, 0]) for i in range(T)]
    left = list(range(T))
    dropped = []
    for _ in range(n_drop):                       # repeated minimum over (word, step)
        best = left[0]
        for i in left[1:]:
            if words[i] < words[best] or (words[i] == words[best] and i < best):
                best = i
        dropped.append(best)
        left.remove(best)
    cases.append(dict(T=T, n_drop=n_drop, seed=seed, words=words, dropped=sorted(dropped)))

with open(os.path.join(ROOT, "tests", "golden", "depth_mask_seeded.json"), "w") as f:
    json.dump(dict(note="generator word 0 of counter (0, 0, step, depth tag) per step, and the n_drop steps "
                        "with the smallest (word, step); written by make_depth_mask_golden.py from oracle/philox",
                   cases=cases), f, indent=1)
print("wrote %d cases" % len(cases))
