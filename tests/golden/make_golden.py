"""Writes tests/golden/tiny_decode_trace.txt from the CPU oracle alone (run from the repository root:
`python tests/golden/make_golden.py`).

The file freezes what the oracle decodes on the seeded `tiny` and `tiny_t123` workloads: the token that follows
the prompt, and for each of 16 steps the tree's tokens, the accepted path and the emitted tokens.  It is a
regression pin, not an independent one: a change to the oracle's arithmetic or to the seeded generators shows up
as a diff of this file and has to be justified by the passage of the paper it follows.  Nothing here reads the GPU
library.
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.join(HERE, "..", ".."))
sys.path.insert(0, os.path.join(HERE, ".."))

from ht_inputs import WORKLOADS                      # noqa: E402
from helpers import oracle_decoder, oracle_model, prompt_of   # noqa: E402

STEPS = 16
NAMES = ("tiny", "tiny_t123")


def trace_lines(name):
    wl = WORKLOADS[name]
    dec = oracle_decoder(wl, oracle_model(wl))
    prompt = prompt_of(wl)
    dec.prefill(prompt)
    lines = [f"workload {name} seed {wl.seed} prompt_len {len(prompt)} tree_size {wl.tree_size}",
             f"root {dec.root}"]
    for s in range(STEPS):
        res = dec.step()
        lines.append(f"step {s} tok " + " ".join(map(str, res["tok"])))
        lines.append(f"step {s} path " + " ".join(map(str, res["path"])))
        lines.append(f"step {s} emitted " + " ".join(map(str, res["emitted"])))
        lines.append(f"step {s} next_root {res['root']} cache_len {res['n']}")
    return lines


def main():
    out = ["# written by tests/golden/make_golden.py from oracle/ht_oracle.py (fp64) on the seeded inputs of ht_inputs/",
           "# one decode per workload: schedule of Sec. 3.2-3.4 (transfer, draft rows, candidates, tree, verify,",
           "# greedy acceptance, compaction), 16 steps"]
    for name in NAMES:
        out += trace_lines(name)
    with open(os.path.join(HERE, "tiny_decode_trace.txt"), "w") as f:
        f.write("\n".join(out) + "\n")


if __name__ == "__main__":
    main()
