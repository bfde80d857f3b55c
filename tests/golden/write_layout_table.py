"""Writes layout_table.txt: chunk count and padding per (parameter set, chunk length, policy).

Calls only the oracle's planner and the synthetic shape lists.  Run from the repo root:
    python tests/golden/write_layout_table.py
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import elixir_oracle as orc  # noqa: E402
from synth import gen  # noqa: E402


def main():
    lines = ["# set chunk_elems policy n_chunks padding_elems"]
    for name, cfg in gen.CONFIGS.items():
        sizes = gen.SWEEP_CHUNK_ELEMS if name == "gpt2_1p5b" else [cfg.chunk_elems]
        for C in sizes:
            for pol in (orc.NEXT_FIT, orc.FIRST_FIT, orc.DENSE):
                _, _, valid = orc.layout_plan(cfg.numels(), C, pol)
                lines.append(f"{name} {C} {pol} {len(valid)} {len(valid) * C - sum(valid)}")
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "layout_table.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
