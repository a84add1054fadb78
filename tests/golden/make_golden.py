"""Writes the stored expected values under tests/golden/ from the CPU oracle alone.

Run from the repo root:  python tests/golden/make_golden.py
Nothing here touches the HIP library.  The paper prints no worked numeric
example, so these fixtures are oracle outputs on the seeded benchmark
workloads (Methods, "Assigning Memory Budgets to KV-Caches": one budget per
KV cache), kept so that the host allocator of the library can be compared
against fixed text instead of a live call.
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import baklava_oracle as O            # noqa: E402
from paper_2502_13176_amd import synth            # noqa: E402


def main():
    for name in synth.WORKLOAD_ORDER:
        w = synth.WORKLOADS[name]
        b = synth.budgets_for(w, O.alloc_proportional)
        path = os.path.join(HERE, f"budgets_{name}.txt")
        with open(path, "w") as f:
            f.write(f"# per-(layer, KV head) token budgets, layer-major; workload {name}; "
                    f"sum {sum(b)}; written by make_golden.py from oracle.alloc_proportional\n")
            f.write("\n".join(str(x) for x in b) + "\n")
        print(path, len(b), sum(b), min(b), max(b))


if __name__ == "__main__":
    main()
