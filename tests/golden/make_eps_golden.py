"""Writes tests/golden/eps_draw_seed42.txt from the CPU oracle (and from nothing else): a frozen
sample of the eps draw's definition, so that a later change to the generator, the counter layout or
the Box-Muller mapping cannot go unnoticed.  Run from the repository root:
    python tests/golden/make_eps_golden.py
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402

SEED, STEP, FIRST, N, S, COL0 = 42, 3, 5, 8, 2, 4 * ((1 << 32) + 1) - 4

out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "eps_draw_seed42.txt")
bits = oracle.eps_bits(N, S, SEED, STEP, FIRST, col0=COL0)
eps = oracle.eps_normal(N, S, SEED, STEP, FIRST, col0=COL0)
with open(out, "w") as f:
    f.write("# eps draw of oracle/eps_oracle.c: Philox-4x32-10 words and Box-Muller normals for\n")
    f.write(f"# seed={SEED} step={STEP} first_sample={FIRST} weights {COL0}..{COL0 + N - 1} (the quads straddle 2^32), {S} samples\n")
    f.write("# written by tests/golden/make_eps_golden.py, which calls only the oracle\n")
    f.write("# columns: sample weight word(hex) eps(%.17g)\n")
    for s in range(S):
        for i in range(N):
            f.write(f"{s} {COL0 + i} {int(bits[s, i]):08x} {eps[s, i]:.17g}\n")
print(out)
