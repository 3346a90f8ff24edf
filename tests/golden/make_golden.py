"""Writes tests/golden/config0_enumeration.txt.

Calls only the enumeration of all plans under oracle/ (never the HIP path):
the stored optimum of configuration 0 is the minimum over its 6^4 plans as
defined in paper section 3.3 (problem formulation, Eq. 1 unrolled).
Run from the repository root:  python tests/golden/make_golden.py
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle.bruteforce import brute_force  # noqa: E402
from paper_2211_13878_amd import workloads  # noqa: E402

w = workloads.config(0)
cost, plan = brute_force(*w.instance(0))
out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config0_enumeration.txt")
with open(out, "w") as f:
    f.write("# configuration 0 (1 instance, L=4, S=6, E=256, seed 0): cheapest admissible plan\n")
    f.write("# found by enumerating all 6^4 plans (paper section 3.3, Eq. 1 unrolled);\n")
    f.write("# ties resolved towards the plan that is smallest read from the last layer.\n")
    f.write(f"cost {cost}\n")
    f.write("plan " + " ".join(str(s) for s in plan) + "\n")
print(open(out).read())
