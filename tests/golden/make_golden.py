"""Writes the stored expected values under tests/golden/.

Calls only code under oracle/ (never the HIP path) and the seeded input generators.

  python tests/golden/make_golden.py            config0_enumeration.txt: the optimum of
      configuration 0 as the minimum over its 6^4 plans (paper section 3.3, problem
      formulation, Eq. 1 unrolled).
  python tests/golden/make_golden.py config4 [threads]
      config4_full_budget.txt: the serial oracle's results for all 16 instances of the
      stress configuration at their full budget (optimum, last strategy, plan, number of
      tied minima, checksums of the last layer's cost table and of the whole back-pointer
      table).  About two minutes and 5 GB of host memory per instance and thread.
Run from the repository root.
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle.bruteforce import brute_force  # noqa: E402
from paper_2211_13878_amd import workloads  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def config4(threads: int) -> None:
    """The oracle on every instance of configuration 4 at full size."""
    from concurrent.futures import ThreadPoolExecutor

    import oracle
    from oracle.checksum import table_checksum

    w = workloads.config(4)

    def one(b):
        r = oracle.solve(*w.instance(b), want_C_last=True, want_bp=True)
        line = (f"{b} {r.best_cost} {r.best_last} {r.n_tied} {table_checksum(r.C_last)} "
                f"{table_checksum(r.bp)} " + " ".join(str(int(s)) for s in r.plan))
        print(line, flush=True)
        return line

    with ThreadPoolExecutor(max_workers=threads) as ex:
        lines = list(ex.map(one, range(w.B)))
    with open(os.path.join(HERE, "config4_full_budget.txt"), "w") as f:
        f.write("# configuration 4 (16 instances, L=128, S=128, E=65536, seeds 4000 + instance) at full budget,\n")
        f.write("# from the serial CPU oracle (oracle/galv_oracle.c: paper section 3.3, Eq. 1 with the former\n")
        f.write("# layer's strategy in the state, lowest index on ties).  Checksums: oracle/checksum.py over\n")
        f.write("# C_last [E+1][S] and bp [L][E+1][S] in row-major order.\n")
        f.write("# instance cost last n_tied checksum_C_last checksum_bp plan[0..127]\n")
        f.write("\n".join(lines) + "\n")


if len(sys.argv) > 1 and sys.argv[1] == "config4":
    config4(int(sys.argv[2]) if len(sys.argv) > 2 else 4)
    sys.exit(0)

w = workloads.config(0)
cost, plan = brute_force(*w.instance(0))
out = os.path.join(HERE, "config0_enumeration.txt")
with open(out, "w") as f:
    f.write("# configuration 0 (1 instance, L=4, S=6, E=256, seed 0): cheapest admissible plan\n")
    f.write("# found by enumerating all 6^4 plans (paper section 3.3, Eq. 1 unrolled);\n")
    f.write("# ties resolved towards the plan that is smallest read from the last layer.\n")
    f.write(f"cost {cost}\n")
    f.write("plan " + " ".join(str(s) for s in plan) + "\n")
print(open(out).read())
