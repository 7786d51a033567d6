"""Communication loads of the schemes the paper compares (Definition 1:
scheduled bits over J*Q*T), taken from the library's own plans.

    python -m paper_1805_01993_amd.loads K r Q N [T]

prints the table of the remark after the K = 4 example for any (K, r, Q, N):
compressed CDC (the paper's J-job schedule), the single-job schedule used by
the workloads, compression only (appendix) and the CDC-only formula of Sec. III
(the paper gives that scheme's load, not its construction).
Host-side only: no GPU is needed.
"""
from __future__ import annotations

import sys
from fractions import Fraction

from . import binding as B


def _load(plan, T):
    plan.bind(T, "u32")
    return Fraction(plan.scheduled_elems, plan.J * plan.Q * T)


def comparison(K, r, Q, N, T=None):
    """dict name -> Fraction load (None where N does not fit that scheme's batches)."""
    T = T or 4 * r * 8                      # any T with 4r | c*T makes the split exact
    out = {}
    for name, ctor in (("compressed CDC (Theorem 1, J jobs)", lambda: B.ccdc_plan_jobs(K, r, Q, N)),
                       ("compressed CDC, single-job schedule", lambda: B.ccdc_plan(K, r, Q, N)),
                       ("compression only (appendix)", lambda: B.ccdc_plan_compression(K, r, Q, N))):
        try:
            plan = ctor()
            out[name] = _load(plan, T)
            plan.close()
        except B.CcdcError:
            out[name] = None
    mu = Fraction(r, K)
    out["CDC only (formula of Sec. III)"] = (1 - mu) * N / (mu * K)
    return out


def main(argv):
    if len(argv) not in (4, 5):
        print(__doc__)
        return 2
    K, r, Q, N = (int(v) for v in argv[:4])
    T = int(argv[4]) if len(argv) == 5 else None
    rows = comparison(K, r, Q, N, T)
    width = max(len(k) for k in rows)
    print(f"K={K} r={r} (mu={Fraction(r, K)}) Q={Q} N={N}")
    for name, val in rows.items():
        shown = "n/a (N does not split into this scheme's batches)" if val is None else f"{str(val):>8s} = {float(val):.4f}"
        print(f"  {name:<{width}s}  {shown}")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
