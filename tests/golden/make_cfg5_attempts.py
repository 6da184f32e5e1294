"""Certify the random-DAG workload against the CPU oracle.

For each DAG index k, redraws (attempt = 0, 1, ...) until the oracle finds the
candidate well behaved, and records the accepted attempt in
workloads/cfg5_attempts.txt.  A candidate is accepted when, evaluated op by op
in fp64 on its real inputs,
  * every node value is finite and at most 1e6 in magnitude,
  * every divisor and every rsqrt argument is at least 1e-3 in magnitude,
  * the same definition evaluated in fp32 agrees with fp64 on every output to a
    quarter of the comparison tolerance of the DAG's dtype (so the subgraph is
    well conditioned: an fp32 engine can be expected to meet the tolerance).
Calls only oracle/ and the input generators.  Usage:
    python tests/golden/make_cfg5_attempts.py [first_k last_k]
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import dag  # noqa: E402
from workloads import configs, dags  # noqa: E402


class Rejected(Exception):
    pass


def _observer(node, value, operands):
    if not np.isfinite(value).all():
        raise Rejected("non-finite at %%%d (%s)" % (node.id, node.op))
    if value.size and np.abs(value).max() > 1e6:
        raise Rejected("magnitude at %%%d (%s)" % (node.id, node.op))
    if node.op == "div" and np.abs(operands[1]).min() < 1e-3:
        raise Rejected("small divisor at %%%d" % node.id)
    if node.op == "rsqrt" and operands[0].min() < 1e-3:
        raise Rejected("small rsqrt argument at %%%d" % node.id)


def check(w):
    ref = dag.run(w.text, w.inputs, observer=_observer)
    low = dag.run(w.text, w.inputs, dtype=np.float32)
    rtol = configs.RTOL[w.meta["dtype"]] / 4
    atol = configs.ATOL[w.meta["dtype"]] / 4
    for r, l in zip(ref, low):
        bad = np.abs(l.astype(np.float64) - r) > atol + rtol * np.abs(r)
        if bad.any():
            raise Rejected("ill conditioned in fp32 (%d elements)" % int(bad.sum()))


def certify(k, max_attempts=64):
    for attempt in range(max_attempts):
        try:
            check(dags.draw_dag(k, attempt, max_rows=32))     # cheap screen, same structure
            check(dags.draw_dag(k, attempt))
            return attempt
        except Rejected as e:
            print("  dag %d attempt %d rejected: %s" % (k, attempt, e), flush=True)
    raise RuntimeError("no acceptable draw for dag %d" % k)


def main():
    lo, hi = (int(sys.argv[1]), int(sys.argv[2])) if len(sys.argv) > 2 else (0, dags.N_DAGS)
    path = os.path.join(ROOT, "workloads", "cfg5_attempts.txt")
    have = dags.accepted_attempts(path) if os.path.exists(path) else {}
    t0 = time.time()
    for k in range(lo, hi):
        have[k] = certify(k)
        print("dag %d -> attempt %d (%.0f s)" % (k, have[k], time.time() - t0), flush=True)
    with open(path, "w") as f:
        f.write("# DAG index, accepted attempt; written by tests/golden/make_cfg5_attempts.py\n")
        for k in sorted(have):
            f.write("%d %d\n" % (k, have[k]))


if __name__ == "__main__":
    main()
