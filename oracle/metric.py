"""CPU oracle: tolerance ladder and the error-aware speedup scores.

TEST INFRASTRUCTURE ONLY; the product path never imports this.

Follows the paper's Sec. 3.4 (Eq. 2: rectified speedup, Eq. 3: ES_t, Eq. 4: AS),
Appendix E (weights W_t) and Appendix F (atol(t), rtol(t) per dtype), written
out step by step.

Readings where the text is silent or garbled:
  * the tolerance index runs over t = -10 .. |E|+1 with |E| = 3 error
    categories (accuracy 1, compilation 2, runtime 3), i.e. t = -10 .. 4;
  * for t <= 0 a subgraph is correct at t when it compiled, ran, and every
    output element passes |a-b| <= atol(t) + rtol(t)*|b| for the output's
    dtype; for t > 0 the numerical test is the one of t = 0;
  * a subgraph that is not correct at t has category 2 or 3 if it failed to
    compile / run and category 1 otherwise, and contributes b if t < c, else 1;
  * fast_p counts subgraphs that are correct at a stated t and faster than p,
    over all subgraphs.
"""
import math

import numpy as np

from .score import score_pair

T_MIN, N_CATEGORIES = -10, 3
T_MAX = N_CATEGORIES + 1
LADDER = list(range(T_MIN, 1))          # the tolerance indices with a numerical meaning

_RTOL_SLOPE = {"bf16": 1.796 / 5, "f16": 3.0 / 5, "f32": 5.886 / 5, "f64": 7.0 / 5}
_ATOL_SLOPE = {"bf16": 1.0, "f16": 1.0, "f32": 1.0, "f64": 7.0 / 5}


def tolerance(dtype, t):
    """(rtol, atol) at tolerance index t <= 0: log-linear between the table's anchor points."""
    if t > 0:
        t = 0
    return 10.0 ** (_RTOL_SLOPE[dtype] * t), 10.0 ** (_ATOL_SLOPE[dtype] * t)


def ladder_violations(cand, cand_dtype, ref, ref_dtype):
    """Number of elements outside the tolerance, for t = -10 .. 0 (11 counts)."""
    out = []
    for t in LADDER:
        rtol, atol = tolerance(cand_dtype, t)
        out.append(score_pair(cand, cand_dtype, ref, ref_dtype, rtol, atol)["n_viol"])
    return out


def weight(t):
    if t <= -6 or t >= N_CATEGORIES + 1:
        return 0.001
    if t <= -3:
        return 1.0
    return 0.8 ** (t + 3)


def correct_at(case, t):
    """case: dict(speedup, error_class in {0,2,3}, viol = 11 ladder counts summed over outputs)."""
    if case["error_class"] != 0:
        return False
    return case["viol"][min(t, 0) - T_MIN] == 0


def rectified_speedup(case, t, b=0.1, p=0.0):
    s = case["speedup"]
    if correct_at(case, t):
        return s if s >= 1.0 else s ** (p + 1.0)
    c = case["error_class"] if case["error_class"] != 0 else 1
    return b if t < c else 1.0


def es(cases, t, b=0.1, p=0.0):
    logs = [math.log(rectified_speedup(c, t, b, p)) for c in cases]
    return math.exp(sum(logs) / len(logs))


def aggregated_score(cases, b=0.1, p=0.0):
    ts = list(range(T_MIN, T_MAX + 1))
    wsum = sum(weight(t) for t in ts)
    return math.exp(sum(weight(t) / wsum * math.log(es(cases, t, b, p)) for t in ts))


def fast_p(cases, p_threshold, t=0):
    return sum(1 for c in cases if correct_at(c, t) and c["speedup"] > p_threshold) / len(cases)
