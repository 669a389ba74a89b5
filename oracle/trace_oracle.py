"""Plain reference for the expert-utilisation trace statistics (paper Sec. 3.3.1 and Sec. 3.2):
T[t][e] = number of tokens routed to expert e at step t; u[e] = its mean over the steps; Pearson's
correlation coefficient of two experts' loads across the steps.

TEST INFRASTRUCTURE ONLY: imported by tests/, never by the package.  Plain Python loops, textbook
definitions (r = cov(a, b) / (sigma_a sigma_b)); shares no code with paper_2605_19945_amd/trace.py.
"""
import math


def trace_from_indices(idx_per_step, E):
    """idx_per_step: for every step a [T][k] table of selected experts -> T[t][e]."""
    trace = []
    for idx in idx_per_step:
        row = [0] * E
        for tok in idx:
            for e in tok:
                row[int(e)] += 1
        trace.append(row)
    return trace


def mean_utilisation(trace):
    S = len(trace)
    return [sum(trace[t][e] for t in range(S)) / S for e in range(len(trace[0]))]


def pearson(trace, e1, e2):
    S = len(trace)
    ma = sum(trace[t][e1] for t in range(S)) / S
    mb = sum(trace[t][e2] for t in range(S)) / S
    cov = sum((trace[t][e1] - ma) * (trace[t][e2] - mb) for t in range(S))
    va = sum((trace[t][e1] - ma) ** 2 for t in range(S))
    vb = sum((trace[t][e2] - mb) ** 2 for t in range(S))
    if va == 0 or vb == 0:
        return float("nan")
    return cov / math.sqrt(va * vb)
