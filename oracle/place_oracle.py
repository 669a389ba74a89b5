"""Plain reference for the paper's expert-to-GPU mapping search (Sec. 3.3.3 "Step-3", Eq. 1, and the
appendix "Expert Mapping Algorithm": initial mapping, iterative refinement, K restarts).

TEST INFRASTRUCTURE ONLY: imported by tests/, never by the package.  Plain Python, the algorithm's
steps in the paper's order and notation (M mapping, T trace, C_g curves, u mean utilisation, S score);
shares no code with the native implementation.

Readings where the paper is silent or ambiguous:
  * C_g(n): the straight line between the neighbouring samples of GPU g's profiled curve (the first
    sample's value below it, the last one's above it, 0 for n <= 0).
  * every GPU hosts exactly E / G experts (Sec. 3.3.3), so the greedy initial placement only
    considers GPUs that still have a free slot; S of a partial mapping counts placed experts only.
  * "20 % noise": u_e * (1 + 0.2 * xi_e) with xi_e in [-1, 1) supplied by the caller (one row per
    restart; the first restart uses u as it is).
  * ties: sort by utilisation keeps the lower expert index first; arg min over GPUs takes the lowest
    GPU index; the best swap is the first pair (e_a < e_b, ascending) with the strictly largest drop.
  * refinement follows the appendix listing: the best swap is committed, then the loop stops if
    bestDrop / s_prev < 0.001 (or if no swap improves the score at all).
"""


def curve_value(counts, ms, n):
    if n <= 0:
        return 0.0
    prev_c, prev_v = None, None
    for c, v in zip(counts, ms):
        if c == n:
            return float(v)
        if c > n:
            if prev_c is None:
                return float(v)
            return float(prev_v + (v - prev_v) * (n - prev_c) / (c - prev_c))
        prev_c, prev_v = c, v
    return float(prev_v)


def score(M, T, curves):
    """Eq. 1: S(M) = sum over steps t of max over GPUs g of C_g(n_g(M, t)); M[e] = GPU of expert e or
    None if e is not placed yet."""
    G = len(curves)
    total = 0.0
    for row in T:
        worst = 0.0
        for g in range(G):
            n = sum(row[e] for e in range(len(M)) if M[e] == g)
            worst = max(worst, curve_value(curves[g][0], curves[g][1], n))
        total += worst
    return total


def mean_utilisation(T):
    S = len(T)
    return [sum(T[t][e] for t in range(S)) / S for e in range(len(T[0]))]


def initial_mapping(u, noise_row, T, curves):
    """Appendix Alg. "Initialmapping": heaviest experts first, each on the GPU that gives the lowest
    score of the partial mapping."""
    E, G = len(u), len(curves)
    cap = E // G
    key = [u[e] * (1.0 + 0.2 * noise_row[e]) if noise_row is not None else u[e] for e in range(E)]
    order = sorted(range(E), key=lambda e: (-key[e], e))
    M = [None] * E
    for e in order:
        best_g, best_s = None, None
        for g in range(G):
            if sum(1 for x in M if x == g) >= cap:
                continue
            M[e] = g
            s = score(M, T, curves)
            M[e] = None
            if best_s is None or s < best_s:
                best_g, best_s = g, s
        M[e] = best_g
    return M


def refine(M, T, curves):
    """Appendix Alg. "Refine": commit the cross-GPU swap with the largest drop of S until the drop
    falls below 0.1 % of the score."""
    M = list(M)
    E = len(M)
    history = [score(M, T, curves)]
    while True:
        s_prev = score(M, T, curves)
        best, best_drop = None, 0.0
        for a in range(E):
            for b in range(a + 1, E):
                if M[a] == M[b]:
                    continue
                M[a], M[b] = M[b], M[a]
                drop = s_prev - score(M, T, curves)
                M[a], M[b] = M[b], M[a]
                if drop > best_drop:
                    best_drop, best = drop, (a, b)
        if best is None:
            break
        a, b = best
        M[a], M[b] = M[b], M[a]
        history.append(score(M, T, curves))
        if best_drop / s_prev < 0.001:
            break
    return M, history


def gem_place(K, T, curves, noise):
    """Appendix Alg. "Place": K restarts, the lowest-scoring refined mapping wins (the earliest on a
    tie).  noise: K rows of E values in [-1, 1) (row 0 is not used)."""
    u = mean_utilisation(T)
    best_M, best_s = None, float("inf")
    for i in range(K):
        M0 = initial_mapping(u, noise[i] if i > 0 else None, T, curves)
        Mm, _ = refine(M0, T, curves)
        s = score(Mm, T, curves)
        if s < best_s:
            best_s, best_M = s, Mm
    return best_M, best_s
