"""CPU oracle of the per-GPU MoE expert layer.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path may import this module: it exists so that tests, the smoke check and
the benchmark's `cpu_baseline` leg have an independent, slow, plainly written definition of what
the HIP kernels must compute.  It shares no code with the HIP path.

The paper (GEM, Sec. 1 and Sec. 2.1) describes the layer only in words: a router picks the top-k
of E experts for every token, the token is sent to those experts, each expert is a feed-forward
network, and the per-expert token counts fall out of the router (Sec. 3.3.1, Step 1).  It prints
no formula and no worked example of the layer.  The formulas below are therefore the standard
definition named by the build target (softmax over the k selected logits, SwiGLU experts
W2^T(silu(W1^T x) * W3^T x), no biases in the experts).

Arithmetic: inputs are bf16 bit patterns or fp32, widened exactly to fp64; all sums are fp64
(numpy matmul is the contraction primitive).  Router logits are rounded once to fp32 and every
integer decision (which experts, in which order) is taken on those fp32 values.

Pins (tests/test_oracle_pins.py): brute-force top-k with forced ties, gate-weight identities,
count/permutation invariants and an O(T^2) literal stable-rank definition, a hand-derived worked
example, identical experts == dense SwiGLU FFN evaluated by pure-Python loops and by a second
library (torch fp64), one-hot inputs, W2 scaling, token-permutation equivariance and per-token
independence; the diagnostic bf16 rounding against hand-picked bit patterns and against an expert
FFN whose intermediate is rebuilt by scalar loops; layer_forward under a given routing against the
staged calls.  No function here is unpinned.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------- input decoding
def widen_bf16(bits: np.ndarray) -> np.ndarray:
    """bf16 bit pattern (uint16) -> fp64, exact."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


# ----------------------------------------------------------------------------- router (Sec. 2.1)
def router_logits(x_bits: np.ndarray, Wg: np.ndarray, bias=None) -> np.ndarray:
    """logit[t, e] = sum_i x[t, i] * Wg[i, e] (+ bias[e]); fp64 sum, rounded once to fp32."""
    z = widen_bf16(x_bits) @ np.asarray(Wg, dtype=np.float64)
    if bias is not None:
        z = z + np.asarray(bias, dtype=np.float64)[None, :]
    return z.astype(np.float32)


def topk_experts(logits: np.ndarray, k: int) -> np.ndarray:
    """The k experts with the largest logit per token, slot 0 = largest.  Equal logits: the
    lower expert index comes first (stable sort of the negated logits)."""
    order = np.argsort(-logits.astype(np.float32), axis=1, kind="stable")
    return order[:, :k].astype(np.int32)


def topk_gap(logits: np.ndarray, k: int) -> np.ndarray:
    """logit of the k-th selected expert minus the best logit left out (+inf when k == E).
    Tokens whose gap is below the near-tie threshold are excluded from index parity."""
    s = -np.sort(-logits.astype(np.float64), axis=1)
    if k >= logits.shape[1]:
        return np.full(logits.shape[0], np.inf)
    return s[:, k - 1] - s[:, k]


def gate_weights(logits: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """Softmax over the k selected logits only: w_j = exp(l_j - l_0) / sum_j' exp(l_j' - l_0)."""
    sel = np.take_along_axis(logits.astype(np.float64), idx.astype(np.int64), axis=1)
    ex = np.exp(sel - sel[:, :1])
    return (ex / ex.sum(axis=1, keepdims=True)).astype(np.float32)


def expert_counts(idx: np.ndarray, E: int) -> np.ndarray:
    """counts[e] = number of (token, slot) pairs routed to expert e (one row of the paper's
    expert-utilisation trace, Sec. 3.3.1)."""
    return np.bincount(idx.reshape(-1), minlength=E).astype(np.int32)


def route(x_bits, Wg, bias, k):
    logits = router_logits(x_bits, Wg, bias)
    idx = topk_experts(logits, k)
    w = gate_weights(logits, idx)
    return logits, idx, w, expert_counts(idx, Wg.shape[1])


# ----------------------------------------------------------------------------- dispatch by expert
def permutation(idx: np.ndarray, E: int, e_lo: int = 0, E_local: int = -1):
    """Expert-contiguous, token-stable ordering of the local assignments.

    offsets[e'] = number of local assignments to experts before e_lo + e';
    row_of[t, j] = offsets[e'] + #{t' < t : expert e'+e_lo selected by t'}   (-1 if not local);
    tok_of[row] = t.
    """
    if E_local < 0:
        E_local = E
    T, k = idx.shape
    counts = expert_counts(idx, E)[e_lo:e_lo + E_local]
    offsets = np.zeros(E_local + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    row_of = np.full((T, k), -1, dtype=np.int32)
    tok_of = np.full(int(offsets[-1]), -1, dtype=np.int32)
    seen = np.zeros(E_local, dtype=np.int64)          # tokens so far that selected each expert
    for t in range(T):
        for j in range(k):
            e = int(idx[t, j]) - e_lo
            if 0 <= e < E_local:
                r = int(offsets[e] + seen[e])
                seen[e] += 1
                row_of[t, j] = r
                tok_of[r] = t
    return offsets, row_of, tok_of


def gather_rows(x_bits: np.ndarray, tok_of: np.ndarray) -> np.ndarray:
    """xp[r, :] = x[tok_of[r], :] (bit copy)."""
    return x_bits[tok_of]


# ----------------------------------------------------------------------------- experts
def silu(g: np.ndarray) -> np.ndarray:
    return g / (1.0 + np.exp(-g))


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp64 -> nearest bf16 (ties to even) -> fp64.  Diagnostic only."""
    f = a.astype(np.float32).view(np.uint32)
    r = ((f + np.uint32(0x7FFF) + ((f >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)) << np.uint32(16)
    return r.view(np.float32).astype(np.float64)


def expert_ffn(X: np.ndarray, W1e_bits, W3e_bits, W2e_bits, round_h_bf16: bool = False) -> np.ndarray:
    """One expert on rows X [n, d] (fp64): y = (silu(X W1) * (X W3)) W2, with W1, W3 [d, f] and
    W2 [f, d] given as bf16 bits."""
    g = X @ widen_bf16(W1e_bits)
    u = X @ widen_bf16(W3e_bits)
    h = silu(g) * u
    if round_h_bf16:
        h = round_to_bf16(h)
    return h @ widen_bf16(W2e_bits)


def grouped_ffn(xp_bits: np.ndarray, offsets: np.ndarray, W1, W3, W2, rows=None,
                round_h_bf16: bool = False) -> np.ndarray:
    """Rows offsets[e]..offsets[e+1] of xp go through local expert e.  `rows` (sorted) restricts
    the evaluation to a subset; the result then has one line per requested row."""
    E_local = len(offsets) - 1
    if rows is None:
        rows = np.arange(int(offsets[-1]))
    rows = np.asarray(rows, dtype=np.int64)
    Y = np.zeros((len(rows), W2.shape[2]), dtype=np.float64)
    for e in range(E_local):
        sel = np.nonzero((rows >= offsets[e]) & (rows < offsets[e + 1]))[0]
        if len(sel) == 0:
            continue
        Y[sel] = expert_ffn(widen_bf16(xp_bits[rows[sel]]), W1[e], W3[e], W2[e], round_h_bf16)
    return Y


# ----------------------------------------------------------------------------- combine
def combine(Y: np.ndarray, row_of: np.ndarray, w: np.ndarray) -> np.ndarray:
    """out[t] = sum_j w[t, j] * Y[row_of[t, j]] in slot order; non-local slots contribute 0."""
    T, k = row_of.shape
    out = np.zeros((T, Y.shape[1]), dtype=np.float64)
    for j in range(k):
        ok = row_of[:, j] >= 0
        out[ok] += w[ok, j].astype(np.float64)[:, None] * Y[row_of[ok, j]]
    return out


# ----------------------------------------------------------------------------- whole layer
def layer_forward(x_bits, Wg, bias, W1, W3, W2, k, e_lo=0, tokens=None, idx=None, w=None,
                  round_h_bf16=False):
    """Router -> dispatch -> experts -> weighted combine, evaluated for `tokens` (default all).

    Each out[t] depends only on x[t], its k experts and the weights, so any subset of tokens is
    exact.  `idx`/`w` [T, k] may be supplied to evaluate the experts under a given routing (used
    for tokens whose top-k is a near-tie).  Returns dict(out, logits, idx, w, counts).
    """
    E = Wg.shape[1]
    E_local = W1.shape[0]
    logits = router_logits(x_bits, Wg, bias)
    if idx is None:
        idx = topk_experts(logits, k)
    if w is None:
        w = gate_weights(logits, idx)
    counts = expert_counts(idx, E)
    T = x_bits.shape[0]
    tokens = np.arange(T) if tokens is None else np.asarray(tokens, dtype=np.int64)
    # y of every local (token, slot) pair, then the weighted sum over slots in slot order
    contrib = np.zeros((len(tokens), k, W2.shape[2]), dtype=np.float64)
    for e in range(E_local):
        hit_t, hit_j = np.nonzero(idx[tokens] == e + e_lo)
        if len(hit_t) == 0:
            continue
        contrib[hit_t, hit_j] = expert_ffn(widen_bf16(x_bits[tokens[hit_t]]), W1[e], W3[e], W2[e],
                                           round_h_bf16)
    out = np.zeros((len(tokens), W2.shape[2]), dtype=np.float64)
    for j in range(k):
        out += w[tokens, j].astype(np.float64)[:, None] * contrib[:, j]
    return dict(out=out, logits=logits, idx=idx, w=w, counts=counts)
