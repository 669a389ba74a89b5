"""Seeded generators for the MoE-layer workloads.

Every tensor is a function of (seed, tensor id, shape) only: a tensor is cut into fixed-size
chunks, chunk c is drawn from its own SFC64 stream seeded by SeedSequence([seed, tensor_id, c]),
so the result does not depend on the number of worker threads.  Floating-point tensors that the
layer consumes as bf16 are produced as uint16 bit patterns (fp32 draw, scaled, rounded to
nearest-even); both consumers widen those bits themselves.

Workload structure follows the paper's description of MoE serving loads: skewed expert
popularity (hottest expert a few times the uniform share, Sec. 2.1 / Fig. "expert imbalance"),
"consistent" experts that are busy almost always and "temporal" experts that are co-activated in
pairs for a minority of the load (Sec. 3.2, Fig. "expert pair heatmaps"), and per-GPU token loads
from a handful up to ~16K tokens (Sec. 3.3.2).  The paper's datasets and trained weights are not
available; these draws stand in for them.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

_CHUNK = 1 << 22  # elements per independently seeded chunk
_THREADS = 8

# tensor ids (second word of the seed sequence)
_TID_X, _TID_WG, _TID_BIAS, _TID_W1, _TID_W3, _TID_W2, _TID_DIR, _TID_GROUPS, _TID_XP = range(1, 10)
_TID_STEPS = 10


@dataclass(frozen=True)
class MoEShape:
    T: int          # tokens in this call
    d: int          # model width
    f: int          # expert FFN width
    E: int          # experts seen by the router
    k: int          # experts per token
    e_lo: int = 0   # first expert resident on this GPU
    E_local: int = -1  # number of resident experts (-1: all)

    def __post_init__(self):
        if self.E_local < 0:
            object.__setattr__(self, "E_local", self.E)

    @property
    def A(self) -> int:
        return self.T * self.k


@dataclass
class MoEInputs:
    name: str
    shape: MoEShape
    x: np.ndarray                      # uint16 [T, d]   bf16 bits
    Wg: np.ndarray                     # float32 [d, E]
    bias: Optional[np.ndarray]         # float32 [E] or None
    W1: Optional[np.ndarray] = None    # uint16 [E_local, d, f]
    W3: Optional[np.ndarray] = None    # uint16 [E_local, d, f]
    W2: Optional[np.ndarray] = None    # uint16 [E_local, f, d]
    notes: dict = field(default_factory=dict)


def bf16_bits_from_f32(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern, round to nearest, ties to even (inputs are finite)."""
    b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def _chunk_f32(seed: int, tid: int, c: int, n: int, std: float) -> np.ndarray:
    g = np.random.Generator(np.random.SFC64(np.random.SeedSequence([seed, tid, c])))
    a = g.standard_normal(n, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def gaussian_f32(seed: int, tid: int, shape, std: float = 1.0) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    nchunks = (n + _CHUNK - 1) // _CHUNK

    def work(c):
        lo = c * _CHUNK
        hi = min(n, lo + _CHUNK)
        out[lo:hi] = _chunk_f32(seed, tid, c, hi - lo, std)

    if nchunks <= 1:
        for c in range(nchunks):
            work(c)
    else:
        with ThreadPoolExecutor(_THREADS) as ex:
            list(ex.map(work, range(nchunks)))
    return out.reshape(shape)


def gaussian_bf16_bits(seed: int, tid: int, shape, std: float = 1.0) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    nchunks = (n + _CHUNK - 1) // _CHUNK

    def work(c):
        lo = c * _CHUNK
        hi = min(n, lo + _CHUNK)
        out[lo:hi] = bf16_bits_from_f32(_chunk_f32(seed, tid, c, hi - lo, std))

    if nchunks <= 1:
        for c in range(nchunks):
            work(c)
    else:
        with ThreadPoolExecutor(_THREADS) as ex:
            list(ex.map(work, range(nchunks)))
    return out.reshape(shape)


def expert_weights(seed: int, E_local: int, d: int, f: int, std: float = 0.02):
    """W1, W3 as [E_local, d, f] and W2 as [E_local, f, d], bf16 bits, N(0, std)."""
    W1 = gaussian_bf16_bits(seed, _TID_W1, (E_local, d, f), std)
    W3 = gaussian_bf16_bits(seed, _TID_W3, (E_local, d, f), std)
    W2 = gaussian_bf16_bits(seed, _TID_W2, (E_local, f, d), std)
    return W1, W3, W2


def _attach_weights(inp: MoEInputs, seed: int, weights) -> MoEInputs:
    s = inp.shape
    if weights is None:
        weights = expert_weights(seed, s.E_local, s.d, s.f)
    if weights is not False:
        inp.W1, inp.W3, inp.W2 = weights
        assert inp.W1.shape == (s.E_local, s.d, s.f) and inp.W2.shape == (s.E_local, s.f, s.d)
    return inp


def custom(name, T, d, f, E, k, seed=0, e_lo=0, E_local=-1, wg_std=0.02, bias_std=0.0,
           w_std=0.02, weights=None) -> MoEInputs:
    """Free-form Gaussian workload used by edge-case tests."""
    s = MoEShape(T, d, f, E, k, e_lo, E_local)
    x = gaussian_bf16_bits(seed, _TID_X, (T, d), 1.0)
    Wg = gaussian_f32(seed, _TID_WG, (d, E), wg_std)
    bias = gaussian_f32(seed, _TID_BIAS, (E,), bias_std) if bias_std > 0 else None
    inp = MoEInputs(name, s, x, Wg, bias)
    if weights is None:
        weights = expert_weights(seed, s.E_local, d, f, w_std)
    return _attach_weights(inp, seed, weights)


def tiny(seed: int = 0) -> MoEInputs:
    """T=64, d=128, f=256, E=8, top-2."""
    return custom("tiny", 64, 128, 256, 8, 2, seed)


MIXTRAL_D, MIXTRAL_F, MIXTRAL_E, MIXTRAL_K = 4096, 14336, 8, 2


def mixtral(T: int = 4096, seed: int = 0, weights=None) -> MoEInputs:
    """Mixtral-8x7B-shaped layer, Gaussian router (near-uniform expert load).

    `weights`: None -> draw them; False -> leave them out (routing-only use);
    or a (W1, W3, W2) tuple drawn earlier with `expert_weights` to avoid redrawing 2.8 GB.
    """
    s = MoEShape(T, MIXTRAL_D, MIXTRAL_F, MIXTRAL_E, MIXTRAL_K)
    x = gaussian_bf16_bits(seed, _TID_X, (T, s.d), 1.0)
    Wg = gaussian_f32(seed, _TID_WG, (s.d, s.E), 0.02)
    return _attach_weights(MoEInputs(f"mixtral_T{T}", s, x, Wg, None), seed, weights)


# Planted structure of the skewed Mixtral-shaped workload.  Experts 0,1 are "consistent";
# (2,3) and (4,5) are "temporal" pairs, each switched on for one contiguous 15 % burst of the
# tokens; popularity of experts 2..7 outside the bursts follows Zipf(1.2).
SKEW_CONSISTENT = (0, 1)
SKEW_PAIRS = ((2, 3), (4, 5))
SKEW_BURSTS = ((0.20, 0.35), (0.60, 0.75))
SKEW_ZIPF_S = 1.2
SKEW_BIAS_CONSISTENT = 2.4   # router-bias lead of the consistent experts (logit noise std is 1.28)
SKEW_ALPHA = 20.0            # burst tokens: x += alpha * u_p          (|u_p| = 1)
SKEW_BETA = 0.5              # pair columns: Wg[:, e] += beta * u_p    -> logit lead alpha*beta = 10


def mixtral_skewed(T: int, seed: int = 0, weights=None) -> MoEInputs:
    s = MoEShape(T, MIXTRAL_D, MIXTRAL_F, MIXTRAL_E, MIXTRAL_K)
    xf = gaussian_f32(seed, _TID_X, (T, s.d), 1.0)
    Wg = gaussian_f32(seed, _TID_WG, (s.d, s.E), 0.02)
    bias = np.zeros(s.E, dtype=np.float32)
    for e in SKEW_CONSISTENT:
        bias[e] = SKEW_BIAS_CONSISTENT
    others = [e for e in range(s.E) if e not in SKEW_CONSISTENT]
    for r, e in enumerate(others, start=1):
        bias[e] = -SKEW_ZIPF_S * math.log(r)          # ln of the Zipf weight r^-s
    bursts = []
    for p, (pair, (lo, hi)) in enumerate(zip(SKEW_PAIRS, SKEW_BURSTS)):
        u = gaussian_f32(seed, _TID_DIR, (len(SKEW_PAIRS), s.d), 1.0)[p].astype(np.float64)
        u /= np.sqrt((u * u).sum())
        t0, t1 = int(round(lo * T)), int(round(hi * T))
        xf[t0:t1] += (SKEW_ALPHA * u).astype(np.float32)
        for e in pair:
            Wg[:, e] += (SKEW_BETA * u).astype(np.float32)
        bursts.append((pair, t0, t1))
    inp = MoEInputs(f"mixtral_skewed_T{T}", s, bf16_bits_from_f32(xf), Wg, bias,
                    notes={"bursts": bursts, "consistent": SKEW_CONSISTENT})
    return _attach_weights(inp, seed, weights)


def fine_grained(T: int = 8192, seed: int = 0, weights=None, d=2048, f=768, E=128, k=8) -> MoEInputs:
    """d=2048, f=768, E=128, top-8; unit-variance logits plus a N(0, 0.5) per-expert bias."""
    s = MoEShape(T, d, f, E, k)
    x = gaussian_bf16_bits(seed, _TID_X, (T, d), 1.0)
    Wg = gaussian_f32(seed, _TID_WG, (d, E), 1.0 / math.sqrt(d))
    bias = gaussian_f32(seed, _TID_BIAS, (E,), 0.5)
    return _attach_weights(MoEInputs(f"fine_grained_T{T}", s, x, Wg, bias), seed, weights)


EP_D, EP_F, EP_E, EP_K, EP_ELO, EP_ELOCAL = 7168, 2048, 256, 8, 64, 32


def ep_share_layer(T: int, seed: int = 0, weights=None, d=EP_D, f=EP_F, E=EP_E, k=EP_K,
                   e_lo=EP_ELO, E_local=EP_ELOCAL) -> MoEInputs:
    """One GPU's expert-parallel share: routing over all E experts, experts
    [e_lo, e_lo+E_local) resident.  The local experts' router bias is the log of a Zipf(1.0)
    popularity; the other experts have zero bias."""
    s = MoEShape(T, d, f, E, k, e_lo, E_local)
    x = gaussian_bf16_bits(seed, _TID_X, (T, d), 1.0)
    Wg = gaussian_f32(seed, _TID_WG, (d, E), 1.0 / math.sqrt(d))
    bias = np.zeros(E, dtype=np.float32)
    for r in range(1, E_local + 1):
        bias[e_lo + r - 1] = 1.5 - math.log(r)
    return _attach_weights(MoEInputs(f"ep_share_T{T}", s, x, Wg, bias), seed, weights)


def ep_share_groups(N: int, seed: int = 0, d=EP_D, E_local=EP_ELOCAL, zipf_s: float = 1.0):
    """Already-routed form of the expert-parallel share: N incoming rows split over the local
    experts by one multinomial draw with Zipf(zipf_s) probabilities.
    Returns (xp bits [N, d], offsets int32 [E_local+1])."""
    p = np.array([r ** -zipf_s for r in range(1, E_local + 1)], dtype=np.float64)
    p /= p.sum()
    g = np.random.Generator(np.random.SFC64(np.random.SeedSequence([seed, _TID_GROUPS, N])))
    n_e = g.multinomial(N, p)
    offsets = np.zeros(E_local + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(n_e)
    xp = gaussian_bf16_bits(seed, _TID_XP, (N, d), 1.0)
    return xp, offsets


TRACE_CONSISTENT = (1, 6)     # lead the router in every step
TRACE_PAIR = (2, 5)           # correlated temporal experts: heavily used together in a few steps
TRACE_ACTIVE_FRACTION = 0.17  # share of the steps in which the pair is active
TRACE_BURST_TOKENS = 0.6      # share of a step's tokens whose top-2 is the pair when it is active


def trace_steps(S: int = 16, T: int = 256, seed: int = 0, d: int = 512, E: int = 8, k: int = 2):
    """S consecutive time steps of one router (the structure the paper describes for expert
    utilisation over time): two consistent experts lead in every step; a pair of temporal experts is
    active together in about 17 % of the steps (at least two of them, never the first), where it takes
    the top-2 of 60 % of that step's tokens.  Returns (list of S routing-only MoEInputs sharing Wg and
    bias, list of S booleans: pair active)."""
    s = MoEShape(T, d, 64, E, k)
    Wg = gaussian_f32(seed, _TID_WG, (d, E), 1.0 / math.sqrt(d))
    bias = np.zeros(E, dtype=np.float32)
    for e in TRACE_CONSISTENT:
        bias[e] = 1.5
    u = gaussian_f32(seed, _TID_DIR, (1, d), 1.0)[0].astype(np.float64)
    u /= np.sqrt((u * u).sum())
    for e in TRACE_PAIR:
        Wg[:, e] += (SKEW_BETA * u).astype(np.float32)
    g = np.random.Generator(np.random.SFC64(np.random.SeedSequence([seed, _TID_STEPS, S])))
    n_active = max(2, int(round(TRACE_ACTIVE_FRACTION * S)))
    active_steps = set((1 + g.permutation(S - 1)[:n_active]).tolist()) if S > 2 else set()
    steps, active = [], []
    for t in range(S):
        xf = gaussian_f32(seed + 1000 * (t + 1), _TID_X, (T, d), 1.0)
        on = t in active_steps
        if on:
            xf[: int(round(TRACE_BURST_TOKENS * T))] += (SKEW_ALPHA * u).astype(np.float32)
        steps.append(MoEInputs(f"trace_step{t}", s, bf16_bits_from_f32(xf), Wg, bias))
        active.append(on)
    return steps, active


def wide_few_experts(T: int = 8192, seed: int = 0, weights=None) -> MoEInputs:
    """A second shape family: few wide experts, top-1 (d=5120, f=8192, E=16, k=1 -- the proportions of
    the 16-expert model the paper evaluates; its exact dimensions are not in the paper)."""
    s = MoEShape(T, 5120, 8192, 16, 1)
    x = gaussian_bf16_bits(seed, _TID_X, (T, s.d), 1.0)
    Wg = gaussian_f32(seed, _TID_WG, (s.d, s.E), 1.0 / math.sqrt(s.d))
    bias = gaussian_f32(seed, _TID_BIAS, (s.E,), 0.5)
    return _attach_weights(MoEInputs(f"wide_few_T{T}", s, x, Wg, bias), seed, weights)


def mid_grained(T: int = 8192, seed: int = 0, weights=None) -> MoEInputs:
    """A third shape family: 64 medium experts, top-8 (d=4096, f=3072, E=64, k=8 -- the proportions of
    the 64-expert model the paper evaluates; its exact dimensions are not in the paper)."""
    s = MoEShape(T, 4096, 3072, 64, 8)
    x = gaussian_bf16_bits(seed, _TID_X, (T, s.d), 1.0)
    Wg = gaussian_f32(seed, _TID_WG, (s.d, s.E), 1.0 / math.sqrt(s.d))
    bias = gaussian_f32(seed, _TID_BIAS, (s.E,), 0.5)
    return _attach_weights(MoEInputs(f"mid_grained_T{T}", s, x, Wg, bias), seed, weights)
