"""Seeded synthetic inputs for the MoE-layer forward (shapes and skew of the five workloads).

This module only DRAWS inputs: activations, router weights, router biases, expert weights and
(for the pre-routed workload) expert ids.  It holds none of the layer's arithmetic -- no router
product, no top-k, no permutation, no FFN -- so that the CPU oracle and the GPU library can both
be fed from it without sharing any part of the method.

Workloads (T tokens, d = d_model, F = d_ff, E experts, k = top-k):

  c1  tiny, fp32            T=256   d=64   F=128   E=8   k=2 renormalised, ReLU,
                            router bias b_e = 1.5*ln(1/(e+1))
  c2  Switch-style, bf16    T=16384 d=768  F=3072  E=128 k=1, ReLU, first-choice loads ~ Zipf(1.0)
                            over a seeded expert order (also with b = 0: uniform)
  c3  fine-grained, bf16    T=8192  d=2048 F=1408  E=60  k=4, SwiGLU, + shared SwiGLU expert
                            F=5632, first-choice loads ~ Zipf(1.2)
  c4  large experts, bf16   T=8192  d=4096 F=14336 E=8   k=2 renormalised, SwiGLU, one hot expert
                            in ~95% of the tokens' top-2, the rest Zipf(0.8)
  c5  pre-routed, bf16      T=32768 d=768  F=3072  16 local + 16 foreign experts, k=1, ReLU,
                            expert ids drawn directly: 70% local / 30% foreign, Zipf(1.5) inside
                            each group

The shapes follow the paper's two models (Switch128: 128 experts of 18 MB; Qwen1.5-MoE: 60
experts of 33 MB, model table in the appendix); the skew stands in for the expert-popularity
ECDFs the paper measures on its text datasets (introduction, Fig. 1), which are not reproduced.

Weights are stored in the paper's orientation (section 4.4: W1 is m x p = d x F, W2 is p x m).
bf16 tensors are returned as uint16 bit patterns (numpy has no bf16); fp32 tensors as float32.
All values come from numpy's PCG64 `default_rng([seed, stream])`, one stream per tensor, so any
tensor can be regenerated alone.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Optional

import numpy as np

SEED0 = 2506124170

# stream ids (second word of the PCG64 seed sequence)
_S_X, _S_WG, _S_ORDER, _S_MC, _S_IDS, _S_SHARED = 1, 2, 3, 4, 5, 6
_S_W = 1000  # + 3*e + {0,1,2} per expert tensor


@dataclasses.dataclass(frozen=True)
class MoEWorkload:
    name: str
    index: int            # position in the list of workloads (fixes the seed)
    T: int
    d: int
    F: int
    E: int
    k: int
    act: str              # "relu" | "swiglu"
    dtype: str            # "f32" | "bf16"
    renorm: int           # 1: gate weights renormalised over the k selected experts
    shared_F: int = 0     # d_ff of the always-on shared expert (0: none)
    skew: str = "zipf"    # "c1bias" | "zipf" | "hot" | "uniform" | "ids"
    zipf_s: float = 1.0
    hot_top2: float = 0.95   # "hot": target P(hot expert in a token's top-2)
    n_local: int = 0         # "ids": experts [0, n_local) are device-resident
    foreign_share: float = 0.0

    @property
    def A(self) -> int:
        return self.T * self.k

    def seed(self) -> int:
        return SEED0 + 10 * self.index

    def scaled(self, **kw) -> "MoEWorkload":
        """Same family at other sizes (used by the parity tests)."""
        return dataclasses.replace(self, **kw)


WORKLOADS: Dict[str, MoEWorkload] = {
    "c1": MoEWorkload("c1", 0, T=256, d=64, F=128, E=8, k=2, act="relu", dtype="f32", renorm=1,
                      skew="c1bias"),
    "c2": MoEWorkload("c2", 1, T=16384, d=768, F=3072, E=128, k=1, act="relu", dtype="bf16",
                      renorm=0, skew="zipf", zipf_s=1.0),
    "c2u": MoEWorkload("c2u", 1, T=16384, d=768, F=3072, E=128, k=1, act="relu", dtype="bf16",
                       renorm=0, skew="uniform"),
    "c3": MoEWorkload("c3", 2, T=8192, d=2048, F=1408, E=60, k=4, act="swiglu", dtype="bf16",
                      renorm=0, shared_F=5632, skew="zipf", zipf_s=1.2),
    "c4": MoEWorkload("c4", 3, T=8192, d=4096, F=14336, E=8, k=2, act="swiglu", dtype="bf16",
                      renorm=1, skew="hot", zipf_s=0.8),
    "c5": MoEWorkload("c5", 4, T=32768, d=768, F=3072, E=32, k=1, act="relu", dtype="bf16",
                      renorm=0, skew="ids", zipf_s=1.5, n_local=16, foreign_share=0.30),
}


# ----------------------------------------------------------------------------- number formats
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(stream)])


def _normal(seed: int, stream: int, shape, std: float, dtype: str) -> np.ndarray:
    a = _rng(seed, stream).standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return f32_to_bf16_bits(a) if dtype == "bf16" else a


# ----------------------------------------------------------------------------- router bias
def zipf_shares(E: int, s: float, seed: int) -> np.ndarray:
    """Target load share of each expert: Zipf(s) over a seeded random expert order."""
    order = _rng(seed, _S_ORDER).permutation(E)
    p = 1.0 / np.arange(1, E + 1, dtype=np.float64) ** s
    p /= p.sum()
    shares = np.empty(E, dtype=np.float64)
    shares[order] = p
    return shares


def _calibrate_bias(target: np.ndarray, seed: int, n_mc: int = 131072, iters: int = 16) -> np.ndarray:
    """Biases b such that argmax_e(z_e + b_e), z ~ N(0, I), picks expert e with probability
    target[e].  The router's logits x.W_g are close to i.i.d. N(0,1) for x ~ N(0, I) and
    W_g ~ N(0, 1/d), so this discrete-choice calibration on plain Gaussian noise gives the
    first-choice loads their Zipf shape without evaluating the router here."""
    E = target.shape[0]
    z = _rng(seed, _S_MC).standard_normal(size=(n_mc, E), dtype=np.float32)
    lt = np.log(target)
    b = lt.copy()
    for _ in range(iters):
        pick = np.argmax(z + b.astype(np.float32), axis=1)
        h = np.bincount(pick, minlength=E).astype(np.float64) / n_mc
        # Gaussian tails react to a bias shift about z ~ 2-3 times as strongly as the
        # log-share asks for, so the fixed point needs a step well below 1/z
        b += 0.3 * (lt - np.log(np.maximum(h, 0.25 / n_mc)))
        b -= b.max()
    return b


def _hot_bias(wl: MoEWorkload, seed: int, n_mc: int = 131072) -> np.ndarray:
    """One seeded-chosen expert in ~hot_top2 of the tokens' top-2 (so ~hot_top2/2 of all
    assignments); the other experts share the rest Zipf(s) over a seeded order."""
    E = wl.E
    r = _rng(seed, _S_ORDER)
    hot = int(r.integers(E))
    rest = np.array([e for e in range(E) if e != hot])
    order = r.permutation(E - 1)
    p = 1.0 / np.arange(1, E, dtype=np.float64) ** wl.zipf_s
    p /= p.sum()
    tgt = np.empty(E - 1)
    tgt[order] = p
    b_rest = _calibrate_bias(tgt, seed, n_mc=n_mc)
    z = _rng(seed, _S_MC + 100).standard_normal(size=(n_mc, E), dtype=np.float32)
    b = np.zeros(E)
    b[rest] = b_rest
    lo, hi = -5.0, 15.0
    for _ in range(40):   # bisection on the hot expert's bias
        mid = 0.5 * (lo + hi)
        b[hot] = mid
        l = z + b.astype(np.float32)
        second = np.partition(l, E - 2, axis=1)[:, E - 2]
        frac = float(np.mean(l[:, hot] >= second))
        if frac < wl.hot_top2:
            lo = mid
        else:
            hi = mid
    b[hot] = 0.5 * (lo + hi)
    return b


def router_bias(wl: MoEWorkload, seed: Optional[int] = None) -> np.ndarray:
    seed = wl.seed() if seed is None else seed
    if wl.skew == "c1bias":
        return (1.5 * np.log(1.0 / (np.arange(wl.E, dtype=np.float64) + 1.0))).astype(np.float32)
    if wl.skew == "uniform" or wl.skew == "ids":
        return np.zeros(wl.E, dtype=np.float32)
    if wl.skew == "zipf":
        return _calibrate_bias(zipf_shares(wl.E, wl.zipf_s, seed), seed).astype(np.float32)
    if wl.skew == "hot":
        return _hot_bias(wl, seed).astype(np.float32)
    raise ValueError(wl.skew)


# ----------------------------------------------------------------------------- pre-routed ids
def routed_ids(wl: MoEWorkload, seed: Optional[int] = None) -> np.ndarray:
    """Expert id of each incoming token for the pre-routed workload: the local group
    [0, n_local) gets 1 - foreign_share of the tokens, the foreign group the rest, each group
    Zipf(s) over its own seeded order; ids are sampled independently per token."""
    seed = wl.seed() if seed is None else seed
    r = _rng(seed, _S_IDS)
    nl, nf = wl.n_local, wl.E - wl.n_local
    p = np.empty(wl.E)
    for lo, n, share in ((0, nl, 1.0 - wl.foreign_share), (nl, nf, wl.foreign_share)):
        z = 1.0 / np.arange(1, n + 1, dtype=np.float64) ** wl.zipf_s
        z *= share / z.sum()
        p[lo + r.permutation(n)] = z
    return r.choice(wl.E, size=wl.T, p=p).astype(np.int32)


def alpha_skew_ids(T: int, E: int, alpha: float, n_hot: int, seed: int) -> np.ndarray:
    """The paper's synthetic skew (section 5.1): the first n_hot experts share probability
    alpha evenly, the others share 1 - alpha evenly; ids sampled independently per token."""
    p = np.empty(E)
    p[:n_hot] = alpha / n_hot
    p[n_hot:] = (1.0 - alpha) / max(E - n_hot, 1)
    if n_hot == E:
        p[:] = 1.0 / E
    return _rng(seed, _S_IDS + 1).choice(E, size=T, p=p).astype(np.int32)


# ----------------------------------------------------------------------------- tensors
def activations(wl: MoEWorkload, seed: Optional[int] = None) -> np.ndarray:
    seed = wl.seed() if seed is None else seed
    return _normal(seed, _S_X, (wl.T, wl.d), 1.0, wl.dtype)


def router_weights(wl: MoEWorkload, seed: Optional[int] = None) -> np.ndarray:
    seed = wl.seed() if seed is None else seed
    return _normal(seed, _S_WG, (wl.d, wl.E), wl.d ** -0.5, wl.dtype)


def expert_weights(wl: MoEWorkload, e: int, seed: Optional[int] = None) -> Dict[str, np.ndarray]:
    """One expert's matrices in the paper's orientation.  ReLU: W1 [d,F], W2 [F,d].
    SwiGLU: Wg, Wu [d,F], Wd [F,d].  N(0, 1/fan_in)."""
    seed = wl.seed() if seed is None else seed
    d, F = wl.d, wl.F
    if wl.act == "relu":
        return {"W1": _normal(seed, _S_W + 3 * e, (d, F), d ** -0.5, wl.dtype),
                "W2": _normal(seed, _S_W + 3 * e + 1, (F, d), F ** -0.5, wl.dtype)}
    return {"Wg": _normal(seed, _S_W + 3 * e, (d, F), d ** -0.5, wl.dtype),
            "Wu": _normal(seed, _S_W + 3 * e + 1, (d, F), d ** -0.5, wl.dtype),
            "Wd": _normal(seed, _S_W + 3 * e + 2, (F, d), F ** -0.5, wl.dtype)}


def shared_expert_weights(wl: MoEWorkload, seed: Optional[int] = None) -> Dict[str, np.ndarray]:
    seed = wl.seed() if seed is None else seed
    d, F = wl.d, wl.shared_F
    return {"Wg": _normal(seed, _S_SHARED, (d, F), d ** -0.5, wl.dtype),
            "Wu": _normal(seed, _S_SHARED + 1, (d, F), d ** -0.5, wl.dtype),
            "Wd": _normal(seed, _S_SHARED + 2, (F, d), F ** -0.5, wl.dtype)}


def all_expert_weights(wl: MoEWorkload, seed: Optional[int] = None, threads: int = 8) -> Dict[str, np.ndarray]:
    """Stacked [E, ...] arrays of every expert's matrices (drawn in parallel, one stream each)."""
    seed = wl.seed() if seed is None else seed
    with ThreadPoolExecutor(max_workers=threads) as ex:
        per = list(ex.map(lambda e: expert_weights(wl, e, seed), range(wl.E)))
    return {name: np.stack([p[name] for p in per]) for name in per[0]}


def make_inputs(wl: MoEWorkload, seed: Optional[int] = None, weights: bool = True) -> Dict[str, np.ndarray]:
    """Everything one layer forward needs: x, W_g, b (or ids for the pre-routed workload) and,
    if asked, the stacked expert weights and the shared expert."""
    seed = wl.seed() if seed is None else seed
    out: Dict[str, np.ndarray] = {"x": activations(wl, seed)}
    if wl.skew == "ids":
        out["ids"] = routed_ids(wl, seed)
    else:
        out["W_g"] = router_weights(wl, seed)
        out["b"] = router_bias(wl, seed)
    if weights:
        out.update(all_expert_weights(wl, seed))
        if wl.shared_F:
            out.update({"s" + n: a for n, a in shared_expert_weights(wl, seed).items()})
    return out
