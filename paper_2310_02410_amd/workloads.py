"""Seeded synthetic MoE layers and token batches (numpy only).

This module only draws random inputs; it holds none of the method's
arithmetic (no quantizer, no router, no FFN) and is the one module both the
tests' CPU reference and the HIP path are fed from.

The layers take the shapes the paper reports for its translation MoE
(App. B "Model architecture": d_model 1024, d_ff 4096, 32 experts, top-1
gating; Table 1: batch 24) and the distributional facts it reports for expert
weights (zero mean, skew ~ 0: App. E Table "skewness"; outliers stretch the
scale: Sec. 2.1).  They stand in for the trained model and its corpora, which
are not available.

Draw order inside a layer (one numpy Generator, PCG64): for each expert in
order W1, b1, W2, b2; then W_g.  Tokens come from their own Generator.

Router inputs sit on a binary lattice: x is a multiple of 2^-4 and W_g a
multiple of 2^-9 (the bias row of 2^-6), both small enough that every product
and every partial sum of a logit is exactly representable in fp32 (and fp64).
The logits are therefore the same numbers in any summation order, so the
top-1 expert of every token is unique up to exact ties, which the lowest
index breaks.  The lattice changes N(0,1) by a rounding of at most 2^-5.
"""

from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

SIGMA_W = 0.02          # expert weight std
SIGMA_B = 0.01          # bias std
OUTLIER_SIGMAS = 8.0    # planted outliers at +-8 sigma


@dataclass(frozen=True)
class Workload:
    name: str
    E: int
    d: int
    f: int
    T: int
    bits: tuple
    seed: int
    outlier_prob: float = 0.0
    routing: str = "uniform"     # "uniform" | "zipf"
    zipf_s: float = 1.1
    n_empty: int = 0             # experts forced empty under zipf routing
    layers: int = 1


# The five benchmark configurations.
CONFIGS = {
    "c0": Workload("c0", E=4, d=64, f=256, T=32, bits=(4,), seed=0),
    "c1": Workload("c1", E=32, d=1024, f=4096, T=24, bits=(4,), seed=1, outlier_prob=1e-3),
    "c2": Workload("c2", E=32, d=1024, f=4096, T=24, bits=(3, 2), seed=2, outlier_prob=1e-3),
    "c3": Workload("c3", E=32, d=1024, f=4096, T=1536, bits=(4,), seed=3, outlier_prob=1e-3,
                   routing="zipf", n_empty=4),
    "c4": Workload("c4", E=32, d=1024, f=4096, T=24, bits=(2,), seed=4, outlier_prob=1e-3,
                   layers=12),
}


# Shapes beyond the five configurations: the paper's second model (App. B: 128 experts,
# d_model 768, d_ff 3072) and a dense FFN (one expert) run through the same calls, at batch 24.
EXTRA = {
    "n2_e128": Workload("n2_e128", E=128, d=768, f=3072, T=24, bits=(4,), seed=5, outlier_prob=1e-3),
    "n2_dense": Workload("n2_dense", E=1, d=1024, f=4096, T=24, bits=(4,), seed=6, outlier_prob=1e-3),
    # the largest batch the decode-sized kernels take (64 tokens), uniform and Zipf(1.1) load
    "c1_T64": Workload("c1_T64", E=32, d=1024, f=4096, T=64, bits=(4,), seed=7, outlier_prob=1e-3),
    "c1_T64_zipf": Workload("c1_T64_zipf", E=32, d=1024, f=4096, T=64, bits=(4,), seed=8, outlier_prob=1e-3,
                            routing="zipf", n_empty=4),
}


def c4_variants():
    """Config 4 runs at T in {24, 4096} with uniform and Zipf(1.1) routing."""
    base = CONFIGS["c4"]
    out = []
    for T in (24, 4096):
        for routing in ("uniform", "zipf"):
            out.append(replace(base, name=f"c4_T{T}_{routing}", T=T, routing=routing,
                               n_empty=4 if routing == "zipf" else 0))
    return out


def zipf_probs(E: int, s: float, n_empty: int, rng) -> np.ndarray:
    """Target load: a seeded random ranking of the experts, p_rank ~ rank^-s over
    the first E - n_empty ranks, the last n_empty ranks get probability 0."""
    ranking = rng.permutation(E)
    live = E - n_empty
    p = np.zeros(E)
    w = np.arange(1, live + 1, dtype=np.float64) ** (-s)
    p[ranking[:live]] = w / w.sum()
    return p


def _calibrate_bias(p_target: np.ndarray, sigma_logit: float, seed: int) -> np.ndarray:
    """Bias row beta (multiples of 2^-6) such that argmax_e(beta_e + z_e), with
    z_e iid N(0, sigma_logit^2), lands on e with probability ~ p_target.
    Fitted on a seeded Gaussian sample - a statistical model of the load, the
    real logits are never formed here.  Zero-probability experts get -50."""
    rng = np.random.default_rng([seed, 0xCA11B])
    E = p_target.size
    live = p_target > 0
    z = rng.standard_normal((8192, E)) * sigma_logit
    beta = np.where(live, 0.0, -50.0)
    for _ in range(300):
        hit = np.bincount(np.argmax(z + beta, axis=1), minlength=E) / z.shape[0]
        step = np.log(p_target[live]) - np.log(np.maximum(hit[live], 0.25 / z.shape[0]))
        beta[live] += 0.3 * sigma_logit * step
        beta[live] -= beta[live].max()
    beta[live] = np.clip(np.rint(beta[live] * 64.0) / 64.0, -15.0, 0.0)
    return beta


def make_layer(wl: Workload, layer: int = 0, zipf_gate: bool = False, lattice: bool = True) -> dict:
    """One MoE layer: fp32 'w1' [E,d,f], 'w2' [E,f,d]; fp16 'b1' [E,f], 'b2' [E,d];
    fp16 'w_gate' [d,E].  With zipf_gate a uniform-routing workload also gets
    'w_gate_zipf': the same router with the Zipf bias row (4 experts empty), so that one
    set of expert weights serves both load shapes.  lattice=False: W_g ~ N(0, 0.02) cast
    straight to fp16 (same draws, no rounding to the 2^-9 lattice)."""
    rng = np.random.default_rng([wl.seed, 1000 + layer])
    E, d, f = wl.E, wl.d, wl.f
    w1 = np.empty((E, d, f), dtype=np.float32)
    w2 = np.empty((E, f, d), dtype=np.float32)
    b1 = np.empty((E, f), dtype=np.float16)
    b2 = np.empty((E, d), dtype=np.float16)

    def matrix(K, N):
        a = rng.standard_normal((K, N), dtype=np.float32) * np.float32(SIGMA_W)
        if wl.outlier_prob > 0.0:
            cnt = int(rng.binomial(K * N, wl.outlier_prob))
            pos = rng.choice(K * N, size=cnt, replace=False)
            sign = rng.integers(0, 2, size=cnt).astype(np.float32) * 2.0 - 1.0
            a.reshape(-1)[pos] = sign * np.float32(OUTLIER_SIGMAS * SIGMA_W)
        return a

    for e in range(E):
        w1[e] = matrix(d, f)
        b1[e] = (rng.standard_normal(f) * SIGMA_B).astype(np.float16)
        w2[e] = matrix(f, d)
        b2[e] = (rng.standard_normal(d) * SIGMA_B).astype(np.float16)

    wg = rng.standard_normal((d, E)) * SIGMA_W
    if lattice:
        wg = np.clip(np.rint(wg * 512.0), -96, 96) / 512.0
    out = dict(w1=w1, b1=b1, w2=w2, b2=b2)
    if wl.routing == "zipf":
        p = zipf_probs(E, wl.zipf_s, wl.n_empty, rng)
        wg[0, :] = _calibrate_bias(p, SIGMA_W * np.sqrt(d - 1.0), wl.seed * 131 + layer)
    elif wl.routing != "uniform":
        raise ValueError(f"unknown routing {wl.routing!r}")
    elif zipf_gate:
        p = zipf_probs(E, wl.zipf_s, 4, rng)
        wz = wg.copy()
        wz[0, :] = _calibrate_bias(p, SIGMA_W * np.sqrt(d - 1.0), wl.seed * 131 + layer)
        out["w_gate_zipf"] = wz.astype(np.float16)
    out["w_gate"] = wg.astype(np.float16)
    return out


def make_tokens(wl: Workload, lattice: bool = True) -> np.ndarray:
    """fp16 activations [T,d] ~ N(0,1) on the 2^-4 lattice; under zipf routing
    feature 0 is the constant 1 that the router's bias row multiplies.
    lattice=False: the same draws cast straight to fp16."""
    rng = np.random.default_rng([wl.seed, 7])
    x = rng.standard_normal((wl.T, wl.d))
    if lattice:
        x = np.clip(np.rint(x * 16.0), -112, 112) / 16.0
    if wl.routing == "zipf":
        x[:, 0] = 1.0
    return x.astype(np.float16)


def small(name: str = "small", **kw) -> Workload:
    """A reduced layer for quick tests; keyword overrides."""
    base = Workload(name, E=8, d=128, f=256, T=37, bits=(4, 3, 2), seed=11, outlier_prob=1e-3)
    return replace(base, **kw)
