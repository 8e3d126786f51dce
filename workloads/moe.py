"""Seeded synthetic inputs for the sparsely gated mixture-of-experts layer (configs 3-4).

The paper's MoE experiment only fixes "n experts, k active per example, one
hidden layer"; sizes, the noisy top-k gate and the Zipf-shaped expert load come
from the benchmark configurations.  Everything is bf16-representable float32 on
the host (the oracle consumes it as is, the HIP path as bf16 bit patterns).

Load shaping.  With zero-mean tokens and a bias-free linear gate no expert can be
selected by much more than half of the tokens, yet Zipf(s=1.2) over ~1000 experts
with k=4 asks the head expert for ~92 % of them.  Tokens therefore carry a shared
component, x_t = sqrt(1-rho) z_t + sqrt(rho) c  (z_t, c ~ N(0,1) i.i.d., so each
entry is still marginally N(0,1)), and every gate column gets a multiple of c
added: Wg[:,e] = G[:,e] + beta_e c/|c|^2.  The shifts beta_e are calibrated on
the host by a few multiplicative-style updates until the routed histogram
follows the Zipf target.  Experts forced empty get zero Wg and Wn columns and
a constant -64 in their noise column, so their logit is -64 softplus(0) = -44 for
every token, far below every active expert's.  The calibration loop below is input shaping written
with library matmuls; it produces no expected values for any test.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

from .rng import BASE_SEED, bf16_bits, round_bf16, stream

_S_X, _S_C, _S_G, _S_N, _S_NOISE, _S_PERM, _S_EMPTY, _S_W = 1, 2, 3, 4, 5, 6, 7, 8


@dataclass
class MoeWorkload:
    name: str
    seed: int
    T: int
    d: int
    h: int
    E: int
    k: int
    x: np.ndarray         # float32 [T,d]   bf16-representable
    Wg: np.ndarray        # float32 [d,E]   bf16-representable
    Wn: np.ndarray        # float32 [d,E]   bf16-representable
    noise: np.ndarray     # float32 [T,E]
    empty: np.ndarray     # int32 ids of experts forced empty
    target_load: np.ndarray   # float64 [E] Zipf target (assignments per expert)
    meta: dict = field(default_factory=dict)
    _cache: dict = field(default_factory=dict, repr=False)

    @property
    def A(self) -> int:
        return self.T * self.k

    def expert_weights(self, e: int):
        """(W1_e [h,d], W2_e [d,h]) float32, bf16-representable, He-normal; regenerable per expert.

        Layout follows the library's boundary: each output neuron's weights are contiguous
        (W1_e[j,:] produces hidden unit j, W2_e[c,:] produces output channel c).
        """
        g = stream(self.seed, _S_W, e)
        w1 = g.standard_normal((self.h, self.d), dtype=np.float32) * np.float32(np.sqrt(2.0 / self.d))
        w2 = g.standard_normal((self.d, self.h), dtype=np.float32) * np.float32(np.sqrt(2.0 / self.h))
        return round_bf16(w1), round_bf16(w2)

    def all_expert_weights_bits(self, W1_bits: np.ndarray, W2_bits: np.ndarray, threads: int = 8) -> None:
        """Fill uint16 arrays [E,h,d] and [E,d,h] with bf16 bit patterns (threaded: Philox is per expert)."""
        def one(e):
            w1, w2 = self.expert_weights(e)
            W1_bits[e] = bf16_bits(w1)
            W2_bits[e] = bf16_bits(w2)
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(one, range(self.E)))


def zipf_target(E_active: int, A: int, s: float, T: int) -> np.ndarray:
    """Assignments per rank under Zipf(s), capped at T (an expert is used at most once per token)."""
    w = np.arange(1, E_active + 1, dtype=np.float64) ** (-s)
    return np.minimum(w / w.sum() * A, 0.98 * T)


def _route_hist(clean, noisy_part, k, E):
    logits = clean + noisy_part
    idx = np.argpartition(-logits, k - 1, axis=1)[:, :k]
    return np.bincount(idx.ravel(), minlength=E)


def make(name: str, seed: int, T: int, d: int, h: int, E: int, k: int, zipf_s: float,
         empty_frac: float = 0.0, rho: float = 0.25, iters: int = 30) -> MoeWorkload:
    z = stream(seed, _S_X).standard_normal((T, d), dtype=np.float32)
    c = stream(seed, _S_C).standard_normal(d, dtype=np.float32)
    x = round_bf16(np.sqrt(1 - rho, dtype=np.float32) * z + np.sqrt(rho, dtype=np.float32) * c[None, :])
    G = stream(seed, _S_G).standard_normal((d, E), dtype=np.float32) / np.float32(np.sqrt(d))
    Wn = 0.1 * stream(seed, _S_N).standard_normal((d, E), dtype=np.float32) / np.float32(np.sqrt(d))
    noise = stream(seed, _S_NOISE).standard_normal((T, E), dtype=np.float32)

    n_empty = int(np.floor(empty_frac * E))
    empty = np.sort(stream(seed, _S_EMPTY).permutation(E)[:n_empty]).astype(np.int32)
    active = np.setdiff1d(np.arange(E), empty)
    rank_to_expert = active[stream(seed, _S_PERM).permutation(len(active))]
    target = np.zeros(E)
    target[rank_to_expert] = zipf_target(len(active), T * k, zipf_s, T)

    G[:, empty] = 0
    Wn[:, empty] = 0
    noise[:, empty] = -64.0     # times softplus(0) = ln 2: logit -44 for every token
    Wn = round_bf16(Wn)

    # input shaping: shifts beta_e along the shared direction c
    u = c / np.float32(c @ c)
    shift_dir = x @ u                       # [T], close to sqrt(rho)
    xG = x @ G                              # [T,E]
    zn = x @ Wn
    nz = noise * (np.maximum(zn, 0) + np.log1p(np.exp(-np.abs(zn))))
    beta = np.zeros(E, np.float32)
    act_mask = np.zeros(E, bool)
    act_mask[active] = True
    for it in range(iters):
        hist = _route_hist(xG + shift_dir[:, None] * beta[None, :], nz, k, E)
        step = np.log((target + 1.0) / (hist + 1.0))
        beta[act_mask] += (0.7 * step[act_mask]).astype(np.float32)
    Wg = round_bf16(G + u[:, None] * beta[None, :])
    hist = _route_hist(x @ Wg, nz, k, E)
    assert (hist[empty] == 0).all() and E - n_empty >= k
    meta = {"zipf_s": zipf_s, "rho": rho, "host_load_hist_max": int(hist.max()),
            "host_load_hist_empty": int((hist == 0).sum())}
    return MoeWorkload(name, seed, T, d, h, E, k, x, Wg, Wn, noise, empty, target, meta)


def config3(seed: int = BASE_SEED * 10 + 3, **kw) -> MoeWorkload:
    """4096 tokens, d=512, 256 experts 512->1024->512, top-2, Zipf(1.1)."""
    a = dict(T=4096, d=512, h=1024, E=256, k=2, zipf_s=1.1)
    a.update(kw)
    return make("cfg3-moe-bf16", seed, **a)


def config4(seed: int = BASE_SEED * 10 + 4, **kw) -> MoeWorkload:
    """16384 tokens, d=1024, 1024 experts 1024->2048->1024, top-4, Zipf(1.2), 5 % empty experts."""
    a = dict(T=16384, d=1024, h=2048, E=1024, k=4, zipf_s=1.2, empty_frac=0.05)
    a.update(kw)
    return make("cfg4-moe-large-bf16", seed, **a)


def small(seed: int, T: int, d: int, h: int, E: int, k: int, zipf_s: float = 1.0,
          empty_frac: float = 0.0) -> MoeWorkload:
    """Small parity workload of arbitrary shape."""
    return make(f"moe-T{T}-d{d}-h{h}-E{E}-k{k}", seed, T, d, h, E, k, zipf_s, empty_frac, iters=20)
