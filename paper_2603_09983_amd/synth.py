"""Seeded synthetic inputs for the verify-step MoE layer.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests/bench.  It draws random tensors, rounds them to bf16 bit
patterns, builds slot tables and packs slot-major weight pools.  It holds none
of the layer's arithmetic, with one stated exception: to honour the "top-k
logit margin" requirement of the workloads it evaluates the router logits with
a library fp64 matmul and uses them ONLY to accept or reject a candidate hidden
row (and to scale the Zipf router bias).  No expected value is ever derived
from that.

Shapes follow the paper's notation (Sec. 2.2): T tokens in the verification
batch (gamma draft + 1 bonus), hidden size H (the paper's d), E routed experts
(the paper's N), top-k, expert FFN width F, and the cache capacity C (number
of HBM-resident expert slots, App. D).
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Sequence

import numpy as np

MARGIN = 1e-3  # minimum gap between adjacent sorted logits among the top k+1


@dataclass(frozen=True)
class Shape:
    T: int
    H: int
    E: int
    k: int
    F: int
    C: int
    n_shared: int = 0
    F_shared: int = 0


@dataclass(frozen=True)
class Recipe:
    """One workload: shape plus the distributions that fill it."""
    name: str
    shape: Shape
    seed: int
    w_std: float = 0.02          # expert / shared weights, bf16(N(0, w_std))
    router_std: float = 0.05     # router weight, fp32 N(0, router_std)
    hidden: str = "n002"         # "n002": bf16(N(0,0.02)); "unit": bf16(N(0,1)/sqrt(H))
    residency: str = "uniform"   # "all" | "uniform" | "zipf"
    zipf_s: float = 0.0          # >0: router bias and residency follow Zipf(s)


RECIPES: Dict[str, Recipe] = {
    # tiny verify step (all experts resident)
    "cfg1": Recipe("cfg1", Shape(T=5, H=256, E=8, k=2, F=512, C=8), seed=0, residency="all"),
    # small-MoE verify step: 64 experts, top-6, 2 shared experts, half-size cache
    "cfg2": Recipe("cfg2", Shape(T=9, H=2048, E=64, k=6, F=1408, C=32, n_shared=2, F_shared=1408),
                   seed=2),
    # fine-grained MoE, Zipf-skewed routing and residency, one wide shared expert
    "cfg3": Recipe("cfg3", Shape(T=5, H=2048, E=60, k=4, F=1408, C=24, n_shared=1, F_shared=5632),
                   seed=3, residency="zipf", zipf_s=1.1),
    # large experts, all resident / half resident
    "cfg4_c8": Recipe("cfg4_c8", Shape(T=8, H=4096, E=8, k=2, F=14336, C=8), seed=4,
                      hidden="unit", residency="all"),
    "cfg4_c4": Recipe("cfg4_c4", Shape(T=8, H=4096, E=8, k=2, F=14336, C=4), seed=4,
                      hidden="unit"),
}

SWEEP_T = (1, 5, 9, 17, 33, 64, 128)
SWEEP_LAYERS = 24


def sweep_recipe(T: int, layer: int) -> Recipe:
    """Batched verification sweep: layer `layer` of 24 independent layers."""
    return Recipe(f"cfg5_T{T}_L{layer}", Shape(T=T, H=2048, E=64, k=6, F=1408, C=48),
                  seed=5000 + layer)


def sweep_hidden_seed(T: int) -> int:
    return 5900 + T


# --------------------------------------------------------------------------
# bf16 bit handling (data formatting only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_bf16(seed_seq: Sequence[int], n: int, std: float) -> np.ndarray:
    rng = np.random.default_rng(list(seed_seq))
    x = rng.standard_normal(n, dtype=np.float32)
    x *= np.float32(std)
    return f32_to_bf16_bits(x)


# stream tags keep the per-tensor random streams apart
_TAG_ROUTER, _TAG_HIDDEN, _TAG_EXPERT, _TAG_SHARED, _TAG_RESIDENT, _TAG_ZIPF = 11, 12, 13, 14, 15, 16


def expert_weights(seed: int, e: int, H: int, F: int, std: float = 0.02):
    """(gate[F,H], up[F,H], down[H,F]) bf16 bit patterns of routed expert e."""
    g = _normal_bf16((seed, _TAG_EXPERT, e, 0), F * H, std).reshape(F, H)
    u = _normal_bf16((seed, _TAG_EXPERT, e, 1), F * H, std).reshape(F, H)
    d = _normal_bf16((seed, _TAG_EXPERT, e, 2), H * F, std).reshape(H, F)
    return g, u, d


def shared_weights(seed: int, s: int, H: int, Fs: int, std: float = 0.02):
    g = _normal_bf16((seed, _TAG_SHARED, s, 0), Fs * H, std).reshape(Fs, H)
    u = _normal_bf16((seed, _TAG_SHARED, s, 1), Fs * H, std).reshape(Fs, H)
    d = _normal_bf16((seed, _TAG_SHARED, s, 2), H * Fs, std).reshape(H, Fs)
    return g, u, d


def router_weight(seed: int, E: int, H: int, std: float = 0.05) -> np.ndarray:
    rng = np.random.default_rng([seed, _TAG_ROUTER])
    return (rng.standard_normal((E, H), dtype=np.float32) * np.float32(std)).astype(np.float32)


def zipf_popularity(seed: int, E: int, s: float) -> np.ndarray:
    """p_e proportional to rank_e^-s with a seeded rank permutation."""
    rng = np.random.default_rng([seed, _TAG_ZIPF])
    rank = rng.permutation(E) + 1
    p = rank.astype(np.float64) ** (-s)
    return p / p.sum()


def _margin_logits(x_bits: np.ndarray, router_w: np.ndarray, bias: Optional[np.ndarray]) -> np.ndarray:
    # accept/reject filter only (see module docstring)
    s = bf16_bits_to_f32(x_bits).astype(np.float64) @ router_w.astype(np.float64).T
    if bias is not None:
        s = s + bias.astype(np.float64)
    return s


def margin_ok(logit_row: np.ndarray, k: int, margin: float = MARGIN) -> bool:
    srt = np.sort(logit_row)[::-1]
    top = srt[: min(k + 1, srt.size)]
    return bool(np.all(top[:-1] - top[1:] >= margin)) if top.size > 1 else True


def hidden_states(seed: int, T: int, H: int, mode: str, router_w: np.ndarray,
                  bias: Optional[np.ndarray], k: int, margin: float = MARGIN) -> np.ndarray:
    """[T,H] bf16 bit patterns; each row is redrawn until its top-(k+1) sorted
    logits are pairwise at least `margin` apart."""
    out = np.empty((T, H), dtype=np.uint16)
    scale = 0.02 if mode == "n002" else 1.0 / np.sqrt(H)
    for t in range(T):
        rng = np.random.default_rng([seed, _TAG_HIDDEN, t])
        for _ in range(10000):
            row = f32_to_bf16_bits(rng.standard_normal(H, dtype=np.float32) * np.float32(scale))
            if margin <= 0 or margin_ok(_margin_logits(row[None, :], router_w, bias)[0], k, margin):
                break
        else:  # pragma: no cover
            raise RuntimeError("could not satisfy the logit margin")
        out[t] = row
    return out


def zipf_router_bias(seed: int, H: int, mode: str, router_w: np.ndarray, p: np.ndarray) -> np.ndarray:
    """bias_e = (sigma_s / 1.2825) ln p_e with sigma_s the measured logit std of
    unbiased draws: Gaussian logit noise of std sigma_s is close to a Gumbel of
    scale sigma_s/1.2825, so top-k then samples experts roughly in proportion to p."""
    rng = np.random.default_rng([seed, _TAG_ZIPF, 1])
    scale = 0.02 if mode == "n002" else 1.0 / np.sqrt(H)
    probe = f32_to_bf16_bits(rng.standard_normal((256, H), dtype=np.float32) * np.float32(scale))
    sigma = float(_margin_logits(probe, router_w, None).std())
    return ((sigma / 1.2825) * np.log(p)).astype(np.float32)


def slot_table(seed: int, E: int, C: int, residency: str, p: Optional[np.ndarray] = None) -> np.ndarray:
    """int32[E]: slot of each expert or -1.  Resident experts get distinct slots
    in a seeded random order, so slot id and expert id never coincide by design."""
    rng = np.random.default_rng([seed, _TAG_RESIDENT])
    tab = np.full(E, -1, dtype=np.int32)
    n = min(C, E)
    if residency == "all":
        assert C >= E
        chosen = np.arange(E)
    elif residency == "zipf":
        chosen = rng.choice(E, size=n, replace=False, p=p)
    else:
        chosen = rng.choice(E, size=n, replace=False)
    slots = rng.permutation(C)[: len(chosen)]
    tab[chosen] = slots.astype(np.int32)
    return tab


# --------------------------------------------------------------------------
# whole-layer bundles
# --------------------------------------------------------------------------
@dataclass
class LayerInputs:
    recipe: Recipe
    shape: Shape
    hidden: np.ndarray                 # uint16 [T,H]
    router_w: np.ndarray               # float32 [E,H]
    router_bias: Optional[np.ndarray]  # float32 [E] or None
    slot_table: np.ndarray             # int32 [E]
    # full expert set, indexed by EXPERT id (what the oracle reads); experts
    # that were not generated are all-zero rows and listed in `missing`
    w_gate: np.ndarray                 # uint16 [E,F,H]
    w_up: np.ndarray                   # uint16 [E,F,H]
    w_down: np.ndarray                 # uint16 [E,H,F]
    sh_gate: Optional[np.ndarray]      # uint16 [n_shared,Fs,H]
    sh_up: Optional[np.ndarray]
    sh_down: Optional[np.ndarray]      # uint16 [n_shared,H,Fs]
    missing: List[int] = field(default_factory=list)

    def pools(self):
        """Slot-major pools [C,F,H],[C,F,H],[C,H,F] (what the HIP path reads).
        Empty slots are filled with a bf16 NaN pattern so any read of a slot
        that holds no expert poisons the output."""
        s = self.shape
        pg = np.full((s.C, s.F, s.H), 0x7FC0, dtype=np.uint16)
        pu = np.full((s.C, s.F, s.H), 0x7FC0, dtype=np.uint16)
        pd = np.full((s.C, s.H, s.F), 0x7FC0, dtype=np.uint16)
        for e in range(s.E):
            c = int(self.slot_table[e])
            if c >= 0:
                pg[c], pu[c], pd[c] = self.w_gate[e], self.w_up[e], self.w_down[e]
        return pg, pu, pd


def _n_workers() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def make_layer(recipe: Recipe, hidden_seed: Optional[int] = None, experts: str = "all",
               margin: float = MARGIN) -> LayerInputs:
    """Draw every tensor of one layer.  experts="resident" skips the weights of
    non-resident experts (they are never read by a correct implementation and
    stay zero), which keeps the large workloads quick to build."""
    s = recipe.shape
    rw = router_weight(recipe.seed, s.E, s.H, recipe.router_std)
    bias = None
    p = None
    if recipe.zipf_s > 0:
        p = zipf_popularity(recipe.seed, s.E, recipe.zipf_s)
        bias = zipf_router_bias(recipe.seed, s.H, recipe.hidden, rw, p)
    tab = slot_table(recipe.seed, s.E, s.C, recipe.residency, p)
    hs = recipe.seed if hidden_seed is None else hidden_seed
    hid = hidden_states(hs, s.T, s.H, recipe.hidden, rw, bias, s.k, margin)

    wg = np.zeros((s.E, s.F, s.H), dtype=np.uint16)
    wu = np.zeros((s.E, s.F, s.H), dtype=np.uint16)
    wd = np.zeros((s.E, s.H, s.F), dtype=np.uint16)
    want = [e for e in range(s.E) if experts == "all" or tab[e] >= 0]
    missing = [e for e in range(s.E) if e not in set(want)]

    def fill(e):
        wg[e], wu[e], wd[e] = expert_weights(recipe.seed, e, s.H, s.F, recipe.w_std)

    with ThreadPoolExecutor(_n_workers()) as ex:
        list(ex.map(fill, want))

    sg = su = sd = None
    if s.n_shared > 0:
        sg = np.empty((s.n_shared, s.F_shared, s.H), dtype=np.uint16)
        su = np.empty((s.n_shared, s.F_shared, s.H), dtype=np.uint16)
        sd = np.empty((s.n_shared, s.H, s.F_shared), dtype=np.uint16)
        for i in range(s.n_shared):
            sg[i], su[i], sd[i] = shared_weights(recipe.seed, i, s.H, s.F_shared, recipe.w_std)
    return LayerInputs(recipe, s, hid, rw, bias, tab, wg, wu, wd, sg, su, sd, missing)


def small_recipe(name: str, seed: int, **shape_kw) -> Recipe:
    """Ad-hoc recipe for parity/edge-case tests."""
    residency = shape_kw.pop("residency", "uniform")
    zipf_s = shape_kw.pop("zipf_s", 0.0)
    hidden = shape_kw.pop("hidden", "n002")
    sh = Shape(**shape_kw)
    if residency == "all" and sh.C < sh.E:
        residency = "uniform"
    return Recipe(name, sh, seed, residency=residency, zipf_s=zipf_s, hidden=hidden)


def with_T(recipe: Recipe, T: int) -> Recipe:
    return replace(recipe, shape=replace(recipe.shape, T=T))
