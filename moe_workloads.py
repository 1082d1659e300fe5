"""Seeded synthetic workloads for one GPU's share of an expert-parallel MoE layer.

This module only *draws inputs*: shapes, seeds, random tensors, storage rounding
and the expert-to-rank placement arrays of the five benchmark configurations.
It contains none of the layer's arithmetic (no gating, packing, FFN or combine),
so that the CPU oracle and the HIP path can both take their inputs from here
without sharing any code of the method itself.

Recipe (one `numpy.random.default_rng(seed)` stream, fp32 draws, in this order):
    x  [T,d]  ~ N(0,1)
    Wg [E,d]  ~ N(0,1/d)
    for e in 0..E-1: W1[e] [f,d] ~ N(0,1/d)
    for e in 0..E-1: W3[e] [f,d] ~ N(0,1/d)
    for e in 0..E-1: W2[e] [d,f] ~ N(0,1/f)
    dOut [T,d] ~ N(0,1)            (training configuration only; its own stream,
                                    default_rng(seed + 7919), so that cases which
                                    skip the weights draw the same gradient)
Every tensor is then rounded to the configuration's storage type (bf16:
round-to-nearest-even on the fp32 bit pattern) and both sides see exactly the
stored values.

The placement arrays follow the expert-parallel setting of the paper (Sec. 2.1,
"Expert Parallelism"; Sec. 3.2 "Relationships between Two Communications"):
expert e lives on virtual rank e // (E/R); an expert that was migrated to the
local rank (fetched by all-gather) is computed locally, so its destination rank
becomes the local rank.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class MoEConfig:
    name: str
    seed: int
    dtype: str            # "f32" or "bf16": storage type of x, weights, outputs
    T: int                # tokens on this GPU
    d: int                # d_model
    E: int                # experts
    k: int                # top-k
    f: int                # ffn_dim
    R: int                # virtual ranks
    local_rank: int = 0
    migrated: Tuple[int, ...] = ()    # experts fetched to the local rank
    all_resident: bool = False        # every expert computed locally
    bias_scale: float = 0.0           # per-expert gate bias b_e = bias_scale*ln(1/(e+1))
    backward: bool = False
    gated: bool = True                # False: the paper's two-matrix expert (no W3)

    @property
    def S(self) -> int:
        return self.T * self.k


CONFIGS: Dict[str, MoEConfig] = {
    "tiny": MoEConfig("tiny", 1001, "f32", T=256, d=128, E=8, k=2, f=256, R=2),
    "small": MoEConfig("small", 1002, "bf16", T=4096, d=1024, E=16, k=2, f=4096, R=4,
                       migrated=(5, 9)),
    "mixtral": MoEConfig("mixtral", 1003, "bf16", T=8192, d=4096, E=8, k=2, f=14336, R=8,
                         all_resident=True),
    "finegrained": MoEConfig("finegrained", 1004, "bf16", T=16384, d=2048, E=64, k=6, f=1408,
                             R=8, migrated=(8, 9, 10, 11), bias_scale=1.2),
    "train": MoEConfig("train", 1005, "bf16", T=8192, d=2048, E=32, k=4, f=2048, R=8,
                       migrated=(5, 9), backward=True),
}
# Not one of the five configurations of the benchmark spec: a layer of the paper's own sweep
# (Table 3: E = 32, H = 1024, M = 4096, K = 2, B*L = 16*512 tokens) with its two-matrix expert.
CONFIGS["paper"] = MoEConfig("paper", 1006, "bf16", T=8192, d=1024, E=32, k=2, f=4096, R=8,
                             migrated=(4, 5, 6, 7), gated=False)
# ... and its training step (forward + backward of the same layer)
CONFIGS["paper_train"] = replace(CONFIGS["paper"], name="paper_train", backward=True)
CONFIG_ORDER = ["tiny", "small", "mixtral", "finegrained", "train"]


def scaled(cfg: MoEConfig, **kw) -> MoEConfig:
    """A copy of `cfg` with some sizes replaced (used for reduced test cases)."""
    return replace(cfg, **kw)


# ---------------------------------------------------------------- storage types
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even), returned as uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact upcast of bf16 bit patterns (uint16) to fp32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def store(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round an fp32 array to the storage type: fp32 array or uint16 bf16 bits."""
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    raise ValueError(dtype)


def stored_to_f32(a: np.ndarray, dtype: str) -> np.ndarray:
    """The exact values a stored array holds, as fp32."""
    return a if dtype == "f32" else bf16_bits_to_f32(a)


# ------------------------------------------------------------------- placement
def home_rank(cfg: MoEConfig) -> np.ndarray:
    per = cfg.E // cfg.R
    return (np.arange(cfg.E, dtype=np.int32) // max(per, 1)).astype(np.int32)


def expert_dest_rank(cfg: MoEConfig) -> np.ndarray:
    """dest_rank[e]: the virtual rank whose buffer the tokens of expert e go to.
    dest_rank[e] == local_rank means expert e is resident (home or migrated)."""
    if cfg.all_resident:
        return np.full(cfg.E, cfg.local_rank, dtype=np.int32)
    dest = home_rank(cfg)
    for e in cfg.migrated:
        dest[e] = cfg.local_rank
    return dest


def resident_experts(cfg: MoEConfig) -> List[int]:
    dest = expert_dest_rank(cfg)
    return [int(e) for e in range(cfg.E) if dest[e] == cfg.local_rank]


def gate_bias(cfg: MoEConfig) -> Optional[np.ndarray]:
    if cfg.bias_scale == 0.0:
        return None
    e = np.arange(cfg.E, dtype=np.float64)
    return (cfg.bias_scale * np.log(1.0 / (e + 1.0))).astype(np.float32)


# ---------------------------------------------------------------------- inputs
@dataclass
class MoEInputs:
    cfg: MoEConfig
    x: np.ndarray                 # stored [T,d]
    Wg: np.ndarray                # stored [E,d]
    bias: Optional[np.ndarray]    # fp32 [E] or None
    W1: List[Optional[np.ndarray]] = field(default_factory=list)   # stored [f,d] or None
    W3: List[Optional[np.ndarray]] = field(default_factory=list)
    W2: List[Optional[np.ndarray]] = field(default_factory=list)   # stored [d,f] or None
    dOut: Optional[np.ndarray] = None
    dest_rank: Optional[np.ndarray] = None


def make_inputs(cfg: MoEConfig, experts: str = "all") -> MoEInputs:
    """Draw the inputs of `cfg`.

    experts = "all": weights for every expert (loopback tests run all segments);
              "resident": only the resident experts keep their weights (the
              others are drawn, to keep the stream position, and dropped);
              "none": no expert weights (routing/dispatch-only cases)."""
    rng = np.random.default_rng(cfg.seed)
    T, d, E, f = cfg.T, cfg.d, cfg.E, cfg.f
    x = store(rng.standard_normal((T, d), dtype=np.float32), cfg.dtype)
    Wg = store(rng.standard_normal((E, d), dtype=np.float32) * np.float32(1.0 / np.sqrt(d)),
               cfg.dtype)
    inp = MoEInputs(cfg=cfg, x=x, Wg=Wg, bias=gate_bias(cfg), dest_rank=expert_dest_rank(cfg))
    keep = set(range(E)) if experts == "all" else \
        set(resident_experts(cfg)) if experts == "resident" else set()
    if experts != "none":
        for name, shape, fan_in in (("W1", (f, d), d), ("W3", (f, d), d), ("W2", (d, f), f)):
            lst = getattr(inp, name)
            if name == "W3" and not cfg.gated:   # two-matrix expert: nothing drawn for W3
                lst.extend([None] * E)
                continue
            s = np.float32(1.0 / np.sqrt(fan_in))
            for e in range(E):
                w = rng.standard_normal(shape, dtype=np.float32)
                if e in keep:
                    w *= s
                    lst.append(store(w, cfg.dtype))
                else:
                    lst.append(None)
                del w
    else:
        inp.W1 = [None] * E
        inp.W3 = [None] * E
        inp.W2 = [None] * E
    if cfg.backward:
        inp.dOut = store(np.random.default_rng(cfg.seed + 7919)
                         .standard_normal((T, d), dtype=np.float32), cfg.dtype)
    return inp


def random_logits(T: int, E: int, seed: int, ties: bool = False) -> np.ndarray:
    """fp32 logits for selection tests. ties=True quantises them so that many
    exact ties occur (exercises the lower-id-first rule)."""
    rng = np.random.default_rng(seed)
    L = rng.standard_normal((T, E), dtype=np.float32)
    if ties:
        L = np.round(L * 2.0) / 2.0
    return L.astype(np.float32)


def random_routing(T: int, E: int, k: int, seed: int, skew: float = 0.0) -> np.ndarray:
    """Random distinct top-k expert ids per token [T,k] int32 (for dispatch tests
    that do not go through gating). skew>0 biases towards low expert ids."""
    rng = np.random.default_rng(seed)
    g = rng.standard_normal((T, E)) - skew * np.log(np.arange(E) + 1.0)[None, :]
    return np.argsort(-g, axis=1, kind="stable")[:, :k].astype(np.int32)


# ------------------------------------------------------------ shared/residual compression
def make_sr_inputs(shape: Tuple[int, int], seed: int, dtype: str, n_experts: int = 2,
                   ties: bool = False):
    """Weights for the shared/residual expert compression (paper Sec. 4.2): a shared
    expert and `n_experts` experts that differ from it by a residual concentrated in few
    entries (Fig. "SRexpert"(a): the residuals' distribution is much narrower than the
    weights', the differences sit in a small number of parameters).

    Recipe (one default_rng(seed) stream, fp32 draws): shared [rows, cols] ~ N(0, 1/cols);
    per expert: a dense part ~ N(0, (0.05)^2 / cols) and, on a random 2 % of the entries, a
    large part ~ N(0, 1/cols) added on top; expert = shared + residual.  With `ties`, the
    residual is quantised to multiples of 2^-7/sqrt(cols) so that many magnitudes are equal.
    Everything is rounded to the storage type; returns (shared, [experts]) as stored arrays.
    """
    rows, cols = shape
    rng = np.random.default_rng(seed)
    sd = 1.0 / np.sqrt(cols)
    shared = (rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(sd)).astype(np.float32)
    experts = []
    for _ in range(n_experts):
        res = rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(0.05 * sd)
        big = rng.random((rows, cols), dtype=np.float32) < np.float32(0.02)
        res = res + big * (rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(sd))
        if ties:
            q = np.float32(sd / 128.0)
            res = np.round(res / q) * q
        experts.append(store((shared + res).astype(np.float32), dtype))
    return store(shared, dtype), experts
