"""Seeded synthetic inputs for the padding-free MoE layer: the one module that both the CPU oracle's tests
and the GPU tests / benchmark draw their tensors from.

This module holds no arithmetic of the method itself (no softmax, no top-k, no GEMM): it only draws random
tensors of the layer's shapes and, for bf16 workloads, rounds them once to bf16 so that both sides consume
bit-identical values.

Shapes follow the paper's model table (Table 3: the "Small" model is H=2048, H_FFN=1408, E=64, k=6; the
"Large" model is H=7168, H_FFN=2048, E=256, k=8).  The paper trains on a corpus that is not available here;
these tensors stand in for one MoE layer's input activations, gate weights and expert weights.

Every tensor is drawn from its own counter-based Philox stream keyed by (seed, tensor id, expert index), so a
single expert's weights can be regenerated anywhere without materialising the whole tensor.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import numpy as np

# tensor ids: fixed, part of the recipe
_TENSOR_IDS = {
    "x": 1, "w_router": 2, "wg": 3, "wu": 4, "wd": 5, "dout": 6,
    "shared_wg": 7, "shared_wu": 8, "shared_wd": 9, "rank_perm": 10, "logits": 11, "w1": 12, "w2": 13, "rbd_key": 14,
}


@dataclasses.dataclass(frozen=True)
class MoEConfig:
    """One MoE-layer workload.  T tokens, d model width (paper: S, H), E routed experts, E_s shared experts
    (always active), k experts per token, f expert FFN width (paper: H_FFN)."""
    name: str
    T: int
    d: int
    E: int
    k: int
    f: int
    dtype: str = "bf16"          # "f32" | "bf16": storage type of activations and weights
    E_s: int = 0
    router_std: Optional[float] = None   # None -> 1/sqrt(d), which makes gate logits ~ N(0,1)
    w_std: float = 0.02
    skew_alpha: float = 0.0      # 0 -> no per-expert bias; else bias[e] = -alpha*1.2*ln(rank_e)
    seed: int = 0
    expert: str = "swiglu"       # "swiglu": three matrices wg, wu, wd; "mlp2": the paper's two matrices w1, w2
    act: str = "gelu"            # activation of the two-matrix expert: identity | gelu | silu

    @property
    def B(self) -> int:
        return self.T * self.k

    def with_T(self, T: int) -> "MoEConfig":
        return dataclasses.replace(self, T=T, name=f"{self.name}-T{T}")


# The five workloads of the benchmark definition, plus reduced shapes for element-by-element parity.
CONFIGS = {
    # config 1: tiny fp32 layer
    "tiny_f32": MoEConfig("tiny_f32", T=256, d=128, E=8, k=2, f=64, dtype="f32", router_std=0.02),
    # config 2: DeepSeek-MoE-16B-shaped layer, near-uniform load
    "dsmoe16b": MoEConfig("dsmoe16b", T=8192, d=2048, E=64, k=6, f=1408, E_s=2),
    # config 3: same, Zipf(s=1.2)-skewed load (alpha chosen by tests/golden/make_skew_alpha.py)
    "dsmoe16b_skew": MoEConfig("dsmoe16b_skew", T=8192, d=2048, E=64, k=6, f=1408, E_s=2, skew_alpha=1.25),
    # config 4: large fine-grained layer
    "large": MoEConfig("large", T=4096, d=7168, E=256, k=8, f=2048, E_s=1),
    # config 5: long-sequence sweep base (T set with .with_T)
    "longseq": MoEConfig("longseq", T=16384, d=2048, E=64, k=6, f=1408, E_s=0),
    # reduced shapes: several tiles plus a ragged tail, small enough for the oracle to finish in seconds
    "mini_bf16": MoEConfig("mini_bf16", T=600, d=256, E=8, k=3, f=192, E_s=1),
    "mini_bf16_skew": MoEConfig("mini_bf16_skew", T=600, d=256, E=8, k=3, f=192, E_s=1, skew_alpha=3.0),
    "mini_f32": MoEConfig("mini_f32", T=200, d=96, E=5, k=2, f=40, dtype="f32", E_s=1, router_std=0.05),
    "odd_f32": MoEConfig("odd_f32", T=77, d=50, E=7, k=3, f=22, dtype="f32", router_std=0.1),
    "odd_bf16": MoEConfig("odd_bf16", T=131, d=72, E=6, k=2, f=24, router_std=0.2),
    "mid_bf16": MoEConfig("mid_bf16", T=1024, d=512, E=16, k=4, f=384, E_s=2),
    # the paper's own two-matrix expert at the shapes of its Table 3, one GPU's share of tokens, near-uniform load
    "small_mlp2": MoEConfig("small_mlp2", T=8192, d=2048, E=64, k=6, f=1408, expert="mlp2"),
    "medium_mlp2": MoEConfig("medium_mlp2", T=8192, d=5120, E=128, k=6, f=1536, expert="mlp2"),
    "large_mlp2": MoEConfig("large_mlp2", T=4096, d=7168, E=256, k=8, f=2048, expert="mlp2"),
    "super_mlp2": MoEConfig("super_mlp2", T=4096, d=7168, E=256, k=8, f=2560, expert="mlp2"),
    # the share of one rank under expert parallelism of degree 8 (the paper's breakdown runs the Small model with
    # EP = 8): 8 local experts, the same number of rows, segments 8 times as long
    "small_ep8_mlp2": MoEConfig("small_ep8_mlp2", T=8192, d=2048, E=8, k=6, f=1408, expert="mlp2"),
    # reduced two-matrix shapes
    "mini_mlp2_bf16": MoEConfig("mini_mlp2_bf16", T=600, d=256, E=8, k=3, f=192, expert="mlp2"),
    "mini_mlp2_skew": MoEConfig("mini_mlp2_skew", T=600, d=256, E=8, k=3, f=192, expert="mlp2", skew_alpha=3.0,
                                act="silu"),
    "mini_mlp2_f32": MoEConfig("mini_mlp2_f32", T=200, d=96, E=5, k=2, f=40, dtype="f32", router_std=0.05,
                               expert="mlp2"),
    "odd_mlp2_bf16": MoEConfig("odd_mlp2_bf16", T=131, d=72, E=6, k=2, f=24, router_std=0.2, expert="mlp2",
                               act="identity"),
    "mid_mlp2_bf16": MoEConfig("mid_mlp2_bf16", T=1024, d=512, E=16, k=4, f=384, expert="mlp2"),
}


# ----------------------------------------------------------------------------------------------------------
# bf16 storage helpers (pure data conversion)
# ----------------------------------------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even) and return the 16-bit patterns as uint16."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = (u + 0x7FFF + lsb) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    return (b.astype(np.uint32) << 16).view(np.float32)


def round_to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """Return float32 values that are exactly representable in the storage type."""
    a = np.asarray(a, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(a)).reshape(a.shape)
    return a


# ----------------------------------------------------------------------------------------------------------
# random draws
# ----------------------------------------------------------------------------------------------------------
def _rng(seed: int, tensor: str, index: int = 0) -> np.random.Generator:
    tid = _TENSOR_IDS[tensor]
    return np.random.Generator(np.random.Philox(key=[(int(seed) << 32) | tid, int(index)]))


def _normal(seed, tensor, index, shape, std, dtype) -> np.ndarray:
    g = _rng(seed, tensor, index)
    a = g.standard_normal(size=shape, dtype=np.float32) * np.float32(std)
    return round_to_storage(a, dtype)


def router_std(cfg: MoEConfig) -> float:
    return cfg.router_std if cfg.router_std is not None else 1.0 / math.sqrt(cfg.d)


def make_x(cfg: MoEConfig) -> np.ndarray:
    """Layer input x [T, d] ~ N(0,1)."""
    return _normal(cfg.seed, "x", 0, (cfg.T, cfg.d), 1.0, cfg.dtype)


def make_dout(cfg: MoEConfig) -> np.ndarray:
    """Upstream gradient dL/dy [T, d] ~ N(0,1)."""
    return _normal(cfg.seed, "dout", 0, (cfg.T, cfg.d), 1.0, cfg.dtype)


def make_w_router(cfg: MoEConfig) -> np.ndarray:
    """Gate projection Wr [d, E] ~ N(0, router_std)."""
    return _normal(cfg.seed, "w_router", 0, (cfg.d, cfg.E), router_std(cfg), cfg.dtype)


def make_gate_bias(cfg: MoEConfig) -> Optional[np.ndarray]:
    """Per-expert logit bias [E] float32, or None.  bias[e] = -alpha * 1.2 * ln(rank_e) with rank a seeded
    permutation of 1..E: expert load then follows a Zipf(s=1.2)-shaped profile sharpened by alpha."""
    if cfg.skew_alpha == 0.0:
        return None
    perm = _rng(cfg.seed, "rank_perm").permutation(cfg.E) + 1
    return (-cfg.skew_alpha * 1.2 * np.log(perm.astype(np.float64))).astype(np.float32)


def make_expert_weight(cfg: MoEConfig, which: str, e: int) -> np.ndarray:
    """One routed expert's matrix.  which in {"wg","wu","w1"} -> [d, f]; "wd","w2" -> [f, d]  (in x out, Y = X W)."""
    shape = (cfg.d, cfg.f) if which in ("wg", "wu", "w1") else (cfg.f, cfg.d)
    return _normal(cfg.seed, which, e, shape, cfg.w_std, cfg.dtype)


def iter_expert_weights(cfg: MoEConfig, which: str, batch: int = 16):
    """Yields (e, matrix) for every routed expert in order, drawing `batch` experts at a time on host threads
    (numpy's generators release the GIL), so that large workloads never hold a whole tensor on the host."""
    import concurrent.futures
    with concurrent.futures.ThreadPoolExecutor(max_workers=batch) as pool:
        for e0 in range(0, cfg.E, batch):
            es = list(range(e0, min(cfg.E, e0 + batch)))
            for e, a in zip(es, pool.map(lambda e: make_expert_weight(cfg, which, e), es)):
                yield e, a


def make_expert_weights(cfg: MoEConfig, which: str) -> np.ndarray:
    """All routed experts' matrices stacked: [E, d, f] or [E, f, d]."""
    shape = (cfg.d, cfg.f) if which in ("wg", "wu", "w1") else (cfg.f, cfg.d)
    out = np.empty((cfg.E,) + shape, dtype=np.float32)
    for e, a in iter_expert_weights(cfg, which):
        out[e] = a
    return out


def make_shared_weight(cfg: MoEConfig, which: str, s: int) -> np.ndarray:
    """One shared expert's matrix (same shapes as a routed expert)."""
    shape = (cfg.d, cfg.f) if which in ("wg", "wu") else (cfg.f, cfg.d)
    return _normal(cfg.seed, "shared_" + which, s, shape, cfg.w_std, cfg.dtype)


def make_shared_weights(cfg: MoEConfig, which: str) -> np.ndarray:
    """All shared experts stacked [E_s, d, f] / [E_s, f, d]; shape (0, ...) when E_s == 0."""
    shape = (cfg.d, cfg.f) if which in ("wg", "wu") else (cfg.f, cfg.d)
    if cfg.E_s == 0:
        return np.zeros((0,) + shape, dtype=np.float32)
    return np.stack([make_shared_weight(cfg, which, s) for s in range(cfg.E_s)])


def make_logits(T: int, E: int, seed: int = 0, std: float = 1.0) -> np.ndarray:
    """Free-standing gate logits [T, E] float32 ~ N(0, std) for tests of routing in isolation."""
    g = _rng(seed, "logits")
    return g.standard_normal(size=(T, E), dtype=np.float32) * np.float32(std)


def make_rbd_keys(n: int, seed: int = 0) -> np.ndarray:
    """The random draws of the redundancy-bypassing dispatch's pilot selection: one uint32 per flat (token, slot)
    entry."""
    return _rng(seed, "rbd_key").integers(0, 2 ** 32, size=n, dtype=np.uint32)


def make_layer_inputs(cfg: MoEConfig) -> dict:
    """Every input of one forward+backward pass, as float32 arrays holding storage-exact values."""
    if cfg.expert == "mlp2":
        return {
            "x": make_x(cfg),
            "w_router": make_w_router(cfg),
            "bias": make_gate_bias(cfg),
            "w1": make_expert_weights(cfg, "w1"),
            "w2": make_expert_weights(cfg, "w2"),
            "dout": make_dout(cfg),
        }
    return {
        "x": make_x(cfg),
        "w_router": make_w_router(cfg),
        "bias": make_gate_bias(cfg),
        "wg": make_expert_weights(cfg, "wg"),
        "wu": make_expert_weights(cfg, "wu"),
        "wd": make_expert_weights(cfg, "wd"),
        "shared_wg": make_shared_weights(cfg, "wg"),
        "shared_wu": make_shared_weights(cfg, "wu"),
        "shared_wd": make_shared_weights(cfg, "wd"),
        "dout": make_dout(cfg),
    }
