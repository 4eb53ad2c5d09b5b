"""Seeded synthetic inputs for the MoE expert layer (shared by the tests, the benchmark and the CPU oracle).

This module only *makes inputs*: shapes, random tensors, bf16 rounding of those tensors and the routing
inputs (logits or expert ids) of each workload.  It holds none of the layer's arithmetic: no top-k, no
softmax, no permutation, no FFN.  Both the HIP path and the oracle consume exactly the arrays made here.

Symbols follow the paper's notation table (Section III-A, "Symbol definitions"): T tokens (= b*s), d = d_model,
f = d_ffn of an expert, E routed experts, E_s shared (always-active) experts, k = top-k.  Derived:
E' = E + E_s expert ids, K' = k + E_s slots per token, N = T*K' rows after the permutation.

Value distributions: x ~ N(0,1), expert weights ~ N(0,0.02), router weights ~ N(0,0.02), dout ~ N(0,1); all
rounded to bf16 (round-to-nearest-even) before anyone sees them, so the GPU and the oracle start from the same
bits.  Logits are the fp32 rounding of an fp64 x.Wg product (the router GEMM is an input here, not a step of
the path).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

# --------------------------------------------------------------------------------------------------------------
# bf16 helpers (input preparation only)
# --------------------------------------------------------------------------------------------------------------


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (round-to-nearest-even); returns the 16-bit patterns as uint16."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    # in-place friendly chunks keep the temporary small for multi-GB weight tensors
    out = np.empty(a.shape, dtype=np.uint16)
    flat_u = u.reshape(-1)
    flat_o = out.reshape(-1)
    step = 1 << 24
    for i in range(0, flat_u.size, step):
        c = flat_u[i:i + step]
        r = ((c >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
        flat_o[i:i + step] = ((c + r) >> np.uint32(16)).astype(np.uint16)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------------------------------------------
# shapes
# --------------------------------------------------------------------------------------------------------------


@dataclass(frozen=True)
class MoEShape:
    T: int          # tokens
    d_model: int    # d
    d_ffn: int      # f
    E: int          # routed experts
    k: int          # top-k
    E_shared: int = 0
    renorm: int = 1

    @property
    def E_total(self) -> int:
        return self.E + self.E_shared

    @property
    def K_slots(self) -> int:
        return self.k + self.E_shared

    @property
    def N(self) -> int:
        return self.T * self.K_slots

    def flops_fwd_bwd(self) -> float:
        """18*d*f per permuted row: three GEMMs of 2*d*f each in forward, twice that again in backward."""
        return 18.0 * self.d_model * self.d_ffn * self.N


@dataclass(frozen=True)
class Workload:
    name: str
    shape: MoEShape
    routing: str            # "router" | "router_bias" | "zipf_shard" | "forced_imbalance"
    note: str = ""


WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", MoEShape(256, 512, 1024, 8, 2), "router",
                     "unit-test scale layer"),
    "mixtral": Workload("mixtral", MoEShape(4096, 4096, 14336, 8, 2), "router",
                        "Mixtral-8x7B-shaped layer (Table I row), near-uniform load"),
    "finegrained": Workload("finegrained", MoEShape(8192, 2048, 1408, 64, 6, E_shared=2), "router_bias",
                            "fine-grained layer, 64 routed top-6 + 2 shared, mild imbalance"),
    "shard": Workload("shard", MoEShape(4096, 7168, 2048, 32, 1), "zipf_shard",
                      "one expert-parallel shard: 4096 incoming rows, 32 local experts, Zipf(1.2) popularity"),
    "imbalance": Workload("imbalance", MoEShape(16384, 4096, 1024, 128, 4), "forced_imbalance",
                          "10% of experts get ~60% of slots, 20% get none"),
}


def scaled_down(w: Workload, dim_div: int = 8, tok_div: int = 4) -> Workload:
    """Same E, k and routing recipe with d, f divided by dim_div (rounded up to a multiple of 64) and T by
    tok_div: a copy small enough for the full fp64 oracle."""
    s = w.shape
    r64 = lambda v: max(64, -(-v // 64) * 64)  # noqa: E731
    return replace(w, name=w.name + "_small",
                   shape=replace(s, T=max(s.T // tok_div, 1), d_model=r64(s.d_model // dim_div),
                                 d_ffn=r64(s.d_ffn // dim_div)))


# --------------------------------------------------------------------------------------------------------------
# tensors
# --------------------------------------------------------------------------------------------------------------


def _normal_bf16(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return f32_to_bf16_bits(a)


def make_tokens(shape: MoEShape, seed: int = 0) -> np.ndarray:
    """x[T,d] ~ N(0,1) as bf16 bits."""
    return _normal_bf16(np.random.default_rng([seed, 1]), (shape.T, shape.d_model), 1.0)


def make_dout(shape: MoEShape, seed: int = 0) -> np.ndarray:
    """Upstream gradient dout[T,d] ~ N(0,1) as bf16 bits."""
    return _normal_bf16(np.random.default_rng([seed, 2]), (shape.T, shape.d_model), 1.0)


def make_expert_weights(shape: MoEShape, seed: int = 0, std: float = 0.02):
    """W_gate[E',d,f], W_up[E',d,f], W_down[E',f,d] ~ N(0,std) as bf16 bits (the paper's layouts, Section III-A)."""
    Et, d, f = shape.E_total, shape.d_model, shape.d_ffn
    wg = np.empty((Et, d, f), dtype=np.uint16)
    wu = np.empty((Et, d, f), dtype=np.uint16)
    wd = np.empty((Et, f, d), dtype=np.uint16)
    for e in range(Et):
        rng = np.random.default_rng([seed, 3, e])
        wg[e] = _normal_bf16(rng, (d, f), std)
        wu[e] = _normal_bf16(rng, (d, f), std)
        wd[e] = _normal_bf16(rng, (f, d), std)
    return wg, wu, wd


def make_router_weight(shape: MoEShape, seed: int = 0, std: float = 0.02) -> np.ndarray:
    """Router weight W_r [E, d_model] (bf16 bits): row e is column e of the matrix make_router_logits multiplies by."""
    rng = np.random.default_rng([seed, 4])
    return np.ascontiguousarray(_normal_bf16(rng, (shape.d_model, shape.E), std).T)


def make_router_logits(shape: MoEShape, x_bits: np.ndarray, seed: int = 0, bias_std: float = 0.0,
                       std: float = 0.02) -> np.ndarray:
    """logits[T,E] = fp32( x . Wg_router (+ b) ) with Wg_router ~ N(0,std) (bf16) and b_e ~ N(0,bias_std)."""
    rng = np.random.default_rng([seed, 4])
    wr = bf16_bits_to_f32(_normal_bf16(rng, (shape.d_model, shape.E), std)).astype(np.float64)
    x = bf16_bits_to_f32(x_bits).astype(np.float64)
    logits = x @ wr
    if bias_std > 0.0:
        logits = logits + rng.standard_normal(shape.E) * bias_std
    return logits.astype(np.float32)


def make_zipf_shard_routing(shape: MoEShape, seed: int = 0, s: float = 1.2):
    """Post-all-to-all shard: each of the T incoming rows carries one local expert id and one gate weight.

    Expert ids ~ Zipf(s) over a seeded random ranking of the E local experts; gate weight ~ U(0,1) (fp32).
    Returns (topk_idx[T,1] int32, topk_w[T,1] float32)."""
    assert shape.k == 1 and shape.E_shared == 0
    rng = np.random.default_rng([seed, 5])
    ranking = rng.permutation(shape.E)
    p = 1.0 / np.arange(1, shape.E + 1, dtype=np.float64) ** s
    p /= p.sum()
    ids = ranking[rng.choice(shape.E, size=shape.T, p=p)]
    w = rng.random(shape.T, dtype=np.float32)
    return ids.astype(np.int32).reshape(shape.T, 1), w.reshape(shape.T, 1)


# Popularity ratio hot:warm of the forced-imbalance logits.  Calibrated once (with the oracle's routing) so that
# for E=128, k=4 the 10% hot experts receive 58-62% of the slots; a CPU test re-checks the realised share.
HOT_WARM_LOG_RATIO = 2.4


def make_forced_imbalance_logits(shape: MoEShape, seed: int = 0, frac_hot: float = 0.10,
                                 frac_dead: float = 0.20, log_ratio: float = HOT_WARM_LOG_RATIO):
    """logits[T,E] that force a skewed load: `frac_dead` of the experts sit at -1e30 (never chosen),
    `frac_hot` get log-popularity `log_ratio`, the rest 0; i.i.d. Gumbel(0,1) noise per (token, expert) makes
    top-k on these logits a draw without replacement proportional to popularity.
    Returns (logits fp32, roles int8[E]: 2 hot, 1 warm, 0 dead)."""
    rng = np.random.default_rng([seed, 6])
    E = shape.E
    n_hot = max(1, int(round(frac_hot * E)))
    n_dead = int(round(frac_dead * E))
    if E - n_dead < shape.k:
        n_dead = max(0, E - shape.k)
    n_hot = min(n_hot, E - n_dead)
    order = rng.permutation(E)
    roles = np.ones(E, dtype=np.int8)
    roles[order[:n_hot]] = 2
    roles[order[n_hot:n_hot + n_dead]] = 0
    base = np.where(roles == 2, log_ratio, 0.0)
    u = rng.random((shape.T, E))
    gumbel = -np.log(-np.log(np.clip(u, 1e-300, 1.0 - 1e-16)))
    logits = (base[None, :] + gumbel).astype(np.float32)
    logits[:, roles == 0] = np.float32(-1e30)
    return logits, roles


def make_layer_inputs(w: Workload, seed: int = 0, with_weights: bool = True) -> dict:
    """Everything one forward+backward of workload `w` consumes.

    Keys: shape, x, dout (bf16 bits), w_gate, w_up, w_down (bf16 bits, unless with_weights=False), and either
    `logits` (fp32 [T,E]) or, for the shard workload, `topk_idx` / `topk_w` given directly."""
    s = w.shape
    out = {"shape": s, "workload": w.name}
    out["x"] = make_tokens(s, seed)
    out["dout"] = make_dout(s, seed)
    if with_weights:
        out["w_gate"], out["w_up"], out["w_down"] = make_expert_weights(s, seed)
    if w.routing == "router":
        out["logits"] = make_router_logits(s, out["x"], seed)
    elif w.routing == "router_bias":
        out["logits"] = make_router_logits(s, out["x"], seed, bias_std=0.5)
    elif w.routing == "zipf_shard":
        out["topk_idx"], out["topk_w"] = make_zipf_shard_routing(s, seed)
    elif w.routing == "forced_imbalance":
        out["logits"], out["roles"] = make_forced_imbalance_logits(s, seed)
    else:
        raise ValueError(w.routing)
    return out


def random_layer_inputs(shape: MoEShape, seed: int = 0, logit_std: float = 1.0,
                        dead_experts: Optional[int] = None) -> dict:
    """Free-form small case for tests: random logits ~ N(0,logit_std) instead of a router product.
    `dead_experts` experts (the highest ids) get -1e30 logits so that they receive no token."""
    rng = np.random.default_rng([seed, 7])
    out = {"shape": shape, "workload": "random"}
    out["x"] = make_tokens(shape, seed)
    out["dout"] = make_dout(shape, seed)
    out["w_gate"], out["w_up"], out["w_down"] = make_expert_weights(shape, seed)
    logits = (rng.standard_normal((shape.T, shape.E)) * logit_std).astype(np.float32)
    if dead_experts:
        assert shape.E - dead_experts >= shape.k
        logits[:, shape.E - dead_experts:] = np.float32(-1e30)
    out["logits"] = logits
    return out
