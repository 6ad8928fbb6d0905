"""Seeded synthetic inputs for the Top-K+phi decode path.

This module only *draws* inputs (queries, KV caches, feature-map weights) and
rounds them to their storage type.  It contains none of the method's
arithmetic: no scores, no feature maps, no selection.  Both the CPU oracle's
tests and the HIP path's tests/bench consume the buffers produced here, so the
two sides see bit-identical stored inputs.

The shapes are those of Llama-3.2-1B/3B attention layers (head counts, head
dimension, layer counts) at the context lengths the paper evaluates
(Sec. "Models, tasks, and protocol") and beyond; the value distributions are a
synthetic stand-in for real activations: Gaussian keys with a few
large-magnitude channels, Gaussian values and a handful of "needle" keys
aligned with the query so that attention has sharp peaks on top of diffuse
mass (the regime the paper's entropy analysis singles out).

bf16 tensors are carried on the host as uint16 bit patterns.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

__all__ = [
    "Workload", "WORKLOADS", "f32_to_bf16_bits", "bf16_bits_to_f32", "to_f64",
    "make_layer", "make_mlp_phi", "ragged_lengths", "mid_budget",
]


# --------------------------------------------------------------------------
# storage rounding helpers (pure bit manipulation)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 -> bfloat16 (round-to-nearest-even), returned as uint16."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    # NaN stays NaN (not produced by the generators, kept for safety)
    rounding = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    out = ((u + rounding) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact bfloat16 (uint16 bits) -> float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(a: np.ndarray) -> np.ndarray:
    """Exact upcast of a stored tensor (float32, or uint16 = bf16 bits) to float64."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return np.asarray(a, dtype=np.float64)


def _store(x32: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return f32_to_bf16_bits(x32)
    if dtype == "f32":
        return np.ascontiguousarray(x32, dtype=np.float32)
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class Workload:
    """One synthetic attention-layer workload.

    budget_bp is the retrieved-token budget in basis points of the mid-region
    size (100 = 1 %); `mid_budget` turns it into the integer K.
    """
    name: str
    dtype: str                 # "f32" | "bf16": storage type of q, K, V, W
    n_q_heads: int
    n_kv_heads: int
    d_head: int
    d_phi: int
    L: int                     # prefill length (max length for ragged sets)
    n_sink: int = 4
    n_tail: int = 64
    budget_bp: int = 100
    n_needles: int = 16        # per KV head
    n_outlier_channels: int = 4
    outlier_scale: float = 5.0
    n_layers: int = 1
    n_seqs: int = 1
    L_min: int = 0             # >0: ragged per-sequence lengths in [L_min, L]
    seed: int = 20260405

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    # scalar constants of the feature map and of the scores, as the float32
    # values that both implementations are handed
    @property
    def score_scale(self) -> float:
        return float(np.float32(1.0 / math.sqrt(self.d_head)))

    @property
    def phi_in_scale(self) -> float:      # "a": input scale d^(-1/4)
        return float(np.float32(self.d_head ** -0.25))

    @property
    def phi_norm_coef(self) -> float:     # "c": 1 / (2 sqrt d)
        return float(np.float32(1.0 / (2.0 * math.sqrt(self.d_head))))

    @property
    def phi_bias(self) -> float:          # "b": -0.5 ln d_phi on both maps
        return float(np.float32(-0.5 * math.log(self.d_phi)))


WORKLOADS = {
    # tiny single head, fp32 storage
    "tiny_f32": Workload("tiny_f32", "f32", 1, 1, 64, 64, 4096, n_needles=8,
                         n_outlier_channels=0, seed=20260405),
    # Llama-3.2-1B-shaped single layer
    "l1b_32k": Workload("l1b_32k", "bf16", 32, 8, 64, 64, 32768, seed=20260406),
    # Llama-3.2-3B-shaped single layer at 128K
    "l3b_128k": Workload("l3b_128k", "bf16", 24, 8, 128, 128, 131072, seed=20260407),
    # batched ragged decode over all 16 layers of a 1B-shaped model
    "l1b_ragged": Workload("l1b_ragged", "bf16", 32, 8, 64, 64, 65536, n_layers=16,
                           n_seqs=16, L_min=16384, seed=20260408),
    # build + 64 decode queries over all 28 layers of a 3B-shaped model
    "l3b_128k_model": Workload("l3b_128k_model", "bf16", 24, 8, 128, 128, 131072,
                               n_layers=28, seed=20260409),
}


def mid_budget(L: int, budget_bp: int, n_sink: int, n_tail: int) -> int:
    """Retrieved tokens for a budget given as basis points of the mid-region
    size, in integer arithmetic (floor)."""
    n_mid = max(0, L - n_sink - n_tail)
    return (n_mid * budget_bp) // 10000


def ragged_lengths(w: Workload) -> np.ndarray:
    """Per-sequence prefill lengths, uniform integers in [L_min, L]."""
    if w.L_min <= 0:
        return np.full(w.n_seqs, w.L, dtype=np.int64)
    rng = np.random.Generator(np.random.Philox(key=w.seed + 7777))
    return rng.integers(w.L_min, w.L + 1, size=w.n_seqs, dtype=np.int64)


def _unit(v: np.ndarray) -> np.ndarray:
    return v / np.linalg.norm(v)


def make_layer(w: Workload, layer: int = 0, seq: int = 0, L: int | None = None,
               query_index: int = 0, with_kv: bool = True) -> dict:
    """Draw one (sequence, layer) problem.

    Returns a dict of stored tensors:
      q  [Hq][d]            K, V [Hkv][L][d]
      Wq [Hq][dphi][d]  bq [Hq][dphi] (float32)
      Wk [Hkv][dphi][d] bk [Hkv][dphi] (float32)
    plus "needle_pos" [Hkv][n_needles] (token indices) for reference.

    Every stream (q, K, V, W) has its own counter-based generator keyed by
    (seed, layer, seq, tensor id), so tensors can be drawn independently and
    a different `query_index` redraws only q: the cache is fixed, and its
    needles are aligned with query 0.
    """
    L = w.L if L is None else int(L)
    Hq, Hkv, d, dphi, G = w.n_q_heads, w.n_kv_heads, w.d_head, w.d_phi, w.group

    def gen(tensor_id: int, extra: int = 0) -> np.random.Generator:
        key = (w.seed * 1_000_003 + layer * 10_007 + seq * 101 + tensor_id) % (2 ** 63)
        return np.random.Generator(np.random.Philox(key=[key, extra]))

    out: dict = {"L": L}

    # query: N(0,1)
    q32 = gen(1, query_index).standard_normal((Hq, d), dtype=np.float32)
    out["q"] = _store(q32, w.dtype)

    # feature-map weights: W ~ N(0,1), shared between a KV head and the query
    # heads of its group; constant bias on both maps
    Wk32 = gen(2).standard_normal((Hkv, dphi, d), dtype=np.float32)
    out["Wk"] = _store(Wk32, w.dtype)
    out["Wq"] = _store(np.repeat(Wk32, G, axis=0), w.dtype)
    out["bk"] = np.full((Hkv, dphi), w.phi_bias, dtype=np.float32)
    out["bq"] = np.full((Hq, dphi), w.phi_bias, dtype=np.float32)

    if not with_kv:
        return out

    # keys: N(0,1) background, a few large channels per KV head
    K32 = gen(3).standard_normal((Hkv, L, d), dtype=np.float32)
    if w.n_outlier_channels > 0:
        crng = gen(4)
        for h in range(Hkv):
            ch = crng.choice(d, size=w.n_outlier_channels, replace=False)
            K32[h][:, ch] *= np.float32(w.outlier_scale)

    # needles: keys with cosine 0.8 to a query of the group, norm sqrt(d),
    # planted at distinct positions of the mid-region
    n_mid = L - w.n_sink - w.n_tail
    n_needles = min(w.n_needles, max(n_mid, 0))
    pos = np.zeros((Hkv, n_needles), dtype=np.int64)
    if n_needles > 0:
        prng = gen(5)
        nrng = gen(6)
        # the stored (rounded) query 0 is what the needles align with
        q0 = gen(1, 0).standard_normal((Hq, d), dtype=np.float32)
        q_st = to_f64(_store(q0, w.dtype))
        for h in range(Hkv):
            pos[h] = w.n_sink + prng.choice(n_mid, size=n_needles, replace=False)
            for j in range(n_needles):
                qh = _unit(q_st[h * G + (j % G)])
                r = nrng.standard_normal(d)
                r = _unit(r - np.dot(r, qh) * qh)
                K32[h, pos[h, j]] = (math.sqrt(d) * (0.8 * qh + 0.6 * r)).astype(np.float32)
    out["needle_pos"] = pos
    out["K"] = _store(K32, w.dtype)
    del K32

    # values: N(0,1)
    V32 = gen(7).standard_normal((Hkv, L, d), dtype=np.float32)
    out["V"] = _store(V32, w.dtype)
    return out


def make_mlp_phi(w: Workload, layer: int = 0, d_emb: int = 512) -> dict:
    """Random weights of the shapes of the head-wise one-block ReZero MLP feature maps
    (stem d -> d_emb, gated residual MLP d_emb -> d_emb -> d_emb, output d_emb -> d_phi, then
    exp), one map per query head ("q") and one per KV head ("k").

    Returns {"q": {...}, "k": {...}} with stacked per-head tensors
      Ws [H][d_emb][d], W1, W2 [H][d_emb][d_emb], Wo [H][d_phi][d_emb]   (storage type of w)
      bs, b1, b2 [H][d_emb], bo [H][d_phi], alpha [H]                     (float32)
    Weight entries are N(0, 1/fan_in) so that activations stay O(1) for N(0,1) inputs; biases
    N(0, 0.1^2); bo is centred on -0.5 ln d_phi; alpha = 0.5.  No trained weights exist for
    these shapes: the maps are not calibrated to exp(q.k), only their cost and arithmetic matter."""
    d, dphi = w.d_head, w.d_phi
    out = {}
    for side, H, tid in (("q", w.n_q_heads, 40), ("k", w.n_kv_heads, 50)):
        key = (w.seed * 1_000_003 + layer * 10_007 + tid) % (2 ** 63)
        rng = np.random.Generator(np.random.Philox(key=[key, d_emb]))

        def mat(rows, cols):
            return _store((rng.standard_normal((H, rows, cols), dtype=np.float32) / np.float32(math.sqrt(cols))), w.dtype)

        def vec(n, centre=0.0):
            return (np.float32(centre) + np.float32(0.1) * rng.standard_normal((H, n), dtype=np.float32)).astype(np.float32)

        out[side] = {
            "Ws": mat(d_emb, d), "bs": vec(d_emb),
            "W1": mat(d_emb, d_emb), "b1": vec(d_emb),
            "W2": mat(d_emb, d_emb), "b2": vec(d_emb),
            "Wo": mat(dphi, d_emb), "bo": vec(dphi, -0.5 * math.log(dphi)),
            "alpha": np.full((H,), 0.5, dtype=np.float32),
        }
    return out
