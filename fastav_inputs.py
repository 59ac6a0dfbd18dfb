"""Seeded synthetic inputs for the FastAV pruned-prefill path.

This module only *draws numbers and describes shapes*: model dimensions, token
layouts (modality spans), prune schedules, random weights and random token
embeddings.  It holds none of the method's arithmetic (no norm, attention,
score, keep-count or selection logic), so both the CPU oracle and the HIP path
may consume what it produces without sharing any computation.

The paper evaluates on audio-visual question answering prompts (video tokens,
then audio tokens, then the question text) fed to a 28-layer decoder
(Section 3.1, "Implementation details"); neither the datasets nor the trained
weights are available here, so these generators stand in for them with the same
*shape*: a [video | audio | text] sequence of a few thousand tokens in which
audio is a large share, a middle-layer global prune and later fine prunes.

Values
------
* matrices  ~ N(0, 0.02), norm gains ~ 1 + N(0, 0.02); one NumPy stream per
  layer, ``default_rng([seed, layer])``, drawn in a fixed order;
* embeddings ~ N(mu_modality, 1), mu = {text 0, video +0.5, audio -0.5};
* for bf16 models every array is rounded (nearest-even) to a bf16-representable
  fp32 value, so both sides start from bit-identical numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import numpy as np

TEXT, VIDEO, AUDIO = 0, 1, 2
MODALITY_MEAN = {TEXT: 0.0, VIDEO: 0.5, AUDIO: -0.5}
GLOBAL, FINE = 0, 1

WEIGHT_NAMES = ("g_attn", "wq", "wk", "wv", "wo", "g_mlp", "w_gate", "w_up", "w_down")


@dataclass(frozen=True)
class Model:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    mlp_dim: int
    rope_base: float = 1.0e4
    rms_eps: float = 1.0e-6
    dtype: str = "bf16"          # "bf16" or "f32": storage type of weights/activations


@dataclass(frozen=True)
class Prune:
    layer: int
    kind: int                    # GLOBAL or FINE
    keep_ratio: float
    selector: int = 0            # which tokens go (Tables 2-3): 0 = the paper's rule for this kind
    seed: int = 0                # keys the draws of the random selector


@dataclass
class Workload:
    name: str
    model: Model
    # one entry per sample: list of (modality, length) spans in sequence order
    samples: List[List[Tuple[int, int]]]
    prunes: List[Prune]
    n_last: int = 1
    seed: int = 0                # embedding seed
    weight_seed: int = 0

    @property
    def seqlens(self) -> List[int]:
        return [sum(l for _, l in s) for s in self.samples]

    @property
    def total_tokens(self) -> int:
        return sum(self.seqlens)


MODEL_TINY = Model(4, 256, 4, 2, 64, 688, 1.0e4, 1.0e-6, "f32")
MODEL_7B_1L = Model(1, 4096, 32, 8, 128, 14336, 1.0e4, 1.0e-6, "bf16")
MODEL_7B = Model(32, 4096, 32, 8, 128, 14336, 1.0e4, 1.0e-6, "bf16")
MODEL_LONG = Model(28, 3584, 28, 4, 128, 18944, 1.0e6, 1.0e-6, "bf16")


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round an fp32 array to the nearest bf16-representable value (ties to even), in place."""
    assert a.dtype == np.float32
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    u += np.uint32(0x7FFF)
    u += lsb
    u &= np.uint32(0xFFFF0000)
    return a


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of an already bf16-representable fp32 array (uint16, same shape)."""
    assert a.dtype == np.float32
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _ragged_samples(batch: int, seed: int) -> List[List[Tuple[int, int]]]:
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(batch):
        n = int(rng.integers(2048, 6144 + 1))
        fv = float(rng.uniform(0.60, 0.75))
        fa = float(rng.uniform(0.20, 0.30))
        nv = max(144, int(round(fv * n / 144.0)) * 144)       # whole 144-token frames
        na = int(round(fa * n))
        if nv + na > n - 8:
            na = n - 8 - nv
        out.append([(VIDEO, nv), (AUDIO, na), (TEXT, n - nv - na)])
    return out


def config(i: int) -> Workload:
    """The five benchmark/parity workloads (1-based index)."""
    if i == 1:
        return Workload("cfg1_tiny_f32_n512", MODEL_TINY,
                        [[(TEXT, 16), (VIDEO, 192), (AUDIO, 288), (TEXT, 16)]],
                        [Prune(2, GLOBAL, 0.5), Prune(3, FINE, 0.5)], seed=1001)
    if i == 2:
        return Workload("cfg2_7b_1layer_n2048", MODEL_7B_1L,
                        [[(VIDEO, 1152), (AUDIO, 768), (TEXT, 128)]],
                        [Prune(0, FINE, 0.6)], seed=1002)
    if i == 3:
        return Workload("cfg3_7b_32layer_n4096", MODEL_7B,
                        [[(VIDEO, 2880), (AUDIO, 1000), (TEXT, 216)]],
                        [Prune(14, GLOBAL, 0.6), Prune(20, FINE, 0.7), Prune(26, FINE, 0.7)], seed=1003)
    if i == 4:
        return Workload("cfg4_long_28layer_n16384", MODEL_LONG,
                        [[(VIDEO, 11520), (AUDIO, 4000), (TEXT, 864)]],
                        [Prune(12, GLOBAL, 0.5), Prune(18, FINE, 0.7), Prune(24, FINE, 0.7)], seed=1004)
    if i == 5:
        return Workload("cfg5_7b_ragged_b8", MODEL_7B, _ragged_samples(8, 5),
                        [Prune(14, GLOBAL, 0.6), Prune(20, FINE, 0.7), Prune(26, FINE, 0.7)], seed=1005)
    raise ValueError("config index must be 1..5")


def unpruned(w: Workload) -> Workload:
    return Workload(w.name + "_unpruned", w.model, w.samples, [], w.n_last, w.seed, w.weight_seed)


def paper_schedule(w: Workload, global_keep: float = 0.6, fine_drop: float = 0.2) -> Workload:
    """Same workload under the schedule the paper runs (Section 3.1, implementation details; Section 2.2, "Fine
    pruning": at each layer following global pruning): one global prune on the input of the middle layer, then a
    fine prune at the middle layer itself and at every layer after it, each dropping ``fine_drop`` (the paper's
    P = 20 %) of the tokens that are left.  This is the placement that reproduces Table 4's FLOPs column."""
    mid = w.model.n_layers // 2
    prunes = [Prune(mid, GLOBAL, global_keep)] + [Prune(l, FINE, 1.0 - fine_drop) for l in range(mid, w.model.n_layers)]
    return Workload(w.name + "_paper_schedule", w.model, w.samples, prunes, w.n_last, w.seed, w.weight_seed)


def with_layers(w: Workload, n_layers: int) -> Workload:
    """Same workload on a decoder truncated to its first ``n_layers`` layers (prunes beyond are dropped)."""
    m = w.model
    m2 = Model(n_layers, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.mlp_dim, m.rope_base, m.rms_eps, m.dtype)
    return Workload(f"{w.name}_first{n_layers}", m2, w.samples,
                    [p for p in w.prunes if p.layer < n_layers], w.n_last, w.seed, w.weight_seed)


def weight_shapes(m: Model) -> Dict[str, Tuple[int, ...]]:
    """Shapes of one layer's parameters.  Matrices are stored [out_features, in_features]."""
    qd, kd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    return {"g_attn": (m.hidden,), "wq": (qd, m.hidden), "wk": (kd, m.hidden), "wv": (kd, m.hidden),
            "wo": (m.hidden, qd), "g_mlp": (m.hidden,), "w_gate": (m.mlp_dim, m.hidden),
            "w_up": (m.mlp_dim, m.hidden), "w_down": (m.hidden, m.mlp_dim)}


def layer_weights(m: Model, layer: int, seed: int = 0) -> Dict[str, np.ndarray]:
    """fp32 arrays (bf16-representable when ``m.dtype == 'bf16'``) for one decoder layer."""
    rng = np.random.default_rng([seed, layer])
    out = {}
    for name, shape in weight_shapes(m).items():
        a = rng.standard_normal(shape, dtype=np.float32)
        a *= np.float32(0.02)
        if len(shape) == 1:
            a += np.float32(1.0)
        if m.dtype == "bf16":
            round_bf16(a)
        out[name] = a
    return out


def embeddings(w: Workload) -> np.ndarray:
    """Packed token embeddings [total_tokens, hidden], fp32 (bf16-representable for bf16 models)."""
    rng = np.random.default_rng(w.seed)
    d = w.model.hidden
    x = rng.standard_normal((w.total_tokens, d), dtype=np.float32)
    row = 0
    for sample in w.samples:
        for modality, length in sample:
            x[row:row + length] += np.float32(MODALITY_MEAN[modality])
            row += length
    if w.model.dtype == "bf16":
        round_bf16(x)
    return x


def cu_seqlens(w: Workload) -> np.ndarray:
    return np.concatenate([[0], np.cumsum(w.seqlens)]).astype(np.int32)


def span_table(w: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """(spans [S,3] int32 rows of (start, len, modality) relative to their sample, span_offsets [B+1])."""
    rows, offs = [], [0]
    for sample in w.samples:
        start = 0
        for modality, length in sample:
            rows.append((start, length, modality))
            start += length
        offs.append(len(rows))
    return np.asarray(rows, dtype=np.int32).reshape(-1, 3), np.asarray(offs, dtype=np.int32)


def random_scores(n: int, seed: int, kind: str = "softmax") -> np.ndarray:
    """Score vectors for select/gather tests: 'softmax' (positive, sums to 1), 'ties' (few distinct
    values), 'equal' (all the same), 'mixed' (signed values with zeros, infinities and NaNs)."""
    rng = np.random.default_rng(seed)
    if kind == "softmax":
        z = rng.standard_normal(n).astype(np.float32) * np.float32(1.6)
        e = np.exp(z - z.max())
        return (e / e.sum()).astype(np.float32)
    if kind == "ties":
        vals = rng.random(7).astype(np.float32)
        return vals[rng.integers(0, 7, n)]
    if kind == "equal":
        return np.full(n, np.float32(1.0 / max(n, 1)), dtype=np.float32)
    if kind == "mixed":
        s = rng.standard_normal(n).astype(np.float32)
        idx = rng.integers(0, n, max(1, n // 8))
        s[idx] = np.float32(0.0)
        s[rng.integers(0, n, max(1, n // 16))] = np.float32(-0.0)
        s[rng.integers(0, n, max(1, n // 32))] = np.float32(np.inf)
        s[rng.integers(0, n, max(1, n // 32))] = np.float32(-np.inf)
        s[rng.integers(0, n, max(1, n // 32))] = np.float32(np.nan)
        return s
    raise ValueError(kind)
