"""CPU oracle for the FastAV pruned prefill — TEST INFRASTRUCTURE, not product code.

Only the test-suite, the smoke check and the benchmark's ``cpu_baseline`` leg
may import this module; the HIP library never does, and the two share no code.

It is a plain, slow NumPy implementation (fp64 unless told otherwise) of what the
pruned prefill computes, written from the paper:

* Section 2.1 / Eq. 1     – the decoder consumes one concatenated sequence
                            [video | audio | text] of K = M + U + E tokens;
* Section 2.2, "Global pruning" – at a middle layer, video/audio tokens in later
                            positions are removed (no scores involved);
* Section 2.2, "Fine pruning", Eq. 4 – s = mean over heads of
                            softmax(Q_last K^T); the lowest-P% tokens are removed
                            at each later layer;
* Section 3.1, "Implementation details" – video tokens precede audio tokens
                            (or are frame-interleaved), P = 20 %.

The decoder-layer arithmetic itself (RMSNorm, QKV projection, rotate-half RoPE,
causal grouped-query attention, output projection, SwiGLU MLP, residuals) is the
standard pre-norm decoder the paper's two models use; the paper does not restate
it.

Readings taken where the paper is silent (each is repeated at the function that
implements it):
  R1  logits are scaled by 1/sqrt(head_dim): Eq. 4 scores are "the attention
      weight" of the last query, i.e. the model's own softmax.
  R2  Q and K in Eq. 4 are the post-RoPE features attention consumes.
  R3  grouped-query attention: query head h reads KV head h // (Hq/Hkv); the mean
      of Eq. 4 runs over the Hq query heads.
  R4  keep count k = min(n, max(n_protected, ceil(r*n - 1e-9))), r = 1 - P.
  R5  only video/audio tokens are candidates; text tokens and the last n_last
      positions are always kept and count toward k.
  R6  ties: higher score wins, equal scores -> lower index wins; NaN ranks as -inf,
      -0.0 equals +0.0; the kept set is returned in ascending order.
  R7  a GLOBAL prune at layer l acts on the input of layer l; a FINE prune at
      layer l uses layer l's own attention and every later layer sees the
      survivors only.  Both may share a layer (global first).
  R8  survivors keep their ORIGINAL position ids for RoPE.
  R9  with only a ratio given, global pruning keeps the protected tokens plus the
      earliest candidates by position (this reproduces "all video + first 10
      audio" and "first 4 frames" when k is chosen accordingly).
  R10 n_last > 1 averages the last n_last causal rows (each sums to 1 over its own
      visible keys).
  R18 the rollout threshold of the global-pruning analysis: a token's influence is
      its column mean in R^l (all rows), measured in uniform shares 1/n; a sample's
      cut-off is one past the last video/audio position that reaches the threshold.
  R17 the ablation strategies of Tables 2-3 are named by what they REMOVE:
      low attentive = lowest Eq. 4 scores (the fine rule), top attentive = highest
      Eq. 4 scores, low informative = latest positions (the global rule, R9), top
      informative = earliest positions (the mirror image: the tokens rollout
      concentrates on), random = lowest values of a counter-based uniform draw per
      (seed, layer, sample, original position).  Protected tokens stay in all of
      them, so every strategy keeps the same count ("FLOPs constant").

Pins (tests/test_oracle_pins.py): brute-force loops on tiny inputs, library
special cases (torch SDPA / rms_norm / silu, numpy stable argsort), closed forms
(zero queries -> uniform scores; one dominant key -> one-hot), invariants (rows
sum to 1, keep ratio 1.0 is the identity, RoPE relative-position property,
batched == per-sample; a decode step on unpruned caches equals the last row of a
prefill one token longer; cache order does not matter; rollout rows sum to 1, alpha = 0
gives the identity, uniform attention has a closed form; influences of uniform causal
attention are differences of harmonic numbers; the ablation selectors against
sorted brute force, mirror symmetry and complement identities, the random draw against the
inverse of its mixing function and uniformity statistics), and the paper's printed
FLOPs column of Table 4 for the schedule semantics.  Parity unpinned: the absolute hidden-state values for random
weights (the paper prints no worked numeric example).
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

TEXT, VIDEO, AUDIO = 0, 1, 2
GLOBAL, FINE = 0, 1
# Which tokens a prune step removes (Tables 2-3, reading R17).  DEFAULT: GLOBAL -> LOW_INFORMATIVE, FINE -> LOW_ATTENTIVE.
DEFAULT, LOW_ATTENTIVE, TOP_ATTENTIVE, LOW_INFORMATIVE, TOP_INFORMATIVE, RANDOM = 0, 1, 2, 3, 4, 5


# --------------------------------------------------------------------------- schedule
def keep_count(n: int, keep_ratio: float, n_protected: int) -> int:
    """Number of tokens kept out of n (reading R4); "lowest P% removed", Section 2.2 Fine pruning."""
    k = int(math.ceil(float(keep_ratio) * n - 1e-9))
    return min(n, max(int(n_protected), k))


def protected_mask(spans: Sequence[Tuple[int, int]], n_last: int) -> np.ndarray:
    """True where a token may never be pruned (reading R5): text spans and the last n_last positions.

    ``spans`` is a list of (modality, length) in sequence order."""
    n = sum(l for _, l in spans)
    prot = np.zeros(n, dtype=bool)
    at = 0
    for modality, length in spans:
        if modality == TEXT:
            prot[at:at + length] = True
        at += length
    if n_last > 0:
        prot[max(0, n - n_last):] = True
    return prot


def token_schedule(n: int, n_protected: int, prunes, n_layers: int) -> List[int]:
    """Tokens that enter attention at each layer for a sample of n tokens (reading R7).

    A GLOBAL prune at layer l shrinks the input of layer l; a FINE prune at layer l shrinks the input of
    layer l + 1.  Counts depend only on (n, ratios, n_protected), never on the data."""
    counts, cur = [], n
    for l in range(n_layers):
        here = sorted([p for p in prunes if p.layer == l], key=lambda p: p.kind)
        for p in here:
            if p.kind == GLOBAL:
                cur = keep_count(cur, p.keep_ratio, n_protected)
        counts.append(cur)
        for p in here:
            if p.kind == FINE:
                cur = keep_count(cur, p.keep_ratio, n_protected)
    return counts


# --------------------------------------------------------------------------- selection
def _rank_value(scores: np.ndarray) -> np.ndarray:
    """Scores as comparable fp32 values: NaN -> -inf, -0.0 -> +0.0 (reading R6)."""
    s = np.asarray(scores, dtype=np.float32).copy()
    s[np.isnan(s)] = -np.inf
    s[s == 0] = 0.0
    return s


def select_keep(scores: np.ndarray, prot: np.ndarray, k: int) -> np.ndarray:
    """Indices kept by a fine prune, ascending (Section 2.2 Fine pruning; readings R5, R6).

    All protected tokens are kept; the remaining k - n_protected slots go to the candidates with the
    highest score, equal scores resolved toward the lower index."""
    prot = np.asarray(prot, dtype=bool)
    n = prot.shape[0]
    n_prot = int(prot.sum())
    if not (n_prot <= k <= n):
        raise ValueError("k must satisfy n_protected <= k <= n")
    cand = np.nonzero(~prot)[0]
    s = _rank_value(scores)[cand]
    order = np.argsort(-s, kind="stable")            # descending score, ascending index among equals
    chosen = cand[order[: k - n_prot]]
    keep = np.concatenate([np.nonzero(prot)[0], chosen])
    keep.sort()
    return keep.astype(np.int64)


def global_keep(prot: np.ndarray, k: int) -> np.ndarray:
    """Indices kept by global pruning, ascending (Section 2.2 Global pruning; reading R9):
    every protected token plus the earliest candidates by position."""
    prot = np.asarray(prot, dtype=bool)
    n = prot.shape[0]
    n_prot = int(prot.sum())
    if not (n_prot <= k <= n):
        raise ValueError("k must satisfy n_protected <= k <= n")
    cand = np.nonzero(~prot)[0]
    keep = np.concatenate([np.nonzero(prot)[0], cand[: k - n_prot]])
    keep.sort()
    return keep.astype(np.int64)


def latest_keep(prot: np.ndarray, k: int) -> np.ndarray:
    """Indices kept when the EARLIEST candidates are removed ("top informative", Table 2; reading R17):
    every protected token plus the latest candidates by position."""
    prot = np.asarray(prot, dtype=bool)
    n = prot.shape[0]
    n_prot = int(prot.sum())
    if not (n_prot <= k <= n):
        raise ValueError("k must satisfy n_protected <= k <= n")
    cand = np.nonzero(~prot)[0]
    keep = np.concatenate([np.nonzero(prot)[0], cand[len(cand) - (k - n_prot):]])
    keep.sort()
    return keep.astype(np.int64)


def mix32(h) -> np.ndarray:
    """The 32-bit avalanche mix (xor-shift 16, multiply, xor-shift 13, multiply, xor-shift 16) that ends the
    published MurmurHash3 hash; a bijection on 32-bit words."""
    h = np.asarray(h, dtype=np.uint64) & np.uint64(0xFFFFFFFF)
    h ^= h >> np.uint64(16)
    h = (h * np.uint64(0x85EBCA6B)) & np.uint64(0xFFFFFFFF)
    h ^= h >> np.uint64(13)
    h = (h * np.uint64(0xC2B2AE35)) & np.uint64(0xFFFFFFFF)
    h ^= h >> np.uint64(16)
    return h


def random_scores(seed: int, layer: int, sample: int, pos: np.ndarray) -> np.ndarray:
    """Uniform fp32 draws in [0, 1) for the "random" strategy of Tables 2-3 (reading R17): a counter-based
    generator keyed by (seed, layer, sample, original position), so the draw of a token does not depend on
    what was pruned before.  word = mix32(mix32(mix32(seed + G*(layer+1)) + G*(sample+1)) + pos), G = 0x9E3779B9;
    the draw is the word's top 24 bits times 2**-24 (exact in fp32)."""
    G, M = 0x9E3779B9, 0xFFFFFFFF
    h = mix32((int(seed) + G * (int(layer) + 1)) & M)
    h = mix32((int(h) + G * (int(sample) + 1)) & M)
    w = mix32((np.asarray(pos, dtype=np.uint64) + np.uint64(int(h))) & np.uint64(M))
    return ((w >> np.uint64(8)).astype(np.float64) * 2.0 ** -24).astype(np.float32)


def keep_by_selector(selector: int, kind: int, prot: np.ndarray, k: int, scores=None, rand=None) -> np.ndarray:
    """Kept indices (ascending) of one prune step under an ablation strategy of Tables 2-3 (reading R17).

    ``scores``: Eq. 4 scores (attentive strategies; FINE steps only, a GLOBAL step acts before the layer's
    attention exists); ``rand``: the uniform draws of the random strategy."""
    if selector == DEFAULT:
        selector = LOW_INFORMATIVE if kind == GLOBAL else LOW_ATTENTIVE
    if selector in (LOW_ATTENTIVE, TOP_ATTENTIVE):
        if kind != FINE:
            raise ValueError("attentive strategies need the layer's own attention: FINE steps only")
        s = np.asarray(scores, dtype=np.float32)
        return select_keep(s if selector == LOW_ATTENTIVE else -s, prot, k)
    if selector == LOW_INFORMATIVE:
        return global_keep(prot, k)
    if selector == TOP_INFORMATIVE:
        return latest_keep(prot, k)
    if selector == RANDOM:
        return select_keep(np.asarray(rand, dtype=np.float32), prot, k)
    raise ValueError("unknown selector")


# --------------------------------------------------------------------------- layer math
def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    ms = np.mean(np.square(x), axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotate-half rotary embedding on x[n, H, dh] with integer positions pos[n] (reading R8).

    Pair (i, i + dh/2) is rotated by the angle pos * base**(-2i/dh)."""
    n, H, dh = x.shape
    half = dh // 2
    inv_freq = np.asarray(base, dtype=np.float64) ** (-np.arange(half, dtype=np.float64) * 2.0 / dh)
    ang = pos.astype(np.float64)[:, None] * inv_freq[None, :]          # [n, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1).astype(x.dtype)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def _softmax_rows(z: np.ndarray) -> np.ndarray:
    z = z - np.max(z, axis=-1, keepdims=True)
    e = np.exp(z)
    return e / np.sum(e, axis=-1, keepdims=True)


def causal_gqa_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, row_block: int = 1024) -> np.ndarray:
    """softmax(q k^T / sqrt(dh) + causal mask) v for one sample (readings R1, R3).

    q[n,Hq,dh], k,v[n,Hkv,dh] -> [n,Hq,dh].  Every row is the plain definition (full softmax over its
    visible keys); the loop over row blocks only bounds the size of the materialised map."""
    n, Hq, dh = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    out = np.empty_like(q)
    scale = 1.0 / math.sqrt(dh)
    for h in range(Hq):
        kh, vh = k[:, h // G, :], v[:, h // G, :]
        for r0 in range(0, n, row_block):
            r1 = min(n, r0 + row_block)
            z = (q[r0:r1, h, :] @ kh[:r1].T) * scale                      # rows r0..r1-1 see keys < r1 at most
            rows = np.arange(r0, r1)[:, None]
            cols = np.arange(r1)[None, :]
            z = np.where(cols <= rows, z, -np.inf)
            out[r0:r1, h, :] = _softmax_rows(z) @ vh[:r1]
    return out


def causal_gqa_attention_rows(q: np.ndarray, k: np.ndarray, v: np.ndarray, rows: Sequence[int]) -> np.ndarray:
    """The rows ``rows`` of causal_gqa_attention(q, k, v), each written out from the definition on its own:
    row r of head h is softmax_j(q[r,h] . k[j,g(h)] / sqrt(dh), j <= r) applied to v[0..r, g(h)].  O(n) work per
    row and head, so single rows of a long sequence can be checked without forming anything n x n.
    -> [len(rows), Hq, dh]"""
    n, Hq, dh = q.shape
    G = Hq // k.shape[1]
    scale = 1.0 / math.sqrt(dh)
    out = np.empty((len(rows), Hq, dh), dtype=np.float64)
    for i, r in enumerate(rows):
        for h in range(Hq):
            z = (k[: r + 1, h // G, :].astype(np.float64) @ q[r, h, :].astype(np.float64)) * scale
            e = np.exp(z - z.max())
            out[i, h, :] = (e / e.sum()) @ v[: r + 1, h // G, :].astype(np.float64)
    return out


def last_query_scores(q: np.ndarray, k: np.ndarray, n_last: int = 1) -> np.ndarray:
    """Eq. 4: s = mean over heads of softmax(Q_last K^T)  (readings R1, R2, R3, R10).

    q[n,Hq,dh] and k[n,Hkv,dh] are the post-RoPE features of one sample; the result has length n.
    For n_last > 1 the mean also runs over the last n_last query rows, row r seeing keys 0..r."""
    n, Hq, dh = q.shape
    G = Hq // k.shape[1]
    scale = 1.0 / math.sqrt(dh)
    s = np.zeros(n, dtype=np.float64)
    rows = range(max(0, n - n_last), n)
    for r in rows:
        for h in range(Hq):
            z = (k[: r + 1, h // G, :].astype(np.float64) @ q[r, h, :].astype(np.float64)) * scale
            z -= z.max()
            e = np.exp(z)
            s[: r + 1] += e / e.sum()
    return s / (Hq * len(rows))


# --------------------------------------------------------------------------- decoder + pruning
def layer_qkv(x: np.ndarray, W: Dict[str, np.ndarray], pos: np.ndarray, m) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """RMSNorm -> Q/K/V projections -> RoPE on Q and K.  Weights are [out, in]."""
    n = x.shape[0]
    h = rmsnorm(x, W["g_attn"], m.rms_eps)
    q = (h @ W["wq"].T).reshape(n, m.n_q_heads, m.head_dim)
    k = (h @ W["wk"].T).reshape(n, m.n_kv_heads, m.head_dim)
    v = (h @ W["wv"].T).reshape(n, m.n_kv_heads, m.head_dim)
    return rope(q, pos, m.rope_base), rope(k, pos, m.rope_base), v


def layer_finish(x: np.ndarray, attn: np.ndarray, W: Dict[str, np.ndarray], m) -> np.ndarray:
    """x + attn Wo^T, then x + SwiGLU MLP of its RMSNorm."""
    n = x.shape[0]
    x = x + attn.reshape(n, -1) @ W["wo"].T
    h = rmsnorm(x, W["g_mlp"], m.rms_eps)
    return x + (silu(h @ W["w_gate"].T) * (h @ W["w_up"].T)) @ W["w_down"].T


def prefill_sample(m, weights, x: np.ndarray, spans: Sequence[Tuple[int, int]], prunes, n_last: int = 1,
                   dtype=np.float64, keep_kv: bool = True, trace: bool = False, sample_index: int = 0) -> Dict:
    """Pruned prefill of ONE sample (Fig. 3; Section 2.2).

    ``weights``: a sequence of per-layer dicts, or a callable ``layer -> dict`` (so big models need not
    be resident).  ``prunes``: objects with ``layer``, ``kind`` (GLOBAL/FINE), ``keep_ratio`` and optionally
    ``selector`` / ``seed`` (the ablation strategies of Tables 2-3, reading R17; ``sample_index`` keys the
    random strategy's draws).
    Returns x_out [n_final, d], kept_pos [n_final] (original positions), per-layer K/V (post-RoPE, of
    the tokens that survive that layer), and for every prune its scores / kept indices / counts."""
    get_w = weights if callable(weights) else (lambda l: weights[l])
    x = np.asarray(x, dtype=dtype)
    n0 = x.shape[0]
    pos = np.arange(n0, dtype=np.int64)
    prot = protected_mask(spans, n_last)
    out = {"kv": [], "prunes": [], "n_per_layer": []}
    if trace:
        out["trace"] = []
    for l in range(m.n_layers):
        W = {name: np.asarray(a, dtype=dtype) for name, a in get_w(l).items()}
        here = sorted([p for p in prunes if p.layer == l], key=lambda p: p.kind)
        for p in here:
            if p.kind == GLOBAL:                                            # reading R7: acts on the layer input
                k_keep = keep_count(x.shape[0], p.keep_ratio, int(prot.sum()))
                sel = getattr(p, "selector", DEFAULT)
                rand = random_scores(getattr(p, "seed", 0), l, sample_index, pos) if sel == RANDOM else None
                keep = keep_by_selector(sel, GLOBAL, prot, k_keep, None, rand)
                out["prunes"].append({"layer": l, "kind": GLOBAL, "n_in": x.shape[0], "k": k_keep, "selector": sel,
                                      "keep": keep, "pos_in": pos.copy(), "scores": None})
                x, pos, prot = x[keep], pos[keep], prot[keep]
        n = x.shape[0]
        out["n_per_layer"].append(n)
        q, k, v = layer_qkv(x, W, pos, m)
        attn = causal_gqa_attention(q, k, v)
        keep = None
        for p in here:
            if p.kind == FINE:
                s = last_query_scores(q, k, n_last)
                k_keep = keep_count(n, p.keep_ratio, int(prot.sum()))
                sel = getattr(p, "selector", DEFAULT)
                rand = random_scores(getattr(p, "seed", 0), l, sample_index, pos) if sel == RANDOM else None
                keep = keep_by_selector(sel, FINE, prot, k_keep, s.astype(np.float32), rand)
                out["prunes"].append({"layer": l, "kind": FINE, "n_in": n, "k": k_keep, "keep": keep, "selector": sel,
                                      "pos_in": pos.copy(), "scores": s})
        x_new = layer_finish(x, attn, W, m)
        if trace:
            out["trace"].append({"x_in": x, "q": q, "k": k, "v": v, "attn": attn, "x_out": x_new, "pos": pos.copy()})
        x = x_new
        if keep is not None:                                                # survivors only from here on
            x, pos, prot = x[keep], pos[keep], prot[keep]
            k, v = k[keep], v[keep]
        if keep_kv:
            out["kv"].append((k, v))
    out["x_out"] = x
    out["kept_pos"] = pos
    return out


def prefill(workload, weights, x: np.ndarray, dtype=np.float64, keep_kv: bool = True, trace: bool = False) -> List[Dict]:
    """Batched pruned prefill: samples never interact, so the batch is a loop over samples."""
    outs, row = [], 0
    for b, spans in enumerate(workload.samples):
        n = sum(l for _, l in spans)
        outs.append(prefill_sample(workload.model, weights, x[row:row + n], spans, workload.prunes,
                                   workload.n_last, dtype, keep_kv, trace, b))
        row += n
    return outs


# --------------------------------------------------------------------------- one decode step on the caches
def single_query_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """softmax(q k^T / sqrt(dh)) v for ONE query that sees every key (readings R1, R3).

    q[Hq,dh], k,v[n,Hkv,dh] -> [Hq,dh].  The generated token is the last position, so no mask applies."""
    Hq, dh = q.shape
    G = Hq // k.shape[1]
    out = np.empty_like(q)
    for h in range(Hq):
        z = (k[:, h // G, :] @ q[h]) / math.sqrt(dh)
        out[h] = _softmax_rows(z[None, :])[0] @ v[:, h // G, :]
    return out


def decode_step(m, weights, x_new: np.ndarray, pos_new: int, kv: Sequence[Tuple[np.ndarray, np.ndarray]],
                dtype=np.float64) -> Dict:
    """Forward of ONE new token of one sample over the per-layer K/V caches a (pruned) prefill left behind
    (Section 3.1: the paper's latency is the time to generate a single token; the memory it saves is these
    compacted caches).

    ``kv[l]`` = (K [n_l,Hkv,dh], V [n_l,Hkv,dh]) of layer l: post-RoPE keys of the tokens that survived that
    layer, plus anything generated since; n_l differs per layer once pruning has happened.  The new token
    carries RoPE position ``pos_new`` (its index in the ORIGINAL sequence, reading R8) and attends to the
    cache and to itself.  Returns x_out [d] and the token's own (k, v) per layer, to be appended."""
    get_w = weights if callable(weights) else (lambda l: weights[l])
    x = np.asarray(x_new, dtype=dtype)[None, :]
    pos = np.array([pos_new], dtype=np.int64)
    new_kv = []
    for l in range(m.n_layers):
        W = {name: np.asarray(a, dtype=dtype) for name, a in get_w(l).items()}
        q, k, v = layer_qkv(x, W, pos, m)                                   # [1,H,dh] each
        K = np.concatenate([np.asarray(kv[l][0], dtype=dtype), k], axis=0)
        V = np.concatenate([np.asarray(kv[l][1], dtype=dtype), v], axis=0)
        attn = single_query_attention(q[0], K, V)
        x = layer_finish(x, attn[None], W, m)
        new_kv.append((k[0], v[0]))
    return {"x_out": x[0], "kv": new_kv}


# --------------------------------------------------------------------------- attention rollout (Eq. 2-3)
def head_mean_attention_map(q: np.ndarray, k: np.ndarray) -> np.ndarray:
    """A^l of Section 2.2: the causal attention weights of one layer averaged over the query heads.

    q[n,Hq,dh], k[n,Hkv,dh] post-RoPE (readings R1-R3) -> A[n,n]; row i is token i's attention distribution
    over tokens 0..i (it sums to 1, entries right of the diagonal are 0)."""
    n, Hq, dh = q.shape
    G = Hq // k.shape[1]
    A = np.zeros((n, n), dtype=np.float64)
    rows, cols = np.arange(n)[:, None], np.arange(n)[None, :]
    for h in range(Hq):
        z = (q[:, h, :].astype(np.float64) @ k[:, h // G, :].astype(np.float64).T) / math.sqrt(dh)
        A += _softmax_rows(np.where(cols <= rows, z, -np.inf))
    return A / Hq


def rollout_step(R_prev: np.ndarray, A: np.ndarray, alpha: float) -> np.ndarray:
    """Eq. 2 then one factor of Eq. 3: R^l = (alpha A^l + (1 - alpha) I) R^{l-1}."""
    n = A.shape[0]
    return (alpha * A + (1.0 - alpha) * np.eye(n)) @ R_prev


def attention_rollout(m, weights, x: np.ndarray, alpha: float, dtype=np.float64) -> List[np.ndarray]:
    """R^1 .. R^L of Eq. 3 for one sample run through the UNPRUNED decoder (the paper computes the rollout on
    the full model to decide where to prune).  Entry [i, j] of R^l says how much input token j influences token
    i after l layers; every row sums to 1 and the matrices are lower triangular."""
    get_w = weights if callable(weights) else (lambda l: weights[l])
    x = np.asarray(x, dtype=dtype)
    n = x.shape[0]
    pos = np.arange(n, dtype=np.int64)
    R = np.eye(n)
    out = []
    for l in range(m.n_layers):
        W = {name: np.asarray(a, dtype=dtype) for name, a in get_w(l).items()}
        q, k, v = layer_qkv(x, W, pos, m)
        R = rollout_step(R, head_mean_attention_map(q, k), alpha)
        out.append(R)
        x = layer_finish(x, causal_gqa_attention(q, k, v), W, m)
    return out


def rollout_influence(R: np.ndarray) -> np.ndarray:
    """Influence of every input token under a rollout matrix (Section 2.2: entry [i, j] of R^l is how much input
    token j influences token i): the mean of column j over all n rows (reading R18).  Rows of R sum to 1, so the
    influences sum to 1 and a token with the uniform share has influence 1/n."""
    R = np.asarray(R, dtype=np.float64)
    return R.sum(axis=0) / R.shape[0]


def rollout_cutoff(R: np.ndarray, prot: np.ndarray, threshold: float) -> int:
    """Cut-off position of one sample (Section 2.2, Global pruning: a rollout threshold at the middle layer
    removes the less influential video/audio tokens, "typically those beyond position ..."; reading R18):
    one past the last candidate (unprotected) position whose influence is at least ``threshold`` uniform
    shares, i.e. influence * n >= threshold; 0 when no candidate reaches it.  Positional global pruning with
    this cut-off keeps every candidate before it."""
    prot = np.asarray(prot, dtype=bool)
    infl = rollout_influence(R)
    n = infl.shape[0]
    hit = np.nonzero((~prot) & (infl * n >= threshold))[0]
    return int(hit[-1]) + 1 if hit.size else 0


# --------------------------------------------------------------------------- FLOPs accounting
def decoder_flops(token_counts: Sequence[int], d: int, m_dim: int) -> float:
    """Theoretical FLOPs in the counting the paper adopts for its FLOPs column (Section 3.1,
    Evaluation protocol): per layer with n tokens, 4 n d^2 + 2 n^2 d + 2 n d m."""
    return float(sum(4.0 * n * d * d + 2.0 * n * n * d + 2.0 * n * d * m_dim for n in token_counts))
