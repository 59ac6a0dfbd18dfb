"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without any GPU.

Each test is chosen so that a plausible mistake in ``oracle/fastav_oracle.py`` (a dropped scale, a wrong
KV-head mapping, an off-by-one in the causal mask, a transposed weight, a wrong tie rule, a misplaced
prune) fails at least one of them.
"""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import fastav_inputs as fi
from oracle import brute
from oracle import fastav_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_qkv(n, Hq, Hkv, dh, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((n, Hq, dh)) * scale, rng.standard_normal((n, Hkv, dh)) * scale,
            rng.standard_normal((n, Hkv, dh)))


# ---------------------------------------------------------------- attention and Eq. 4 vs brute force
@pytest.mark.parametrize("n,Hq,Hkv,dh", [(1, 2, 1, 4), (7, 4, 2, 8), (19, 6, 2, 4), (12, 3, 3, 6)])
def test_attention_matches_bruteforce(n, Hq, Hkv, dh):
    q, k, v = _rand_qkv(n, Hq, Hkv, dh, 10 + n)
    got = orc.causal_gqa_attention(q, k, v, row_block=5)           # row blocks smaller than n
    want = np.asarray(brute.attention_output(q.tolist(), k.tolist(), v.tolist(), Hq // Hkv))
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_attention_rows_match_bruteforce_and_closed_forms():
    """The row-sampled form used for long sequences: chosen rows against the pure-loop brute force, against SDPA
    on a longer sequence, and two closed forms (one dominant key -> that key's value; zero query -> running mean)."""
    n, Hq, Hkv, dh = 19, 6, 2, 4
    q, k, v = _rand_qkv(n, Hq, Hkv, dh, 77)
    rows = [0, 1, 7, 18]
    got = orc.causal_gqa_attention_rows(q, k, v, rows)
    want = np.asarray(brute.attention_output(q.tolist(), k.tolist(), v.tolist(), Hq // Hkv))[rows]
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    n, Hq, Hkv, dh = 96, 8, 2, 16
    q, k, v = _rand_qkv(n, Hq, Hkv, dh, 78)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)[None]
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)[None]
    sdpa = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    rows = [0, 5, 50, 95]
    np.testing.assert_allclose(orc.causal_gqa_attention_rows(q, k, v, rows), sdpa[rows], rtol=1e-10, atol=1e-12)
    # key 30 dominates every later row (its logit exceeds all others by > 700 * ln 2): the output is v[30]
    kk = k.copy()
    qq = np.abs(q) + 0.1
    kk[30] = 1000.0
    out = orc.causal_gqa_attention_rows(qq, kk, v, [29, 30, 60])
    for h in range(Hq):
        np.testing.assert_allclose(out[1, h], v[30, h // (Hq // Hkv)], rtol=1e-12)
        np.testing.assert_allclose(out[2, h], v[30, h // (Hq // Hkv)], rtol=1e-12)
        assert np.abs(out[0, h] - v[30, h // (Hq // Hkv)]).max() > 1e-3          # row 29 cannot see key 30
    out0 = orc.causal_gqa_attention_rows(np.zeros_like(q), k, v, [9])
    np.testing.assert_allclose(out0[0, 3], v[:10, 0].mean(axis=0), rtol=1e-12)


@pytest.mark.parametrize("n_last", [1, 2, 5])
def test_scores_equal_last_rows_of_head_mean_map(n_last):
    """Eq. 4 == last row(s) of the head-averaged full attention map A of Section 2.2."""
    n, Hq, Hkv, dh = 17, 4, 2, 8
    q, k, _ = _rand_qkv(n, Hq, Hkv, dh, 3)
    got = orc.last_query_scores(q, k, n_last)
    want = np.asarray(brute.head_mean_last_rows(q.tolist(), k.tolist(), Hq // Hkv, n_last))
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-15)
    assert abs(got.sum() - 1.0) < 1e-12                           # mean of distributions is a distribution


def test_attention_matches_torch_sdpa():
    n, Hq, Hkv, dh = 96, 8, 2, 16
    q, k, v = _rand_qkv(n, Hq, Hkv, dh, 4)
    got = orc.causal_gqa_attention(q, k, v, row_block=40)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)[None]
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)[None]
    want = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)


def test_softmax_rows_sum_to_one_and_scores_sum_to_one():
    n, Hq, Hkv, dh = 33, 4, 1, 8
    q, k, v = _rand_qkv(n, Hq, Hkv, dh, 5, scale=3.0)
    ones = np.ones_like(v)
    out = orc.causal_gqa_attention(q, k, ones, row_block=8)        # P @ 1 = row sums
    np.testing.assert_allclose(out, 1.0, rtol=0, atol=1e-12)
    for n_last in (1, 3, 33):
        s = orc.last_query_scores(q, k, n_last)
        assert abs(s.sum() - 1.0) < 1e-12 and (s >= 0).all()


def test_scores_closed_forms():
    n, Hq, Hkv, dh = 40, 4, 2, 8
    q, k, _ = _rand_qkv(n, Hq, Hkv, dh, 6)
    # zero query -> zero logits -> exactly uniform
    s = orc.last_query_scores(np.zeros_like(q), k, 1)
    np.testing.assert_allclose(s, 1.0 / n, rtol=1e-15)
    # one key aligned with every head's last query and scaled up -> one-hot
    k2 = k * 0.01
    j = 11
    for g in range(Hkv):
        k2[j, g] = 50.0 * q[n - 1, g * (Hq // Hkv)] / np.linalg.norm(q[n - 1, g * (Hq // Hkv)])
    q2 = q.copy()
    for h in range(Hq):
        q2[n - 1, h] = q[n - 1, (h // (Hq // Hkv)) * (Hq // Hkv)] * 5.0
    s = orc.last_query_scores(q2, k2, 1)
    assert s[j] > 1 - 1e-9
    # 1/sqrt(dh) scale: two keys with logits differing by known amount
    q3 = np.zeros((2, 1, 4)); k3 = np.zeros((2, 1, 4))
    q3[1, 0, 0] = 2.0; k3[0, 0, 0] = 3.0                         # logit(0) = 6/sqrt(4) = 3, logit(1) = 0
    s = orc.last_query_scores(q3, k3, 1)
    np.testing.assert_allclose(s, [math.exp(3) / (1 + math.exp(3)), 1 / (1 + math.exp(3))], rtol=1e-14)


def test_gqa_head_mapping():
    """Query head h must read KV head h // G: make KV heads distinguishable."""
    n, Hq, Hkv, dh = 6, 4, 2, 4
    q, k, v = _rand_qkv(n, Hq, Hkv, dh, 7)
    v[:, 0, :] = 1.0
    v[:, 1, :] = -2.0
    out = orc.causal_gqa_attention(q, k, v)
    np.testing.assert_allclose(out[:, :2], 1.0, atol=1e-12)
    np.testing.assert_allclose(out[:, 2:], -2.0, atol=1e-12)


# ---------------------------------------------------------------- row-wise ops vs library routines / loops
def test_rmsnorm_silu_match_torch_and_loops():
    rng = np.random.default_rng(8)
    x = rng.standard_normal((5, 24)); g = 1 + 0.1 * rng.standard_normal(24)
    got = orc.rmsnorm(x, g, 1e-6)
    want = F.rms_norm(torch.from_numpy(x), (24,), torch.from_numpy(g), 1e-6).numpy()
    np.testing.assert_allclose(got, want, rtol=1e-12)
    np.testing.assert_allclose(got[2], brute.rmsnorm_row(x[2].tolist(), g.tolist(), 1e-6), rtol=1e-12)
    np.testing.assert_allclose(orc.silu(x), F.silu(torch.from_numpy(x)).numpy(), rtol=1e-12)


def test_rope_invariants_and_loops():
    rng = np.random.default_rng(9)
    n, H, dh, base = 9, 3, 16, 1.0e4
    x = rng.standard_normal((n, H, dh))
    pos = np.array([0, 1, 2, 5, 9, 100, 101, 4000, 16383])
    y = orc.rope(x, pos, base)
    np.testing.assert_allclose(y[0], x[0], rtol=0, atol=0)                       # position 0 is the identity
    half = dh // 2
    np.testing.assert_allclose(y[..., :half] ** 2 + y[..., half:] ** 2,
                               x[..., :half] ** 2 + x[..., half:] ** 2, rtol=1e-12)  # per-pair norm preserved
    for t in (3, 7):
        np.testing.assert_allclose(y[t, 1], brute.rope_vec(x[t, 1].tolist(), int(pos[t]), base), rtol=1e-10, atol=1e-12)
    # <rope(a,p1), rope(b,p2)> depends only on p1 - p2
    a, b = rng.standard_normal((1, 1, dh)), rng.standard_normal((1, 1, dh))
    def dot(p1, p2):
        return float(np.sum(orc.rope(a, np.array([p1]), base) * orc.rope(b, np.array([p2]), base)))
    assert abs(dot(7, 3) - dot(1004, 1000)) < 1e-9
    assert abs(dot(7, 3) - dot(3, 7)) > 1e-3                                       # and is not symmetric


def test_weights_are_out_by_in():
    """layer_qkv / layer_finish multiply by W^T with W stored [out, in]: compare with torch linear."""
    m = fi.Model(1, 16, 4, 2, 4, 24, 1.0e4, 1e-6, "f32")
    W = {k: v.astype(np.float64) for k, v in fi.layer_weights(m, 0, seed=3).items()}
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 16))
    pos = np.zeros(5, dtype=np.int64)                                              # RoPE identity
    q, k, v = orc.layer_qkv(x, W, pos, m)
    h = F.rms_norm(torch.from_numpy(x), (16,), torch.from_numpy(W["g_attn"]), 1e-6)
    np.testing.assert_allclose(q.reshape(5, -1), F.linear(h, torch.from_numpy(W["wq"])).numpy(), rtol=1e-12)
    np.testing.assert_allclose(v.reshape(5, -1), F.linear(h, torch.from_numpy(W["wv"])).numpy(), rtol=1e-12)
    attn = rng.standard_normal((5, 4, 4))
    got = orc.layer_finish(x, attn, W, m)
    t = torch.from_numpy(x) + F.linear(torch.from_numpy(attn.reshape(5, -1)), torch.from_numpy(W["wo"]))
    h2 = F.rms_norm(t, (16,), torch.from_numpy(W["g_mlp"]), 1e-6)
    t = t + F.linear(F.silu(F.linear(h2, torch.from_numpy(W["w_gate"]))) * F.linear(h2, torch.from_numpy(W["w_up"])),
                     torch.from_numpy(W["w_down"]))
    np.testing.assert_allclose(got, t.numpy(), rtol=1e-12)


# ---------------------------------------------------------------- selection
@pytest.mark.parametrize("kind", ["softmax", "ties", "equal", "mixed"])
@pytest.mark.parametrize("n", [1, 2, 13, 64, 257])
def test_select_equals_full_sort(kind, n):
    rng = np.random.default_rng(n)
    s = fi.random_scores(n, 100 + n, kind)
    for prot_kind in ("none", "ends", "random"):
        prot = np.zeros(n, dtype=bool)
        if prot_kind == "ends":
            prot[: min(2, n)] = True; prot[-1] = True
        elif prot_kind == "random":
            prot = rng.random(n) < 0.3
        n_prot = int(prot.sum())
        for k in sorted({n_prot, n, (n_prot + n) // 2, min(n, n_prot + 1)}):
            got = orc.select_keep(s, prot, k)
            want = brute.topk_by_full_sort(s.tolist(), prot.tolist(), k)
            assert got.tolist() == want
            assert len(got) == k and (np.diff(got) > 0).all() and prot[got].sum() == n_prot


def test_select_signed_zero_and_nan_rules():
    s = np.array([0.0, -0.0, np.nan, -np.inf, 1.0], dtype=np.float32)
    prot = np.zeros(5, dtype=bool)
    assert orc.select_keep(s, prot, 2).tolist() == [0, 4]          # +0 and -0 tie -> lower index
    assert orc.select_keep(s, prot, 3).tolist() == [0, 1, 4]
    assert orc.select_keep(s, prot, 4).tolist() == [0, 1, 2, 4]    # NaN ties with -inf -> lower index


def test_keep_count_rule():
    assert orc.keep_count(2048, 0.6, 0) == 1229
    assert orc.keep_count(2458, 0.7, 0) == 1721
    assert orc.keep_count(1721, 0.7, 0) == 1205
    assert orc.keep_count(5735, 0.7, 0) == 4015
    assert orc.keep_count(16384, 0.5, 0) == 8192
    assert orc.keep_count(10, 0.3, 0) == 3                         # 0.3*10 = 3.0000000000000004 must not give 4
    assert orc.keep_count(10, 0.1, 4) == 4                         # never below the protected count
    assert orc.keep_count(10, 1.0, 0) == 10


def test_global_rule_reproduces_paper_rules():
    """Section 3.1 Implementation details: VideoLLaMA2 keeps all video + the first 10 audio tokens;
    video-SALMONN2 (frame-interleaved) keeps the first 4 frames."""
    M, U, E = 676, 1496, 64
    spans = [(orc.VIDEO, M), (orc.AUDIO, U), (orc.TEXT, E)]
    prot = orc.protected_mask(spans, 1)
    keep = orc.global_keep(prot, E + M + 10)
    assert keep.tolist() == list(range(M + 10)) + list(range(M + U, M + U + E))
    frames = []
    for _ in range(10):
        frames += [(orc.VIDEO, 30), (orc.AUDIO, 12)]
    spans = [(orc.TEXT, 5)] + frames + [(orc.TEXT, 9)]
    prot = orc.protected_mask(spans, 1)
    keep = orc.global_keep(prot, 5 + 9 + 4 * 42)
    assert keep.tolist() == list(range(5 + 4 * 42)) + list(range(5 + 10 * 42, 5 + 10 * 42 + 9))


def test_table4_flops_fix_prune_placement():
    """The paper's FLOPs column (Table 4) is reproduced within +-1 point by the schedule semantics of
    reading R7 on a VideoLLaMA2-shaped sequence; shifting the global prune by one layer, or not
    compounding the fine prune per layer, misses it."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table4_flops.txt")) if l.strip() and not l.startswith("#")]
    printed = {int(p): float(v) for p, v in rows}
    L, d, mlp = 28, 3584, 18944
    M, U, E = 676, 1496, 64                       # 1,496 audio tokens; M + E + 10 = 750 survivors
    n = M + U + E
    g = (M + 10 + E) / n
    base = orc.decoder_flops([n] * L, d, mlp)

    def rel(global_layer, P, compound=True):
        prunes = [fi.Prune(global_layer, fi.GLOBAL, g)]
        if P > 0:
            last = L if compound else global_layer + 1
            prunes += [fi.Prune(l, fi.FINE, 1.0 - P) for l in range(global_layer, last)]
        counts = orc.token_schedule(n, E, prunes, L)
        return 100.0 * orc.decoder_flops(counts, d, mlp) / base

    for P, want in printed.items():
        assert abs(rel(14, P / 100.0) - want) <= 1.0, (P, rel(14, P / 100.0), want)
    assert abs(rel(13, 0.0) - printed[0]) > 1.0 and abs(rel(15, 0.0) - printed[0]) > 1.0
    assert abs(rel(14, 0.2, compound=False) - printed[20]) > 1.0


def test_paper_schedule_helper_reproduces_table4():
    """The schedule helper the benchmark and the GPU parity test use (global prune on the input of the middle layer,
    fine prunes from that layer on) gives Table 4's FLOPs column within +-1 point for P = 10 / 20 / 30 % on the
    VideoLLaMA2-shaped sequence; starting the fine prunes one layer later misses P = 30 %."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table4_flops.txt")) if l.strip() and not l.startswith("#")]
    printed = {int(p): float(v) for p, v in rows}
    L, d, mlp = 28, 3584, 18944
    M, U, E = 676, 1496, 64
    n = M + U + E
    g = (M + 10 + E) / n
    m = fi.Model(L, d, 28, 4, 128, mlp, 1.0e6, 1e-6, "bf16")
    base_w = fi.Workload("vl2", m, [[(fi.VIDEO, M), (fi.AUDIO, U), (fi.TEXT, E)]], [])
    base = orc.decoder_flops([n] * L, d, mlp)
    for P in (10, 20, 30):
        w = fi.paper_schedule(base_w, global_keep=g, fine_drop=P / 100.0)
        assert w.prunes[0].kind == fi.GLOBAL and w.prunes[0].layer == 14
        assert [(p.layer, p.kind) for p in w.prunes[1:]] == [(l, fi.FINE) for l in range(14, L)]
        counts = orc.token_schedule(n, E, w.prunes, L)
        got = 100.0 * orc.decoder_flops(counts, d, mlp) / base
        assert abs(got - printed[P]) <= 1.0, (P, got, printed[P])
    late = [fi.Prune(14, fi.GLOBAL, g)] + [fi.Prune(l, fi.FINE, 0.7) for l in range(15, L)]
    got_late = 100.0 * orc.decoder_flops(orc.token_schedule(n, E, late, L), d, mlp) / base
    assert abs(got_late - printed[30]) > 1.0, got_late


# ---------------------------------------------------------------- the pruned prefill as a whole
def _tiny():
    m = fi.Model(4, 32, 4, 2, 8, 48, 1.0e4, 1e-6, "f32")
    w = fi.Workload("t", m, [[(fi.TEXT, 3), (fi.VIDEO, 20), (fi.AUDIO, 14), (fi.TEXT, 4)]],
                    [fi.Prune(1, fi.GLOBAL, 0.6), fi.Prune(2, fi.FINE, 0.7), fi.Prune(3, fi.FINE, 0.7)], seed=77)
    weights = [fi.layer_weights(m, l, 5) for l in range(m.n_layers)]
    for W in weights:                                # larger weights so attention is far from uniform
        for name in ("wq", "wk"):
            W[name] = W[name] * 30.0
    return m, w, weights, fi.embeddings(w)


def test_keep_ratio_one_is_identity():
    m, w, weights, x = _tiny()
    plain = orc.prefill(fi.unpruned(w), weights, x)[0]
    w1 = fi.Workload("t1", m, w.samples, [fi.Prune(p.layer, p.kind, 1.0) for p in w.prunes], seed=w.seed)
    same = orc.prefill(w1, weights, x)[0]
    assert np.array_equal(plain["x_out"], same["x_out"])
    assert np.array_equal(same["kept_pos"], np.arange(41))


def test_prefill_schedule_structure_and_original_positions():
    m, w, weights, x = _tiny()
    out = orc.prefill(w, weights, x, trace=True)[0]
    n_prot = 7
    assert out["n_per_layer"] == orc.token_schedule(41, n_prot, w.prunes, m.n_layers)
    assert out["n_per_layer"] == [41, 25, 25, 18]
    assert out["x_out"].shape[0] == 13 == len(out["kept_pos"])
    kp = out["kept_pos"]
    assert (np.diff(kp) > 0).all() and kp[-1] == 40 and set(range(3)) <= set(kp) and set(range(37, 41)) <= set(kp)
    # global prune kept the earliest candidates
    assert out["prunes"][0]["keep"].tolist() == list(range(3 + 18)) + list(range(37, 41))
    # K/V of a fine layer are compacted, earlier layers untouched
    assert [kv[0].shape[0] for kv in out["kv"]] == [41, 25, 18, 13]
    # RoPE used original positions after pruning: layer 3's K equals a fresh projection with pos = kept positions
    t3 = out["trace"][3]
    W3 = {k: v.astype(np.float64) for k, v in weights[3].items()}
    q, k, v = orc.layer_qkv(t3["x_in"], W3, t3["pos"], m)
    np.testing.assert_array_equal(k, t3["k"])
    assert t3["pos"].max() == 40 and len(t3["pos"]) == 18
    # fine scores are a distribution over the tokens present at that layer
    s = out["prunes"][1]["scores"]
    assert len(s) == 25 and abs(s.sum() - 1) < 1e-12


def test_in_layer_compaction_equals_end_of_layer():
    """O-projection, RMSNorm, MLP and residual are row-wise, so removing rows right after attention gives
    the same surviving rows as removing them at the end of the layer."""
    m, w, weights, x = _tiny()
    out = orc.prefill(w, weights, x, trace=True)[0]
    t2 = out["trace"][2]
    keep = out["prunes"][1]["keep"]
    W2 = {k: v.astype(np.float64) for k, v in weights[2].items()}
    early = orc.layer_finish(t2["x_in"][keep], t2["attn"][keep], W2, m)
    np.testing.assert_allclose(early, t2["x_out"][keep], rtol=1e-12, atol=1e-13)


def test_uniform_scores_make_fine_equal_earliest_first():
    """With Wq = 0 every logit is 0, s_j = 1/n exactly, every candidate ties, and the tie rule makes the
    fine prune keep the earliest candidates — the global rule."""
    m, w, weights, x = _tiny()
    for W in weights:
        W["wq"] = np.zeros_like(W["wq"])
    w2 = fi.Workload("t2", m, w.samples, [fi.Prune(2, fi.FINE, 0.5)], seed=w.seed)
    out = orc.prefill(w2, weights, x)[0]
    p = out["prunes"][0]
    np.testing.assert_allclose(p["scores"], 1.0 / 41, rtol=1e-14)
    prot = orc.protected_mask(w.samples[0], 1)
    assert p["keep"].tolist() == orc.global_keep(prot, p["k"]).tolist()


def test_batch_is_a_loop_over_samples():
    m, w, weights, x = _tiny()
    w_b = fi.Workload("tb", m, [w.samples[0], [(fi.VIDEO, 10), (fi.AUDIO, 9), (fi.TEXT, 2)]], w.prunes, seed=3)
    xb = fi.embeddings(w_b)
    outs = orc.prefill(w_b, weights, xb)
    solo = orc.prefill_sample(m, weights, xb[41:], w_b.samples[1], w.prunes)
    assert np.array_equal(outs[1]["x_out"], solo["x_out"]) and np.array_equal(outs[1]["kept_pos"], solo["kept_pos"])


def test_input_generators_shapes():
    for i in range(1, 6):
        w = fi.config(i)
        assert all(n > 0 for n in w.seqlens)
    assert fi.config(1).seqlens == [512] and fi.config(2).seqlens == [2048]
    assert fi.config(3).seqlens == [4096] and fi.config(4).seqlens == [16384]
    w5 = fi.config(5)
    assert len(w5.seqlens) == 8 and all(2048 <= n <= 6144 for n in w5.seqlens)
    for s in w5.samples:
        n = sum(l for _, l in s)
        assert 0.55 <= s[0][1] / n <= 0.80 and 0.15 <= s[1][1] / n <= 0.35 and s[2][1] >= 8
    a = np.array([1.0, 1.00390625, 1.01171875, 3.14159], dtype=np.float32)      # 1+2^-8 ties to even (down), 1+3*2^-8 ties up
    r = fi.round_bf16(a.copy())
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == np.float32(1.015625)
    assert r[3] == torch.tensor(3.14159).to(torch.bfloat16).float().item()


# ------------------------------------------------------------------------------------ decode step
def test_decode_step_equals_last_row_of_a_longer_prefill():
    """With unpruned caches, the forward of token n over the caches of tokens 0..n-1 IS row n of a causal
    prefill over n+1 tokens: the definition the decode step must reproduce."""
    m, w, weights, x = _tiny()
    n = x.shape[0] - 1
    spans = [(fi.TEXT, n)]
    head = orc.prefill_sample(m, weights, x[:n], spans, [])
    full = orc.prefill_sample(m, weights, x, [(fi.TEXT, n + 1)], [])
    step = orc.decode_step(m, weights, x[n], n, head["kv"])
    np.testing.assert_allclose(step["x_out"], full["x_out"][n], rtol=1e-11, atol=1e-12)
    for l in range(m.n_layers):
        np.testing.assert_allclose(step["kv"][l][0], full["kv"][l][0][n], rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(step["kv"][l][1], full["kv"][l][1][n], rtol=1e-11, atol=1e-12)
    # a second step on the grown caches equals row n+1 of a prefill over n+2 tokens
    x2 = np.concatenate([x, x[3:4] * 0.5 + 0.1], axis=0)
    grown = [(np.concatenate([head["kv"][l][0], step["kv"][l][0][None]]), np.concatenate([head["kv"][l][1], step["kv"][l][1][None]]))
             for l in range(m.n_layers)]
    step2 = orc.decode_step(m, weights, x2[n + 1], n + 1, grown)
    full2 = orc.prefill_sample(m, weights, x2, [(fi.TEXT, n + 2)], [])
    np.testing.assert_allclose(step2["x_out"], full2["x_out"][n + 1], rtol=1e-11, atol=1e-12)


def test_decode_step_on_pruned_caches_sees_a_set_of_keys():
    """On pruned caches the layers hold different numbers of keys; the step depends on each cache as a SET
    (keys carry their rotary position already), and matches brute-force loops."""
    m, w, weights, x = _tiny()
    out = orc.prefill(w, weights, x)[0]
    assert [kv[0].shape[0] for kv in out["kv"]] == [41, 25, 18, 13]
    x_new = x[5] * 0.7 - 0.2
    step = orc.decode_step(m, weights, x_new, 41, out["kv"])
    rng = np.random.default_rng(0)
    shuffled = []
    for K, V in out["kv"]:
        p = rng.permutation(K.shape[0])
        shuffled.append((K[p], V[p]))
    step_p = orc.decode_step(m, weights, x_new, 41, shuffled)
    np.testing.assert_allclose(step_p["x_out"], step["x_out"], rtol=1e-11, atol=1e-12)
    # layer 0 attention by explicit loops: query = the new token, keys = cache + itself
    W0 = {k: v.astype(np.float64) for k, v in weights[0].items()}
    q, k, v = orc.layer_qkv(x_new[None].astype(np.float64), W0, np.array([41]), m)
    K = np.concatenate([out["kv"][0][0], k]); V = np.concatenate([out["kv"][0][1], v])
    nk = K.shape[0]
    qq = np.concatenate([np.zeros((nk - 1,) + q.shape[1:]), q])          # brute works on causal rows: use the last
    want = np.array(brute.attention_output(qq.tolist(), K.tolist(), V.tolist(), m.n_q_heads // m.n_kv_heads)[nk - 1])
    got = orc.single_query_attention(q[0], K, V)
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)


# ------------------------------------------------------------------------------------ attention rollout (Eq. 2-3)
def test_attention_map_is_the_head_mean_of_brute_force_maps():
    rng = np.random.default_rng(4)
    n, Hq, Hkv, dh = 9, 4, 2, 8
    q, k = rng.standard_normal((n, Hq, dh)), rng.standard_normal((n, Hkv, dh))
    A = orc.head_mean_attention_map(q, k)
    want = np.mean([np.array(brute.attention_map(q.tolist(), k.tolist(), h, Hq // Hkv)) for h in range(Hq)], axis=0)
    np.testing.assert_allclose(A, want, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(A.sum(axis=1), 1.0, rtol=1e-13)
    assert np.all(np.triu(A, 1) == 0.0)
    # its last row is Eq. 4's score vector: the fine prune and the rollout look at the same attention weights
    np.testing.assert_allclose(A[-1], orc.last_query_scores(q, k), rtol=1e-12, atol=1e-15)


def test_rollout_matches_explicit_products_and_closed_forms():
    m, w, weights, x = _tiny()
    alpha = 0.6
    R = orc.attention_rollout(m, weights, x, alpha)
    assert len(R) == m.n_layers
    # Eq. 3 by explicit loops over the layer maps, in the printed order (newest factor on the left)
    out = orc.prefill(fi.unpruned(w), weights, x, trace=True)[0]
    n = x.shape[0]
    At = [alpha * orc.head_mean_attention_map(t["q"], t["k"]) + (1 - alpha) * np.eye(n) for t in out["trace"]]
    prod = [[float(i == j) for j in range(n)] for i in range(n)]
    for A in At:                                            # triple loop: prod = A @ prod
        prod = [[sum(A[i][kk] * prod[kk][j] for kk in range(n)) for j in range(n)] for i in range(n)]
    np.testing.assert_allclose(R[-1], np.array(prod), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(R[1], At[1] @ At[0], rtol=1e-12, atol=1e-14)
    for r in R:
        np.testing.assert_allclose(r.sum(axis=1), 1.0, rtol=1e-12)      # product of row-stochastic matrices
        assert np.all(np.triu(r, 1) == 0.0) and (r >= 0).all()
    # alpha = 0 keeps every token's own representation only
    for r in orc.attention_rollout(m, weights, x, 0.0):
        np.testing.assert_array_equal(r, np.eye(n))
    # uniform attention (Wq = 0): A[i][j] = 1/(i+1) for j <= i in every layer
    flat = [dict(W, wq=np.zeros_like(W["wq"])) for W in weights]
    U = np.tril(np.ones((n, n))) / np.arange(1, n + 1)[:, None]
    R1 = orc.attention_rollout(m, flat, x, 1.0)
    np.testing.assert_allclose(R1[0], U, rtol=1e-12)
    np.testing.assert_allclose(R1[2], U @ U @ U, rtol=1e-11)


# ---------------------------------------------------------------- ablation selectors (Tables 2-3)
def _unmix32(h: int) -> int:
    """Inverse of the 32-bit avalanche mix, from the algebra alone: an xor-shift by s >= 11 undoes itself in at
    most three applications, an odd multiplier has an inverse modulo 2**32."""
    M = 0xFFFFFFFF
    h ^= h >> 16
    h = (h * pow(0xC2B2AE35, -1, 1 << 32)) & M
    h ^= (h >> 13) ^ (h >> 26)
    h = (h * pow(0x85EBCA6B, -1, 1 << 32)) & M
    h ^= h >> 16
    return h


def test_mix32_is_the_bijection_its_inverse_undoes():
    rng = np.random.default_rng(5)
    xs = np.concatenate([np.arange(0, 4096, dtype=np.uint64), rng.integers(0, 1 << 32, 4096, dtype=np.uint64),
                         np.array([0xFFFFFFFF, 0x80000000, 0x7FFFFFFF], dtype=np.uint64)])
    ys = orc.mix32(xs)
    assert int(orc.mix32(0)) == 0                                   # every step maps 0 to 0
    assert ys.max() <= 0xFFFFFFFF and len(set(ys.tolist())) == len(set(xs.tolist()))
    assert [_unmix32(int(y)) for y in ys] == [int(x) for x in xs]
    # avalanche: flipping one input bit flips about half of the output bits
    flips = [bin(int(orc.mix32(int(x) ^ (1 << b))) ^ int(y)).count("1") for x, y in zip(xs[:512], ys[:512]) for b in (0, 13, 31)]
    assert 14.5 < np.mean(flips) < 17.5


def test_random_scores_are_uniform_counter_based_draws():
    pos = np.arange(20000)
    u = orc.random_scores(7, 3, 1, pos)
    assert u.dtype == np.float32 and u.min() >= 0.0 and u.max() < 1.0
    assert np.array_equal(u * 2.0 ** 24, np.floor(u * 2.0 ** 24))    # 24-bit fractions
    assert abs(u.mean() - 0.5) < 0.01 and abs(u.var() - 1.0 / 12.0) < 0.004
    hist = np.bincount((u * 16).astype(int), minlength=16)
    assert (((hist - 1250.0) ** 2) / 1250.0).sum() < 45.0             # chi-square, 15 dof (p ~ 1e-4)
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.03               # neighbouring counters uncorrelated
    # counter-based: a token's draw depends on its own position only, not on which others are present
    sub = np.array([5, 17, 400, 19999])
    assert np.array_equal(orc.random_scores(7, 3, 1, sub), u[sub])
    # every key component matters
    for other in (orc.random_scores(8, 3, 1, pos), orc.random_scores(7, 4, 1, pos), orc.random_scores(7, 3, 2, pos)):
        assert (other == u).mean() < 0.001 and abs(np.corrcoef(other, u)[0, 1]) < 0.03


@pytest.mark.parametrize("n", [1, 2, 13, 64, 257])
def test_selectors_against_sorted_brute_force(n):
    rng = np.random.default_rng(300 + n)
    s = fi.random_scores(n, 500 + n, "softmax")
    prot = rng.random(n) < 0.25
    n_prot = int(prot.sum())
    cand = [j for j in range(n) if not prot[j]]
    r = orc.random_scores(11, 2, 0, np.arange(n))
    for k in sorted({n_prot, n, (n_prot + n) // 2, min(n, n_prot + 1)}):
        c = k - n_prot
        want = {
            orc.LOW_ATTENTIVE: sorted(cand, key=lambda j: (-float(s[j]), j))[:c],
            orc.TOP_ATTENTIVE: sorted(cand, key=lambda j: (float(s[j]), j))[:c],
            orc.LOW_INFORMATIVE: cand[:c],
            orc.TOP_INFORMATIVE: cand[len(cand) - c:],
            orc.RANDOM: sorted(cand, key=lambda j: (-float(r[j]), j))[:c],
        }
        for sel, chosen in want.items():
            got = orc.keep_by_selector(sel, orc.FINE if sel in (orc.LOW_ATTENTIVE, orc.TOP_ATTENTIVE) else orc.GLOBAL,
                                       prot, k, s, r)
            assert got.tolist() == sorted([j for j in range(n) if prot[j]] + chosen), (sel, k)
            assert len(got) == k                                        # every strategy keeps the same count
    # defaults are the paper's own rules
    k = (n_prot + n) // 2
    assert np.array_equal(orc.keep_by_selector(orc.DEFAULT, orc.GLOBAL, prot, k), orc.global_keep(prot, k))
    assert np.array_equal(orc.keep_by_selector(orc.DEFAULT, orc.FINE, prot, k, s), orc.select_keep(s, prot, k))


def test_selector_symmetries():
    rng = np.random.default_rng(9)
    n = 90
    prot = rng.random(n) < 0.2
    n_prot, n_cand = int(prot.sum()), int((~prot).sum())
    s = rng.permutation(n).astype(np.float32)                          # distinct scores: no ties
    for c in (0, 1, n_cand // 3, n_cand):
        lo = orc.keep_by_selector(orc.LOW_ATTENTIVE, orc.FINE, prot, n_prot + c, s)
        hi = orc.keep_by_selector(orc.TOP_ATTENTIVE, orc.FINE, prot, n_prot + n_cand - c, s)
        # keeping the c best and keeping the n_cand - c worst split the candidates between them
        both = np.intersect1d(lo, hi)
        assert np.array_equal(both, np.nonzero(prot)[0]) and len(np.union1d(lo, hi)) == n
        # top informative is low informative on the reversed sequence
        early = orc.keep_by_selector(orc.LOW_INFORMATIVE, orc.GLOBAL, prot, n_prot + c)
        late_rev = orc.keep_by_selector(orc.TOP_INFORMATIVE, orc.GLOBAL, prot[::-1], n_prot + c)
        assert np.array_equal(np.sort(n - 1 - late_rev), early)
    with pytest.raises(ValueError):
        orc.keep_by_selector(orc.TOP_ATTENTIVE, orc.GLOBAL, prot, n_prot + 1, s)


def test_prefill_with_ablation_selectors_keeps_counts_and_rules():
    m, w, weights, x = _tiny()
    base = orc.prefill(w, weights, x)[0]
    n_prot = 7
    for sel_g, sel_f in [(orc.TOP_INFORMATIVE, orc.TOP_ATTENTIVE), (orc.RANDOM, orc.RANDOM), (orc.LOW_INFORMATIVE, orc.LOW_ATTENTIVE)]:
        prunes = [fi.Prune(p.layer, p.kind, p.keep_ratio, sel_g if p.kind == fi.GLOBAL else sel_f, 123) for p in w.prunes]
        wv = fi.Workload("tv", m, w.samples, prunes, seed=w.seed)
        out = orc.prefill(wv, weights, x)[0]
        assert out["n_per_layer"] == base["n_per_layer"]               # same FLOPs for every strategy
        kp = out["kept_pos"]
        assert set(range(3)) <= set(kp) and set(range(37, 41)) <= set(kp)
        g = out["prunes"][0]
        if sel_g == orc.TOP_INFORMATIVE:
            assert g["keep"].tolist() == list(range(3)) + list(range(37 - 18, 37)) + list(range(37, 41))
            f = out["prunes"][1]                                       # removed = the highest-scored candidates
            removed = np.setdiff1d(np.arange(f["n_in"]), f["keep"])
            kept_cand = [j for j in f["keep"] if 3 <= f["pos_in"][j] < 37]
            assert f["scores"][removed].min() >= f["scores"][kept_cand].max()
        elif sel_g == orc.RANDOM:
            r = orc.random_scores(123, 1, 0, g["pos_in"])
            removed = np.setdiff1d(np.arange(g["n_in"]), g["keep"])
            kept_cand = [j for j in g["keep"] if 3 <= j < 37]
            assert r[removed].max() <= r[kept_cand].min()
            f = out["prunes"][2]                                       # draws are keyed by ORIGINAL positions
            r = orc.random_scores(123, 3, 0, f["pos_in"])
            removed = np.setdiff1d(np.arange(f["n_in"]), f["keep"])
            kept_cand = [j for j in f["keep"] if 3 <= f["pos_in"][j] < 37]
            assert r[removed].max() <= r[kept_cand].min()
        else:
            assert np.array_equal(out["x_out"], base["x_out"])         # explicit names of the defaults


# ---------------------------------------------------------------- rollout threshold -> cut-off position
def test_rollout_influence_and_cutoff_closed_forms():
    n = 40
    # one layer of uniform causal attention, alpha = 1: R[i, j] = 1/(i+1) for j <= i, so the influence of token j
    # is (H_n - H_j)/n with H the harmonic numbers: earlier tokens are seen by more rows
    A = np.tril(np.ones((n, n))) / np.arange(1, n + 1)[:, None]
    R = orc.rollout_step(np.eye(n), A, 1.0)
    H = np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, n + 1))])
    infl = orc.rollout_influence(R)
    np.testing.assert_allclose(infl, (H[n] - H[:n]) / n, rtol=1e-13)
    assert abs(infl.sum() - 1.0) < 1e-13 and (np.diff(infl) < 0).all()
    # brute-force column means
    want = [sum(R[i][j] for i in range(n)) / n for j in range(n)]
    np.testing.assert_allclose(infl, want, rtol=1e-13)
    prot = np.zeros(n, dtype=bool); prot[:3] = True; prot[-5:] = True
    for thr in (0.25, 0.5, 1.0, 2.0, 4.0):
        # influences decrease with j: the cut-off is the number of leading positions with H_n - H_j >= thr,
        # clipped to the candidates [3, n-5)
        lead = sum(1 for j in range(n) if H[n] - H[j] >= thr)
        want_c = min(lead, n - 5) if lead > 3 else 0
        assert orc.rollout_cutoff(R, prot, thr) == want_c, thr
    # alpha = 0: R = I, every token has exactly the uniform share
    I = orc.rollout_step(np.eye(n), A, 0.0)
    np.testing.assert_allclose(orc.rollout_influence(I), 1.0 / n, rtol=1e-15)
    assert orc.rollout_cutoff(I, prot, 1.0) == n - 5 and orc.rollout_cutoff(I, prot, 1.0 + 1e-9) == 0
    # a late influential candidate moves the cut-off past it; a protected one does not
    R2 = R.copy(); R2[:, 30] += 1.0
    assert orc.rollout_cutoff(R2, prot, 4.0) == 31
    R3 = R.copy(); R3[:, n - 2] += 1.0
    assert orc.rollout_cutoff(R3, prot, 4.0) == orc.rollout_cutoff(R, prot, 4.0)
    assert orc.rollout_cutoff(R, np.ones(n, dtype=bool), 0.0) == 0        # no candidates at all
