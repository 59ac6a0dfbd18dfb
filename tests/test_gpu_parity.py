"""GPU parity: every stage of the HIP path against the CPU oracle, element by element, through the C ABI.

Integer / index work (selection, compaction) must match bit for bit; floating-point stages stay within the
tolerances in gpu_util (bf16: max-abs 2e-2, relative L2 1e-2 on O(1)-scale outputs).  End-to-end kept sets
may differ only on tokens whose oracle score lies within 1e-3 of the k-th score."""
import os

import numpy as np
import pytest
import torch

import fastav_inputs as fi
from oracle import fastav_oracle as orc
import paper_2601_13143_amd as fa
from gpu_util import (TIE_BAND, assert_close, dev, host, make_decoder, make_decoder_streamed, model_struct, prune_tuples,
                      rel_l2)

pytestmark = pytest.mark.gpu


def _cu(lens):
    return np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)


# ------------------------------------------------------------------------------------ select + gather
def _select_case(lens, score_kind, seed, prot_frac=0.1, ratio=0.6, positional=False, negate=False):
    rng = np.random.default_rng(seed)
    cu = _cu(lens)
    T = int(cu[-1])
    kind = score_kind or "softmax"
    scores = np.concatenate([fi.random_scores(n, seed + i, kind) if n else np.zeros(0, np.float32) for i, n in enumerate(lens)])
    if negate:
        scores = -scores
    prot = (rng.random(T) < prot_frac)
    for b in range(len(lens)):
        if lens[b] > 0:
            prot[cu[b + 1] - 1] = True
    kc, want = [], []
    for b, n in enumerate(lens):
        p = prot[cu[b]:cu[b + 1]]
        k = orc.keep_count(n, ratio, int(p.sum())) if n else 0
        kc.append(k)
        keep = orc.global_keep(p, k) if positional else orc.select_keep(scores[cu[b]:cu[b + 1]], p, k)
        want.append(keep + cu[b])
    want = np.concatenate(want) if want else np.zeros(0, np.int64)
    x = rng.standard_normal((T, 24)).astype(np.float32)           # 96-byte rows (16-byte path)
    ids = np.arange(T, dtype=np.int32)                            # 4-byte rows
    by = rng.integers(0, 255, (T, 3)).astype(np.uint8)            # 3-byte rows (bytewise path)
    s_dev = None if positional else torch.from_numpy(scores).cuda()
    keep_idx, cu_out, (gx, gi, gb) = fa.fastav_select_gather(
        s_dev, torch.from_numpy(prot.astype(np.uint8)).cuda(), cu, kc,
        [torch.from_numpy(x).cuda(), torch.from_numpy(ids).cuda(), torch.from_numpy(by).cuda()])
    torch.cuda.synchronize()
    got = keep_idx.cpu().numpy()
    assert np.array_equal(got, want), f"kept indices differ: {np.sum(got != want)} of {len(want)}"
    assert np.array_equal(cu_out.cpu().numpy(), _cu(kc))
    assert np.array_equal(gx.cpu().numpy(), x[want]) and np.array_equal(gi.cpu().numpy(), ids[want])
    assert np.array_equal(gb.cpu().numpy(), by[want])


@pytest.mark.parametrize("kind", ["softmax", "ties", "equal", "mixed"])
def test_select_gather_single_samples(kind):
    for n in (1, 2, 63, 64, 65, 1000, 1025, 4096, 5000):
        _select_case([n], kind, 11 + n)


def test_select_gather_ragged_batch_and_edges():
    _select_case([2048, 6144, 3000, 1, 77, 4095, 2049, 5120], "softmax", 5)
    _select_case([300, 1, 1, 900], "ties", 6, prot_frac=0.5, ratio=0.3)
    _select_case([500, 700], "softmax", 7, ratio=1.0)              # keep everything
    _select_case([500, 700], "softmax", 8, prot_frac=0.0, ratio=0.001)   # keep only the forced last row
    _select_case([500, 700], "equal", 9, prot_frac=1.0, ratio=0.5)  # everything protected
    _select_case([128, 0, 64], "softmax", 10)                      # an empty sample in the batch


def test_select_gather_long_samples():
    _select_case([16384], "softmax", 21, ratio=0.7)
    _select_case([32768, 33000], "ties", 22, ratio=0.5)            # second sample exceeds the LDS-resident limit
    _select_case([70001], "softmax", 23, ratio=0.35)


def test_select_variant_strategies_of_the_ablation_tables():
    """Tables 2-3 compare selectors: keeping the LEAST attended tokens is the same selection on negated
    scores (signed zeros and ties included), a random selector the same selection on random scores."""
    _select_case([4096, 777], "softmax", 41, ratio=0.5, negate=True)
    _select_case([300, 1, 900], "ties", 42, prot_frac=0.3, ratio=0.4, negate=True)
    _select_case([2000], "equal", 43, ratio=0.5, negate=True)


def test_select_positional_is_the_global_rule():
    _select_case([4096, 1000, 37], None, 31, prot_frac=0.05, ratio=0.6, positional=True)
    _select_case([16384], None, 32, prot_frac=0.05, ratio=0.5, positional=True)


# ------------------------------------------------------------------------------------ Eq. 4 scores
@pytest.mark.parametrize("dtype,Hq,Hkv,dh", [("bf16", 32, 8, 128), ("bf16", 28, 4, 128), ("bf16", 6, 3, 64), ("bf16", 8, 8, 128),
                                            ("f32", 4, 2, 64), ("f32", 8, 2, 128), ("bf16", 16, 2, 64)])
@pytest.mark.parametrize("n_last", [1, 3])
def test_score_matches_oracle(dtype, Hq, Hkv, dh, n_last):
    lens = [300, 129, 2, 1, 517]
    rng = np.random.default_rng(Hq * 100 + dh + n_last)
    T = sum(lens)
    q = rng.standard_normal((T, Hq, dh)).astype(np.float32) * 1.3
    k = rng.standard_normal((T, Hkv, dh)).astype(np.float32) * 1.3
    if dtype == "bf16":
        fi.round_bf16(q); fi.round_bf16(k)
    m = fa.make_model(1, 64, Hq, Hkv, dh, 64, dtype=fa.BF16 if dtype == "bf16" else fa.F32)
    cu = _cu(lens)
    got = host(fa.fastav_score(m, dev(q, dtype), dev(k, dtype), torch.from_numpy(cu).cuda(), max(lens), n_last))
    for b, n in enumerate(lens):
        want = orc.last_query_scores(q[cu[b]:cu[b + 1]].astype(np.float64), k[cu[b]:cu[b + 1]].astype(np.float64), n_last)
        g = got[cu[b]:cu[b + 1]]
        assert abs(g.sum() - 1.0) < 1e-4
        # scores are O(1/n): compare after scaling by n; inputs are identical so fp32 accumulation is the only error
        assert np.max(np.abs(g - want)) * n <= 1e-3 and rel_l2(g, want) <= 1e-4, (b, np.max(np.abs(g - want)) * n, rel_l2(g, want))


def test_score_strided_views_of_a_fused_qkv_buffer():
    Hq, Hkv, dh, n = 8, 2, 128, 700
    rng = np.random.default_rng(3)
    qkv = fi.round_bf16(rng.standard_normal((n, (Hq + 2 * Hkv) * dh)).astype(np.float32))
    t = dev(qkv, "bf16")
    m = fa.make_model(1, 64, Hq, Hkv, dh, 64)
    got = host(fa.fastav_score(m, t, t[:, Hq * dh:], torch.tensor([0, n], dtype=torch.int32).cuda(), n, 1,
                               q_row_stride=t.stride(0), k_row_stride=t.stride(0)))
    q = qkv[:, :Hq * dh].reshape(n, Hq, dh).astype(np.float64)
    k = qkv[:, Hq * dh:(Hq + Hkv) * dh].reshape(n, Hkv, dh).astype(np.float64)
    want = orc.last_query_scores(q, k, 1)
    assert np.max(np.abs(got - want)) * n <= 1e-3


# ------------------------------------------------------------------------------------ row-wise ops
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("rows,d", [(1, 256), (77, 4096), (33, 3584), (5, 250)])
def test_rmsnorm(dtype, rows, d):
    rng = np.random.default_rng(rows + d)
    x = (rng.standard_normal((rows, d)) * 3 + 0.5).astype(np.float32)
    g = (1 + 0.02 * rng.standard_normal(d)).astype(np.float32)
    if dtype == "bf16":
        fi.round_bf16(g)
    got = host(fa.fastav_rmsnorm(torch.from_numpy(x).cuda(), dev(g, dtype), 1e-6))
    assert_close(got, orc.rmsnorm(x.astype(np.float64), g.astype(np.float64), 1e-6), dtype, what="rmsnorm")


@pytest.mark.parametrize("dtype,dh,base", [("bf16", 128, 1e4), ("bf16", 128, 1e6), ("f32", 64, 1e4), ("bf16", 64, 1e4)])
def test_rope_with_original_positions(dtype, dh, base):
    rng = np.random.default_rng(dh)
    n, H, extra = 50, 5, 2 * dh                                     # rows wider than the rotated heads (V part untouched)
    x = rng.standard_normal((n, H * dh + extra)).astype(np.float32)
    if dtype == "bf16":
        fi.round_bf16(x)
    pos = np.sort(rng.choice(16384, n, replace=False)).astype(np.int32)
    pos[0] = 0; pos[-1] = 16383
    t = dev(x, dtype)
    fa.fastav_rope(t, torch.from_numpy(pos).cuda(), H, dh, base)
    got = host(t)
    want = orc.rope(x[:, :H * dh].reshape(n, H, dh).astype(np.float64), pos, base).reshape(n, H * dh)
    assert_close(got[:, :H * dh], want, dtype, what="rope")
    assert np.array_equal(got[:, H * dh:], x[:, H * dh:].astype(np.float64))


# ------------------------------------------------------------------------------------ linear layers
LINEAR_SHAPES = [("f32", 100, 688, 256), ("f32", 37, 256, 688), ("bf16", 100, 200, 72),
                 ("bf16", 300, 1024, 512), ("bf16", 1205, 512, 1024), ("bf16", 257, 6144, 4096), ("bf16", 129, 3584, 1024),
                 ("bf16", 2100, 6144, 256), ("bf16", 4000, 2048, 192),
                 ("bf16", 1205, 4096, 2048),      # < 1 round of big tiles: split-K for the residual epilogue
                 ("bf16", 2458, 2048, 1536),      # 80 big tiles -> split 3
                 ("bf16", 3000, 8192, 256),       # 384 big tiles = 1.5 rounds
                 ("bf16", 2458, 4608, 192),       # SwiGLU: 360 big tiles = 1.4 rounds
                 ("bf16", 1721, 2816, 320),       # 77 tiles; SwiGLU has 154
                 ("bf16", 8200, 4096, 256),       # 33 x 16 = 528 big tiles: several rounds (hardware-add residual epilogue)
                 ("bf16", 2458, 4096, 512),       # residual epilogue: 208 tiles of 192 rows instead of 160 of 256
                 ("bf16", 300, 512, 128),         # two 64-k stages: the shortest pipeline
                 ("bf16", 1, 1024, 320),          # one row; five stages (the unrolled loop's remainder path only)
                 ("bf16", 257, 256, 448),         # one row past a tile; seven stages (unrolled loop + remainder)
                 ("bf16", 5000, 14336, 128)]      # 20 x 56 = 1120 big tiles of two stages each: rounds + tail columns


@pytest.mark.parametrize("dtype,M,N,K", LINEAR_SHAPES)
@pytest.mark.parametrize("epi", [fa.EPI_STORE, fa.EPI_RESADD, fa.EPI_SWIGLU])
def test_linear(dtype, M, N, K, epi):
    rng = np.random.default_rng(M + N + K + epi)
    a = rng.standard_normal((M, K)).astype(np.float32)
    w = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32)
    w2 = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32)
    if dtype == "bf16":
        fi.round_bf16(a); fi.round_bf16(w); fi.round_bf16(w2)
    a64, w64, w264 = a.astype(np.float64), w.astype(np.float64), w2.astype(np.float64)
    if epi == fa.EPI_STORE:
        got = host(fa.fastav_linear(dev(a, dtype), dev(w, dtype)))
        want = a64 @ w64.T
    elif epi == fa.EPI_RESADD:
        r = rng.standard_normal((M, N)).astype(np.float32)
        c = torch.from_numpy(r.copy()).cuda()
        fa.fastav_linear(dev(a, dtype), dev(w, dtype), fa.EPI_RESADD, c=c)
        got, want = host(c), r.astype(np.float64) + a64 @ w64.T
    else:
        got = host(fa.fastav_linear(dev(a, dtype), dev(w, dtype), fa.EPI_SWIGLU, w2=dev(w2, dtype)))
        want = orc.silu(a64 @ w64.T) * (a64 @ w264.T)
    assert_close(got, want, dtype, what=f"linear epi={epi}")


def test_linear_seeded_random_shapes():
    """Thirty seeded shapes around the tile, stage and row-block boundaries, every epilogue in turn."""
    rng = np.random.default_rng(20260113)
    for case in range(30):
        M = int(rng.choice([1, 15, 16, 17, 127, 128, 129, 191, 192, 193, 255, 256, 257, 300, 511, 600]))
        N = 128 * int(rng.choice([1, 2, 3, 5, 8]))
        K = 64 * int(rng.choice([2, 3, 5, 6, 7, 8]))
        epi = [fa.EPI_STORE, fa.EPI_RESADD, fa.EPI_SWIGLU][case % 3]
        a = rng.standard_normal((M, K)).astype(np.float32)
        w = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32)
        w2 = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32)
        fi.round_bf16(a); fi.round_bf16(w); fi.round_bf16(w2)
        a64, w64, w264 = a.astype(np.float64), w.astype(np.float64), w2.astype(np.float64)
        if epi == fa.EPI_STORE:
            got, want = host(fa.fastav_linear(dev(a, "bf16"), dev(w, "bf16"))), a64 @ w64.T
        elif epi == fa.EPI_RESADD:
            r = rng.standard_normal((M, N)).astype(np.float32)
            c = torch.from_numpy(r.copy()).cuda()
            fa.fastav_linear(dev(a, "bf16"), dev(w, "bf16"), fa.EPI_RESADD, c=c)
            got, want = host(c), r.astype(np.float64) + a64 @ w64.T
        else:
            got = host(fa.fastav_linear(dev(a, "bf16"), dev(w, "bf16"), fa.EPI_SWIGLU, w2=dev(w2, "bf16")))
            want = orc.silu(a64 @ w64.T) * (a64 @ w264.T)
        assert_close(got, want, "bf16", what=f"linear case {case}: M={M} N={N} K={K} epi={epi}")


@pytest.mark.parametrize("epi", [fa.EPI_STORE, fa.EPI_RESADD, fa.EPI_SWIGLU])
def test_linear_output_not_16_byte_aligned(epi):
    """An output that starts one element past a 16-byte boundary takes the element-wise store path."""
    M, N, K = 300, 1024, 512
    rng = np.random.default_rng(7 + epi)
    a = rng.standard_normal((M, K)).astype(np.float32)
    w = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32)
    w2 = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32)
    fi.round_bf16(a); fi.round_bf16(w); fi.round_bf16(w2)
    a64, w64, w264 = a.astype(np.float64), w.astype(np.float64), w2.astype(np.float64)
    if epi == fa.EPI_RESADD:
        r = rng.standard_normal((M, N)).astype(np.float32)
        buf = torch.zeros(M * N + 8, dtype=torch.float32, device="cuda")
        c = buf[1:1 + M * N].view(M, N)
        c.copy_(torch.from_numpy(r))
        want = r.astype(np.float64) + a64 @ w64.T
    else:
        buf = torch.zeros(M * N + 8, dtype=torch.bfloat16, device="cuda")
        c = buf[1:1 + M * N].view(M, N)
        want = a64 @ w64.T if epi == fa.EPI_STORE else orc.silu(a64 @ w64.T) * (a64 @ w264.T)
    assert c.data_ptr() % 16 != 0
    fa.fastav_linear(dev(a, "bf16"), dev(w, "bf16"), epi, w2=dev(w2, "bf16") if epi == fa.EPI_SWIGLU else None, c=c)
    assert_close(host(c), want, "bf16", what=f"linear (unaligned output) epi={epi}")
    assert float(buf[0]) == 0.0 and float(buf[1 + M * N:].abs().max()) == 0.0


# ------------------------------------------------------------------------------------ attention (+ side output)
@pytest.mark.parametrize("dtype,Hq,Hkv,dh,lens", [("f32", 4, 2, 64, [130, 1, 77]), ("bf16", 8, 2, 128, [300, 129, 64]),
                                                 ("bf16", 4, 4, 64, [200, 65]), ("bf16", 32, 8, 128, [700]),
                                                 ("bf16", 28, 4, 128, [257, 500]),
                                                 ("bf16", 8, 2, 128, [1, 2, 33, 63, 128, 256, 191]),   # shorter than a tile, exact tile multiples
                                                 ("bf16", 4, 2, 64, [1, 31, 64, 127, 385])])
def test_attention_and_last_row_side_output(dtype, Hq, Hkv, dh, lens):
    rng = np.random.default_rng(Hq + dh + len(lens))
    T = sum(lens)
    qkv = rng.standard_normal((T, (Hq + 2 * Hkv) * dh)).astype(np.float32)
    qkv[:, :(Hq + Hkv) * dh] *= 1.3
    if dtype == "bf16":
        fi.round_bf16(qkv)
    t = dev(qkv, dtype)
    q = t.as_strided((T, Hq, dh), (t.stride(0), dh, 1))
    k = t.as_strided((T, Hkv, dh), (t.stride(0), dh, 1), Hq * dh)
    v = t.as_strided((T, Hkv, dh), (t.stride(0), dh, 1), (Hq + Hkv) * dh)
    m = fa.make_model(1, 64, Hq, Hkv, dh, 64, dtype=fa.BF16 if dtype == "bf16" else fa.F32)
    cu = _cu(lens)
    cu_dev = torch.from_numpy(cu).cuda()
    o, ll, ml = fa.fastav_attention(m, q, k, v, cu_dev, max(lens), want_last=True)
    o2 = fa.fastav_attention(m, q, k, v, cu_dev, max(lens))
    assert torch.equal(o, o2)                                     # the side output does not change the result
    got, ll, ml = host(o), host(ll), host(ml)
    q64 = qkv[:, :Hq * dh].reshape(T, Hq, dh).astype(np.float64)
    k64 = qkv[:, Hq * dh:(Hq + Hkv) * dh].reshape(T, Hkv, dh).astype(np.float64)
    v64 = qkv[:, (Hq + Hkv) * dh:].reshape(T, Hkv, dh).astype(np.float64)
    G = Hq // Hkv
    for b, n in enumerate(lens):
        sl = slice(cu[b], cu[b + 1])
        want = orc.causal_gqa_attention(q64[sl], k64[sl], v64[sl])
        assert_close(got[sl], want, dtype, what=f"attention sample {b}")
        # side output: scaled logits of the last row and its (max, sum exp)
        for h in range(Hq):
            z = (k64[sl, h // G] @ q64[cu[b + 1] - 1, h]) / np.sqrt(dh)
            assert np.max(np.abs(ll[h, sl] - z)) <= 1e-3 * max(1.0, np.abs(z).max())
            assert abs(ml[b, h, 0] - z.max()) <= 1e-3 * max(1.0, abs(z.max()))
            assert abs(ml[b, h, 1] - np.exp(z - ml[b, h, 0]).sum()) <= 2e-3 * np.exp(z - z.max()).sum()


def _attention_case(qkv, Hq, Hkv, dh, lens, rows_per_sample=None, what=""):
    """Runs fastav_attention with the side output on a fused [T, (Hq+2Hkv)dh] bf16-representable buffer and compares
    O (all rows, or the given rows of each sample), the last row's logits, (max, sum) and the Eq. 4 scores they
    imply against the oracle."""
    T = sum(lens)
    t = dev(qkv, "bf16")
    q = t.as_strided((T, Hq, dh), (t.stride(0), dh, 1))
    k = t.as_strided((T, Hkv, dh), (t.stride(0), dh, 1), Hq * dh)
    v = t.as_strided((T, Hkv, dh), (t.stride(0), dh, 1), (Hq + Hkv) * dh)
    m = fa.make_model(1, 64, Hq, Hkv, dh, 64, dtype=fa.BF16)
    cu = _cu(lens)
    o, ll, ml = fa.fastav_attention(m, q, k, v, torch.from_numpy(cu).cuda(), max(lens), want_last=True)
    torch.cuda.synchronize()
    got, ll, ml = host(o), host(ll), host(ml)
    assert np.isfinite(got).all() and np.isfinite(ml).all()
    q3 = qkv[:, :Hq * dh].reshape(T, Hq, dh)
    k3 = qkv[:, Hq * dh:(Hq + Hkv) * dh].reshape(T, Hkv, dh)
    v3 = qkv[:, (Hq + Hkv) * dh:].reshape(T, Hkv, dh)
    G = Hq // Hkv
    for b, n in enumerate(lens):
        sl = slice(cu[b], cu[b + 1])
        if rows_per_sample is None:
            want = orc.causal_gqa_attention(q3[sl].astype(np.float64), k3[sl].astype(np.float64), v3[sl].astype(np.float64))
            assert_close(got[sl], want, "bf16", what=f"{what} attention sample {b}")
        else:
            rows = [r for r in rows_per_sample[b] if 0 <= r < n]
            want = orc.causal_gqa_attention_rows(q3[sl], k3[sl], v3[sl], rows)
            assert_close(got[sl][rows], want, "bf16", what=f"{what} attention sample {b} rows {rows[:4]}..")
        s_side = np.zeros(n)
        for h in range(Hq):
            z = (k3[sl, h // G].astype(np.float64) @ q3[cu[b + 1] - 1, h].astype(np.float64)) / np.sqrt(dh)
            assert np.max(np.abs(ll[h, sl] - z)) <= 1e-3 * max(1.0, np.abs(z).max()), (what, b, h)
            assert abs(ml[b, h, 0] - z.max()) <= 1e-3 * max(1.0, abs(z.max())), (what, b, h)
            assert abs(ml[b, h, 1] - np.exp(z - ml[b, h, 0]).sum()) <= 4e-3 * np.exp(z - z.max()).sum(), (what, b, h)
            s_side += np.exp(ll[h, sl] - ml[b, h, 0]) / ml[b, h, 1] / Hq      # what the finalize kernel forms
        want_s = orc.last_query_scores(q3[sl], k3[sl], 1)
        assert np.max(np.abs(s_side - want_s)) <= 2e-2 * max(1.0 / n, want_s.max()), (what, b)


def _ramped_qkv(T, Hq, Hkv, dh, seed, log2_per_key, lens, row_mix=False):
    """q = noise + a e, k_j = noise + b_j e along one unit direction e, so that every query's logits climb with the key
    index by `log2_per_key` (in units of log2, per key, inside each sample): the running row max then keeps rising
    across key tiles.  row_mix: every other query row has a ~ 0 and sees flat logits instead."""
    rng = np.random.default_rng(seed)
    qkv = rng.standard_normal((T, (Hq + 2 * Hkv) * dh)).astype(np.float32)
    a = 8.0
    slope = log2_per_key * np.log(2.0) * np.sqrt(dh) / a             # b_(j+1) - b_j
    cu = _cu(lens)
    j_in = np.concatenate([np.arange(n) for n in lens]).astype(np.float64)
    for h in range(Hq):
        amp = np.full(T, a)
        if row_mix:
            amp[1::2] = 0.0
        qkv[:, h * dh] += amp.astype(np.float32)                    # e = first coordinate of every head
    for g in range(Hkv):
        qkv[:, (Hq + g) * dh] += (slope * j_in).astype(np.float32)
    return fi.round_bf16(qkv)


@pytest.mark.parametrize("dh,Hq,Hkv", [(128, 8, 2), (64, 4, 4)])
@pytest.mark.parametrize("log2_per_tile", [5.0, 7.5, 9.0, 20.0])
def test_attention_running_max_climbs_across_key_tiles(dh, Hq, Hkv, log2_per_tile):
    """Rows whose maximum rises by less than, just under, just over and far over 8 log2 units per 64-key tile: the
    accumulator is then rescaled on some tiles and left on a stale reference on others, and the probabilities of a
    tile reach up to 2^8 before they are rounded.  O, the last row's logits and its (max, sum) against the oracle."""
    lens = [700, 333, 64, 129]
    qkv = _ramped_qkv(sum(lens), Hq, Hkv, dh, int(dh + log2_per_tile * 10), log2_per_tile / 64.0, lens)
    _attention_case(qkv, Hq, Hkv, dh, lens, what=f"ramp {log2_per_tile}/tile")
    qkv = _ramped_qkv(sum(lens), Hq, Hkv, dh, int(dh + log2_per_tile * 10) + 1, log2_per_tile / 64.0, lens, row_mix=True)
    _attention_case(qkv, Hq, Hkv, dh, lens, what=f"ramp {log2_per_tile}/tile, every other row flat")


@pytest.mark.parametrize("dh,Hq,Hkv", [(128, 8, 2), (64, 4, 2)])
def test_attention_one_dominant_late_key(dh, Hq, Hkv):
    """One key far down the sequence outweighs everything before it (the closed form the oracle is pinned with):
    rows at and after it return that key's value, the last row's scores are one-hot on it, and the rows before it
    are ordinary.  The maximum jumps by hundreds of log2 units in the middle of a tile."""
    lens = [600, 257]
    T = sum(lens)
    rng = np.random.default_rng(dh)
    qkv = rng.standard_normal((T, (Hq + 2 * Hkv) * dh)).astype(np.float32)
    cu = _cu(lens)
    hot = [417, 130]
    for h in range(Hq):
        qkv[:, h * dh:(h + 1) * dh] = np.abs(qkv[:, h * dh:(h + 1) * dh]) + 0.25
    for b, j in enumerate(hot):
        qkv[cu[b] + j, Hq * dh:(Hq + Hkv) * dh] = 6.0
    qkv = fi.round_bf16(qkv)
    _attention_case(qkv, Hq, Hkv, dh, lens, what="dominant key")
    # and the closed form itself, on the GPU result
    t = dev(qkv, "bf16")
    q = t.as_strided((T, Hq, dh), (t.stride(0), dh, 1))
    k = t.as_strided((T, Hkv, dh), (t.stride(0), dh, 1), Hq * dh)
    v = t.as_strided((T, Hkv, dh), (t.stride(0), dh, 1), (Hq + Hkv) * dh)
    o, ll, ml = fa.fastav_attention(fa.make_model(1, 64, Hq, Hkv, dh, 64), q, k, v, torch.from_numpy(cu).cuda(), max(lens), want_last=True)
    o = host(o)
    v3 = qkv[:, (Hq + Hkv) * dh:].reshape(T, Hkv, dh)
    for b, j in enumerate(hot):
        for h in range(Hq):
            want = v3[cu[b] + j, h // (Hq // Hkv)]
            assert np.max(np.abs(o[cu[b] + j:cu[b + 1], h] - want)) <= 2e-2 * max(1.0, np.abs(want).max())


@pytest.mark.parametrize("n,Hq,Hkv,dh", [(4096, 32, 8, 128), (16384, 28, 4, 128)])
def test_attention_and_score_at_benchmark_lengths_on_sampled_rows(n, Hq, Hkv, dh):
    """The sequence lengths the benchmark runs (64 and 256 key tiles, query-tile pairs far apart): attention output on
    a sample of rows the oracle evaluates one by one (tile edges, the paired tiles' first and last rows, random
    rows), the last row's side output, and the standalone Eq. 4 kernel over the whole sequence."""
    rng = np.random.default_rng(n + Hq)
    qkv = rng.standard_normal((n, (Hq + 2 * Hkv) * dh)).astype(np.float32)
    qkv[:, :(Hq + Hkv) * dh] *= 1.3
    qkv = fi.round_bf16(qkv)
    rows = sorted(set([0, 1, 31, 32, 63, 64, 127, 128, 129, 191, 255, 256, n // 2 - 1, n // 2, n // 2 + 64, n - 129, n - 128,
                       n - 65, n - 64, n - 2, n - 1] + rng.integers(0, n, 12).tolist()))
    _attention_case(qkv, Hq, Hkv, dh, [n], rows_per_sample=[rows], what=f"n={n}")
    t = dev(qkv, "bf16")
    m = fa.make_model(1, 64, Hq, Hkv, dh, 64)
    for n_last in (1, 2):
        got = host(fa.fastav_score(m, t, t[:, Hq * dh:], torch.tensor([0, n], dtype=torch.int32).cuda(), n, n_last,
                                   q_row_stride=t.stride(0), k_row_stride=t.stride(0)))
        want = orc.last_query_scores(qkv[:, :Hq * dh].reshape(n, Hq, dh), qkv[:, Hq * dh:(Hq + Hkv) * dh].reshape(n, Hkv, dh), n_last)
        assert abs(got.sum() - 1.0) < 1e-4
        assert np.max(np.abs(got - want)) * n <= 1e-3 * max(1.0, want.max() * n) and rel_l2(got, want) <= 1e-4, \
            (n_last, np.max(np.abs(got - want)) * n, rel_l2(got, want))


# ------------------------------------------------------------------------------------ prefill end to end
def _oracle_and_gpu(w: fi.Workload, weights, x, want_kv=True):
    dec = make_decoder(w.model, weights)
    spans, offs = fi.span_table(w)
    out = dec.fastav_prefill(dev(x, w.model.dtype), fi.cu_seqlens(w), spans, offs, prune_tuples(w), w.n_last,
                             want_kv=want_kv, want_trace=True, want_layers=True)
    torch.cuda.synchronize()
    ref = orc.prefill(w, weights, x)
    return out, ref


def _check_prefill(w: fi.Workload, out, ref, x_scale_from_ref=True):
    """Kept sets (tie band), surviving positions, hidden states on the common survivors, K/V."""
    dtype = w.model.dtype
    cu0 = fi.cu_seqlens(w)
    B = len(w.samples)
    got_pos = out["kept_pos"].cpu().numpy()
    got_cu = out["cu_seqlens_out"].cpu().numpy()
    assert got_cu[-1] == len(got_pos) == out["x_out"].shape[0]
    x_out = host(out["x_out"])
    stats = {"flipped": 0, "flips_per_prune": [], "jaccard": [], "outside_strict_band": []}
    # per prune: compare kept sets in terms of ORIGINAL positions
    for b in range(B):
        r = ref[b]
        prot0 = orc.protected_mask(w.samples[b], w.n_last)
        inherited = set()                      # positions that already differed at an earlier prune
        for i, pr in enumerate(r["prunes"]):
            want_pos = set(pr["pos_in"][pr["keep"]].tolist())
            # GPU kept rows of prune i, mapped to original positions through the previous prunes
            idx = out["prune_keep_idx"][i].cpu().numpy()
            cu_in = _cu([rr["prunes"][i]["n_in"] for rr in ref])
            mine = idx[(idx >= cu_in[b]) & (idx < cu_in[b + 1])] - cu_in[b]
            pos_in = np.arange(cu0[b + 1] - cu0[b])
            for j in range(i):
                idx_j = out["prune_keep_idx"][j].cpu().numpy()
                cu_j = _cu([rr["prunes"][j]["n_in"] for rr in ref])
                sel = idx_j[(idx_j >= cu_j[b]) & (idx_j < cu_j[b + 1])] - cu_j[b]
                pos_in = pos_in[sel]
            got_set = set(pos_in[mine].tolist())
            assert len(got_set) == pr["k"] and (np.diff(mine) > 0).all()
            assert set(np.nonzero(prot0)[0].tolist()) <= got_set, "a protected token was pruned"
            diff = (got_set ^ want_pos) - inherited
            if diff:
                sel = pr.get("selector", orc.DEFAULT)
                assert pr["kind"] == fi.FINE and sel in (orc.DEFAULT, orc.LOW_ATTENTIVE, orc.TOP_ATTENTIVE), \
                    "positional and random selections are integer work and must match exactly"
                s_ref = pr["scores"]
                cand_kept = [j for j in pr["keep"] if not prot0[pr["pos_in"][j]]]
                edge = max if sel == orc.TOP_ATTENTIVE else min       # the kept candidate next to the cut
                kth = edge(s_ref[j] for j in cand_kept) if cand_kept else 0.0
                pos_to_local = {int(p): j for j, p in enumerate(pr["pos_in"])}
                for p in diff:
                    # a token the oracle no longer holds can only be the partner of an earlier flip
                    assert p in pos_to_local, (b, i, p, "differs, yet was never within a tie band")
                    assert abs(s_ref[pos_to_local[p]] - kth) <= TIE_BAND, (b, i, p, s_ref[pos_to_local[p]], kth)
                # beyond the literal band (loose where scores are ~1/n): bf16 noise may only exchange a small part of
                # the kept set.  Measured on the full-size configurations: 0.3-1.0 % of k exchanged per prune, moving by
                # a few tokens between builds whose bf16 rounding differs (profiles/parity_cfg*.txt); the cap is 1.5 %
                # of k exchanged = 3 % of k in the symmetric difference
                assert len(diff) <= max(4, int(0.03 * pr["k"])), (b, i, len(diff), pr["k"])
            stats["flips_per_prune"].append((b, i, len(diff) // 2, pr["k"]))
            stats["flipped"] += (len(diff) + 1) // 2
            # diagnostics: overlap of the two kept sets, and how many differing tokens lie outside a STRICT band
            # (1 % of the k-th score) around the cut - the literal band is wide where scores are ~1/n
            both = got_set ^ want_pos
            stats["jaccard"].append((b, i, len(got_set & want_pos) / max(1, len(got_set | want_pos))))
            n_strict = 0
            if both and pr["kind"] == fi.FINE and pr.get("scores") is not None:
                cand_kept = [j for j in pr["keep"] if not prot0[pr["pos_in"][j]]]
                if cand_kept:
                    top = pr.get("selector", orc.DEFAULT) == orc.TOP_ATTENTIVE
                    kth = (max if top else min)(pr["scores"][j] for j in cand_kept)
                    p2l = {int(p): j for j, p in enumerate(pr["pos_in"])}
                    n_strict = sum(1 for p in both if p in p2l and abs(pr["scores"][p2l[p]] - kth) > 1e-2 * abs(kth))
            stats["outside_strict_band"].append((b, i, n_strict))
            inherited |= (got_set ^ want_pos)
            if pr["kind"] == fi.FINE and out["prune_scores"][i] is not None and not inherited \
                    and pr.get("selector", orc.DEFAULT) != orc.RANDOM:
                g = host(out["prune_scores"][i])[cu_in[b]:cu_in[b + 1]]
                n = len(g)
                lim = 2e-2 if dtype == "bf16" else 1e-4
                assert np.max(np.abs(g - pr["scores"])) * n <= lim * max(1.0, pr["scores"].max() * n), \
                    (np.max(np.abs(g - pr["scores"])) * n, pr["scores"].max() * n)
        # final hidden state on the common survivors
        mine_pos = got_pos[got_cu[b]:got_cu[b + 1]]
        assert (np.diff(mine_pos) > 0).all()
        common, gi, ri = np.intersect1d(mine_pos, r["kept_pos"], return_indices=True)
        assert len(common) >= len(mine_pos) - stats["flipped"]
        gx, rx = x_out[got_cu[b]:got_cu[b + 1]][gi], r["x_out"][ri]
        have = np.isfinite(rx).all(axis=1)      # a stored oracle result holds a sample of the rows only
        gx, rx = gx[have], rx[have]
        assert len(rx) > 0
        scale = float(np.sqrt(np.mean(rx ** 2)))
        stats[f"x_rel_l2_{b}"] = rel_l2(gx, rx)
        stats[f"x_max_abs_over_rms_{b}"] = float(np.max(np.abs(gx - rx))) / scale
    return stats


def test_prefill_cfg1_tiny_fp32():
    w = fi.config(1)
    weights = [fi.layer_weights(w.model, l, w.weight_seed) for l in range(w.model.n_layers)]
    x = fi.embeddings(w)
    out, ref = _oracle_and_gpu(w, weights, x)
    st = _check_prefill(w, out, ref)
    assert st["flipped"] == 0
    assert st["x_rel_l2_0"] <= 2e-5 and st["x_max_abs_over_rms_0"] <= 2e-4, st
    assert out["x_out"].shape[0] == 128 and out["tokens_in"].tolist() == [512, 512, 256, 256]
    # K/V caches: layer 3's are compacted to the survivors
    for l, (k, v) in enumerate(out["kv"]):
        rk, rv = ref[0]["kv"][l]
        assert_close(host(k), rk, "f32", what=f"K layer {l}")
        assert_close(host(v), rv, "f32", what=f"V layer {l}")
    # per-layer hidden states
    r_trace = orc.prefill(w, weights, x, trace=True)[0]["trace"]
    for l in range(3):
        assert rel_l2(host(out["layer_x"][l]), r_trace[l]["x_out"]) <= 2e-5


def _small_bf16():
    m = fi.Model(3, 512, 8, 2, 128, 1024, 1.0e4, 1e-6, "bf16")
    w = fi.Workload("small_bf16", m, [[(fi.VIDEO, 288), (fi.AUDIO, 150), (fi.TEXT, 30)], [(fi.VIDEO, 144), (fi.AUDIO, 97), (fi.TEXT, 9)]],
                    [fi.Prune(1, fi.GLOBAL, 0.6), fi.Prune(1, fi.FINE, 0.7), fi.Prune(2, fi.FINE, 0.7)], seed=41)
    weights = [fi.layer_weights(m, l, 7) for l in range(m.n_layers)]
    return w, weights, fi.embeddings(w)


def test_prefill_small_bf16_ragged_batch():
    w, weights, x = _small_bf16()
    out, ref = _oracle_and_gpu(w, weights, x)
    st = _check_prefill(w, out, ref)
    for b in range(2):
        assert st[f"x_rel_l2_{b}"] <= 1e-2 and st[f"x_max_abs_over_rms_{b}"] <= 5e-2, st


def test_prefill_kv_cache_written_in_place_or_not_is_the_same_forward():
    """Layers without a fine prune produce K and V directly in the caller's cache; without a cache they stay in
    the workspace.  Both must give the same forward, and the cache of the unpruned first layer the oracle's K, V."""
    w, weights, x = _small_bf16()
    dec = make_decoder(w.model, weights)
    spans, offs = fi.span_table(w)
    xd = dev(x, "bf16")
    with_kv = dec.fastav_prefill(xd, fi.cu_seqlens(w), spans, offs, prune_tuples(w), 1, want_kv=True)
    x_with, pos_with = with_kv["x_out"].clone(), with_kv["kept_pos"].clone()
    k0, v0 = with_kv["kv"][0]
    k0, v0 = host(k0), host(v0)
    without = dec.fastav_prefill(xd, fi.cu_seqlens(w), spans, offs, prune_tuples(w), 1, want_kv=False)
    torch.cuda.synchronize()
    assert torch.equal(x_with, without["x_out"]) and torch.equal(pos_with, without["kept_pos"])
    ref = orc.prefill(w, weights, x)
    rk = np.concatenate([ref[b]["kv"][0][0] for b in range(len(ref))])
    rv = np.concatenate([ref[b]["kv"][0][1] for b in range(len(ref))])
    assert_close(k0.reshape(rk.shape), rk, "bf16", what="K layer 0")
    assert_close(v0.reshape(rv.shape), rv, "bf16", what="V layer 0")


def test_prefill_keep_ratio_one_is_the_unpruned_forward():
    w, weights, x = _small_bf16()
    dec = make_decoder(w.model, weights)
    spans, offs = fi.span_table(w)
    xd = dev(x, "bf16")
    plain = dec.fastav_prefill(xd, fi.cu_seqlens(w), spans, offs, [], 1)
    x_plain = plain["x_out"].clone()
    ones = dec.fastav_prefill(xd, fi.cu_seqlens(w), spans, offs, [(p.layer, p.kind, 1.0) for p in w.prunes], 1)
    torch.cuda.synchronize()
    assert torch.equal(x_plain, ones["x_out"])
    assert np.array_equal(ones["kept_pos"].cpu().numpy(), np.concatenate([np.arange(n) for n in w.seqlens]))
    assert np.array_equal(ones["cu_seqlens_out"].cpu().numpy(), fi.cu_seqlens(w))


def test_prefill_batched_equals_per_sample():
    w, weights, x = _small_bf16()
    dec = make_decoder(w.model, weights)
    spans, offs = fi.span_table(w)
    both = dec.fastav_prefill(dev(x, "bf16"), fi.cu_seqlens(w), spans, offs, prune_tuples(w), 1)
    xb, posb, cub = both["x_out"].clone(), both["kept_pos"].clone(), both["cu_seqlens_out"].cpu().numpy()
    row = 0
    for b, s in enumerate(w.samples):
        n = sum(l for _, l in s)
        wb = fi.Workload("one", w.model, [s], w.prunes)
        sp, of = fi.span_table(wb)
        one = dec.fastav_prefill(dev(x[row:row + n], "bf16"), [0, n], sp, of, prune_tuples(w), 1)
        torch.cuda.synchronize()
        assert torch.equal(one["kept_pos"], posb[cub[b]:cub[b + 1]])
        assert torch.equal(one["x_out"], xb[cub[b]:cub[b + 1]])
        row += n


def test_prefill_fused_score_select_equals_separate_kernels():
    """A FINE prune finishes Eq. 4 inside the selection kernel (one launch less per prune); with the switch off it
    runs the separate finishing kernel.  Scores, kept rows, surviving positions and hidden states must agree bit for
    bit, on a ragged batch with several FINE prunes."""
    m = fi.Model(6, 512, 8, 2, 128, 1024, 1.0e4, 1e-6, "bf16")
    base = fi.Workload("small6", m, [[(fi.VIDEO, 288), (fi.AUDIO, 150), (fi.TEXT, 30)], [(fi.VIDEO, 144), (fi.AUDIO, 97), (fi.TEXT, 9)],
                                     [(fi.VIDEO, 1000), (fi.AUDIO, 301), (fi.TEXT, 5)]], [], seed=51)
    w = fi.paper_schedule(base, global_keep=0.6, fine_drop=0.2)
    weights = [fi.layer_weights(m, l, 13) for l in range(m.n_layers)]
    dec = make_decoder(m, weights)
    spans, offs = fi.span_table(w)
    xd = dev(fi.embeddings(w), "bf16")
    res = []
    try:
        for fused in (1, 0):
            fa.fastav_set_option(fa.OPT_FUSED_SCORE_SELECT, fused)
            o = dec.fastav_prefill(xd, fi.cu_seqlens(w), spans, offs, prune_tuples(w), 1, want_trace=True)
            torch.cuda.synchronize()
            res.append((o["x_out"].clone(), o["kept_pos"].clone(), [t.clone() for t in o["prune_keep_idx"]],
                        [None if t is None else t.clone() for t in o["prune_scores"]]))
    finally:
        fa.fastav_set_option(fa.OPT_FUSED_SCORE_SELECT, 1)
    (xa, pa, ka, sa), (xb, pb, kb, sb) = res
    assert torch.equal(xa, xb) and torch.equal(pa, pb)
    for i, (a, b) in enumerate(zip(ka, kb)):
        assert torch.equal(a, b), i
    n_scored = 0
    for i, (a, b) in enumerate(zip(sa, sb)):
        if a is not None:
            assert torch.equal(a, b), i
            n_scored += int(float(a.sum()) > 0)
    assert n_scored == 3                                            # the three FINE prunes wrote their scores


@pytest.mark.parametrize("dh,Hq,Hkv,hidden", [(128, 8, 2, 512), (64, 8, 4, 512), (128, 32, 8, 1024)])
def test_prefill_rope_in_the_projection_epilogue(dh, Hq, Hkv, hidden):
    """bf16 prefill rotates Q and K inside the epilogue of the Q/K/V projection (one rounding); with the switch off
    the separate RoPE kernel runs on the rounded projection (two roundings).  Both must give the oracle's rotated
    keys at the stage tolerance (the first layer's cache: no pruning before it, original positions), agree with each
    other to bf16 rounding, and leave V alone.  Ragged batch: row tiles with a tail, small and large tile shapes."""
    m = fi.Model(2, hidden, Hq, Hkv, dh, 1024, 1.0e4, 1e-6, "bf16")
    w = fi.Workload("rope", m, [[(fi.VIDEO, 700), (fi.AUDIO, 150), (fi.TEXT, 30)], [(fi.VIDEO, 144), (fi.AUDIO, 97), (fi.TEXT, 9)]],
                    [fi.Prune(1, fi.GLOBAL, 0.6)], seed=61)
    weights = [fi.layer_weights(m, l, 17) for l in range(m.n_layers)]
    x = fi.embeddings(w)
    dec = make_decoder(m, weights)
    spans, offs = fi.span_table(w)
    xd = dev(x, "bf16")
    res = {}
    try:
        for fused in (1, 0):
            fa.fastav_set_option(fa.OPT_FUSED_ROPE, fused)
            for want_kv in (True, False):                          # K/V produced in the caller's cache, or in the workspace
                o = dec.fastav_prefill(xd, fi.cu_seqlens(w), spans, offs, prune_tuples(w), 1, want_kv=want_kv)
                torch.cuda.synchronize()
                res[(fused, want_kv)] = (o["x_out"].clone(), [(k.clone(), v.clone()) for k, v in o["kv"]] if want_kv else None)
    finally:
        fa.fastav_set_option(fa.OPT_FUSED_ROPE, 1)
    ref = orc.prefill(w, weights, x)
    rk = np.concatenate([ref[b]["kv"][0][0] for b in range(len(ref))])
    rv = np.concatenate([ref[b]["kv"][0][1] for b in range(len(ref))])
    for fused in (1, 0):
        k0, v0 = res[(fused, True)][1][0]
        assert_close(host(k0).reshape(rk.shape), rk, "bf16", what=f"K layer 0, fused={fused}")
        assert_close(host(v0).reshape(rv.shape), rv, "bf16", what=f"V layer 0, fused={fused}")
        assert torch.equal(res[(fused, True)][0], res[(fused, False)][0])      # cache or workspace: the same forward
    assert torch.equal(res[(1, True)][1][0][1], res[(0, True)][1][0][1])       # V of layer 0 is untouched by either form
    xa, xb = host(res[(1, True)][0]), host(res[(0, True)][0])
    assert rel_l2(xa, xb) <= 1e-2
    k_f, k_u = host(res[(1, True)][1][0][0]), host(res[(0, True)][1][0][0])
    assert np.max(np.abs(k_f - k_u)) <= 2e-2 * max(1.0, np.abs(k_u).max())


def test_prefill_splitk_sum_left_to_the_next_rmsnorm_is_the_same_forward():
    """The residual projections of short sequences split K over workgroups; the ordered sum of their partial tiles is
    then done by the RMSNorm that follows (or, where something else reads the residual first - a per-layer output, a
    GLOBAL prune, the end of the stack - by the reduction kernel).  Every combination must give the same bits as
    always reducing separately."""
    m = fi.Model(5, 512, 8, 2, 128, 1024, 1.0e4, 1e-6, "bf16")
    w = fi.Workload("splitk", m, [[(fi.VIDEO, 288), (fi.AUDIO, 150), (fi.TEXT, 30)], [(fi.VIDEO, 1000), (fi.AUDIO, 301), (fi.TEXT, 5)]],
                    [fi.Prune(2, fi.GLOBAL, 0.6), fi.Prune(3, fi.FINE, 0.7)], seed=71)
    weights = [fi.layer_weights(m, l, 19) for l in range(m.n_layers)]
    dec = make_decoder(m, weights)
    spans, offs = fi.span_table(w)
    xd = dev(fi.embeddings(w), "bf16")
    res = {}
    try:
        for fused in (1, 0):
            fa.fastav_set_option(fa.OPT_FUSED_SPLITK_NORM, fused)
            for layers in (False, True):
                o = dec.fastav_prefill(xd, fi.cu_seqlens(w), spans, offs, prune_tuples(w), 1, want_kv=True, want_layers=layers)
                torch.cuda.synchronize()
                res[(fused, layers)] = (o["x_out"].clone(), o["kept_pos"].clone(), [k.clone() for k, _ in o["kv"]],
                                        [t.clone() for t in o["layer_x"]] if layers else None)
    finally:
        fa.fastav_set_option(fa.OPT_FUSED_SPLITK_NORM, 1)
    base = res[(0, True)]
    for key, r in res.items():
        assert torch.equal(r[0], base[0]) and torch.equal(r[1], base[1]), key
        assert all(torch.equal(a, b) for a, b in zip(r[2], base[2])), key
        if r[3] is not None:
            assert all(torch.equal(a, b) for a, b in zip(r[3], base[3])), key
    # and the forward is the oracle's
    out, ref = _oracle_and_gpu(w, weights, fi.embeddings(w), want_kv=False)
    st = _check_prefill(w, out, ref)
    for b in range(2):
        assert st[f"x_rel_l2_{b}"] <= 1e-2, st


def test_prefill_n_last_greater_than_one():
    w, weights, x = _small_bf16()
    w.n_last = 3
    out, ref = _oracle_and_gpu(w, weights, x, want_kv=False)
    st = _check_prefill(w, out, ref)
    for b in range(2):
        assert st[f"x_rel_l2_{b}"] <= 1e-2, st


def test_prefill_paper_schedule_fine_prune_at_every_later_layer():
    """The schedule the paper runs (global prune on the input of the middle layer, a 20 % fine prune at that layer
    and at every later one) on a small 8-layer model and a ragged batch: 1 + 4 prune steps' worth of kept sets
    against the oracle."""
    m = fi.Model(8, 512, 8, 2, 128, 1024, 1.0e4, 1e-6, "bf16")
    base = fi.Workload("small8", m, [[(fi.VIDEO, 288), (fi.AUDIO, 150), (fi.TEXT, 30)], [(fi.VIDEO, 144), (fi.AUDIO, 97), (fi.TEXT, 9)]],
                       [], seed=43)
    w = fi.paper_schedule(base, global_keep=0.6, fine_drop=0.2)
    assert [(p.layer, p.kind) for p in w.prunes] == [(4, fi.GLOBAL)] + [(l, fi.FINE) for l in (4, 5, 6, 7)]
    weights = [fi.layer_weights(m, l, 9) for l in range(m.n_layers)]
    out, ref = _oracle_and_gpu(w, weights, fi.embeddings(w), want_kv=False)
    st = _check_prefill(w, out, ref)
    for b in range(2):
        assert st[f"x_rel_l2_{b}"] <= 2e-2 and st[f"x_max_abs_over_rms_{b}"] <= 0.1, st


def test_prefill_frame_interleaved_spans():
    """video-SALMONN2 layout (Section 3.1, implementation details): video and audio tokens interleaved frame by
    frame; the global prune keeps the first frames (earliest candidates), text stays."""
    m = fi.Model(3, 512, 8, 2, 128, 1024, 1.0e4, 1e-6, "bf16")
    frames = []
    for f in range(10):
        frames += [(fi.VIDEO, 36), (fi.AUDIO, 13)]
    s0 = [(fi.TEXT, 7)] + frames + [(fi.TEXT, 21)]
    s1 = frames[:8] + [(fi.TEXT, 5)]
    # keep 4 of 10 frames: 4 * 49 candidates + 28 text of 518 tokens
    w = fi.Workload("interleaved", m, [s0, s1], [fi.Prune(1, fi.GLOBAL, (4 * 49 + 28) / 518), fi.Prune(2, fi.FINE, 0.8)], seed=47)
    weights = [fi.layer_weights(m, l, 11) for l in range(m.n_layers)]
    out, ref = _oracle_and_gpu(w, weights, fi.embeddings(w), want_kv=False)
    st = _check_prefill(w, out, ref)
    g = ref[0]["prunes"][0]
    assert g["k"] == 4 * 49 + 28 and g["keep"].tolist() == list(range(7 + 4 * 49)) + list(range(497, 518))
    for b in range(2):
        assert st[f"x_rel_l2_{b}"] <= 1e-2, st


def test_prefill_cfg2_7b_single_layer():
    w = fi.config(2)
    weights = [fi.layer_weights(w.model, 0, w.weight_seed)]
    x = fi.embeddings(w)
    out, ref = _oracle_and_gpu(w, weights, x)
    st = _check_prefill(w, out, ref)
    assert out["x_out"].shape[0] == 1229
    assert st["x_rel_l2_0"] <= 1e-2 and st["x_max_abs_over_rms_0"] <= 5e-2, st
    rk, rv = ref[0]["kv"][0]
    common, gi, ri = np.intersect1d(out["kept_pos"].cpu().numpy(), ref[0]["kept_pos"], return_indices=True)
    assert_close(host(out["kv"][0][0])[gi], rk[ri], "bf16", scale=float(np.sqrt(np.mean(rk ** 2))), what="K")
    assert_close(host(out["kv"][0][1])[gi], rv[ri], "bf16", scale=float(np.sqrt(np.mean(rv ** 2))), what="V")


# ------------------------------------------------------------------------ full-size configs vs stored oracle
def _stored_oracle(cfg: int, w: fi.Workload):
    """The fp64 oracle's results for a full-size config, written by tests/golden/make_goldens.py (which calls
    the oracle only), in the shape _check_prefill reads: hidden states are NaN outside the stored rows."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", f"cfg{cfg}_oracle.npz")
    if not os.path.exists(path):
        pytest.skip(f"{os.path.basename(path)} has not been generated (python tests/golden/make_goldens.py {cfg})")
    z = np.load(path)
    ref = []
    for b in range(len(w.samples)):
        prunes = []
        for i, p in enumerate(w.prunes):
            pos_in, keep_pos = z[f"s{b}_p{i}_pos_in"], z[f"s{b}_p{i}_keep_pos"]
            keep = np.searchsorted(pos_in, keep_pos)
            assert np.array_equal(pos_in[keep], keep_pos)
            prunes.append({"kind": p.kind, "n_in": len(pos_in), "k": len(keep_pos), "keep": keep, "pos_in": pos_in,
                           "scores": z[f"s{b}_p{i}_scores"] if f"s{b}_p{i}_scores" in z else None})
        kept = z[f"s{b}_kept_pos"]
        x = np.full((len(kept), w.model.hidden), np.nan)
        x[z[f"s{b}_x_rows"]] = z[f"s{b}_x_out"]
        ref.append({"prunes": prunes, "kept_pos": kept, "x_out": x, "x_rms": float(z[f"s{b}_x_rms"])})
    return ref


def _record_parity(cfg, w, st):
    """Writes the measured end-to-end figures of a full-size run to <FASTAV_PARITY_DIR or gpurun_out>/parity_cfgN.txt
    (a plain-text record; the run passes or fails on the asserts, not on this file)."""
    out_dir = os.environ.get("FASTAV_PARITY_DIR", os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out"))
    try:
        os.makedirs(out_dir, exist_ok=True)
        with open(os.path.join(out_dir, f"parity_cfg{cfg}.txt"), "w") as f:
            f.write(f"end-to-end parity of fastav_prefill vs the stored fp64 oracle, workload {w.name}\n")
            f.write("command: python -u -m pytest tests/test_gpu_parity.py -m gpu -k full_size -v\n")
            f.write("sample  x_rel_l2  x_max_abs_over_rms\n")
            for b in range(len(w.samples)):
                f.write(f"{b:6d}  {st[f'x_rel_l2_{b}']:.4e}  {st[f'x_max_abs_over_rms_{b}']:.4e}\n")
            f.write("limits asserted: x_rel_l2 <= 3e-2, x_max_abs_over_rms <= 0.25, tokens exchanged per prune <= max(2, 1.5 % of k), "
                    "every exchanged token within 1e-3 of the k-th score\n")
            f.write("sample  prune  kept_k  tokens_exchanged  share_of_k  jaccard  differing_tokens_outside_1pct_band_of_kth_score\n")
            for (b, i, fl, k), (_, _, jac), (_, _, ns) in zip(st["flips_per_prune"], st["jaccard"], st["outside_strict_band"]):
                f.write(f"{b:6d}  {i:5d}  {k:6d}  {fl:16d}  {fl / max(1, k):.4f}  {jac:.5f}  {ns}\n")
    except OSError:
        pass


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_prefill_full_size_against_stored_oracle(cfg):
    """The benchmark configurations at their full sizes, launched as bench.py launches them: kept sets, surviving
    positions and a sample of final hidden-state rows against the stored fp64 oracle results."""
    w = fi.config(cfg)
    ref = _stored_oracle(cfg, w)
    print(f"cfg{cfg}: generating and uploading {w.model.n_layers} layers", flush=True)
    dec = make_decoder_streamed(w.model, w.weight_seed)
    spans, offs = fi.span_table(w)
    x = dev(fi.embeddings(w), w.model.dtype)
    print(f"cfg{cfg}: prefill of {sum(w.seqlens)} tokens", flush=True)
    out = dec.fastav_prefill(x, fi.cu_seqlens(w), spans, offs, prune_tuples(w), w.n_last, want_kv=False, want_trace=True)
    torch.cuda.synchronize()
    st = _check_prefill(w, out, ref)
    print(f"cfg{cfg}: {st}", flush=True)
    _record_parity(cfg, w, st)
    for b in range(len(w.samples)):
        # 28-32 bf16 layers against fp64: the error of a deep stack, not of one stage
        assert st[f"x_rel_l2_{b}"] <= 3e-2 and st[f"x_max_abs_over_rms_{b}"] <= 0.25, st
    del dec
    torch.cuda.empty_cache()


def test_prefill_and_decode_replay_from_a_hip_graph():
    """Nothing in the path allocates, synchronises or copies through the host, so a caller may capture it in a
    HIP graph.  The graph is replayed several times, with eager work and synchronisations in between, and every
    replay must reproduce the eager result bit for bit."""
    w, weights, x = _small_bf16()
    m = w.model
    dec = make_decoder(m, weights)
    spans, offs = fi.span_table(w)
    xd = dev(x, "bf16")
    cu = fi.cu_seqlens(w)
    prunes = prune_tuples(w)
    out = dec.fastav_prefill(xd, cu, spans, offs, prunes, 1, want_kv=True)       # allocates outputs + workspace
    lens = fa.fastav_schedule_lens(cu, spans, offs, prunes, 1, m.n_layers)
    x_new = dev(fi.round_bf16(np.random.default_rng(2).standard_normal((2, m.hidden)).astype(np.float32)), "bf16")
    pos = torch.from_numpy(np.array(w.seqlens, dtype=np.int32)).cuda()
    st = dec.fastav_decode_step(x_new, pos, out["kv"], lens)["state"]
    torch.cuda.synchronize()
    eager_x, eager_pos = out["x_out"].clone(), out["kept_pos"].clone()
    eager_k = [k.clone() for k, _ in out["kv"]]
    eager_dec = st["x_out"].clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=torch.cuda.Stream()):
        dec.fastav_prefill(xd, cu, spans, offs, prunes, 1, outputs=out)
        dec.fastav_decode_step(x_new, pos, out["kv"], lens, state=st)
    for rep in range(3):
        out["x_out"].zero_(); out["kept_pos"].zero_(); st["x_out"].zero_()
        for k, v in out["kv"]:
            k.zero_(); v.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out["x_out"], eager_x) and torch.equal(out["kept_pos"], eager_pos), rep
        assert all(torch.equal(k, ek) for (k, _), ek in zip(out["kv"], eager_k)), rep
        assert torch.equal(st["x_out"], eager_dec), rep
        # eager work of the same kind between the replays
        other = dec.fastav_prefill(xd, cu, spans, offs, [], 1)
        torch.cuda.synchronize()
        assert other["x_out"].shape[0] == sum(w.seqlens)


def test_achievable_peak_probes_run_and_report_their_work():
    """The measurement aids of the benchmark: both enqueue one kernel, report the work of the launch and leave the sink
    untouched; operands drawn like activations must not raise the matrix-only rate above the constant-operand one by
    more than measurement noise (they toggle more bits, the chip holds a lower clock)."""
    sink = torch.zeros(1 << 20, dtype=torch.float32, device="cuda")
    ops = torch.randn(32768, device="cuda").bfloat16()

    def rate(operands):
        fa.fastav_probe_mfma(200, sink, operands)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fl = sum(fa.fastav_probe_mfma(2000, sink, operands) for _ in range(4))
        e1.record()
        torch.cuda.synchronize()
        return fl, fl / (e0.elapsed_time(e1) * 1e-3) / 1e12

    fl_c, r_c = rate(None)
    fl_n, r_n = rate(ops)
    assert fl_c == fl_n == 4 * 2048 * 4 * 2000 * 32 * (2 * 16 * 16 * 32)
    assert 500.0 < r_n <= r_c * 1.05 and r_c < 2600.0, (r_c, r_n)      # TFLOP/s: below the datasheet peak, well above a stall
    src = torch.zeros(1 << 24, dtype=torch.float32, device="cuda")
    assert fa.fastav_probe_read(src, sink) == src.numel() * 4
    torch.cuda.synchronize()
    assert float(sink.abs().max()) == 0.0
    with pytest.raises(ValueError):
        fa.fastav_probe_mfma(10, sink, torch.zeros(16, device="cuda").bfloat16())


@pytest.mark.parametrize("case", ["short", "long"])
def test_prefill_o_projection_reads_surviving_rows_through_the_keep_list(case):
    """After a FINE prune the O projection can fetch the surviving rows of the attention output through the keep list
    in its operand copies instead of having them compacted first.  Same values into the same arithmetic: every output
    must have the same bits either way (short samples take the split-K form of the projection, the long one whole
    tiles), and the forward is the oracle's."""
    if case == "short":
        m = fi.Model(4, 512, 8, 2, 128, 1024, 1.0e4, 1e-6, "bf16")
        samples = [[(fi.VIDEO, 288), (fi.AUDIO, 150), (fi.TEXT, 30)], [(fi.VIDEO, 1000), (fi.AUDIO, 301), (fi.TEXT, 5)]]
        prunes = [fi.Prune(1, fi.GLOBAL, 0.6), fi.Prune(1, fi.FINE, 0.7), fi.Prune(2, fi.FINE, 0.8)]
    else:
        m = fi.Model(3, 1024, 8, 2, 128, 2048, 1.0e4, 1e-6, "bf16")
        samples = [[(fi.VIDEO, 2600), (fi.AUDIO, 700), (fi.TEXT, 23)]]
        prunes = [fi.Prune(1, fi.FINE, 0.75), fi.Prune(2, fi.FINE, 0.5)]
    w = fi.Workload("rowlist_" + case, m, samples, prunes, seed=83)
    weights = [fi.layer_weights(m, l, 29) for l in range(m.n_layers)]
    dec = make_decoder(m, weights)
    spans, offs = fi.span_table(w)
    xd = dev(fi.embeddings(w), "bf16")
    res = {}
    try:
        for fused in (1, 0):
            fa.fastav_set_option(fa.OPT_FUSED_GATHER_OPROJ, fused)
            o = dec.fastav_prefill(xd, fi.cu_seqlens(w), spans, offs, prune_tuples(w), 1, want_kv=True, want_layers=True)
            torch.cuda.synchronize()
            res[fused] = (o["x_out"].clone(), o["kept_pos"].clone(), [k.clone() for k, _ in o["kv"]], [v.clone() for _, v in o["kv"]],
                          [t.clone() for t in o["layer_x"]])
    finally:
        fa.fastav_set_option(fa.OPT_FUSED_GATHER_OPROJ, 1)
    a, b = res[1], res[0]
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    for i in (2, 3, 4):
        assert all(torch.equal(x, y) for x, y in zip(a[i], b[i])), i
    out, ref = _oracle_and_gpu(w, weights, fi.embeddings(w), want_kv=False)
    st = _check_prefill(w, out, ref)
    for bb in range(len(samples)):
        assert st[f"x_rel_l2_{bb}"] <= 1e-2, st
