"""GPU parity of one decode step on the per-layer pruned caches (Section 3.1: single-token latency, compacted
caches) against the CPU oracle, through the C ABI.

Stage-wise cases feed both sides the SAME bf16-rounded caches (written by the oracle's pruned prefill), so the
only difference is bf16 arithmetic inside the step; the end-to-end case chains the GPU prefill into the GPU
decode step and compares with the oracle's chain."""
import numpy as np
import pytest
import torch

import fastav_inputs as fi
from oracle import fastav_oracle as orc
import paper_2601_13143_amd as fa
from gpu_util import assert_close, dev, host, make_decoder, prune_tuples, rel_l2

pytestmark = pytest.mark.gpu


def _skinny_case(B, N, K, epi, seed):
    rng = np.random.default_rng(seed)
    a = fi.round_bf16(rng.standard_normal((B, K)).astype(np.float32))
    w = fi.round_bf16((rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32))
    w2 = fi.round_bf16((rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32))
    a64, w64, w264 = a.astype(np.float64), w.astype(np.float64), w2.astype(np.float64)
    if epi == fa.EPI_STORE:
        return host(fa.fastav_linear(dev(a, "bf16"), dev(w, "bf16"))), a64 @ w64.T
    if epi == fa.EPI_RESADD:
        r = rng.standard_normal((B, N)).astype(np.float32)
        c = torch.from_numpy(r.copy()).cuda()
        fa.fastav_linear(dev(a, "bf16"), dev(w, "bf16"), fa.EPI_RESADD, c=c)
        return host(c), r.astype(np.float64) + a64 @ w64.T
    return host(fa.fastav_linear(dev(a, "bf16"), dev(w, "bf16"), fa.EPI_SWIGLU, w2=dev(w2, "bf16"))), \
        orc.silu(a64 @ w64.T) * (a64 @ w264.T)


@pytest.mark.parametrize("epi", [fa.EPI_STORE, fa.EPI_RESADD, fa.EPI_SWIGLU])
@pytest.mark.parametrize("B,N,K", [(1, 256, 128), (3, 4096, 512), (8, 6144, 4096), (16, 1024, 14336), (5, 3584, 3584),
                                   (1, 4096, 3584), (1, 1024, 18944), (1, 272, 512), (1, 4096, 4096), (2, 512, 4096)])
def test_decode_linear_few_rows(B, N, K, epi):
    """Linear layers of a decode step: 1-16 rows against weight matrices of the model's shapes.  A single row with
    K a multiple of 512 takes the one-row kernel (7, 37, 1 and 8 chunks per lane: whole and ragged batches of loads),
    everything else the matrix-core one."""
    got, want = _skinny_case(B, N, K, epi, B + N + K + epi)
    assert_close(got, want, "bf16", what=f"skinny linear {B}x{N}x{K} epi {epi}")


def _caches_from_oracle(w, weights, x):
    """Oracle pruned prefill -> per layer bf16-rounded (K, V) packed over the batch, rows per sample."""
    ref = orc.prefill(w, weights, x)
    L = w.model.n_layers
    lens = np.array([[ref[b]["kv"][l][0].shape[0] for b in range(len(ref))] for l in range(L)], dtype=np.int32)
    kv = []
    for l in range(L):
        K = fi.round_bf16(np.concatenate([ref[b]["kv"][l][0] for b in range(len(ref))]).astype(np.float32))
        V = fi.round_bf16(np.concatenate([ref[b]["kv"][l][1] for b in range(len(ref))]).astype(np.float32))
        kv.append((K, V))
    return ref, kv, lens


def _small():
    m = fi.Model(3, 512, 8, 2, 128, 1024, 1.0e4, 1e-6, "bf16")
    w = fi.Workload("small_bf16", m, [[(fi.VIDEO, 288), (fi.AUDIO, 150), (fi.TEXT, 30)], [(fi.VIDEO, 144), (fi.AUDIO, 97), (fi.TEXT, 9)]],
                    [fi.Prune(1, fi.GLOBAL, 0.6), fi.Prune(1, fi.FINE, 0.7), fi.Prune(2, fi.FINE, 0.7)], seed=41)
    weights = [fi.layer_weights(m, l, 7) for l in range(m.n_layers)]
    return w, weights, fi.embeddings(w)


def _oracle_steps(m, weights, kv, lens, x_steps, pos0):
    """Oracle decode of len(x_steps) consecutive tokens per sample; kv are the packed bf16 caches."""
    B = lens.shape[1]
    cu = np.concatenate([np.zeros((lens.shape[0], 1), np.int64), np.cumsum(lens, axis=1)], axis=1)
    outs = []
    caches = [[(kv[l][0][cu[l, b]:cu[l, b + 1]].astype(np.float64), kv[l][1][cu[l, b]:cu[l, b + 1]].astype(np.float64))
               for l in range(m.n_layers)] for b in range(B)]
    for t, x_new in enumerate(x_steps):
        row = []
        for b in range(B):
            r = orc.decode_step(m, weights, x_new[b].astype(np.float64), int(pos0[b]) + t, caches[b])
            row.append(r["x_out"])
            # the GPU appends bf16-rounded keys / values: do the same so both sides read identical caches
            caches[b] = [(np.concatenate([caches[b][l][0], fi.round_bf16(r["kv"][l][0][None].astype(np.float32)).astype(np.float64)]),
                          np.concatenate([caches[b][l][1], fi.round_bf16(r["kv"][l][1][None].astype(np.float32)).astype(np.float64)]))
                         for l in range(m.n_layers)]
        outs.append(np.stack(row))
    return outs


def test_decode_step_on_oracle_caches_ragged_batch():
    """Two samples whose layers hold 468/250 -> 281/150 -> 197/105 -> 138/74 keys: one step, then two more with
    the generated-token caches, against the oracle on identical bf16 caches."""
    w, weights, x = _small()
    m = w.model
    ref, kv, lens = _caches_from_oracle(w, weights, x)
    assert lens[:, 0].tolist() == [468, 197, 138] and lens[:, 1].tolist() == [250, 105, 74]
    dec = make_decoder(m, weights)
    B = 2
    rng = np.random.default_rng(5)
    x_steps = [fi.round_bf16(rng.standard_normal((B, m.hidden)).astype(np.float32)) for _ in range(3)]
    pos0 = np.array(w.seqlens, dtype=np.int32)
    want = _oracle_steps(m, weights, kv, lens, x_steps, pos0)
    kv_dev = [(dev(K, "bf16"), dev(V, "bf16")) for K, V in kv]
    gen_cap = 4
    gen = [(torch.zeros((B, gen_cap, m.n_kv_heads, m.head_dim), dtype=torch.bfloat16, device="cuda"),
            torch.zeros((B, gen_cap, m.n_kv_heads, m.head_dim), dtype=torch.bfloat16, device="cuda")) for _ in range(m.n_layers)]
    state = None
    for t in range(3):
        pos = torch.from_numpy(pos0 + t).cuda()
        r = dec.fastav_decode_step(dev(x_steps[t], "bf16"), pos, kv_dev, lens, gen=gen, gen_len=t, state=state)
        state = r["state"]
        torch.cuda.synchronize()
        got = host(r["x_out"])
        scale = float(np.sqrt(np.mean(want[t] ** 2)))
        assert_close(got, want[t], "bf16", scale=scale, what=f"decode step {t}")
    # the appended keys are the rotated keys of the new tokens (compare slot 0 of layer 0 with the oracle's)
    W0 = {k: v.astype(np.float64) for k, v in weights[0].items()}
    q, k, v = orc.layer_qkv(x_steps[0].astype(np.float64), W0, pos0.astype(np.int64), m)
    assert_close(host(gen[0][0][:, 0]), k, "bf16", what="appended K")
    assert_close(host(gen[0][1][:, 0]), v, "bf16", what="appended V")


def test_decode_step_without_generated_cache_equals_with_empty_one():
    w, weights, x = _small()
    m = w.model
    _, kv, lens = _caches_from_oracle(w, weights, x)
    dec = make_decoder(m, weights)
    kv_dev = [(dev(K, "bf16"), dev(V, "bf16")) for K, V in kv]
    x_new = dev(fi.round_bf16(np.random.default_rng(1).standard_normal((2, m.hidden)).astype(np.float32)), "bf16")
    pos = torch.from_numpy(np.array(w.seqlens, dtype=np.int32)).cuda()
    a = dec.fastav_decode_step(x_new, pos, kv_dev, lens)["x_out"].clone()
    gen = [(torch.zeros((2, 2, m.n_kv_heads, m.head_dim), dtype=torch.bfloat16, device="cuda"),
            torch.zeros((2, 2, m.n_kv_heads, m.head_dim), dtype=torch.bfloat16, device="cuda")) for _ in range(m.n_layers)]
    b = dec.fastav_decode_step(x_new, pos, kv_dev, lens, gen=gen, gen_len=0)["x_out"]
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def _positions_per_layer(n0, keep_local_per_prune, prune_layers, n_layers):
    """Original positions of the tokens in each layer's cache, from the per-prune kept row indices (relative to the
    sample's rows entering that prune): the cache of layer l holds what survives every prune at layers <= l."""
    pos, out, pi = np.arange(n0), [], 0
    for l in range(n_layers):
        while pi < len(prune_layers) and prune_layers[pi] == l:
            pos = pos[keep_local_per_prune[pi]]
            pi += 1
        out.append(pos)
    return out


def test_prefill_then_decode_end_to_end():
    """GPU pruned prefill -> GPU decode step on ITS caches, against the oracle's chain.  A near-tie may put a
    different token in the two kept sets, so both sides decode on the rows of their own caches that belong to
    tokens BOTH kept (per layer and sample); on this input that is every row or all but a few."""
    w, weights, x = _small()
    m = w.model
    dec = make_decoder(m, weights)
    spans, offs = fi.span_table(w)
    cu0 = fi.cu_seqlens(w)
    out = dec.fastav_prefill(dev(x, "bf16"), cu0, spans, offs, prune_tuples(w), w.n_last, want_kv=True, want_trace=True)
    lens = fa.fastav_schedule_lens(cu0, spans, offs, prune_tuples(w), w.n_last, m.n_layers)
    ref = orc.prefill(w, weights, x)
    B, L = len(ref), m.n_layers
    assert lens.tolist() == [[ref[b]["kv"][l][0].shape[0] for b in range(B)] for l in range(L)]
    prune_layers = [p.layer for p in w.prunes]
    # rows entering each prune, per sample, are known from the schedule
    n_in = [[ref[b]["prunes"][i]["n_in"] for b in range(B)] for i in range(len(w.prunes))]
    gpu_pos, ref_pos = [], []
    for b in range(B):
        keeps = []
        for i in range(len(w.prunes)):
            idx = out["prune_keep_idx"][i].cpu().numpy()
            cu_in = np.concatenate([[0], np.cumsum(n_in[i])])
            keeps.append(idx[(idx >= cu_in[b]) & (idx < cu_in[b + 1])] - cu_in[b])
        gpu_pos.append(_positions_per_layer(w.seqlens[b], keeps, prune_layers, L))
        ref_pos.append(_positions_per_layer(w.seqlens[b], [pr["keep"] for pr in ref[b]["prunes"]], prune_layers, L))
        assert np.array_equal(ref_pos[b][L - 1], ref[b]["kept_pos"])
    cu_l = np.concatenate([np.zeros((L, 1), np.int64), np.cumsum(lens, axis=1)], axis=1)
    kv_gpu, kv_ref, lens_common = [], [[] for _ in range(B)], np.zeros((L, B), dtype=np.int32)
    for l in range(L):
        rows_g = []
        for b in range(B):
            common, gi, ri = np.intersect1d(gpu_pos[b][l], ref_pos[b][l], return_indices=True)
            assert len(common) >= lens[l, b] - 4, (l, b, len(common), lens[l, b])
            lens_common[l, b] = len(common)
            rows_g.append(cu_l[l, b] + gi)
            kv_ref[b].append((ref[b]["kv"][l][0][ri], ref[b]["kv"][l][1][ri]))
        rows_g = torch.from_numpy(np.concatenate(rows_g)).cuda()
        kv_gpu.append((out["kv"][l][0][rows_g].contiguous(), out["kv"][l][1][rows_g].contiguous()))
    x_new = fi.round_bf16(np.random.default_rng(9).standard_normal((2, m.hidden)).astype(np.float32))
    pos = torch.from_numpy(np.array(w.seqlens, dtype=np.int32)).cuda()
    r = dec.fastav_decode_step(dev(x_new, "bf16"), pos, kv_gpu, lens_common)
    torch.cuda.synchronize()
    got = host(r["x_out"])
    for b in range(2):
        want = orc.decode_step(m, weights, x_new[b].astype(np.float64), w.seqlens[b], kv_ref[b])["x_out"]
        assert rel_l2(got[b], want) <= 2e-2, (b, rel_l2(got[b], want))


def test_decode_step_7b_layer_shape():
    """One layer at the 7B shape (hidden 4096, 32/8 heads, mlp 14336), 2048-token cache pruned to 1229."""
    w = fi.config(2)
    m = w.model
    weights = [fi.layer_weights(m, 0, w.weight_seed)]
    x = fi.embeddings(w)
    ref, kv, lens = _caches_from_oracle(w, weights, x)
    assert lens.tolist() == [[1229]]
    dec = make_decoder(m, weights)
    x_new = fi.round_bf16(np.random.default_rng(3).standard_normal((1, m.hidden)).astype(np.float32))
    want = _oracle_steps(m, weights, kv, lens, [x_new], np.array([2048]))[0]
    r = dec.fastav_decode_step(dev(x_new, "bf16"), torch.tensor([2048], dtype=torch.int32, device="cuda"),
                               [(dev(kv[0][0], "bf16"), dev(kv[0][1], "bf16"))], lens)
    torch.cuda.synchronize()
    assert_close(host(r["x_out"]), want, "bf16", scale=float(np.sqrt(np.mean(want ** 2))), what="7B-shape decode step")


@pytest.mark.parametrize("hq,hkv,dh,batch", [(28, 4, 128, 3), (8, 8, 64, 16), (16, 2, 64, 5), (28, 4, 128, 1), (16, 16, 64, 1),
                                             (16, 2, 64, 1)])
def test_decode_step_head_layouts(hq, hkv, dh, batch):
    """Seven and eight query heads per KV head, one query head per KV head, head_dim 64, a full batch of 16, and
    single samples (the one-row projections with the rotation folded in): ragged caches written by the oracle,
    two layers."""
    m = fi.Model(2, hq * dh // 2 if hq * dh >= 1024 else 512, hq, hkv, dh, 1024, 1.0e4, 1e-6, "bf16")
    rng = np.random.default_rng(hq + batch)
    lens1 = rng.integers(70, 330, size=batch)
    samples = [[(fi.VIDEO, int(n) - 20), (fi.TEXT, 20)] for n in lens1]
    w = fi.Workload("heads", m, samples, [fi.Prune(1, fi.FINE, 0.5)], seed=77)
    weights = [fi.layer_weights(m, l, 3) for l in range(m.n_layers)]
    ref, kv, lens = _caches_from_oracle(w, weights, fi.embeddings(w))
    dec = make_decoder(m, weights)
    x_new = fi.round_bf16(rng.standard_normal((batch, m.hidden)).astype(np.float32))
    pos0 = np.array(w.seqlens, dtype=np.int32)
    want = _oracle_steps(m, weights, kv, lens, [x_new], pos0)[0]
    r = dec.fastav_decode_step(dev(x_new, "bf16"), torch.from_numpy(pos0).cuda(), [(dev(K, "bf16"), dev(V, "bf16")) for K, V in kv], lens)
    torch.cuda.synchronize()
    assert_close(host(r["x_out"]), want, "bf16", scale=float(np.sqrt(np.mean(want ** 2))), what=f"decode Hq{hq} Hkv{hkv} dh{dh} B{batch}")


def test_decode_step_rejects_bad_arguments():
    w, weights, x = _small()
    m = w.model
    _, kv, lens = _caches_from_oracle(w, weights, x)
    dec = make_decoder(m, weights)
    kv_dev = [(dev(K, "bf16"), dev(V, "bf16")) for K, V in kv]
    pos = torch.from_numpy(np.array(w.seqlens, dtype=np.int32)).cuda()
    x_new = torch.zeros((2, m.hidden), dtype=torch.bfloat16, device="cuda")
    gen = [(torch.zeros((2, 1, m.n_kv_heads, m.head_dim), dtype=torch.bfloat16, device="cuda"),) * 2 for _ in range(m.n_layers)]
    with pytest.raises(fa.FastavError):                       # generated-token cache already full
        dec.fastav_decode_step(x_new, pos, kv_dev, lens, gen=gen, gen_len=1)
    with pytest.raises(fa.FastavError):                       # more samples than one step serves
        big = torch.zeros((17, m.hidden), dtype=torch.bfloat16, device="cuda")
        dec.fastav_decode_step(big, torch.zeros(17, dtype=torch.int32, device="cuda"), kv_dev, np.zeros((m.n_layers, 17), np.int32))
