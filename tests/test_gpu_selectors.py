"""GPU parity of the ablation strategies of Tables 2-3 (top / low attentive, top / low informative, random) inside
the pruned prefill, through the C ABI, against the CPU oracle.  Positional and random selections are integer work
and must match exactly; attentive ones may differ inside the tie band of the score at the cut."""
import numpy as np
import pytest
import torch

import fastav_inputs as fi
import paper_2601_13143_amd as fa
from oracle import fastav_oracle as orc
from gpu_util import dev, host, make_decoder, prune_tuples, rel_l2
from test_gpu_parity import _check_prefill, _oracle_and_gpu

pytestmark = pytest.mark.gpu

STRATEGIES = [(orc.TOP_INFORMATIVE, orc.TOP_ATTENTIVE), (orc.RANDOM, orc.RANDOM), (orc.RANDOM, orc.LOW_ATTENTIVE),
              (orc.LOW_INFORMATIVE, orc.TOP_ATTENTIVE), (orc.TOP_INFORMATIVE, orc.RANDOM)]


def _with_selectors(w: fi.Workload, sel_g: int, sel_f: int, seed: int) -> fi.Workload:
    prunes = [fi.Prune(p.layer, p.kind, p.keep_ratio, sel_g if p.kind == fi.GLOBAL else sel_f, seed) for p in w.prunes]
    return fi.Workload(w.name + f"_sel{sel_g}{sel_f}", w.model, w.samples, prunes, w.n_last, w.seed, w.weight_seed)


def test_selector_constants_agree():
    assert [fa.SEL_DEFAULT, fa.SEL_LOW_ATTENTIVE, fa.SEL_TOP_ATTENTIVE, fa.SEL_LOW_INFORMATIVE, fa.SEL_TOP_INFORMATIVE,
            fa.SEL_RANDOM] == [orc.DEFAULT, orc.LOW_ATTENTIVE, orc.TOP_ATTENTIVE, orc.LOW_INFORMATIVE,
                               orc.TOP_INFORMATIVE, orc.RANDOM]


@pytest.mark.parametrize("sel_g,sel_f", STRATEGIES)
def test_prefill_tiny_fp32_with_ablation_selectors(sel_g, sel_f):
    w = _with_selectors(fi.config(1), sel_g, sel_f, 2024)
    weights = [fi.layer_weights(w.model, l, w.weight_seed) for l in range(w.model.n_layers)]
    x = fi.embeddings(w)
    out, ref = _oracle_and_gpu(w, weights, x)
    st = _check_prefill(w, out, ref)
    assert st["flipped"] == 0                                   # fp32: every strategy's kept sets are exact
    assert st["x_rel_l2_0"] <= 2e-5 and st["x_max_abs_over_rms_0"] <= 2e-4, st
    assert np.array_equal(out["kept_pos"].cpu().numpy(), ref[0]["kept_pos"])
    assert out["tokens_in"].tolist() == [512, 512, 256, 256]    # same FLOPs as the paper's own strategy
    for l, (k, v) in enumerate(out["kv"]):
        assert rel_l2(host(k), ref[0]["kv"][l][0]) <= 2e-5 and rel_l2(host(v), ref[0]["kv"][l][1]) <= 2e-5


@pytest.mark.parametrize("sel_g,sel_f", STRATEGIES)
def test_prefill_small_bf16_ragged_batch_with_ablation_selectors(sel_g, sel_f):
    m = fi.Model(3, 512, 8, 2, 128, 1024, 1.0e4, 1e-6, "bf16")
    base = fi.Workload("small_bf16", m, [[(fi.VIDEO, 288), (fi.AUDIO, 150), (fi.TEXT, 30)], [(fi.VIDEO, 144), (fi.AUDIO, 97), (fi.TEXT, 9)]],
                       [fi.Prune(1, fi.GLOBAL, 0.6), fi.Prune(1, fi.FINE, 0.7), fi.Prune(2, fi.FINE, 0.7)], seed=41)
    w = _with_selectors(base, sel_g, sel_f, 7)
    weights = [fi.layer_weights(m, l, 7) for l in range(m.n_layers)]
    out, ref = _oracle_and_gpu(w, weights, fi.embeddings(w), want_kv=False)
    st = _check_prefill(w, out, ref)
    for b in range(2):
        assert st[f"x_rel_l2_{b}"] <= 1e-2 and st[f"x_max_abs_over_rms_{b}"] <= 5e-2, st
    if sel_f == orc.RANDOM:                                      # nothing floating point decides a kept set
        assert st["flipped"] == 0
        for b in range(2):
            cu = out["cu_seqlens_out"].cpu().numpy()
            assert np.array_equal(out["kept_pos"].cpu().numpy()[cu[b]:cu[b + 1]], ref[b]["kept_pos"])


@pytest.mark.parametrize("sel_g", [orc.RANDOM, orc.TOP_INFORMATIVE])
def test_global_selectors_on_a_sample_longer_than_the_lds_key_buffer(sel_g):
    """40 000 tokens: the select kernel re-reads its keys from memory instead of LDS; the draws of the random
    strategy are keyed by original positions, two samples draw differently."""
    m = fi.Model(1, 256, 4, 2, 64, 688, 1.0e4, 1e-6, "f32")
    w = fi.Workload("long1", m, [[(fi.VIDEO, 30000), (fi.AUDIO, 9990), (fi.TEXT, 10)], [(fi.VIDEO, 900), (fi.AUDIO, 90), (fi.TEXT, 10)]],
                    [fi.Prune(0, fi.GLOBAL, 0.03, sel_g, 5)], seed=53)
    weights = [fi.layer_weights(m, 0, 3)]
    out, ref = _oracle_and_gpu(w, weights, fi.embeddings(w), want_kv=False)
    st = _check_prefill(w, out, ref)
    assert st["flipped"] == 0
    cu = out["cu_seqlens_out"].cpu().numpy()
    kept = [out["kept_pos"].cpu().numpy()[cu[b]:cu[b + 1]] for b in range(2)]
    for b in range(2):
        assert np.array_equal(kept[b], ref[b]["kept_pos"])
        assert st[f"x_rel_l2_{b}"] <= 2e-5, st
    if sel_g == orc.RANDOM:
        assert not np.array_equal(kept[0][kept[0] < 900][:20], kept[1][:20])
