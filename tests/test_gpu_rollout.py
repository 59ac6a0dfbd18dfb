"""GPU parity of the attention-rollout analysis (Eq. 2-3) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import fastav_inputs as fi
from oracle import fastav_oracle as orc
import paper_2601_13143_amd as fa
from gpu_util import dev, host, make_decoder, rel_l2

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("Hq,Hkv,dh,n", [(8, 2, 128, 300), (4, 4, 64, 132), (28, 4, 128, 260), (32, 8, 128, 1028), (4, 2, 128, 4)])
def test_attention_map_matches_oracle(Hq, Hkv, dh, n):
    """Head-mean causal attention map of one layer on identical bf16 inputs: entries are probabilities (<= 1),
    written as bf16, so they are compared relative to the row's own scale."""
    rng = np.random.default_rng(Hq + n)
    q = fi.round_bf16((rng.standard_normal((n, Hq, dh)) * 1.3).astype(np.float32))
    k = fi.round_bf16((rng.standard_normal((n, Hkv, dh)) * 1.3).astype(np.float32))
    m = fa.make_model(1, 64, Hq, Hkv, dh, 64)
    got = host(fa.fastav_attention_map(m, dev(q, "bf16"), dev(k, "bf16")))
    want = orc.head_mean_attention_map(q.astype(np.float64), k.astype(np.float64))
    assert np.all(np.triu(got, 1) == 0.0)
    assert np.max(np.abs(got.sum(axis=1) - 1.0)) <= 5e-3               # bf16 entries: each within 2^-9 of itself
    assert rel_l2(got, want) <= 5e-3, rel_l2(got, want)
    assert np.max(np.abs(got - want) / np.maximum(want, 1.0 / n)) <= 2e-2


def _small(n_layers=3):
    m = fi.Model(n_layers, 512, 8, 2, 128, 1024, 1.0e4, 1e-6, "bf16")
    w = fi.Workload("roll", m, [[(fi.TEXT, 8), (fi.VIDEO, 144), (fi.AUDIO, 92), (fi.TEXT, 12)]], [], seed=51)
    weights = [fi.layer_weights(m, l, 13) for l in range(m.n_layers)]
    for W in weights:                                # sharper attention than N(0, 0.02) weights give
        W["wq"] = fi.round_bf16((W["wq"] * 6.0).astype(np.float32))
        W["wk"] = fi.round_bf16((W["wk"] * 6.0).astype(np.float32))
    return m, w, weights, fi.embeddings(w)


@pytest.mark.parametrize("alpha", [0.5, 1.0, 0.0])
def test_rollout_matches_oracle(alpha):
    m, w, weights, x = _small()
    dec = make_decoder(m, weights)
    n = x.shape[0]
    want = orc.attention_rollout(m, weights, x, alpha)
    for upto in (1, 2, 3):
        got = host(dec.fastav_rollout(dev(x, "bf16"), alpha, upto))
        torch.cuda.synchronize()
        assert np.max(np.abs(got.sum(axis=1) - 1.0)) <= 1e-2            # rows of a rollout sum to 1
        assert np.all(np.abs(np.triu(got, 1)) <= 1e-6)
        assert rel_l2(got, want[upto - 1]) <= 1e-2, (alpha, upto, rel_l2(got, want[upto - 1]))
    if alpha == 0.0:
        assert np.array_equal(got, np.eye(n))


def test_rollout_is_deterministic_and_rejects_bad_arguments():
    m, w, weights, x = _small(2)
    dec = make_decoder(m, weights)
    a = dec.fastav_rollout(dev(x, "bf16"), 0.7).clone()
    b = dec.fastav_rollout(dev(x, "bf16"), 0.7)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    with pytest.raises(fa.FastavError):
        dec.fastav_rollout(dev(x, "bf16"), 1.5)
    with pytest.raises(fa.FastavError):
        dec.fastav_rollout(dev(x, "bf16"), 0.5, 3)             # more layers than the model has
    with pytest.raises(fa.FastavError):
        dec.fastav_rollout(dev(x[:254], "bf16"), 0.5)          # n not a multiple of 4
