"""Helpers shared by the GPU parity tests: host<->device conversion of the seeded inputs, error metrics
and the stated tolerances."""
import numpy as np
import torch

import fastav_inputs as fi
import paper_2601_13143_amd as fa

# bf16 kernels vs the fp64 oracle on identical bf16-rounded inputs (stage-wise, outputs of O(1) scale)
BF16_MAX_ABS, BF16_REL_L2 = 2e-2, 1e-2
# fp32 kernels vs the fp64 oracle: fp32 accumulation over K <= ~1e3 terms plus fp32 exp/rsqrt
F32_MAX_ABS, F32_REL_L2 = 2e-4, 2e-5
# end-to-end kept sets may differ only on tokens whose oracle score is within this of the k-th score
TIE_BAND = 1e-3


def torch_dtype(code_or_name):
    if code_or_name in (fa.BF16, "bf16"):
        return torch.bfloat16
    return torch.float32


def dev(a: np.ndarray, dtype) -> torch.Tensor:
    """fp32 numpy (already bf16-representable when dtype is bf16) -> device tensor, exactly."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda").to(torch_dtype(dtype))


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_l2(got: np.ndarray, want: np.ndarray) -> float:
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30))


def max_abs(got: np.ndarray, want: np.ndarray) -> float:
    return float(np.max(np.abs(got - want))) if got.size else 0.0


def assert_close(got, want, dtype, scale: float = 1.0, what: str = ""):
    """Relative L2, and max-abs after dividing by ``scale`` (the output's natural magnitude, so that the
    absolute bound applies to O(1) values); an element larger than 1 in magnitude is judged relative to
    itself, since a bf16 result carries a rounding error proportional to its own size (2^-9 |x|)."""
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    err = np.abs(got - want) / scale / np.maximum(1.0, np.abs(want) / scale)
    ma, rl = (float(err.max()) if err.size else 0.0), rel_l2(got, want)
    lim_a, lim_r = (BF16_MAX_ABS, BF16_REL_L2) if dtype in (fa.BF16, "bf16") else (F32_MAX_ABS, F32_REL_L2)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    assert ma <= lim_a and rl <= lim_r, f"{what}: max_abs/scale={ma:.3e} (lim {lim_a}), rel_l2={rl:.3e} (lim {lim_r})"
    return ma, rl


def model_struct(m: fi.Model):
    return fa.make_model(m.n_layers, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.mlp_dim, m.rope_base, m.rms_eps,
                         fa.BF16 if m.dtype == "bf16" else fa.F32)


def make_decoder(m: fi.Model, weights):
    """weights: list of per-layer dicts of fp32 numpy arrays -> Decoder with device weights set."""
    dec = fa.Decoder(model_struct(m))
    for l, W in enumerate(weights):
        dec.fastav_set_weights(l, {k: dev(v, m.dtype) for k, v in W.items()})
    return dec


def prune_tuples(w: fi.Workload):
    return [(p.layer, p.kind, p.keep_ratio, p.selector, p.seed) for p in w.prunes]


def make_decoder_streamed(m: fi.Model, seed: int, threads: int = 8):
    """Full-size models: generate each layer's seeded weights on host threads and upload it at once, so that
    only a few layers of fp32 host copies are alive at any time."""
    from concurrent.futures import ThreadPoolExecutor

    dec = fa.Decoder(model_struct(m))

    def gen(l):
        W = fi.layer_weights(m, l, seed)
        return l, {k: (fi.bf16_bits(v) if m.dtype == "bf16" else v) for k, v in W.items()}

    with ThreadPoolExecutor(max_workers=threads) as ex:
        for l, W in ex.map(gen, range(m.n_layers)):
            d = {}
            for k, v in W.items():
                t = torch.from_numpy(v).cuda()
                d[k] = t.view(torch.bfloat16) if m.dtype == "bf16" else t
            dec.fastav_set_weights(l, d)
    return dec
