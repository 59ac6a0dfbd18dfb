"""Writes the oracle's results for the large benchmark configs (3, 4, 5) to tests/golden/cfgN_oracle.npz.

Only the CPU oracle and the seeded input generators are used here; nothing comes from the HIP path.  The
full-size oracle runs take minutes to tens of minutes (fp64 NumPy), which is why their results are stored
instead of being recomputed inside the GPU tests.

    python tests/golden/make_goldens.py 3 4 5

Stored per config: the kept original positions of every prune and sample, the fine-prune scores, the
surviving positions, and the final hidden state on a fixed sample of surviving rows (all of them when
there are fewer than 96 per sample)."""
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import fastav_inputs as fi  # noqa: E402
from oracle import fastav_oracle as orc  # noqa: E402

ROWS_PER_SAMPLE = 96


def run(cfg: int) -> None:
    w = fi.config(cfg)
    x = fi.embeddings(w)
    cache = {}

    def weights(l):                     # one layer resident at a time
        if l not in cache:
            cache.clear()
            cache[l] = fi.layer_weights(w.model, l, w.weight_seed)
        return cache[l]

    t0 = time.time()
    out = {}
    row = 0
    for b, spans in enumerate(w.samples):
        n = sum(l for _, l in spans)
        r = orc.prefill_sample(w.model, weights, x[row:row + n], spans, w.prunes, w.n_last, keep_kv=False)
        row += n
        for i, pr in enumerate(r["prunes"]):
            out[f"s{b}_p{i}_keep_pos"] = pr["pos_in"][pr["keep"]].astype(np.int32)
            out[f"s{b}_p{i}_pos_in"] = pr["pos_in"].astype(np.int32)
            if pr["scores"] is not None:
                out[f"s{b}_p{i}_scores"] = pr["scores"].astype(np.float64)
        kp = r["kept_pos"].astype(np.int32)
        out[f"s{b}_kept_pos"] = kp
        rng = np.random.default_rng(1000 * cfg + b)
        sel = np.sort(rng.choice(len(kp), min(ROWS_PER_SAMPLE, len(kp)), replace=False))
        sel[-1] = len(kp) - 1                                      # always include the last token
        out[f"s{b}_x_rows"] = sel.astype(np.int32)
        out[f"s{b}_x_out"] = r["x_out"][sel].astype(np.float32)
        out[f"s{b}_x_rms"] = np.float64(np.sqrt(np.mean(r["x_out"] ** 2)))
        print(f"cfg{cfg} sample {b}: n={n} -> {len(kp)} survivors, {time.time() - t0:.0f} s", flush=True)
    np.savez_compressed(os.path.join(HERE, f"cfg{cfg}_oracle.npz"), **out)


if __name__ == "__main__":
    for a in sys.argv[1:]:
        run(int(a))
