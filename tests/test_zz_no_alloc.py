"""The entry point that allocates nothing (fastav_score_static): same result as fastav_score, which takes its
scratch from the caller, on two calls in a row — the second on a smaller input, so that whatever the first call left
in the library's built-in scratch array is still there — and both against the CPU oracle."""
import ctypes as C

import numpy as np
import pytest
import torch

import fastav_inputs as fi
from oracle import fastav_oracle as orc
import paper_2601_13143_amd as fa
from paper_2601_13143_amd import binding as B
from gpu_util import dev, host, rel_l2

pytestmark = pytest.mark.gpu


def _case(lens, Hq, Hkv, dh, n_last, seed):
    rng = np.random.default_rng(seed)
    T = sum(lens)
    q = fi.round_bf16(rng.standard_normal((T, Hq, dh)).astype(np.float32) * 1.3)
    k = fi.round_bf16(rng.standard_normal((T, Hkv, dh)).astype(np.float32) * 1.3)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    return q, k, cu


def test_score_static_equals_score_with_workspace_on_two_calls_in_a_row():
    Hq, Hkv, dh = 32, 8, 128
    m = fa.make_model(1, 64, Hq, Hkv, dh, 64, dtype=fa.BF16)
    lib = fa.lib()
    for lens, n_last, seed in (([3000, 517, 1, 129], 2, 1), ([700, 130], 1, 2)):      # the second call is the smaller one
        q, k, cu = _case(lens, Hq, Hkv, dh, n_last, seed)
        T = int(cu[-1])
        qd, kd, cud = dev(q, "bf16"), dev(k, "bf16"), torch.from_numpy(cu).cuda()
        out = torch.full((T,), -1.0, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        # raw C-ABI call: inputs and the output only, no workspace
        st = lib.fastav_score_static(C.byref(m), qd.data_ptr(), qd.stride(0), kd.data_ptr(), kd.stride(0), cud.data_ptr(),
                                     len(lens), T, max(lens), n_last, out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        assert st == B.OK, lib.fastav_last_error()
        want_ws = fa.fastav_score(m, qd, kd, cud, max(lens), n_last)
        torch.cuda.synchronize()
        assert torch.equal(out, want_ws), float((out - want_ws).abs().max())
        got = host(out)
        for b, n in enumerate(lens):
            ref = orc.last_query_scores(q[cu[b]:cu[b + 1]], k[cu[b]:cu[b + 1]], n_last)
            g = got[cu[b]:cu[b + 1]]
            assert abs(g.sum() - 1.0) < 1e-4
            assert np.max(np.abs(g - ref)) * n <= 1e-3 * max(1.0, ref.max() * n) and rel_l2(g, ref) <= 1e-4


def test_score_static_rejects_what_does_not_fit_before_any_launch():
    m = fa.make_model(1, 64, 32, 8, 128, 64, dtype=fa.BF16)
    lib = fa.lib()
    T = 80000                                                      # 32 heads x 80000 tokens x 4 bytes > 8 MiB
    assert lib.fastav_score_workspace_bytes(32, T, 1, 1) > B.SCORE_STATIC_BYTES
    st = lib.fastav_score_static(C.byref(m), 4096, 4096, 4096, 1024, 4096, 1, T, T, 1, 4096, None)
    assert st == B.EWORKSPACE and b"built-in buffer" in lib.fastav_last_error()
