"""Benchmark of the FastAV pruned prefill on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3]

A step is one pass of the whole hot path (every layer, every prune step) over one batch of synthetic
audio-visual tokens already resident in HBM.  Prints ONE JSON line: pruned-prefill tokens/s as `value`,
the unpruned rate and the prune-step times beside it, a `roofline` object for the dominant kernel (the
gate/up SwiGLU GEMM) measured with HIP events around its launches, one entry per other kernel kind, and
the CPU oracle timed on this host (`cpu_baseline`)."""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import fastav_inputs as fi  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E

WORKLOADS = {"cfg1": 1, "cfg2": 2, "cfg3": 3, "cfg4": 4, "cfg5": 5}


def _recorded_traffic(workload):
    """-> (bytes per launch of the gate/up GEMM, where the figure comes from).  A profiler cannot run inside this
    process, so the figure is NOT measured by this run: it is read back from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, calibrated on a copy kernel) and labelled as such; (None, None) when there is no
    summary for this workload."""
    rel = os.path.join("profiles", f"prefill_{workload}_pmc_traffic.txt")
    try:
        for line in open(os.path.join(ROOT, rel)):
            if line.startswith("traffic_bytes_per_launch_gemm_swiglu:"):
                return float(line.split(":")[1]), f"recorded, not measured in this run: {rel} (two rocprofv3 --pmc runs of this script)"
    except OSError:
        pass
    return None, None


def _upload_weights(dec, m, seed, threads):
    import torch

    def gen(l):
        W = fi.layer_weights(m, l, seed)
        return l, {k: (fi.bf16_bits(v) if m.dtype == "bf16" else v) for k, v in W.items()}

    with ThreadPoolExecutor(max_workers=threads) as ex:
        for l, W in ex.map(gen, range(m.n_layers)):
            dev = {}
            for k, v in W.items():
                t = torch.from_numpy(v).cuda()
                dev[k] = t.view(torch.bfloat16) if m.dtype == "bf16" else t
            dec.fastav_set_weights(l, dev)


def _cpu_baseline(w, threads):
    """Times the oracle, as it stands, on a bounded sample of the workload: a 4-layer surrogate that runs one
    layer at each token count of the schedule (n0; after the global prune with the first fine prune; after
    it with the second; after that), each layer timed through the oracle's own per-layer weight callback,
    then weighted by how many layers of the real model run at that count."""
    from oracle import fastav_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        used = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        used = threads
    m = w.model
    globals_ = [p for p in w.prunes if p.kind == fi.GLOBAL]
    fines = [p for p in w.prunes if p.kind == fi.FINE]
    if not (len(w.samples) == 1 and len(globals_) == 1 and len(fines) == 2):
        return None
    m4 = fi.Model(4, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.mlp_dim, m.rope_base, m.rms_eps, m.dtype)
    prunes4 = [fi.Prune(1, fi.GLOBAL, globals_[0].keep_ratio), fi.Prune(1, fi.FINE, fines[0].keep_ratio),
               fi.Prune(2, fi.FINE, fines[1].keep_ratio)]
    w4 = fi.Workload("surrogate", m4, w.samples, prunes4, w.n_last, w.seed, w.weight_seed)
    x = fi.embeddings(w4)
    W = fi.layer_weights(m4, 0, w.weight_seed)
    marks = []

    def get_w(l):
        marks.append(time.perf_counter())
        return W

    reps = 2                                         # two passes of the surrogate: 10-20 s of CPU work on the box
    per_layer = np.zeros(4)
    for _ in range(reps):
        marks.clear()
        orc.prefill(w4, get_w, x, keep_kv=False)
        marks.append(time.perf_counter())
        per_layer += np.diff(marks) / reps           # seconds at token counts n0, n1, n2, n3
    g, f1, f2 = globals_[0].layer, fines[0].layer, fines[1].layer
    # real schedule: layers [0,g) at n0; [g,f1] at n1; (f1,f2] at n2; (f2,L) at n3
    counts = [g, f1 - g + 1, f2 - f1, m.n_layers - 1 - f2]
    total = float(np.dot(per_layer, counts))
    return {"value": w.total_tokens / total, "unit": "tokens/s", "cores": int(used), "kind": "oracle",
            "sample": f"fp64 NumPy oracle on a 4-layer surrogate (one layer per token count of the pruned schedule, "
                      f"mean of {reps} passes, {per_layer.sum() * reps:.1f} s measured), extrapolated to {m.n_layers} layers by layer counts {counts}"}


def _prune_stress(fa, torch, model_struct, hq, hkv, dh, d):
    """Score, select and gather on a batch large enough that bytes, not launch latency, set the time
    (16 samples x 16384 tokens, 7B shapes): achieved GB/s of algorithmic bytes against the 8 TB/s peak."""
    B, n = 16, 16384
    T = B * n
    cu = np.arange(B + 1, dtype=np.int32) * n
    cu_dev = torch.from_numpy(cu).cuda()
    g = torch.Generator(device="cuda").manual_seed(7)

    def timeit(fn, kind, iters=8):
        """GPU time per call of one kernel kind, from the library's own HIP events around its launches (the
        Python call around them also allocates outputs, which is not part of the kernels' time)."""
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        fa.fastav_profile_enable([kind])
        ms0, n0, _ = fa.fastav_profile_collect(kind)
        for _ in range(iters):
            fn()
        torch.cuda.synchronize()
        ms1, n1, _ = fa.fastav_profile_collect(kind)
        fa.fastav_profile_enable([])
        return (ms1 - ms0) / iters * 1e-3

    q = torch.randn(T, hq, dh, device="cuda", generator=g).bfloat16()
    k = torch.randn(T, hkv, dh, device="cuda", generator=g).bfloat16()
    t_score = timeit(lambda: fa.fastav_score(model_struct, q, k, cu_dev, n, 1), "score")
    del q
    scores = torch.rand(T, device="cuda", generator=g)
    prot = (torch.rand(T, device="cuda", generator=g) < 0.05).to(torch.uint8)
    kc = [int(0.7 * n)] * B
    t_sel = timeit(lambda: fa.fastav_select_gather(scores, prot, cu, kc, []), "select")
    x = torch.randn(T, d, device="cuda", generator=g)
    o = torch.randn(T, hq * dh, device="cuda", generator=g).bfloat16()
    v = torch.randn(T, hkv * dh, device="cuda", generator=g).bfloat16()
    pos = torch.arange(T, device="cuda", dtype=torch.int32)
    tens = [x, o, k.view(T, hkv * dh), v, pos, prot]
    t_gather = timeit(lambda: fa.fastav_select_gather(scores, prot, cu, kc, tens), "gather", iters=4)
    rows = sum(kc)
    b_score = T * hkv * dh * 2 + 4 * T
    b_sel = 5 * T + 4 * rows
    b_gather = 2 * rows * (d * 4 + hq * dh * 2 + 2 * hkv * dh * 2 + 4 + 1) + 4 * rows
    mk = lambda byt, t: {"us": t * 1e6, "achieved": byt / t / 1e9, "unit": "GB/s", "frac": byt / t / 1e9 / PEAK_HBM_GBS}
    return {"shape": f"{B} samples x {n} tokens, Hq {hq}, Hkv {hkv}, head_dim {dh}, hidden {d}, keep 0.7",
            "score": mk(b_score, t_score), "select": mk(b_sel, t_sel), "gather": mk(b_gather, t_gather)}


def _achievable_peak(fa, torch):
    """What the chip sustains with nothing in the way, next to the datasheet peaks the roofline fractions use: a loop
    of bf16 matrix instructions only (no memory traffic, two waves per SIMD on every CU) and one streaming read of a
    1 GiB buffer (four times the memory-side cache).  Timed with events on the launch stream."""
    sink = torch.zeros(1 << 20, dtype=torch.float32, device="cuda")
    src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")          # 1 GiB

    def timed(fn, reps):
        fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        torch.cuda.synchronize()
        work = 0.0
        for i in range(reps):
            ev[i].record()
            work = fn()
        ev[reps].record()
        torch.cuda.synchronize()
        return work, min(ev[i].elapsed_time(ev[i + 1]) for i in range(reps)) * 1e-3

    fl, t_m = timed(lambda: fa.fastav_probe_mfma(2000, sink), 3)
    # the same loop on operands drawn like activations: a matrix instruction's power, and with it the clock the chip
    # holds, depends on how many operand bits toggle; several back-to-back launches so that the clock settles
    ops = torch.randn(32768, device="cuda", generator=torch.Generator(device="cuda").manual_seed(11)).bfloat16()
    fl_n, t_n = timed(lambda: [fa.fastav_probe_mfma(2000, sink, ops) for _ in range(8)][0], 4)
    t_n /= 8
    by, t_r = timed(lambda: fa.fastav_probe_read(src, sink), 5)
    del src
    return {"mfma_bf16": {"achieved": fl / t_m / 1e12, "unit": "TFLOP/s", "of_datasheet": fl / t_m / 1e12 / PEAK_BF16_TFLOPS,
                          "what": "v_mfma_f32_16x16x32_bf16 only, 32 independent accumulator chains per SIMD, small-integer operands"},
            "mfma_bf16_normal_operands": {"achieved": fl_n / t_n / 1e12, "unit": "TFLOP/s", "of_datasheet": fl_n / t_n / 1e12 / PEAK_BF16_TFLOPS,
                                          "what": "the same loop on standard-normal operands, sustained over 8 launches: the ceiling "
                                                  "under the switching activity of real data (the chip lowers its clock)"},
            "hbm_read": {"achieved": by / t_r / 1e9, "unit": "GB/s", "of_datasheet": by / t_r / 1e9 / PEAK_HBM_GBS,
                         "what": "streaming read of 1 GiB, 16 bytes per lane and load"}}


def _by_shape(fa, torch, dec, m, cu, spans, offs, prunes, n_last, iters=6):
    """Every kernel of a layer at every token count of the schedule, on its own: us per launch and the fraction of
    its roofline (flops over the bf16 MFMA peak for the GEMMs and attention, algorithmic bytes over the HBM peak
    for RMSNorm and RoPE).  The GEMMs rotate through the layers' weights, so the weights stream from HBM as they do
    in the model.  Timed with the library's events on the launch stream."""
    if m.dtype != "bf16":
        return None
    L = m.n_layers
    qd, kd, d, mlp, dh = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim, m.hidden, m.mlp_dim, m.head_dim
    tin, tout, _ = fa.fastav_schedule(cu, spans, offs, prunes, n_last, L)
    stages = [fa.fastav_schedule(cu, spans, offs, prunes[:i], n_last, L)[2] for i in range(len(prunes) + 1)]
    g = torch.Generator(device="cuda").manual_seed(3)
    nw = min(L, 4)
    wqkv = [torch.cat([dec._weights[l]["wq"], dec._weights[l]["wk"], dec._weights[l]["wv"]]) for l in range(nw)]
    out = []
    for lens in stages:
        T = int(lens.sum())
        n_attn = int((tin == T).sum())
        n_mlp = int((tout == T).sum())
        if n_attn == 0 and n_mlp == 0:
            continue
        cu_s = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).cuda()
        hn = torch.randn(T, d, device="cuda", generator=g).bfloat16()
        ao = torch.randn(T, qd, device="cuda", generator=g).bfloat16()
        hm = torch.randn(T, mlp, device="cuda", generator=g).bfloat16() * 0.1
        res = torch.randn(T, d, device="cuda", generator=g)
        qkv = torch.randn(T, qd + 2 * kd, device="cuda", generator=g).bfloat16()
        pos = torch.arange(T, device="cuda", dtype=torch.int32)
        q = qkv.as_strided((T, m.n_q_heads, dh), (qkv.stride(0), dh, 1))
        k = qkv.as_strided((T, m.n_kv_heads, dh), (qkv.stride(0), dh, 1), qd)
        v = qkv.as_strided((T, m.n_kv_heads, dh), (qkv.stride(0), dh, 1), qd + kd)
        gain = dec._weights[0]["g_attn"]
        c_qkv = torch.empty(T, qd + 2 * kd, device="cuda", dtype=torch.bfloat16)
        c_mlp = torch.empty(T, mlp, device="cuda", dtype=torch.bfloat16)
        attn_flops = float(sum(2.0 * m.n_q_heads * dh * n * (n + 1.0) for n in lens.tolist()))
        cases = [
            ("qkv_store", "linear_store", lambda i: fa.fastav_linear(hn, wqkv[i % nw], fa.EPI_STORE, c=c_qkv), 2.0 * T * (qd + 2 * kd) * d, True),
            ("attention", "attention", lambda i: fa.fastav_attention(dec.model, q, k, v, cu_s, int(lens.max())), attn_flops, True),
            ("o_resadd", "linear_resadd", lambda i: fa.fastav_linear(ao, dec._weights[i % L]["wo"], fa.EPI_RESADD, c=res), 2.0 * T * d * qd, True),
            ("gateup_swiglu", "linear_swiglu", lambda i: fa.fastav_linear(hn, dec._weights[i % L]["w_gate"], fa.EPI_SWIGLU, w2=dec._weights[i % L]["w_up"], c=c_mlp), 4.0 * T * mlp * d, True),
            ("down_resadd", "linear_resadd", lambda i: fa.fastav_linear(hm, dec._weights[i % L]["w_down"], fa.EPI_RESADD, c=res), 2.0 * T * d * mlp, True),
            ("rmsnorm", "rmsnorm", lambda i: fa.fastav_rmsnorm(res, gain, 1e-6), T * d * 6.0, False),
            ("rope", "rope", lambda i: fa.fastav_rope(qkv, pos, m.n_q_heads + m.n_kv_heads, dh, m.rope_base), 2.0 * T * (qd + kd) * 2.0, False),
        ]
        row = {"tokens": T, "layers_with_attention_at_this_count": n_attn, "layers_with_mlp_at_this_count": n_mlp, "kernels": {}}
        for name, kind, fn, work, is_flops in cases:
            fn(0); fn(1)
            torch.cuda.synchronize()
            fa.fastav_profile_enable([kind])
            ms0, n0, _ = fa.fastav_profile_collect(kind)
            for i in range(iters):
                fn(i + 2)
            torch.cuda.synchronize()
            ms1, n1, _ = fa.fastav_profile_collect(kind)
            fa.fastav_profile_enable([])
            t = (ms1 - ms0) * 1e-3 / max(1, n1 - n0)
            rate = work / t / (1e12 if is_flops else 1e9)
            row["kernels"][name] = {"us": t * 1e6, "achieved": rate, "unit": "TFLOP/s" if is_flops else "GB/s",
                                    "frac": rate / (PEAK_BF16_TFLOPS if is_flops else PEAK_HBM_GBS)}
        out.append(row)
        del hn, ao, hm, res, qkv, c_qkv, c_mlp
    return out


def _decode_bench(fa, torch, dec, m, w, x, cu, spans, offs, prunes, iters=20):
    """One generated token's forward (the paper's latency metric, Section 3.1) on the caches the pruned prefill
    left, and on the unpruned caches: ms per step and bytes moved (all weights once + every layer's cache once)
    against the HBM peak.  Not part of `value`."""
    if m.dtype != "bf16" or len(w.samples) > 16:
        return None
    B = len(w.samples)
    qd, kd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    w_bytes = m.n_layers * 2.0 * ((qd + 2 * kd) * m.hidden + m.hidden * qd + 3 * m.hidden * m.mlp_dim)
    g = torch.Generator(device="cuda").manual_seed(11)
    x_new = torch.randn(B, m.hidden, device="cuda", generator=g).bfloat16()
    pos = torch.tensor(w.seqlens, dtype=torch.int32, device="cuda")
    res = {}
    for name, pr in (("pruned", prunes), ("unpruned", [])):
        out = dec.fastav_prefill(x, cu, spans, offs, pr, w.n_last, want_kv=True)
        lens = fa.fastav_schedule_lens(cu, spans, offs, pr, w.n_last, m.n_layers)
        st = None
        for _ in range(3):
            st = dec.fastav_decode_step(x_new, pos, out["kv"], lens, state=st)["state"]
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
        torch.cuda.synchronize()
        for i in range(iters):
            ev[i].record()
            dec.fastav_decode_step(x_new, pos, out["kv"], lens, state=st)
        ev[iters].record()
        torch.cuda.synchronize()
        ts = [ev[i].elapsed_time(ev[i + 1]) for i in range(iters)]
        cache_bytes = float(lens.sum()) * 2 * kd * 2
        med = float(np.median(ts))
        res[name] = {"ms_per_token_median": med, "ms_per_token_min": float(np.min(ts)),
                     "cache_MB": cache_bytes / 1e6, "weights_MB": w_bytes / 1e6,
                     "achieved": (w_bytes + cache_bytes) / (med * 1e-3) / 1e9, "unit": "GB/s",
                     "frac": (w_bytes + cache_bytes) / (med * 1e-3) / 1e9 / PEAK_HBM_GBS}
        del out
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3", choices=sorted(WORKLOADS))
    ap.add_argument("--paper-schedule", action="store_true",
                    help="prune as the paper does: global at the middle layer, then 20 %% fine at every later layer")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-passes", action="store_true", help="skip the per-kernel timing passes")
    ap.add_argument("--shapes-only", action="store_true",
                    help="run only the per-shape kernel table and the achievable-peak probes (short: for counter runs under rocprofv3)")
    ap.add_argument("--stress-only", action="store_true",
                    help="run only the prune kernels at the stress shape (short: for counter runs under rocprofv3)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the path is single-GPU by design: no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2601_13143_amd as fa

    fa.lib()
    if os.environ.get("FASTAV_BENCH_ROPE") == "0":            # A/B aid: the separate RoPE kernel instead of the fused epilogue
        fa.fastav_set_option(fa.OPT_FUSED_ROPE, 0)
    host_threads = len(os.sched_getaffinity(0))
    w = fi.config(WORKLOADS[args.workload])
    if args.paper_schedule:
        w = fi.paper_schedule(w, global_keep=w.prunes[0].keep_ratio if w.prunes else 0.6)
    m = w.model
    dec = fa.Decoder(fa.make_model(m.n_layers, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.mlp_dim, m.rope_base,
                                   m.rms_eps, fa.BF16 if m.dtype == "bf16" else fa.F32))
    t0 = time.time()
    _upload_weights(dec, m, w.weight_seed, min(16, host_threads))
    x_np = fi.embeddings(w)
    x = torch.from_numpy(fi.bf16_bits(x_np)).cuda().view(torch.bfloat16) if m.dtype == "bf16" else torch.from_numpy(x_np).cuda()
    setup_s = time.time() - t0
    cu, (spans, offs) = fi.cu_seqlens(w), fi.span_table(w)
    prunes = [(p.layer, p.kind, p.keep_ratio) for p in w.prunes]
    tokens = w.total_tokens

    if args.shapes_only or args.stress_only:
        line = {"workload": w.name}
        if args.shapes_only:
            line["achievable_peak"] = _achievable_peak(fa, torch)
            line["by_shape"] = _by_shape(fa, torch, dec, m, cu, spans, offs, prunes, w.n_last, iters=3)
        else:
            line["prune_kernels_stress"] = _prune_stress(fa, torch, dec.model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.hidden)
        print(json.dumps(line))
        return

    dominant = "linear_swiglu"

    def run(pr, steps, outputs=None):
        o = outputs
        for _ in range(steps):
            o = dec.fastav_prefill(x, cu, spans, offs, pr, w.n_last, want_kv=True, outputs=o)
        return o

    def timed(pr, steps, warmup):
        """-> (wall seconds per step over exactly `steps` steps, per-step GPU times in ms from events on the
        launch stream)."""
        o = run(pr, warmup)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(steps):
            ev[i].record()
            o = dec.fastav_prefill(x, cu, spans, offs, pr, w.n_last, want_kv=True, outputs=o)
        ev[steps].record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t) / steps
        return wall, [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]

    fa.fastav_profile_reset()
    fa.fastav_profile_enable([dominant])              # events around the dominant kernel only, whole run
    s_pruned, per_pruned = timed(prunes, args.steps, args.warmup)
    s_plain, per_plain = timed([], args.steps, args.warmup)
    dom_ms, dom_n, dom_wk = fa.fastav_profile_collect(dominant)
    achieved = dom_wk / (dom_ms * 1e-3) / 1e12 if dom_ms > 0 else 0.0
    # the same steps once more with the event bracket off: what the bracket itself costs (not `value`)
    fa.fastav_profile_enable([])
    s_pruned_noev, _ = timed(prunes, args.steps, 1)

    # ---- per-kernel passes (not part of `value`): all kinds timed with events, pruned then unpruned
    kernels = {}
    if not args.no_kernel_passes:
        kinds = list(fa.PROF_KINDS)          # "other" = plain row copies: KV-cache writes and outputs
        fa.fastav_profile_enable(kinds)
        o = run(prunes, 1)
        torch.cuda.synchronize()
        base = {k: fa.fastav_profile_collect(k) for k in kinds}
        run(prunes, 3, o)
        torch.cuda.synchronize()
        after = {k: fa.fastav_profile_collect(k) for k in kinds}
        o2 = run([], 1)
        torch.cuda.synchronize()
        mid = {k: fa.fastav_profile_collect(k) for k in kinds}
        run([], 3, o2)
        torch.cuda.synchronize()
        for k in kinds:
            ms, n, wk = (after[k][i] - base[k][i] for i in range(3))
            if n == 0:
                continue
            flops = k.startswith("linear") or k == "attention"
            rate = wk / (ms * 1e-3) / (1e12 if flops else 1e9) if ms > 0 else 0.0
            kernels[k] = {"launches_per_step": n / 3, "ms_per_step": ms / 3, "us_per_launch": 1e3 * ms / n,
                          "achieved": rate, "unit": "TFLOP/s" if flops else "GB/s",
                          "frac": rate / (PEAK_BF16_TFLOPS if flops else PEAK_HBM_GBS)}
        prune_us = sum(kernels[k]["ms_per_step"] for k in ("score", "select", "gather") if k in kernels) * 1e3
    else:
        prune_us = None
    fa.fastav_profile_enable([])

    peak = by_shape = None
    if not args.no_kernel_passes:
        peak = _achievable_peak(fa, torch)
        by_shape = _by_shape(fa, torch, dec, m, cu, spans, offs, prunes, w.n_last)

    stress = None
    if not args.no_kernel_passes and m.dtype == "bf16":
        stress = _prune_stress(fa, torch, dec.model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.hidden)

    decode = None
    if not args.no_kernel_passes:
        decode = _decode_bench(fa, torch, dec, m, w, x, cu, spans, offs, prunes)

    rollout = None
    if not args.no_kernel_passes and m.dtype == "bf16" and len(w.samples) == 1 and w.prunes and tokens % 4 == 0:
        # the analysis behind the global prune (Eq. 2-3): rollout up to the global-prune layer, alpha 0.5
        upto = max(1, w.prunes[0].layer)
        dec.fastav_rollout(x, 0.5, upto)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        R = dec.fastav_rollout(x, 0.5, upto)
        torch.cuda.synchronize()
        rollout = {"layers": upto, "alpha": 0.5, "ms": (time.perf_counter() - t0) * 1e3,
                   "max_row_sum_error": float((R.sum(dim=1) - 1.0).abs().max())}
        del R

    cpu = None
    if not args.no_cpu_baseline:
        cpu = _cpu_baseline(w, host_threads)

    traffic, traffic_src = _recorded_traffic(args.workload)
    line = {
        "metric": "pruned prefill tokens/sec at 7B shape (unpruned rate, prune-step us and % roofline alongside)",
        "value": tokens / s_pruned, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": s_pruned * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": m.dtype, "data": "synthetic",
        "config": {"workload": w.name, "layers": m.n_layers, "hidden": m.hidden, "q_heads": m.n_q_heads,
                   "kv_heads": m.n_kv_heads, "head_dim": m.head_dim, "mlp": m.mlp_dim, "batch": len(w.samples),
                   "tokens": tokens, "prunes": [[p.layer, "global" if p.kind == fi.GLOBAL else "fine", p.keep_ratio] for p in w.prunes],
                   "kv_cache_written": True},
        "ms_per_step_median": float(np.median(per_pruned)), "ms_per_step_min": float(np.min(per_pruned)),
        "unpruned_tokens_per_s": tokens / s_plain, "unpruned_ms_per_step": s_plain * 1e3,
        "unpruned_ms_per_step_median": float(np.median(per_plain)), "unpruned_ms_per_step_min": float(np.min(per_plain)),
        "pruned_over_unpruned": s_plain / s_pruned,
        "prune_steps_us_per_prefill": prune_us,
        "roofline": {"kernel": "k_gemm_mfma16<SwiGLU> (gate/up projection)", "bound": "mfma", "achieved": achieved,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic, "traffic_source": traffic_src,
                     "launches": dom_n, "avg_launch_us": 1e3 * dom_ms / max(dom_n, 1),
                     # against what a loop of nothing but matrix instructions sustains on operands like the model's
                     "frac_of_achievable": (achieved / peak["mfma_bf16_normal_operands"]["achieved"]) if peak else None},
        "ms_per_step_without_kernel_events": s_pruned_noev * 1e3,
        "achievable_peak": peak,
        "kernels": kernels,
        "by_shape": by_shape,
        "prune_kernels_stress": stress,
        "decode_step": decode,
        "rollout": rollout,
        "cpu_baseline": cpu,
        "setup_s": setup_s,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
