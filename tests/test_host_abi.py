"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares, its schedule
helpers agree with the oracle's, and every argument error is reported before any GPU work (so these run on a
machine with no GPU)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import fastav_inputs as fi
from oracle import fastav_oracle as orc
import paper_2601_13143_amd as fa
from paper_2601_13143_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "fastav.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(fastav_[a-z_]+)\s*\(", header))
    assert {"fastav_prefill", "fastav_score", "fastav_select_gather"} <= names
    lib = fa.lib()
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in fastav.h but not exported"
    assert names == set(B._SIGS), "binding signatures and header declarations differ"


def test_keep_count_matches_oracle_rule():
    rng = np.random.default_rng(0)
    for _ in range(2000):
        n = int(rng.integers(1, 20000))
        r = float(rng.choice([0.5, 0.6, 0.7, 0.8, 0.3, 1.0, rng.uniform(0.01, 1.0)]))
        p = int(rng.integers(0, n + 1))
        assert fa.fastav_keep_count(n, r, p) == orc.keep_count(n, r, p)
    assert fa.fastav_keep_count(10, 0.0, 0) == -1 and fa.fastav_keep_count(10, 1.5, 0) == -1
    assert fa.fastav_keep_count(10, 0.5, 11) == -1 and fa.fastav_keep_count(-1, 0.5, 0) == -1


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_schedule_matches_oracle(cfg):
    w = fi.config(cfg)
    spans, offs = fi.span_table(w)
    prunes = [(p.layer, p.kind, p.keep_ratio) for p in w.prunes]
    tin, tout, fl = fa.fastav_schedule(fi.cu_seqlens(w), spans, offs, prunes, w.n_last, w.model.n_layers)
    want_in = np.zeros(w.model.n_layers, dtype=np.int64)
    finals = []
    for s in w.samples:
        n = sum(l for _, l in s)
        n_prot = int(orc.protected_mask(s, w.n_last).sum())
        counts = orc.token_schedule(n, n_prot, w.prunes, w.model.n_layers)
        want_in += np.asarray(counts)
        cur = counts[-1]
        for p in w.prunes:
            if p.layer == w.model.n_layers - 1 and p.kind == fi.FINE:
                cur = orc.keep_count(cur, p.keep_ratio, n_prot)
        finals.append(cur)
    assert tin.tolist() == want_in.tolist()
    assert fl.tolist() == finals
    # the ablation selectors of Tables 2-3 change which tokens go, never how many
    for sel_g, sel_f in [(fa.SEL_TOP_INFORMATIVE, fa.SEL_TOP_ATTENTIVE), (fa.SEL_RANDOM, fa.SEL_RANDOM)]:
        alt = [(p.layer, p.kind, p.keep_ratio, sel_g if p.kind == fi.GLOBAL else sel_f, 99) for p in w.prunes]
        tin2, tout2, fl2 = fa.fastav_schedule(fi.cu_seqlens(w), spans, offs, alt, w.n_last, w.model.n_layers)
        assert tin2.tolist() == tin.tolist() and tout2.tolist() == tout.tolist() and fl2.tolist() == fl.tolist()
    assert tout[-1] == sum(finals) and (tout <= tin).all() and (tout[:-1] >= tin[1:]).all()
    if cfg == 3:
        assert tin[0] == 4096 and tin[14] == 2458 and tin[21] == 1721 and tin[27] == 1205 and tout[20] == 1721


def test_schedule_n_last_counts_non_text_tail_once():
    # last 3 positions: one audio + two text -> protected = 4 text + 1 audio
    cu = [0, 20]
    spans = [(0, 2, fi.TEXT), (2, 10, fi.VIDEO), (12, 6, fi.AUDIO), (18, 2, fi.TEXT)]
    _, _, fl = fa.fastav_schedule(cu, spans, [0, 4], [(0, fi.FINE, 0.05)], 3, 1)
    assert fl.tolist() == [5]
    assert int(orc.protected_mask([(fi.TEXT, 2), (fi.VIDEO, 10), (fi.AUDIO, 6), (fi.TEXT, 2)], 3).sum()) == 5


def _expect(status, fn, *a, **k):
    with pytest.raises(fa.FastavError) as e:
        fn(*a, **k)
    assert e.value.status == status, str(e.value)
    assert len(str(e.value)) > 20


def test_batch_and_prune_validation():
    ok_spans, ok_off = [(0, 4, fi.VIDEO), (4, 4, fi.TEXT)], [0, 2]
    sched = fa.fastav_schedule
    _expect(B.EINVAL, sched, [1, 8], ok_spans, ok_off, [], 1, 2)                          # cu[0] != 0
    _expect(B.EINVAL, sched, [0, 0], ok_spans, ok_off, [], 1, 2)                          # empty sample
    _expect(B.EINVAL, sched, [0, 9], ok_spans, ok_off, [], 1, 2)                          # spans do not cover
    _expect(B.EINVAL, sched, [0, 8], [(0, 4, 1), (5, 3, 0)], ok_off, [], 1, 2)            # gap
    _expect(B.EINVAL, sched, [0, 8], [(0, 4, 7), (4, 4, 0)], ok_off, [], 1, 2)            # bad modality
    _expect(B.EINVAL, sched, [0, 8], ok_spans, ok_off, [(2, fi.FINE, 0.5)], 1, 2)         # layer out of range
    _expect(B.EINVAL, sched, [0, 8], ok_spans, ok_off, [(1, fi.FINE, 0.0)], 1, 2)         # ratio 0
    _expect(B.EINVAL, sched, [0, 8], ok_spans, ok_off, [(1, fi.FINE, 1.5)], 1, 2)
    _expect(B.EINVAL, sched, [0, 8], ok_spans, ok_off, [(1, 3, 0.5)], 1, 2)               # bad kind
    _expect(B.EINVAL, sched, [0, 8], ok_spans, ok_off, [(1, fi.FINE, 0.5), (0, fi.FINE, 0.5)], 1, 2)   # unsorted
    _expect(B.EINVAL, sched, [0, 8], ok_spans, ok_off, [(1, fi.FINE, 0.5), (1, fi.FINE, 0.5)], 1, 2)   # duplicate
    _expect(B.EINVAL, sched, [0, 8], ok_spans, ok_off, [(1, fi.FINE, 0.5), (1, fi.GLOBAL, 0.5)], 1, 2)  # global after fine
    _expect(B.EINVAL, sched, [0, 8], ok_spans, ok_off, [(1, fi.FINE, 0.5, 6)], 1, 2)      # selector out of range
    _expect(B.EINVAL, sched, [0, 8], ok_spans, ok_off, [(1, fi.FINE, 0.5, -1)], 1, 2)
    _expect(B.EINVAL, sched, [0, 8], ok_spans, ok_off, [(1, fi.GLOBAL, 0.5, fa.SEL_TOP_ATTENTIVE)], 1, 2)    # no attention yet
    _expect(B.EINVAL, sched, [0, 8], ok_spans, ok_off, [(1, fi.GLOBAL, 0.5, fa.SEL_LOW_ATTENTIVE)], 1, 2)
    _expect(B.EINVAL, sched, [0, 8], ok_spans, ok_off, [(1, fi.FINE, 0.5, fa.SEL_TOP_INFORMATIVE)], 1, 2)    # positional on FINE
    _expect(B.EINVAL, sched, [0, 8], ok_spans, ok_off, [], 0, 2)                          # n_last < 1
    _expect(B.EINVAL, sched, [0, 8], ok_spans, ok_off, [], B.MAX_N_LAST + 1, 2)
    tin, tout, fl = sched([0, 8], ok_spans, ok_off, [(1, fi.GLOBAL, 0.5), (1, fi.FINE, 0.75)], 1, 2)
    assert tin.tolist() == [8, 4] and tout.tolist() == [8, 4] and fl.tolist() == [4]       # text (4) is the floor


def test_model_validation_and_handle_errors():
    lib = fa.lib()
    h = C.c_void_p()
    for bad in [fa.make_model(0, 64, 4, 2, 64, 64), fa.make_model(1, 64, 4, 3, 64, 64), fa.make_model(1, 64, 4, 2, 64, 64, dtype=5),
                fa.make_model(1, 64, 4, 2, 64, 64, rope_base=1.0)]:
        assert lib.fastav_create(C.byref(bad), C.byref(h)) == B.EINVAL and not h.value
    assert lib.fastav_create(C.byref(fa.make_model(1, 64, 4, 2, 96, 64)), C.byref(h)) == B.EUNSUPPORTED
    assert b"head_dim" in lib.fastav_last_error()
    assert lib.fastav_create(None, C.byref(h)) == B.EINVAL
    dec = fa.Decoder(fa.make_model(2, 64, 4, 2, 64, 96, dtype=B.F32))
    assert dec.fastav_workspace_bytes(100, 2) > 100 * 64 * 4 * 2
    _expect(B.EINVAL, dec.fastav_workspace_bytes, 0, 1)
    lw = B.LayerWeights(*([16] * 9))
    assert lib.fastav_set_weights(dec._h, 2, C.byref(lw)) == B.EINVAL                      # layer out of range
    lw0 = B.LayerWeights(*([16] * 8 + [None]))
    assert lib.fastav_set_weights(dec._h, 0, C.byref(lw0)) == B.EINVAL                     # NULL weight
    lw1 = B.LayerWeights(*([16] * 8 + [24]))
    assert lib.fastav_set_weights(dec._h, 0, C.byref(lw1)) == B.EINVAL                     # misaligned
    assert lib.fastav_set_weights(dec._h, 0, C.byref(lw)) == B.OK


def test_prefill_rejects_bad_arguments_before_any_launch():
    """Fake (never dereferenced) device addresses: every one of these must fail on the host."""
    lib = fa.lib()
    m = fa.make_model(2, 64, 4, 2, 64, 96, dtype=B.F32)
    dec = fa.Decoder(m)
    hb = B._HostBatch(4096, [0, 8], [(0, 4, fi.VIDEO), (4, 4, fi.TEXT)], [0, 2])
    out = B.PrefillOut(4096, 4096, 4096, None, None, None, None)
    pr = B._prune_array([(1, fi.FINE, 0.5)])
    ws_need = dec.fastav_workspace_bytes(8, 1)

    def call(h=dec._h, batch=hb.c, prunes=pr, n_prunes=1, n_last=1, ws=4096, ws_bytes=ws_need, o=out):
        return lib.fastav_prefill(h, C.byref(batch) if batch is not None else None, prunes, n_prunes, n_last, ws, ws_bytes,
                                  C.byref(o) if o is not None else None, None)

    assert call() == B.EINVAL and b"never set" in lib.fastav_last_error()                  # weights missing
    lw = B.LayerWeights(*([16] * 9))
    for l in range(2):
        assert lib.fastav_set_weights(dec._h, l, C.byref(lw)) == B.OK
    assert call(h=None) == B.EINVAL
    assert call(batch=None) == B.EINVAL
    assert call(o=None) == B.EINVAL
    assert call(o=B.PrefillOut(None, 4096, 4096, None, None, None, None)) == B.EINVAL
    assert call(ws=None) == B.EINVAL
    assert call(ws=4100) == B.EINVAL                                                        # misaligned workspace
    assert call(ws_bytes=ws_need - 1) == B.EWORKSPACE and b"needed" in lib.fastav_last_error()
    assert call(n_last=0) == B.EINVAL
    assert call(n_prunes=B.MAX_PRUNES + 1) == B.EINVAL
    hb2 = B._HostBatch(None, [0, 8], [(0, 4, fi.VIDEO), (4, 4, fi.TEXT)], [0, 2])
    assert call(batch=hb2.c) == B.EINVAL                                                    # x NULL
    kv_bad = (C.c_void_p * 4)(4096, 4096, 4096 + 8, 4096)                                   # a cache pointer off a 16-byte boundary
    assert call(o=B.PrefillOut(4096, 4096, 4096, kv_bad, None, None, None)) == B.EINVAL and b"kv_out[2]" in lib.fastav_last_error()


def test_score_and_select_reject_bad_arguments():
    lib = fa.lib()
    m = fa.make_model(1, 64, 4, 2, 64, 96, dtype=B.BF16)
    need = lib.fastav_score_workspace_bytes(4, 100, 1, 1)
    assert need >= 4 * 100 * 4
    f = lambda **k: lib.fastav_score(C.byref(m), k.get("q", 4096), k.get("qs", 256), k.get("k", 4096), k.get("ks", 128),
                                     k.get("cu", 4096), 1, 100, k.get("maxlen", 100), k.get("n_last", 1), 4096,
                                     k.get("ws", 4096), k.get("wsb", need), None)
    assert f(q=None) == B.EINVAL and f(qs=100) == B.EINVAL and f(ks=4) == B.EINVAL
    assert f(n_last=9) == B.EINVAL and f(maxlen=101) == B.EINVAL and f(wsb=need - 1) == B.EWORKSPACE
    assert f(q=4098) == B.EINVAL                                                            # misaligned q
    # the entry point without a workspace: what does not fit its built-in scratch is refused on the host
    big = 80000
    assert lib.fastav_score_workspace_bytes(4, big * 8, 1, 1) > B.SCORE_STATIC_BYTES
    assert lib.fastav_score_static(C.byref(m), 4096, 256, 4096, 128, 4096, 1, big * 8, big * 8, 1, 4096, None) == B.EWORKSPACE
    assert b"built-in buffer" in lib.fastav_last_error()
    assert lib.fastav_score_static(C.byref(m), 4096, 256, 4096, 128, 4096, 1, 100, 100, 9, 4096, None) == B.EINVAL
    cu = np.array([0, 10, 30], dtype=np.int32)
    kc = np.array([5, 25], dtype=np.int32)
    ip = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    g = lambda **k: lib.fastav_select_gather(4096, k.get("prot", 4096), ip(k.get("cu", cu)), ip(k.get("kc", kc)), 2, k.get("nt", 0),
                                             None, None, None, 4096, 4096, 4096, k.get("wsb", 256), None)
    assert g(prot=None) == B.EINVAL
    assert g(kc=np.array([5, 25], dtype=np.int32)) == B.EINVAL and b"exceeds" in lib.fastav_last_error()   # 25 > 20 rows
    assert g(kc=np.array([-1, 2], dtype=np.int32)) == B.EINVAL
    assert g(cu=np.array([0, 10, 5], dtype=np.int32)) == B.EINVAL
    assert g(nt=9) == B.EINVAL and g(nt=1) == B.EINVAL and g(wsb=4, kc=np.array([5, 15], dtype=np.int32)) == B.EWORKSPACE


@pytest.mark.parametrize("cfg", [1, 3, 5])
def test_schedule_lens_matches_oracle_cache_rows(cfg):
    """Rows per sample of every layer's K/V cache (what a decode step needs) equal the oracle's token schedule."""
    w = fi.config(cfg)
    spans, offs = fi.span_table(w)
    prunes = [(p.layer, p.kind, p.keep_ratio) for p in w.prunes]
    lens = fa.fastav_schedule_lens(fi.cu_seqlens(w), spans, offs, prunes, w.n_last, w.model.n_layers)
    assert lens.shape == (w.model.n_layers, len(w.samples))
    for b, s in enumerate(w.samples):
        n = sum(l for _, l in s)
        n_prot = int(orc.protected_mask(s, w.n_last).sum())
        cur, want = n, []
        for l in range(w.model.n_layers):
            for p in sorted([p for p in w.prunes if p.layer == l], key=lambda p: p.kind):
                cur = orc.keep_count(cur, p.keep_ratio, n_prot)
            want.append(cur)                                         # tokens that leave layer l
        assert lens[:, b].tolist() == want
    _, tout, _ = fa.fastav_schedule(fi.cu_seqlens(w), spans, offs, prunes, w.n_last, w.model.n_layers)
    assert lens.sum(axis=1).tolist() == tout.tolist()


def test_decode_step_rejects_bad_arguments_before_any_launch():
    lib = fa.lib()
    h = C.c_void_p()
    assert lib.fastav_create(C.byref(fa.make_model(2, 256, 4, 2, 64, 256)), C.byref(h)) == B.OK
    need = C.c_size_t()
    assert lib.fastav_decode_workspace_bytes(h, 4, C.byref(need)) == B.OK and need.value > 0 and need.value % 256 == 0
    assert lib.fastav_decode_workspace_bytes(h, 0, C.byref(need)) == B.EINVAL
    assert lib.fastav_decode_workspace_bytes(h, 17, C.byref(need)) == B.EINVAL
    assert lib.fastav_decode_workspace_bytes(None, 4, C.byref(need)) == B.EINVAL
    di = B.DecodeIn()
    assert lib.fastav_decode_step(None, C.byref(di), None, None, 0, None) == B.EINVAL
    assert lib.fastav_decode_step(h, None, None, None, 0, None) == B.EINVAL
    fake = C.c_void_p(4096)
    di.batch = 0
    assert lib.fastav_decode_step(h, C.byref(di), fake, fake, 1 << 20, None) == B.EINVAL     # batch out of range
    di.batch = 2
    assert lib.fastav_decode_step(h, C.byref(di), fake, fake, 1 << 20, None) == B.EINVAL     # NULL inputs
    assert b"must be non-NULL" in lib.fastav_last_error()
    f32 = C.c_void_p()
    assert lib.fastav_create(C.byref(fa.make_model(1, 256, 4, 2, 64, 256, dtype=fa.F32)), C.byref(f32)) == B.OK
    assert lib.fastav_decode_step(f32, C.byref(di), fake, fake, 1 << 20, None) == B.EUNSUPPORTED   # fp32 model
    lib.fastav_destroy(h)
    lib.fastav_destroy(f32)


def test_probes_and_options_reject_bad_arguments():
    """The measurement aids validate on the host like every other entry point (no launch happens here)."""
    lib = fa.lib()
    fl = C.c_double()
    assert lib.fastav_probe_mfma(0, None, 4096, C.byref(fl), None) == B.EINVAL            # iters < 1
    assert lib.fastav_probe_mfma(10, None, None, C.byref(fl), None) == B.EINVAL           # no sink
    assert lib.fastav_probe_mfma(10, 4096 + 8, 4096, C.byref(fl), None) == B.EINVAL       # operands off a 16-byte boundary
    assert b"operands" in lib.fastav_last_error()
    assert lib.fastav_probe_read(None, 1 << 20, 4096, None) == B.EINVAL
    assert lib.fastav_probe_read(4096, 1024, 4096, None) == B.EINVAL                        # under 16 KB
    assert lib.fastav_probe_read(4096 + 4, 1 << 20, 4096, None) == B.EINVAL                 # misaligned
    assert lib.fastav_set_option(-1, 1) == B.EINVAL and lib.fastav_set_option(4, 1) == B.EINVAL
    for opt in (B.OPT_FUSED_SCORE_SELECT, B.OPT_FUSED_ROPE, B.OPT_FUSED_SPLITK_NORM, B.OPT_FUSED_GATHER_OPROJ):
        assert lib.fastav_set_option(opt, 0) == B.OK and lib.fastav_set_option(opt, 1) == B.OK

