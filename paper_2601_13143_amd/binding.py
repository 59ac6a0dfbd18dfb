"""ctypes binding of libfastav.so: argument marshalling only — every step of the path runs in the HIP
kernels behind the C ABI declared in include/fastav.h.  PyTorch supplies device memory and streams.

There is no fallback: if the shared library has not been built this module raises on import of the
library handle (``lib()``), and nothing here computes on the CPU.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
# FASTAV_LIBRARY selects another build of the same library (e.g. the host-sanitized one the CPU tests make)
LIB_PATH = os.environ.get("FASTAV_LIBRARY") or os.path.join(HERE, "libfastav.so")

OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP = 0, 1, 2, 3, 4
TEXT, VIDEO, AUDIO = 0, 1, 2
GLOBAL, FINE = 0, 1
SEL_DEFAULT, SEL_LOW_ATTENTIVE, SEL_TOP_ATTENTIVE, SEL_LOW_INFORMATIVE, SEL_TOP_INFORMATIVE, SEL_RANDOM = range(6)
BF16, F32 = 0, 1
EPI_STORE, EPI_RESADD, EPI_SWIGLU = 0, 1, 2
MAX_N_LAST, MAX_PRUNES, MAX_GATHER_TENSORS = 8, 128, 8


class FastavError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"fastav status {status}: {msg}")
        self.status = status


class Span(C.Structure):
    _fields_ = [("start", C.c_int32), ("len", C.c_int32), ("modality", C.c_int32)]


class Prune(C.Structure):
    _fields_ = [("layer", C.c_int32), ("kind", C.c_int32), ("keep_ratio", C.c_double), ("selector", C.c_int32),
                ("seed", C.c_uint32)]


class Model(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("mlp_dim", C.c_int32), ("rope_base", C.c_float), ("rms_eps", C.c_float),
                ("dtype", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("g_attn", "wq", "wk", "wv", "wo", "g_mlp", "w_gate", "w_up", "w_down")]


class Batch(C.Structure):
    _fields_ = [("x", C.c_void_p), ("cu_seqlens", C.POINTER(C.c_int32)), ("batch", C.c_int32),
                ("spans", C.POINTER(Span)), ("span_offsets", C.POINTER(C.c_int32))]


class PrefillOut(C.Structure):
    _fields_ = [("x_out", C.c_void_p), ("cu_seqlens_out", C.c_void_p), ("kept_pos_out", C.c_void_p),
                ("kv_out", C.POINTER(C.c_void_p)), ("prune_scores_out", C.POINTER(C.c_void_p)),
                ("prune_keep_idx_out", C.POINTER(C.c_void_p)), ("layer_x_out", C.POINTER(C.c_void_p))]


_lib = None

class DecodeIn(C.Structure):
    _fields_ = [("batch", C.c_int32), ("x_new", C.c_void_p), ("pos_new", C.c_void_p),
                ("k_prefix", C.POINTER(C.c_void_p)), ("v_prefix", C.POINTER(C.c_void_p)),
                ("cu_prefix", C.POINTER(C.c_void_p)), ("max_prefix", C.POINTER(C.c_int32)),
                ("k_gen", C.POINTER(C.c_void_p)), ("v_gen", C.POINTER(C.c_void_p)),
                ("gen_len", C.c_int32), ("gen_cap", C.c_int32)]


_SIGS = {
    "fastav_last_error": (C.c_char_p, []),
    "fastav_set_option": (C.c_int, [C.c_int32, C.c_int32]),
    "fastav_keep_count": (C.c_int64, [C.c_int64, C.c_double, C.c_int64]),
    "fastav_schedule": (C.c_int, [C.POINTER(Batch), C.POINTER(Prune), C.c_int32, C.c_int32, C.c_int32,
                                  C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int32)]),
    "fastav_schedule_lens": (C.c_int, [C.POINTER(Batch), C.POINTER(Prune), C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]),
    "fastav_decode_workspace_bytes": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_size_t)]),
    "fastav_decode_step": (C.c_int, [C.c_void_p, C.POINTER(DecodeIn), C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "fastav_attention_map_workspace_bytes": (C.c_size_t, [C.c_int32, C.c_int32]),
    "fastav_attention_map": (C.c_int, [C.POINTER(Model), C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p,
                                       C.c_void_p, C.c_size_t, C.c_void_p]),
    "fastav_rollout_workspace_bytes": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_size_t)]),
    "fastav_rollout": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t,
                                 C.c_void_p]),
    "fastav_rollout_cutoff": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]),
    "fastav_create": (C.c_int, [C.POINTER(Model), C.POINTER(C.c_void_p)]),
    "fastav_destroy": (None, [C.c_void_p]),
    "fastav_set_weights": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(LayerWeights)]),
    "fastav_workspace_bytes": (C.c_int, [C.c_void_p, C.c_int64, C.c_int32, C.POINTER(C.c_size_t)]),
    "fastav_prefill": (C.c_int, [C.c_void_p, C.POINTER(Batch), C.POINTER(Prune), C.c_int32, C.c_int32, C.c_void_p,
                                 C.c_size_t, C.POINTER(PrefillOut), C.c_void_p]),
    "fastav_score_workspace_bytes": (C.c_size_t, [C.c_int32, C.c_int64, C.c_int32, C.c_int32]),
    "fastav_score": (C.c_int, [C.POINTER(Model), C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32,
                               C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "fastav_score_static": (C.c_int, [C.POINTER(Model), C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32,
                                      C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "fastav_select_workspace_bytes": (C.c_size_t, [C.c_int32]),
    "fastav_select_gather": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int32,
                                       C.c_int32, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_int64),
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "fastav_rmsnorm": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_float, C.c_int32, C.c_void_p]),
    "fastav_rope": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_float, C.c_int32, C.c_void_p]),
    "fastav_linear_workspace_bytes": (C.c_size_t, []),
    "fastav_linear": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32,
                                C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]),
    "fastav_attention": (C.c_int, [C.POINTER(Model), C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                   C.c_int64, C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "fastav_profile_enable": (C.c_int, [C.c_uint32]),
    "fastav_profile_collect": (C.c_int, [C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_double)]),
    "fastav_profile_reset": (C.c_int, []),
    "fastav_probe_mfma": (C.c_int, [C.c_int32, C.c_void_p, C.c_void_p, C.POINTER(C.c_double), C.c_void_p]),
    "fastav_probe_read": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]),
}

PROF_KINDS = {"linear_store": 0, "linear_resadd": 1, "linear_swiglu": 2, "attention": 3, "score": 4, "select": 5,
              "gather": 6, "rmsnorm": 7, "rope": 8, "other": 9}


def lib() -> C.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built (there is no CPU fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2601_13143_amd.build` "
                                    "(or __graft_entry__.build()); the HIP library is the only implementation")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def _check(st: int) -> None:
    if st != OK:
        raise FastavError(st, lib().fastav_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError("tensors must be bfloat16 or float32")


def make_model(n_layers, hidden, n_q_heads, n_kv_heads, head_dim, mlp_dim, rope_base=1e4, rms_eps=1e-6, dtype=BF16) -> Model:
    return Model(n_layers, hidden, n_q_heads, n_kv_heads, head_dim, mlp_dim, rope_base, rms_eps, dtype)


def _prune_array(prunes: Sequence) -> "C.Array":
    arr = (Prune * max(1, len(prunes)))()
    for i, p in enumerate(prunes):
        arr[i] = Prune(int(p[0]), int(p[1]), float(p[2]), int(p[3]) if len(p) > 3 else 0, int(p[4]) if len(p) > 4 else 0)
    return arr


class _HostBatch:
    """Keeps the host arrays of a fastav_batch_t alive."""

    def __init__(self, x_ptr, cu_seqlens, spans, span_offsets):
        self.cu = _i32(cu_seqlens)
        self.spans_np = _i32(spans).reshape(-1, 3)
        self.off = _i32(span_offsets)
        self.spans = (Span * max(1, len(self.spans_np)))()
        for i, (s, l, m) in enumerate(self.spans_np):
            self.spans[i] = Span(int(s), int(l), int(m))
        self.c = Batch(x_ptr, self.cu.ctypes.data_as(C.POINTER(C.c_int32)), len(self.cu) - 1, self.spans,
                       self.off.ctypes.data_as(C.POINTER(C.c_int32)))


def fastav_keep_count(n: int, keep_ratio: float, n_protected: int) -> int:
    return int(lib().fastav_keep_count(n, keep_ratio, n_protected))


def fastav_schedule(cu_seqlens, spans, span_offsets, prunes: Sequence, n_last: int, n_layers: int):
    """-> (tokens_in [n_layers], tokens_out [n_layers], final_lens [batch]) as numpy arrays."""
    hb = _HostBatch(None, cu_seqlens, spans, span_offsets)
    tin = np.zeros(max(1, n_layers), dtype=np.int64)
    tout = np.zeros(max(1, n_layers), dtype=np.int64)
    fl = np.zeros(hb.c.batch if hb.c.batch > 0 else 1, dtype=np.int32)
    _check(lib().fastav_schedule(C.byref(hb.c), _prune_array(prunes), len(prunes), n_last, n_layers,
                                 tin.ctypes.data_as(C.POINTER(C.c_int64)), tout.ctypes.data_as(C.POINTER(C.c_int64)),
                                 fl.ctypes.data_as(C.POINTER(C.c_int32))))
    return tin[:n_layers], tout[:n_layers], fl


def fastav_schedule_lens(cu_seqlens, spans, span_offsets, prunes: Sequence, n_last: int, n_layers: int) -> np.ndarray:
    """-> int32 [n_layers, batch]: tokens of each sample that leave each layer (rows per sample of its K/V cache)."""
    hb = _HostBatch(None, cu_seqlens, spans, span_offsets)
    out = np.zeros((n_layers, hb.c.batch), dtype=np.int32)
    _check(lib().fastav_schedule_lens(C.byref(hb.c), _prune_array(prunes), len(prunes), n_last, n_layers,
                                      out.ctypes.data_as(C.POINTER(C.c_int32))))
    return out


class Decoder:
    """Owns a fastav handle, the device weights handed to it and a reusable workspace tensor."""

    def __init__(self, model: Model):
        self.model = model
        self._h = C.c_void_p()
        _check(lib().fastav_create(C.byref(model), C.byref(self._h)))
        self._weights: Dict[int, Dict[str, torch.Tensor]] = {}
        self._ws: Optional[torch.Tensor] = None

    def __del__(self):
        if getattr(self, "_h", None) and self._h.value and _lib is not None:
            _lib.fastav_destroy(self._h)
            self._h = C.c_void_p()

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.model.dtype == BF16 else torch.float32

    def fastav_set_weights(self, layer: int, weights: Dict[str, torch.Tensor]) -> None:
        """weights: name -> device tensor in the model dtype ([out, in] matrices); kept alive by the decoder."""
        w = {k: v.contiguous() for k, v in weights.items()}
        lw = LayerWeights(*[w[n].data_ptr() for n, _ in LayerWeights._fields_])
        _check(lib().fastav_set_weights(self._h, layer, C.byref(lw)))
        self._weights[layer] = w

    def fastav_workspace_bytes(self, max_total_tokens: int, max_batch: int) -> int:
        out = C.c_size_t()
        _check(lib().fastav_workspace_bytes(self._h, max_total_tokens, max_batch, C.byref(out)))
        return out.value

    def workspace(self, total_tokens: int, batch: int) -> torch.Tensor:
        need = self.fastav_workspace_bytes(total_tokens, batch)
        if self._ws is None or self._ws.numel() < need:
            self._ws = None
            self._ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        return self._ws

    def fastav_prefill(self, x: torch.Tensor, cu_seqlens, spans, span_offsets, prunes: Sequence, n_last: int = 1,
                       want_kv: bool = False, want_trace: bool = False, want_layers: bool = False,
                       outputs: Optional[Dict] = None) -> Dict:
        """Runs fastav_prefill on the current stream.  ``prunes``: sequence of (layer, kind, keep_ratio[, selector
        [, seed]]).
        Output tensors are allocated here (or reused from ``outputs``, the dict a previous call returned)."""
        m = self.model
        hb = _HostBatch(x.data_ptr(), cu_seqlens, spans, span_offsets)
        B, T0 = hb.c.batch, int(hb.cu[-1])
        if x.dtype != self.torch_dtype or not x.is_contiguous() or tuple(x.shape) != (T0, m.hidden):
            raise ValueError("x must be a contiguous [total_tokens, hidden] tensor in the model dtype")
        tin, tout, fl = fastav_schedule(hb.cu, hb.spans_np, hb.off, prunes, n_last, m.n_layers)
        Tf = int(fl.sum())
        dev = x.device
        o = outputs if outputs is not None else {}
        if outputs is None:
            o["x_out"] = torch.empty((Tf, m.hidden), dtype=torch.float32, device=dev)
            o["cu_seqlens_out"] = torch.empty(B + 1, dtype=torch.int32, device=dev)
            o["kept_pos"] = torch.empty(Tf, dtype=torch.int32, device=dev)
            if want_kv:
                kd = (m.n_kv_heads, m.head_dim)
                o["kv"] = [(torch.empty((int(tout[l]),) + kd, dtype=self.torch_dtype, device=dev),
                            torch.empty((int(tout[l]),) + kd, dtype=self.torch_dtype, device=dev)) for l in range(m.n_layers)]
            if want_trace:
                # packed tokens entering prune i = survivors of the schedule truncated to its first i prunes
                stage_tot = [int(fastav_schedule(hb.cu, hb.spans_np, hb.off, prunes[:i], n_last, m.n_layers)[2].sum())
                             for i in range(len(prunes) + 1)]
                o["prune_scores"] = [torch.zeros(stage_tot[i], dtype=torch.float32, device=dev) if p[1] == FINE else None
                                     for i, p in enumerate(prunes)]
                o["prune_keep_idx"] = [torch.empty(stage_tot[i + 1], dtype=torch.int32, device=dev) for i in range(len(prunes))]
            if want_layers:
                o["layer_x"] = [torch.empty((int(tout[l]), m.hidden), dtype=torch.float32, device=dev) for l in range(m.n_layers)]
        po = PrefillOut(o["x_out"].data_ptr(), o["cu_seqlens_out"].data_ptr(), o["kept_pos"].data_ptr(), None, None, None, None)
        keep = []
        if "kv" in o:
            arr = (C.c_void_p * (2 * m.n_layers))(*[t.data_ptr() for kv in o["kv"] for t in kv])
            po.kv_out = arr; keep.append(arr)
        if "prune_scores" in o:
            a1 = (C.c_void_p * max(1, len(prunes)))(*[_ptr(t) for t in o["prune_scores"]])
            a2 = (C.c_void_p * max(1, len(prunes)))(*[_ptr(t) for t in o["prune_keep_idx"]])
            po.prune_scores_out, po.prune_keep_idx_out = a1, a2; keep += [a1, a2]
        if "layer_x" in o:
            a3 = (C.c_void_p * m.n_layers)(*[t.data_ptr() for t in o["layer_x"]])
            po.layer_x_out = a3; keep.append(a3)
        ws = self.workspace(T0, B)
        _check(lib().fastav_prefill(self._h, C.byref(hb.c), _prune_array(prunes), len(prunes), n_last, ws.data_ptr(),
                                    ws.numel(), C.byref(po), _stream()))
        o["tokens_in"], o["tokens_out"], o["final_lens"] = tin, tout, fl
        return o


    def fastav_decode_step(self, x_new: torch.Tensor, pos_new: torch.Tensor, kv: Sequence, lens: np.ndarray,
                           gen: Optional[Sequence] = None, gen_len: int = 0, state: Optional[Dict] = None) -> Dict:
        """One decode step on the current stream.  ``kv``: per layer (K, V) device tensors [T_l, Hkv, dh] as
        fastav_prefill returned them; ``lens``: int32 [n_layers, batch] rows per sample of every layer's cache
        (fastav_schedule_lens); ``gen``: per layer (K, V) tensors [batch, gen_cap, Hkv, dh] holding ``gen_len``
        generated tokens, slot gen_len is written.  -> {"x_out": fp32 [batch, hidden], "state": reusable}."""
        m = self.model
        B = x_new.shape[0]
        if x_new.dtype != self.torch_dtype or not x_new.is_contiguous() or tuple(x_new.shape) != (B, m.hidden):
            raise ValueError("x_new must be a contiguous [batch, hidden] tensor in the model dtype")
        st = state if state is not None else {}
        if "cu" not in st:                                   # per-layer prefix sums of the cache rows, on the device
            lens = np.asarray(lens, dtype=np.int32).reshape(m.n_layers, B)
            cu = np.zeros((m.n_layers, B + 1), dtype=np.int32)
            cu[:, 1:] = np.cumsum(lens, axis=1)
            st["cu"] = torch.from_numpy(cu).to(x_new.device)
            st["max_prefix"] = np.ascontiguousarray(lens.max(axis=1).astype(np.int32))
            st["x_out"] = torch.empty((B, m.hidden), dtype=torch.float32, device=x_new.device)
            need = C.c_size_t()
            _check(lib().fastav_decode_workspace_bytes(self._h, B, C.byref(need)))
            st["ws"] = torch.empty(need.value, dtype=torch.uint8, device=x_new.device)
        L = m.n_layers
        kp = (C.c_void_p * L)(*[kv[l][0].data_ptr() for l in range(L)])
        vp = (C.c_void_p * L)(*[kv[l][1].data_ptr() for l in range(L)])
        cup = (C.c_void_p * L)(*[st["cu"][l].data_ptr() for l in range(L)])
        kg = vg = None
        gen_cap = 0
        if gen is not None:
            kg = (C.c_void_p * L)(*[gen[l][0].data_ptr() for l in range(L)])
            vg = (C.c_void_p * L)(*[gen[l][1].data_ptr() for l in range(L)])
            gen_cap = gen[0][0].shape[1]
        di = DecodeIn(B, x_new.data_ptr(), pos_new.data_ptr(), kp, vp, cup,
                      st["max_prefix"].ctypes.data_as(C.POINTER(C.c_int32)), kg, vg, gen_len, gen_cap)
        _check(lib().fastav_decode_step(self._h, C.byref(di), st["x_out"].data_ptr(), st["ws"].data_ptr(), st["ws"].numel(), _stream()))
        return {"x_out": st["x_out"], "state": st}


    def fastav_rollout(self, x: torch.Tensor, alpha: float, upto_layers: Optional[int] = None) -> torch.Tensor:
        """Eq. 3 for one sample x [n, hidden] through the first ``upto_layers`` layers of the unpruned decoder.
        -> fp32 [n, n] view of R^l (the library writes its transpose; the view flips it back)."""
        m = self.model
        n = x.shape[0]
        L = m.n_layers if upto_layers is None else upto_layers
        if x.dtype != self.torch_dtype or not x.is_contiguous() or x.shape[1] != m.hidden:
            raise ValueError("x must be a contiguous [n, hidden] tensor in the model dtype")
        need = C.c_size_t()
        _check(lib().fastav_rollout_workspace_bytes(self._h, n, C.byref(need)))
        ws = torch.empty(need.value, dtype=torch.uint8, device=x.device)
        rt = torch.empty((n, n), dtype=torch.float32, device=x.device)
        _check(lib().fastav_rollout(self._h, x.data_ptr(), n, alpha, L, rt.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
        return rt.t()


def fastav_rollout_cutoff(r: torch.Tensor, protected_mask: torch.Tensor, threshold: float):
    """``r``: the fp32 [n, n] view fastav_rollout returned (or any tensor whose transpose is contiguous);
    ``protected_mask``: uint8 [n] on the device.  -> (influence fp32 [n], cutoff int32 [1]), both on the device."""
    rt = r.t()
    n = rt.shape[0]
    if rt.dtype != torch.float32 or not rt.is_contiguous() or rt.shape[1] != n:
        raise ValueError("r must be the transposed view of a contiguous fp32 [n, n] tensor")
    if protected_mask.dtype != torch.uint8 or protected_mask.numel() != n or not protected_mask.is_contiguous():
        raise ValueError("protected_mask must be a contiguous uint8 [n] tensor")
    infl = torch.empty(n, dtype=torch.float32, device=rt.device)
    cut = torch.empty(1, dtype=torch.int32, device=rt.device)
    _check(lib().fastav_rollout_cutoff(rt.data_ptr(), n, protected_mask.data_ptr(), threshold, infl.data_ptr(),
                                       cut.data_ptr(), _stream()))
    return infl, cut


def fastav_attention_map(model: Model, q: torch.Tensor, k: torch.Tensor) -> torch.Tensor:
    """q [n, Hq, dh], k [n, Hkv, dh] (bf16, post-RoPE, one sample; views with a row stride are fine)
    -> bf16 [n, n] head-mean causal attention map."""
    n = q.shape[0]
    a = torch.empty((n, n), dtype=torch.bfloat16, device=q.device)
    need = lib().fastav_attention_map_workspace_bytes(n, model.n_q_heads)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    _check(lib().fastav_attention_map(C.byref(model), q.data_ptr(), q.stride(0), k.data_ptr(), k.stride(0), n, a.data_ptr(),
                                      ws.data_ptr(), ws.numel(), _stream()))
    return a


def fastav_score(model: Model, q: torch.Tensor, k: torch.Tensor, cu_seqlens_dev: torch.Tensor, max_seqlen: int,
                 n_last: int = 1, q_row_stride: Optional[int] = None, k_row_stride: Optional[int] = None) -> torch.Tensor:
    """q [T, Hq, dh], k [T, Hkv, dh] (or 2-D views with explicit row strides) -> fp32 scores [T]."""
    T = q.shape[0]
    B = cu_seqlens_dev.numel() - 1
    qs = q_row_stride if q_row_stride is not None else q.stride(0)
    ks = k_row_stride if k_row_stride is not None else k.stride(0)
    out = torch.empty(T, dtype=torch.float32, device=q.device)
    need = lib().fastav_score_workspace_bytes(model.n_q_heads, T, B, n_last)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    _check(lib().fastav_score(C.byref(model), q.data_ptr(), qs, k.data_ptr(), ks, cu_seqlens_dev.data_ptr(), B, T,
                              max_seqlen, n_last, out.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
    return out


SCORE_STATIC_BYTES = 8 << 20


def fastav_score_static(model: Model, q: torch.Tensor, k: torch.Tensor, cu_seqlens_dev: torch.Tensor, max_seqlen: int,
                        n_last: int = 1, out: Optional[torch.Tensor] = None, q_row_stride: Optional[int] = None,
                        k_row_stride: Optional[int] = None) -> torch.Tensor:
    """fastav_score through the entry point that allocates nothing: the scratch is the library's built-in array.
    Pass ``out`` (fp32 [T]) to keep this wrapper from allocating as well."""
    T = q.shape[0]
    B = cu_seqlens_dev.numel() - 1
    qs = q_row_stride if q_row_stride is not None else q.stride(0)
    ks = k_row_stride if k_row_stride is not None else k.stride(0)
    if out is None:
        out = torch.empty(T, dtype=torch.float32, device=q.device)
    _check(lib().fastav_score_static(C.byref(model), q.data_ptr(), qs, k.data_ptr(), ks, cu_seqlens_dev.data_ptr(), B, T,
                                     max_seqlen, n_last, out.data_ptr(), _stream()))
    return out


def fastav_select_gather(scores: Optional[torch.Tensor], protected_mask: torch.Tensor, cu_seqlens, keep_counts,
                         tensors: Sequence[torch.Tensor] = ()):
    """-> (keep_idx int32 [total_keep], cu_seqlens_out int32 [B+1] (device), [gathered tensors]).
    ``tensors`` are contiguous [T, ...] device tensors gathered along dim 0."""
    cu = _i32(cu_seqlens)
    kc = _i32(keep_counts)
    B = len(cu) - 1
    dev = protected_mask.device
    total_keep = int(kc.sum())
    keep_idx = torch.empty(max(total_keep, 1), dtype=torch.int32, device=dev)
    cu_out = torch.empty(B + 1, dtype=torch.int32, device=dev)
    dsts = [torch.empty((total_keep,) + tuple(t.shape[1:]), dtype=t.dtype, device=dev) for t in tensors]
    nt = len(tensors)
    src = (C.c_void_p * max(1, nt))(*[t.data_ptr() for t in tensors])
    dst = (C.c_void_p * max(1, nt))(*[t.data_ptr() if t.numel() else None for t in dsts])
    rb = (C.c_int64 * max(1, nt))(*[t.stride(0) * t.element_size() if t.dim() > 1 else t.element_size() for t in tensors])
    need = lib().fastav_select_workspace_bytes(B)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    _check(lib().fastav_select_gather(_ptr(scores), protected_mask.data_ptr(), cu.ctypes.data_as(C.POINTER(C.c_int32)),
                                      kc.ctypes.data_as(C.POINTER(C.c_int32)), B, nt, src, dst, rb, keep_idx.data_ptr(),
                                      cu_out.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
    return keep_idx[:total_keep], cu_out, dsts


def fastav_rmsnorm(x: torch.Tensor, g: torch.Tensor, eps: float) -> torch.Tensor:
    y = torch.empty(x.shape, dtype=g.dtype, device=x.device)
    _check(lib().fastav_rmsnorm(x.data_ptr(), g.data_ptr(), y.data_ptr(), x.shape[0], x.shape[1], eps, _dtype_code(g), _stream()))
    return y


def fastav_rope(x: torch.Tensor, pos: torch.Tensor, n_heads: int, head_dim: int, base: float) -> torch.Tensor:
    """In place on x [rows, row_stride]; returns x."""
    _check(lib().fastav_rope(x.data_ptr(), x.stride(0), pos.data_ptr(), x.shape[0], n_heads, head_dim, base,
                             _dtype_code(x), _stream()))
    return x


_linear_ws: Dict = {}


def fastav_linear(a: torch.Tensor, w: torch.Tensor, epilogue: int = EPI_STORE, w2: Optional[torch.Tensor] = None,
                  c: Optional[torch.Tensor] = None, use_workspace: bool = True) -> torch.Tensor:
    m, k = a.shape
    n = w.shape[0]
    if c is None:
        if epilogue == EPI_RESADD:
            raise ValueError("the residual epilogue updates c in place: pass it")
        c = torch.empty((m, n), dtype=a.dtype, device=a.device)
    ws = None
    if use_workspace and epilogue == EPI_RESADD and a.dtype == torch.bfloat16:
        key = a.device.index
        if key not in _linear_ws:
            _linear_ws[key] = torch.empty(lib().fastav_linear_workspace_bytes(), dtype=torch.uint8, device=a.device)
        ws = _linear_ws[key]
    _check(lib().fastav_linear(a.data_ptr(), w.data_ptr(), _ptr(w2), c.data_ptr(), m, n, k, epilogue, _dtype_code(a),
                               _ptr(ws), ws.numel() if ws is not None else 0, _stream()))
    return c


def fastav_attention(model: Model, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cu_seqlens_dev: torch.Tensor,
                     max_seqlen: int, want_last: bool = False):
    """q [T,Hq,dh], k,v [T,Hkv,dh] (row strides taken from the tensors) -> o [T,Hq,dh] (, last_logits [Hq,T], last_ml [B,Hq,2])."""
    T = q.shape[0]
    B = cu_seqlens_dev.numel() - 1
    o = torch.empty((T, model.n_q_heads, model.head_dim), dtype=q.dtype, device=q.device)
    ll = torch.full((model.n_q_heads, T), float("-inf"), dtype=torch.float32, device=q.device) if want_last else None
    ml = torch.zeros((B, model.n_q_heads, 2), dtype=torch.float32, device=q.device) if want_last else None
    if k.stride(0) != v.stride(0):
        raise ValueError("k and v must share a row stride")
    _check(lib().fastav_attention(C.byref(model), q.data_ptr(), q.stride(0), k.data_ptr(), v.data_ptr(), k.stride(0),
                                  o.data_ptr(), o.stride(0), cu_seqlens_dev.data_ptr(), B, T, max_seqlen, _ptr(ll), _ptr(ml), _stream()))
    return (o, ll, ml) if want_last else o


def fastav_profile_enable(kinds: Sequence[str]) -> None:
    mask = 0
    for k in kinds:
        mask |= 1 << PROF_KINDS[k]
    _check(lib().fastav_profile_enable(mask))


def fastav_profile_collect(kind: str):
    """-> (total_ms, launches, total_work) accumulated for one kernel kind since the last reset."""
    ms, n, w = C.c_double(), C.c_int64(), C.c_double()
    _check(lib().fastav_profile_collect(PROF_KINDS[kind], C.byref(ms), C.byref(n), C.byref(w)))
    return ms.value, n.value, w.value


def fastav_profile_reset() -> None:
    _check(lib().fastav_profile_reset())


def fastav_probe_mfma(iters: int, sink: torch.Tensor, operands: Optional[torch.Tensor] = None) -> float:
    """Enqueues the matrix-instruction-only probe on the current stream; -> flops of the launch.  ``operands``:
    optional bf16 tensor of at least 32768 elements that fills the operand registers."""
    fl = C.c_double()
    if operands is not None and (operands.dtype != torch.bfloat16 or operands.numel() < 32768 or not operands.is_contiguous()):
        raise ValueError("operands: contiguous bf16 tensor of at least 32768 elements")
    _check(lib().fastav_probe_mfma(iters, operands.data_ptr() if operands is not None else None, sink.data_ptr(), C.byref(fl), _stream()))
    return fl.value


def fastav_probe_read(src: torch.Tensor, sink: torch.Tensor) -> int:
    """Enqueues one streaming read of ``src`` on the current stream; -> bytes read."""
    nbytes = src.numel() * src.element_size()
    _check(lib().fastav_probe_read(src.data_ptr(), nbytes, sink.data_ptr(), _stream()))
    return nbytes


OPT_FUSED_SCORE_SELECT = 0
OPT_FUSED_ROPE = 1
OPT_FUSED_SPLITK_NORM = 2
OPT_FUSED_GATHER_OPROJ = 3


def fastav_set_option(option: int, value: int) -> None:
    _check(lib().fastav_set_option(option, value))
