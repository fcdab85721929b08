"""Thin ctypes binding of libdmoe.so: argument marshalling only.

PyTorch is used for device memory and streams; every step of the path runs in the library's own
kernels.  There is no fallback: if the library has not been built, importing `lib()` raises.
The functions carry the names of the C entry points (include/dmoe.h).
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "_lib", "libdmoe.so")

DMOE_OK, DMOE_ERR_NULL, DMOE_ERR_SHAPE, DMOE_ERR_UNSUPPORTED = 0, 1, 2, 3
DMOE_ERR_TAU, DMOE_ERR_WORKSPACE, DMOE_ERR_HIP = 4, 5, 6
DMOE_F32, DMOE_BF16 = 0, 1
ACT_CODES = {"relu": 0, "gelu_erf": 1, "gelu_tanh": 2}
DTYPE_CODES = {"f32": DMOE_F32, "bf16": DMOE_BF16}
DMOE_W_NATIVE, DMOE_W_FP8_E4M3, DMOE_W_FP8_E4M3_X8, DMOE_W_FP8_E4M3_A8 = 0, 1, 2, 3

EXPORTS = (
    "dmoe_version", "dmoe_last_error", "dmoe_workspace_bytes", "dmoe_select_workspace_bytes",
    "dmoe_packed_bytes", "dmoe_pack_weights", "dmoe_router", "dmoe_select", "dmoe_expert_ffn",
    "dmoe_forward", "dmoe_forward_static", "dmoe_select_topk", "dmoe_forward_topk", "dmoe_group_workspace_bytes",
    "dmoe_forward_group", "dmoe_timing_enable", "dmoe_timing_reset", "dmoe_timing_slots",
    "dmoe_timing_read",
)


class DmoeLayerStruct(ctypes.Structure):
    _fields_ = [
        ("d_model", ctypes.c_int32), ("n_experts", ctypes.c_int32),
        ("expert_size", ctypes.c_int32), ("router_hidden", ctypes.c_int32),
        ("gated", ctypes.c_int32), ("act", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("weight_format", ctypes.c_int32),
        ("w_up", ctypes.c_void_p), ("w_gate", ctypes.c_void_p), ("b_up", ctypes.c_void_p),
        ("w_down", ctypes.c_void_p), ("b_down", ctypes.c_void_p),
        ("r_w1", ctypes.c_void_p), ("r_b1", ctypes.c_void_p), ("r_w2", ctypes.c_void_p),
        ("r_b2", ctypes.c_void_p), ("packed", ctypes.c_void_p), ("w_scales", ctypes.c_void_p),
    ]


class DmoeError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"dmoe status {code}: {text}")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2310_04361_amd.build` "
                "(or __graft_entry__.build()); the HIP library is the only implementation")
        L = ctypes.CDLL(LIB_PATH)
        P, I, V, F = ctypes.POINTER, ctypes.c_int32, ctypes.c_void_p, ctypes.c_float
        SZ = ctypes.c_size_t
        LP = P(DmoeLayerStruct)
        L.dmoe_version.restype = I
        L.dmoe_last_error.restype = ctypes.c_char_p
        L.dmoe_workspace_bytes.argtypes = [LP, I, P(SZ)]
        L.dmoe_select_workspace_bytes.argtypes = [I, I, P(SZ)]
        L.dmoe_packed_bytes.argtypes = [LP, P(SZ)]
        L.dmoe_pack_weights.argtypes = [LP, V, SZ, V]
        L.dmoe_router.argtypes = [LP, V, I, V, V]
        L.dmoe_select.argtypes = [V, I, I, F, V, V, V, V, V, V, SZ, V]
        L.dmoe_expert_ffn.argtypes = [LP, V, I, V, V, V, V, SZ, V]
        L.dmoe_forward.argtypes = [LP, V, I, F, V, V, V, V, V, V, SZ, V]
        L.dmoe_forward_static.argtypes = [LP, V, I, F, V, V]
        L.dmoe_select_topk.argtypes = [V, I, I, I, V, V, V, V, V, V, SZ, V]
        L.dmoe_forward_topk.argtypes = [LP, V, I, I, V, V, V, V, V, V, SZ, V]
        L.dmoe_group_workspace_bytes.argtypes = [P(LP), I, I, P(SZ)]
        L.dmoe_forward_group.argtypes = [P(LP), I, V, I, P(F), P(V), V, SZ, V]
        L.dmoe_timing_enable.argtypes = [I]
        L.dmoe_timing_read.argtypes = [I, P(ctypes.c_char_p), P(ctypes.c_int64), P(ctypes.c_double)]
        for name in EXPORTS:
            if name != "dmoe_last_error":
                getattr(L, name).restype = I
        _lib = L
    return _lib


def check(rc: int) -> None:
    if rc != DMOE_OK:
        raise DmoeError(rc, lib().dmoe_last_error().decode())


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _torch_dtype(dtype: str):
    import torch
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def to_device(a: Optional[np.ndarray], dtype: str, device="cuda"):
    """fp64 array of storage-representable values -> device tensor of the storage type."""
    import torch
    from . import workloads
    if a is None:
        return None
    s = workloads.to_storage(a, dtype)
    if dtype == "bf16":
        return torch.from_numpy(s.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(s).to(device)


def from_device(t, dtype: str) -> np.ndarray:
    """Device tensor of the storage type -> fp64 NumPy array."""
    import torch
    return t.detach().to("cpu", torch.float64).numpy()


class Layer:
    """Device copy of one converted layer plus its C descriptor."""

    def __init__(self, params: dict, dtype: str, device="cuda"):
        import torch
        self.dtype = dtype
        self.device = device
        E, m, d = params["w_up"].shape
        self.E, self.m, self.d = E, m, d
        self.d_h = params["r_w1"].shape[0]
        self.gated = bool(params.get("gated", False))
        self.act = params["act"]
        self.t = {k: to_device(params.get(k), dtype, device)
                  for k in ("w_up", "w_gate", "b_up", "w_down", "b_down", "r_w1", "r_b1", "r_w2", "r_b2")}
        # params["x8"] (with "w8"): the experts' input is quantised row-wise to 8 bits as well;
        # params["a8"]: ... and every row of hidden activations too
        # 8-bit expert weights (params["w8"]: E4M3 codes and power-of-two scales): the library gets
        # the codes; self.t keeps the bf16 values of the same weights for dense comparisons
        w8 = params.get("w8")
        self.w8 = None
        ptrs = {k: _ptr(v) for k, v in self.t.items()}
        if w8 is not None:
            self.w8 = {k: torch.from_numpy(np.ascontiguousarray(w8[k])).to(device)
                       for k in ("w_up", "w_gate", "w_down", "scales") if w8.get(k) is not None}
            for k in ("w_up", "w_gate", "w_down"):
                ptrs[k] = _ptr(self.w8.get(k))
        self.c = DmoeLayerStruct(
            d_model=d, n_experts=E, expert_size=m, router_hidden=self.d_h,
            gated=int(self.gated), act=ACT_CODES[self.act], dtype=DTYPE_CODES[dtype],
            weight_format=(DMOE_W_FP8_E4M3_A8 if params.get("a8") else DMOE_W_FP8_E4M3_X8 if params.get("x8") else DMOE_W_FP8_E4M3) if w8 is not None else DMOE_W_NATIVE,
            **ptrs, packed=None, w_scales=_ptr(self.w8["scales"]) if w8 is not None else None)
        nbytes = ctypes.c_size_t(0)
        check(lib().dmoe_packed_bytes(ctypes.byref(self.c), ctypes.byref(nbytes)))
        self.packed = None
        if nbytes.value:
            self.packed = torch.empty(nbytes.value, dtype=torch.uint8, device=device)
            check(lib().dmoe_pack_weights(ctypes.byref(self.c), self.packed.data_ptr(),
                                          nbytes.value, _stream()))
            self.c.packed = self.packed.data_ptr()
        self._ws = None

    def ref(self):
        return ctypes.byref(self.c)

    def workspace(self, T: int):
        """Cached scratch tensor large enough for T tokens."""
        import torch
        n = ctypes.c_size_t(0)
        check(lib().dmoe_workspace_bytes(self.ref(), T, ctypes.byref(n)))
        if self._ws is None or self._ws.numel() < n.value:
            self._ws = torch.empty(max(n.value, 256), dtype=torch.uint8, device=self.device)
        return self._ws


def dmoe_router(layer: Layer, x):
    """scores[T, E] fp32 (Sec. 3.3)."""
    import torch
    T = x.shape[0]
    scores = torch.empty((T, layer.E), dtype=torch.float32, device=x.device)
    check(lib().dmoe_router(layer.ref(), x.data_ptr(), T, scores.data_ptr(), _stream()))
    return scores


def dmoe_select(scores, tau: float, want_mask=True, want_k=True, top_k=None):
    """Dynamic-k gate + bucketing (Eq. 4), or the top-k gate when top_k is given.  Returns a dict
    of device tensors: mask_bits [T, ceil(E/64)] int64, k_per_token [T], counts [E],
    offsets [E+1], token_lists [T*E] (only the first offsets[E] entries are meaningful)."""
    import torch
    T, E = scores.shape
    dev = scores.device
    W = (E + 63) // 64
    out = {
        "mask_bits": torch.empty((T, W), dtype=torch.int64, device=dev) if want_mask else None,
        "k_per_token": torch.empty((T,), dtype=torch.int32, device=dev) if want_k else None,
        "counts": torch.empty((E,), dtype=torch.int32, device=dev),
        "offsets": torch.empty((E + 1,), dtype=torch.int32, device=dev),
        "token_lists": torch.empty((max(T * E, 1),), dtype=torch.int32, device=dev),
    }
    n = ctypes.c_size_t(0)
    check(lib().dmoe_select_workspace_bytes(T, E, ctypes.byref(n)))
    ws = torch.empty(max(n.value, 256), dtype=torch.uint8, device=dev)
    tail = (_ptr(out["mask_bits"]), _ptr(out["k_per_token"]), out["counts"].data_ptr(),
            out["offsets"].data_ptr(), out["token_lists"].data_ptr(), ws.data_ptr(), ws.numel(),
            _stream())
    if top_k is None:
        check(lib().dmoe_select(scores.data_ptr(), T, E, float(tau), *tail))
    else:
        check(lib().dmoe_select_topk(scores.data_ptr(), T, E, int(top_k), *tail))
    return out


def dmoe_select_topk(scores, k: int, want_mask=True, want_k=True):
    """Top-k gate + bucketing: exactly k experts per token (ties to the lower index)."""
    return dmoe_select(scores, 0.0, want_mask, want_k, top_k=k)


def dmoe_expert_ffn(layer: Layer, x, offsets, token_lists):
    """y[T, d] from explicit per-expert token lists (Sec. 3.2, Appendix G)."""
    import torch
    T = x.shape[0]
    y = torch.empty((T, layer.d), dtype=_torch_dtype(layer.dtype), device=x.device)
    ws = layer.workspace(T)
    check(lib().dmoe_expert_ffn(layer.ref(), x.data_ptr(), T, offsets.data_ptr(),
                                token_lists.data_ptr(), y.data_ptr(), ws.data_ptr(), ws.numel(),
                                _stream()))
    return y


def dmoe_forward(layer: Layer, x, tau: float, want_scores=False, want_mask=False,
                 want_lists=False, y=None, top_k=None):
    """Whole layer (top-k gate instead of the dynamic-k one when top_k is given).  Returns
    (y, extras) with extras holding the requested optional outputs."""
    import torch
    T = x.shape[0]
    dev = x.device
    if y is None:
        y = torch.empty((T, layer.d), dtype=_torch_dtype(layer.dtype), device=dev)
    ex = {}
    if want_scores:
        ex["scores"] = torch.empty((T, layer.E), dtype=torch.float32, device=dev)
    if want_mask:
        ex["mask_bits"] = torch.empty((T, (layer.E + 63) // 64), dtype=torch.int64, device=dev)
    if want_lists:
        ex["offsets"] = torch.empty((layer.E + 1,), dtype=torch.int32, device=dev)
        ex["token_lists"] = torch.empty((max(T * layer.E, 1),), dtype=torch.int32, device=dev)
    ws = layer.workspace(T)
    tail = (y.data_ptr(), _ptr(ex.get("scores")), _ptr(ex.get("mask_bits")),
            _ptr(ex.get("offsets")), _ptr(ex.get("token_lists")), ws.data_ptr(), ws.numel(),
            _stream())
    if top_k is None:
        check(lib().dmoe_forward(layer.ref(), x.data_ptr(), T, float(tau), *tail))
    else:
        check(lib().dmoe_forward_topk(layer.ref(), x.data_ptr(), T, int(top_k), *tail))
    return y, ex


def dmoe_forward_static(layer: Layer, x, tau: float, y=None):
    """Whole layer on the library's static per-GPU workspace (no allocation inside the call;
    y is allocated here only when the caller passes none)."""
    import torch
    T = x.shape[0]
    if y is None:
        y = torch.empty((T, layer.d), dtype=_torch_dtype(layer.dtype), device=x.device)
    check(lib().dmoe_forward_static(layer.ref(), x.data_ptr(), T, float(tau), y.data_ptr(), _stream()))
    return y


_group_ws = {}


def dmoe_forward_group(layers, x, taus, ys=None):
    """1 to 4 layers of one shape on the same input (the attention projections of Sec. 3.5).
    Returns the list of outputs."""
    import torch
    n, T = len(layers), x.shape[0]
    if ys is None:
        ys = [torch.empty((T, L.d), dtype=_torch_dtype(L.dtype), device=x.device) for L in layers]
    LP = ctypes.POINTER(DmoeLayerStruct)
    refs = (LP * n)(*[ctypes.pointer(L.c) for L in layers])
    need = ctypes.c_size_t(0)
    check(lib().dmoe_group_workspace_bytes(refs, n, T, ctypes.byref(need)))
    key = (x.device, max(need.value, 256))
    ws = _group_ws.get(key)
    if ws is None:
        _group_ws.clear()
        ws = _group_ws[key] = torch.empty(key[1], dtype=torch.uint8, device=x.device)
    tau_arr = (ctypes.c_float * n)(*[float(t) for t in taus])
    y_arr = (ctypes.c_void_p * n)(*[y.data_ptr() for y in ys])
    check(lib().dmoe_forward_group(refs, n, x.data_ptr(), T, tau_arr, y_arr, ws.data_ptr(),
                                   ws.numel(), _stream()))
    return ys


def dmoe_forward_topk(layer: Layer, x, k: int, **kw):
    """Whole layer with the top-k gate."""
    return dmoe_forward(layer, x, 0.0, top_k=k, **kw)


def mask_bits_to_bool(mask_bits, E: int) -> np.ndarray:
    """[T, W] int64 words -> [T, E] uint8 (host)."""
    words = mask_bits.detach().cpu().numpy().view(np.uint64)
    T, W = words.shape
    bits = ((words[:, :, None] >> np.arange(64, dtype=np.uint64)[None, None, :]) & np.uint64(1))
    return bits.reshape(T, W * 64)[:, :E].astype(np.uint8)


def timing(enable: bool) -> None:
    check(lib().dmoe_timing_enable(1 if enable else 0))
    check(lib().dmoe_timing_reset())


def timing_read() -> dict:
    """{kernel name: (launches, total_ms)} since the last reset; waits for the events."""
    out = {}
    for i in range(lib().dmoe_timing_slots()):
        name, n, ms = ctypes.c_char_p(), ctypes.c_int64(0), ctypes.c_double(0.0)
        check(lib().dmoe_timing_read(i, ctypes.byref(name), ctypes.byref(n), ctypes.byref(ms)))
        out[name.value.decode()] = (n.value, ms.value)
    return out
