"""Thin ctypes binding of libcq.so: argument marshalling only.

Every step of the layer runs in the HIP kernels behind the C ABI declared in include/cq.h; the
functions here carry the same names, allocate outputs and workspaces as torch tensors (device
memory and streams are all torch is used for) and pass raw device pointers through.  There is no
CPU fallback: if the library has not been built, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libcq.so")

CQ_OK = 0
CQ_A_INT8_CODES, CQ_A_F16, CQ_A_F32, CQ_A_BF16 = 0, 1, 2, 3
CQ_EPI_NONE, CQ_EPI_SWIGLU = 0, 1
CQ_OUT_F32, CQ_OUT_F16 = 0, 1

EXPORTS = [
    "cq_status_string", "cq_rotate_quant_workspace_bytes", "cq_rotate_quant",
    "cq_route_permute_workspace_bytes", "cq_route_permute", "cq_grouped_gemm_workspace_bytes",
    "cq_codebook_grouped_gemm", "cq_combine", "cq_moe_workspace_bytes", "cq_moe_workspace_layout",
    "cq_moe_forward", "cq_moe_forward_static", "cq_moe_forward_timed", "cq_prepack_bytes", "cq_prepack", "cq_decode_dense", "cq_device_info",
    "cq_stream_read", "cq_mfma_loop", "cq_rotation_split_bytes", "cq_rotation_split",
    "cq_rotate_quant_split_workspace_bytes", "cq_rotate_quant_split", "cq_hadamard_quant",
    "cq_codebook_grouped_gemm_lut", "cq_expand_centroid_budget",
]


class CodebookWeights(ctypes.Structure):
    _fields_ = [("idx", ctypes.c_void_p), ("cent", ctypes.c_void_p), ("prepacked", ctypes.c_void_p),
                ("G", ctypes.c_int), ("N", ctypes.c_int), ("K", ctypes.c_int), ("group_k", ctypes.c_int),
                ("index_bits", ctypes.c_int)]


class Layer(ctypes.Structure):
    _fields_ = [("H", ctypes.c_int), ("I", ctypes.c_int), ("E", ctypes.c_int), ("top_k", ctypes.c_int),
                ("S", ctypes.c_int), ("act_bits", ctypes.c_int),
                ("R", ctypes.c_void_p), ("Wr", ctypes.c_void_p), ("bias", ctypes.c_void_p),
                ("gate_up", CodebookWeights), ("down", CodebookWeights), ("R_split", ctypes.c_void_p),
                ("h_bits", ctypes.c_int), ("r_hadamard", ctypes.c_int)]


class MoeLayout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in
                ("total", "XR", "Q", "Q16", "scale", "logits", "topk_ids", "topk_w", "offsets", "perm", "inv_perm",
                 "src_token", "Hbuf", "Obuf", "scratch", "HQ", "HQ16", "hscale")]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libcq.so (after torch when torch is importable, so both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_10496_amd.build` "
                           "(there is no fallback path)")
    try:
        import torch  # noqa: F401  (maps torch's libamdhip64 first)
    except ImportError:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.cq_status_string.restype = ctypes.c_char_p
    lib.cq_status_string.argtypes = [ci]
    lib.cq_rotate_quant_workspace_bytes.restype = sz
    lib.cq_rotate_quant_workspace_bytes.argtypes = [ci, ci]
    lib.cq_rotate_quant.restype = ci
    lib.cq_rotate_quant.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp, vp, sz, vp]
    lib.cq_route_permute_workspace_bytes.restype = sz
    lib.cq_route_permute_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.cq_route_permute.restype = ci
    lib.cq_route_permute.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.cq_grouped_gemm_workspace_bytes.restype = sz
    lib.cq_grouped_gemm_workspace_bytes.argtypes = [ctypes.POINTER(CodebookWeights), ci]
    lib.cq_codebook_grouped_gemm.restype = ci
    lib.cq_codebook_grouped_gemm.argtypes = [ctypes.POINTER(CodebookWeights), vp, ci, vp, vp, vp, ci, ci, vp, ci,
                                             vp, sz, vp]
    lib.cq_combine.restype = ci
    lib.cq_combine.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp, vp]
    lib.cq_moe_workspace_bytes.restype = sz
    lib.cq_moe_workspace_bytes.argtypes = [ctypes.POINTER(Layer), ci]
    lib.cq_moe_workspace_layout.restype = ci
    lib.cq_moe_workspace_layout.argtypes = [ctypes.POINTER(Layer), ci, ctypes.POINTER(MoeLayout)]
    lib.cq_moe_forward.restype = ci
    lib.cq_moe_forward.argtypes = [ctypes.POINTER(Layer), vp, ci, vp, vp, sz, vp]
    lib.cq_moe_forward_static.restype = ci
    lib.cq_moe_forward_static.argtypes = [ctypes.POINTER(Layer), vp, ci, vp, vp]
    lib.cq_moe_forward_timed.restype = ci
    lib.cq_moe_forward_timed.argtypes = [ctypes.POINTER(Layer), vp, ci, vp, vp, sz, vp, ctypes.POINTER(ctypes.c_float)]
    lib.cq_rotation_split_bytes.restype = sz
    lib.cq_rotation_split_bytes.argtypes = [ci]
    lib.cq_rotation_split.restype = ci
    lib.cq_rotation_split.argtypes = [vp, ci, vp, sz, vp]
    lib.cq_rotate_quant_split_workspace_bytes.restype = sz
    lib.cq_rotate_quant_split_workspace_bytes.argtypes = [ci, ci]
    lib.cq_rotate_quant_split.restype = ci
    lib.cq_rotate_quant_split.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp, vp, sz, vp]
    lib.cq_hadamard_quant.restype = ci
    lib.cq_hadamard_quant.argtypes = [vp, ci, ci, ci, vp, vp, vp, vp]
    lib.cq_prepack_bytes.restype = sz
    lib.cq_prepack_bytes.argtypes = [ctypes.POINTER(CodebookWeights)]
    lib.cq_prepack.restype = ci
    lib.cq_prepack.argtypes = [ctypes.POINTER(CodebookWeights), vp, sz, vp]
    lib.cq_codebook_grouped_gemm_lut.restype = ci
    lib.cq_codebook_grouped_gemm_lut.argtypes = [ctypes.POINTER(CodebookWeights), vp, vp, vp, vp, ci, ci, vp, ci, vp]
    lib.cq_expand_centroid_budget.restype = ci
    lib.cq_expand_centroid_budget.argtypes = [vp, vp, ci, ci, ci, ci, ci, vp, vp, vp]
    lib.cq_decode_dense.restype = ci
    lib.cq_decode_dense.argtypes = [ctypes.POINTER(CodebookWeights), ci, vp, vp]
    lib.cq_device_info.restype = ci
    lib.cq_device_info.argtypes = [ctypes.POINTER(ci)] * 5
    lib.cq_stream_read.restype = ci
    lib.cq_stream_read.argtypes = [vp, sz, vp, vp]
    lib.cq_mfma_loop.restype = ci
    lib.cq_mfma_loop.argtypes = [ci, ci, vp, vp]
    _lib = lib
    return lib


class CqError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(load_library().cq_status_string(status).decode())


def _check(st: int) -> None:
    if st != CQ_OK:
        raise CqError(st)


def _torch():
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("libcq needs a GPU: torch.cuda.is_available() is False and there is no CPU path")
    return torch


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _ws(nbytes: int):
    torch = _torch()
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


# ------------------------------------------------------------------------------------------------
# weights
# ------------------------------------------------------------------------------------------------
class DeviceCodebook:
    """Device-resident [G, N, K/2] indices + [G, N, 16] bf16 tables, optionally prepacked.

    group_k = g > 0: block-wise tables, cent is [G, N, ceil(K/g), 16].
    index_bits = 2: the W2 budget streamed as stored, idx [G, N, K/4] (2-bit stream), cent [G, N, 4]."""

    def __init__(self, idx, cent, prepack: bool = True, keep_canonical: bool = True, group_k: int = 0,
                 index_bits: int = 4):
        torch = _torch()
        import numpy as np
        if isinstance(idx, np.ndarray):
            idx = torch.from_numpy(np.ascontiguousarray(idx))
        if isinstance(cent, np.ndarray):
            cent = torch.from_numpy(np.ascontiguousarray(cent).view(np.int16))
        assert idx.dtype == torch.uint8 and idx.dim() == 3 and cent.dtype == torch.int16
        self.index_bits = int(index_bits)
        per_byte = 4 if self.index_bits == 2 else 2
        self.G, self.N, self.K = int(idx.shape[0]), int(idx.shape[1]), int(idx.shape[2]) * per_byte
        self.group_k = int(group_k)
        if self.index_bits == 2:
            assert self.group_k == 0 and tuple(cent.shape) == (self.G, self.N, 4)
        elif self.group_k > 0:
            assert tuple(cent.shape) == (self.G, self.N, -(-self.K // self.group_k), 16)
        else:
            assert tuple(cent.shape) == (self.G, self.N, 16)
        self.cent = cent.to("cuda").contiguous()
        self.idx = idx.to("cuda").contiguous()
        self.prepacked = None
        if prepack:
            self.prepacked = cq_prepack(self)
            if not keep_canonical:
                self.idx = None

    def struct(self, use_prepacked: bool = True) -> CodebookWeights:
        pre = self.prepacked if use_prepacked else None
        return CodebookWeights(_ptr(self.idx), _ptr(self.cent), _ptr(pre), self.G, self.N, self.K, self.group_k,
                               self.index_bits)


def cq_prepack(W: DeviceCodebook):
    torch = _torch()
    lib = load_library()
    s = W.struct(use_prepacked=False)
    n = lib.cq_prepack_bytes(ctypes.byref(s))
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    _check(lib.cq_prepack(ctypes.byref(s), _ptr(dst), n, _stream()))
    return dst


def cq_rotation_split(R):
    """Split copy of R [H, H] (device fp32) for the f16 matrix cores; returns a device byte buffer."""
    torch = _torch()
    lib = load_library()
    H = R.shape[0]
    n = lib.cq_rotation_split_bytes(H)
    if n == 0:
        raise CqError(2)
    out = torch.empty(n, dtype=torch.uint8, device="cuda")
    _check(lib.cq_rotation_split(_ptr(R), H, _ptr(out), n, _stream()))
    return out


def cq_codebook_grouped_gemm_lut(W: DeviceCodebook, codes, row_scale, row_gather, group_offsets, M_total: int,
                                 epilogue: int, out_kind: int, out=None):
    """The lookup formulation of the product (4-bit codes in an int8 container); see include/cq.h."""
    torch = _torch()
    lib = load_library()
    n_out = W.N // 2 if epilogue == CQ_EPI_SWIGLU else W.N
    if out is None:
        out = torch.empty((M_total, n_out), dtype=torch.float16 if out_kind == CQ_OUT_F16 else torch.float32,
                          device="cuda")
    s = W.struct(use_prepacked=False)
    _check(lib.cq_codebook_grouped_gemm_lut(ctypes.byref(s), _ptr(codes), _ptr(row_scale), _ptr(row_gather),
                                            _ptr(group_offsets), M_total, epilogue, _ptr(out), out_kind, _stream()))
    return out


def cq_expand_centroid_budget(idx_bits, cent_bits, bits: int, K: int, group_k: int = 0, prepack: bool = True):
    """W2 / W3 weights ([G, N, K*bits/8] bit-stream bytes, [G, N, (tables,) 2^bits] bf16 tables, numpy or torch)
    -> a DeviceCodebook in the 16-entry format the kernels read."""
    torch = _torch()
    import numpy as np
    lib = load_library()
    if isinstance(idx_bits, np.ndarray):
        idx_bits = torch.from_numpy(np.ascontiguousarray(idx_bits))
    if isinstance(cent_bits, np.ndarray):
        cent_bits = torch.from_numpy(np.ascontiguousarray(cent_bits).view(np.int16))
    idx_bits, cent_bits = idx_bits.to("cuda").contiguous(), cent_bits.to("cuda").contiguous()
    G, N = int(idx_bits.shape[0]), int(idx_bits.shape[1])
    tables = -(-K // group_k) if group_k > 0 else 1
    assert idx_bits.shape[2] * 8 == K * bits and cent_bits.numel() == G * N * tables * (1 << bits)
    idx4 = torch.empty((G, N, K // 2), dtype=torch.uint8, device="cuda")
    shape = (G, N, tables, 16) if group_k > 0 else (G, N, 16)
    cent16 = torch.empty(shape, dtype=torch.int16, device="cuda")
    _check(lib.cq_expand_centroid_budget(_ptr(idx_bits), _ptr(cent_bits), bits, G, N, K, tables, _ptr(idx4),
                                         _ptr(cent16), _stream()))
    return DeviceCodebook(idx4, cent16, prepack=prepack, group_k=group_k)


def cq_decode_dense(W: DeviceCodebook, g: int, use_prepacked: bool = True):
    torch = _torch()
    lib = load_library()
    out = torch.empty((W.N, W.K), dtype=torch.int16, device="cuda")
    s = W.struct(use_prepacked)
    _check(lib.cq_decode_dense(ctypes.byref(s), g, _ptr(out), _stream()))
    return out


# ------------------------------------------------------------------------------------------------
# steps
# ------------------------------------------------------------------------------------------------
def cq_rotate_quant(X, R, act_bits: int) -> Dict[str, object]:
    torch = _torch()
    lib = load_library()
    T, H = X.shape
    XR = torch.empty((T, H), dtype=torch.float32, device="cuda")
    Q = torch.empty((T, H), dtype=torch.int8, device="cuda")
    scale = torch.empty((T,), dtype=torch.float32, device="cuda")
    n = lib.cq_rotate_quant_workspace_bytes(T, H)
    ws = _ws(n)
    _check(lib.cq_rotate_quant(_ptr(X), _ptr(R), T, H, act_bits, _ptr(XR), _ptr(Q), _ptr(scale), _ptr(ws), ws.numel(),
                               _stream()))
    return {"XR": XR, "Q": Q, "scale": scale}


def cq_rotate_quant_split(X, R_split, act_bits: int) -> Dict[str, object]:
    torch = _torch()
    lib = load_library()
    T, H = X.shape
    XR = torch.empty((T, H), dtype=torch.float32, device="cuda")
    Q = torch.empty((T, H), dtype=torch.int8, device="cuda")
    scale = torch.empty((T,), dtype=torch.float32, device="cuda")
    ws = _ws(lib.cq_rotate_quant_split_workspace_bytes(T, H))
    _check(lib.cq_rotate_quant_split(_ptr(X), _ptr(R_split), T, H, act_bits, _ptr(XR), _ptr(Q), _ptr(scale), _ptr(ws),
                                     ws.numel(), _stream()))
    return {"XR": XR, "Q": Q, "scale": scale}


def cq_hadamard_quant(Hrows, bits: int) -> Dict[str, object]:
    """h' = h H / sqrt(I) per row (device fp32 [M, I]) and its integer codes and scales."""
    torch = _torch()
    lib = load_library()
    M, I = Hrows.shape
    HR = torch.empty((M, I), dtype=torch.float32, device="cuda")
    Q = torch.empty((M, I), dtype=torch.int8, device="cuda")
    scale = torch.empty((M,), dtype=torch.float32, device="cuda")
    _check(lib.cq_hadamard_quant(_ptr(Hrows), M, I, bits, _ptr(HR), _ptr(Q), _ptr(scale), _stream()))
    return {"HR": HR, "Q": Q, "scale": scale}


def cq_route_permute(XR, Wr, bias, top_k: int, n_shared: int = 0, logits_in=None) -> Dict[str, object]:
    torch = _torch()
    lib = load_library()
    if XR is not None:
        T, H = XR.shape
        E = Wr.shape[0]
    else:
        T, E = logits_in.shape
        H = 64
    A = T * top_k
    i32 = dict(dtype=torch.int32, device="cuda")
    out = {
        "logits": torch.empty((T, E), dtype=torch.float32, device="cuda"),
        "ids": torch.empty((T, top_k), **i32),
        "w": torch.empty((T, top_k), dtype=torch.float32, device="cuda"),
        "offsets": torch.empty((E + n_shared + 1,), **i32),
        "perm": torch.empty((A,), **i32),
        "inv_perm": torch.empty((A,), **i32),
        "src_token": torch.empty((T * (top_k + n_shared),), **i32),
    }
    n = lib.cq_route_permute_workspace_bytes(T, H, E, top_k)
    ws = _ws(n)
    _check(lib.cq_route_permute(_ptr(XR), _ptr(Wr), _ptr(bias), _ptr(logits_in), T, H, E, top_k, n_shared,
                                _ptr(out["logits"]), _ptr(out["ids"]), _ptr(out["w"]), _ptr(out["offsets"]),
                                _ptr(out["perm"]), _ptr(out["inv_perm"]), _ptr(out["src_token"]), _ptr(ws),
                                ws.numel(), _stream()))
    return out


def cq_codebook_grouped_gemm(W: DeviceCodebook, A, a_kind: int, row_scale, row_gather, group_offsets, M_total: int,
                             epilogue: int, out_kind: int, use_prepacked: bool = True):
    torch = _torch()
    lib = load_library()
    n_out = W.N // 2 if epilogue == CQ_EPI_SWIGLU else W.N
    out = torch.empty((M_total, n_out), dtype=torch.float16 if out_kind == CQ_OUT_F16 else torch.float32,
                      device="cuda")
    s = W.struct(use_prepacked)
    n = lib.cq_grouped_gemm_workspace_bytes(ctypes.byref(s), M_total)
    ws = _ws(n)
    _check(lib.cq_codebook_grouped_gemm(ctypes.byref(s), _ptr(A), a_kind, _ptr(row_scale), _ptr(row_gather),
                                        _ptr(group_offsets), M_total, epilogue, _ptr(out), out_kind, _ptr(ws),
                                        ws.numel(), _stream()))
    return out


def cq_combine(O, topk_w, inv_perm, T: int, H: int, top_k: int, n_shared: int = 0):
    torch = _torch()
    lib = load_library()
    Y = torch.empty((T, H), dtype=torch.float32, device="cuda")
    _check(lib.cq_combine(_ptr(O), _ptr(topk_w), _ptr(inv_perm), T, H, top_k, n_shared, _ptr(Y), _stream()))
    return Y


class DeviceLayer:
    """All constant inputs of one layer on the device, plus a reusable workspace."""

    def __init__(self, cfg, R, Wr, bias, gate_up: DeviceCodebook, down: DeviceCodebook, use_prepacked: bool = True):
        torch = _torch()
        self.cfg = cfg
        self.R = None if R is None else torch.as_tensor(R).to("cuda").contiguous()
        self.Wr = torch.as_tensor(Wr).to("cuda").contiguous()
        self.bias = None if bias is None else torch.as_tensor(bias).to("cuda").contiguous()
        self.gate_up, self.down = gate_up, down
        self.use_prepacked = use_prepacked
        # set-up work, like prepacking the indices: the split copy of R for the f16 matrix cores
        self.R_split = (cq_rotation_split(self.R)
                        if use_prepacked and cfg.H % 32 == 0 and self.R is not None
                        and not getattr(cfg, "r_hadamard", False) else None)
        self._ws = None
        self._ws_T = -1

    def struct(self) -> Layer:
        c = self.cfg
        return Layer(c.H, c.I, c.E, c.top_k, c.S, c.act_bits, _ptr(self.R), _ptr(self.Wr), _ptr(self.bias),
                     self.gate_up.struct(self.use_prepacked), self.down.struct(self.use_prepacked),
                     _ptr(self.R_split), getattr(c, "h_bits", 0), 1 if getattr(c, "r_hadamard", False) else 0)

    def workspace(self, T: int):
        if self._ws is None or self._ws_T != T:
            lib = load_library()
            s = self.struct()
            n = lib.cq_moe_workspace_bytes(ctypes.byref(s), T)
            if n == 0:
                raise CqError(2)
            self._ws = _ws(n)
            self._ws_T = T
        return self._ws


def cq_moe_forward(layer: DeviceLayer, X, Y=None):
    torch = _torch()
    lib = load_library()
    T = X.shape[0]
    if Y is None:
        Y = torch.empty((T, layer.cfg.H), dtype=torch.float32, device="cuda")
    ws = layer.workspace(T)
    s = layer.struct()
    _check(lib.cq_moe_forward(ctypes.byref(s), _ptr(X), T, _ptr(Y), _ptr(ws), ws.numel(), _stream()))
    return Y


def cq_moe_forward_static(layer: DeviceLayer, X, Y):
    """cq_moe_forward on the library's own scratch array: no workspace, nothing allocated (Y is the caller's)."""
    lib = load_library()
    s = layer.struct()
    _check(lib.cq_moe_forward_static(ctypes.byref(s), _ptr(X), X.shape[0], _ptr(Y), _stream()))
    return Y


STAGES = ("rotate_quant", "route_permute", "gate_up", "down", "combine")


def cq_moe_forward_timed(layer: DeviceLayer, X, Y=None):
    """Same launches as cq_moe_forward plus stage-boundary events; returns (Y, {stage: ms})."""
    torch = _torch()
    lib = load_library()
    T = X.shape[0]
    if Y is None:
        Y = torch.empty((T, layer.cfg.H), dtype=torch.float32, device="cuda")
    ws = layer.workspace(T)
    s = layer.struct()
    ms = (ctypes.c_float * len(STAGES))()
    _check(lib.cq_moe_forward_timed(ctypes.byref(s), _ptr(X), T, _ptr(Y), _ptr(ws), ws.numel(), _stream(), ms))
    return Y, dict(zip(STAGES, [float(v) for v in ms]))


def moe_intermediates(layer: DeviceLayer, T: int) -> Dict[str, object]:
    """Views of the intermediates the last cq_moe_forward(layer, X[T]) left in the workspace."""
    torch = _torch()
    lib = load_library()
    lay = MoeLayout()
    s = layer.struct()
    _check(lib.cq_moe_workspace_layout(ctypes.byref(s), T, ctypes.byref(lay)))
    ws = layer.workspace(T)
    c = layer.cfg
    A, M = T * c.top_k, T * (c.top_k + c.S)

    def view(off, nbytes, dtype, shape):
        return ws[off:off + nbytes].view(dtype).view(shape)
    return {
        "XR": view(lay.XR, T * c.H * 4, torch.float32, (T, c.H)),
        "Q": view(lay.Q, T * c.H, torch.int8, (T, c.H)),
        "scale": view(lay.scale, T * 4, torch.float32, (T,)),
        "logits": view(lay.logits, T * c.E * 4, torch.float32, (T, c.E)),
        "ids": view(lay.topk_ids, A * 4, torch.int32, (T, c.top_k)),
        "w": view(lay.topk_w, A * 4, torch.float32, (T, c.top_k)),
        "offsets": view(lay.offsets, (c.E + c.S + 1) * 4, torch.int32, (c.E + c.S + 1,)),
        "perm": view(lay.perm, A * 4, torch.int32, (A,)),
        "inv_perm": view(lay.inv_perm, A * 4, torch.int32, (A,)),
        "src_token": view(lay.src_token, M * 4, torch.int32, (M,)),
        "h": (view(lay.Hbuf, M * c.I * 4, torch.float32, (M, c.I)) if getattr(c, "h_bits", 0)
              else view(lay.Hbuf, M * c.I * 2, torch.float16, (M, c.I))),
        "o": view(lay.Obuf, M * c.H * 4, torch.float32, (M, c.H)),
        "hq": view(lay.HQ, M * c.I, torch.int8, (M, c.I)) if getattr(c, "h_bits", 0) else None,
        "hscale": view(lay.hscale, M * 4, torch.float32, (M,)) if getattr(c, "h_bits", 0) else None,
    }


def device_layer_from_inputs(inputs, use_prepacked: bool = True) -> DeviceLayer:
    """Upload a synth.LayerInputs (layout work only: stacking experts, interleaving gate/up rows)."""
    from . import synth
    st = synth.stack_experts(inputs)
    g = getattr(inputs.cfg, "group_k", 0)
    bits = getattr(inputs.cfg, "index_bits", 4)
    gu = DeviceCodebook(st["gate_up_idx"], st["gate_up_cent"], prepack=use_prepacked, group_k=g, index_bits=bits)
    dn = DeviceCodebook(st["down_idx"], st["down_cent"], prepack=use_prepacked, group_k=g, index_bits=bits)
    return DeviceLayer(inputs.cfg, inputs.R, inputs.Wr, inputs.bias, gu, dn, use_prepacked)


def cq_device_info() -> Dict[str, int]:
    lib = load_library()
    vals = [ctypes.c_int(0) for _ in range(5)]
    _check(lib.cq_device_info(*[ctypes.byref(v) for v in vals]))
    keys = ["cu_count", "clock_khz", "mem_clock_khz", "bus_bits", "lds_bytes"]
    return {k: v.value for k, v in zip(keys, vals)}


def cq_stream_read(buf):
    torch = _torch()
    lib = load_library()
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    _check(lib.cq_stream_read(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), _stream()))
    return sink


def cq_mfma_loop(workgroups: int, iters: int):
    """Launch the bare MFMA loop; returns its flop count (time it with events around the call)."""
    torch = _torch()
    lib = load_library()
    sink = torch.empty(workgroups * 256, dtype=torch.float32, device="cuda")
    _check(lib.cq_mfma_loop(workgroups, iters, _ptr(sink), _stream()))
    return workgroups * 4 * iters * 16 * 32768.0
