"""Thin ctypes binding of libwq.so (include/wq.h).  Argument marshalling only:
every step of the convolution runs in the library's HIP kernels.  PyTorch is
used for device memory and streams, nothing else.  There is no fallback: if the
library is not built, importing a symbol raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libwq.so")

WQ_OK = 0
STATIC_WORKSPACE_BYTES = 32 << 20   # WQ_STATIC_WORKSPACE_BYTES of include/wq.h
STATUS_NAMES = {0: "WQ_OK", 1: "WQ_ERR_INVALID_ARG", 2: "WQ_ERR_UNSUPPORTED",
                3: "WQ_ERR_BAD_TRANSFORM", 4: "WQ_ERR_NOT_PREPARED", 5: "WQ_ERR_WORKSPACE",
                6: "WQ_ERR_DEVICE"}

EXPORTS = ["wq_standard_transforms", "wq_scaled_transforms", "wq_plan_create", "wq_plan_destroy",
           "wq_plan_layout", "wq_plan_tune", "wq_plan_set_integer_transforms", "wq_conv_forward_debug_slab", "wq_direct_plan_tune",
           "wq_contract_output_part", "wq_microbench_dequant", "wq_conv_forward_static",
           "wq_weight_prepare", "wq_input_transform", "wq_contract_output", "wq_contract",
           "wq_output_transform", "wq_conv_forward",
           "wq_direct_plan_create", "wq_linear_plan_create", "wq_direct_plan_create_bits",
           "wq_linear_plan_create_bits", "wq_direct_plan_destroy", "wq_direct_plan_layout",
           "wq_direct_weight_prepare", "wq_direct_quantize", "wq_direct_conv", "wq_direct_forward",
           "wq_conv_forward_debug", "wq_status_string"]


class Layout(ctypes.Structure):
    _fields_ = ([(k, ctypes.c_int32) for k in
                 ("N", "H", "W", "Cin", "Cout", "m", "n", "group_size", "groups",
                  "TH", "TW", "T", "T_pad", "Cout_pad", "kstep", "k2_kernels", "k2_variant",
                  "k1_rows")] +
                [(k, ctypes.c_uint64) for k in
                 ("blob_bytes", "blob_Wq_off", "blob_sW_off", "blob_bias_off",
                  "ws_bytes", "ws_Xq_off", "ws_sX_off", "ws_M_off", "debug_P_bytes")])


class DirectLayout(ctypes.Structure):
    _fields_ = ([(k, ctypes.c_int32) for k in
                 ("N", "H", "W", "Cin", "Cout", "group_size", "groups", "P", "Cout_pad", "kstep",
                  "splits", "taps", "weight_bits", "reserved")] +
                [(k, ctypes.c_uint64) for k in
                 ("blob_bytes", "blob_Wq_off", "blob_sW_off", "blob_bias_off",
                  "ws_bytes", "ws_xq_off", "ws_sx_off", "ws_part_off")])


# wq_k2_variant_t (include/wq.h): the kernel instance of stages 2+3
K2_VARIANTS = {"auto": -1, "fused_16x16": 0, "fused_ksplit": 1, "fused_32x16": 2, "fused_32x32": 3,
               "gemm_64x64": 10, "gemm_32x128": 11, "gemm_128x128": 12,
               "lds_full_64x64": 20, "lds_full_32x64": 21, "lds_full_32x32": 22, "lds_row_64x64": 30, "lds_row_32x64": 31,
               "lds_tap_64x64": 40, "lds_tap_128x128": 41}
K2_VARIANT_NAMES = {v: k for k, v in K2_VARIANTS.items()}


class WqError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {STATUS_NAMES.get(status, status)} ({status_string(status)})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load libwq.so; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run __graft_entry__.build() "
                              "(python -m paper_2412_19867_amd.build)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, ip = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        L.wq_standard_transforms.argtypes = [ip, vp, vp, vp]
        L.wq_scaled_transforms.argtypes = [ip, vp, vp, vp, vp, vp]
        L.wq_plan_create.argtypes = [ctypes.POINTER(vp), ip, ip, ip, ip, ip, ip, ip, vp, vp, vp]
        L.wq_plan_tune.argtypes = [vp, ip, ip]
        L.wq_plan_set_integer_transforms.argtypes = [vp, ip]
        L.wq_conv_forward_debug_slab.argtypes = [vp, vp, vp, vp, sz, vp, sz, vp, vp, sz, ip, ip, ip, ip]
        L.wq_direct_plan_tune.argtypes = [vp, ip]
        L.wq_plan_destroy.argtypes = [vp]
        L.wq_plan_layout.argtypes = [vp, ctypes.POINTER(Layout)]
        L.wq_weight_prepare.argtypes = [vp, vp, vp, vp, vp, sz]
        L.wq_input_transform.argtypes = [vp, vp, vp, vp, sz]
        L.wq_contract_output.argtypes = [vp, vp, vp, sz, vp, sz, vp]
        L.wq_contract_output_part.argtypes = [vp, vp, vp, sz, vp, sz, vp, ip]
        L.wq_contract.argtypes = [vp, vp, vp, sz, vp, sz]
        L.wq_microbench_dequant.argtypes = [vp, ip, ip, ip, ip, ip, vp, vp, vp]
        L.wq_output_transform.argtypes = [vp, vp, vp, sz, vp, sz, vp]
        L.wq_conv_forward.argtypes = [vp, vp, vp, vp, sz, vp, sz, vp]
        L.wq_conv_forward_static.argtypes = [vp, vp, vp, vp, sz, vp]
        L.wq_conv_forward_debug.argtypes = [vp, vp, vp, vp, sz, vp, sz, vp, vp, sz]
        L.wq_direct_plan_create.argtypes = [ctypes.POINTER(vp), ip, ip, ip, ip, ip, ip]
        L.wq_linear_plan_create.argtypes = [ctypes.POINTER(vp), ip, ip, ip, ip]
        L.wq_direct_plan_create_bits.argtypes = [ctypes.POINTER(vp), ip, ip, ip, ip, ip, ip, ip]
        L.wq_linear_plan_create_bits.argtypes = [ctypes.POINTER(vp), ip, ip, ip, ip, ip]
        L.wq_direct_plan_destroy.argtypes = [vp]
        L.wq_direct_plan_layout.argtypes = [vp, ctypes.POINTER(DirectLayout)]
        L.wq_direct_weight_prepare.argtypes = [vp, vp, vp, vp, vp, sz]
        L.wq_direct_quantize.argtypes = [vp, vp, vp, vp, sz]
        L.wq_direct_conv.argtypes = [vp, vp, vp, sz, vp, sz, vp]
        L.wq_direct_forward.argtypes = [vp, vp, vp, vp, sz, vp, sz, vp]
        L.wq_status_string.argtypes = [ip]
        L.wq_status_string.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name != "wq_status_string":
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().wq_status_string(int(status)).decode()


def _check(status: int, what: str):
    if status != WQ_OK:
        raise WqError(status, what)


def standard_transforms(m: int):
    """The library's standard (A^T, B^T, G) as float64 arrays."""
    n = m + 2
    BT, G, AT = np.empty((n, n)), np.empty((n, 3)), np.empty((m, n))
    _check(lib().wq_standard_transforms(m, BT.ctypes.data, G.ctypes.data, AT.ctypes.data),
           "wq_standard_transforms")
    return AT, BT, G


def scaled_transforms(m: int, u_B, u_G):
    """(A^T, B^T, G) in fp32 with learned diagonal scales applied to the standard matrices
    (wq_scaled_transforms: rows of B^T by u_B, rows of G by u_G, columns of A^T by
    1/(u_B u_G))."""
    n = m + 2
    u_B, u_G = np.ascontiguousarray(u_B, np.float64), np.ascontiguousarray(u_G, np.float64)
    if u_B.shape != (n,) or u_G.shape != (n,):
        raise ValueError("need one scale per row of B^T and of G")
    BT, G, AT = (np.empty((n, n), np.float32), np.empty((n, 3), np.float32),
                 np.empty((m, n), np.float32))
    _check(lib().wq_scaled_transforms(m, u_B.ctypes.data, u_G.ctypes.data, BT.ctypes.data,
                                      G.ctypes.data, AT.ctypes.data), "wq_scaled_transforms")
    return AT, BT, G


def _stream_handle(stream) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _dev_ptr(t, dtype, what: str, numel: Optional[int] = None) -> int:
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{what}: expected a device tensor")
    if t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{what}: expected contiguous {dtype}")
    if numel is not None and t.numel() != numel:
        raise ValueError(f"{what}: expected {numel} elements, got {t.numel()}")
    return t.data_ptr()


class Plan:
    """One layer shape.  Owns only the host-side plan object."""

    def __init__(self, N, H, W, Cin, Cout, m, group_size, AT=None, BT=None, G=None):
        self._h = ctypes.c_void_p()
        mats = [None, None, None]
        if AT is not None or BT is not None or G is not None:
            mats = [np.ascontiguousarray(a, np.float32) if a is not None else None
                    for a in (BT, G, AT)]
            n = m + 2
            for a, shp in zip(mats, ((n, n), (n, 3), (m, n))):
                if a is not None and a.shape != shp:
                    raise ValueError(f"transform matrix shape {a.shape}, expected {shp}")
        self._mats = mats  # keep alive during the call
        ptrs = [a.ctypes.data if a is not None else None for a in mats]
        _check(lib().wq_plan_create(ctypes.byref(self._h), N, H, W, Cin, Cout, m, group_size, *ptrs),
               "wq_plan_create")
        self.layout = Layout()
        _check(lib().wq_plan_layout(self._h, ctypes.byref(self.layout)), "wq_plan_layout")

    def __del__(self):
        h = getattr(self, "_h", None)
        if h and _lib is not None:
            _lib.wq_plan_destroy(h)
            self._h = None

    def tune(self, k1_rows: int = 0, k2_variant=-1):
        """Override the plan's kernel choices (wq_plan_tune); k2_variant by number or name."""
        v = K2_VARIANTS[k2_variant] if isinstance(k2_variant, str) else int(k2_variant)
        _check(lib().wq_plan_tune(self._h, int(k1_rows), v), "wq_plan_tune")
        _check(lib().wq_plan_layout(self._h, ctypes.byref(self.layout)), "wq_plan_layout")
        return self

    def set_integer_transforms(self, mode: int = 1):
        """Fully-integer input and output transforms (wq_plan_set_integer_transforms): 0 off,
        1 one scale per transform matrix, 2 one scale per matrix row."""
        _check(lib().wq_plan_set_integer_transforms(self._h, int(mode)), "wq_plan_set_integer_transforms")
        _check(lib().wq_plan_layout(self._h, ctypes.byref(self.layout)), "wq_plan_layout")
        return self

    @property
    def k2_variant_name(self) -> str:
        return K2_VARIANT_NAMES.get(self.layout.k2_variant, str(self.layout.k2_variant))

    # ---- buffers (device memory comes from torch) ----
    def alloc_blob(self, device="cuda"):
        import torch
        return torch.empty(self.layout.blob_bytes, dtype=torch.uint8, device=device)

    def alloc_workspace(self, device="cuda"):
        import torch
        return torch.empty(self.layout.ws_bytes, dtype=torch.uint8, device=device)

    def alloc_output(self, device="cuda"):
        import torch
        L = self.layout
        return torch.empty((L.N, L.H, L.W, L.Cout), dtype=torch.float32, device=device)

    def alloc_debug_P(self, device="cuda"):
        import torch
        L = self.layout
        return torch.empty((L.n * L.n, L.T, L.groups, L.Cout), dtype=torch.int32, device=device)

    # ---- views of the library's formats (for tests): pure index permutations ----
    def _unblock(self, flat, rows):
        """[n*n][rows/16][Cin/kstep][4][16][kstep/4] -> [n*n][rows][Cin]"""
        L = self.layout
        n2, ks = L.n * L.n, L.kstep
        v = flat.view(n2, rows // 16, L.Cin // ks, 4, 16, ks // 4)
        return v.permute(0, 1, 4, 2, 3, 5).reshape(n2, rows, L.Cin)

    def blob_views(self, blob):
        """(Wq [n*n][Cout_pad][Cin] int8, sW [n*n][groups][Cout_pad] fp32, bias [Cout_pad])"""
        import torch
        L = self.layout
        n2 = L.n * L.n
        Wq = self._unblock(blob[L.blob_Wq_off:L.blob_Wq_off + n2 * L.Cout_pad * L.Cin]
                           .view(torch.int8), L.Cout_pad)
        sW = blob[L.blob_sW_off:L.blob_sW_off + n2 * L.groups * L.Cout_pad * 4].view(torch.float32) \
            .view(n2, L.groups, L.Cout_pad)
        bias = blob[L.blob_bias_off:L.blob_bias_off + L.Cout_pad * 4].view(torch.float32)
        return Wq, sW, bias

    def workspace_views(self, ws):
        """(Xq [n*n][T_pad][Cin] int8, sX [n*n][T_pad][groups] fp32)"""
        import torch
        L = self.layout
        n2 = L.n * L.n
        Xq = self._unblock(ws[L.ws_Xq_off:L.ws_Xq_off + n2 * L.T_pad * L.Cin].view(torch.int8),
                           L.T_pad)
        sX = ws[L.ws_sX_off:L.ws_sX_off + n2 * L.T_pad * L.groups * 4].view(torch.float32) \
            .view(n2, L.T_pad // 16, L.groups, 16).permute(0, 1, 3, 2).reshape(n2, L.T_pad, L.groups)
        return Xq, sX

    def product_view(self, ws):
        """M [n*n][T][Cout] fp32: the dequantized Winograd-domain products wq_contract left
        in the workspace (a strided view, no copy)."""
        import torch
        L = self.layout
        n2 = L.n * L.n
        M = ws[L.ws_M_off:L.ws_M_off + n2 * L.T_pad * L.Cout_pad * 4].view(torch.float32) \
            .view(L.T_pad, n2, L.Cout_pad)
        return M[:L.T, :, :L.Cout].permute(1, 0, 2)

    # ---- entry points ----
    def weight_prepare(self, w, bias, blob, stream=None):
        import torch
        L = self.layout
        wp = _dev_ptr(w, torch.float32, "w", L.Cout * L.Cin * 9)
        bp = None if bias is None else _dev_ptr(bias, torch.float32, "bias", L.Cout)
        _check(lib().wq_weight_prepare(self._h, _stream_handle(stream), wp, bp,
                                       _dev_ptr(blob, torch.uint8, "blob"), blob.numel()),
               "wq_weight_prepare")

    def input_transform(self, x, ws, stream=None):
        import torch
        L = self.layout
        _check(lib().wq_input_transform(self._h, _stream_handle(stream),
                                        _dev_ptr(x, torch.float32, "x", L.N * L.H * L.W * L.Cin),
                                        _dev_ptr(ws, torch.uint8, "workspace"), ws.numel()),
               "wq_input_transform")

    def contract_output(self, ws, blob, y, stream=None):
        import torch
        L = self.layout
        _check(lib().wq_contract_output(self._h, _stream_handle(stream),
                                        _dev_ptr(ws, torch.uint8, "workspace"), ws.numel(),
                                        _dev_ptr(blob, torch.uint8, "blob"), blob.numel(),
                                        _dev_ptr(y, torch.float32, "y", L.N * L.H * L.W * L.Cout)),
               "wq_contract_output")

    def contract_output_part(self, ws, blob, y, part, stream=None):
        import torch
        L = self.layout
        _check(lib().wq_contract_output_part(self._h, _stream_handle(stream),
                                             _dev_ptr(ws, torch.uint8, "workspace"), ws.numel(),
                                             _dev_ptr(blob, torch.uint8, "blob"), blob.numel(),
                                             _dev_ptr(y, torch.float32, "y", L.N * L.H * L.W * L.Cout), int(part)),
               "wq_contract_output_part")

    def contract(self, ws, blob, stream=None):
        import torch
        _check(lib().wq_contract(self._h, _stream_handle(stream),
                                 _dev_ptr(ws, torch.uint8, "workspace"), ws.numel(),
                                 _dev_ptr(blob, torch.uint8, "blob"), blob.numel()),
               "wq_contract")

    def output_transform(self, ws, blob, y, stream=None):
        import torch
        L = self.layout
        _check(lib().wq_output_transform(self._h, _stream_handle(stream),
                                         _dev_ptr(ws, torch.uint8, "workspace"), ws.numel(),
                                         _dev_ptr(blob, torch.uint8, "blob"), blob.numel(),
                                         _dev_ptr(y, torch.float32, "y", L.N * L.H * L.W * L.Cout)),
               "wq_output_transform")

    def forward(self, x, blob, ws, y, stream=None):
        import torch
        L = self.layout
        _check(lib().wq_conv_forward(self._h, _stream_handle(stream),
                                     _dev_ptr(x, torch.float32, "x", L.N * L.H * L.W * L.Cin),
                                     _dev_ptr(blob, torch.uint8, "blob"), blob.numel(),
                                     _dev_ptr(ws, torch.uint8, "workspace"), ws.numel(),
                                     _dev_ptr(y, torch.float32, "y", L.N * L.H * L.W * L.Cout)),
               "wq_conv_forward")

    def forward_static(self, x, blob, y, stream=None):
        """wq_conv_forward_static: the library's own static workspace, nothing allocated."""
        import torch
        L = self.layout
        _check(lib().wq_conv_forward_static(self._h, _stream_handle(stream),
                                            _dev_ptr(x, torch.float32, "x", L.N * L.H * L.W * L.Cin),
                                            _dev_ptr(blob, torch.uint8, "blob"), blob.numel(),
                                            _dev_ptr(y, torch.float32, "y", L.N * L.H * L.W * L.Cout)),
               "wq_conv_forward_static")

    def forward_debug(self, x, blob, ws, y, P, stream=None):
        import torch
        L = self.layout
        _check(lib().wq_conv_forward_debug(self._h, _stream_handle(stream),
                                           _dev_ptr(x, torch.float32, "x", L.N * L.H * L.W * L.Cin),
                                           _dev_ptr(blob, torch.uint8, "blob"), blob.numel(),
                                           _dev_ptr(ws, torch.uint8, "workspace"), ws.numel(),
                                           _dev_ptr(y, torch.float32, "y", L.N * L.H * L.W * L.Cout),
                                           _dev_ptr(P, torch.int32, "P"), P.numel() * 4),
               "wq_conv_forward_debug")


    def _forward_debug_slab(self, x, blob, ws, y, P, tap0, ntaps, tile0, ntiles, stream=None):
        import torch
        L = self.layout
        _check(lib().wq_conv_forward_debug_slab(
            self._h, _stream_handle(stream), _dev_ptr(x, torch.float32, "x", L.N * L.H * L.W * L.Cin),
            _dev_ptr(blob, torch.uint8, "blob"), blob.numel(), _dev_ptr(ws, torch.uint8, "workspace"),
            ws.numel(), _dev_ptr(y, torch.float32, "y", L.N * L.H * L.W * L.Cout),
            _dev_ptr(P, torch.int32, "P"), P.numel() * 4, tap0, ntaps, tile0, ntiles),
            "wq_conv_forward_debug_slab")

    def forward_debug_slab(self, x, blob, ws, y, tap0, ntaps, tile0, ntiles, stream=None):
        """Forward pass that also returns P[tap0:tap0+ntaps, tile0:tile0+ntiles] (int32 device tensor)."""
        import torch
        L = self.layout
        P = torch.empty((ntaps, ntiles, L.groups, L.Cout), dtype=torch.int32, device=x.device)
        self._forward_debug_slab(x, blob, ws, y, P, tap0, ntaps, tile0, ntiles, stream)
        return P


def microbench_dequant(mode: int, group_size: int, blocks_per_wave: int, workgroups: int, iters: int,
                       stream=None):
    """Runs wq_microbench_dequant once; returns the per-workgroup (cycle-counter, 100 MHz wall-clock)
    tick counts of the loop as a [workgroups, 2] device tensor."""
    import torch
    seed = torch.arange(64, dtype=torch.int32, device="cuda")
    out = torch.empty(workgroups * 256, dtype=torch.float32, device="cuda")
    cyc = torch.zeros((workgroups, 2), dtype=torch.int64, device="cuda")
    _check(lib().wq_microbench_dequant(_stream_handle(stream), mode, group_size, blocks_per_wave, workgroups,
                                       iters, seed.data_ptr(), out.data_ptr(), cyc.data_ptr()),
           "wq_microbench_dequant")
    return cyc


class DirectPlan:
    """The group-wise quantized standard 3x3 convolution (the paper's runtime
    comparison point) for one layer shape.  Owns only the host-side plan object."""

    def __init__(self, N, H, W, Cin, Cout, group_size, linear: bool = False, weight_bits: int = 8):
        self._h = ctypes.c_void_p()
        if linear:   # N rows, H = W = 1: a group-wise quantized linear layer
            _check(lib().wq_linear_plan_create_bits(ctypes.byref(self._h), N * H * W, Cin, Cout, group_size,
                                                    weight_bits), "wq_linear_plan_create_bits")
        else:
            _check(lib().wq_direct_plan_create_bits(ctypes.byref(self._h), N, H, W, Cin, Cout, group_size,
                                                    weight_bits), "wq_direct_plan_create_bits")
        self.layout = DirectLayout()
        _check(lib().wq_direct_plan_layout(self._h, ctypes.byref(self.layout)), "wq_direct_plan_layout")

    def tune(self, splits: int):
        """Override how many workgroups share an output tile's reduction (wq_direct_plan_tune)."""
        _check(lib().wq_direct_plan_tune(self._h, int(splits)), "wq_direct_plan_tune")
        _check(lib().wq_direct_plan_layout(self._h, ctypes.byref(self.layout)), "wq_direct_plan_layout")
        return self

    def __del__(self):
        h = getattr(self, "_h", None)
        if h and _lib is not None:
            _lib.wq_direct_plan_destroy(h)
            self._h = None

    def alloc_blob(self, device="cuda"):
        import torch
        return torch.empty(self.layout.blob_bytes, dtype=torch.uint8, device=device)

    def alloc_workspace(self, device="cuda"):
        import torch
        return torch.empty(self.layout.ws_bytes, dtype=torch.uint8, device=device)

    def alloc_output(self, device="cuda"):
        import torch
        L = self.layout
        return torch.empty((L.N, L.H, L.W, L.Cout), dtype=torch.float32, device=device)

    def blob_views(self, blob):
        """(Wq [taps][Cout_pad][Cin] int8, sW [taps][groups][Cout_pad] fp32, bias [Cout_pad]) - the
        int8 tensor un-blocked (a pure index permutation)."""
        import torch
        L = self.layout
        R, ks, nt = L.Cout_pad, L.kstep, L.taps
        if L.weight_bits == 4:   # two codes per byte: back to one int8 per code, same blocked order
            pk = blob[L.blob_Wq_off:L.blob_Wq_off + nt * R * L.Cin // 2].view(-1, 2, 4)   # pieces p0 p1
            lo = ((pk & 0x0f) ^ 0x08).to(torch.int16) - 8      # sign-extend the low nibbles: d0, d2
            hi = ((pk >> 4) ^ 0x08).to(torch.int16) - 8        # and the high ones: d1, d3
            raw = torch.stack((lo, hi), dim=2).to(torch.int8).reshape(-1)   # d0 d1 d2 d3 per piece
        else:
            raw = blob[L.blob_Wq_off:L.blob_Wq_off + nt * R * L.Cin].view(torch.int8)
        Wq = raw.view(nt, R // 16, L.Cin // ks, 4, 16, ks // 4).permute(0, 1, 4, 2, 3, 5) \
            .reshape(nt, R, L.Cin)
        sW = blob[L.blob_sW_off:L.blob_sW_off + nt * L.groups * R * 4].view(torch.float32) \
            .view(nt, L.groups, R)
        bias = blob[L.blob_bias_off:L.blob_bias_off + R * 4].view(torch.float32)
        return Wq, sW, bias

    def workspace_views(self, ws):
        """(xq [P][Cin] int8, sx [P][groups] fp32)"""
        import torch
        L = self.layout
        xq = ws[L.ws_xq_off:L.ws_xq_off + L.P * L.Cin].view(torch.int8).view(L.P, L.Cin)
        sx = ws[L.ws_sx_off:L.ws_sx_off + L.P * L.groups * 4].view(torch.float32).view(L.P, L.groups)
        return xq, sx

    def weight_prepare(self, w, bias, blob, stream=None):
        import torch
        L = self.layout
        wp = _dev_ptr(w, torch.float32, "w", L.Cout * L.Cin * L.taps)
        bp = None if bias is None else _dev_ptr(bias, torch.float32, "bias", L.Cout)
        _check(lib().wq_direct_weight_prepare(self._h, _stream_handle(stream), wp, bp,
                                              _dev_ptr(blob, torch.uint8, "blob"), blob.numel()),
               "wq_direct_weight_prepare")

    def quantize(self, x, ws, stream=None):
        import torch
        L = self.layout
        _check(lib().wq_direct_quantize(self._h, _stream_handle(stream),
                                        _dev_ptr(x, torch.float32, "x", L.P * L.Cin),
                                        _dev_ptr(ws, torch.uint8, "workspace"), ws.numel()),
               "wq_direct_quantize")

    def conv(self, ws, blob, y, stream=None):
        import torch
        L = self.layout
        _check(lib().wq_direct_conv(self._h, _stream_handle(stream),
                                    _dev_ptr(ws, torch.uint8, "workspace"), ws.numel(),
                                    _dev_ptr(blob, torch.uint8, "blob"), blob.numel(),
                                    _dev_ptr(y, torch.float32, "y", L.P * L.Cout)),
               "wq_direct_conv")

    def forward(self, x, blob, ws, y, stream=None):
        import torch
        L = self.layout
        _check(lib().wq_direct_forward(self._h, _stream_handle(stream),
                                       _dev_ptr(x, torch.float32, "x", L.P * L.Cin),
                                       _dev_ptr(blob, torch.uint8, "blob"), blob.numel(),
                                       _dev_ptr(ws, torch.uint8, "workspace"), ws.numel(),
                                       _dev_ptr(y, torch.float32, "y", L.P * L.Cout)),
               "wq_direct_forward")
