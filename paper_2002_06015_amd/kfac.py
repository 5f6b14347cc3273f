"""Python binding of the C-ABI HIP library (``include/kfac.h``): argument marshalling only.

torch is used for device memory and the stream handle; every step of the path runs
in the HIP kernels of ``libkfac_hip.so``.  There is no CPU fallback: if the library
is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import contextlib
import ctypes
import os
from typing import List, Optional, Sequence


import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkfac_hip.so")

KFAC_OK, KFAC_ERR_INVALID, KFAC_ERR_WORKSPACE, KFAC_ERR_NOT_PD, KFAC_ERR_DEVICE = range(5)
KFAC_F32, KFAC_BF16 = 0, 1

EXPORTS = [
    "kfac_status_string", "kfac_layer_dims", "kfac_workspace_bytes", "kfac_create", "kfac_destroy",
    "kfac_options_default", "kfac_workspace_bytes_opt", "kfac_create_opt", "kfac_step_workspace_bytes",
    "kfac_im2col", "kfac_stats", "kfac_invert", "kfac_precondition", "kfac_step",
    "bn_unitwise_precondition", "bn_unitwise_reduce_nchw", "bn_unitwise_reduce_nhwc", "kfac_profile_enable", "kfac_profile_read",
    "kfac_packed_elems", "kfac_pack_upper", "kfac_unpack_upper",
    "kfac_lr_polynomial", "kfac_momentum_coupled", "kfac_update_weights",
    "bn_full_workspace_bytes", "bn_full_precondition", "kfac_nhwc_to_nchw", "kfac_stats_nhwc", "kfac_step_nhwc",
    "kfac_staleness", "kfac_staleness_static", "kfac_next_interval", "kfac_refresh_init", "kfac_refresh_due", "kfac_refresh_advance",
]

KERNEL_NAMES = ["gemm_f32", "gemm_bf16", "gemm_reduce", "patch", "trace", "copy_damp", "leaf_inverse", "zero",
                "bn_unit", "bn_reduce", "pad", "assemble", "border", "staleness", "pack", "update", "bn_full", "layout", "gemm_f32_split"]


class kfac_profile_entry(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int32), ("variant", ctypes.c_int32), ("workgroups", ctypes.c_int32),
                ("ms", ctypes.c_float), ("flops", ctypes.c_double), ("bytes", ctypes.c_double),
                ("start_ms", ctypes.c_float), ("stream", ctypes.c_int32)]


KFAC_PRODUCTS_SPLIT_BF16, KFAC_PRODUCTS_FP32_MFMA = 0, 1


class kfac_options(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("struct_size", "fp32_products", "streams", "staging_slots", "correlation_form", "pipeline_phases",
                 "early_n", "target_workgroups", "min_k_per_split", "max_k_per_workgroup", "recursion_leaf",
                 "force_tile", "group_by_depth")] + [("chunk_gflop", ctypes.c_float)]


def options(**fields) -> kfac_options:
    """The library's default options with the given fields replaced."""
    o = kfac_options()
    lib().kfac_options_default(ctypes.addressof(o))
    for k, v in fields.items():
        if not hasattr(o, k):
            raise ValueError("unknown option %r" % k)
        setattr(o, k, v)
    return o


_default_opts: Optional[kfac_options] = None


@contextlib.contextmanager
def default_options(**fields):
    """Within the block, contexts created (and workspaces sized) without explicit options take these
    instead of the library's defaults.  A convenience of this binding; the library itself has no such state."""
    global _default_opts
    prev, _default_opts = _default_opts, options(**fields)
    try:
        yield _default_opts
    finally:
        _default_opts = prev


class kfac_layer(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "c_in", "c_out", "k", "stride", "pad", "h_in", "w_in", "bias")]


class KfacError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (where, status_string(status), status))


_lib = None


def lib() -> ctypes.CDLL:
    """Loads the HIP library built in-tree (``python -m paper_2002_06015_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("HIP library %s is not built; run __graft_entry__.build()" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float
        L.kfac_status_string.restype = ctypes.c_char_p
        L.kfac_status_string.argtypes = [ctypes.c_int]
        L.kfac_layer_dims.argtypes = [vp, vp, vp, vp, vp]
        L.kfac_workspace_bytes.restype = ctypes.c_size_t
        L.kfac_workspace_bytes.argtypes = [vp, i32, ctypes.c_int]
        L.kfac_create.argtypes = [vp, vp, vp, ctypes.c_size_t]
        L.kfac_create_opt.argtypes = [vp, vp, vp, ctypes.c_size_t, vp]
        L.kfac_options_default.restype = None
        L.kfac_options_default.argtypes = [vp]
        L.kfac_workspace_bytes_opt.restype = ctypes.c_size_t
        L.kfac_workspace_bytes_opt.argtypes = [vp, i32, ctypes.c_int, vp]
        L.kfac_step_workspace_bytes.restype = ctypes.c_size_t
        L.kfac_step_workspace_bytes.argtypes = [vp, i32, ctypes.c_int, vp, vp]
        L.kfac_destroy.restype = None
        L.kfac_destroy.argtypes = [vp]
        L.kfac_im2col.argtypes = [vp, vp, ctypes.c_int, vp, vp, ctypes.c_int64]
        L.kfac_stats.argtypes = [vp, i32, vp, ctypes.c_int, vp, vp, f32, i32, vp, vp]
        L.kfac_stats_nhwc.argtypes = L.kfac_stats.argtypes
        L.kfac_invert.argtypes = [vp, i32, vp, vp, vp, f32, vp, vp, vp, vp]
        L.kfac_precondition.argtypes = [vp, i32, vp, vp, vp, vp, vp]
        L.kfac_step.argtypes = [vp, i32, vp, ctypes.c_int, vp, vp, f32, i32, vp, vp, vp, f32, vp, vp, vp, vp, vp, vp]
        L.kfac_step_nhwc.argtypes = L.kfac_step.argtypes
        L.bn_unitwise_precondition.argtypes = [vp, i32, i32, vp, vp, vp, f32, f32, vp, vp, vp]
        L.bn_unitwise_reduce_nchw.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp]
        L.bn_unitwise_reduce_nhwc.argtypes = L.bn_unitwise_reduce_nchw.argtypes
        L.kfac_profile_enable.argtypes = [vp, i32]
        L.kfac_profile_read.restype = i32
        L.kfac_profile_read.argtypes = [vp, vp, i32]
        L.kfac_nhwc_to_nchw.argtypes = [vp, i32, vp, i32, i32, vp, vp]
        L.bn_full_workspace_bytes.restype = ctypes.c_size_t
        L.bn_full_workspace_bytes.argtypes = [i32, i32, vp]
        L.bn_full_precondition.argtypes = [vp, i32, i32, vp, vp, vp, f32, f32, vp, vp, vp, vp, vp, vp]
        f64 = ctypes.c_double
        L.kfac_lr_polynomial.restype = f64
        L.kfac_lr_polynomial.argtypes = [f64, f64, f64, f64, f64]
        L.kfac_momentum_coupled.restype = f64
        L.kfac_momentum_coupled.argtypes = [f64, f64, f64]
        L.kfac_update_weights.argtypes = [vp, i32, vp, vp, f32, f32, i32, f32, vp, vp]
        L.kfac_packed_elems.restype = ctypes.c_size_t
        L.kfac_packed_elems.argtypes = [i32, vp]
        L.kfac_pack_upper.argtypes = [vp, i32, vp, vp, ctypes.c_int, vp]
        L.kfac_unpack_upper.argtypes = [vp, i32, vp, ctypes.c_int, vp, vp]
        L.kfac_staleness.argtypes = [vp, i32, vp, vp, vp, vp, vp]
        L.kfac_staleness_static.argtypes = [vp, i32, vp, vp, vp, vp, vp]
        L.kfac_next_interval.restype = i32
        L.kfac_next_interval.argtypes = [i32, i32, i32, i32]
        L.kfac_refresh_init.restype = None
        L.kfac_refresh_init.argtypes = [vp, i32]
        L.kfac_refresh_due.restype = i32
        L.kfac_refresh_due.argtypes = [vp, i32]
        L.kfac_refresh_advance.restype = None
        L.kfac_refresh_advance.argtypes = [vp, ctypes.c_double, ctypes.c_double, ctypes.c_double]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().kfac_status_string(int(status)).decode()


def _layers(layers: Sequence) -> ctypes.Array:
    arr = (kfac_layer * len(layers))()
    for i, L in enumerate(layers):
        arr[i] = kfac_layer(*[int(v) for v in L])
    return arr


def _ptrs(tensors: Optional[Sequence[Optional[torch.Tensor]]], n: int, dtype=None,
          numels: Optional[Sequence[int]] = None, what: str = "tensor") -> Optional[ctypes.Array]:
    """Host array of device pointers; None entries become NULL; None list becomes NULL.
    numels: the element count the library will read or write behind each pointer; a smaller
    tensor is refused here (the library sees only the pointer)."""
    if tensors is None:
        return None
    if len(tensors) != n:
        raise ValueError("expected %d %ss, got %d" % (n, what, len(tensors)))
    arr = (ctypes.c_void_p * n)()
    for i, t in enumerate(tensors):
        if t is None:
            arr[i] = None
            continue
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("%s %d must be a contiguous device tensor" % (what, i))
        if dtype is not None and t.dtype != dtype:
            raise ValueError("%s %d must be %s" % (what, i, dtype))
        if numels is not None and t.numel() < int(numels[i]):
            raise ValueError("%s %d has %d elements, the layer needs %d" % (what, i, t.numel(), int(numels[i])))
        arr[i] = t.data_ptr()
    return arr


_sizes_cache: dict = {}


def _sizes(layers: Sequence) -> dict:
    """Element counts of the per-layer tensors, from the library's own kfac_layer_dims (kept per layer
    list: a training loop passes the same list every step)."""
    key = tuple(tuple(int(v) for v in L) for L in layers)
    hit = _sizes_cache.get(key)
    if hit is not None:
        return hit
    if len(_sizes_cache) > 64:
        _sizes_cache.clear()
    out = _sizes_cache[key] = {"act": [], "grad_out": [], "A": [], "G": [], "W": []}
    for L in layers:
        dA, dG, h, w = kfac_layer_dims(L)
        N, c_in, c_out, _, _, _, h_in, w_in, _ = [int(v) for v in L]
        out["act"].append(N * c_in * h_in * w_in)
        out["grad_out"].append(N * c_out * h * w)
        out["A"].append(dA * dA)
        out["G"].append(dG * dG)
        out["W"].append(dG * dA)
    return out


def _i32(values: Sequence[int]) -> ctypes.Array:
    return (ctypes.c_int32 * len(values))(*[int(v) for v in values])


def kfac_layer_dims(layer) -> tuple:
    L = kfac_layer(*[int(v) for v in layer])
    out = [ctypes.c_int32() for _ in range(4)]
    st = lib().kfac_layer_dims(ctypes.addressof(L), *[ctypes.addressof(o) for o in out])
    if st != KFAC_OK:
        raise KfacError(st, "kfac_layer_dims")
    return tuple(o.value for o in out)


def kfac_workspace_bytes(layers: Sequence, in_dtype: int = KFAC_F32, opts: Optional[kfac_options] = None) -> int:
    arr = _layers(layers)
    opts = opts if opts is not None else _default_opts
    return int(lib().kfac_workspace_bytes_opt(ctypes.addressof(arr), len(layers), int(in_dtype),
                                              None if opts is None else ctypes.addressof(opts)))


def kfac_step_workspace_bytes(layers: Sequence, in_dtype: int = KFAC_F32, invert_mask: Optional[Sequence[bool]] = None,
                              opts: Optional[kfac_options] = None) -> int:
    arr = _layers(layers)
    mask = None if invert_mask is None else (ctypes.c_uint8 * len(layers))(*[1 if m else 0 for m in invert_mask])
    return int(lib().kfac_step_workspace_bytes(ctypes.addressof(arr), len(layers), int(in_dtype),
                                               None if mask is None else ctypes.addressof(mask),
                                               None if opts is None else ctypes.addressof(opts)))


class Context:
    """kfac_create/kfac_destroy with a torch-allocated workspace on the current device and
    torch's current stream."""

    def __init__(self, layers: Sequence, in_dtype: int = KFAC_F32, extra_layer_lists: Sequence[Sequence] = (),
                 workspace_bytes: Optional[int] = None, stream: Optional[torch.cuda.Stream] = None,
                 opts: Optional[kfac_options] = None):
        opts = opts if opts is not None else _default_opts
        need = kfac_workspace_bytes(layers, in_dtype, opts)
        if need == 0:
            raise KfacError(KFAC_ERR_INVALID, "kfac_workspace_bytes")
        for other in extra_layer_lists:
            need = max(need, kfac_workspace_bytes(other, in_dtype, opts))
        if workspace_bytes is not None:
            need = int(workspace_bytes)
        self.workspace = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
        base = (self.workspace.data_ptr() + 255) // 256 * 256
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        handle = ctypes.c_void_p()
        st = lib().kfac_create_opt(ctypes.addressof(handle), ctypes.c_void_p(self.stream.cuda_stream),
                                   ctypes.c_void_p(base), need, None if opts is None else ctypes.addressof(opts))
        if st != KFAC_OK:
            raise KfacError(st, "kfac_create")
        self.handle = handle

    def close(self):
        if getattr(self, "handle", None) is not None and self.handle.value:
            lib().kfac_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _tdtype(in_dtype: int):
    return torch.bfloat16 if in_dtype == KFAC_BF16 else torch.float32


def kfac_im2col(ctx: Context, layer, in_dtype: int, act: torch.Tensor, patches: torch.Tensor, ld: int) -> None:
    L = kfac_layer(*[int(v) for v in layer])
    if act.dtype != _tdtype(in_dtype) or patches.dtype != _tdtype(in_dtype):
        raise ValueError("dtype mismatch")
    dA, dG, h, w = kfac_layer_dims(layer)
    N, c_in, k = int(layer[0]), int(layer[1]), int(layer[3])
    if not (act.is_cuda and act.is_contiguous() and patches.is_cuda and patches.is_contiguous()):
        raise ValueError("act and patches must be contiguous device tensors")
    if act.numel() < N * c_in * int(layer[6]) * int(layer[7]) or int(ld) < N * h * w or patches.numel() < c_in * k * k * int(ld):
        raise ValueError("act or patches too small for the layer (need [N,c_in,h_in,w_in] and [c_in*k*k, ld], ld >= N*h*w)")
    st = lib().kfac_im2col(ctx.handle, ctypes.addressof(L), int(in_dtype), act.data_ptr(), patches.data_ptr(), int(ld))
    if st != KFAC_OK:
        raise KfacError(st, "kfac_im2col")


def kfac_stats(ctx: Context, layers: Sequence, in_dtype: int, act, grad_out, decay: float,
               g_spatial_mean: bool, A_ema, G_ema, nhwc: bool = False) -> None:
    """nhwc: act / grad_out are stored [N, H, W, C] (kfac_stats_nhwc); same element counts."""
    n = len(layers)
    arr = _layers(layers)
    sz = _sizes(layers)
    pa = _ptrs(act, n, _tdtype(in_dtype), sz["act"], "act")
    pg = _ptrs(grad_out, n, _tdtype(in_dtype), sz["grad_out"], "grad_out")
    pA, pG = _ptrs(A_ema, n, torch.float32, sz["A"], "A_ema"), _ptrs(G_ema, n, torch.float32, sz["G"], "G_ema")
    entry = lib().kfac_stats_nhwc if nhwc else lib().kfac_stats
    st = entry(ctx.handle, n, ctypes.addressof(arr), int(in_dtype),
               pa and ctypes.addressof(pa), pg and ctypes.addressof(pg),
               float(decay), int(bool(g_spatial_mean)),
               pA and ctypes.addressof(pA), pG and ctypes.addressof(pG))
    if st != KFAC_OK:
        raise KfacError(st, "kfac_stats_nhwc" if nhwc else "kfac_stats")


def kfac_invert(ctx: Context, layers: Sequence, A_ema, G_ema, gamma: float, A_inv, G_inv,
                pi_out: Optional[torch.Tensor] = None, info: Optional[torch.Tensor] = None) -> None:
    n = len(layers)
    arr = _layers(layers)
    sz = _sizes(layers)
    pA, pG = _ptrs(A_ema, n, torch.float32, sz["A"], "A_ema"), _ptrs(G_ema, n, torch.float32, sz["G"], "G_ema")
    pAi, pGi = _ptrs(A_inv, n, torch.float32, sz["A"], "A_inv"), _ptrs(G_inv, n, torch.float32, sz["G"], "G_inv")
    if pi_out is not None and (pi_out.dtype != torch.float32 or pi_out.numel() < n):
        raise ValueError("pi_out must be float32 [n_layers]")
    if info is not None and (info.dtype != torch.int32 or info.numel() < 2 * n):
        raise ValueError("info must be int32 [2*n_layers]")
    st = lib().kfac_invert(ctx.handle, n, ctypes.addressof(arr),
                           pA and ctypes.addressof(pA), pG and ctypes.addressof(pG), float(gamma),
                           pAi and ctypes.addressof(pAi), pGi and ctypes.addressof(pGi),
                           None if pi_out is None else pi_out.data_ptr(),
                           None if info is None else info.data_ptr())
    if st != KFAC_OK:
        raise KfacError(st, "kfac_invert")


def kfac_precondition(ctx: Context, layers: Sequence, G_inv, A_inv, grad_W, out) -> None:
    n = len(layers)
    arr = _layers(layers)
    sz = _sizes(layers)
    ps = [_ptrs(x, n, torch.float32, sz[k], w) for x, k, w in ((G_inv, "G", "G_inv"), (A_inv, "A", "A_inv"),
                                                               (grad_W, "W", "grad_W"), (out, "W", "out"))]
    st = lib().kfac_precondition(ctx.handle, n, ctypes.addressof(arr), *[p and ctypes.addressof(p) for p in ps])
    if st != KFAC_OK:
        raise KfacError(st, "kfac_precondition")


def kfac_step(ctx: Context, layers: Sequence, in_dtype: int, act, grad_out, decay: float, g_spatial_mean: bool,
              A_ema, G_ema, invert_mask: Optional[Sequence[bool]], gamma: float, A_inv, G_inv,
              pi_out: Optional[torch.Tensor], info: Optional[torch.Tensor], grad_W, out, nhwc: bool = False) -> None:
    """nhwc: act / grad_out are stored [N, H, W, C] (kfac_step_nhwc); same element counts."""
    n = len(layers)
    arr = _layers(layers)
    sz = _sizes(layers)
    ps = [_ptrs(act, n, _tdtype(in_dtype), sz["act"], "act"), _ptrs(grad_out, n, _tdtype(in_dtype), sz["grad_out"], "grad_out")]
    ps += [_ptrs(x, n, torch.float32, sz[k], w) for x, k, w in ((A_ema, "A", "A_ema"), (G_ema, "G", "G_ema"),
                                                                (A_inv, "A", "A_inv"), (G_inv, "G", "G_inv"),
                                                                (grad_W, "W", "grad_W"), (out, "W", "out"))]
    pa, pg, pA, pG, pAi, pGi, pW, pO = [p and ctypes.addressof(p) for p in ps]
    mask = None
    if invert_mask is not None:
        if len(invert_mask) != n:
            raise ValueError("invert_mask must have one entry per layer")
        mask = (ctypes.c_uint8 * n)(*[1 if m else 0 for m in invert_mask])
    if pi_out is not None and (pi_out.dtype != torch.float32 or pi_out.numel() < n):
        raise ValueError("pi_out must be float32 [n_layers]")
    if info is not None and (info.dtype != torch.int32 or info.numel() < 2 * n):
        raise ValueError("info must be int32 [2*n_layers]")
    entry = lib().kfac_step_nhwc if nhwc else lib().kfac_step
    st = entry(ctx.handle, n, ctypes.addressof(arr), int(in_dtype), pa, pg, float(decay),
               int(bool(g_spatial_mean)), pA, pG, mask and ctypes.addressof(mask), float(gamma),
               pAi, pGi, None if pi_out is None else pi_out.data_ptr(),
               None if info is None else info.data_ptr(), pW, pO)
    if st != KFAC_OK:
        raise KfacError(st, "kfac_step_nhwc" if nhwc else "kfac_step")


def bn_unitwise_precondition(ctx: Context, N: int, C: Sequence[int], g_gamma, g_beta, decay: float, lam: float,
                             F_ema, out_gamma, out_beta) -> None:
    n = len(C)
    cs = _i32(C)
    nc, c3, c1 = [int(N) * int(c) for c in C], [3 * int(c) for c in C], [int(c) for c in C]
    ps = [_ptrs(x, n, torch.float32, nc, w) for x, w in ((g_gamma, "g_gamma"), (g_beta, "g_beta"))]
    qs = [_ptrs(x, n, torch.float32, m, w) for x, m, w in ((F_ema, c3, "F_ema"), (out_gamma, c1, "out_gamma"), (out_beta, c1, "out_beta"))]
    st = lib().bn_unitwise_precondition(ctx.handle, n, int(N), ctypes.addressof(cs),
                                        *[p and ctypes.addressof(p) for p in ps], float(decay), float(lam),
                                        *[p and ctypes.addressof(p) for p in qs])
    if st != KFAC_OK:
        raise KfacError(st, "bn_unitwise_precondition")


def bn_unitwise_reduce_nchw(ctx: Context, N: int, C: Sequence[int], HW: Sequence[int], dy, xhat,
                            g_gamma, g_beta, nhwc: bool = False) -> None:
    """nhwc: dy / xhat are stored [N, HW, C] (bn_unitwise_reduce_nhwc)."""
    n = len(C)
    cs, hs = _i32(C), _i32(HW)
    big = [int(N) * int(c) * int(h) for c, h in zip(C, HW)]
    nc = [int(N) * int(c) for c in C]
    ps = [_ptrs(x, n, torch.float32, m, w) for x, m, w in ((dy, big, "dy"), (xhat, big, "xhat"), (g_gamma, nc, "g_gamma"), (g_beta, nc, "g_beta"))]
    entry = lib().bn_unitwise_reduce_nhwc if nhwc else lib().bn_unitwise_reduce_nchw
    st = entry(ctx.handle, n, int(N), ctypes.addressof(cs), ctypes.addressof(hs), *[p and ctypes.addressof(p) for p in ps])
    if st != KFAC_OK:
        raise KfacError(st, "bn_unitwise_reduce_nhwc" if nhwc else "bn_unitwise_reduce_nchw")


def bn_unitwise_reduce_nhwc(ctx: Context, N: int, C: Sequence[int], HW: Sequence[int], dy, xhat, g_gamma, g_beta) -> None:
    bn_unitwise_reduce_nchw(ctx, N, C, HW, dy, xhat, g_gamma, g_beta, nhwc=True)


def kfac_nhwc_to_nchw(ctx: Context, layers: Sequence, which: int, type_: int, src, dst) -> None:
    n = len(layers)
    ls = _layers(layers)
    szl = _sizes(layers)["act" if int(which) == 0 else "grad_out"]
    ps, pd = _ptrs(src, n, _tdtype(type_), szl, "src"), _ptrs(dst, n, _tdtype(type_), szl, "dst")
    st = lib().kfac_nhwc_to_nchw(ctx.handle, n, ctypes.addressof(ls), int(which), int(type_),
                                 ps and ctypes.addressof(ps), pd and ctypes.addressof(pd))
    if st != KFAC_OK:
        raise KfacError(st, "kfac_nhwc_to_nchw")


def bn_full_workspace_bytes(N: int, C: Sequence[int]) -> int:
    c = _i32(C)
    return int(lib().bn_full_workspace_bytes(len(C), int(N), ctypes.addressof(c)))


def bn_full_precondition(ctx: Context, N: int, C: Sequence[int], g_gamma, g_beta, decay: float, lam: float,
                         F_ema, F_inv, out_gamma, out_beta, invert_mask: Optional[Sequence[int]] = None,
                         info: Optional[torch.Tensor] = None) -> None:
    n = len(C)
    c = _i32(C)
    nc, cc, c1 = [int(N) * int(v) for v in C], [4 * int(v) * int(v) for v in C], [int(v) for v in C]
    ps = [_ptrs(x, n, torch.float32, m, w) for x, m, w in ((g_gamma, nc, "g_gamma"), (g_beta, nc, "g_beta"), (F_ema, cc, "F_ema"),
                                                           (F_inv, cc, "F_inv"), (out_gamma, c1, "out_gamma"), (out_beta, c1, "out_beta"))]
    mask = None if invert_mask is None else (ctypes.c_uint8 * n)(*[1 if m else 0 for m in invert_mask])
    if info is not None and (info.dtype != torch.int32 or info.numel() < n):
        raise ValueError("info must be int32 [n_layers]")
    ad = [p and ctypes.addressof(p) for p in ps]
    st = lib().bn_full_precondition(ctx.handle, n, int(N), ctypes.addressof(c), ad[0], ad[1], float(decay), float(lam),
                                    ad[2], None if mask is None else ctypes.addressof(mask), ad[3],
                                    None if info is None else info.data_ptr(), ad[4], ad[5])
    if st != KFAC_OK:
        raise KfacError(st, "bn_full_precondition")


def kfac_lr_polynomial(eta0: float, e: float, e_start: float, e_end: float, p_decay: float) -> float:
    return float(lib().kfac_lr_polynomial(eta0, e, e_start, e_end, p_decay))


def kfac_momentum_coupled(m0: float, eta0: float, eta: float) -> float:
    return float(lib().kfac_momentum_coupled(m0, eta0, eta))


def kfac_update_weights(ctx: Context, layers: Sequence, U, eta: float, momentum: float, rescale: bool, eps: float,
                        W, W_prev) -> None:
    n = len(layers)
    ls = _layers(layers)
    szw = _sizes(layers)["W"]
    ps = [_ptrs(x, n, torch.float32, szw, w) for x, w in ((U, "U"), (W, "W"), (W_prev, "W_prev"))]
    st = lib().kfac_update_weights(ctx.handle, n, ctypes.addressof(ls), ps[0] and ctypes.addressof(ps[0]), float(eta),
                                   float(momentum), int(bool(rescale)), float(eps), ps[1] and ctypes.addressof(ps[1]),
                                   ps[2] and ctypes.addressof(ps[2]))
    if st != KFAC_OK:
        raise KfacError(st, "kfac_update_weights")


def kfac_packed_elems(dims: Sequence[int]) -> int:
    ds = _i32(dims)
    return int(lib().kfac_packed_elems(len(dims), ctypes.addressof(ds)))


def _packed_ok(packed: torch.Tensor, dims: Sequence[int], type_: int) -> None:
    want = torch.bfloat16 if type_ == KFAC_BF16 else torch.float32
    if not (packed.is_cuda and packed.is_contiguous() and packed.dtype == want and
            packed.numel() >= kfac_packed_elems(dims)):
        raise ValueError("packed must be a contiguous device tensor of the packed type and size")


def kfac_pack_upper(ctx: Context, dims: Sequence[int], X, type_: int, packed: torch.Tensor) -> None:
    n = len(dims)
    ds, ps = _i32(dims), _ptrs(X, n, torch.float32, [int(d) * int(d) for d in dims], "X")
    _packed_ok(packed, dims, type_)
    st = lib().kfac_pack_upper(ctx.handle, n, ctypes.addressof(ds), ps and ctypes.addressof(ps), int(type_),
                               packed.data_ptr())
    if st != KFAC_OK:
        raise KfacError(st, "kfac_pack_upper")


def kfac_unpack_upper(ctx: Context, dims: Sequence[int], type_: int, packed: torch.Tensor, X) -> None:
    n = len(dims)
    ds, ps = _i32(dims), _ptrs(X, n, torch.float32, [int(d) * int(d) for d in dims], "X")
    _packed_ok(packed, dims, type_)
    st = lib().kfac_unpack_upper(ctx.handle, n, ctypes.addressof(ds), int(type_), packed.data_ptr(),
                                 ps and ctypes.addressof(ps))
    if st != KFAC_OK:
        raise KfacError(st, "kfac_unpack_upper")


def kfac_staleness(ctx: Context, dims: Sequence[int], X, X_m1, X_m2, ratios: torch.Tensor) -> None:
    """ratios: device float64 [2 * len(dims)] (contiguous)."""
    n = len(dims)
    ds = _i32(dims)
    dd = [int(d) * int(d) for d in dims]
    ps = [_ptrs(x, n, torch.float32, dd, w) for x, w in ((X, "X"), (X_m1, "X_m1"), (X_m2, "X_m2"))]
    if not (ratios.is_cuda and ratios.is_contiguous() and ratios.dtype == torch.float64 and ratios.numel() >= 2 * n):
        raise ValueError("ratios must be a contiguous device float64 tensor of at least 2 n elements")
    st = lib().kfac_staleness(ctx.handle, n, ctypes.addressof(ds), *[p and ctypes.addressof(p) for p in ps],
                              ratios.data_ptr())
    if st != KFAC_OK:
        raise KfacError(st, "kfac_staleness")


def kfac_staleness_static(stream: Optional[torch.cuda.Stream], dims: Sequence[int], X, X_m1, X_m2,
                          ratios: torch.Tensor) -> None:
    """kfac_staleness without a context: scratch in the library's fixed device array, nothing allocated."""
    n = len(dims)
    ds = _i32(dims)
    dd = [int(d) * int(d) for d in dims]
    ps = [_ptrs(x, n, torch.float32, dd, w) for x, w in ((X, "X"), (X_m1, "X_m1"), (X_m2, "X_m2"))]
    if not (ratios.is_cuda and ratios.is_contiguous() and ratios.dtype == torch.float64 and ratios.numel() >= 2 * n):
        raise ValueError("ratios must be a contiguous device float64 tensor of at least 2 n elements")
    s = stream if stream is not None else torch.cuda.current_stream()
    st = lib().kfac_staleness_static(ctypes.c_void_p(s.cuda_stream), n, ctypes.addressof(ds),
                                     *[p and ctypes.addressof(p) for p in ps], ratios.data_ptr())
    if st != KFAC_OK:
        raise KfacError(st, "kfac_staleness_static")


class kfac_refresh_state(ctypes.Structure):
    _fields_ = [("t_next", ctypes.c_int32), ("delta", ctypes.c_int32), ("delta_m1", ctypes.c_int32)]


def kfac_next_interval(similar_to_last: bool, similar_to_before_last: bool, delta_m1: int, delta_m2: int) -> int:
    return int(lib().kfac_next_interval(int(bool(similar_to_last)), int(bool(similar_to_before_last)), int(delta_m1),
                                        int(delta_m2)))


def kfac_refresh_init(n: int):
    """A ctypes array of n refresh states, initialised by the library."""
    arr = (kfac_refresh_state * n)()
    lib().kfac_refresh_init(ctypes.addressof(arr), n)
    return arr


def kfac_refresh_due(state: kfac_refresh_state, t: int) -> bool:
    return bool(lib().kfac_refresh_due(ctypes.addressof(state), int(t)))


def kfac_refresh_advance(state: kfac_refresh_state, ratio_m1: float, ratio_m2: float, alpha: float) -> None:
    lib().kfac_refresh_advance(ctypes.addressof(state), float(ratio_m1), float(ratio_m2), float(alpha))


def kfac_profile_enable(ctx: Context, on: bool) -> None:
    st = lib().kfac_profile_enable(ctx.handle, int(bool(on)))
    if st != KFAC_OK:
        raise KfacError(st, "kfac_profile_enable")


def kfac_profile_read(ctx: Context, max_entries: int = 4096) -> list:
    """Per-launch records since the last read: dicts with kernel, variant, workgroups, ms, flops, bytes,
    start_ms (from the start of the first recorded launch) and stream."""
    arr = (kfac_profile_entry * max_entries)()
    n = lib().kfac_profile_read(ctx.handle, ctypes.addressof(arr), max_entries)
    if n < 0:
        raise KfacError(KFAC_ERR_DEVICE, "kfac_profile_read")
    return [dict(kernel=KERNEL_NAMES[e.kernel], variant=e.variant, workgroups=e.workgroups, ms=e.ms,
                 flops=e.flops, bytes=e.bytes, start_ms=e.start_ms, stream=e.stream)
            for e in arr[:min(n, max_entries)]]
