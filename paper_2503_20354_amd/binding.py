"""ctypes binding of libsurgeon.so: the same names as the C ABI, argument marshalling only.

The ``surgeon_*`` functions mirror ``include/surgeon.h`` one to one (torch tensors stand in for device
pointers, the current torch stream for ``stream``).  ``prune_pack`` / ``dw_from_packed`` / ``grad_importance``
are conveniences that also allocate the outputs and workspaces with torch.  There is no fallback: if the
library is missing or a call fails, an exception is raised.
"""
import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

F32, BF16 = 0, 1
_STATUS = {0: "SURGEON_OK", 1: "SURGEON_EINVAL", 2: "SURGEON_ESIZE", 3: "SURGEON_EUNSUPPORTED", 4: "SURGEON_EHIP"}
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("SURGEON_LIBRARY", os.path.join(_HERE, "libsurgeon.so"))  # override: another build of the same ABI
_lib = None


class SurgeonError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("%s: %s" % (_STATUS.get(status, status), message))
        self.status = status


class LayerDesc(ctypes.Structure):
    """surgeon_layer_desc"""
    _fields_ = [("kind", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("M", ctypes.c_int64), ("K", ctypes.c_int64), ("N", ctypes.c_int64),
                ("Nb", ctypes.c_int64), ("Ci", ctypes.c_int64), ("H", ctypes.c_int64), ("W", ctypes.c_int64),
                ("Co", ctypes.c_int64), ("kh", ctypes.c_int64), ("kw", ctypes.c_int64),
                ("stride", ctypes.c_int64), ("pad", ctypes.c_int64), ("k_total", ctypes.c_int64),
                ("group_len", ctypes.c_int64), ("r", ctypes.c_float), ("groups", ctypes.c_int64)]


def library_path():
    return _LIB_PATH


def load_library():
    """Loads libsurgeon.so (built in-tree by ``__graft_entry__.build()``); fails loudly if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise SurgeonError(4, "libsurgeon.so is not built: run `python __graft_entry__.py` (hipcc, gfx950) first")
    L = ctypes.CDLL(_LIB_PATH)
    i64, f32, vp, ci, sz = ctypes.c_int64, ctypes.c_float, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    L.surgeon_keep_count.restype = i64
    L.surgeon_keep_count.argtypes = [i64, f32]
    L.surgeon_packed_sizes.restype = ci
    L.surgeon_packed_sizes.argtypes = [i64, i64, f32, ci, ctypes.POINTER(i64), ctypes.POINTER(sz), ctypes.POINTER(sz),
                                       ctypes.POINTER(sz)]
    L.surgeon_layer_ratios.restype = ci
    L.surgeon_layer_ratios.argtypes = [vp, vp, ci, f32, f32, vp]
    L.surgeon_prune_pack.restype = ci
    L.surgeon_prune_pack.argtypes = [vp, i64, i64, f32, ci, vp, vp, vp, vp, sz, vp]
    L.surgeon_set_select_margin.restype = ci
    L.surgeon_set_select_margin.argtypes = [f32]
    L.surgeon_select_pack_pattern_probe.restype = ci
    L.surgeon_select_pack_pattern_probe.argtypes = [vp, i64, ci, ctypes.c_uint32, i64, vp, vp, vp]
    L.surgeon_prune_pack_batched.restype = ci
    L.surgeon_prune_pack_batched.argtypes = [ci, vp, vp, vp, vp, ci, vp, vp, vp]
    L.surgeon_dw_ws_bytes.restype = ci
    L.surgeon_dw_ws_bytes.argtypes = [ctypes.POINTER(LayerDesc), ctypes.POINTER(sz)]
    L.surgeon_dw_kernel_class.restype = ci
    L.surgeon_dw_kernel_class.argtypes = [ctypes.POINTER(LayerDesc), ctypes.POINTER(ci)]
    L.surgeon_dw_from_packed.restype = ci
    L.surgeon_dw_from_packed.argtypes = [ctypes.POINTER(LayerDesc), vp, vp, vp, vp, vp, sz, vp]
    L.surgeon_dw_gi_ws_bytes.restype = ci
    L.surgeon_dw_gi_ws_bytes.argtypes = [ctypes.POINTER(LayerDesc), ctypes.POINTER(sz)]
    L.surgeon_dw_from_packed_gi.restype = ci
    L.surgeon_dw_from_packed_gi.argtypes = [ctypes.POINTER(LayerDesc), vp, vp, vp, vp, vp, vp, sz, vp]
    L.surgeon_da.restype = ci
    L.surgeon_da.argtypes = [ctypes.POINTER(LayerDesc), vp, vp, vp, vp]
    L.surgeon_da_ws_bytes.restype = ci
    L.surgeon_da_ws_bytes.argtypes = [ctypes.POINTER(LayerDesc), ctypes.POINTER(sz)]
    L.surgeon_da_ws.restype = ci
    L.surgeon_da_ws.argtypes = [ctypes.POINTER(LayerDesc), vp, vp, vp, vp, sz, vp]
    L.surgeon_weight_update.restype = ci
    L.surgeon_weight_update.argtypes = [vp, vp, i64, f32, ci, vp]
    L.surgeon_weight_update_batched.restype = ci
    L.surgeon_weight_update_batched.argtypes = [ci, vp, vp, vp, f32, ci, vp]
    L.surgeon_affine_grad_ws_bytes.restype = ci
    L.surgeon_affine_grad_ws_bytes.argtypes = [i64, i64, i64, ctypes.POINTER(sz)]
    L.surgeon_affine_grad.restype = ci
    L.surgeon_affine_grad.argtypes = [vp, vp, vp, i64, i64, i64, ci, i64, vp, vp, vp, sz, vp]
    L.surgeon_grad_importance_ws_bytes.restype = sz
    L.surgeon_grad_importance_ws_bytes.argtypes = [i64]
    L.surgeon_grad_importance.restype = ci
    L.surgeon_grad_importance.argtypes = [vp, i64, vp, vp, sz, vp]
    L.surgeon_grad_importance_static.restype = ci
    L.surgeon_grad_importance_static.argtypes = [vp, i64, vp, vp]
    L.surgeon_grad_importance_batched_ws_bytes.restype = sz
    L.surgeon_grad_importance_batched_ws_bytes.argtypes = [vp, ci]
    L.surgeon_grad_importance_batched.restype = ci
    L.surgeon_grad_importance_batched.argtypes = [vp, vp, ci, vp, vp, sz, vp]
    L.surgeon_profile_begin.restype = ci
    L.surgeon_profile_begin.argtypes = []
    L.surgeon_profile_end.restype = ci
    L.surgeon_profile_end.argtypes = [ci, vp, vp]
    L.surgeon_last_error.restype = ctypes.c_char_p
    L.surgeon_version.restype = ctypes.c_char_p
    _lib = L
    return L


def _check(status):
    if status != 0:
        raise SurgeonError(status, load_library().surgeon_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(device):
    return ctypes.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def _dt(t: torch.Tensor):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("activations are float32 or bfloat16, got %s" % t.dtype)


def _dev(t: torch.Tensor, name):
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)


# ----------------------------------------------------------------------------------------------------
# one-to-one mirrors of the C ABI
# ----------------------------------------------------------------------------------------------------
def surgeon_version():
    return load_library().surgeon_version().decode()


def surgeon_last_error():
    return load_library().surgeon_last_error().decode()


def surgeon_keep_count(length: int, r: float) -> int:
    return int(load_library().surgeon_keep_count(int(length), float(r)))


def surgeon_packed_sizes(n: int, group_len: int, r: float, dt: int):
    """Returns (k_total, vals_bytes, mask_bytes, ws_bytes)."""
    k = ctypes.c_int64()
    vb, mb, wb = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(load_library().surgeon_packed_sizes(int(n), int(group_len), float(r), int(dt), ctypes.byref(k),
                                               ctypes.byref(vb), ctypes.byref(mb), ctypes.byref(wb)))
    return k.value, vb.value, mb.value, wb.value


def surgeon_layer_ratios(G, m, r_lo: float = 0.0, r_hi: float = 1.0):
    """Eq. 5-7 on the host.  G: float32 sequence/tensor (host), m: sizes.  Returns a float32 CPU tensor."""
    G = torch.as_tensor(G, dtype=torch.float32, device="cpu").contiguous()
    m64 = torch.as_tensor([int(x) for x in m], dtype=torch.int64)  # uint64 values passed through int64 storage
    out = torch.empty(G.numel(), dtype=torch.float32)
    _check(load_library().surgeon_layer_ratios(_ptr(G), _ptr(m64), int(G.numel()), float(r_lo), float(r_hi), _ptr(out)))
    return out


def surgeon_prune_pack(A, group_len, r, vals, mask, idx=None, ws=None):
    _dev(A, "A")
    _dev(mask, "mask")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(load_library().surgeon_prune_pack(_ptr(A), A.numel(), int(group_len), float(r), _dt(A), _ptr(vals),
                                             _ptr(mask), _ptr(idx), _ptr(ws), ws_bytes, _stream(A.device)))


def surgeon_set_select_margin(deviations: float):
    """Bracket width (standard deviations of the sample rank) of the two-read selection of long groups."""
    _check(load_library().surgeon_set_select_margin(float(deviations)))


def surgeon_select_pack_pattern_probe(A, threshold_bits: int, k_cap: int, vals, mask):
    """Benchmark aid: the memory pattern of the fused select+pack kernel with a fixed threshold instead of a search."""
    _dev(A, "A")
    _dev(vals, "vals")
    _dev(mask, "mask")
    _check(load_library().surgeon_select_pack_pattern_probe(_ptr(A), A.numel(), _dt(A), int(threshold_bits), int(k_cap),
                                                            _ptr(vals), _ptr(mask), _stream(A.device)))


def surgeon_prune_pack_batched(As, group_lens, ratios, vals, masks):
    """Alg. 1 lines 6-7 for a list of tensors (one dtype) in one call; vals / masks: pre-sized tensors per layer."""
    l = len(As)
    for t in list(As) + list(masks):
        _dev(t, "tensor")
    dt = _dt(As[0])
    a_p = (ctypes.c_void_p * l)(*[t.data_ptr() for t in As])
    v_p = (ctypes.c_void_p * l)(*[t.data_ptr() for t in vals])
    m_p = (ctypes.c_void_p * l)(*[t.data_ptr() for t in masks])
    n_a = (ctypes.c_int64 * l)(*[t.numel() for t in As])
    g_a = (ctypes.c_int64 * l)(*[int(g) for g in group_lens])
    r_a = (ctypes.c_float * l)(*[float(r) for r in ratios])
    _check(load_library().surgeon_prune_pack_batched(l, a_p, n_a, g_a, r_a, dt, v_p, m_p, _stream(As[0].device)))


def surgeon_dw_ws_bytes(desc: LayerDesc) -> int:
    wb = ctypes.c_size_t()
    _check(load_library().surgeon_dw_ws_bytes(ctypes.byref(desc), ctypes.byref(wb)))
    return wb.value


def surgeon_dw_kernel_class(desc: LayerDesc) -> str:
    """Name of the kernel class ("dw" or "dw_sparse") surgeon_dw_from_packed will use for this descriptor."""
    c = ctypes.c_int()
    _check(load_library().surgeon_dw_kernel_class(ctypes.byref(desc), ctypes.byref(c)))
    return PROF_CLASSES[c.value]


def surgeon_dw_from_packed(desc: LayerDesc, vals, mask, dY, dW, ws):
    _dev(dY, "dY")
    _dev(dW, "dW")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(load_library().surgeon_dw_from_packed(ctypes.byref(desc), _ptr(vals), _ptr(mask), _ptr(dY), _ptr(dW),
                                                 _ptr(ws), ws_bytes, _stream(dY.device)))


def surgeon_dw_gi_ws_bytes(desc: LayerDesc) -> int:
    wb = ctypes.c_size_t()
    _check(load_library().surgeon_dw_gi_ws_bytes(ctypes.byref(desc), ctypes.byref(wb)))
    return wb.value


def surgeon_dw_from_packed_gi(desc: LayerDesc, vals, mask, dY, dW, G_out, ws):
    """dW from the packed activation plus Eq. 4 of that gradient into G_out[0], in one call."""
    _dev(dY, "dY")
    _dev(dW, "dW")
    _dev(G_out, "G_out")
    if G_out.dtype != torch.float32:
        raise TypeError("G_out is float32")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(load_library().surgeon_dw_from_packed_gi(ctypes.byref(desc), _ptr(vals), _ptr(mask), _ptr(dY), _ptr(dW),
                                                    _ptr(G_out), _ptr(ws), ws_bytes, _stream(dY.device)))


def surgeon_da(desc: LayerDesc, dY, W, dA):
    """Eq. 2, first line: dA = dY . W (all three tensors of the layer's dtype, on the device)."""
    for t, name in ((dY, "dY"), (W, "W"), (dA, "dA")):
        _dev(t, name)
        if _dt(t) != desc.dtype:
            raise TypeError("%s does not have the layer's dtype" % name)
    _check(load_library().surgeon_da(ctypes.byref(desc), _ptr(dY), _ptr(W), _ptr(dA), _stream(dY.device)))


def surgeon_da_ws_bytes(desc: LayerDesc) -> int:
    wb = ctypes.c_size_t()
    _check(load_library().surgeon_da_ws_bytes(ctypes.byref(desc), ctypes.byref(wb)))
    return wb.value


def surgeon_da_ws(desc: LayerDesc, dY, W, dA, ws):
    """Eq. 2, first line, with a workspace: bf16 linear layers run on the bf16 matrix cores."""
    for t, name in ((dY, "dY"), (W, "W"), (dA, "dA")):
        _dev(t, name)
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(load_library().surgeon_da_ws(ctypes.byref(desc), _ptr(dY), _ptr(W), _ptr(dA), _ptr(ws), ws_bytes,
                                        _stream(dY.device)))


def surgeon_weight_update(W, dW, lr: float):
    """Alg. 1 line 14 as one plain gradient step, in place: W <- W - lr * dW."""
    _dev(W, "W")
    _dev(dW, "dW")
    if dW.dtype != torch.float32 or dW.numel() != W.numel():
        raise TypeError("dW is float32 with as many elements as W")
    _check(load_library().surgeon_weight_update(_ptr(W), _ptr(dW), W.numel(), float(lr), _dt(W), _stream(W.device)))


def surgeon_weight_update_batched(Ws, dWs, lr: float):
    """Alg. 1 line 14 for a list of weight tensors (one dtype) in one call."""
    l = len(Ws)
    for t in list(Ws) + list(dWs):
        _dev(t, "tensor")
    w_p = (ctypes.c_void_p * l)(*[t.data_ptr() for t in Ws])
    g_p = (ctypes.c_void_p * l)(*[t.data_ptr() for t in dWs])
    n_a = (ctypes.c_int64 * l)(*[t.numel() for t in Ws])
    for w, g in zip(Ws, dWs):
        if g.numel() != w.numel() or g.dtype != torch.float32:
            raise SurgeonError(1, "weight_update_batched: dW must be fp32 with W's element count")
    _check(load_library().surgeon_weight_update_batched(l, w_p, g_p, n_a, float(lr), _dt(Ws[0]), _stream(Ws[0].device)))


def surgeon_affine_grad_ws_bytes(outer: int, C: int, inner: int) -> int:
    wb = ctypes.c_size_t()
    _check(load_library().surgeon_affine_grad_ws_bytes(int(outer), int(C), int(inner), ctypes.byref(wb)))
    return wb.value


def surgeon_affine_grad(vals, mask, dY, outer, C, inner, k_total, dgamma, dbeta, ws):
    """Scale / shift gradients of a normalisation layer from the packed normalised activation."""
    _dev(dY, "dY")
    _dev(dgamma, "dgamma")
    _dev(dbeta, "dbeta")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(load_library().surgeon_affine_grad(_ptr(vals), _ptr(mask), _ptr(dY), int(outer), int(C), int(inner), _dt(dY),
                                              int(k_total), _ptr(dgamma), _ptr(dbeta), _ptr(ws), ws_bytes,
                                              _stream(dY.device)))


def surgeon_grad_importance_ws_bytes(n_w: int) -> int:
    return int(load_library().surgeon_grad_importance_ws_bytes(int(n_w)))


def surgeon_grad_importance(dW, G_out, ws=None):
    _dev(dW, "dW")
    _dev(G_out, "G_out")
    if dW.dtype != torch.float32 or G_out.dtype != torch.float32:
        raise TypeError("dW and G_out are float32")
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(load_library().surgeon_grad_importance(_ptr(dW), dW.numel(), _ptr(G_out), _ptr(ws), ws_bytes,
                                                  _stream(dW.device)))


def surgeon_grad_importance_static(dW, G_out):
    """Eq. 4 with the partial sums in the library's own device array: no workspace, nothing allocated."""
    _dev(dW, "dW")
    _dev(G_out, "G_out")
    if dW.dtype != torch.float32 or G_out.dtype != torch.float32:
        raise TypeError("dW and G_out are float32")
    _check(load_library().surgeon_grad_importance_static(_ptr(dW), dW.numel(), _ptr(G_out), _stream(dW.device)))


def _batched_args(dWs):
    l = len(dWs)
    ptrs = (ctypes.c_void_p * l)(*[t.data_ptr() for t in dWs])
    sizes = (ctypes.c_int64 * l)(*[t.numel() for t in dWs])
    return l, ptrs, sizes


def surgeon_grad_importance_batched_ws_bytes(dWs) -> int:
    l, _, sizes = _batched_args(dWs)
    return int(load_library().surgeon_grad_importance_batched_ws_bytes(sizes, l))


def surgeon_grad_importance_batched(dWs, G_out, ws):
    """Eq. 4 for a list of per-layer dW tensors in one call; G_out: float32 device tensor of len(dWs)."""
    for t in dWs:
        _dev(t, "dW")
        if t.dtype != torch.float32:
            raise TypeError("dW is float32")
    _dev(G_out, "G_out")
    if G_out.numel() < len(dWs):
        raise ValueError("G_out is too short")
    l, ptrs, sizes = _batched_args(dWs)
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(load_library().surgeon_grad_importance_batched(ptrs, sizes, l, _ptr(G_out), _ptr(ws), ws_bytes,
                                                          _stream(G_out.device)))


PROF_CLASSES = ("select_pack", "dw", "importance", "dw_aux", "select_other", "dw_sparse", "da", "update", "affine",
                "dw_grouped", "dw_sparse_aux")


def surgeon_profile_begin():
    _check(load_library().surgeon_profile_begin())


def surgeon_profile_end():
    """Returns {class name: (milliseconds, launches)} for the kernels launched since surgeon_profile_begin()."""
    n = len(PROF_CLASSES)
    ms = (ctypes.c_double * n)()
    launches = (ctypes.c_int64 * n)()
    _check(load_library().surgeon_profile_end(n, ms, launches))
    return {name: (ms[i], launches[i]) for i, name in enumerate(PROF_CLASSES)}


# ----------------------------------------------------------------------------------------------------
# conveniences: the same calls with torch doing the allocation
# ----------------------------------------------------------------------------------------------------
@dataclass
class PackedActivation:
    """Cached form of one pruned activation (Alg. 1 line 7): kept values + one bit per element."""
    vals: torch.Tensor   # [k_total], dtype of A
    mask: torch.Tensor   # [ceil(n/64)] int64 holding the uint64 words
    idx: Optional[torch.Tensor]
    k_total: int
    n: int
    group_len: int
    r: float


def _workspace(nbytes, device):
    return torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device) if nbytes > 0 else None


def prune_pack(A: torch.Tensor, group_len: int, r: float, want_idx: bool = False) -> PackedActivation:
    n = A.numel()
    k, _, mask_bytes, ws_bytes = surgeon_packed_sizes(n, group_len, r, _dt(A))
    vals = torch.empty(k, dtype=A.dtype, device=A.device)
    mask = torch.empty(mask_bytes // 8, dtype=torch.int64, device=A.device)
    idx = torch.empty(k, dtype=torch.int32, device=A.device) if want_idx else None
    surgeon_prune_pack(A, group_len, r, vals, mask, idx, _workspace(ws_bytes, A.device))
    return PackedActivation(vals, mask, idx, k, n, group_len, r)


def linear_desc(M, K, N, dtype, k_total, group_len=0, r=0.0) -> LayerDesc:
    d = LayerDesc()
    d.kind, d.dtype, d.M, d.K, d.N, d.k_total = 0, dtype, M, K, N, k_total
    d.group_len, d.r = group_len, r  # optional hint: the arguments the packing used
    return d


def conv2d_desc(Nb, Ci, H, W, Co, kh, kw, stride, pad, dtype, k_total, group_len=0, r=0.0, groups=1) -> LayerDesc:
    d = LayerDesc()
    d.kind, d.dtype, d.k_total, d.groups = 1, dtype, k_total, groups
    d.group_len, d.r = group_len, r
    d.Nb, d.Ci, d.H, d.W, d.Co, d.kh, d.kw, d.stride, d.pad = Nb, Ci, H, W, Co, kh, kw, stride, pad
    return d


def dw_from_packed(desc: LayerDesc, packed: PackedActivation, dY: torch.Tensor, dW: Optional[torch.Tensor] = None,
                   ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    if desc.kind == 0:
        shape = (desc.N, desc.K)
    else:
        shape = (desc.Co, desc.Ci // max(desc.groups, 1), desc.kh, desc.kw)
    if dW is None:
        dW = torch.empty(shape, dtype=torch.float32, device=dY.device)
    if ws is None:
        ws = _workspace(surgeon_dw_ws_bytes(desc), dY.device)
    if desc.group_len == 0:  # pass the packing's arguments along as the hint
        desc.group_len, desc.r = packed.group_len, packed.r
    surgeon_dw_from_packed(desc, packed.vals, packed.mask, dY, dW, ws)
    return dW


def affine_grad(packed: PackedActivation, dY: torch.Tensor, outer: int, C: int, inner: int):
    """(dgamma, dbeta) of a normalisation layer from its packed normalised activation."""
    dgamma = torch.empty(C, dtype=torch.float32, device=dY.device)
    dbeta = torch.empty(C, dtype=torch.float32, device=dY.device)
    ws = _workspace(surgeon_affine_grad_ws_bytes(outer, C, inner), dY.device)
    surgeon_affine_grad(packed.vals, packed.mask, dY, outer, C, inner, packed.k_total, dgamma, dbeta, ws)
    return dgamma, dbeta


def grad_importance(dW: torch.Tensor, G_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    if G_out is None:
        G_out = torch.empty(1, dtype=torch.float32, device=dW.device)
    ws = _workspace(surgeon_grad_importance_ws_bytes(dW.numel()), dW.device)
    surgeon_grad_importance(dW, G_out, ws)
    return G_out
