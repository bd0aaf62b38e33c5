"""CPU oracle for SURGEON's activation-pruning hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes marshalling around ``surgeon_oracle.c`` (the plain definition of Alg. 1 lines 6-7 and 11-12,
Eq. 2 and Eq. 4-7).  Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import this
package; the product package never does.  Arrays are numpy: float32 for fp32 tensors, uint16 holding the
raw bit patterns for bfloat16 tensors.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "surgeon_oracle.c")
_SO = os.path.join(_HERE, "libsurgeon_oracle.so")
_lib = None

F32, BF16 = 0, 1


def build(force=True):
    """Compile the oracle with gcc (-O2, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall",
               "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_SO)
        i64, f32, vp, ci = ctypes.c_int64, ctypes.c_float, ctypes.c_void_p, ctypes.c_int
        L.oracle_keep_count.restype = i64
        L.oracle_keep_count.argtypes = [i64, f32]
        L.oracle_prune_pack.restype = ci
        L.oracle_prune_pack.argtypes = [vp, i64, i64, f32, ci, vp, vp, vp, ctypes.POINTER(i64)]
        L.oracle_unpack.restype = None
        L.oracle_unpack.argtypes = [vp, vp, i64, ci, vp]
        L.oracle_dw_linear.restype = ci
        L.oracle_dw_linear.argtypes = [vp, vp, vp, i64, i64, i64, ci, vp]
        L.oracle_dw_linear_at.restype = ci
        L.oracle_dw_linear_at.argtypes = [vp, vp, vp, i64, i64, i64, ci, vp, i64, vp]
        L.oracle_dw_conv2d.restype = ci
        L.oracle_dw_conv2d.argtypes = [vp, vp, vp] + [i64] * 9 + [ci, vp]
        L.oracle_dw_conv2d_at.restype = ci
        L.oracle_dw_conv2d_at.argtypes = [vp, vp, vp] + [i64] * 9 + [ci, vp, i64, vp]
        L.oracle_grad_importance.restype = f32
        L.oracle_grad_importance.argtypes = [vp, i64]
        L.oracle_layer_scores.restype = ci
        L.oracle_layer_scores.argtypes = [vp, vp, ci, vp, vp, vp]
        L.oracle_layer_ratios.restype = ci
        L.oracle_layer_ratios.argtypes = [vp, vp, ci, f32, f32, vp]
        L.oracle_da_linear.restype = ci
        L.oracle_da_linear.argtypes = [vp, vp, i64, i64, i64, ci, vp]
        L.oracle_da_linear_at.restype = ci
        L.oracle_da_linear_at.argtypes = [vp, vp, i64, i64, i64, ci, vp, i64, vp]
        L.oracle_da_conv2d.restype = ci
        L.oracle_da_conv2d.argtypes = [vp, vp] + [i64] * 9 + [ci, vp]
        L.oracle_da_conv2d_grouped.restype = ci
        L.oracle_da_conv2d_grouped.argtypes = [vp, vp] + [i64] * 10 + [ci, vp]
        L.oracle_da_conv2d_at.restype = ci
        L.oracle_da_conv2d_at.argtypes = [vp, vp] + [i64] * 9 + [ci, vp, i64, vp]
        L.oracle_weight_update.restype = ci
        L.oracle_weight_update.argtypes = [vp, vp, i64, f32, ci, vp]
        L.oracle_affine_grad.restype = ci
        L.oracle_affine_grad.argtypes = [vp, vp, vp, i64, i64, i64, ci, vp, vp]
        L.oracle_dw_conv2d_grouped.restype = ci
        L.oracle_dw_conv2d_grouped.argtypes = [vp, vp, vp] + [i64] * 10 + [ci, vp]
        L.oracle_dw_conv2d_grouped_at.restype = ci
        L.oracle_dw_conv2d_grouped_at.argtypes = [vp, vp, vp] + [i64] * 10 + [ci, vp, i64, vp]
        _lib = L
    return _lib


def threads():
    """Number of host threads the OpenMP loops of the oracle will use."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    return len(os.sched_getaffinity(0))


def _dt(a):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError("oracle arrays are float32, or uint16 holding bfloat16 bits; got %s" % a.dtype)


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype=None):
    return np.ascontiguousarray(a, dtype=dtype)


def keep_count(length, r):
    return int(lib().oracle_keep_count(int(length), float(np.float32(r))))


def total_kept(n, group_len, r):
    """Sum over groups of keep_count(len_g, r)."""
    if n == 0:
        return 0
    group_len = min(group_len, n)
    full, rem = divmod(n, group_len)
    return full * keep_count(group_len, r) + (keep_count(rem, r) if rem else 0)


def prune_pack(A, group_len, r):
    """Alg. 1 lines 6-7.  Returns (vals, mask uint64[ceil(n/64)], idx uint32[k], k_total)."""
    A = _c(A).reshape(-1)
    n = A.size
    k = total_kept(n, group_len, r)
    vals = np.empty(k, dtype=A.dtype)
    mask = np.zeros((n + 63) // 64, dtype=np.uint64)
    idx = np.empty(k, dtype=np.uint32)
    k_out = ctypes.c_int64(-1)
    rc = lib().oracle_prune_pack(_p(A), n, int(group_len), float(np.float32(r)), _dt(A), _p(vals), _p(mask),
                                 _p(idx), ctypes.byref(k_out))
    if rc != 0:
        raise ValueError("oracle_prune_pack failed with %d" % rc)
    assert k_out.value == k
    return vals, mask, idx, k


def unpack(vals, mask, n):
    """Alg. 1 line 11: dense pruned activation in the storage dtype."""
    vals, mask = _c(vals), _c(mask, np.uint64)
    dense = np.empty(n, dtype=vals.dtype)
    lib().oracle_unpack(_p(vals), _p(mask), n, _dt(vals), _p(dense))
    return dense


def dw_linear(vals, mask, dY, M, K, N):
    """Eq. 2 weight gradient of a linear layer as [N, K] float32."""
    vals, mask, dY = _c(vals), _c(mask, np.uint64), _c(dY)
    assert _dt(vals) == _dt(dY) and dY.size == M * N
    dW = np.empty((N, K), dtype=np.float32)
    rc = lib().oracle_dw_linear(_p(vals), _p(mask), _p(dY), M, K, N, _dt(vals), _p(dW))
    assert rc == 0
    return dW


def dw_linear_at(vals, mask, dY, M, K, N, where):
    vals, mask, dY = _c(vals), _c(mask, np.uint64), _c(dY)
    where = _c(where, np.int64)
    out = np.empty(where.size, dtype=np.float32)
    rc = lib().oracle_dw_linear_at(_p(vals), _p(mask), _p(dY), M, K, N, _dt(vals), _p(where), where.size, _p(out))
    assert rc == 0
    return out


def dw_conv2d(vals, mask, dY, Nb, Ci, H, W, Co, kh, kw, stride, pad):
    """Weight gradient of a 2-D convolution as [Co, Ci, kh, kw] float32."""
    vals, mask, dY = _c(vals), _c(mask, np.uint64), _c(dY)
    OH, OW = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    assert _dt(vals) == _dt(dY) and dY.size == Nb * Co * OH * OW
    dW = np.empty((Co, Ci, kh, kw), dtype=np.float32)
    rc = lib().oracle_dw_conv2d(_p(vals), _p(mask), _p(dY), Nb, Ci, H, W, Co, kh, kw, stride, pad, _dt(vals), _p(dW))
    assert rc == 0
    return dW


def dw_conv2d_at(vals, mask, dY, Nb, Ci, H, W, Co, kh, kw, stride, pad, where):
    vals, mask, dY = _c(vals), _c(mask, np.uint64), _c(dY)
    where = _c(where, np.int64)
    out = np.empty(where.size, dtype=np.float32)
    rc = lib().oracle_dw_conv2d_at(_p(vals), _p(mask), _p(dY), Nb, Ci, H, W, Co, kh, kw, stride, pad, _dt(vals),
                                   _p(where), where.size, _p(out))
    assert rc == 0
    return out


def grad_importance(dW):
    dW = _c(dW, np.float32).reshape(-1)
    return float(lib().oracle_grad_importance(_p(dW), dW.size))


def layer_scores(G, m):
    """Eq. 5-7 in double: returns (M, I, p)."""
    G, m = _c(G, np.float32), _c(m, np.uint64)
    l = G.size
    M, I, p = (np.empty(l, dtype=np.float64) for _ in range(3))
    rc = lib().oracle_layer_scores(_p(G), _p(m), l, _p(M), _p(I), _p(p))
    if rc != 0:
        raise ValueError("oracle_layer_scores: bad input")
    return M, I, p


def layer_ratios(G, m, r_lo=0.0, r_hi=1.0):
    G, m = _c(G, np.float32), _c(m, np.uint64)
    out = np.empty(G.size, dtype=np.float32)
    rc = lib().oracle_layer_ratios(_p(G), _p(m), G.size, float(r_lo), float(r_hi), _p(out))
    if rc != 0:
        raise ValueError("oracle_layer_ratios: bad input")
    return out


def da_linear(dY, W, M, K, N):
    """Eq. 2, first line: dA [M, K] = dY [M, N] . W [N, K], in the dtype of the inputs."""
    dY, W = _c(dY), _c(W)
    assert _dt(dY) == _dt(W) and dY.size == M * N and W.size == N * K
    dA = np.empty((M, K), dtype=dY.dtype)
    assert lib().oracle_da_linear(_p(dY), _p(W), M, K, N, _dt(dY), _p(dA)) == 0
    return dA


def da_linear_at(dY, W, M, K, N, where):
    dY, W, where = _c(dY), _c(W), _c(where, np.int64)
    out = np.empty(where.size, dtype=dY.dtype)
    assert lib().oracle_da_linear_at(_p(dY), _p(W), M, K, N, _dt(dY), _p(where), where.size, _p(out)) == 0
    return out


def da_conv2d(dY, W, Nb, Ci, H, Wd, Co, kh, kw, stride, pad):
    """Activation gradient of a 2-D convolution: dA [Nb, Ci, H, Wd] in the dtype of the inputs."""
    dY, W = _c(dY), _c(W)
    OH, OW = (H + 2 * pad - kh) // stride + 1, (Wd + 2 * pad - kw) // stride + 1
    assert _dt(dY) == _dt(W) and dY.size == Nb * Co * OH * OW and W.size == Co * Ci * kh * kw
    dA = np.empty((Nb, Ci, H, Wd), dtype=dY.dtype)
    assert lib().oracle_da_conv2d(_p(dY), _p(W), Nb, Ci, H, Wd, Co, kh, kw, stride, pad, _dt(dY), _p(dA)) == 0
    return dA


def da_conv2d_grouped(dY, W, Nb, Ci, H, Wd, Co, kh, kw, stride, pad, groups):
    """Activation gradient of a convolution with channel groups (W is [Co, Ci/groups, kh, kw])."""
    dY, W = _c(dY), _c(W)
    OH, OW = (H + 2 * pad - kh) // stride + 1, (Wd + 2 * pad - kw) // stride + 1
    assert Ci % groups == 0 and Co % groups == 0
    assert _dt(dY) == _dt(W) and dY.size == Nb * Co * OH * OW and W.size == Co * (Ci // groups) * kh * kw
    dA = np.empty((Nb, Ci, H, Wd), dtype=dY.dtype)
    assert lib().oracle_da_conv2d_grouped(_p(dY), _p(W), Nb, Ci, H, Wd, Co, kh, kw, stride, pad, groups, _dt(dY),
                                          _p(dA)) == 0
    return dA


def da_conv2d_at(dY, W, Nb, Ci, H, Wd, Co, kh, kw, stride, pad, where):
    dY, W, where = _c(dY), _c(W), _c(where, np.int64)
    out = np.empty(where.size, dtype=dY.dtype)
    assert lib().oracle_da_conv2d_at(_p(dY), _p(W), Nb, Ci, H, Wd, Co, kh, kw, stride, pad, _dt(dY), _p(where),
                                     where.size, _p(out)) == 0
    return out


def weight_update(W, dW, lr):
    """Alg. 1 line 14 as one plain gradient step: W - lr * dW in the dtype of W."""
    W, dW = _c(W), _c(dW, np.float32)
    assert W.size == dW.size
    out = np.empty(W.shape, dtype=W.dtype)
    assert lib().oracle_weight_update(_p(W), _p(dW), W.size, float(np.float32(lr)), _dt(W), _p(out)) == 0
    return out


def affine_grad(vals, mask, dY, outer, C, inner):
    """Scale / shift gradients of a normalisation layer from the pruned normalised activation: (dgamma, dbeta)."""
    vals, mask, dY = _c(vals), _c(mask, np.uint64), _c(dY)
    assert _dt(vals) == _dt(dY) and dY.size == outer * C * inner
    dgamma, dbeta = np.empty(C, dtype=np.float32), np.empty(C, dtype=np.float32)
    assert lib().oracle_affine_grad(_p(vals), _p(mask), _p(dY), outer, C, inner, _dt(vals), _p(dgamma), _p(dbeta)) == 0
    return dgamma, dbeta


def dw_conv2d_grouped(vals, mask, dY, Nb, Ci, H, W, Co, kh, kw, stride, pad, groups):
    """Weight gradient of a convolution with channel groups as [Co, Ci/groups, kh, kw] float32."""
    vals, mask, dY = _c(vals), _c(mask, np.uint64), _c(dY)
    dW = np.empty((Co, Ci // groups, kh, kw), dtype=np.float32)
    rc = lib().oracle_dw_conv2d_grouped(_p(vals), _p(mask), _p(dY), Nb, Ci, H, W, Co, kh, kw, stride, pad, groups,
                                        _dt(vals), _p(dW))
    assert rc == 0
    return dW


def dw_conv2d_grouped_at(vals, mask, dY, Nb, Ci, H, W, Co, kh, kw, stride, pad, groups, where):
    vals, mask, dY, where = _c(vals), _c(mask, np.uint64), _c(dY), _c(where, np.int64)
    out = np.empty(where.size, dtype=np.float32)
    rc = lib().oracle_dw_conv2d_grouped_at(_p(vals), _p(mask), _p(dY), Nb, Ci, H, W, Co, kh, kw, stride, pad, groups,
                                           _dt(vals), _p(where), where.size, _p(out))
    assert rc == 0
    return out
