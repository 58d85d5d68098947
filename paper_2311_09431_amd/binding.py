"""ctypes binding of libstriped_attn.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/striped_attn.h)
and takes torch tensors living on the GPU; torch supplies device memory and the
current stream, nothing else.  There is no CPU fallback: if the library is not
built, or a tensor is not on the GPU, the call raises.
"""
import ctypes
import math
import os

import torch

CONTIGUOUS, STRIPED = 0, 1
F32, BF16 = 0, 1
MASK_EMPTY, MASK_TRI, MASK_FULL = 0, 1, 2

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libstriped_attn.so")
_lib = None


class SaShape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("c", ctypes.c_int32),
                ("d", ctypes.c_int32), ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64),
                ("stride_s", ctypes.c_int64), ("stat_stride_b", ctypes.c_int64), ("stat_stride_h", ctypes.c_int64),
                ("dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("H_kv", ctypes.c_int32), ("kv_stride_b", ctypes.c_int64), ("kv_stride_h", ctypes.c_int64),
                ("kv_stride_s", ctypes.c_int64)]


class StripedAttnError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, lib().sa_status_str(status).decode(), status))


def lib():
    """The loaded shared library (loads on first use; raises if it is not built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("libstriped_attn.so is not built: run "
                               "`python -m paper_2311_09431_amd.build` (needs hipcc)")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        shp = ctypes.POINTER(SaShape)
        sig = {
            "sa_stripe_permute": (i32, [vp, vp, i64, i64, i64, i32, vp]),
            "sa_unstripe_permute": (i32, [vp, vp, i64, i64, i64, i32, vp]),
            "sa_state_init": (i32, [vp, vp, shp, vp]),
            "sa_rope": (i32, [vp, vp, vp, i64, shp, ctypes.c_float, i32, vp]),
            "sa_attn_step_fwd": (i32, [vp, vp, vp, vp, vp, i32, i32, i32, i32, shp, vp]),
            "sa_attn_step_fwd_rope": (i32, [vp, vp, vp, vp, vp, vp, i64, ctypes.c_float, i32, i32, i32, i32, shp, vp]),
            "sa_finalize": (i32, [vp, vp, shp, vp]),
            "sa_bwd_preprocess": (i32, [vp, vp, vp, shp, vp]),
            "sa_attn_step_bwd": (i32, [vp] * 9 + [i32, i32, i32, i32, shp, vp]),
            "sa_ring_fwd": (i32, [vp] * 5 + [i32, i32, shp, i32, vp, vp]),
            "sa_ring_bwd": (i32, [vp] * 10 + [i32, i32, shp, i32, vp, vp]),
            "sa_attn_step_fwd_tiled": (i32, [vp, vp, vp, vp, vp, i32, i32, i32, i32, shp, i32, i32, vp]),
            "sa_attn_step_bwd_tiled": (i32, [vp] * 9 + [i32, i32, i32, i32, shp, i32, i32, vp]),
            "sa_ring_fwd_tiled": (i32, [vp] * 5 + [i32, i32, shp, i32, i32, i32, vp, vp]),
            "sa_ring_bwd_tiled": (i32, [vp] * 10 + [i32, i32, shp, i32, i32, i32, vp, vp]),
            "sa_step_tiles": (i32, [i32, i32, i32, i32, i64, i64, i64, ctypes.POINTER(i64),
                                    ctypes.POINTER(i64)]),
            "sa_step_mask": (i32, [i32, i32, i32, i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]),
            "sa_step_pairs": (i64, [i32, i32, i32, i32, i64]),
            "sa_device_props": (i32, [ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i64)]),
            "sa_status_str": (ctypes.c_char_p, [i32]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


EXPORTS = ("sa_stripe_permute", "sa_unstripe_permute", "sa_rope", "sa_state_init", "sa_attn_step_fwd",
           "sa_attn_step_fwd_rope",
           "sa_finalize", "sa_bwd_preprocess", "sa_attn_step_bwd", "sa_ring_fwd", "sa_ring_bwd",
           "sa_attn_step_fwd_tiled", "sa_attn_step_bwd_tiled", "sa_ring_fwd_tiled", "sa_ring_bwd_tiled",
           "sa_step_tiles", "sa_step_mask", "sa_step_pairs", "sa_device_props", "sa_status_str")


def _ptr(t):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("expected a GPU tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status, where):
    if status != 0:
        raise StripedAttnError(status, where)


def _dtype_code(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("Q/K/V must be float32 or bfloat16")


def shard_shape(x, c, lse=None, scale=None, kv=None):
    """sa_shape of a c-row shard of x indexed [B, H, rows, d] (d contiguous; any batch, head
    and row strides, e.g. a [B, rows, H, d] tensor viewed through permute(0, 2, 1, 3)).
    kv: a key/value tensor [B, H_kv, rows, d] when K, V, dK, dV have fewer heads than x or
    strides of their own (all four must share them)."""
    B, H, rows, d = x.shape
    if x.stride(3) != 1:
        raise ValueError("the head dimension must be contiguous")
    ssb, ssh = (lse.stride(0), lse.stride(1)) if lse is not None else (H * rows, rows)
    shape = SaShape(B, H, c, d, x.stride(0), x.stride(1), x.stride(2), ssb, ssh, _dtype_code(x),
                    float(scale) if scale else 0.0)
    if kv is not None:
        if kv.shape[0] != B or kv.shape[3] != d or kv.stride(3) != 1:
            raise ValueError("K/V must be [B, H_kv, rows, d] with the head dimension contiguous")
        shape.H_kv, shape.kv_stride_b, shape.kv_stride_h, shape.kv_stride_s = (
            kv.shape[1], kv.stride(0), kv.stride(1), kv.stride(2))
    return shape


def _rows(t, dev, c):
    """View of rows [dev*c, (dev+1)*c) along the sequence axis (axis 2)."""
    return t[:, :, dev * c:(dev + 1) * c]


def sa_stripe_permute(src, dst, N, seq_axis=2):
    """dst <- stripe permutation of src along seq_axis (both contiguous, same shape)."""
    _permute("sa_stripe_permute", src, dst, N, seq_axis)


def sa_unstripe_permute(src, dst, N, seq_axis=2):
    _permute("sa_unstripe_permute", src, dst, N, seq_axis)


def _permute(name, src, dst, N, seq_axis):
    if not (src.is_contiguous() and dst.is_contiguous()) or src.shape != dst.shape \
            or src.dtype != dst.dtype:
        raise ValueError("src and dst must be contiguous with equal shape and dtype")
    outer = math.prod(src.shape[:seq_axis])
    inner = math.prod(src.shape[seq_axis + 1:]) * src.element_size()
    _check(getattr(lib(), name)(_ptr(src), _ptr(dst), outer, src.shape[seq_axis], inner, N, _stream()),
           name)


def sa_rope(x, y, pos, shape, base=10000.0, inverse=False):
    """y <- x with rows rotated by their position ids pos (int32 [c] or [B, c], on the GPU)."""
    if pos.dtype != torch.int32 or not pos.is_contiguous():
        raise TypeError("pos must be a contiguous int32 tensor")
    stride_b = pos.stride(0) if pos.dim() == 2 else 0
    _check(lib().sa_rope(_ptr(x), _ptr(y), _ptr(pos), stride_b, ctypes.byref(shape), float(base),
                         1 if inverse else 0, _stream()), "sa_rope")


def sa_state_init(o, lse, shape):
    _check(lib().sa_state_init(_ptr(o), _ptr(lse), ctypes.byref(shape), _stream()), "sa_state_init")


def sa_attn_step_fwd(q, k, v, o, lse, q_dev, kv_dev, N, layout, shape):
    _check(lib().sa_attn_step_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), q_dev, kv_dev, N,
                                  layout, ctypes.byref(shape), _stream()), "sa_attn_step_fwd")


def sa_attn_step_fwd_rope(q, k, v, o, lse, q_pos, q_dev, kv_dev, N, layout, shape, base=10000.0):
    """Forward step with the query rows rotated by q_pos (int32 [c] or [B, c]) as they are loaded;
    k must already be rotated (sa_rope)."""
    if q_pos.dtype != torch.int32 or not q_pos.is_contiguous():
        raise TypeError("q_pos must be a contiguous int32 tensor")
    stride_b = q_pos.stride(0) if q_pos.dim() == 2 else 0
    _check(lib().sa_attn_step_fwd_rope(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(q_pos), stride_b,
                                       float(base), q_dev, kv_dev, N, layout, ctypes.byref(shape), _stream()),
           "sa_attn_step_fwd_rope")


def sa_finalize(o, out, shape):
    _check(lib().sa_finalize(_ptr(o), _ptr(out), ctypes.byref(shape), _stream()), "sa_finalize")


def sa_bwd_preprocess(o, dout, delta, shape):
    _check(lib().sa_bwd_preprocess(_ptr(o), _ptr(dout), _ptr(delta), ctypes.byref(shape), _stream()),
           "sa_bwd_preprocess")


def sa_attn_step_bwd(q, k, v, dout, lse, delta, dq, dk, dv, q_dev, kv_dev, N, layout, shape):
    _check(lib().sa_attn_step_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(lse), _ptr(delta),
                                  _ptr(dq), _ptr(dk), _ptr(dv), q_dev, kv_dev, N, layout,
                                  ctypes.byref(shape), _stream()), "sa_attn_step_bwd")


def sa_ring_fwd(Q, K, V, O, LSE, N, layout, shape, q_dev_only=-1, timed=False):
    """Returns None, or (timed=True) an [N][N] list of step durations in ms."""
    buf = (ctypes.c_float * (N * N))() if timed else None
    _check(lib().sa_ring_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), N, layout,
                             ctypes.byref(shape), q_dev_only, buf, _stream()), "sa_ring_fwd")
    return [[buf[i * N + j] for j in range(N)] for i in range(N)] if timed else None


def sa_ring_bwd(Q, K, V, dO, O, LSE, delta, dQ, dK, dV, N, layout, shape, q_dev_only=-1, timed=False):
    buf = (ctypes.c_float * (N * N))() if timed else None
    _check(lib().sa_ring_bwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(dO), _ptr(O), _ptr(LSE), _ptr(delta),
                             _ptr(dQ), _ptr(dK), _ptr(dV), N, layout, ctypes.byref(shape), q_dev_only,
                             buf, _stream()), "sa_ring_bwd")
    return [[buf[i * N + j] for j in range(N)] for i in range(N)] if timed else None


def sa_attn_step_fwd_tiled(q, k, v, o, lse, q_dev, kv_dev, N, layout, shape, skip_bq, skip_bk):
    _check(lib().sa_attn_step_fwd_tiled(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), q_dev, kv_dev, N,
                                        layout, ctypes.byref(shape), skip_bq, skip_bk, _stream()),
           "sa_attn_step_fwd_tiled")


def sa_attn_step_bwd_tiled(q, k, v, dout, lse, delta, dq, dk, dv, q_dev, kv_dev, N, layout, shape,
                           skip_bq, skip_bk):
    _check(lib().sa_attn_step_bwd_tiled(_ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(lse), _ptr(delta),
                                        _ptr(dq), _ptr(dk), _ptr(dv), q_dev, kv_dev, N, layout,
                                        ctypes.byref(shape), skip_bq, skip_bk, _stream()),
           "sa_attn_step_bwd_tiled")


def sa_ring_fwd_tiled(Q, K, V, O, LSE, N, layout, shape, skip_bq, skip_bk, q_dev_only=-1, timed=False):
    buf = (ctypes.c_float * (N * N))() if timed else None
    _check(lib().sa_ring_fwd_tiled(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), N, layout,
                                   ctypes.byref(shape), skip_bq, skip_bk, q_dev_only, buf, _stream()),
           "sa_ring_fwd_tiled")
    return [[buf[i * N + j] for j in range(N)] for i in range(N)] if timed else None


def sa_ring_bwd_tiled(Q, K, V, dO, O, LSE, delta, dQ, dK, dV, N, layout, shape, skip_bq, skip_bk,
                      q_dev_only=-1, timed=False):
    buf = (ctypes.c_float * (N * N))() if timed else None
    _check(lib().sa_ring_bwd_tiled(_ptr(Q), _ptr(K), _ptr(V), _ptr(dO), _ptr(O), _ptr(LSE), _ptr(delta),
                                   _ptr(dQ), _ptr(dK), _ptr(dV), N, layout, ctypes.byref(shape), skip_bq,
                                   skip_bk, q_dev_only, buf, _stream()), "sa_ring_bwd_tiled")
    return [[buf[i * N + j] for j in range(N)] for i in range(N)] if timed else None


def sa_step_tiles(q_dev, kv_dev, N, layout, c, skip_bq, skip_bk):
    """(computed, total) tiles of the step's block at granularity skip_bq x skip_bk."""
    computed, total = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().sa_step_tiles(q_dev, kv_dev, N, layout, c, skip_bq, skip_bk, ctypes.byref(computed),
                               ctypes.byref(total)), "sa_step_tiles")
    return computed.value, total.value


def sa_step_mask(q_dev, kv_dev, N, layout):
    """(kind, off): kind 0 empty / 1 triangular (b <= a - off) / 2 full."""
    kind, off = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().sa_step_mask(q_dev, kv_dev, N, layout, ctypes.byref(kind), ctypes.byref(off)),
           "sa_step_mask")
    return kind.value, off.value


def sa_step_pairs(q_dev, kv_dev, N, layout, c):
    return lib().sa_step_pairs(q_dev, kv_dev, N, layout, c)


def sa_device_props():
    """(compute units, peak clock in kHz, device memory in bytes) of the current device."""
    cus, khz, mem = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int64()
    _check(lib().sa_device_props(ctypes.byref(cus), ctypes.byref(khz), ctypes.byref(mem)), "sa_device_props")
    return cus.value, khz.value, mem.value


def sa_status_str(status):
    return lib().sa_status_str(status).decode()
