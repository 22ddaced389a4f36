"""ctypes binding of libsq.so; see include/sq.h for the contract of each call."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsq.so")

if not os.path.exists(_LIB_PATH):
    raise ImportError(
        f"{_LIB_PATH} is missing: build it with `python paper_1611_07151_amd/build.py` "
        "(there is no fallback path)")

lib = ctypes.CDLL(_LIB_PATH)

SQ_F32, SQ_BF16 = 0, 1
SQ_ALGO_AUTO, SQ_ALGO_DIRECT, SQ_ALGO_VARIANT0 = 0, 1, 2
SQ_SQUEEZENET_MAX_BATCH, SQ_SQUEEZENET_BF16_MAX_BATCH = 453, 907   # as in include/sq.h

_vp, _i, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
lib.sq_strerror.restype = ctypes.c_char_p
lib.sq_strerror.argtypes = [_i]
lib.sq_last_hip_error.restype = _i
lib.sq_set_stream.argtypes = [_vp]
lib.sq_set_dtype.argtypes = [_i]
lib.sq_init.argtypes = []
lib.sq_conv_variant_count.restype = _i
lib.sq_conv_variant_name.restype = ctypes.c_char_p
lib.sq_conv_variant_name.argtypes = [_i]
lib.sq_conv2d_forward.argtypes = [_vp] * 4 + [_i] * 9
lib.sq_conv2d_forward_ex.argtypes = [_vp] * 4 + [_i] * 13
lib.sq_conv2d_forward_ws.argtypes = [_vp] * 4 + [_i] * 13 + [_vp, _sz]
lib.sq_conv2d_workspace_bytes.restype = _sz
lib.sq_conv2d_workspace_bytes.argtypes = [_i] * 5
lib.sq_conv2d_strided_workspace_bytes.restype = _sz
lib.sq_conv2d_strided_workspace_bytes.argtypes = [_i] * 8
lib.sq_conv2d_bf16_workspace_bytes.restype = _sz
lib.sq_conv2d_bf16_workspace_bytes.argtypes = [_i] * 8
lib.sq_maxpool.argtypes = [_vp, _vp] + [_i] * 6
lib.sq_maxpool_conv2d_forward.argtypes = [_vp] * 4 + [_i] * 9
lib.sq_tune_conv2d_forward_poolcols.argtypes = [_vp] * 4 + [_i] * 8 + [ctypes.POINTER(_i)]
lib.sq_tune_fire_forward_poolcols.argtypes = [_vp] * 8 + [_i] * 7 + [_vp, ctypes.c_size_t, ctypes.POINTER(_i)]
lib.sq_tune_poolrows_conv2d_forward.argtypes = [_vp] * 4 + [_i] * 9 + [ctypes.POINTER(_i)]
lib.sq_avgpool_global.argtypes = [_vp, _vp] + [_i] * 4
lib.sq_softmax.argtypes = [_vp, _vp, _i, _i]
lib.sq_fire_forward.argtypes = [_vp] * 8 + [_i] * 7 + [_vp, _sz]
lib.sq_fire_workspace_bytes.restype = _sz
lib.sq_fire_workspace_bytes.argtypes = [_i] * 5
lib.sq_squeezenet_forward.argtypes = [_vp, ctypes.POINTER(_vp), _vp, _i, _vp, _sz, ctypes.POINTER(_vp)]
lib.sq_squeezenet_workspace_bytes.restype = _sz
lib.sq_squeezenet_workspace_bytes.argtypes = [_i]
lib.sq_classifier_workspace_bytes.restype = _sz
lib.sq_classifier_workspace_bytes.argtypes = [_i] * 5
lib.sq_classifier_forward.argtypes = [_vp] * 5 + [_i] * 5 + [_vp, _sz]
lib.sq_fire_forward_static.argtypes = [_vp] * 8 + [_i] * 7
lib.sq_fire_packed_bytes.restype = _sz
lib.sq_fire_packed_bytes.argtypes = [_i, _i]
lib.sq_fire_pack_weights.argtypes = [_vp, _vp, _sz, _i, _i]
lib.sq_fire_forward_packed.argtypes = [_vp] * 9 + [_i] * 7 + [_vp, _sz]
lib.sq_packed_weights_bytes.restype = _sz
lib.sq_packed_weights_bytes.argtypes = [_i]
lib.sq_pack_weights.argtypes = [ctypes.POINTER(_vp), _i, _vp, _sz]
lib.sq_squeezenet_forward_packed.argtypes = [_vp, ctypes.POINTER(_vp), _vp, _vp, _i, _vp, _sz, ctypes.POINTER(_vp)]

lib.sq_blocked_map_bytes.restype = _sz
lib.sq_blocked_map_bytes.argtypes = [_i] * 4
lib.sq_blocked_pack.argtypes = [_vp, _i, _vp] + [_i] * 4
lib.sq_blocked_unpack.argtypes = [_vp, _vp] + [_i] * 4
lib.sq_blocked_kernel_bytes.restype = _sz
lib.sq_blocked_kernel_bytes.argtypes = [_i] * 3
lib.sq_blocked_pack_kernels.argtypes = [_vp, _i, _vp] + [_i] * 3
lib.sq_blocked_conv2d_forward.argtypes = [_vp] * 4 + [_i] * 10
lib.sq_blocked_kernel7_bytes.restype = _sz
lib.sq_blocked_kernel7_bytes.argtypes = []
lib.sq_blocked_pack_kernels7.argtypes = [_vp, _i, _vp, _i]
lib.sq_blocked_conv7s2_forward.argtypes = [_vp, _i, _vp, _vp, _vp] + [_i] * 8
lib.sq_blocked_pool_conv2d_forward.argtypes = [_vp] * 4 + [_i] * 8
lib.sq_blocked_fire_forward.argtypes = [_vp] * 8 + [_i] * 7 + [_vp, _sz]
lib.sq_blocked_maxpool.argtypes = [_vp, _vp] + [_i] * 6
lib.sq_blocked_avgpool_global.argtypes = [_vp, _vp] + [_i] * 4
lib.sq_squeezenet_bf16_packed_bytes.restype = _sz
lib.sq_squeezenet_bf16_packed_bytes.argtypes = []
lib.sq_squeezenet_bf16_pack_params.argtypes = [ctypes.POINTER(_vp), _vp, _sz]
lib.sq_squeezenet_bf16_workspace_bytes.restype = _sz
lib.sq_squeezenet_bf16_workspace_bytes.argtypes = [_i]
lib.sq_squeezenet_forward_bf16.argtypes = [_vp, _i, ctypes.POINTER(_vp), _vp, _vp, _i, _vp, _sz, ctypes.POINTER(_vp)]

lib.sq_profile_begin.argtypes = [_i]
lib.sq_profile_get_mfma_flops.argtypes = [_i, ctypes.POINTER(ctypes.c_double)]
lib.sq_profile_get.argtypes = [_i, ctypes.c_char_p, _i, ctypes.POINTER(ctypes.c_longlong),
                               ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                               ctypes.POINTER(ctypes.c_double)]

TAP_NAMES = ("conv1", "pool1", "fire2", "fire3", "fire4", "pool4", "fire5", "fire6",
             "fire7", "fire8", "pool8", "fire9", "conv10", "means", "probs")
TAP_SHAPES = ((96, 111), (96, 55), (128, 55), (128, 55), (256, 55), (256, 27), (256, 27),
              (384, 27), (384, 27), (512, 27), (512, 13), (512, 13), (1000, 13))


class SqError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        msg = lib.sq_strerror(status).decode()
        if status == -5:
            msg += f" (hipError {lib.sq_last_hip_error()})"
        super().__init__(f"{what}: {msg} [{status}]")


def sq_strerror(status: int) -> str:
    return lib.sq_strerror(int(status)).decode()


def _check(status: int, what: str) -> None:
    if status != 0:
        raise SqError(status, what)


def _dev(t, dtype=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}")
    return t.data_ptr()


def _use_current_stream():
    lib.sq_set_stream(torch.cuda.current_stream().cuda_stream)


_mode = SQ_F32   # mirror of the library's per-thread arithmetic mode, for the tensor type checks below


def sq_set_dtype(dtype: int) -> None:
    global _mode
    _check(lib.sq_set_dtype(int(dtype)), "sq_set_dtype")
    _mode = int(dtype)


def sq_init() -> None:
    _check(lib.sq_init(), "sq_init")


def sq_conv_variant_count() -> int:
    return int(lib.sq_conv_variant_count())


def sq_conv_variant_name(i: int) -> str:
    return lib.sq_conv_variant_name(int(i)).decode()


def _out_extent(h, k, s, p):
    return (h + 2 * p - k) // s + 1


def sq_conv2d_forward(x, w, b=None, stride=1, pad=0, relu=False):
    N, Cin, H, W = x.shape
    Cout, _, K, _ = w.shape
    if w.shape[1] != Cin or w.shape[3] != K:
        raise ValueError("kernel shape does not match the input")
    if H + 2 * pad < K or W + 2 * pad < K:
        _check(-2, "sq_conv2d_forward")
    out = torch.empty((N, Cout, _out_extent(H, K, stride, pad), _out_extent(W, K, stride, pad)),
                      device=x.device, dtype=torch.float32)
    _use_current_stream()
    tin = torch.float32 if _mode == SQ_F32 else torch.bfloat16
    rc = lib.sq_conv2d_forward(_dev(x, tin, "x"), _dev(w, tin, "w"),
                               _dev(b, torch.float32, "b"), _dev(out), N, Cin, H, W, Cout, K,
                               int(stride), int(pad), int(bool(relu)))
    _check(rc, "sq_conv2d_forward")
    return out


def sq_conv2d_forward_ex(x, w, b=None, stride=1, pad=0, relu=False, out=None, c_offset=0,
                         algo=SQ_ALGO_AUTO):
    """x and w float32 or both bfloat16.  `out` may be a larger [N][C'][Ho][Wo] tensor; the
    result lands in layers [c_offset, c_offset+Cout)."""
    return _conv_ex(x, w, b, stride, pad, relu, out, c_offset, algo, None, False)


def sq_conv2d_workspace_bytes(Cin, Cout, K, stride, pad) -> int:
    return int(lib.sq_conv2d_workspace_bytes(Cin, Cout, K, stride, pad))


def sq_conv2d_strided_workspace_bytes(N, Cin, H, W, Cout, K, stride, pad) -> int:
    return int(lib.sq_conv2d_strided_workspace_bytes(N, Cin, H, W, Cout, K, stride, pad))


def sq_conv2d_bf16_workspace_bytes(N, Cin, H, W, Cout, K, stride, pad) -> int:
    return int(lib.sq_conv2d_bf16_workspace_bytes(N, Cin, H, W, Cout, K, stride, pad))


def sq_conv2d_forward_ws(x, w, b=None, stride=1, pad=0, relu=False, out=None, c_offset=0,
                         algo=SQ_ALGO_AUTO, workspace=None):
    """sq_conv2d_forward_ex with device scratch (a uint8 tensor; allocated here at the largest of the sizes
    sq_conv2d_workspace_bytes, sq_conv2d_strided_workspace_bytes and, for bfloat16 operands,
    sq_conv2d_bf16_workspace_bytes report when None), which makes the kernel-transforming algorithms, the
    space-to-depth form of strided layers and the bf16 matrix instructions available."""
    if workspace is None:
        shape = (x.shape[0], x.shape[1], x.shape[2], x.shape[3], w.shape[0], w.shape[2], stride, pad)
        need = max(sq_conv2d_workspace_bytes(x.shape[1], w.shape[0], w.shape[2], stride, pad),
                   sq_conv2d_strided_workspace_bytes(*shape),
                   sq_conv2d_bf16_workspace_bytes(*shape) if x.dtype == torch.bfloat16 else 0)
        workspace = torch.empty(max(need, 256), device=x.device, dtype=torch.uint8)
    return _conv_ex(x, w, b, stride, pad, relu, out, c_offset, algo, workspace, True)


def _conv_ex(x, w, b, stride, pad, relu, out, c_offset, algo, workspace, with_ws):
    N, Cin, H, W = x.shape
    Cout, _, K, _ = w.shape
    if w.shape[1] != Cin or w.shape[3] != K:
        raise ValueError("kernel shape does not match the input")
    if x.dtype != w.dtype or x.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("x and w must both be float32 or both bfloat16")
    if H + 2 * pad < K or W + 2 * pad < K:
        _check(-2, "sq_conv2d_forward_ex")
    Ho, Wo = _out_extent(H, K, stride, pad), _out_extent(W, K, stride, pad)
    if out is None:
        out = torch.empty((N, Cout + c_offset, Ho, Wo), device=x.device, dtype=torch.float32)
    if out.shape[0] != N or out.shape[2] != Ho or out.shape[3] != Wo:
        raise ValueError("out has the wrong shape")
    dt = SQ_F32 if x.dtype == torch.float32 else SQ_BF16
    _use_current_stream()
    args = (_dev(x, None, "x"), _dev(w, None, "w"), _dev(b, torch.float32, "b"),
            _dev(out, torch.float32, "out"), N, Cin, H, W, Cout, K, int(stride),
            int(pad), int(bool(relu)), out.shape[1], int(c_offset), dt, int(algo))
    if with_ws:
        rc = lib.sq_conv2d_forward_ws(*args, _dev(workspace, torch.uint8, "workspace"), workspace.numel())
        _check(rc, "sq_conv2d_forward_ws")
    else:
        rc = lib.sq_conv2d_forward_ex(*args)
        _check(rc, "sq_conv2d_forward_ex")
    return out


def sq_maxpool(x, k=3, stride=2):
    N, C, H, W = x.shape
    if k > H or k > W:
        _check(-2, "sq_maxpool")
    out = torch.empty((N, C, (H - k) // stride + 1, (W - k) // stride + 1), device=x.device,
                      dtype=torch.float32)
    _use_current_stream()
    _check(lib.sq_maxpool(_dev(x, torch.float32, "x"), _dev(out), N, C, H, W, int(k), int(stride)),
           "sq_maxpool")
    return out


def sq_maxpool_conv2d_forward(x, w, b=None, relu=True, out=None, c_offset=0, algo=SQ_ALGO_AUTO):
    N, Cin, H, W = x.shape
    Cout = w.shape[0]
    if H < 3 or W < 3:
        _check(-2, "sq_maxpool_conv2d_forward")
    Hp, Wp = (H - 3) // 2 + 1, (W - 3) // 2 + 1
    if out is None:
        out = torch.empty((N, Cout, Hp, Wp), device=x.device, dtype=torch.float32)
    _use_current_stream()
    _check(lib.sq_maxpool_conv2d_forward(_dev(x, torch.float32, "x"), _dev(w, torch.float32, "w"),
                                         _dev(b, torch.float32, "b") if b is not None else None, _dev(out),
                                         N, Cin, H, W, Cout, int(bool(relu)), out.shape[1], int(c_offset), int(algo)),
           "sq_maxpool_conv2d_forward")
    return out


def sq_tune_conv2d_forward_poolcols(x, w, b, pad=2):
    """conv1-type layer writing the column-pooled map of its result -> (map [N, Cout, Ho, row stride], geometry)."""
    N, Cin, H, W = x.shape
    Cout, K, S = w.shape[0], w.shape[2], 2
    Ho, Wo = (H + 2 * pad - K) // S + 1, (W + 2 * pad - K) // S + 1
    out = torch.full((N * Cout * Ho * Wo,), float("nan"), device=x.device, dtype=torch.float32)
    g = (_i * 4)()
    _use_current_stream()
    _check(lib.sq_tune_conv2d_forward_poolcols(_dev(x, torch.float32, "x"), _dev(w, torch.float32, "w"), _dev(b, torch.float32, "b"),
                                               _dev(out), N, Cin, H, W, Cout, K, S, int(pad), g), "sq_tune_conv2d_forward_poolcols")
    g = list(g)
    return out[:N * Cout * Ho * g[3]].view(N, Cout, Ho, g[3]), g


def sq_tune_fire_forward_poolcols(x, w_sq, b_sq, w_e1, b_e1, w_e3, b_e3):
    """sq_fire_forward writing the column-pooled map of its result -> (map [N, Ce1 + Ce3, H, row stride], geometry)."""
    N, Cin, H, W = x.shape
    Csq, Ce1, Ce3 = w_sq.shape[0], w_e1.shape[0], w_e3.shape[0]
    ws = torch.empty(max(sq_fire_workspace_bytes(N, H, W, Csq, Ce3), 256), device=x.device, dtype=torch.uint8)
    out = torch.full((N * (Ce1 + Ce3) * H * W,), float("nan"), device=x.device, dtype=torch.float32)
    g = (_i * 4)()
    _use_current_stream()
    _check(lib.sq_tune_fire_forward_poolcols(_dev(x, torch.float32, "x"), _dev(w_sq, torch.float32, "w_sq"), _dev(b_sq, torch.float32, "b_sq"),
                                             _dev(w_e1, torch.float32, "w_e1"), _dev(b_e1, torch.float32, "b_e1"),
                                             _dev(w_e3, torch.float32, "w_e3"), _dev(b_e3, torch.float32, "b_e3"), _dev(out),
                                             N, Cin, H, W, Csq, Ce1, Ce3, _dev(ws), ws.numel(), g), "sq_tune_fire_forward_poolcols")
    g = list(g)
    return out[:N * (Ce1 + Ce3) * H * g[3]].view(N, Ce1 + Ce3, H, g[3]), g


def sq_tune_poolrows_conv2d_forward(x, W, w, b, geometry, relu=True, algo=SQ_ALGO_AUTO):
    """1x1 convolution of a column-pooled map x [N, Cin, H, row stride] of H x W results per layer."""
    N, Cin, H, rs = x.shape
    Cout = w.shape[0]
    if rs != geometry[3]:
        raise ValueError("row stride of the map and of the geometry differ")
    out = torch.empty((N, Cout, (H - 3) // 2 + 1, (W - 3) // 2 + 1), device=x.device, dtype=torch.float32)
    g = (_i * 4)(*[int(v) for v in geometry])
    _use_current_stream()
    _check(lib.sq_tune_poolrows_conv2d_forward(_dev(x, torch.float32, "x"), _dev(w, torch.float32, "w"),
                                               _dev(b, torch.float32, "b") if b is not None else None, _dev(out),
                                               N, Cin, H, int(W), Cout, int(bool(relu)), Cout, 0, int(algo), g),
           "sq_tune_poolrows_conv2d_forward")
    return out


def sq_avgpool_global(x):
    N, C, H, W = x.shape
    out = torch.empty((N, C), device=x.device, dtype=torch.float32)
    _use_current_stream()
    _check(lib.sq_avgpool_global(_dev(x, torch.float32, "x"), _dev(out), N, C, H, W), "sq_avgpool_global")
    return out


def sq_softmax(x):
    N, C = x.shape
    out = torch.empty((N, C), device=x.device, dtype=torch.float32)
    _use_current_stream()
    _check(lib.sq_softmax(_dev(x, torch.float32, "x"), _dev(out), N, C), "sq_softmax")
    return out


def sq_classifier_forward(x, w, b=None, want_means=False, workspace=None):
    """relu(conv1x1) -> global average pooling -> softmax.  x [N][Cin][H][W], w [Cout][Cin][1][1] or [Cout][Cin];
    returns probs [N][Cout], or (probs, means) with want_means."""
    N, Cin, H, W = x.shape
    Cout = w.shape[0]
    if w.numel() != Cout * Cin:
        raise ValueError("kernel shape does not match the input")
    if workspace is None:
        workspace = torch.empty(max(256, int(lib.sq_classifier_workspace_bytes(N, Cin, H, W, Cout))), device=x.device, dtype=torch.uint8)
    probs = torch.empty((N, Cout), device=x.device, dtype=torch.float32)
    means = torch.empty((N, Cout), device=x.device, dtype=torch.float32) if want_means else None
    _use_current_stream()
    rc = lib.sq_classifier_forward(_dev(x, torch.float32, "x"), _dev(w, torch.float32, "w"), _dev(b, torch.float32, "b"),
                                   _dev(means), _dev(probs), N, Cin, H, W, Cout, _dev(workspace), workspace.numel())
    _check(rc, "sq_classifier_forward")
    return (probs, means) if want_means else probs


def sq_fire_workspace_bytes(N, H, W, Csq, Ce3) -> int:
    return int(lib.sq_fire_workspace_bytes(N, H, W, Csq, Ce3))


def sq_fire_forward(x, w_sq, b_sq, w_e1, b_e1, w_e3, b_e3, workspace=None, out=None):
    N, Cin, H, W = x.shape
    Csq, Ce1, Ce3 = w_sq.shape[0], w_e1.shape[0], w_e3.shape[0]
    if tuple(w_sq.shape) != (Csq, Cin, 1, 1) or tuple(w_e1.shape) != (Ce1, Csq, 1, 1) \
            or tuple(w_e3.shape) != (Ce3, Csq, 3, 3):
        raise ValueError("fire kernel shapes")
    need = sq_fire_workspace_bytes(N, H, W, Csq, Ce3)
    if workspace is None:
        workspace = torch.empty(need, device=x.device, dtype=torch.uint8)
    if out is None:
        out = torch.empty((N, Ce1 + Ce3, H, W), device=x.device, dtype=torch.float32)
    f32 = torch.float32
    _use_current_stream()
    rc = lib.sq_fire_forward(_dev(x, f32, "x"), _dev(w_sq, f32, "w_sq"), _dev(b_sq, f32, "b_sq"),
                             _dev(w_e1, f32, "w_e1"), _dev(b_e1, f32, "b_e1"), _dev(w_e3, f32, "w_e3"),
                             _dev(b_e3, f32, "b_e3"), _dev(out, f32, "out"), N, Cin, H, W, Csq, Ce1, Ce3,
                             _dev(workspace), workspace.numel() * workspace.element_size())
    _check(rc, "sq_fire_forward")
    return out


SQ_FIRE_STATIC_SCRATCH_BYTES = 32 << 20   # as in include/sq.h


def sq_fire_forward_static(x, w_sq, b_sq, w_e1, b_e1, w_e3, b_e3, out):
    """The fire layer with its scratch inside the library: the caller passes inputs and the output tensor,
    and nothing is allocated here or in the library."""
    N, Cin, H, W = x.shape
    Csq, Ce1, Ce3 = w_sq.shape[0], w_e1.shape[0], w_e3.shape[0]
    if tuple(w_sq.shape) != (Csq, Cin, 1, 1) or tuple(w_e1.shape) != (Ce1, Csq, 1, 1) \
            or tuple(w_e3.shape) != (Ce3, Csq, 3, 3) or tuple(out.shape) != (N, Ce1 + Ce3, H, W):
        raise ValueError("fire kernel or output shapes")
    f32 = torch.float32
    _use_current_stream()
    rc = lib.sq_fire_forward_static(_dev(x, f32, "x"), _dev(w_sq, f32, "w_sq"), _dev(b_sq, f32, "b_sq"),
                                    _dev(w_e1, f32, "w_e1"), _dev(b_e1, f32, "b_e1"), _dev(w_e3, f32, "w_e3"),
                                    _dev(b_e3, f32, "b_e3"), _dev(out, f32, "out"), N, Cin, H, W, Csq, Ce1, Ce3)
    _check(rc, "sq_fire_forward_static")
    return out


def sq_fire_packed_bytes(Csq, Ce3) -> int:
    return int(lib.sq_fire_packed_bytes(int(Csq), int(Ce3)))


def sq_fire_pack_weights(w_e3):
    """Expand3x3 kernels [Ce3][Csq][3][3] float32 -> their re-ordered form (uint8 tensor), written once."""
    Ce3, Csq = w_e3.shape[0], w_e3.shape[1]
    if tuple(w_e3.shape[2:]) != (3, 3):
        raise ValueError("expects [Ce3][Csq][3][3]")
    out = torch.empty(max(sq_fire_packed_bytes(Csq, Ce3), 256), device=w_e3.device, dtype=torch.uint8)
    _use_current_stream()
    _check(lib.sq_fire_pack_weights(_dev(w_e3, torch.float32, "w_e3"), _dev(out), out.numel(), Csq, Ce3), "sq_fire_pack_weights")
    return out


def sq_fire_forward_packed(x, w_sq, b_sq, w_e1, b_e1, w_e3, b_e3, packed_e3, workspace=None, out=None):
    N, Cin, H, W = x.shape
    Csq, Ce1, Ce3 = w_sq.shape[0], w_e1.shape[0], w_e3.shape[0]
    if tuple(w_sq.shape) != (Csq, Cin, 1, 1) or tuple(w_e1.shape) != (Ce1, Csq, 1, 1) \
            or tuple(w_e3.shape) != (Ce3, Csq, 3, 3):
        raise ValueError("fire kernel shapes")
    if workspace is None:
        workspace = torch.empty((N * Csq * H * W * 4 + 255) // 256 * 256, device=x.device, dtype=torch.uint8)
    if out is None:
        out = torch.empty((N, Ce1 + Ce3, H, W), device=x.device, dtype=torch.float32)
    f32 = torch.float32
    _use_current_stream()
    rc = lib.sq_fire_forward_packed(_dev(x, f32, "x"), _dev(w_sq, f32, "w_sq"), _dev(b_sq, f32, "b_sq"),
                                    _dev(w_e1, f32, "w_e1"), _dev(b_e1, f32, "b_e1"), _dev(w_e3, f32, "w_e3"),
                                    _dev(b_e3, f32, "b_e3"), _dev(packed_e3, torch.uint8, "packed_e3"), _dev(out, f32, "out"),
                                    N, Cin, H, W, Csq, Ce1, Ce3, _dev(workspace), workspace.numel() * workspace.element_size())
    _check(rc, "sq_fire_forward_packed")
    return out


def sq_squeezenet_workspace_bytes(N) -> int:
    return int(lib.sq_squeezenet_workspace_bytes(int(N)))


def sq_squeezenet_forward(x, params, workspace=None, probs=None, want_taps=False):
    """x [N,3,224,224] float32; params: 52 device tensors (kernel, bias per convolution in
    network order).  Returns probs [N,1000], or (probs, {stage: tensor}) with want_taps."""
    N = x.shape[0]
    if tuple(x.shape[1:]) != (3, 224, 224) or len(params) != 52:
        raise ValueError("expects [N,3,224,224] and 52 parameter tensors")
    if workspace is None:
        workspace = torch.empty(sq_squeezenet_workspace_bytes(N), device=x.device, dtype=torch.uint8)
    if probs is None:
        probs = torch.empty((N, 1000), device=x.device, dtype=torch.float32)
    parr = (_vp * 52)(*[_dev(p, torch.float32, f"params[{i}]") for i, p in enumerate(params)])
    taps, tarr = {}, None
    if want_taps:
        for name, (c, h) in zip(TAP_NAMES, TAP_SHAPES):
            taps[name] = torch.empty((N, c, h, h), device=x.device, dtype=torch.float32)
        taps["means"] = torch.empty((N, 1000), device=x.device, dtype=torch.float32)
        taps["probs"] = torch.empty((N, 1000), device=x.device, dtype=torch.float32)
        tarr = (_vp * 16)(*([taps[n].data_ptr() for n in TAP_NAMES] + [None]))
    _use_current_stream()
    rc = lib.sq_squeezenet_forward(_dev(x, torch.float32, "x"), parr, _dev(probs, torch.float32, "probs"),
                                   N, _dev(workspace), workspace.numel() * workspace.element_size(), tarr)
    _check(rc, "sq_squeezenet_forward")
    return (probs, taps) if want_taps else probs


def sq_packed_weights_bytes(dtype=SQ_F32) -> int:
    return int(lib.sq_packed_weights_bytes(int(dtype)))


def sq_pack_weights(params, dtype=SQ_F32):
    """One-time re-ordering of the network's kernels for the given arithmetic mode -> packed uint8 tensor."""
    if len(params) != 52:
        raise ValueError("expects 52 parameter tensors")
    out = torch.empty(sq_packed_weights_bytes(dtype), device=params[0].device, dtype=torch.uint8)
    parr = (_vp * 52)(*[_dev(p, torch.float32, f"params[{i}]") for i, p in enumerate(params)])
    _use_current_stream()
    _check(lib.sq_pack_weights(parr, int(dtype), _dev(out), out.numel()), "sq_pack_weights")
    return out


def sq_squeezenet_forward_packed(x, params, packed, workspace=None, probs=None, want_taps=False):
    """sq_squeezenet_forward on kernels packed by sq_pack_weights for the mode of sq_set_dtype."""
    N = x.shape[0]
    if tuple(x.shape[1:]) != (3, 224, 224) or len(params) != 52:
        raise ValueError("expects [N,3,224,224] and 52 parameter tensors")
    if workspace is None:
        workspace = torch.empty(sq_squeezenet_workspace_bytes(N), device=x.device, dtype=torch.uint8)
    if probs is None:
        probs = torch.empty((N, 1000), device=x.device, dtype=torch.float32)
    parr = (_vp * 52)(*[_dev(p, torch.float32, f"params[{i}]") for i, p in enumerate(params)])
    taps, tarr = {}, None
    if want_taps:
        for name, (c, h) in zip(TAP_NAMES, TAP_SHAPES):
            taps[name] = torch.empty((N, c, h, h), device=x.device, dtype=torch.float32)
        taps["means"] = torch.empty((N, 1000), device=x.device, dtype=torch.float32)
        taps["probs"] = torch.empty((N, 1000), device=x.device, dtype=torch.float32)
        tarr = (_vp * 16)(*([taps[n].data_ptr() for n in TAP_NAMES] + [None]))
    _use_current_stream()
    rc = lib.sq_squeezenet_forward_packed(_dev(x, torch.float32, "x"), parr, _dev(packed, torch.uint8, "packed"),
                                          _dev(probs, torch.float32, "probs"), N, _dev(workspace),
                                          workspace.numel() * workspace.element_size(), tarr)
    _check(rc, "sq_squeezenet_forward_packed")
    return (probs, taps) if want_taps else probs


def _dtype_code(t, name):
    if t.dtype == torch.float32:
        return SQ_F32
    if t.dtype == torch.bfloat16:
        return SQ_BF16
    raise ValueError(f"{name} must be float32 or bfloat16")


def sq_blocked_map_bytes(N, C, H, W) -> int:
    return int(lib.sq_blocked_map_bytes(N, C, H, W))


def _new_map(N, C, H, W, device):
    """Blocked map [N][ceil(C/8)][H][W][8] as a bfloat16 tensor."""
    return torch.empty((N, (C + 7) // 8, H, W, 8), device=device, dtype=torch.bfloat16)


def sq_blocked_pack(x):
    """NCHW float32 / bfloat16 -> blocked bfloat16 map [N][ceil(C/8)][H][W][8]."""
    N, C, H, W = x.shape
    out = _new_map(N, C, H, W, x.device)
    _use_current_stream()
    _check(lib.sq_blocked_pack(_dev(x, None, "x"), _dtype_code(x, "x"), _dev(out), N, C, H, W), "sq_blocked_pack")
    return out


def sq_blocked_unpack(m, C):
    """Blocked map -> NCHW float32 with C layers."""
    N, CB, H, W, _ = m.shape
    if m.shape[4] != 8 or (C + 7) // 8 != CB:
        raise ValueError("not a blocked map of C layers")
    out = torch.empty((N, C, H, W), device=m.device, dtype=torch.float32)
    _use_current_stream()
    _check(lib.sq_blocked_unpack(_dev(m, torch.bfloat16, "m"), _dev(out), N, C, H, W), "sq_blocked_unpack")
    return out


def sq_blocked_kernel_bytes(Cout, Cin, K) -> int:
    return int(lib.sq_blocked_kernel_bytes(Cout, Cin, K))


def sq_blocked_pack_kernels(w):
    """Kernels [Cout][Cin][K][K] (float32 / bfloat16) -> packed buffer (uint8 tensor)."""
    Cout, Cin, K, K2 = w.shape
    if K != K2:
        raise ValueError("square kernels only")
    out = torch.empty(sq_blocked_kernel_bytes(Cout, Cin, K), device=w.device, dtype=torch.uint8)
    _use_current_stream()
    _check(lib.sq_blocked_pack_kernels(_dev(w, None, "w"), _dtype_code(w, "w"), _dev(out), Cout, Cin, K),
           "sq_blocked_pack_kernels")
    return out


def sq_blocked_conv2d_forward(m, packed_w, b, Cin, Cout, K, pad, relu=False, out=None, c_offset=0):
    """m: blocked map of Cin layers; out: blocked map (default: a new one of Cout layers)."""
    N, CB, H, W, _ = m.shape
    if m.shape[4] != 8 or (Cin + 7) // 8 != CB:
        raise ValueError("not a blocked map of Cin layers")
    if out is None:
        out = _new_map(N, Cout, H, W, m.device)
    if tuple(out.shape[:1] + out.shape[2:]) != (N, H, W, 8):
        raise ValueError("output map shape")
    _use_current_stream()
    rc = lib.sq_blocked_conv2d_forward(_dev(m, torch.bfloat16, "m"), _dev(packed_w, torch.uint8, "packed_w"),
                                       _dev(b, torch.float32, "b"), _dev(out, torch.bfloat16, "out"), N, Cin, H, W,
                                       Cout, int(K), int(pad), 1 if relu else 0, out.shape[1] * 8, int(c_offset))
    _check(rc, "sq_blocked_conv2d_forward")
    return out


def sq_blocked_kernel7_bytes() -> int:
    return int(lib.sq_blocked_kernel7_bytes())


def sq_blocked_pack_kernels7(w):
    """conv1-type kernels [Cout][3][7][7] (float32 / bfloat16) -> packed buffer (uint8 tensor)."""
    if tuple(w.shape[1:]) != (3, 7, 7):
        raise ValueError("expects [Cout][3][7][7]")
    out = torch.empty(sq_blocked_kernel7_bytes(), device=w.device, dtype=torch.uint8)
    _use_current_stream()
    _check(lib.sq_blocked_pack_kernels7(_dev(w, None, "w"), _dtype_code(w, "w"), _dev(out), w.shape[0]),
           "sq_blocked_pack_kernels7")
    return out


def sq_blocked_conv7s2_forward(x, packed_w, b, Cout, pad, relu=False, out=None, c_offset=0):
    """x: NCHW image [N][3][H][W], float32 or bfloat16; out: blocked map (default: a new one of Cout layers)."""
    N, C, H, W = x.shape
    if C != 3:
        raise ValueError("three input layers")
    if H + 2 * pad < 7 or W + 2 * pad < 7:
        _check(-2, "sq_blocked_conv7s2_forward")
    Ho, Wo = (H + 2 * pad - 7) // 2 + 1, (W + 2 * pad - 7) // 2 + 1
    if out is None:
        out = _new_map(N, Cout, Ho, Wo, x.device)
    _use_current_stream()
    rc = lib.sq_blocked_conv7s2_forward(_dev(x, None, "x"), _dtype_code(x, "x"), _dev(packed_w, torch.uint8, "packed_w"),
                                        _dev(b, torch.float32, "b"), _dev(out, torch.bfloat16, "out"), N, H, W, Cout,
                                        int(pad), 1 if relu else 0, out.shape[1] * 8, int(c_offset))
    _check(rc, "sq_blocked_conv7s2_forward")
    return out


def sq_blocked_pool_conv2d_forward(m, packed_w, b, Cin, Cout, relu=False, out=None, c_offset=0):
    """3x3 stride-2 max pooling of a blocked map of Cin layers, then a 1x1 convolution to Cout layers."""
    N, CB, Hin, Win, _ = m.shape
    if m.shape[4] != 8 or (Cin + 7) // 8 != CB:
        raise ValueError("not a blocked map of Cin layers")
    if Hin < 3 or Win < 3:
        _check(-2, "sq_blocked_pool_conv2d_forward")
    if out is None:
        out = _new_map(N, Cout, (Hin - 3) // 2 + 1, (Win - 3) // 2 + 1, m.device)
    _use_current_stream()
    rc = lib.sq_blocked_pool_conv2d_forward(_dev(m, torch.bfloat16, "m"), _dev(packed_w, torch.uint8, "packed_w"),
                                            _dev(b, torch.float32, "b"), _dev(out, torch.bfloat16, "out"), N, Cin, Hin, Win,
                                            Cout, 1 if relu else 0, out.shape[1] * 8, int(c_offset))
    _check(rc, "sq_blocked_pool_conv2d_forward")
    return out


def sq_blocked_fire_forward(m, Cin, packed_sq, b_sq, packed_e1, b_e1, packed_e3, b_e3, Csq, Ce1, Ce3, workspace=None):
    """Fire layer on a blocked map of Cin layers; returns the blocked map of Ce1 + Ce3 layers."""
    N, CB, H, W, _ = m.shape
    if m.shape[4] != 8 or (Cin + 7) // 8 != CB:
        raise ValueError("not a blocked map of Cin layers")
    if workspace is None:
        workspace = torch.empty(sq_blocked_map_bytes(N, Csq, H, W), device=m.device, dtype=torch.uint8)
    out = _new_map(N, Ce1 + Ce3, H, W, m.device)
    u8, f32 = torch.uint8, torch.float32
    _use_current_stream()
    rc = lib.sq_blocked_fire_forward(_dev(m, torch.bfloat16, "m"), _dev(packed_sq, u8, "packed_sq"), _dev(b_sq, f32, "b_sq"),
                                     _dev(packed_e1, u8, "packed_e1"), _dev(b_e1, f32, "b_e1"),
                                     _dev(packed_e3, u8, "packed_e3"), _dev(b_e3, f32, "b_e3"), _dev(out), N, Cin, H, W,
                                     Csq, Ce1, Ce3, _dev(workspace), workspace.numel() * workspace.element_size())
    _check(rc, "sq_blocked_fire_forward")
    return out


def sq_blocked_maxpool(m, C, k, stride):
    N, CB, H, W, _ = m.shape
    if H < k or W < k:
        _check(-2, "sq_blocked_maxpool")
    out = _new_map(N, C, (H - k) // stride + 1, (W - k) // stride + 1, m.device)
    _use_current_stream()
    _check(lib.sq_blocked_maxpool(_dev(m, torch.bfloat16, "m"), _dev(out), N, C, H, W, int(k), int(stride)),
           "sq_blocked_maxpool")
    return out


def sq_blocked_avgpool_global(m, C):
    N, CB, H, W, _ = m.shape
    out = torch.empty((N, C), device=m.device, dtype=torch.float32)
    _use_current_stream()
    _check(lib.sq_blocked_avgpool_global(_dev(m, torch.bfloat16, "m"), _dev(out), N, C, H, W),
           "sq_blocked_avgpool_global")
    return out


def sq_squeezenet_bf16_packed_bytes() -> int:
    return int(lib.sq_squeezenet_bf16_packed_bytes())


def sq_squeezenet_bf16_pack_params(params):
    """One-time re-ordering of the 26 kernels (52 float32 parameter tensors in) -> packed uint8 tensor."""
    if len(params) != 52:
        raise ValueError("expects 52 parameter tensors")
    out = torch.empty(sq_squeezenet_bf16_packed_bytes(), device=params[0].device, dtype=torch.uint8)
    parr = (_vp * 52)(*[_dev(p, torch.float32, f"params[{i}]") for i, p in enumerate(params)])
    _use_current_stream()
    _check(lib.sq_squeezenet_bf16_pack_params(parr, _dev(out), out.numel()), "sq_squeezenet_bf16_pack_params")
    return out


def sq_squeezenet_bf16_workspace_bytes(N) -> int:
    return int(lib.sq_squeezenet_bf16_workspace_bytes(int(N)))


def sq_squeezenet_forward_bf16(x, params, packed, workspace=None, probs=None, want_taps=False):
    """x [N,3,224,224] float32 or bfloat16; params as for sq_squeezenet_forward; packed from
    sq_squeezenet_bf16_pack_params.  Returns probs, or (probs, taps) with float32 NCHW stage copies."""
    N = x.shape[0]
    if tuple(x.shape[1:]) != (3, 224, 224) or len(params) != 52:
        raise ValueError("expects [N,3,224,224] and 52 parameter tensors")
    if workspace is None:
        workspace = torch.empty(sq_squeezenet_bf16_workspace_bytes(N), device=x.device, dtype=torch.uint8)
    if probs is None:
        probs = torch.empty((N, 1000), device=x.device, dtype=torch.float32)
    parr = (_vp * 52)(*[_dev(p, torch.float32, f"params[{i}]") for i, p in enumerate(params)])
    taps, tarr = {}, None
    if want_taps:
        for name, (c, h) in zip(TAP_NAMES, TAP_SHAPES):
            taps[name] = torch.empty((N, c, h, h), device=x.device, dtype=torch.float32)
        taps["means"] = torch.empty((N, 1000), device=x.device, dtype=torch.float32)
        taps["probs"] = torch.empty((N, 1000), device=x.device, dtype=torch.float32)
        tarr = (_vp * 16)(*([taps[n].data_ptr() for n in TAP_NAMES] + [None]))
    _use_current_stream()
    rc = lib.sq_squeezenet_forward_bf16(_dev(x, None, "x"), _dtype_code(x, "x"), parr, _dev(packed, torch.uint8, "packed"),
                                        _dev(probs, torch.float32, "probs"), N, _dev(workspace),
                                        workspace.numel() * workspace.element_size(), tarr)
    _check(rc, "sq_squeezenet_forward_bf16")
    return (probs, taps) if want_taps else probs


def sq_profile_begin(max_launches: int = 4096) -> None:
    _use_current_stream()
    _check(lib.sq_profile_begin(int(max_launches)), "sq_profile_begin")


def sq_profile_end():
    """Returns a list of dicts: name ("stage|kernel"), launches, ms, flops, bytes, mfma_flops."""
    _check(lib.sq_profile_end(), "sq_profile_end")
    out = []
    for i in range(lib.sq_profile_count()):
        name = ctypes.create_string_buffer(128)
        n, ms = ctypes.c_longlong(), ctypes.c_double()
        fl, by = ctypes.c_double(), ctypes.c_double()
        _check(lib.sq_profile_get(i, name, 128, ctypes.byref(n), ctypes.byref(ms), ctypes.byref(fl),
                                  ctypes.byref(by)), "sq_profile_get")
        mf = ctypes.c_double()
        _check(lib.sq_profile_get_mfma_flops(i, ctypes.byref(mf)), "sq_profile_get_mfma_flops")
        out.append(dict(name=name.value.decode(), launches=n.value, ms=ms.value, flops=fl.value,
                        bytes=by.value, mfma_flops=mf.value))
    return out
