"""ctypes binding of include/dp_bk.h.  Same names, same argument order; tensors may be
passed as torch tensors (their data_ptr is taken) or as integer device addresses.
PyTorch is used for nothing but device memory and the current stream."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdp_bk.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2311_11822_amd.build` "
        "(there is no CPU or PyTorch fallback for the HIP kernels)")

lib = C.CDLL(LIB_PATH)

DP_OK, DP_ERR_INVALID_ARG, DP_ERR_UNSUPPORTED, DP_ERR_WORKSPACE, DP_ERR_HIP = range(5)
DP_F32, DP_BF16, DP_F16 = 0, 1, 2
DP_CLIP_STANDARD, DP_CLIP_AUTOMATIC = 0, 1
DP_PATH_GHOST, DP_PATH_PEREX = 0, 1


class dp_layer(C.Structure):
    _fields_ = [("a", C.c_void_p), ("g", C.c_void_p), ("T", C.c_int32), ("d_in", C.c_int32),
                ("d_out", C.c_int32), ("path", C.c_int32)]


_vp, _i, _f, _u64, _sz = C.c_void_p, C.c_int, C.c_float, C.c_uint64, C.c_size_t
_PROTOS = {
    "dp_status_string": (C.c_char_p, [_i]),
    "dp_version": (_i, []),
    "dp_choose_path": (_i, [C.c_int64, C.c_int64, C.c_int64]),
    "dp_norm_workspace_bytes": (_sz, [_i, _i, _i, _i, _i, _i]),
    "dp_ghost_norm": (_i, [_vp, _vp, _i, _i, _i, _i, _i, _vp, _vp, _sz, _vp]),
    "dp_perex_norm": (_i, [_vp, _vp, _i, _i, _i, _i, _i, _vp, _vp, _sz, _vp]),
    "dp_clip_factors": (_i, [_vp, _i, _i, _i, _f, _f, _vp, _vp, _vp]),
    "dp_clipped_grad": (_i, [_vp, _vp, _i, _i, _i, _i, _i, _vp, _vp, _i, _vp]),
    "dp_add_noise": (_i, [_vp, _u64, _u64, _f, _f, _u64, _u64, _vp]),
    "dp_philox_blocks": (_i, [_vp, _u64, _u64, _u64, _u64, _vp]),
    "dp_norms_multi_workspace_bytes": (_sz, [C.POINTER(dp_layer), _i, _i, _i]),
    "dp_norms_multi": (_i, [C.POINTER(dp_layer), _i, _i, _i, _vp, _vp, _sz, _vp]),
    "dp_norms_multi_static": (_i, [C.POINTER(dp_layer), _i, _i, _i, _vp, _vp]),
    "dp_clipped_grad_multi": (_i, [C.POINTER(dp_layer), _i, _i, _i, _vp, C.POINTER(_vp), _i, _vp]),
    "dp_clipped_grad_noise_multi": (_i, [C.POINTER(dp_layer), _i, _i, _i, _vp, C.POINTER(_vp),
                                        C.POINTER(_u64), _i, _u64, _u64, _f, _f, _u64, _u64, _vp]),
    "dp_clipped_grad_noise_multi_h16": (_i, [C.POINTER(dp_layer), _i, _i, _i, _vp, C.POINTER(_vp),
                                            C.POINTER(_u64), _i, _u64, _u64, _f, _f, _u64, _u64, _vp]),
    "dp_clip_factors_grouped": (_i, [_vp, _i, _i, C.POINTER(C.c_int32), _i, C.POINTER(_f), _i, _f, _vp, _vp, _vp]),
    "dp_clipped_grad_grouped": (_i, [C.POINTER(dp_layer), _i, _i, _i, _vp, C.POINTER(C.c_int32), _i,
                                     C.POINTER(_vp), _i, _vp]),
    "dp_group_noise_threshold": (_f, [C.POINTER(_f), _i]),
    "dp_bias_norm": (_i, [_vp, _i, _i, _i, _i, _vp, _vp, _vp]),
    "dp_clipped_bias_grad": (_i, [_vp, _i, _i, _vp, _vp, _i, _vp]),
    "dp_norms_multi_keep": (_i, [C.POINTER(dp_layer), _i, _i, _i, _vp, C.POINTER(_vp), _vp, _sz, _vp]),
    "dp_clipped_grad_kept_multi": (_i, [C.POINTER(dp_layer), _i, _i, _i, _vp, C.POINTER(_vp), C.POINTER(_vp),
                                       C.POINTER(_u64), _i, _u64, _u64, _f, _f, _u64, _u64, _vp]),
    "dp_layerwise_workspace_bytes": (_sz, [C.POINTER(dp_layer), _i, _i, _i]),
    "dp_layerwise_clipped_grad": (_i, [C.POINTER(dp_layer), _i, _i, _i, C.POINTER(_f), _i, _f, C.POINTER(_vp),
                                      C.POINTER(_u64), _i, _u64, _u64, _f, _u64, _u64, _vp, _vp, _vp, _sz, _i, _vp]),
    "dp_clipped_grad_tile_order": (C.c_int64, [_i, _i, _vp, _vp, C.c_int64]),
    "dp_ghost_tile_order": (C.c_int64, [_i, _i, _vp, _vp, _vp, _vp, C.c_int64]),
}
EXPORTS = tuple(_PROTOS)
for _name, (_res, _args) in _PROTOS.items():
    _fn = getattr(lib, _name)          # AttributeError here = header/library mismatch
    _fn.restype, _fn.argtypes = _res, _args


class DpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib.dp_status_string(status).decode()} (dp_status {status})")


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is not None:
        return stream if isinstance(stream, int) else stream.cuda_stream
    import torch
    return torch.cuda.current_stream().cuda_stream


def _nbytes(ws) -> int:
    return 0 if ws is None else ws.numel() * ws.element_size()


def _check(status: int, where: str) -> None:
    if status != DP_OK:
        raise DpError(status, where)


def layer_array(layers: Sequence) -> "C.Array[dp_layer]":
    """layers: sequence of (a, g, T, d_in, d_out, path)."""
    arr = (dp_layer * len(layers))()
    for k, (a, g, T, d_in, d_out, path) in enumerate(layers):
        arr[k] = dp_layer(_ptr(a), _ptr(g), T, d_in, d_out, path)
    return arr


def dp_version() -> int:
    return lib.dp_version()


def dp_choose_path(T: int, d_in: int, d_out: int) -> int:
    return lib.dp_choose_path(T, d_in, d_out)


def dp_norm_workspace_bytes(path, dt, B, T, d_in, d_out) -> int:
    return lib.dp_norm_workspace_bytes(path, dt, B, T, d_in, d_out)


def dp_ghost_norm(a, g, dt, B, T, d_in, d_out, sqnorm_out, ws, stream=None) -> None:
    _check(lib.dp_ghost_norm(_ptr(a), _ptr(g), dt, B, T, d_in, d_out, _ptr(sqnorm_out), _ptr(ws),
                             _nbytes(ws), _stream(stream)), "dp_ghost_norm")


def dp_perex_norm(a, g, dt, B, T, d_in, d_out, sqnorm_out, ws, stream=None) -> None:
    _check(lib.dp_perex_norm(_ptr(a), _ptr(g), dt, B, T, d_in, d_out, _ptr(sqnorm_out), _ptr(ws),
                             _nbytes(ws), _stream(stream)), "dp_perex_norm")


def dp_clip_factors(sqnorm, L, B, mode, R, stability, C_out, norm_out=None, stream=None) -> None:
    _check(lib.dp_clip_factors(_ptr(sqnorm), L, B, mode, R, stability, _ptr(C_out), _ptr(norm_out),
                               _stream(stream)), "dp_clip_factors")


def dp_clipped_grad(a, g, dt, B, T, d_in, d_out, Cf, grad, accumulate=0, stream=None) -> None:
    _check(lib.dp_clipped_grad(_ptr(a), _ptr(g), dt, B, T, d_in, d_out, _ptr(Cf), _ptr(grad),
                               accumulate, _stream(stream)), "dp_clipped_grad")


def dp_add_noise(grad_slice, global_offset, count, sigma, R, seed, step, stream=None) -> None:
    _check(lib.dp_add_noise(_ptr(grad_slice), global_offset, count, sigma, R, seed, step,
                            _stream(stream)), "dp_add_noise")


def dp_philox_blocks(out, first_block, n_blocks, seed, step, stream=None) -> None:
    _check(lib.dp_philox_blocks(_ptr(out), first_block, n_blocks, seed, step, _stream(stream)),
           "dp_philox_blocks")


def dp_norms_multi_workspace_bytes(layers, dt, B) -> int:
    arr = layers if isinstance(layers, C.Array) else layer_array(layers)
    return lib.dp_norms_multi_workspace_bytes(arr, len(arr), dt, B)


def dp_norms_multi(layers, dt, B, sqnorm_out, ws, stream=None) -> None:
    arr = layers if isinstance(layers, C.Array) else layer_array(layers)
    _check(lib.dp_norms_multi(arr, len(arr), dt, B, _ptr(sqnorm_out), _ptr(ws), _nbytes(ws),
                              _stream(stream)), "dp_norms_multi")


def dp_norms_multi_static(layers, dt, B, sqnorm_out, stream=None) -> None:
    arr = layers if isinstance(layers, C.Array) else layer_array(layers)
    _check(lib.dp_norms_multi_static(arr, len(arr), dt, B, _ptr(sqnorm_out), _stream(stream)),
           "dp_norms_multi_static")


def dp_clipped_grad_multi(layers, dt, B, Cf, grads, accumulate=0, stream=None) -> None:
    arr = layers if isinstance(layers, C.Array) else layer_array(layers)
    gp = grads if isinstance(grads, C.Array) else (C.c_void_p * len(grads))(*[_ptr(x) for x in grads])
    _check(lib.dp_clipped_grad_multi(arr, len(arr), dt, B, _ptr(Cf), gp, accumulate, _stream(stream)),
           "dp_clipped_grad_multi")


def dp_clipped_grad_noise_multi(layers, dt, B, Cf, grads, grad_offset, accumulate, shard_offset, shard_count,
                                sigma, R, seed, step, stream=None) -> None:
    arr = layers if isinstance(layers, C.Array) else layer_array(layers)
    gp = grads if isinstance(grads, C.Array) else (C.c_void_p * len(grads))(*[_ptr(x) for x in grads])
    offs = grad_offset if isinstance(grad_offset, C.Array) else (C.c_uint64 * len(grad_offset))(*grad_offset)
    _check(lib.dp_clipped_grad_noise_multi(arr, len(arr), dt, B, _ptr(Cf), gp, offs, accumulate, shard_offset,
                                           shard_count, sigma, R, seed, step, _stream(stream)),
           "dp_clipped_grad_noise_multi")


def dp_clipped_grad_noise_multi_h16(layers, dt, B, Cf, grads16, grad_offset, accumulate, shard_offset, shard_count,
                                    sigma, R, seed, step, stream=None) -> None:
    arr = layers if isinstance(layers, C.Array) else layer_array(layers)
    gp = grads16 if isinstance(grads16, C.Array) else (C.c_void_p * len(grads16))(*[_ptr(x) for x in grads16])
    offs = None
    if grad_offset is not None:
        offs = grad_offset if isinstance(grad_offset, C.Array) else (C.c_uint64 * len(grad_offset))(*grad_offset)
    _check(lib.dp_clipped_grad_noise_multi_h16(arr, len(arr), dt, B, _ptr(Cf), gp, offs, accumulate, shard_offset,
                                               shard_count, sigma, R, seed, step, _stream(stream)),
           "dp_clipped_grad_noise_multi_h16")


def _i32(xs):
    return (C.c_int32 * len(xs))(*xs)


def _f32(xs):
    return (C.c_float * len(xs))(*xs)


def dp_clip_factors_grouped(sqnorm, L, B, group_begin, R, mode, stability, C_out, norm_out=None,
                            stream=None) -> None:
    M = len(R)
    _check(lib.dp_clip_factors_grouped(_ptr(sqnorm), L, B, _i32(group_begin), M, _f32(R), mode, stability,
                                       _ptr(C_out), _ptr(norm_out), _stream(stream)),
           "dp_clip_factors_grouped")


def dp_clipped_grad_grouped(layers, dt, B, Cf, group_of_layer, M, grads, accumulate=0, stream=None) -> None:
    arr = layers if isinstance(layers, C.Array) else layer_array(layers)
    gp = grads if isinstance(grads, C.Array) else (C.c_void_p * len(grads))(*[_ptr(x) for x in grads])
    _check(lib.dp_clipped_grad_grouped(arr, len(arr), dt, B, _ptr(Cf), _i32(group_of_layer), M, gp, accumulate,
                                       _stream(stream)), "dp_clipped_grad_grouped")


def dp_group_noise_threshold(R) -> float:
    return lib.dp_group_noise_threshold(_f32(R), len(R))


def dp_bias_norm(g, dt, B, T, d_out, colsum, sqnorm_out, stream=None) -> None:
    _check(lib.dp_bias_norm(_ptr(g), dt, B, T, d_out, _ptr(colsum), _ptr(sqnorm_out), _stream(stream)),
           "dp_bias_norm")


def dp_clipped_bias_grad(colsum, B, d_out, Cf, grad_b, accumulate=0, stream=None) -> None:
    _check(lib.dp_clipped_bias_grad(_ptr(colsum), B, d_out, _ptr(Cf), _ptr(grad_b), accumulate, _stream(stream)),
           "dp_clipped_bias_grad")


def _ptr_array(xs):
    """HOST array of device pointers; None entries become NULL."""
    if isinstance(xs, C.Array):
        return xs
    return (C.c_void_p * len(xs))(*[_ptr(x) for x in xs])


def dp_norms_multi_keep(layers, dt, B, sqnorm_out, kept, ws, stream=None) -> None:
    arr = layers if isinstance(layers, C.Array) else layer_array(layers)
    _check(lib.dp_norms_multi_keep(arr, len(arr), dt, B, _ptr(sqnorm_out), _ptr_array(kept) if kept is not None else None,
                                   _ptr(ws), _nbytes(ws), _stream(stream)), "dp_norms_multi_keep")


def dp_clipped_grad_kept_multi(layers, dt, B, Cf, kept, grads, grad_offset, accumulate, shard_offset, shard_count,
                               sigma, R, seed, step, stream=None) -> None:
    arr = layers if isinstance(layers, C.Array) else layer_array(layers)
    offs = None
    if grad_offset is not None:
        offs = grad_offset if isinstance(grad_offset, C.Array) else (C.c_uint64 * len(grad_offset))(*grad_offset)
    _check(lib.dp_clipped_grad_kept_multi(arr, len(arr), dt, B, _ptr(Cf), _ptr_array(kept) if kept is not None else None,
                                          _ptr_array(grads), offs, accumulate, shard_offset, shard_count, sigma, R,
                                          seed, step, _stream(stream)), "dp_clipped_grad_kept_multi")


def dp_layerwise_workspace_bytes(layers, dt, B) -> int:
    arr = layers if isinstance(layers, C.Array) else layer_array(layers)
    return lib.dp_layerwise_workspace_bytes(arr, len(arr), dt, B)


def dp_layerwise_clipped_grad(layers, dt, B, R, mode, stability, grads, grad_offset, accumulate, shard_offset,
                              shard_count, sigma, seed, step, sqnorm_out, C_out, ws, layers_per_pass=0,
                              stream=None) -> None:
    arr = layers if isinstance(layers, C.Array) else layer_array(layers)
    gp = grads if isinstance(grads, C.Array) else (C.c_void_p * len(grads))(*[_ptr(x) for x in grads])
    offs = None
    if grad_offset is not None:
        offs = grad_offset if isinstance(grad_offset, C.Array) else (C.c_uint64 * len(grad_offset))(*grad_offset)
    _check(lib.dp_layerwise_clipped_grad(arr, len(arr), dt, B, _f32(R), mode, stability, gp, offs, accumulate,
                                         shard_offset, shard_count, sigma, seed, step, _ptr(sqnorm_out),
                                         _ptr(C_out), _ptr(ws), _nbytes(ws), layers_per_pass, _stream(stream)),
           "dp_layerwise_clipped_grad")


def dp_clipped_grad_tile_order(d_in: int, d_out: int):
    """(tile_row0, tile_col0) numpy int32 arrays in launch order (host function)."""
    import numpy as np
    n = lib.dp_clipped_grad_tile_order(d_in, d_out, None, None, 0)
    if n < 0:
        raise DpError(DP_ERR_INVALID_ARG, "dp_clipped_grad_tile_order")
    r, c = np.zeros(n, dtype=np.int32), np.zeros(n, dtype=np.int32)
    lib.dp_clipped_grad_tile_order(d_in, d_out, r.ctypes.data, c.ctypes.data, n)
    return r, c


def dp_ghost_tile_order(T: int, B: int):
    """(sample, token_row0, token_col0, slot) numpy int32 arrays in launch order (host function)."""
    import numpy as np
    n = lib.dp_ghost_tile_order(T, B, None, None, None, None, 0)
    if n < 0:
        raise DpError(DP_ERR_INVALID_ARG, "dp_ghost_tile_order")
    out = [np.zeros(n, dtype=np.int32) for _ in range(4)]
    lib.dp_ghost_tile_order(T, B, *[x.ctypes.data for x in out], n)
    return tuple(out)
