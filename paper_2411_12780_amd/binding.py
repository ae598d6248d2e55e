"""ctypes binding of libppll.so: same names as include/ppll.h, argument
marshalling only.  Device memory and streams come from PyTorch-ROCm; every step
of the path runs in the library's kernels.  There is no fallback: a missing
library is an error."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libppll.so")

PPLL_OK = 0
ERR_NAMES = {1: "PPLL_ERR_NULL", 2: "PPLL_ERR_CONFIG", 3: "PPLL_ERR_SHAPE", 4: "PPLL_ERR_WORKSPACE",
             5: "PPLL_ERR_HIP", 6: "PPLL_ERR_LABEL", 7: "PPLL_ERR_STATE"}
T_PARAM, T_GRAD, T_MOMENT1, T_MOMENT2, T_BN_MEAN, T_BN_VAR = range(6)


class PpllError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{ERR_NAMES.get(status, status)}: {text}")
        self.status = status


class BlockConfig(C.Structure):
    """Mirror of ppll_block_config."""
    _fields_ = [("struct_size", C.c_uint32), ("arch", C.c_int32), ("precision", C.c_int32),
                ("input_kind", C.c_int32), ("batch", C.c_int32), ("num_classes", C.c_int32),
                ("img_h", C.c_int32), ("img_w", C.c_int32), ("img_c", C.c_int32), ("patch", C.c_int32),
                ("tokens", C.c_int32), ("dim", C.c_int32), ("heads", C.c_int32), ("mlp_dim", C.c_int32),
                ("depth", C.c_int32), ("aux_depth", C.c_int32),
                ("channels", C.c_int32), ("height", C.c_int32), ("width", C.c_int32),
                ("n_basic_blocks", C.c_int32), ("aux_channels", C.c_int32), ("transition_block", C.c_int32),
                ("optimizer", C.c_int32), ("momentum", C.c_float), ("nesterov", C.c_int32),
                ("weight_decay", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("adam_eps", C.c_float), ("ln_eps", C.c_float), ("bn_eps", C.c_float),
                ("bn_momentum", C.c_float), ("seed", C.c_uint64)]


def make_config(wl: dict) -> BlockConfig:
    """Workload dict (see synth.WORKLOADS) -> ppll_block_config; unknown keys are ignored."""
    cfg = BlockConfig()
    defaults = dict(beta1=0.9, beta2=0.999, adam_eps=1e-8, ln_eps=1e-6, bn_eps=1e-5, bn_momentum=0.1)
    names = {f[0] for f in BlockConfig._fields_}
    for k, v in {**defaults, **wl}.items():
        if k in names:
            setattr(cfg, k, v)
    cfg.struct_size = C.sizeof(BlockConfig)
    return cfg


_lib = None
_SIGS = {
    "ppll_last_error": (C.c_char_p, []),
    "ppll_block_workspace_bytes": (C.c_int, [C.POINTER(BlockConfig), C.POINTER(C.c_size_t)]),
    "ppll_block_param_bytes": (C.c_int, [C.POINTER(BlockConfig), C.POINTER(C.c_size_t)]),
    "ppll_block_in_bytes": (C.c_int, [C.POINTER(BlockConfig), C.POINTER(C.c_size_t)]),
    "ppll_block_out_bytes": (C.c_int, [C.POINTER(BlockConfig), C.POINTER(C.c_size_t)]),
    "ppll_block_init": (C.c_int, [C.POINTER(BlockConfig), C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p,
                                  C.POINTER(C.c_void_p)]),
    "ppll_block_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p,
                                  C.c_void_p]),
    "ppll_block_sync": (C.c_int, [C.c_void_p, C.POINTER(C.c_float)]),
    "ppll_block_tensor_count": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]),
    "ppll_block_tensor_info": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_char_p),
                                         C.POINTER(C.c_size_t)]),
    "ppll_block_read_tensor": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t]),
    "ppll_block_write_tensor": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t]),
    "ppll_block_destroy": (C.c_int, [C.c_void_p]),
    "ppll_pipeline_workspace_bytes": (C.c_int, [C.POINTER(BlockConfig), C.c_int32, C.c_int32,
                                                C.POINTER(C.c_size_t)]),
    "ppll_pipeline_init": (C.c_int, [C.POINTER(BlockConfig), C.c_int32, C.c_int32, C.c_void_p, C.c_size_t,
                                     C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p)]),
    "ppll_pipeline_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_void_p]),
    "ppll_pipeline_sync": (C.c_int, [C.c_void_p, C.POINTER(C.c_float)]),
    "ppll_pipeline_block": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_void_p)]),
    "ppll_pipeline_output": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_size_t)]),
    "ppll_pipeline_destroy": (C.c_int, [C.c_void_p]),
    "ppll_probe_copy": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "ppll_block_forward_eval": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "ppll_block_forward_eval_noalloc": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "ppll_block_phase_timers": (C.c_int, [C.c_void_p, C.c_int32]),
    "ppll_block_phase_times": (C.c_int, [C.c_void_p, C.POINTER(C.c_float)]),
    "ppll_block_profile_enable": (C.c_int, [C.c_void_p, C.c_int32]),
    "ppll_block_profile_read": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
    "ppll_block_profile_read_conv": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
    "ppll_block_profile_read_small": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
}
EXPORTS = tuple(_SIGS)


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no CPU fallback)")
        # PyTorch-ROCm ships its own HIP runtime and owns the device memory and streams handed to
        # the library: load it first so that the process holds a single libamdhip64.
        import torch  # noqa: F401
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def _check(status: int) -> None:
    if status != PPLL_OK:
        raise PpllError(status, lib().ppll_last_error().decode())


def _ptr(t) -> Optional[int]:
    """Device/host address of a torch tensor, numpy array, int or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def ppll_last_error() -> str:
    return lib().ppll_last_error().decode()


def _size_query(fn_name: str, cfg: BlockConfig) -> int:
    out = C.c_size_t(0)
    _check(getattr(lib(), fn_name)(C.byref(cfg), C.byref(out)))
    return out.value


def ppll_block_workspace_bytes(cfg): return _size_query("ppll_block_workspace_bytes", cfg)
def ppll_block_param_bytes(cfg): return _size_query("ppll_block_param_bytes", cfg)
def ppll_block_in_bytes(cfg): return _size_query("ppll_block_in_bytes", cfg)
def ppll_block_out_bytes(cfg): return _size_query("ppll_block_out_bytes", cfg)


def ppll_block_init(cfg: BlockConfig, workspace, workspace_bytes: int, init_params: Optional[np.ndarray],
                    stream=None) -> int:
    if init_params is not None:
        init_params = np.ascontiguousarray(init_params, dtype=np.float32)
        if init_params.nbytes != ppll_block_param_bytes(cfg):
            raise PpllError(3, f"parameter blob has {init_params.nbytes} bytes")
    h = C.c_void_p(0)
    _check(lib().ppll_block_init(C.byref(cfg), _ptr(workspace), workspace_bytes, _ptr(init_params), _ptr(stream),
                                 C.byref(h)))
    return h.value


def ppll_block_step(blk: int, x_in, labels, lr: float, x_out, loss=None, stream=None) -> None:
    _check(lib().ppll_block_step(blk, _ptr(x_in), _ptr(labels), lr, _ptr(x_out), _ptr(loss), _ptr(stream)))


def ppll_block_sync(blk: int) -> float:
    out = C.c_float(0)
    _check(lib().ppll_block_sync(blk, C.byref(out)))
    return out.value


def ppll_block_tensor_count(blk: int, kind: int = T_PARAM) -> int:
    n = C.c_int32(0)
    _check(lib().ppll_block_tensor_count(blk, kind, C.byref(n)))
    return n.value


def ppll_block_tensor_info(blk: int, kind: int, index: int):
    name, n = C.c_char_p(), C.c_size_t(0)
    _check(lib().ppll_block_tensor_info(blk, kind, index, C.byref(name), C.byref(n)))
    return name.value.decode(), n.value


def ppll_block_read_tensor(blk: int, kind: int, index: int) -> np.ndarray:
    _, n = ppll_block_tensor_info(blk, kind, index)
    out = np.empty(n, dtype=np.float32)
    _check(lib().ppll_block_read_tensor(blk, kind, index, out.ctypes.data, n))
    return out


def ppll_block_write_tensor(blk: int, kind: int, index: int, values: np.ndarray) -> None:
    values = np.ascontiguousarray(values, dtype=np.float32).reshape(-1)
    _check(lib().ppll_block_write_tensor(blk, kind, index, values.ctypes.data, values.size))


def ppll_block_destroy(blk: int) -> None:
    _check(lib().ppll_block_destroy(blk))


def _cfg_array(cfgs: Sequence[BlockConfig]):
    arr = (BlockConfig * len(cfgs))()
    for i, c in enumerate(cfgs):
        arr[i] = c
    return arr


def ppll_pipeline_workspace_bytes(cfgs: Sequence[BlockConfig], queue_depth: int) -> int:
    out = C.c_size_t(0)
    _check(lib().ppll_pipeline_workspace_bytes(_cfg_array(cfgs), len(cfgs), queue_depth, C.byref(out)))
    return out.value


def ppll_pipeline_init(cfgs: Sequence[BlockConfig], queue_depth: int, workspace, workspace_bytes: int,
                       streams: Sequence, init_params: Optional[Sequence[Optional[np.ndarray]]]) -> int:
    K = len(cfgs)
    s_arr = (C.c_void_p * K)(*[_ptr(s) for s in streams])
    keep: List[np.ndarray] = []
    p_arr = None
    if init_params is not None:
        p_arr = (C.c_void_p * K)()
        for j, p in enumerate(init_params):
            if p is not None:
                a = np.ascontiguousarray(p, dtype=np.float32)
                keep.append(a)
                p_arr[j] = a.ctypes.data
    h = C.c_void_p(0)
    _check(lib().ppll_pipeline_init(_cfg_array(cfgs), K, queue_depth, _ptr(workspace), workspace_bytes, s_arr, p_arr,
                                    C.byref(h)))
    return h.value


def ppll_pipeline_step(pipe: int, x0, labels, lr: float, losses=None) -> None:
    _check(lib().ppll_pipeline_step(pipe, _ptr(x0), _ptr(labels), lr, _ptr(losses)))


def ppll_pipeline_sync(pipe: int, K: int) -> np.ndarray:
    out = (C.c_float * K)()
    _check(lib().ppll_pipeline_sync(pipe, out))
    return np.array(out[:], dtype=np.float32)


def ppll_pipeline_block(pipe: int, j: int) -> int:
    h = C.c_void_p(0)
    _check(lib().ppll_pipeline_block(pipe, j, C.byref(h)))
    return h.value


def ppll_pipeline_output(pipe: int):
    p, n = C.c_void_p(0), C.c_size_t(0)
    _check(lib().ppll_pipeline_output(pipe, C.byref(p), C.byref(n)))
    return p.value, n.value


def ppll_pipeline_destroy(pipe: int) -> None:
    _check(lib().ppll_pipeline_destroy(pipe))


def ppll_block_forward_eval(block, x_in, x_out, logits=None, stream=None) -> None:
    _check(lib().ppll_block_forward_eval(block, _ptr(x_in), _ptr(x_out), _ptr(logits), _ptr(stream)))


EVAL_SCRATCH_BYTES = 64 << 20


def ppll_block_forward_eval_noalloc(block, x_in, x_out, logits=None, stream=None) -> None:
    _check(lib().ppll_block_forward_eval_noalloc(block, _ptr(x_in), _ptr(x_out), _ptr(logits), _ptr(stream)))


def ppll_block_phase_timers(block, on: bool) -> None:
    _check(lib().ppll_block_phase_timers(block, 1 if on else 0))


def ppll_block_phase_times(block):
    """(f, f_a, B, U) of the block's last step in milliseconds."""
    ms = (C.c_float * 4)()
    _check(lib().ppll_block_phase_times(block, ms))
    return tuple(float(v) for v in ms)


def ppll_block_profile_enable(block, on: bool) -> None:
    _check(lib().ppll_block_profile_enable(block, 1 if on else 0))


def ppll_block_profile_read(block):
    """(milliseconds, flops, launches) of the block's GEMM launches bracketed since the last read."""
    ms, fl, n = C.c_double(0), C.c_double(0), C.c_int64(0)
    _check(lib().ppll_block_profile_read(block, C.byref(ms), C.byref(fl), C.byref(n)))
    return ms.value, fl.value, n.value


def ppll_block_profile_read_conv(block):
    """(milliseconds, algorithmic bytes, launches) of the block's convolution launches bracketed since the last read."""
    ms, by, n = C.c_double(0), C.c_double(0), C.c_int64(0)
    _check(lib().ppll_block_profile_read_conv(block, C.byref(ms), C.byref(by), C.byref(n)))
    return ms.value, by.value, n.value


def ppll_block_profile_read_small(block):
    """(milliseconds, flops, launches) of the block's GEMM launches with fewer than 256 output rows since the last read."""
    ms, fl, n = C.c_double(0), C.c_double(0), C.c_int64(0)
    _check(lib().ppll_block_profile_read_small(block, C.byref(ms), C.byref(fl), C.byref(n)))
    return ms.value, fl.value, n.value


def ppll_probe_copy(src, dst, nbytes: int, stream=None) -> None:
    _check(lib().ppll_probe_copy(_ptr(src), _ptr(dst), nbytes, _ptr(stream)))
