"""ctypes binding of the C ABI in include/adam_mini.h -- argument marshalling only.

Every function here has the name of the C entry point it calls.  ``AdamMini`` is
a small convenience holder that keeps the layout handle and the pointer arrays of
a tensor list together; it performs no arithmetic either.  If the HIP library has
not been built, loading fails with an error: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libadam_mini.so")

OK, INVALID_ARG, MISALIGNED, OUT_OF_MEMORY, HIP_ERROR, NO_DEVICE, TOO_LARGE = 0, -1, -2, -3, -4, -5, -6
STATIC_SCRATCH_BYTES = 16 << 20
GRAD_F32, GRAD_BF16 = 0, 1
PATH_ELEMENTWISE, PATH_ROW, PATH_LARGE, PATH_ROW_LDS, PATH_STRIDED, PATH_FUSED = 0, 1, 2, 3, 4, 5
FLAG_STRIDED = 1
# adam_mini_tensor_desc.flags bits 4-6: block statistic of g*g that feeds v
REDUCE_FLAGS = {"mean": 0 << 4, "norm1": 1 << 4, "norm2": 2 << 4, "max": 3 << 4, "min": 4 << 4}


class TensorDesc(ctypes.Structure):
    _fields_ = [("numel", ctypes.c_uint64), ("block_numel", ctypes.c_uint64),
                ("wd_scale", ctypes.c_float), ("flags", ctypes.c_uint32)]


class HParams(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float), ("step", ctypes.c_uint64)]


class BucketInfo(ctypes.Structure):
    _fields_ = [("family", ctypes.c_int32), ("vec", ctypes.c_int32), ("lanes", ctypes.c_int32),
                ("upt", ctypes.c_int32), ("n_tensors", ctypes.c_uint32), ("n_kernels", ctypes.c_uint32),
                ("n_items", ctypes.c_uint64), ("numel", ctypes.c_uint64), ("n_blocks", ctypes.c_uint64),
                ("timed_launches", ctypes.c_uint64), ("total_ms", ctypes.c_double),
                ("kernel", ctypes.c_char * 96)]


class AdamMiniError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = "%s: %s (%d)" % (where, adam_mini_strerror(status), status)
        if status in (HIP_ERROR, OUT_OF_MEMORY):
            msg += " -- " + adam_mini_last_hip_error()
        super().__init__(msg)


_lib = None

EXPORTS = ["adam_mini_init_layout", "adam_mini_num_blocks", "adam_mini_num_tensors",
           "adam_mini_export_layout", "adam_mini_block_id", "adam_mini_write_block_ids",
           "adam_mini_step", "adam_mini_step_static", "adam_mini_step_device_hparams", "adam_mini_set_option", "adam_mini_num_buckets",
           "adam_mini_profile_enable", "adam_mini_profile_read", "adam_mini_destroy_layout",
           "adam_mini_strerror", "adam_mini_last_hip_error"]


def load(path: Optional[str] = None):
    """Load libadam_mini.so (built by paper_2406_16793_amd/build.py).  Raises if absent."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise FileNotFoundError(
            "%s is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')" % p)
    # PyTorch ships its own copy of the HIP runtime (same soname).  Device pointers and
    # streams come from torch, so the library must bind to THAT runtime: load torch first,
    # otherwise the process ends up with two runtimes that do not see each other's memory.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(p)
    vp, u32, u64, i32 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int
    lib.adam_mini_init_layout.restype = i32
    lib.adam_mini_init_layout.argtypes = [ctypes.POINTER(TensorDesc), u32, i32, i32, ctypes.POINTER(vp)]
    lib.adam_mini_num_blocks.restype = u64
    lib.adam_mini_num_blocks.argtypes = [vp]
    lib.adam_mini_num_tensors.restype = u32
    lib.adam_mini_num_tensors.argtypes = [vp]
    lib.adam_mini_export_layout.restype = i32
    lib.adam_mini_export_layout.argtypes = [vp, ctypes.POINTER(u64), ctypes.POINTER(u32)]
    lib.adam_mini_block_id.restype = i32
    lib.adam_mini_block_id.argtypes = [vp, u32, u64, ctypes.POINTER(u64)]
    lib.adam_mini_write_block_ids.restype = i32
    lib.adam_mini_write_block_ids.argtypes = [vp, u32, vp, vp]
    lib.adam_mini_step.restype = i32
    lib.adam_mini_step.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), vp,
                                   ctypes.POINTER(HParams), vp]
    lib.adam_mini_step_static.restype = i32
    lib.adam_mini_step_static.argtypes = lib.adam_mini_step.argtypes
    lib.adam_mini_step_device_hparams.restype = i32
    lib.adam_mini_step_device_hparams.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), vp,
                                                  vp, u32, vp]
    lib.adam_mini_num_buckets.restype = u32
    lib.adam_mini_num_buckets.argtypes = [vp]
    lib.adam_mini_profile_enable.restype = i32
    lib.adam_mini_profile_enable.argtypes = [vp, u32]
    lib.adam_mini_profile_read.restype = i32
    lib.adam_mini_profile_read.argtypes = [vp, ctypes.POINTER(BucketInfo), u32]
    lib.adam_mini_set_option.restype = i32
    lib.adam_mini_set_option.argtypes = [ctypes.c_char_p, ctypes.c_int64]
    lib.adam_mini_destroy_layout.restype = None
    lib.adam_mini_destroy_layout.argtypes = [vp]
    lib.adam_mini_strerror.restype = ctypes.c_char_p
    lib.adam_mini_strerror.argtypes = [i32]
    lib.adam_mini_last_hip_error.restype = ctypes.c_char_p
    lib.adam_mini_last_hip_error.argtypes = []
    if path is None:
        _lib = lib
    return lib


def _check(status: int, where: str) -> None:
    if status != OK:
        raise AdamMiniError(status, where)


# ---- one function per C entry point ----------------------------------------
def adam_mini_strerror(status: int) -> str:
    return load().adam_mini_strerror(int(status)).decode()


def adam_mini_last_hip_error() -> str:
    return load().adam_mini_last_hip_error().decode()


def adam_mini_set_option(key: str, value: int) -> None:
    _check(load().adam_mini_set_option(key.encode(), int(value)), "adam_mini_set_option(%s)" % key)


def adam_mini_init_layout(descs: Sequence[Tuple[int, int, float]], grad_dtype: int, device: int) -> int:
    """descs: (numel, block_numel, wd_scale) per tensor.  Returns the opaque handle."""
    arr = (TensorDesc * max(1, len(descs)))()
    for i, d in enumerate(descs):
        arr[i].numel, arr[i].block_numel, arr[i].wd_scale = int(d[0]), int(d[1]), float(d[2])
        arr[i].flags = int(d[3]) if len(d) > 3 else 0
    out = ctypes.c_void_p()
    _check(load().adam_mini_init_layout(arr, len(descs), int(grad_dtype), int(device), ctypes.byref(out)),
           "adam_mini_init_layout")
    return out.value


def adam_mini_num_blocks(layout: int) -> int:
    return int(load().adam_mini_num_blocks(layout))


def adam_mini_num_tensors(layout: int) -> int:
    return int(load().adam_mini_num_tensors(layout))


def adam_mini_export_layout(layout: int) -> Tuple[List[int], List[int]]:
    n = adam_mini_num_tensors(layout)
    voff = (ctypes.c_uint64 * (n + 1))()
    kind = (ctypes.c_uint32 * max(1, n))()
    _check(load().adam_mini_export_layout(layout, voff, kind), "adam_mini_export_layout")
    return list(voff), list(kind)[:n]


def adam_mini_block_id(layout: int, tensor: int, elem: int) -> int:
    out = ctypes.c_uint64()
    _check(load().adam_mini_block_id(layout, int(tensor), int(elem), ctypes.byref(out)), "adam_mini_block_id")
    return int(out.value)


def adam_mini_write_block_ids(layout: int, tensor: int, ids_dev_ptr: int, stream: int = 0) -> None:
    _check(load().adam_mini_write_block_ids(layout, int(tensor), ctypes.c_void_p(ids_dev_ptr),
                                            ctypes.c_void_p(stream)), "adam_mini_write_block_ids")


def adam_mini_step(layout: int, params, grads, exp_avg, v_dev_ptr: int, hp: HParams, stream: int = 0) -> None:
    """params / grads / exp_avg: ctypes arrays of c_void_p holding device pointers."""
    _check(load().adam_mini_step(layout, params, grads, exp_avg, ctypes.c_void_p(v_dev_ptr),
                                 ctypes.byref(hp), ctypes.c_void_p(stream)), "adam_mini_step")


def adam_mini_step_static(layout: int, params, grads, exp_avg, v_dev_ptr: int, hp: HParams, stream: int = 0) -> None:
    """Same arguments as adam_mini_step; allocates nothing (fixed scratch inside the library)."""
    _check(load().adam_mini_step_static(layout, params, grads, exp_avg, ctypes.c_void_p(v_dev_ptr),
                                        ctypes.byref(hp), ctypes.c_void_p(stream)), "adam_mini_step_static")


STEP_ADVANCE = 1


def adam_mini_step_device_hparams(layout: int, params, grads, exp_avg, v_dev_ptr: int, hp_dev_ptr: int,
                                  flags: int = 0, stream: int = 0) -> None:
    """hp_dev_ptr: device pointer to one HParams (32 bytes).  flags: STEP_ADVANCE or 0."""
    _check(load().adam_mini_step_device_hparams(layout, params, grads, exp_avg, ctypes.c_void_p(v_dev_ptr),
                                                ctypes.c_void_p(hp_dev_ptr), int(flags), ctypes.c_void_p(stream)),
           "adam_mini_step_device_hparams")


def adam_mini_num_buckets(layout: int) -> int:
    return int(load().adam_mini_num_buckets(layout))


def adam_mini_profile_enable(layout: int, max_steps: int) -> None:
    _check(load().adam_mini_profile_enable(layout, int(max_steps)), "adam_mini_profile_enable")


def adam_mini_profile_read(layout: int) -> List[dict]:
    n = adam_mini_num_buckets(layout)
    arr = (BucketInfo * max(1, n))()
    _check(load().adam_mini_profile_read(layout, arr, n), "adam_mini_profile_read")
    return [{f: (getattr(arr[i], f).decode() if f == "kernel" else getattr(arr[i], f))
             for f, _ in BucketInfo._fields_} for i in range(n)]


def adam_mini_destroy_layout(layout: int) -> None:
    load().adam_mini_destroy_layout(layout)


def device_hparams(lr, beta1, beta2, eps, weight_decay, step: int, device: int = 0):
    """One HParams record in GPU memory (a 32-byte torch tensor): marshalling only."""
    import torch
    raw = bytes(HParams(lr, beta1, beta2, eps, weight_decay, step))
    return torch.frombuffer(bytearray(raw), dtype=torch.uint8).to("cuda:%d" % device)


# ---- convenience holder ------------------------------------------------------
def pointer_array(ptrs: Sequence[int]):
    arr = (ctypes.c_void_p * max(1, len(ptrs)))()
    for i, p in enumerate(ptrs):
        arr[i] = p
    return arr


class AdamMini:
    """Keeps a layout handle and the pointer lists of torch tensors together.

    params / grads / exp_avg are lists of flat, contiguous torch tensors on one
    GPU; v is a float32 tensor of num_blocks elements on the same GPU.  step()
    enqueues on torch's current stream.  No computation happens in Python.
    """

    def __init__(self, specs, grad_dtype: str, device: int = 0):
        self.specs = list(specs)
        self.grad_dtype = GRAD_BF16 if grad_dtype == "bf16" else GRAD_F32
        self.device = device
        self.layout = adam_mini_init_layout([(s.numel, s.block_numel, s.wd_scale,
                                              (FLAG_STRIDED if getattr(s, "strided", False) else 0)
                                              | REDUCE_FLAGS[getattr(s, "reducer", "mean")])
                                             for s in self.specs],
                                            self.grad_dtype, device)
        self.num_blocks = adam_mini_num_blocks(self.layout)
        self._ptrs = None
        self._keep = None

    def bind(self, params, grads, exp_avg, v) -> None:
        import torch
        want_g = torch.bfloat16 if self.grad_dtype == GRAD_BF16 else torch.float32
        for s, p, g, m in zip(self.specs, params, grads, exp_avg):
            for t, dt in ((p, torch.float32), (g, want_g), (m, torch.float32)):
                if t.dtype != dt or t.numel() != s.numel or not t.is_contiguous() or not t.is_cuda:
                    raise ValueError("tensor %s: wrong dtype, size, device or layout" % s.name)
        if v.dtype != torch.float32 or v.numel() != self.num_blocks or not v.is_cuda:
            raise ValueError("v must be float32[%d] on the GPU" % self.num_blocks)
        self._keep = (params, grads, exp_avg, v)
        self._ptrs = (pointer_array([t.data_ptr() for t in params]),
                      pointer_array([t.data_ptr() for t in grads]),
                      pointer_array([t.data_ptr() for t in exp_avg]), v.data_ptr())

    def step(self, lr, beta1, beta2, eps, weight_decay, step: int, stream: Optional[int] = None,
             static: bool = False) -> None:
        """static=True calls adam_mini_step_static (no allocation; fixed scratch inside the library)."""
        import torch
        if self._ptrs is None:
            raise RuntimeError("bind() the tensors first")
        if stream is None:
            stream = torch.cuda.current_stream(self.device).cuda_stream
        hp = HParams(lr, beta1, beta2, eps, weight_decay, step)
        entry = adam_mini_step_static if static else adam_mini_step
        entry(self.layout, self._ptrs[0], self._ptrs[1], self._ptrs[2], self._ptrs[3], hp, stream)

    def step_device_hparams(self, hp_dev, advance: bool = True, stream: Optional[int] = None) -> None:
        """hp_dev: a torch uint8 tensor of 32 bytes on the GPU holding one HParams (see device_hparams())."""
        import torch
        if self._ptrs is None:
            raise RuntimeError("bind() the tensors first")
        if stream is None:
            stream = torch.cuda.current_stream(self.device).cuda_stream
        adam_mini_step_device_hparams(self.layout, self._ptrs[0], self._ptrs[1], self._ptrs[2], self._ptrs[3],
                                      hp_dev.data_ptr(), STEP_ADVANCE if advance else 0, stream)

    def block_ids(self, tensor: int):
        import torch
        out = torch.empty(self.specs[tensor].numel, dtype=torch.int64, device="cuda:%d" % self.device)
        adam_mini_write_block_ids(self.layout, tensor, out.data_ptr(),
                                  torch.cuda.current_stream(self.device).cuda_stream)
        return out

    def close(self) -> None:
        if self.layout:
            adam_mini_destroy_layout(self.layout)
            self.layout = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
