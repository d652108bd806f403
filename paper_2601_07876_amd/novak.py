"""Thin ctypes binding over libnovak.so: the C entry points under their own names.

Argument marshalling only; every step of the update runs in the library's HIP kernels.  There is
no fallback: if the shared library is missing or fails to load, importing the functions raises.
PyTorch is imported first so that this library binds to the same HIP runtime that owns the
tensors' memory and streams.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libnovak.so")

# ---- constants of include/novak.h -----------------------------------------------------------------
NOVAK_OK, NOVAK_ERR_INVALID_ARG, NOVAK_ERR_NULL_POINTER, NOVAK_ERR_MISALIGNED = 0, 1, 2, 3
NOVAK_ERR_BAD_STEP, NOVAK_ERR_STATE, NOVAK_ERR_HIP, NOVAK_ERR_NOT_IMPLEMENTED, NOVAK_ERR_NO_MEMORY = 4, 5, 6, 7, 8
NOVAK_NESTEROV_NONE, NOVAK_NESTEROV_APPROX, NOVAK_NESTEROV_CLASSICAL, NOVAK_NESTEROV_TRUE = 0, 1, 2, 3
NOVAK_LOOKAHEAD_NONE, NOVAK_LOOKAHEAD_MEMORY_EFFICIENT, NOVAK_LOOKAHEAD_BASIC = 0, 1, 2
NOVAK_UNRECT_ADAM_DENOM, NOVAK_UNRECT_SGDM = 0, 1
NOVAK_MODE_FAST, NOVAK_MODE_RESEARCH = 0, 1
NOVAK_GRAD_F32, NOVAK_GRAD_BF16 = 0, 1
NOVAK_MOMENT_F32, NOVAK_MOMENT_BF16_M = 0, 1
NOVAK_WARN_TRUE_NESTEROV_DOWNGRADED, NOVAK_WARN_LOOKAHEAD_DOWNGRADED = 1, 2
NOVAK_WARN_LAYER_ADAPTATION_DISABLED, NOVAK_WARN_AUTO_LR_DISABLED, NOVAK_WARN_GC_DISABLED = 4, 8, 16
NOVAK_TUNE_CHUNK_ELEMS, NOVAK_TUNE_NONTEMPORAL, NOVAK_TUNE_VEC_PER_LANE, NOVAK_TUNE_THREADS, NOVAK_TUNE_WAVES_PER_CU = 0, 1, 2, 3, 4
NOVAK_TUNE_PREPASS_WAVES_PER_CU = 5

NOVAK_STATIC_MAX_TENSORS, NOVAK_STATIC_MAX_CHUNKS, NOVAK_STATIC_SCRATCH_BYTES = 1024, 32768, 2 << 20
NOVAK_ARENA_TENSOR_ALIGN, NOVAK_ARENA_ROLE_PERIOD, NOVAK_ARENA_ROLE_SKEW = 256, 8192, 2048

NESTEROV = {"none": 0, "approx": 1, "classical": 2, "true": 3}
LOOKAHEAD = {"none": 0, "memory_efficient": 1, "basic": 2}
UNRECT = {"adam_denom": 0, "sgdm": 1}
MODE = {"fast": 0, "research": 1}
GRAD_DTYPE = {"f32": 0, "bf16": 1}
MOMENT_DTYPE = {"f32": 0, "bf16_m": 1}


class novak_hparams(C.Structure):
    _fields_ = [("struct_size", C.c_size_t),
                ("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
                ("weight_decay", C.c_double), ("beta_n", C.c_double), ("la_alpha", C.c_double),
                ("la_k", C.c_int32), ("rectified", C.c_int32), ("decoupled_decay", C.c_int32),
                ("nesterov_mode", C.c_int32), ("lookahead_mode", C.c_int32), ("unrect_fallback", C.c_int32),
                ("mode", C.c_int32), ("auto_sync", C.c_int32),
                ("layer_adaptation", C.c_int32), ("auto_lr", C.c_int32), ("auto_lr_gamma", C.c_double),
                ("trust_clip_lo", C.c_double), ("trust_clip_hi", C.c_double),
                ("auto_clip_lo", C.c_double), ("auto_clip_hi", C.c_double),
                ("clip_threshold", C.c_double), ("sparse_threshold", C.c_double),
                ("use_gc", C.c_int32), ("adaptive_beta", C.c_int32),
                ("beta_tau1", C.c_double), ("beta_tau2", C.c_double), ("n_taylor", C.c_int64),
                ("moment_dtype", C.c_int32), ("device_step", C.c_int32)]


class novak_tensor_desc(C.Structure):
    _fields_ = [("param", C.c_void_p), ("exp_avg", C.c_void_p), ("exp_avg_sq", C.c_void_p),
                ("la_buf", C.c_void_p), ("numel", C.c_int64), ("rows", C.c_int64)]


class novak_step_scalars(C.Structure):
    _fields_ = [("bc1", C.c_double), ("bc2", C.c_double), ("rho_inf", C.c_double), ("rho_t", C.c_double),
                ("r_t", C.c_double), ("step_size", C.c_double), ("decay", C.c_double),
                ("rectified_now", C.c_int32), ("denom_on", C.c_int32),
                ("beta1_t", C.c_double), ("beta2_t", C.c_double), ("nesterov_mode", C.c_int32), ("reserved0", C.c_int32)]


class novak_chunk(C.Structure):
    _fields_ = [("offset", C.c_int64), ("tensor", C.c_int32), ("len", C.c_int32)]


class novak_info(C.Structure):
    _fields_ = [("struct_size", C.c_size_t), ("nesterov_mode", C.c_int32), ("lookahead_mode", C.c_int32),
                ("warnings", C.c_uint32), ("n_tensors", C.c_int32), ("n_chunks", C.c_int64),
                ("chunk_elems", C.c_int64), ("total_numel", C.c_int64), ("last_step", C.c_int64),
                ("sync_due", C.c_int32), ("device_id", C.c_int32),
                ("layer_adaptation", C.c_int32), ("auto_lr", C.c_int32), ("use_gc", C.c_int32),
                ("n_centralized", C.c_int32), ("moment_dtype", C.c_int32), ("reserved0", C.c_int32)]


EXPORTS = ("novak_validate_hparams", "novak_compute_step_scalars", "novak_plan_chunks", "novak_plan_arena",
           "novak_arena_alloc", "novak_arena_free",
           "novak_bytes_per_param_step", "novak_bytes_per_param_scaled_step", "novak_bytes_per_param_clip",
           "novak_bytes_per_param_moment_saving", "novak_bytes_per_param_sync",
           "novak_status_string", "novak_create", "novak_lookahead_init", "novak_step", "novak_lookahead_sync",
           "novak_destroy", "novak_get_info", "novak_set_tuning", "novak_last_error", "novak_set_auto_lr_state",
           "novak_copy_tensor_scales", "novak_nesterov_extrapolate", "novak_step_static",
           "novak_torch_malloc", "novak_torch_free", "novak_torch_alloc_stats", "novak_set_step_counter")

_lib: Optional[C.CDLL] = None


def load_library() -> C.CDLL:
    """Loads libnovak.so (built in-tree by paper_2601_07876_amd.build).  Raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2601_07876_amd.build`; "
                           "there is no fallback path")
    import torch  # noqa: F401  (loads the HIP runtime this library must share)
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.novak_validate_hparams.argtypes = [C.POINTER(novak_hparams), C.POINTER(novak_hparams), C.POINTER(C.c_uint32)]
    lib.novak_compute_step_scalars.argtypes = [C.POINTER(novak_hparams), i64, C.POINTER(novak_step_scalars)]
    lib.novak_plan_chunks.argtypes = [C.POINTER(i64), i32, i64, C.POINTER(novak_chunk), i64, C.POINTER(i64)]
    lib.novak_plan_arena.argtypes = [C.POINTER(i64), i32, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
    lib.novak_arena_alloc.argtypes = [i32, C.c_size_t, C.POINTER(C.c_void_p), C.POINTER(i32)]
    lib.novak_arena_free.argtypes = [i32, C.c_void_p]
    lib.novak_torch_malloc.argtypes = [C.c_ssize_t, C.c_int, vp]
    lib.novak_torch_malloc.restype = vp
    lib.novak_torch_free.argtypes = [vp, C.c_ssize_t, C.c_int, vp]
    lib.novak_torch_free.restype = None
    lib.novak_torch_alloc_stats.argtypes = [C.POINTER(i64), C.POINTER(i64)]
    lib.novak_torch_alloc_stats.restype = None
    lib.novak_bytes_per_param_step.argtypes = [i32, i32, i32, i32, i32]
    lib.novak_bytes_per_param_step.restype = C.c_double
    lib.novak_bytes_per_param_scaled_step.argtypes = [i32, i32, i32, i32, i32]
    lib.novak_bytes_per_param_scaled_step.restype = C.c_double
    lib.novak_set_auto_lr_state.argtypes = [vp, vp]
    lib.novak_set_step_counter.argtypes = [vp, vp]
    lib.novak_copy_tensor_scales.argtypes = [vp, C.POINTER(C.c_float), vp]
    lib.novak_nesterov_extrapolate.argtypes = [vp, C.POINTER(vp), vp]
    lib.novak_bytes_per_param_moment_saving.argtypes = [i32, i32]
    lib.novak_bytes_per_param_moment_saving.restype = C.c_double
    lib.novak_bytes_per_param_clip.argtypes = [i32]
    lib.novak_bytes_per_param_clip.restype = C.c_double
    lib.novak_bytes_per_param_sync.argtypes = [i32]
    lib.novak_bytes_per_param_sync.restype = C.c_double
    lib.novak_status_string.argtypes = [C.c_int]
    lib.novak_status_string.restype = C.c_char_p
    lib.novak_create.argtypes = [C.POINTER(vp), C.POINTER(novak_hparams), C.POINTER(novak_tensor_desc), i32, i32]
    lib.novak_lookahead_init.argtypes = [vp, vp]
    lib.novak_step.argtypes = [vp, C.POINTER(vp), i32, i64, vp]
    lib.novak_lookahead_sync.argtypes = [vp, vp]
    lib.novak_step_static.argtypes = [C.POINTER(novak_hparams), C.POINTER(novak_tensor_desc), i32, C.POINTER(vp), i32, i64, i32, vp]
    lib.novak_destroy.argtypes = [vp]
    lib.novak_get_info.argtypes = [vp, C.POINTER(novak_info)]
    lib.novak_set_tuning.argtypes = [vp, i32, i64]
    lib.novak_last_error.argtypes = [vp]
    lib.novak_last_error.restype = C.c_char_p
    for name in EXPORTS:
        fn = getattr(lib, name)
        if fn.restype is C.c_int:
            fn.restype = C.c_int
    _lib = lib
    return lib


class NovakError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        msg = f"{where}: status {status} ({novak_status_string(status)})"
        super().__init__(msg + (f": {detail}" if detail else ""))


def make_hparams(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, beta_n=0.9, la_alpha=0.5, la_k=5,
                 rectified=True, decoupled_decay=True, nesterov="approx", lookahead="memory_efficient",
                 unrect_fallback="adam_denom", mode="fast", auto_sync=False, layer_adaptation=False, auto_lr=False,
                 auto_lr_gamma=0.1, trust_clip=(0.1, 10.0), auto_clip=(0.1, 2.0), clip_threshold=0.0,
                 sparse_threshold=0.0, use_gc=False, adaptive_beta=False, beta_tau1=1000.0, beta_tau2=5000.0,
                 n_taylor=0, moment_dtype="f32", device_step=False) -> novak_hparams:
    """Fills a novak_hparams from keyword values (mode names or their integer codes)."""
    def code(table: Dict[str, int], x):
        return table[x] if isinstance(x, str) else int(x)
    return novak_hparams(C.sizeof(novak_hparams), lr, beta1, beta2, eps, weight_decay, beta_n, la_alpha, int(la_k),
                         int(rectified), int(decoupled_decay), code(NESTEROV, nesterov), code(LOOKAHEAD, lookahead),
                         code(UNRECT, unrect_fallback), code(MODE, mode), int(auto_sync), int(layer_adaptation),
                         int(auto_lr), float(auto_lr_gamma), float(trust_clip[0]), float(trust_clip[1]),
                         float(auto_clip[0]), float(auto_clip[1]), float(clip_threshold), float(sparse_threshold),
                         int(use_gc), int(adaptive_beta), float(beta_tau1), float(beta_tau2), int(n_taylor),
                         code(MOMENT_DTYPE, moment_dtype), int(device_step))


# ---- the entry points, same names as the C ABI ------------------------------------------------------
def novak_status_string(status: int) -> str:
    return load_library().novak_status_string(int(status)).decode()


def novak_validate_hparams(hp: novak_hparams):
    """-> (status, effective hparams, warning bits)."""
    eff, warn = novak_hparams(), C.c_uint32(0)
    rc = load_library().novak_validate_hparams(C.byref(hp), C.byref(eff), C.byref(warn))
    return rc, eff, warn.value


def novak_compute_step_scalars(hp: novak_hparams, step: int):
    out = novak_step_scalars()
    rc = load_library().novak_compute_step_scalars(C.byref(hp), int(step), C.byref(out))
    return rc, out


def novak_plan_chunks(numels: Sequence[int], chunk_elems: int):
    """-> (status, list of (tensor, offset, len))."""
    lib = load_library()
    n = len(numels)
    arr = (C.c_int64 * max(n, 1))(*numels)
    count = C.c_int64(0)
    rc = lib.novak_plan_chunks(arr, n, int(chunk_elems), None, 0, C.byref(count))
    if rc != NOVAK_OK:
        return rc, []
    out = (novak_chunk * max(count.value, 1))()
    rc = lib.novak_plan_chunks(arr, n, int(chunk_elems), out, count.value, C.byref(count))
    return rc, [(out[i].tensor, out[i].offset, out[i].len) for i in range(count.value)]


def novak_plan_arena(numels: Sequence[int]):
    """-> (status, tensor offsets in elements, padded elements per role, bytes between consecutive roles)."""
    n = len(numels)
    arr = (C.c_int64 * max(n, 1))(*numels)
    offs = (C.c_int64 * max(n, 1))()
    role_elems, stride = C.c_int64(0), C.c_int64(0)
    rc = load_library().novak_plan_arena(arr, n, offs, C.byref(role_elems), C.byref(stride))
    return rc, [offs[i] for i in range(n)], role_elems.value, stride.value


def novak_arena_alloc(device_id: int, nbytes: int):
    """-> (status, device pointer as int or None, 1 if physically contiguous else 0)."""
    ptr, contiguous = C.c_void_p(), C.c_int32(0)
    rc = load_library().novak_arena_alloc(device_id, nbytes, C.byref(ptr), C.byref(contiguous))
    return rc, ptr.value, contiguous.value


def novak_arena_free(device_id: int, ptr) -> int:
    return load_library().novak_arena_free(device_id, ptr)


def novak_torch_alloc_stats():
    """-> (allocations alive that were made through novak_torch_malloc, how many of them are physically contiguous)."""
    live, contig = C.c_int64(0), C.c_int64(0)
    load_library().novak_torch_alloc_stats(C.byref(live), C.byref(contig))
    return live.value, contig.value


_torch_pool_allocator = None


def torch_mem_pool():
    """A torch.cuda.MemPool whose segments come from novak_torch_malloc (argument marshalling only: the pool and
    the caching on top of it are torch's).  Use as `with torch.cuda.use_mem_pool(pool): ...allocate...`; keep the
    pool alive as long as its tensors."""
    global _torch_pool_allocator
    import torch
    load_library()
    if _torch_pool_allocator is None:      # one allocator object per process: torch keeps function pointers into it
        _torch_pool_allocator = torch.cuda.memory.CUDAPluggableAllocator(LIB_PATH, "novak_torch_malloc", "novak_torch_free")
    return torch.cuda.MemPool(_torch_pool_allocator.allocator())


class _DeviceBytes:
    """Exposes raw device memory to torch through the array-interface protocol (no copy, no ownership)."""

    def __init__(self, ptr: int, nbytes: int):
        self.__cuda_array_interface__ = {"shape": (nbytes,), "typestr": "|u1", "data": (ptr, False), "version": 2}


def arena_as_tensor(ptr: int, nbytes: int, device_id: int = 0):
    """A uint8 torch tensor over memory from novak_arena_alloc.  The tensor does not own the memory: keep
    it (and every view of it) no longer than until novak_arena_free."""
    import torch
    return torch.as_tensor(_DeviceBytes(ptr, nbytes), device=torch.device("cuda", device_id))


def novak_bytes_per_param_step(lookahead_mode: int, grad_dtype: int, la_k: int, window_pos: int, fused_sync: int) -> float:
    return load_library().novak_bytes_per_param_step(lookahead_mode, grad_dtype, la_k, window_pos, fused_sync)


def novak_bytes_per_param_scaled_step(lookahead_mode: int, grad_dtype: int, la_k: int, window_pos: int, fused_sync: int) -> float:
    return load_library().novak_bytes_per_param_scaled_step(lookahead_mode, grad_dtype, la_k, window_pos, fused_sync)


def novak_set_auto_lr_state(handle, ema_ptr: int) -> int:
    return load_library().novak_set_auto_lr_state(handle, C.c_void_p(ema_ptr))


def novak_set_step_counter(handle, counter_ptr: int) -> int:
    return load_library().novak_set_step_counter(handle, C.c_void_p(counter_ptr))


def novak_copy_tensor_scales(handle, n_tensors: int, stream: int = 0):
    """-> (status, list of n_tensors floats)."""
    buf = (C.c_float * max(n_tensors, 1))()
    rc = load_library().novak_copy_tensor_scales(handle, buf, C.c_void_p(stream))
    return rc, [buf[i] for i in range(n_tensors)]


def novak_nesterov_extrapolate(handle, out_ptrs, stream: int = 0) -> int:
    """`out_ptrs`: a ctypes c_void_p array or a sequence of device addresses, one per tensor."""
    if not isinstance(out_ptrs, C.Array):
        out_ptrs = (C.c_void_p * max(len(out_ptrs), 1))(*out_ptrs)
    return load_library().novak_nesterov_extrapolate(handle, out_ptrs, C.c_void_p(stream))


def novak_bytes_per_param_moment_saving(moment_dtype: int, two_pass: int) -> float:
    return load_library().novak_bytes_per_param_moment_saving(moment_dtype, two_pass)


def novak_bytes_per_param_clip(grad_dtype: int) -> float:
    return load_library().novak_bytes_per_param_clip(grad_dtype)


def novak_bytes_per_param_sync(lookahead_mode: int) -> float:
    return load_library().novak_bytes_per_param_sync(lookahead_mode)


def novak_create(hp: novak_hparams, descs: Sequence[novak_tensor_desc], device_id: int = 0):
    """-> (status, handle).  `descs` hold raw device pointers (e.g. tensor.data_ptr())."""
    lib = load_library()
    n = len(descs)
    arr = (novak_tensor_desc * max(n, 1))(*descs)
    handle = C.c_void_p(None)
    rc = lib.novak_create(C.byref(handle), C.byref(hp), arr, n, int(device_id))
    return rc, (handle if rc == NOVAK_OK else None)


def novak_lookahead_init(handle, stream: int = 0) -> int:
    return load_library().novak_lookahead_init(handle, C.c_void_p(stream))


def novak_step(handle, grad_ptrs, grad_dtype: int, step: int, stream: int = 0) -> int:
    """`grad_ptrs`: a ctypes c_void_p array (reused by the caller) or a sequence of device addresses."""
    if not isinstance(grad_ptrs, C.Array):
        grad_ptrs = (C.c_void_p * max(len(grad_ptrs), 1))(*grad_ptrs)
    return load_library().novak_step(handle, grad_ptrs, int(grad_dtype), int(step), C.c_void_p(stream))


def novak_step_static(hp: novak_hparams, descs: Sequence[novak_tensor_desc], grad_ptrs, grad_dtype: int, step: int,
                      device_id: int = 0, stream: int = 0) -> int:
    """One handle-free, allocation-free step (see include/novak.h)."""
    n = len(descs)
    arr = descs if isinstance(descs, C.Array) else (novak_tensor_desc * max(n, 1))(*descs)
    if not isinstance(grad_ptrs, C.Array):
        grad_ptrs = (C.c_void_p * max(len(grad_ptrs), 1))(*grad_ptrs)
    return load_library().novak_step_static(C.byref(hp), arr, n, grad_ptrs, int(grad_dtype), int(step), int(device_id),
                                            C.c_void_p(stream))


def novak_lookahead_sync(handle, stream: int = 0) -> int:
    return load_library().novak_lookahead_sync(handle, C.c_void_p(stream))


def novak_destroy(handle) -> int:
    return load_library().novak_destroy(handle)


def novak_get_info(handle):
    info = novak_info(struct_size=C.sizeof(novak_info))
    rc = load_library().novak_get_info(handle, C.byref(info))
    return rc, info


def novak_set_tuning(handle, key: int, value: int) -> int:
    return load_library().novak_set_tuning(handle, int(key), int(value))


def novak_last_error(handle=None) -> str:
    return load_library().novak_last_error(handle).decode()


# ---- convenience: marshal torch tensors into descriptors -------------------------------------------
def tensor_desc(param, exp_avg, exp_avg_sq, la_buf=None) -> novak_tensor_desc:
    """Descriptor from contiguous fp32 torch tensors that live on the GPU; `rows` (Eq. 26) is the size of
    the parameter's first dimension when it has more than one."""
    for t in (param, exp_avg, exp_avg_sq) + ((la_buf,) if la_buf is not None else ()):
        ok_dtype = str(t.dtype) == "torch.float32" or (t is exp_avg and str(t.dtype) == "torch.bfloat16")
        if not t.is_contiguous() or not ok_dtype or not t.is_cuda:
            raise ValueError("state tensors must be contiguous fp32 GPU tensors (exp_avg may be bfloat16)")
        if t.numel() != param.numel():
            raise ValueError("state tensors must have the parameter's element count")
    return novak_tensor_desc(param.data_ptr(), exp_avg.data_ptr(), exp_avg_sq.data_ptr(),
                             la_buf.data_ptr() if la_buf is not None else None, param.numel(),
                             param.shape[0] if param.dim() > 1 else 0)


def check(rc: int, where: str, handle=None) -> None:
    if rc != NOVAK_OK:
        raise NovakError(rc, where, novak_last_error(handle))
