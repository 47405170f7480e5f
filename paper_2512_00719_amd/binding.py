"""ctypes binding of libsimple_sample.so: argument marshalling only.

The functions carry the names of the C boundary (``include/simple_sample.h``).  Every step of
the sampling path runs in the HIP kernels of the library; PyTorch is used by callers for device
memory and streams only.  If the shared library is missing the import of this module fails --
there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np
import torch  # noqa: F401  imported first so that the library binds to the HIP runtime PyTorch loads

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsimple_sample.so")

SIMPLE_F32, SIMPLE_BF16 = 0, 1
SIMPLE_OK, SIMPLE_EINVAL, SIMPLE_ENOMEM, SIMPLE_EDEVICE, SIMPLE_ECAPACITY = 0, -1, -2, -3, -4

DIAG_ERROR, DIAG_GREEDY, DIAG_WIDE, DIAG_SHVS, DIAG_ACCEPTED, DIAG_CAREFUL, DIAG_REPLAY, DIAG_GENERAL = (
    1 << i for i in range(8))
DIAG_BAD_PARAM, DIAG_BAD_LOGIT, DIAG_BAD_HISTORY_ID, DIAG_HISTORY_TOO_LONG, DIAG_BAD_HOT_SET, DIAG_PATTERN = (
    1 << i for i in range(8, 14))

ROW_DIAG_DTYPE = np.dtype([("alpha", "<f8"), ("s_k", "<f8"), ("p_chosen", "<f4"),
                           ("n_survivors", "<i4"), ("flags", "<u4"), ("reserved", "<u4")])
assert ROW_DIAG_DTYPE.itemsize == 32

STATS_DTYPE = np.dtype([("rows", "<u8"), ("greedy_rows", "<u8"), ("shvs_accepted", "<u8"), ("shvs_rejected", "<u8"),
                        ("second_pass_rows", "<u8"), ("general_rows", "<u8"), ("sum_alpha_q32", "<u8"),
                        ("error_flags", "<u4"), ("reserved", "<u4")])
assert STATS_DTYPE.itemsize == 64

EXPORTS = ("simple_create", "simple_destroy", "simple_set_hot_set", "simple_set_stats", "simple_set_decision_outputs", "simple_sample",
           "simple_sample_static", "simple_static_limit",
           "simple_apply_logit_constraints", "simple_sample_hot_first",
           "simple_state_create", "simple_state_destroy", "simple_state_restart", "simple_state_append", "simple_sample_state",
           "simple_profile_enable", "simple_profile_read", "simple_profile_read_launches",
           "simple_stream_probe",
           "simple_lds_bytes", "simple_strerror", "simple_version")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2512_00719_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, u64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64
    lib.simple_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64, i64, i64]
    lib.simple_create.restype = ctypes.c_int
    lib.simple_destroy.argtypes = [vp]
    lib.simple_destroy.restype = None
    lib.simple_set_hot_set.argtypes = [vp, vp, i32, i64, vp]
    lib.simple_set_hot_set.restype = ctypes.c_int
    lib.simple_set_decision_outputs.argtypes = [vp, vp, vp, ctypes.POINTER(ctypes.c_int32), ctypes.c_int]
    lib.simple_set_decision_outputs.restype = ctypes.c_int
    lib.simple_set_stats.argtypes = [vp, vp]
    lib.simple_set_stats.restype = ctypes.c_int
    lib.simple_sample.argtypes = [vp, vp, i64, i64, ctypes.c_int, i64, vp, vp, vp, vp, i32, u64, u64, u64,
                                  vp, vp, vp]
    lib.simple_sample.restype = ctypes.c_int
    lib.simple_sample_static.argtypes = [vp, i64, i64, ctypes.c_int, i64, vp, vp, vp, vp, i32, u64, u64, u64, vp, vp, vp]
    lib.simple_sample_static.restype = ctypes.c_int
    lib.simple_static_limit.argtypes = [ctypes.c_int]
    lib.simple_static_limit.restype = i64
    lib.simple_sample_hot_first.argtypes = [vp, vp, i64, i64, ctypes.c_int, i64, vp, i32, vp, u64, u64, u64, vp, vp, vp]
    lib.simple_sample_hot_first.restype = ctypes.c_int
    lib.simple_apply_logit_constraints.argtypes = [vp, i64, i64, ctypes.c_int, i64, vp, vp, vp, vp, vp, vp, i64, vp]
    lib.simple_apply_logit_constraints.restype = ctypes.c_int
    lib.simple_state_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64, i64, i64]
    lib.simple_state_create.restype = ctypes.c_int
    lib.simple_state_destroy.argtypes = [vp]
    lib.simple_state_destroy.restype = None
    lib.simple_state_restart.argtypes = [vp, vp, i64, vp, vp, vp, vp]
    lib.simple_state_restart.restype = ctypes.c_int
    lib.simple_state_append.argtypes = [vp, vp, vp, i64, vp]
    lib.simple_state_append.restype = ctypes.c_int
    lib.simple_sample_state.argtypes = [vp, vp, vp, vp, i64, i64, ctypes.c_int, i64, vp, vp, i32, u64, u64, u64, vp, vp, vp]
    lib.simple_sample_state.restype = ctypes.c_int
    lib.simple_profile_enable.argtypes = [vp, ctypes.c_int]
    lib.simple_profile_enable.restype = ctypes.c_int
    lib.simple_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_double)]
    lib.simple_profile_read.restype = ctypes.c_int
    lib.simple_profile_read_launches.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.c_int,
                                                 ctypes.POINTER(ctypes.c_double)]
    lib.simple_profile_read_launches.restype = ctypes.c_int
    lib.simple_stream_probe.argtypes = [vp, i64, i64, ctypes.c_int, i64, vp, vp]
    lib.simple_stream_probe.restype = ctypes.c_int
    lib.simple_lds_bytes.argtypes = [vp]
    lib.simple_lds_bytes.restype = i64
    lib.simple_strerror.argtypes = [ctypes.c_int]
    lib.simple_strerror.restype = ctypes.c_char_p
    lib.simple_version.argtypes = []
    lib.simple_version.restype = ctypes.c_int
    return lib


_lib = _load()


class SimpleError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where}: {simple_strerror(code)} ({code})")
        self.code = code


def simple_version() -> int:
    return int(_lib.simple_version())


def simple_strerror(code: int) -> str:
    return _lib.simple_strerror(int(code)).decode()


def simple_create(device: int, max_B: int, max_V: int, max_nnz_per_row: int) -> int:
    """Returns the context handle (an integer address); raises SimpleError on failure."""
    h = ctypes.c_void_p()
    rc = _lib.simple_create(ctypes.byref(h), int(device), int(max_B), int(max_V), int(max_nnz_per_row))
    if rc != SIMPLE_OK:
        raise SimpleError(rc, "simple_create")
    return h.value


def simple_destroy(ctx: Optional[int]) -> None:
    _lib.simple_destroy(ctypes.c_void_p(ctx))


def simple_lds_bytes(ctx: int) -> int:
    return int(_lib.simple_lds_bytes(ctypes.c_void_p(ctx)))


def simple_profile_enable(ctx: int, on: bool) -> int:
    return int(_lib.simple_profile_enable(ctypes.c_void_p(ctx), 1 if on else 0))


def simple_profile_read(ctx: int) -> tuple[int, float]:
    """Returns (recorded launches, sum of their durations in ms) of the dominant kernel."""
    total = ctypes.c_double(0.0)
    n = int(_lib.simple_profile_read(ctypes.c_void_p(ctx), ctypes.byref(total)))
    if n < 0:
        raise SimpleError(n, "simple_profile_read")
    return n, float(total.value)


def simple_profile_read_launches(ctx: int, cap: int = 1024) -> np.ndarray:
    """Durations in ms of the recorded launches of the dominant kernel, in launch order."""
    buf = (ctypes.c_float * max(cap, 1))()
    total = ctypes.c_double(0.0)
    n = int(_lib.simple_profile_read_launches(ctypes.c_void_p(ctx), buf, int(cap), ctypes.byref(total)))
    if n < 0:
        raise SimpleError(n, "simple_profile_read_launches")
    return np.frombuffer(buf, dtype=np.float32, count=min(n, cap)).copy()


def simple_stream_probe(logits_ptr: int, B: int, V: int, dtype: int, row_stride: int, row_max_ptr: int,
                        stream: int = 0) -> int:
    """Raw call: row maxima by a read-only streaming reduction.  Returns the C status code."""
    vp = ctypes.c_void_p
    return int(_lib.simple_stream_probe(vp(logits_ptr), int(B), int(V), int(dtype), int(row_stride),
                                        vp(row_max_ptr), vp(stream)))


def simple_set_hot_set(ctx: int, hot_ids_ptr: int, H: int, V: int, stream: int = 0) -> int:
    return int(_lib.simple_set_hot_set(ctypes.c_void_p(ctx), ctypes.c_void_p(hot_ids_ptr), int(H), int(V),
                                       ctypes.c_void_p(stream)))


def simple_set_decision_outputs(ctx: int, logprobs_ptr: int, eos_ptr: int, eos_ids=()) -> int:
    """Install per-row log-probability (float32) and EOS-flag (uint8) outputs; eos_ids: up to 8 token ids."""
    ids = (ctypes.c_int32 * max(len(eos_ids), 1))(*[int(x) for x in eos_ids])
    return int(_lib.simple_set_decision_outputs(ctypes.c_void_p(ctx), ctypes.c_void_p(logprobs_ptr), ctypes.c_void_p(eos_ptr), ids,
                                                len(eos_ids)))


def simple_set_stats(ctx: int, stats_ptr: int) -> int:
    return int(_lib.simple_set_stats(ctypes.c_void_p(ctx), ctypes.c_void_p(stats_ptr)))


def simple_sample(ctx: int, logits_ptr: int, B: int, V: int, dtype: int, row_stride: int, params_ptr: int,
                  hist_ptr_ptr: int, hist_ids_ptr: int, hot_ids_ptr: int, H: int, seed: int, step: int,
                  row_offset: int, out_ids_ptr: int, diag_ptr: int, stream: int = 0) -> int:
    """Raw call: every *_ptr is a device address (0 for NULL).  Returns the C status code."""
    vp = ctypes.c_void_p
    return int(_lib.simple_sample(vp(ctx), vp(logits_ptr), int(B), int(V), int(dtype), int(row_stride),
                                  vp(params_ptr), vp(hist_ptr_ptr), vp(hist_ids_ptr), vp(hot_ids_ptr), int(H),
                                  ctypes.c_uint64(seed & (2 ** 64 - 1)), ctypes.c_uint64(step & (2 ** 64 - 1)),
                                  ctypes.c_uint64(row_offset & (2 ** 64 - 1)), vp(out_ids_ptr), vp(diag_ptr),
                                  vp(stream)))


def simple_sample_static(logits_ptr: int, B: int, V: int, dtype: int, row_stride: int, params_ptr: int,
                         hist_ptr_ptr: int, hist_ids_ptr: int, hot_ids_ptr: int, H: int, seed: int, step: int,
                         row_offset: int, out_ids_ptr: int, diag_ptr: int, stream: int = 0) -> int:
    """Raw call of the entry point that allocates nothing (no context).  Returns the C status code."""
    vp = ctypes.c_void_p
    return int(_lib.simple_sample_static(vp(logits_ptr), int(B), int(V), int(dtype), int(row_stride),
                                         vp(params_ptr), vp(hist_ptr_ptr), vp(hist_ids_ptr), vp(hot_ids_ptr), int(H),
                                         ctypes.c_uint64(seed & (2 ** 64 - 1)), ctypes.c_uint64(step & (2 ** 64 - 1)),
                                         ctypes.c_uint64(row_offset & (2 ** 64 - 1)), vp(out_ids_ptr), vp(diag_ptr),
                                         vp(stream)))


def simple_static_limit(what: int) -> int:
    return int(_lib.simple_static_limit(int(what)))


TAIL_STATS_DTYPE = np.dtype([("tail_sum", "<f8"), ("tail_max", "<f4"), ("reserved", "<f4")])
assert TAIL_STATS_DTYPE.itemsize == 16


def simple_sample_hot_first(ctx: int, logits_ptr: int, B: int, V: int, dtype: int, row_stride: int, params_ptr: int, H: int,
                            tail_stats_ptr: int, seed: int, step: int, row_offset: int, out_ids_ptr: int, diag_ptr: int,
                            stream: int = 0) -> int:
    """Raw call: SHVS on a hot-first vocabulary with per-row tail statistics.  Returns the C status code."""
    vp = ctypes.c_void_p
    return int(_lib.simple_sample_hot_first(vp(ctx), vp(logits_ptr), int(B), int(V), int(dtype), int(row_stride), vp(params_ptr), int(H),
                                            vp(tail_stats_ptr), ctypes.c_uint64(seed & (2 ** 64 - 1)),
                                            ctypes.c_uint64(step & (2 ** 64 - 1)), ctypes.c_uint64(row_offset & (2 ** 64 - 1)),
                                            vp(out_ids_ptr), vp(diag_ptr), vp(stream)))


def simple_apply_logit_constraints(logits_ptr: int, B: int, V: int, dtype: int, row_stride: int, bias_ptr_ptr: int, bias_ids_ptr: int,
                                   bias_vals_ptr: int, allow_ptr_ptr: int, allow_ids_ptr: int, out_ptr: int, out_stride: int,
                                   stream: int = 0) -> int:
    """Raw call: logit bias and allow-lists written out as a float32 matrix.  Returns the C status code."""
    vp = ctypes.c_void_p
    return int(_lib.simple_apply_logit_constraints(vp(logits_ptr), int(B), int(V), int(dtype), int(row_stride), vp(bias_ptr_ptr),
                                                   vp(bias_ids_ptr), vp(bias_vals_ptr), vp(allow_ptr_ptr), vp(allow_ids_ptr),
                                                   vp(out_ptr), int(out_stride), vp(stream)))


def simple_state_create(device: int, max_seqs: int, V: int, L_max: int) -> int:
    """Returns the state handle (an integer address); raises SimpleError on failure."""
    h = ctypes.c_void_p()
    rc = _lib.simple_state_create(ctypes.byref(h), int(device), int(max_seqs), int(V), int(L_max))
    if rc != SIMPLE_OK:
        raise SimpleError(rc, "simple_state_create")
    return h.value


def simple_state_destroy(state: Optional[int]) -> None:
    _lib.simple_state_destroy(ctypes.c_void_p(state))


def simple_state_restart(state: int, slots_ptr: int, n: int, prompt_ptr_ptr: int, prompt_ids_ptr: int, n_prompt_ptr: int = 0,
                         stream: int = 0) -> int:
    vp = ctypes.c_void_p
    return int(_lib.simple_state_restart(vp(state), vp(slots_ptr), int(n), vp(prompt_ptr_ptr), vp(prompt_ids_ptr), vp(n_prompt_ptr),
                                         vp(stream)))


def simple_state_append(state: int, slots_ptr: int, new_ids_ptr: int, B: int, stream: int = 0) -> int:
    vp = ctypes.c_void_p
    return int(_lib.simple_state_append(vp(state), vp(slots_ptr), vp(new_ids_ptr), int(B), vp(stream)))


def simple_sample_state(ctx: int, state: int, slots_ptr: int, logits_ptr: int, B: int, V: int, dtype: int, row_stride: int,
                        params_ptr: int, hot_ids_ptr: int, H: int, seed: int, step: int, row_offset: int,
                        out_ids_ptr: int, diag_ptr: int, stream: int = 0) -> int:
    """Raw call: the sampling call with the rows' histories taken from a state.  Returns the C status code."""
    vp = ctypes.c_void_p
    return int(_lib.simple_sample_state(vp(ctx), vp(state), vp(slots_ptr), vp(logits_ptr), int(B), int(V), int(dtype),
                                        int(row_stride), vp(params_ptr), vp(hot_ids_ptr), int(H),
                                        ctypes.c_uint64(seed & (2 ** 64 - 1)), ctypes.c_uint64(step & (2 ** 64 - 1)),
                                        ctypes.c_uint64(row_offset & (2 ** 64 - 1)), vp(out_ids_ptr), vp(diag_ptr), vp(stream)))


class Sampler:
    """Convenience wrapper over torch device tensors (marshalling only)."""

    def __init__(self, max_V: int, max_nnz_per_row: int, device: int = 0, max_B: int = 4096):
        self.ctx = simple_create(device, max_B, max_V, max_nnz_per_row)
        self.device = device

    def close(self) -> None:
        if self.ctx:
            simple_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_hot_set(self, hot_ids, V: int) -> None:
        import torch
        rc = simple_set_hot_set(self.ctx, hot_ids.data_ptr(), hot_ids.numel(), V,
                                torch.cuda.current_stream().cuda_stream)
        if rc != SIMPLE_OK:
            raise SimpleError(rc, "simple_set_hot_set")

    def sample(self, logits, params, hist_ptr=None, hist_ids=None, hot_ids=None, H: int = 0, *, seed: int,
               step: int, row_offset: int = 0, out=None, diag=None, V: Optional[int] = None):
        """logits: [B, stride] float32 or bfloat16/uint16/int16 device tensor; params: uint8 view of
        [B] 32-byte records; hist_ptr int64 [B+1]; hist_ids int32; hot_ids int32 or None (H=-1 uses the
        installed set).  Returns ``out`` (int32 [B]); enqueued on the current stream, not synchronised."""
        import torch
        B = logits.shape[0]
        V = int(V if V is not None else logits.shape[1])
        dtype = SIMPLE_F32 if logits.dtype == torch.float32 else SIMPLE_BF16
        if out is None:
            out = torch.empty(B, dtype=torch.int32, device=logits.device)
        if hot_ids is not None:
            H = hot_ids.numel()
        rc = simple_sample(self.ctx, logits.data_ptr(), B, V, dtype, logits.stride(0) if B else V,
                           params.data_ptr(), 0 if hist_ptr is None else hist_ptr.data_ptr(),
                           0 if hist_ids is None else hist_ids.data_ptr(),
                           0 if hot_ids is None else hot_ids.data_ptr(), H, seed, step, row_offset,
                           out.data_ptr(), 0 if diag is None else diag.data_ptr(),
                           torch.cuda.current_stream().cuda_stream)
        if rc != SIMPLE_OK:
            raise SimpleError(rc, "simple_sample")
        return out
