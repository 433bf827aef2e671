"""ctypes binding of libdba (include/dba.h): same names, argument marshalling only.

Device buffers are passed as integer addresses (e.g. torch.Tensor.data_ptr());
host arrays as contiguous numpy arrays.  Nothing of the method runs here: if the
built library is missing this module raises, it never falls back to anything.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdba.so")

DBA_OK, DBA_EINVAL, DBA_ESTATE, DBA_EHIP, DBA_ENOMEM = 0, -1, -2, -3, -4
DBA_FLAG_FINISHED, DBA_FLAG_DEAD = 1, 2
DBA_MAX_BEAM, DBA_MAX_CONS_TOKENS = 64, 64
DBA_NOALLOC_MAX_ROWS = 8192
DBA_LOGP_F32, DBA_LOGP_F16, DBA_LOGP_BF16 = 0, 1, 2
DBA_STOP_ALL, DBA_STOP_ANY = 1, 2
DBA_OPT_ADJUSTMENT, DBA_OPT_NORMALIZE_FINISHED, DBA_OPT_PRUNE_THRESHOLD = 2, 3, 4
DBA_OPT_TRACK_COMPLETED = 5
DBA_OPT_MERGE_WAVES = 6

_P = ctypes.c_void_p
_I = ctypes.c_int

_SIGNATURES = {
    "dba_workspace_bytes": (ctypes.c_size_t, [_I] * 5),
    "dba_init": (_I, [_P] + [_I] * 6 + [_P] * 4 + [ctypes.c_size_t, _P]),
    "dba_step": (_I, [_P] * 6),
    "dba_step_fmt": (_I, [_P, _P, _I] + [_P] * 4),
    "dba_step_noalloc": (_I, [_P, _P, _I] + [_P] * 4),
    "dba_finalize": (_I, [_P] * 5),
    "dba_get_state": (_I, [_P] * 7),
    "dba_steps_done": (_I, [_P]),
    "dba_set_option": (_I, [_P, _I, ctypes.c_double]),
    "dba_get_finished": (_I, [_P, _P]),
    "dba_destroy": (None, [_P]),
    "dba_last_error": (ctypes.c_char_p, [_P]),
    "dba_debug_allocate": (_I, [_I, _I] + [_P] * 5 + [ctypes.c_size_t, _P]),
    "dba_debug_wave_select": (_I, [_I] + [_P] * 5 + [ctypes.c_size_t, _P]),
    "dba_debug_row_max": (_I, [_P, _I, _I, _P, _P]),
}

_lib = None


class DbaError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libdba error {code}: {text}")
        self.code = code


def load() -> ctypes.CDLL:
    """Loads the built library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1804_06609_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _host(a: Optional[np.ndarray], dtype) -> Optional[int]:
    if a is None:
        return None
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags.c_contiguous
    return a.ctypes.data


def _check(rc: int, ctx=None):
    if rc != DBA_OK:
        raise DbaError(rc, dba_last_error(ctx))
    return rc


def dba_last_error(ctx=None) -> str:
    return load().dba_last_error(ctx).decode()


def dba_workspace_bytes(B: int, k: int, V: int, N: int, max_cons_tokens: int) -> int:
    return int(load().dba_workspace_bytes(B, k, V, N, max_cons_tokens))


def dba_init(B: int, k: int, V: int, N: int, eos_id: int, pad_id: int, cons_tokens: np.ndarray,
             phrase_offsets: np.ndarray, sent_offsets: np.ndarray, workspace_dev: int,
             workspace_bytes: int, hip_stream: int = 0):
    """Returns the ctx handle (an integer address)."""
    ctx = _P()
    toks = np.ascontiguousarray(cons_tokens, dtype=np.int32)
    rc = load().dba_init(ctypes.byref(ctx), B, k, V, N, eos_id, pad_id,
                         toks.ctypes.data if toks.size else None,
                         _host(np.ascontiguousarray(phrase_offsets, dtype=np.int32), np.int32),
                         _host(np.ascontiguousarray(sent_offsets, dtype=np.int32), np.int32),
                         workspace_dev, workspace_bytes, hip_stream or None)
    _check(rc)
    return ctx


def dba_step(ctx, logp_dev: int, out_token_dev: int = 0, out_backptr_dev: int = 0,
             out_score_dev: int = 0, out_flags_dev: int = 0) -> int:
    return _check(load().dba_step(ctx, logp_dev, out_token_dev or None, out_backptr_dev or None,
                                  out_score_dev or None, out_flags_dev or None), ctx)


def dba_step_fmt(ctx, logp_dev: int, logp_format: int, out_token_dev: int = 0, out_backptr_dev: int = 0,
                 out_score_dev: int = 0, out_flags_dev: int = 0) -> int:
    return _check(load().dba_step_fmt(ctx, logp_dev, logp_format, out_token_dev or None,
                                      out_backptr_dev or None, out_score_dev or None,
                                      out_flags_dev or None), ctx)


def dba_step_noalloc(ctx, logp_dev: int, logp_format: int, out_token_dev: int = 0, out_backptr_dev: int = 0,
                     out_score_dev: int = 0, out_flags_dev: int = 0) -> int:
    return _check(load().dba_step_noalloc(ctx, logp_dev, logp_format, out_token_dev or None,
                                          out_backptr_dev or None, out_score_dev or None,
                                          out_flags_dev or None), ctx)


def dba_finalize(ctx, out_tokens: np.ndarray, out_len: np.ndarray, out_score: np.ndarray,
                 out_status: np.ndarray) -> int:
    return _check(load().dba_finalize(ctx, _host(out_tokens, np.int32), _host(out_len, np.int32),
                                      _host(out_score, np.float32), _host(out_status, np.int32)), ctx)


def dba_get_state(ctx, score=None, met_mask=None, inprog_phrase=None, inprog_pos=None, length=None,
                  flags=None) -> int:
    return _check(load().dba_get_state(ctx, _host(score, np.float32), _host(met_mask, np.uint64),
                                       _host(inprog_phrase, np.int32), _host(inprog_pos, np.int32),
                                       _host(length, np.int32), _host(flags, np.uint8)), ctx)


def dba_set_option(ctx, option: int, value: float) -> int:
    return _check(load().dba_set_option(ctx, option, float(value)), ctx)


def dba_get_finished(ctx, all_finished: np.ndarray) -> int:
    return _check(load().dba_get_finished(ctx, _host(all_finished, np.uint8)), ctx)


def dba_steps_done(ctx) -> int:
    return int(load().dba_steps_done(ctx))


def dba_destroy(ctx) -> None:
    load().dba_destroy(ctx)


def dba_debug_allocate(k: np.ndarray, C: np.ndarray, cnt: np.ndarray, alloc: np.ndarray,
                       scratch_dev: int, scratch_bytes: int, hip_stream: int = 0, adjust: bool = True) -> int:
    n = int(k.shape[0])
    assert cnt.shape == (n, 65) and alloc.shape == (n, 65)
    return _check(load().dba_debug_allocate(n, int(bool(adjust)), _host(k, np.int32), _host(C, np.int32),
                                            _host(cnt, np.int32), _host(alloc, np.int32),
                                            scratch_dev, scratch_bytes, hip_stream or None))


def dba_debug_wave_select(keys: np.ndarray, vals: np.ndarray, out: np.ndarray, fout: np.ndarray,
                          scratch_dev: int, scratch_bytes: int, hip_stream: int = 0) -> int:
    n = int(keys.shape[0])
    assert keys.shape == (n, 128) and vals.shape == (n, 64) and out.shape == (n, 256) and fout.shape == (n, 64)
    return _check(load().dba_debug_wave_select(n, _host(keys, np.uint64), _host(vals, np.float32),
                                               _host(out, np.uint64), _host(fout, np.float32),
                                               scratch_dev, scratch_bytes, hip_stream or None))


def dba_debug_row_max(src_dev: int, rows: int, V: int, out_max_dev: int, hip_stream: int = 0) -> int:
    return _check(load().dba_debug_row_max(src_dev, rows, V, out_max_dev, hip_stream or None))
