"""Device-memory plumbing around the binding: PyTorch owns the buffers and the stream.

No arithmetic of the method happens here; every step runs in libdba's kernels.
"""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as _b


class Session:
    """One decoding job: workspace + output buffers on the current CUDA/HIP device."""

    def __init__(self, B: int, k: int, V: int, N: int, eos_id: int, pad_id: int,
                 cons_tokens: np.ndarray, phrase_offsets: np.ndarray, sent_offsets: np.ndarray,
                 stream: Optional[torch.cuda.Stream] = None, options: Optional[dict] = None):
        if not torch.cuda.is_available():
            raise RuntimeError("libdba needs a GPU: no HIP device is visible")
        _b.load()
        self.B, self.k, self.V, self.N = B, k, V, N
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        nbytes = _b.dba_workspace_bytes(B, k, V, N, _b.DBA_MAX_CONS_TOKENS)
        if nbytes == 0:
            raise _b.DbaError(_b.DBA_EINVAL, "shape outside the library's limits")
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
        base = (self.workspace.data_ptr() + 255) // 256 * 256
        self.out_token = torch.empty((B, k), dtype=torch.int32, device="cuda")
        self.out_backptr = torch.empty((B, k), dtype=torch.int32, device="cuda")
        self.out_score = torch.empty((B, k), dtype=torch.float32, device="cuda")
        self.out_flags = torch.empty((B, k), dtype=torch.uint8, device="cuda")
        self.ctx = _b.dba_init(B, k, V, N, eos_id, pad_id, cons_tokens, phrase_offsets, sent_offsets,
                               base, nbytes, self.stream.cuda_stream)
        for opt, val in (options or {}).items():
            _b.dba_set_option(self.ctx, opt, val)

    _FORMATS = {torch.float32: _b.DBA_LOGP_F32, torch.float16: _b.DBA_LOGP_F16, torch.bfloat16: _b.DBA_LOGP_BF16}

    def step(self, logp: torch.Tensor, noalloc: bool = False) -> None:
        """Enqueue one step; logp is a contiguous device tensor [B,k,V] of fp32, fp16 or bf16.
        noalloc: through dba_step_noalloc (the library's own scratch instead of the workspace's)."""
        assert logp.is_cuda and logp.dtype in self._FORMATS and logp.is_contiguous()
        assert tuple(logp.shape) == (self.B, self.k, self.V)
        if noalloc:
            _b.dba_step_noalloc(self.ctx, logp.data_ptr(), self._FORMATS[logp.dtype], self.out_token.data_ptr(),
                                self.out_backptr.data_ptr(), self.out_score.data_ptr(), self.out_flags.data_ptr())
        elif logp.dtype == torch.float32:
            _b.dba_step(self.ctx, logp.data_ptr(), self.out_token.data_ptr(), self.out_backptr.data_ptr(),
                        self.out_score.data_ptr(), self.out_flags.data_ptr())
        else:
            _b.dba_step_fmt(self.ctx, logp.data_ptr(), self._FORMATS[logp.dtype], self.out_token.data_ptr(),
                            self.out_backptr.data_ptr(), self.out_score.data_ptr(), self.out_flags.data_ptr())

    def outputs(self):
        """(token, backptr, score, flags) of the last step as numpy arrays (synchronises)."""
        self.stream.synchronize()
        return (self.out_token.cpu().numpy(), self.out_backptr.cpu().numpy(),
                self.out_score.cpu().numpy(), self.out_flags.cpu().numpy())

    def state(self):
        n = (self.B, self.k)
        st = dict(score=np.empty(n, np.float32), met_mask=np.empty(n, np.uint64),
                  inprog_phrase=np.empty(n, np.int32), inprog_pos=np.empty(n, np.int32),
                  length=np.empty(n, np.int32), flags=np.empty(n, np.uint8))
        _b.dba_get_state(self.ctx, **st)
        return st

    def finished(self) -> np.ndarray:
        """[B] uint8 of DBA_STOP_ALL / DBA_STOP_ANY bits per sentence (synchronises)."""
        done = np.empty(self.B, np.uint8)
        _b.dba_get_finished(self.ctx, done)
        return done

    def finalize(self):
        toks = np.empty((self.B, self.N), np.int32)
        ln = np.empty(self.B, np.int32)
        sc = np.empty(self.B, np.float32)
        status = np.empty(self.B, np.int32)
        _b.dba_finalize(self.ctx, toks, ln, sc, status)
        return toks, ln, sc, status

    def close(self) -> None:
        if self.ctx is not None:
            self.stream.synchronize()
            _b.dba_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
