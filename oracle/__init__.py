"""Python face of the CPU oracle (oracle/dba_oracle.c).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
CPU-baseline leg may import this; the GPU library and its binding never do.
It holds no arithmetic of its own - it marshals arrays into the C functions
and keeps the per-sentence beam between steps.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dba_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

FLAG_FINISHED = 1
FLAG_DEAD = 2
MAX_TOKENS = 64


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-shared",
             "-fPIC", _SRC, "-o", _LIB, "-lm"])
    return _LIB


_lib = None
_P = ctypes.c_void_p


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.dba_oracle_allocate.restype = None
        lib.dba_oracle_allocate.argtypes = [ctypes.c_int, ctypes.c_int, _P, _P]
        lib.dba_oracle_add.restype = None
        lib.dba_oracle_add.argtypes = [ctypes.c_int, _P, _P, ctypes.c_uint64, ctypes.c_int,
                                       ctypes.c_int, ctypes.c_int, _P, _P, _P, _P, _P]
        lib.dba_oracle_step.restype = ctypes.c_int
        lib.dba_oracle_allocate_fixed.restype = None
        lib.dba_oracle_allocate_fixed.argtypes = [ctypes.c_int, ctypes.c_int, _P, _P]
        lib.dba_oracle_step.argtypes = [ctypes.c_int] * 5 + [_P] * 22 + [ctypes.c_int, ctypes.c_int,
                                                                        ctypes.c_float, _P]
        lib.dba_oracle_finalize.restype = ctypes.c_int
        lib.dba_oracle_finalize.argtypes = [ctypes.c_int] * 4 + [_P] * 10 + [ctypes.c_int]
        lib.dba_oracle_track_completed.restype = None
        lib.dba_oracle_track_completed.argtypes = [ctypes.c_int, ctypes.c_int, _P, _P, _P, ctypes.c_int, _P, _P]
        lib.dba_oracle_finalize_tracked.restype = ctypes.c_int
        lib.dba_oracle_finalize_tracked.argtypes = [ctypes.c_int] * 4 + [_P] * 10 + [ctypes.c_int, _P, _P]
        _lib = lib
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def allocate(k: int, cnt: Sequence[int], adjust: bool = True) -> np.ndarray:
    """Slots per bank for bank counts cnt[0..C] (Sec. 3.2); adjust=False: Sec. 5's fixed split."""
    c = np.ascontiguousarray(cnt, dtype=np.int32)
    out = np.zeros_like(c)
    fn = _load().dba_oracle_allocate if adjust else _load().dba_oracle_allocate_fixed
    fn(int(k), len(c) - 1, c.ctypes.data, out.ctypes.data)
    return out


def widen16(bits: np.ndarray, fmt: str) -> np.ndarray:
    """16-bit log-probs (uint16 bit patterns of IEEE binary16 "f16" or bfloat16 "bf16") as the
    fp32 values they stand for; both conversions are exact.  The step then computes, as always,
    one fp32 addition prev + logp on the widened value."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if fmt == "f16":
        return bits.view(np.float16).astype(np.float32)
    if fmt == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    raise ValueError(f"unknown 16-bit format {fmt!r}")


def _phrase_arrays(phrases: Sequence[Sequence[int]]):
    off = [0]
    tok: List[int] = []
    for p in phrases:
        tok.extend(int(x) for x in p)
        off.append(len(tok))
    return (np.asarray(off, dtype=np.int32), np.asarray(tok + [0], dtype=np.int32)[:max(len(tok), 1)])


def add(phrases, met: int, ip: int, iq: int, w: int):
    """(met', ip', iq', expandable tokens of the state before w).  w < 0: no token."""
    off, tok = _phrase_arrays(phrases)
    m = ctypes.c_uint64(0)
    a = ctypes.c_int(0)
    b = ctypes.c_int(0)
    nn = ctypes.c_int(0)
    nxt = np.zeros(MAX_TOKENS, dtype=np.int32)
    _load().dba_oracle_add(len(phrases), off.ctypes.data, tok.ctypes.data, met, ip, iq, w,
                           ctypes.byref(m), ctypes.byref(a), ctypes.byref(b), nxt.ctypes.data,
                           ctypes.byref(nn))
    return m.value, a.value, b.value, [int(x) for x in nxt[:nn.value]]


class SentenceBeam:
    """Beam of one sentence, advanced by dba_oracle_step."""

    def __init__(self, k: int, V: int, phrases, eos_id: int, pad_id: int, adjust: bool = True,
                 normalize_finished: bool = False, prune_threshold: Optional[float] = None,
                 track_completed: bool = False):
        self.k, self.V, self.eos_id, self.pad_id = k, V, eos_id, pad_id
        self.adjust, self.normalize_finished = bool(adjust), bool(normalize_finished)
        # variant: remember the best completed hypothesis seen on any beam (Sec. 3.3)
        self.track_completed = bool(track_completed)
        self.rec_int = np.zeros(4, dtype=np.int32)      # have, step, slot, length
        self.rec_flt = np.zeros(2, dtype=np.float32)    # value per word, stored score
        self.prune_threshold = -1.0 if prune_threshold is None else float(prune_threshold)
        self.all_finished = 0
        self.any_finished = 0
        self.stop_bits = 0
        self.phrases = [list(p) for p in phrases]
        self.off, self.tok = _phrase_arrays(self.phrases)
        self.P = len(self.phrases)
        self.C = int(self.off[-1])
        # decoder-init: one live, empty hypothesis in slot 0 (score +0.0), the rest empty
        self.score = np.full(k, -np.inf, dtype=np.float32)
        self.score[0] = 0.0
        self.met = np.zeros(k, dtype=np.uint64)
        self.ip = np.full(k, -1, dtype=np.int32)
        self.iq = np.zeros(k, dtype=np.int32)
        self.flags = np.full(k, FLAG_DEAD, dtype=np.uint8)
        self.flags[0] = 0
        self.len = np.zeros(k, dtype=np.int32)
        self.token = np.full(k, pad_id, dtype=np.int32)
        self.backptr = np.full(k, -1, dtype=np.int32)
        self.hist_token: List[np.ndarray] = []
        self.hist_backptr: List[np.ndarray] = []
        self.dbg = None

    @property
    def nmet(self) -> np.ndarray:
        return np.array([bin(int(m)).count("1") for m in self.met], dtype=np.int32)

    def step(self, logp: np.ndarray, debug: bool = False):
        k, V = self.k, self.V
        logp = np.ascontiguousarray(logp, dtype=np.float32)
        assert logp.shape == (k, V)
        fin = (self.flags & FLAG_FINISHED).astype(np.uint8)
        o_tok = np.empty(k, np.int32)
        o_bp = np.empty(k, np.int32)
        o_sc = np.empty(k, np.float32)
        o_fl = np.empty(k, np.uint8)
        o_met = np.empty(k, np.uint64)
        o_ip = np.empty(k, np.int32)
        o_iq = np.empty(k, np.int32)
        o_len = np.empty(k, np.int32)
        done = np.zeros(1, np.int32)
        d_n = d_flat = d_bank = d_cnt = d_alloc = None
        if debug:
            cap = max(1, k * (self.P + 2))
            d_n = np.zeros(1, np.int32)
            d_flat = np.zeros(cap, np.int64)
            d_bank = np.zeros(cap, np.int32)
            d_cnt = np.zeros(self.C + 1, np.int32)
            d_alloc = np.zeros(self.C + 1, np.int32)
        rc = _load().dba_oracle_step(
            k, V, self.eos_id, self.pad_id, self.P, _ptr(self.off), _ptr(self.tok),
            _ptr(self.score), _ptr(self.met), _ptr(self.ip), _ptr(self.iq), _ptr(fin),
            _ptr(self.len), _ptr(logp), _ptr(o_tok), _ptr(o_bp), _ptr(o_sc), _ptr(o_fl),
            _ptr(o_met), _ptr(o_ip), _ptr(o_iq), _ptr(o_len), _ptr(d_n), _ptr(d_flat),
            _ptr(d_bank), _ptr(d_cnt), _ptr(d_alloc), int(self.adjust), int(self.normalize_finished),
            self.prune_threshold, _ptr(done))
        self.all_finished = int(done[0]) & 1          # Sec. 4: every hypothesis on the beam is completed
        self.any_finished = (int(done[0]) >> 1) & 1   # Sec. 6.3: some hypothesis is completed
        self.stop_bits = int(done[0])
        if rc != 0:
            raise ValueError("dba_oracle_step rejected its arguments")
        self.token, self.backptr, self.score, self.flags = o_tok, o_bp, o_sc, o_fl
        self.met, self.ip, self.iq, self.len = o_met, o_ip, o_iq, o_len
        self.hist_token.append(o_tok)
        self.hist_backptr.append(o_bp)
        if self.track_completed:
            _load().dba_oracle_track_completed(k, len(self.hist_token) - 1, _ptr(o_sc), _ptr(o_fl), _ptr(o_len),
                                               int(self.normalize_finished), _ptr(self.rec_int), _ptr(self.rec_flt))
        if debug:
            n = int(d_n[0])
            self.dbg = dict(flat=d_flat[:n].copy(), bank=d_bank[:n].copy(), cnt=d_cnt, alloc=d_alloc)
        return self

    def finalize(self, N: int):
        T = len(self.hist_token)
        ht = np.ascontiguousarray(np.stack(self.hist_token) if T else np.zeros((0, self.k), np.int32))
        hb = np.ascontiguousarray(np.stack(self.hist_backptr) if T else np.zeros((0, self.k), np.int32))
        toks = np.empty(N, np.int32)
        ln = np.zeros(1, np.int32)
        sc = np.zeros(1, np.float32)
        stt = np.zeros(1, np.int32)
        nm = self.nmet
        if self.track_completed:
            _load().dba_oracle_finalize_tracked(self.k, T, N, self.pad_id, _ptr(ht), _ptr(hb), _ptr(self.score),
                                                _ptr(self.flags), _ptr(self.len), _ptr(nm), _ptr(toks),
                                                _ptr(ln), _ptr(sc), _ptr(stt), int(self.normalize_finished),
                                                _ptr(self.rec_int), _ptr(self.rec_flt))
        else:
            _load().dba_oracle_finalize(self.k, T, N, self.pad_id, _ptr(ht), _ptr(hb), _ptr(self.score),
                                        _ptr(self.flags), _ptr(self.len), _ptr(nm), _ptr(toks),
                                        _ptr(ln), _ptr(sc), _ptr(stt), int(self.normalize_finished))
        return toks, int(ln[0]), np.float32(sc[0]), int(stt[0])


class BatchBeam:
    """B independent sentence beams; step() may spread sentences over threads."""

    def __init__(self, k: int, V: int, constraints, eos_id: int, pad_id: int,
                 sentences: Optional[Sequence[int]] = None, **variants):
        self.sent_ids = list(range(len(constraints))) if sentences is None else list(sentences)
        self.beams = [SentenceBeam(k, V, constraints[b], eos_id, pad_id, **variants) for b in self.sent_ids]
        self.k, self.V = k, V

    def step(self, logp: np.ndarray, threads: int = 1, debug: bool = False):
        """logp: [len(self.beams), k, V] rows of exactly these sentences."""
        assert logp.shape[0] == len(self.beams)
        if threads <= 1 or len(self.beams) == 1:
            for i, bm in enumerate(self.beams):
                bm.step(logp[i], debug)
        else:
            with ThreadPoolExecutor(max_workers=threads) as ex:
                list(ex.map(lambda i: self.beams[i].step(logp[i], debug), range(len(self.beams))))
        return self

    def stacked(self, name: str) -> np.ndarray:
        return np.stack([getattr(bm, name) for bm in self.beams])

    def finalize(self, N: int):
        res = [bm.finalize(N) for bm in self.beams]
        return (np.stack([r[0] for r in res]), np.array([r[1] for r in res], np.int32),
                np.array([r[2] for r in res], np.float32), np.array([r[3] for r in res], np.int32))
