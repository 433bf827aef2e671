"""Seeded synthetic workloads standing in for a decoder's per-step output.

Everything here manufactures *inputs* only (log-prob tensors, constraint
phrases); none of the beam-allocation arithmetic lives in this package.  The
same bytes are handed to every consumer.

Recipe (all deterministic from one 64-bit seed):
  * reserved ids: PAD=0, 1, EOS=2, 3; constraint ids are drawn from [4, V)
  * a seeded permutation gives every non-reserved id a Zipf rank; ids 0, 1, 3
    take the three worst ranks
  * logit[t, b, h, v] = N(0,1) + alpha * (-s * ln rank(v)) (+ sparse boosts)
  * the EOS logit is N(0,1) - 30 until the last tenth of the run, then
    N(0,1) + 2
  * logp = log_softmax(logit) in double, rounded once to fp32
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.c")
_LIB = os.path.join(_HERE, "libsynth.so")

PAD_ID = 0
EOS_ID = 2
FIRST_FREE_ID = 4
BASE_SEED = 180406609

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15


def build(force: bool = False) -> str:
    """Compile the generator with gcc (host code only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC",
             _SRC, "-o", _LIB, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.synth_logp.restype = None
        lib.synth_logp.argtypes = [
            ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p]
        lib.synth_mix64.restype = ctypes.c_uint64
        lib.synth_mix64.argtypes = [ctypes.c_uint64]
        _lib = lib
    return _lib


def mix64(z: int) -> int:
    """SplitMix64 finaliser on Python ints (same function as in gen.c)."""
    z &= _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


class Stream:
    """Tiny counter-based integer stream for the small, host-side draws."""

    def __init__(self, seed: int, name: int):
        self._key = mix64((seed & _M64) ^ mix64(name + 0x5EED))
        self._n = 0

    def u64(self) -> int:
        self._n += 1
        return mix64((self._key + _GOLDEN * self._n) & _M64)

    def randint(self, lo: int, hi: int) -> int:
        """Uniform integer in [lo, hi] (modulo bias is irrelevant at these ranges)."""
        return lo + self.u64() % (hi - lo + 1)

    def uniform(self) -> float:
        return ((self.u64() >> 11) + 0.5) / 9007199254740992.0


def _mix64_np(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


@dataclass
class Workload:
    """One synthetic decoding job: shapes, constraints and the log-prob recipe."""

    B: int
    k: int
    V: int
    T: int
    seed: int
    constraints: List[List[List[int]]]          # [sentence][phrase][token]
    zipf_s: float = 1.1
    alpha: float = 1.0
    eos_id: int = EOS_ID
    pad_id: int = PAD_ID
    eos_low: float = -30.0
    eos_high: float = 2.0
    eos_switch: Optional[int] = None            # first step with the high EOS logit
    boost_tokens: List[List[int]] = field(default_factory=list)  # config-3 style boosts
    boost_value: float = 3.0
    boost_prob: float = 0.3
    name: str = "custom"

    def __post_init__(self):
        if self.eos_switch is None:
            self.eos_switch = self.T - math.ceil(self.T / 10)
        if not self.boost_tokens:
            self.boost_tokens = [[] for _ in range(self.B)]
        self._zb = None

    # ---- constraints -----------------------------------------------------
    def csr(self):
        """(cons_tokens, phrase_offsets, sent_offsets) as int32 arrays."""
        toks: List[int] = []
        poff = [0]
        soff = [0]
        for sent in self.constraints:
            for ph in sent:
                toks.extend(ph)
                poff.append(len(toks))
            soff.append(len(poff) - 1)
        return (np.asarray(toks, dtype=np.int32), np.asarray(poff, dtype=np.int32),
                np.asarray(soff, dtype=np.int32))

    def n_tokens(self, b: int) -> int:
        return sum(len(p) for p in self.constraints[b])

    # ---- log-probs ---------------------------------------------------------
    def _zbias_base(self) -> np.ndarray:
        if self._zb is None:
            V = self.V
            free = np.arange(FIRST_FREE_ID, V, dtype=np.uint64)
            h = _mix64_np(free * np.uint64(_GOLDEN) + np.uint64(mix64(self.seed ^ 0xA11CE)))
            order = np.argsort(h, kind="stable")
            rank = np.empty(V, dtype=np.float64)
            rank[free[order].astype(np.int64)] = np.arange(1, V - FIRST_FREE_ID + 1)
            worst = [i for i in (0, 1, 3) if i < V]
            for n, i in enumerate(worst):
                rank[i] = V - FIRST_FREE_ID + 1 + n
            if self.eos_id < V:
                rank[self.eos_id] = 1.0
            self._zb = self.alpha * (-self.zipf_s * np.log(rank))
        return self._zb

    def zbias(self, t: int) -> np.ndarray:
        zb = self._zbias_base().copy()
        zb[self.eos_id] = self.eos_high if t >= self.eos_switch else self.eos_low
        return zb

    def _boosts(self, t: int):
        if not any(self.boost_tokens):
            return None
        off = [0]
        tok: List[int] = []
        for b in range(self.B):
            for i, w in enumerate(self.boost_tokens[b]):
                u = mix64(mix64(self.seed ^ 0xB005) + _GOLDEN * ((t * self.B + b) * 64 + i + 1))
                if ((u >> 11) + 0.5) / 9007199254740992.0 < self.boost_prob:
                    tok.append(w)
            off.append(len(tok))
        return (np.asarray(off, dtype=np.int64), np.asarray(tok, dtype=np.int32),
                np.full(len(tok), self.boost_value, dtype=np.float64))

    def logp(self, t: int, sentences: Optional[Sequence[int]] = None,
             out: Optional[np.ndarray] = None) -> np.ndarray:
        """fp32 log-probs of step t: [B, k, V], or [len(sentences), k, V]."""
        lib = _load()
        zb = np.ascontiguousarray(self.zbias(t))
        boosts = self._boosts(t)
        sents = list(range(self.B)) if sentences is None else list(sentences)
        if out is None:
            out = np.empty((len(sents), self.k, self.V), dtype=np.float32)
        assert out.dtype == np.float32 and out.flags.c_contiguous
        assert out.shape == (len(sents), self.k, self.V)
        ex = (None, None, None) if boosts is None else tuple(a.ctypes.data for a in boosts)

        def run(row0, nrows, dst):
            lib.synth_logp(self.seed & _M64, t, row0, nrows, self.k, self.V, zb.ctypes.data,
                           ex[0], ex[1], ex[2], dst)

        if sentences is None:
            run(0, self.B * self.k, out.ctypes.data)
        else:
            for i, b in enumerate(sents):
                run(b * self.k, self.k, out[i].ctypes.data)
        return out


def narrow16(x: np.ndarray, fmt: str) -> np.ndarray:
    """The fp32 log-probs as a 16-bit decoder would hand them over: rounded once more, to nearest
    even, to IEEE binary16 ("f16") or bfloat16 ("bf16"); returned as the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if fmt == "f16":
        with np.errstate(over="ignore"):
            return x.astype(np.float16).view(np.uint16)
    if fmt == "bf16":
        u = x.view(np.uint32)
        nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
        r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
        r = np.where(nan, (u >> np.uint32(16)) | np.uint32(0x40), r)
        return r.astype(np.uint16)
    raise ValueError(f"unknown 16-bit format {fmt!r}")


def _draw_token(rs: Stream, V: int, used: Optional[set] = None) -> int:
    while True:
        w = rs.randint(FIRST_FREE_ID, V - 1)
        if used is None or w not in used:
            if used is not None:
                used.add(w)
            return w


def _phrases_with_total(rs: Stream, total: int, lo: int, hi: int) -> List[int]:
    """Phrase lengths, each uniform in [lo, hi] (last one cut), summing to total."""
    lens = []
    left = total
    while left > 0:
        n = min(rs.randint(lo, hi), left)
        lens.append(n)
        left -= n
    return lens


def fixed_total_constraints(seed: int, B: int, V: int, total: int, max_len: int = 5):
    """Every sentence gets exactly `total` constraint tokens in phrases of 1..max_len."""
    out = []
    for b in range(B):
        rs = Stream(seed, 7000 + b)
        lens = _phrases_with_total(rs, total, 1, max_len)
        out.append([[_draw_token(rs, V) for _ in range(n)] for n in lens])
    return out


def make_config(idx: int, seed: Optional[int] = None, T: Optional[int] = None,
                B: Optional[int] = None) -> Workload:
    """The five named configurations (idx 1..5).  T and B may be cut for quick runs."""
    seed = BASE_SEED + idx if seed is None else seed
    shapes = {1: (1, 5, 1000, 20), 2: (1, 10, 32000, 60), 3: (16, 10, 32000, 80),
              4: (64, 20, 32000, 100), 5: (128, 64, 50000, 120)}
    B0, k, V, T0 = shapes[idx]
    B = B0 if B is None else B
    T = T0 if T is None else T
    cons: List[List[List[int]]] = []
    boost: List[List[int]] = []
    for b in range(B):
        rs = Stream(seed, 1000 + b)
        bt: List[int] = []
        if idx == 1:
            sent = [[_draw_token(rs, V), _draw_token(rs, V)]]
        elif idx == 2:
            used: set = set()
            sent = [[_draw_token(rs, V, used) for _ in range(rs.randint(1, 3))] for _ in range(4)]
        elif idx == 3:
            sent = [[_draw_token(rs, V) for _ in range(rs.randint(1, 4))]
                    for _ in range(rs.randint(1, 8))]
            bt = [w for ph in sent for w in ph if rs.uniform() < 0.2]
        elif idx == 4:
            P = rs.randint(8, 12)
            lens = [1] * P
            for _ in range(32 - P):
                while True:
                    j = rs.randint(0, P - 1)
                    if lens[j] < 5:
                        lens[j] += 1
                        break
            sent = [[_draw_token(rs, V) for _ in range(n)] for n in lens]
        elif idx == 5:
            lens = _phrases_with_total(rs, rs.randint(0, 32), 1, 5)
            sent = [[_draw_token(rs, V) for _ in range(n)] for n in lens]
        else:
            raise ValueError("config index must be 1..5")
        cons.append(sent)
        boost.append(bt)
    return Workload(B=B, k=k, V=V, T=T, seed=seed, constraints=cons,
                    zipf_s=0.9 if idx == 5 else 1.1, boost_tokens=boost,
                    name=f"config{idx}")


def make_small(seed: int, B: int, k: int, V: int, T: int, max_phrases: int = 3,
               max_len: int = 3, dup_prob: float = 0.3, zipf_s: float = 1.1,
               boost: bool = True) -> Workload:
    """Small fuzz workloads: few tokens, repeated ids and shared prefixes on purpose."""
    cons = []
    boosts = []
    for b in range(B):
        rs = Stream(seed, 2000 + b)
        pool: List[int] = []
        sent = []
        for _ in range(rs.randint(0, max_phrases)):
            ph = []
            for _ in range(rs.randint(1, max_len)):
                if pool and rs.uniform() < dup_prob:
                    ph.append(pool[rs.randint(0, len(pool) - 1)])
                else:
                    ph.append(_draw_token(rs, V))
                    pool.append(ph[-1])
            sent.append(ph)
        cons.append(sent)
        boosts.append(sorted(set(pool)) if boost else [])
    return Workload(B=B, k=k, V=V, T=T, seed=seed, constraints=cons, zipf_s=zipf_s,
                    boost_tokens=boosts, boost_value=4.0, boost_prob=0.35, name="small")


def two_profile_logp(seed: int, t: int, B: int, k: int, V: int, eos_id: int = EOS_ID) -> np.ndarray:
    """Log-probs [B, k, V] for decodes in which completed hypotheses get onto the beam and are pushed
    off it again: every row's distribution is one of two profiles over a seeded shuffle of the
    vocabulary - "peaky" (0.85, 0.10, then a thin tail; end-of-sentence often holds the 0.10) or "flat"
    (0.46, 0.44, thin tail).  A weak completion enters behind a peaky row's favourite and loses its
    slot when the survivors' next rows are flat.  log() of the table in double, rounded once to fp32."""
    assert V >= 6
    out = np.empty((B, k, V), dtype=np.float32)
    tail = V - 2
    for b in range(B):
        for h in range(k):
            rs = Stream(seed, (t * B + b) * 64 + h + 90000)
            peaky = rs.randint(0, 2) != 0
            top = (0.85, 0.10) if peaky else (0.46, 0.44)
            rest = (1.0 - top[0] - top[1]) / tail
            order = list(range(V))
            for i in range(V - 1, 0, -1):
                j = rs.randint(0, i)
                order[i], order[j] = order[j], order[i]
            if peaky and rs.randint(0, 1) == 0:          # end-of-sentence takes the second place
                order.remove(eos_id)
                order.insert(1, eos_id)
            p = np.empty(V, dtype=np.float64)
            for place, w in enumerate(order):
                p[w] = top[place] if place < 2 else rest * (1.0 + 0.01 * place)
            out[b, h] = np.log(p / p.sum()).astype(np.float32)
    return out


@dataclass
class TwoProfileWorkload(Workload):
    """A Workload whose log-probs come from two_profile_logp (V is small: 6..64)."""

    def logp(self, t: int, sentences: Optional[Sequence[int]] = None,
             out: Optional[np.ndarray] = None) -> np.ndarray:
        lp = two_profile_logp(self.seed, t, self.B, self.k, self.V, self.eos_id)
        if sentences is not None:
            lp = np.ascontiguousarray(lp[list(sentences)])
        if out is not None:
            out[...] = lp
            return out
        return lp
