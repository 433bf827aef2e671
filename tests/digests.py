"""Chained digests of a decode, one chain per sentence.

A chain is fed, step after step, the bytes of everything a step leaves behind for one sentence
(tokens, parents, fp32 scores, flags, met masks, phrase under way, lengths, stopping bits), so its
value after step t stands for the whole decode up to t: two decodes that differ anywhere up to
step t disagree at t and ever after.  No arithmetic of the method lives here - only hashing of
arrays that someone else computed.
"""
from __future__ import annotations

import hashlib
from typing import Dict, List, Sequence

import numpy as np

FIELDS = (("token", np.int32), ("backptr", np.int32), ("score", np.float32), ("flags", np.uint8),
          ("met", np.uint64), ("ip", np.int32), ("iq", np.int32), ("len", np.int32))


class Chains:
    """One running 64-bit digest per sentence."""

    def __init__(self, n_sentences: int):
        self.h = [b"\0" * 8 for _ in range(n_sentences)]

    def feed(self, i: int, fields: Dict[str, np.ndarray], stop_bits: int) -> None:
        """fields[name] = the k values of sentence i after the step, for every name in FIELDS."""
        m = hashlib.blake2b(self.h[i], digest_size=8)
        for name, dt in FIELDS:
            a = np.ascontiguousarray(fields[name])
            assert a.dtype == dt, (name, a.dtype)
            m.update(a.tobytes())
        m.update(bytes([int(stop_bits) & 0xFF]))
        self.h[i] = m.digest()

    def hex(self) -> List[str]:
        return [x.hex() for x in self.h]


def final_digest(tokens: np.ndarray, length: int, score, status: int) -> str:
    """Digest of what the end of decoding returns for one sentence."""
    m = hashlib.blake2b(digest_size=8)
    m.update(np.ascontiguousarray(tokens, dtype=np.int32).tobytes())
    m.update(np.int32(length).tobytes())
    m.update(np.float32(score).tobytes())
    m.update(np.int32(status).tobytes())
    return m.hexdigest()


def read_table(path: str):
    """-> (header dict, {step: [hex per sentence]}, [final hex per sentence])."""
    head: Dict[str, str] = {}
    steps: Dict[int, List[str]] = {}
    final: List[str] = []
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if not line:
                continue
            if line.startswith("#"):
                if "=" in line:
                    for part in line[1:].split():
                        if "=" in part:
                            key, val = part.split("=", 1)
                            head[key] = val
                continue
            kind, rest = line.split(" ", 1)
            if kind == "final":
                final = rest.split()
            else:
                steps[int(kind)] = rest.split()
    return head, steps, final


def write_table(path: str, comment: Sequence[str], head: Dict[str, object], steps: Dict[int, List[str]],
                final: List[str]) -> None:
    with open(path, "w") as fh:
        for c in comment:
            fh.write(f"# {c}\n")
        fh.write("# " + " ".join(f"{key}={val}" for key, val in head.items()) + "\n")
        for t in sorted(steps):
            fh.write(f"{t} " + " ".join(steps[t]) + "\n")
        fh.write("final " + " ".join(final) + "\n")
