"""Reader and writer of the sandbox's tape file, written from the format stated in include/tm_sandbox.h
(independent of the library's own reader / writer): 16-byte header "TMTAPE01" + uint64 entry count; per
entry a 64-byte record {uint32 kind, scope, site, dtype; uint64 bytes, checksum; 32 zero bytes} and the
payload padded to 64 bytes.  Payloads are handed over as raw bytes."""
from __future__ import annotations

import struct
from typing import List, Tuple

import numpy as np

MAGIC = b"TMTAPE01"
MASK = (1 << 64) - 1


def checksum(payload: bytes) -> int:
    pad = (-len(payload)) % 8
    words = np.frombuffer(payload + b"\0" * pad, dtype="<u8")
    c = 0xcbf29ce484222325
    for w in words.tolist():
        c = ((c ^ w) * 0x100000001b3) & MASK
    return c


def write_tape(path: str, entries: List[Tuple[int, int, int, int, bytes]]) -> None:
    """entries: (kind, scope, site, dtype, payload bytes)."""
    with open(path, "wb") as f:
        f.write(MAGIC + struct.pack("<Q", len(entries)))
        for kind, scope, site, dtype, payload in entries:
            f.write(struct.pack("<IIIIQQ", kind, scope, site, dtype, len(payload), checksum(payload)) + b"\0" * 32)
            f.write(payload + b"\0" * ((-len(payload)) % 64))


def read_tape(path: str, verify: bool = True) -> List[Tuple[int, int, int, int, bytes]]:
    raw = open(path, "rb").read()
    assert raw[:8] == MAGIC
    (count,) = struct.unpack_from("<Q", raw, 8)
    at, out = 16, []
    for _ in range(count):
        kind, scope, site, dtype, nbytes, csum = struct.unpack_from("<IIIIQQ", raw, at)
        assert raw[at + 32:at + 64] == b"\0" * 32
        at += 64
        payload = raw[at:at + nbytes]
        assert len(payload) == nbytes
        if verify:
            assert checksum(payload) == csum
        at += nbytes + ((-nbytes) % 64)
        out.append((kind, scope, site, dtype, payload))
    assert at == len(raw)
    return out


def payload_of(a: np.ndarray, dtype: int) -> bytes:
    """fp32 array -> storage bytes (dtype 1: bf16, the values must lie on the bf16 grid)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == 1:
        bits = a.view(np.uint32)
        assert not (bits & np.uint32(0xFFFF)).any(), "not bf16-exact"
        return (bits >> np.uint32(16)).astype("<u2").tobytes()
    return a.astype("<f4").tobytes()


def array_of(payload: bytes, dtype: int) -> np.ndarray:
    if dtype == 1:
        return (np.frombuffer(payload, dtype="<u2").astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return np.frombuffer(payload, dtype="<f4").astype(np.float64)
