"""Plain Python reference of the paper's context de-duplication (Section 6, appendix
algorithm "Context De-duplication").

TEST INFRASTRUCTURE ONLY: imported by the tests and by the CPU-baseline leg of the benchmark.
The C++ library never imports this module and this module imports nothing from it.

Readings where the paper leaves a choice open:
  * Hash is 64-bit FNV-1a over bytes (the paper names no hash function); the same function
    hashes a text line for the boundary test and a whole sub-block for the lookup.
  * A text line is the bytes up to and including its newline (the last line may lack one); the
    boundary test hashes the line without the newline.  A sub-block ends after every line whose
    hash is a multiple of the chunk modulus M, and at the end of the block.
  * A sub-block found under another block's id is replaced by a reference to that block - the
    first occurrence, because an entry is only ever written when the hash is new or is this
    block's own.
  * The set of seen blocks grows only after the whole turn has been processed, as printed: a
    block id that occurs twice in one turn is processed twice.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Set, Tuple

FNV_OFFSET = 0xCBF29CE484222325
FNV_PRIME = 0x100000001B3


def fnv1a64(data: bytes) -> int:
    h = FNV_OFFSET
    for byte in data:
        h ^= byte
        h = (h * FNV_PRIME) & 0xFFFFFFFFFFFFFFFF
    return h


def lines_of(block: bytes) -> List[bytes]:
    """The block cut after every newline; the pieces concatenate to the block."""
    out, start = [], 0
    for i, byte in enumerate(block):
        if byte == 0x0A:
            out.append(block[start:i + 1])
            start = i + 1
    if start < len(block):
        out.append(block[start:])
    return out


def cdc(block: bytes, modulus: int) -> List[bytes]:
    """Content-defined chunking by text lines: a sub-block ends after a line whose hash is
    0 modulo `modulus`."""
    subs, cur = [], b""
    for line in lines_of(block):
        cur += line
        body = line[:-1] if line.endswith(b"\n") else line
        if fnv1a64(body) % modulus == 0:
            subs.append(cur)
            cur = b""
    if cur:
        subs.append(cur)
    return subs


class Conversation:
    """State of one conversation: block ids seen in earlier turns, and for every sub-block
    hash the block it was first seen in."""

    def __init__(self, modulus: int):
        assert modulus >= 1
        self.modulus = modulus
        self.seen_blocks: Set[int] = set()
        self.seen_subblocks: Dict[int, int] = {}

    def turn(self, ids: Sequence[int], blocks: Sequence[bytes]):
        """One turn.  Returns, per block of the new context, either ("block", id) when the
        whole block is replaced by a reference to the earlier turn, or ("subs", [(begin, end,
        ref), ...]) with the byte range of every sub-block and the block id it is replaced by
        (-1: kept)."""
        out = []
        for b, text in zip(ids, blocks):
            if b in self.seen_blocks:
                out.append(("block", int(b)))
                continue
            subs: List[Tuple[int, int, int]] = []
            at = 0
            for s in cdc(text, self.modulus):
                f = fnv1a64(s)
                owner = self.seen_subblocks.get(f)
                if owner is not None and owner != b:
                    subs.append((at, at + len(s), int(owner)))
                else:
                    self.seen_subblocks[f] = int(b)
                    subs.append((at, at + len(s), -1))
                at += len(s)
            out.append(("subs", subs))
        self.seen_blocks.update(int(b) for b in ids)
        return out


def kept_bytes(result) -> int:
    """Bytes of the turn that still have to be prefilled."""
    return sum(e - b for kind, x in result if kind == "subs" for b, e, ref in x if ref < 0)
