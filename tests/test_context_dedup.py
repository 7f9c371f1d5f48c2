"""Context de-duplication (paper, Section 6 and the appendix algorithm): pins of the Python
oracle (the paper's block-level example, published hash vectors, chunking invariants, the
algorithm's rules by hand) and parity of the C++ library against it - byte ranges, references
and kept bytes must be identical.  Host code only: no GPU needed."""
import os

import numpy as np
import pytest

from oracle import context_dedup as OD
import paper_2511_03475_amd as cp
import workloads as W

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    rows = []
    for line in open(os.path.join(HERE, "golden", "context_dedup_examples.txt")):
        line = line.rstrip("\n")
        if line and not line.startswith("#"):
            rows.append([x.strip() for x in line.split("|")])
    return rows


def _ids(s):
    s = s.split(":", 1)[1].strip() if ":" in s else s
    return [int(x) for x in s.split(",")] if s else []


# ---- oracle pins ---------------------------------------------------------------------------
def test_paper_block_level_example_and_hash_vectors():
    conv = OD.Conversation(modulus=8)
    text = {i: (f"block {i} line one\nblock {i} line two\n").encode() for i in range(10)}
    for kind, a, *rest in _golden():
        if kind == "fnv1a64":
            assert OD.fnv1a64(a.encode()) == int(rest[0], 16)
        else:
            ids = _ids(a)
            res = conv.turn(ids, [text[i] for i in ids])
            replaced = [i for i, (k, x) in zip(ids, res) if k == "block"]
            kept = [i for i, (k, x) in zip(ids, res) if k == "subs"]
            assert replaced == _ids(rest[0]) and kept == _ids(rest[1])


def test_chunking_invariants():
    blocks, _ = W.make_conversation(3, pool_blocks=12)
    for M in (1, 2, 4, 16, 1 << 40):
        for text in blocks.values():
            subs = OD.cdc(text, M)
            assert b"".join(subs) == text and all(subs)
            for s in subs[:-1]:
                assert s.endswith(b"\n")
                last = s[:-1].split(b"\n")[-1]
                assert OD.fnv1a64(last) % M == 0
                # ... and no earlier line of the sub-block is a boundary line
                assert all(OD.fnv1a64(l) % M for l in s[:-1].split(b"\n")[:-1])
            if M == 1:
                assert len(subs) == len(OD.lines_of(text))
    assert OD.cdc(b"", 4) == [] and OD.lines_of(b"x") == [b"x"] and OD.lines_of(b"x\n\ny") == [b"x\n", b"\n", b"y"]


def test_boundaries_are_local():
    """Text inserted in front moves the offsets, not the sub-blocks: the sub-blocks after the
    first boundary of the original are found again unchanged."""
    blocks, _ = W.make_conversation(4, pool_blocks=4)
    text = blocks[1]
    subs = OD.cdc(text, 4)
    assert len(subs) > 3
    shifted = OD.cdc(b"an inserted line\nand another one\n" + text, 4)
    assert shifted[-(len(subs) - 1):] == subs[1:]


def test_rules_of_the_algorithm_by_hand():
    M = 1                                   # every line is a sub-block
    conv = OD.Conversation(M)
    a, b, c = b"x\ny\nx\n", b"y\nz\n", b"q\n"
    r1 = conv.turn([7, 8], [a, b])
    # inside block 7 the repeated "x" is its own, never replaced; block 8's "y" points to 7
    assert r1 == [("subs", [(0, 2, -1), (2, 4, -1), (4, 6, -1)]), ("subs", [(0, 2, 7), (2, 4, -1)])]
    assert OD.kept_bytes(r1) == 8
    # the same id twice in one turn: the seen set grows only after the turn
    r2 = conv.turn([9, 9], [c, c])
    assert r2 == [("subs", [(0, 2, -1)]), ("subs", [(0, 2, -1)])]
    # next turn: 9 and 7 are whole-block references; "z" of a new block points to 8, its first owner
    r3 = conv.turn([9, 5, 7], [c, b"z\nnew\n", a])
    assert r3 == [("block", 9), ("subs", [(0, 2, 8), (2, 6, -1)]), ("block", 7)]


# ---- the C++ library against the oracle ---------------------------------------------------------
def test_hash_and_chunks_match_oracle():
    blocks, _ = W.make_conversation(5, pool_blocks=10)
    for text in list(blocks.values()) + [b"", b"\n", b"no newline", b"\n\n\n"]:
        assert cp.cp_dedup_hash(text) == OD.fnv1a64(text)
        for M in (1, 3, 4, 64):
            want, at = [], 0
            for s in OD.cdc(text, M):
                at += len(s)
                want.append(at)
            assert cp.cp_dedup_chunks(text, M) == want


@pytest.mark.parametrize("seed,M", [(1, 4), (2, 1), (3, 16), (4, 7)])
def test_conversation_matches_oracle_turn_by_turn(seed, M):
    blocks, turns = W.make_conversation(seed)
    ref, lib = OD.Conversation(M), cp.Conversation(M)
    saved = 0
    for ids in turns:
        texts = [blocks[i] for i in ids]
        want = ref.turn(ids, texts)
        got, kept = lib.turn(ids, texts)
        assert got == want
        assert kept == OD.kept_bytes(want)
        saved += sum(len(t) for t in texts) - kept
    assert saved > 0, "the trace has repeated blocks and shared sections"
    lib.close()


def test_through_the_c_abi_paper_example():
    conv = cp.Conversation(8)
    text = {i: (f"block {i} line one\nblock {i} line two\n").encode() for i in range(10)}
    r1, kept1 = conv.turn([1, 2, 4], [text[i] for i in (1, 2, 4)])
    r2, kept2 = conv.turn([1, 5, 2], [text[i] for i in (1, 5, 2)])
    assert [k for k, _ in r1] == ["subs"] * 3 and kept1 == sum(len(text[i]) for i in (1, 2, 4))
    assert [k for k, _ in r2] == ["block", "subs", "block"] and kept2 == len(text[5])
    conv.close()


def test_error_paths_and_unchanged_state_on_small_buffer():
    import ctypes
    lib = cp.load_library()
    h = ctypes.c_void_p()
    assert lib.cp_dedup_create(0, ctypes.byref(h)) == -2
    assert lib.cp_dedup_create(4, None) == -1
    assert lib.cp_dedup_create(1, ctypes.byref(h)) == 0
    data = b"a\nb\nc\n"
    buf = (ctypes.c_uint8 * len(data)).from_buffer_copy(data)
    ids = (ctypes.c_int32 * 1)(3)
    off = (ctypes.c_int64 * 2)(0, len(data))
    ref = (ctypes.c_int32 * 1)()
    subs = (cp.binding.cp_dedup_sub * 3)()
    cnt = ctypes.c_int32(0)
    assert lib.cp_dedup_turn(h, ids, buf, off, 1, ref, subs, 2, ctypes.byref(cnt), None) == -2 and cnt.value == 3
    # nothing was recorded: the same turn with room still sees block 3 as new and keeps all of it
    kept = ctypes.c_int64(0)
    assert lib.cp_dedup_turn(h, ids, buf, off, 1, ref, subs, 3, ctypes.byref(cnt), ctypes.byref(kept)) == 0
    assert ref[0] == 0 and kept.value == len(data) and [subs[i].ref for i in range(3)] == [-1, -1, -1]
    bad = (ctypes.c_int64 * 2)(4, 2)
    assert lib.cp_dedup_turn(h, ids, buf, bad, 1, ref, subs, 3, ctypes.byref(cnt), None) == -2
    assert lib.cp_dedup_turn(None, ids, buf, off, 1, ref, subs, 3, ctypes.byref(cnt), None) == -1
    lib.cp_dedup_free(h)
