"""Host sweep of the tree-visibility arithmetic the matrix-core attention kernel uses.

The kernel header `csrc/tree_window.h` is plain integer code; it is compiled here for the host and
compared with the definition (a position is visible iff it lies in front of the request's new tokens,
or is new token j with bit j of the row's mask word set) over every offset a tile can have: all row
counts 1..21, every alignment of the new tokens against the 16-token tiles, tiles wholly inside the old
context and the slots behind the last new token in the last cache block.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER_DIR = os.path.join(ROOT, "paper_2604_09562_amd", "csrc")

SHIM = r"""
#define SS_HOST_DEVICE
#include "tree_window.h"
extern "C" unsigned tree_visible4_host(unsigned mask, int rel) { return ss::tree_visible4(mask, rel); }
"""


@pytest.fixture(scope="module")
def shim(tmp_path_factory):
    d = tmp_path_factory.mktemp("tree_window")
    src, so = d / "shim.cpp", d / "shim.so"
    src.write_text(SHIM)
    subprocess.run(["g++", "-O1", "-shared", "-fPIC", "-I", HEADER_DIR, str(src), "-o", str(so)], check=True)
    lib = ctypes.CDLL(str(so))
    lib.tree_visible4_host.restype = ctypes.c_uint32
    lib.tree_visible4_host.argtypes = [ctypes.c_uint32, ctypes.c_int32]
    return lib


def test_every_tile_offset_matches_the_definition(shim):
    rng = np.random.default_rng(0)
    checked = 0
    for q_len in range(1, 22):
        full = (1 << q_len) - 1
        masks = [full, 1, 1 << (q_len - 1), (1 << (q_len - 1)) | 1] + [int(rng.integers(1, full + 1)) for _ in range(6)]
        for ctx in range(0, 80):                      # every ctx % 16, with 0..4 whole tiles of old context
            kv_len = ctx + q_len
            tiles = (kv_len + 15) // 16
            for mask in masks:
                for tok0 in range(0, tiles * 16, 4):  # the first position of each lane group of each tile
                    got = shim.tree_visible4_host(mask, tok0 - ctx)
                    for e in range(4):
                        p = tok0 + e
                        want = p < ctx or (p - ctx < 32 and (mask >> (p - ctx)) & 1 == 1)
                        assert ((got >> e) & 1 == 1) == want, (q_len, ctx, hex(mask), tok0, e)
                        checked += 1
    assert checked > 100000


def test_far_offsets(shim):
    # tiles far in front of the new tokens see everything; offsets at and past the end of the 64-position window nothing
    assert shim.tree_visible4_host(0x1FFFFF, -100000) == 0xF
    assert shim.tree_visible4_host(0x1FFFFF, -33) == 0xF
    for rel in (32, 33, 36, 64, 100000):
        assert shim.tree_visible4_host(0xFFFFFFFF, rel) == 0
    assert shim.tree_visible4_host(0x80000000, 28) == 0x8
    assert shim.tree_visible4_host(0x80000000, 31) == 0x1
