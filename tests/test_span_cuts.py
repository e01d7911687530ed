"""Host check of the span-cut arithmetic shared by the plan kernel and the merge kernel of the attention path.

`csrc/span_cuts.h` is plain integer code.  It is compiled here for the host; for many shapes (tile counts per
request, KV heads, span counts, unit weights) the spans are enumerated the way the plan kernel writes them
(for every unit, the waves whose cut falls into the unit's stretch) and checked against what the streaming
and merge kernels rely on:
  * the spans tile the flat sequence: contiguous, in order, nothing lost, nothing twice;
  * every wave gets its descriptor from exactly one unit, and its span begins inside that unit;
  * the waves that hold tiles of a unit are exactly w_first .. w_last of the merge kernel's formula, so the
    partial slots it reads are the ones that were written (also after the division by four that the
    instances with the in-workgroup hand-over apply);
  * slot `wave + unit` (and `workgroup + unit`) is unique along the sequence.
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
#include "span_cuts.h"
using ss::SpanCuts;
// For every unit (b, g) in order: the waves the plan kernel would describe from it, with their first tile and
// span (x0, x1).  out[w] = {unit, t0, x0, x1}; count[w] = how many units claimed wave w.
extern "C" void plan_spans(const int32_t *prefix, int batch, int hkv, int weight, long long nw, long long *out, int *count)
{
    const SpanCuts c = SpanCuts::make(prefix, batch, hkv, weight, nw);
    for (int b = 0; b < batch; ++b)
        for (int g = 0; g < hkv; ++g) {
            const int n = prefix[b + 1] - prefix[b];
            const long long off = c.unit_offset(b, g), ya = c.unit_coord(b, g);
            const long long w_lo = c.first_cut_at_or_after(ya), w_hi = c.first_cut_at_or_after(ya + weight + n);
            for (long long w = w_lo; w < w_hi && w < nw; ++w) {
                const int t0 = c.first_tile(c.cut(w), ya);
                out[4 * w + 0] = (long long)b * hkv + g;
                out[4 * w + 1] = t0;
                out[4 * w + 2] = off + t0;
                out[4 * w + 3] = c.span_end(w);
                ++count[w];
            }
        }
}
extern "C" void merge_waves(const int32_t *prefix, int batch, int hkv, int weight, long long nw, int *first, int *last)
{
    const SpanCuts c = SpanCuts::make(prefix, batch, hkv, weight, nw);
    for (int b = 0; b < batch; ++b)
        for (int g = 0; g < hkv; ++g)
            c.unit_waves(c.unit_coord(b, g), prefix[b + 1] - prefix[b], first[b * hkv + g], last[b * hkv + g]);
}
"""


@pytest.fixture(scope="module")
def shim(tmp_path_factory):
    d = tmp_path_factory.mktemp("span_cuts")
    src, so = d / "shim.cpp", d / "shim.so"
    src.write_text(SHIM)
    subprocess.run(["g++", "-O1", "-shared", "-fPIC", "-I", HEADER_DIR, str(src), "-o", str(so)], check=True)
    return ctypes.CDLL(str(so))


def _check(shim, tiles, hkv, weight, nw):
    batch = len(tiles)
    prefix = np.concatenate([[0], np.cumsum(tiles)]).astype(np.int32)
    total = int(prefix[-1]) * hkv
    out = np.full((nw, 4), -1, np.int64)
    count = np.zeros(nw, np.int32)
    p = prefix.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    shim.plan_spans(p, batch, hkv, weight, ctypes.c_longlong(nw), out.ctypes.data_as(ctypes.POINTER(ctypes.c_longlong)),
                    count.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    label = (list(map(int, tiles)), hkv, weight, nw)
    assert np.all(count == 1), label                       # every wave is described exactly once
    x0, x1 = out[:, 2], out[:, 3]
    assert x0[0] == 0 and x1[-1] == total, label
    assert np.all(x1[:-1] == x0[1:]), label                # contiguous, in order
    assert np.all(x1 >= x0), label
    # the span begins inside the unit that described it (or is empty and sits at that unit's start)
    unit_off = np.array([int(prefix[b]) * hkv + g * int(tiles[b]) for b in range(batch) for g in range(hkv)], np.int64)
    unit_n = np.array([int(tiles[b]) for b in range(batch) for _ in range(hkv)], np.int64)
    u = out[:, 0]
    assert np.all((x0 >= unit_off[u]) & (x0 < unit_off[u] + unit_n[u])), label
    assert np.all(out[:, 1] == x0 - unit_off[u]), label
    # which waves hold tiles of each unit, from the spans themselves
    first = np.zeros(batch * hkv, np.int32)
    last = np.zeros(batch * hkv, np.int32)
    shim.merge_waves(p, batch, hkv, weight, ctypes.c_longlong(nw), first.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                     last.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    slots, wg_slots = set(), set()
    for unit in range(batch * hkv):
        lo, hi = unit_off[unit], unit_off[unit] + unit_n[unit]
        holders = [w for w in range(nw) if max(x0[w], lo) < min(x1[w], hi)]
        assert holders == list(range(first[unit], last[unit] + 1)), (label, unit, holders, int(first[unit]), int(last[unit]))
        for w in holders:
            assert (w + unit) not in slots, (label, unit, w)
            slots.add(w + unit)
        for wg in sorted({w // 4 for w in holders}):
            assert (wg + unit) not in wg_slots, (label, unit, wg)
            wg_slots.add(wg + unit)
        # a unit whose holders share one workgroup is finished inside the streaming kernel: the merge kernel skips it
        assert (first[unit] // 4 == last[unit] // 4) == (len({w // 4 for w in holders}) == 1)


def test_small_shapes_exhaustively(shim):
    n = 0
    for hkv in (1, 2):
        for weight in (0, 1, 3, 7):
            for tiles in ([1], [5], [1, 1], [1, 4], [3, 1, 2], [2, 2, 2, 2], [1, 9, 1], [6, 1, 1, 1, 5]):
                total = sum(tiles) * hkv
                for nw in range(1, total + 1):          # never more spans than tiles (the plan keeps >= 1 tile per wave on average)
                    _check(shim, np.array(tiles), hkv, weight, nw)
                    n += 1
    assert n > 500


def test_random_shapes(shim):
    rng = np.random.default_rng(1)
    for _ in range(300):
        batch = int(rng.integers(1, 40))
        hkv = int(rng.choice([1, 2, 4, 8]))
        kind = rng.integers(0, 3)
        if kind == 0:
            tiles = rng.integers(1, 6, batch)                       # many short units
        elif kind == 1:
            tiles = np.exp(rng.uniform(0, np.log(600), batch)).astype(np.int64) + 1   # ragged
        else:
            tiles = rng.integers(200, 1200, batch)                  # long
        total = int(tiles.sum()) * hkv
        weight = int(rng.choice([0, 1, 3, 4, 17, 64]))
        nw_max = max(1, total // 4)                                 # the plan kernel's bound: at least 4 tiles per span on average
        nw = int(min(nw_max, rng.choice([1, 4, 8, 64, 256, 1024])))
        nw = max(4 * (nw // 4), 1) if nw >= 4 else nw
        _check(shim, tiles, hkv, weight, nw)


def test_bench_workload_shape(shim):
    # configs[1]: 64 requests, contexts uniform on [256, 4096] + 5 new tokens, 8 KV heads, 1024 spans, default weight
    rng = np.random.default_rng(2)
    tiles = (rng.integers(256, 4097, 64) + 5 + 15) // 16
    _check(shim, tiles, 8, 3, 1024)
