// Where the flat KV tile sequence is cut into the spans of the streaming attention kernel.
//
// The tiles of all (request, KV head) units lie end to end, unit major: request b contributes hkv units of
// n_b tiles each.  Spans are equal in a "weighted" coordinate in which every unit is preceded by `weight`
// virtual tiles (what opening a unit costs a wavefront): unit u = b * hkv + g occupies the stretch
// [ya, ya + weight + n_b), ya = (flat index of its first tile) + weight * u, and wave w starts at the cut
// w * total_w / nw.  A cut inside a unit's virtual part starts the span at the unit's first tile.  The plan
// kernel (which writes the spans) and the merge kernel (which has to know which waves hold a part of a unit)
// both use the functions below; plain integer code with no device dependency, so that a host test can check
// them against each other over many shapes.
#pragma once

#include <stdint.h>

#ifndef SS_HOST_DEVICE
#define SS_HOST_DEVICE __host__ __device__
#endif

namespace ss {

struct SpanCuts {
    const int32_t *prefix;   // [batch + 1] exclusive prefix of the tiles per KV head of the requests
    int batch, hkv, weight;
    long long total;         // tiles of all units
    long long total_w;       // tiles of all units plus `weight` per unit
    long long nw;            // number of spans

    SS_HOST_DEVICE static SpanCuts make(const int32_t *prefix, int batch, int hkv, int weight, long long nw)
    {
        SpanCuts c;
        c.prefix = prefix;
        c.batch = batch;
        c.hkv = hkv;
        c.weight = weight;
        c.total = (long long)prefix[batch] * hkv;
        c.total_w = c.total + (long long)weight * batch * hkv;
        c.nw = nw;
        return c;
    }
    // weighted coordinate of wave w's cut
    SS_HOST_DEVICE long long cut(long long w) const { return w * total_w / nw; }
    // flat index of unit (b, g)'s first tile, and the weighted coordinate where its stretch begins
    SS_HOST_DEVICE long long unit_offset(int b, int g) const
    {
        return (long long)prefix[b] * hkv + (long long)g * (prefix[b + 1] - prefix[b]);
    }
    SS_HOST_DEVICE long long unit_coord(int b, int g) const { return unit_offset(b, g) + (long long)weight * ((long long)b * hkv + g); }
    // the waves whose cut falls into the stretch [ya, ya + weight + n): w_lo <= w < w_hi (w_hi may exceed nw)
    SS_HOST_DEVICE long long first_cut_at_or_after(long long y) const { return (y * nw + total_w - 1) / total_w; }
    // tile of the unit at which a span begins whose cut lies `ya <= cut < ya + weight + n`
    SS_HOST_DEVICE int first_tile(long long cut_y, long long ya) const
    {
        const long long in_unit = cut_y - ya - weight;
        return in_unit > 0 ? (int)in_unit : 0;
    }
    // unit and tile that weighted coordinate y (< total_w) falls on; returns the flat tile index
    SS_HOST_DEVICE long long locate(long long y, int &b, int &g, int &tile) const
    {
        int lo = 0, hi = batch - 1;   // last request whose first unit starts at or before y
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (((long long)prefix[mid] + (long long)weight * mid) * hkv <= y)
                lo = mid;
            else
                hi = mid - 1;
        }
        b = lo;
        const int n = prefix[b + 1] - prefix[b];
        const long long r = y - ((long long)prefix[b] + (long long)weight * b) * hkv;
        g = (int)(r / (n + weight));
        const int in_unit = (int)(r - (long long)g * (n + weight)) - weight;
        tile = in_unit > 0 ? in_unit : 0;
        return (long long)prefix[b] * hkv + (long long)g * n + tile;
    }
    // flat index one past wave w's last tile
    SS_HOST_DEVICE long long span_end(long long w) const
    {
        if (w + 1 >= nw) return total;
        if (weight == 0) return (w + 1) * total / nw;
        int b, g, t;
        return locate(cut(w + 1), b, g, t);
    }
    // The waves that hold tiles of a unit with n >= 1 tiles whose stretch begins at ya: the last wave whose cut
    // lies at or before the unit's first tile ... the last wave whose cut lies at or before its last tile.
    SS_HOST_DEVICE void unit_waves(long long ya, int n, int &w_first, int &w_last) const
    {
        w_first = (int)(((ya + weight + 1) * nw - 1) / total_w);
        w_last = (int)(((ya + weight + n) * nw - 1) / total_w);
    }
};

}  // namespace ss
