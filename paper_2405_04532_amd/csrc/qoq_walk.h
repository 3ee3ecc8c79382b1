// Iteration structure of a workgroup's run of work units in the streaming kernel (internal to the library).
//
// Work unit u = block * G + g (64-channel block, quantization group).  A workgroup is dealt the contiguous
// run [u0, u1).  It walks the run R units per iteration (one per wave); an iteration never straddles a block
// boundary or the end of the run, so the run is a sequence of segments (the tail of a first block, whole
// blocks, the head of a last block), each ending with a possibly short iteration.  The closed form below gives,
// for any iteration index, the block, the first group, the number of units and whether the iteration ends a
// segment, so that an iteration can be looked up ahead of time without stepping a state machine.
#pragma once
#include "qoq_layout.h"

namespace qoq {

struct RunShape {
    int G;          // groups per block
    int R;          // units per iteration
    int b0, g0;     // first unit: block, group
    int len0;       // units of the first segment
    int it0;        // iterations of the first segment
    int itG;        // iterations of a whole block = ceil(G / R)
    int full;       // whole blocks after the first segment
    int last_len;   // units of the last (partial) segment, 0 if none
    int T;          // iterations in total
};

QOQ_HD RunShape make_run(int u0, int u1, int G, int R)
{
    RunShape r;
    const int U = u1 - u0;
    r.G = G;
    r.R = R;
    r.b0 = u0 / G;
    r.g0 = u0 - r.b0 * G;
    r.len0 = (G - r.g0) < U ? (G - r.g0) : U;
    r.it0 = (r.len0 + R - 1) / R;
    r.itG = (G + R - 1) / R;
    const int rest = U - r.len0;
    r.full = rest / G;
    r.last_len = rest - r.full * G;
    r.T = r.it0 + r.full * r.itG + (r.last_len + R - 1) / R;
    return r;
}

struct IterInfo {
    int block, g, n;      // block, first group, units (1 .. R)
    bool seg_end;         // last iteration of its segment
    bool complete;        // ... and the segment is a whole block (starts at group 0, reaches group G)
};

// it in [0, T)
QOQ_HD IterInfo run_iteration(const RunShape& r, int it)
{
    int block, g, seg_g0, seg_len;
    if (it < r.it0) {
        block = r.b0; seg_g0 = r.g0; seg_len = r.len0; g = r.g0 + r.R * it;
    } else {
        const int k = it - r.it0;
        const int whole = r.full * r.itG;
        if (k < whole) {
            const int q = k / r.itG;
            block = r.b0 + 1 + q; seg_g0 = 0; seg_len = r.G; g = r.R * (k - q * r.itG);
        } else {
            block = r.b0 + 1 + r.full; seg_g0 = 0; seg_len = r.last_len; g = r.R * (k - whole);
        }
    }
    IterInfo o;
    const int left = seg_g0 + seg_len - g;
    o.block = block;
    o.g = g;
    o.n = left < r.R ? left : r.R;
    o.seg_end = g + o.n == seg_g0 + seg_len;
    o.complete = o.seg_end && seg_g0 == 0 && g + o.n >= r.G;
    return o;
}

}  // namespace qoq
