// Order in which the workgroups of the weights-in-registers kernels walk the (row tile, channel strip)
// units of a linear: shared by those kernels, each with its own row-tile height.
#pragma once
#include "mfma_linear.hpp"

namespace ptq4vm {
namespace mfma {

// Position in the workgroup's list of units.  An XCD owns a contiguous range of row tiles and all
// strips; its units are ordered band by band (a band = `band_h` consecutive row tiles), inside a
// band strip by strip, inside a strip by row tile.  Consecutive workgroups of an XCD take
// consecutive runs of `band_h` units: in a full band that is one strip of the band each, so the
// workgroups of a band read the same row tiles at about the same time and share them through L2.
struct UnitCursor {
    int band, strip, row, band_rows;
};

struct WorkRange {
    int t_lo, tiles_x, band_h, strips, count;
    UnitCursor start;
};

__device__ __forceinline__ WorkRange work_range(const LinearArgs &p) {
    WorkRange w;
    const int xcd = (int)(blockIdx.x % kXcds), ci = (int)(blockIdx.x / kXcds), per_xcd = (int)(gridDim.x / kXcds);
    w.strips = p.tiles_o;
    w.t_lo = (int)((int64_t)xcd * p.tiles_r / kXcds);
    w.tiles_x = (int)((int64_t)(xcd + 1) * p.tiles_r / kXcds) - w.t_lo;
    const int units = w.strips * w.tiles_x;
    w.band_h = max(1, (units + per_xcd - 1) / per_xcd);
    const int first = ci * w.band_h;
    w.count = max(0, min(w.band_h, units - first));
    const int per_band = w.strips * w.band_h;
    w.start.band = first / per_band;
    const int rem = first - w.start.band * per_band;
    w.start.band_rows = max(1, min(w.band_h, w.tiles_x - w.start.band * w.band_h));
    w.start.strip = rem / w.start.band_rows;
    w.start.row = rem - w.start.strip * w.start.band_rows;
    return w;
}

__device__ __forceinline__ void advance(UnitCursor &c, const WorkRange &w) {
    if (++c.row < c.band_rows) return;
    c.row = 0;
    if (++c.strip < w.strips) return;
    c.strip = 0;
    c.band++;
    c.band_rows = max(1, min(w.band_h, w.tiles_x - c.band * w.band_h));
}

}  // namespace mfma
}  // namespace ptq4vm
