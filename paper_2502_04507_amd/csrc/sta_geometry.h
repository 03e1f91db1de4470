// Key-tile window geometry of Sliding Tile Attention, in tile units.
//
// Follows the window-centre and distance test of the appendix algorithm
// "Mask Definition of 3D STA": along each axis the window centre is the query
// tile clamped into [half, n-1-half] (the upper clamp first, the lower clamp
// last), half = floor(window/2), and a key tile is kept when its distance to
// the centre is at most half.  The kept key tiles of a query tile therefore
// form an axis-aligned box, which is all the attention kernel needs: no mask
// is ever materialised.
#pragma once

#if defined(__HIPCC__)
#define STA_HD __host__ __device__ __forceinline__
#else
#define STA_HD inline
#endif

struct StaAxisRange {
    int lo;   // first kept key tile (inclusive)
    int hi;   // last kept key tile (inclusive)
};

// n: tiles along the axis, w: window size in tiles (>= 1), q: query tile.
STA_HD StaAxisRange sta_axis_range(int n, int w, int q)
{
    const int half = w >> 1;
    int c = q < (n - 1 - half) ? q : (n - 1 - half);
    c = c > half ? c : half;
    StaAxisRange r;
    r.lo = (c - half) > 0 ? (c - half) : 0;
    r.hi = (c + half) < (n - 1) ? (c + half) : (n - 1);
    return r;
}

struct StaBox {
    StaAxisRange t, h, w;
    STA_HD int count() const { return (t.hi - t.lo + 1) * (h.hi - h.lo + 1) * (w.hi - w.lo + 1); }
};

// nt/nh/nw: tile grid; wt/wh/ww: window in tiles; q_tile: row-major query tile id.
STA_HD StaBox sta_key_tile_box_of(int nt, int nh, int nw, int wt, int wh, int ww, int q_tile)
{
    const int qw = q_tile % nw;
    const int qh = (q_tile / nw) % nh;
    const int qt = q_tile / (nw * nh);
    StaBox b;
    b.t = sta_axis_range(nt, wt, qt);
    b.h = sta_axis_range(nh, wh, qh);
    b.w = sta_axis_range(nw, ww, qw);
    return b;
}
