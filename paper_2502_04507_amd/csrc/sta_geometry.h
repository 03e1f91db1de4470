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

// The transposed question, needed when gradients are accumulated per key tile: which query tiles keep key
// tile k?  Along one axis the window centre c(q) is q clamped into [half, n-1-half]; k is kept when
// |c(q) - k| <= half.  The centres that qualify form the interval [max(half, k-half), min(n-1-half, k+half)];
// every q below `half` shares the centre `half` and every q above n-1-half shares n-1-half, so the interval is
// widened to the border on the side where it reaches the clamp value.  If the window covers the axis
// (n-1-half < half) every query tile keeps every key tile.
STA_HD StaAxisRange sta_axis_query_range(int n, int w, int k)
{
    const int half = w >> 1;
    StaAxisRange r;
    if (n - 1 - half < half) {
        r.lo = 0;
        r.hi = n - 1;
        return r;
    }
    const int c0 = (k - half) > half ? (k - half) : half;
    const int c1 = (k + half) < (n - 1 - half) ? (k + half) : (n - 1 - half);
    r.lo = c0 == half ? 0 : c0;
    r.hi = c1 == (n - 1 - half) ? (n - 1) : c1;
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

// Query tiles that keep key tile k_tile (a box as well, not symmetric to the key-tile box at the borders).
STA_HD StaBox sta_query_tile_box_of(int nt, int nh, int nw, int wt, int wh, int ww, int k_tile)
{
    const int kw = k_tile % nw;
    const int kh = (k_tile / nw) % nh;
    const int kt = k_tile / (nw * nh);
    StaBox b;
    b.t = sta_axis_query_range(nt, wt, kt);
    b.h = sta_axis_query_range(nh, wh, kh);
    b.w = sta_axis_query_range(nw, ww, kw);
    return b;
}
