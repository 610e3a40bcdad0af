// Pieces shared by the sub-bit convolution kernels (device side, gfx950).
#pragma once

#include "snn_internal.h"

namespace snn {

// Where one output pixel's 3x3 window sits in the row-packed input
// (uint32 [N][C][H][WW], bit (w % 32) of word (w / 32)).
struct PixGeom {
    int n;             // image
    int rowoff[3];     // h * WW of the three window rows (0 if the row is outside the image)
    uint32_t rowmask;  // bit dy set if window row dy is inside the image
    int j;             // word holding column wc - 1 (0 if wc == 0)
    int sh;            // bit of column wc - 1 in that word, or -1 if wc == 0
    bool need_hi;      // the three columns straddle two words
    uint32_t colmask;  // 3-bit mask of the window columns inside the image
};

__device__ inline PixGeom pix_geom(int64_t p, const Geom &g)
{
    PixGeom q;
    if (p >= g.P) p = g.P - 1;
    q.n = (int)(p / g.HoWo);
    const int r = (int)(p - (int64_t)q.n * g.HoWo);
    const int ho = r / g.Wo, wo = r - ho * g.Wo;
    const int hc = ho * g.stride, wc = wo * g.stride;
    q.rowmask = 0;
#pragma unroll
    for (int dy = 0; dy < 3; ++dy) {
        const int h = hc + dy - 1;
        const bool ok = h >= 0 && h < g.H;
        q.rowoff[dy] = ok ? h * g.WW : 0;
        q.rowmask |= ok ? (1u << dy) : 0u;
    }
    const int c = wc - 1;
    q.j = c >= 0 ? (c >> 5) : 0;
    q.sh = c >= 0 ? (c & 31) : -1;
    q.need_hi = q.sh > 29 && q.j + 1 < g.WW;
    q.colmask = (wc > 0 ? 1u : 0u) | 2u | (wc + 1 < g.W ? 4u : 0u);
    return q;
}

// The raw words one window needs: issued early, consumed later (software pipelining).
struct RawWin {
    uint32_t lo[3], hi[3];
};

__device__ inline RawWin window_load(const uint32_t *__restrict__ x, const PixGeom &q, int ci, const Geom &g)
{
    const uint32_t *plane = x + ((int64_t)q.n * g.C_in + ci) * ((int64_t)g.H * g.WW);
    RawWin r;
#pragma unroll
    for (int dy = 0; dy < 3; ++dy) {
        const uint32_t *row = plane + q.rowoff[dy];
        r.lo[dy] = row[q.j];
        r.hi[dy] = q.need_hi ? row[q.j + 1] : 0u;
    }
    return r;
}

// 9-bit window: bit (3*dy + dx) = sign bit of x[h+dy-1][w+dx-1], 0 outside the image.
__device__ inline uint32_t window_extract(const RawWin &r, const PixGeom &q)
{
    uint32_t win = 0;
#pragma unroll
    for (int dy = 0; dy < 3; ++dy) {
        const unsigned long long v = ((unsigned long long)r.hi[dy] << 32) | r.lo[dy];
        uint32_t b3 = q.sh >= 0 ? (uint32_t)(v >> q.sh) : (r.lo[dy] << 1);
        b3 &= q.colmask;
        if (!((q.rowmask >> dy) & 1u)) b3 = 0;
        win |= b3 << (3 * dy);
    }
    return win;
}

__device__ inline uint32_t window9(const uint32_t *__restrict__ x, const PixGeom &q, int ci, const Geom &g)
{
    return window_extract(window_load(x, q, ci, g), q);
}

}  // namespace snn
