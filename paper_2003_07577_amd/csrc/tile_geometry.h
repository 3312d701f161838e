// Host-side geometry of the tiled convolution (plain C++, no HIP): how many
// padded input positions a tile of consecutive output positions can touch.
//
// Output positions are numbered t = (n*OH + oh)*OW + ow.  The packed
// activations are stored with a zero border of `border` positions around every
// image, i.e. as one flat array of positions u = (n*Hp + hp)*Wp + wp with
// Hp = H + 2*border, Wp = W + 2*border.  With pad <= border, output t reads,
// for filter tap (r, s), position base(t) + r*Wp + s where
// base(t) = (n*Hp + oh*stride + border - pad)*Wp + ow*stride + border - pad.
// base() is non-decreasing in t, so a tile of consecutive outputs touches one
// contiguous range of u, and no tap of a valid output leaves the array.
#pragma once

namespace ebs {

struct TileGeom {
    int H, W, R, S, stride, pad, OH, OW, border;
    int Hp() const { return H + 2 * border; }
    int Wp() const { return W + 2 * border; }
    long long base(long long t) const
    {
        long long ow = t % OW;
        long long oh = (t / OW) % OH;
        long long n = t / ((long long)OW * OH);
        return (n * Hp() + oh * stride + border - pad) * Wp() + ow * stride + border - pad;
    }
    // Exact extent (number of positions u) touched by outputs [t0, t1].
    long long extent(long long t0, long long t1) const
    {
        return base(t1) + (long long)(R - 1) * Wp() + (S - 1) - base(t0) + 1;
    }
    // Upper bound of extent() over every tile of `tp` consecutive outputs.
    long long extent_bound(long long tp) const
    {
        if (tp < 1) tp = 1;
        long long steps = tp - 1;
        long long row_wraps = (steps + OW - 1) / OW;
        long long img_wraps = (steps + (long long)OW * OH - 1) / ((long long)OW * OH);
        long long row_extra = (long long)stride * (Wp() - OW);            // >= 0
        long long img_extra = (long long)Wp() * (Hp() - (long long)OH * stride);
        if (row_extra < 0) row_extra = 0;
        if (img_extra < 0) img_extra = 0;
        return steps * stride + row_wraps * row_extra + img_wraps * img_extra
             + (long long)(R - 1) * Wp() + S;
    }
};

}  // namespace ebs
