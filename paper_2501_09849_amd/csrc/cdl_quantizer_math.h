// Device-side arithmetic of the probabilistic quantizer shared by the quantizer kernels and by the backward
// product that applies the quantizer's backward pass in its epilogue (not installed).
//
// The conditional PMF of one entry theta over the levels i*delta is softmax_i(-alpha (theta - i delta)^2)
// (eq. CPMF, Sec. III-A).  With c a level next to theta, u = theta - c*delta and kappa = alpha*delta^2, the weight
// of level c+j relative to level c is w_j = exp(alpha*delta * j * (2u - j*delta)); only a band of W levels on
// each side of c carries weight above fp32 resolution, W depends on kappa alone.  Moments are taken of j.
#pragma once

#include "cdl_internal.h"

#include <math.h>

namespace cdl {

struct QConst {
    float delta;
    float inv_delta;
    float c1;         // alpha * delta * log2(e): base-2 exponent per unit of j*(2u - j delta)
    float b2;         // 2 alpha delta log2(e): t = exp2(b2 u)
    float k1, k4;     // exp(-kappa), exp(-4 kappa)
    float two_kappa;  // 2 alpha delta^2
    float lo_f;
    float hi_f;
    int lo;
    int n_levels;
    int idx_off;      // what is subtracted from a level index before it is stored as an int8 (0, or 128 for sets that reach beyond 127)
    int wgen;         // band half-width of the generic kernel
    int stream;       // 1: the tensor is large, read and write it with non-temporal accesses
    int slide;        // 1: truncated CPMF - the band of 2 wgen + 1 levels slides at the ends of the level set instead of being cut
    float r_clamp;    // |u / delta| beyond which the W = 2 kernels hold the offset fixed (see band_weights), else infinity
};

// Four level indices as the four int8 of one word, each stored as index - off
__device__ __forceinline__ uint32_t pack_indices(int c0, int c1, int c2, int c3, int off)
{
    return (uint32_t)((c0 - off) & 0xff) | ((uint32_t)((c1 - off) & 0xff) << 8) |
           ((uint32_t)((c2 - off) & 0xff) << 16) | ((uint32_t)((c3 - off) & 0xff) << 24);
}

__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float clampf(float x, float lo, float hi) { return __builtin_amdgcn_fmed3f(x, lo, hi); }

// Level next to th.  EXACT: the nearest level, lower index on an exact tie, clamped to [lo, hi]:
// rint(th/delta) can be off by one next to a midpoint; the two fused multiply-adds evaluate
// 2 th - (2r +- 1) delta with a single rounding, so their signs are those of the exact values.
// Not EXACT: rint(th/delta) clamped - within 2e-5 of a midpoint it may pick the other neighbour,
// which changes no moment (the band is centred one level off, u is a hair above delta/2).
template <bool EXACT>
__device__ __forceinline__ float anchor_level(float th, const QConst &k)
{
    float r = rintf(th * k.inv_delta);
    if (EXACT) {
        const float two_th = 2.0f * th;
        const float up = fmaf(-(2.0f * r + 1.0f), k.delta, two_th);  // > 0: r+1 is strictly closer
        const float dn = fmaf(-(2.0f * r - 1.0f), k.delta, two_th);  // <= 0: r-1 is at least as close
        const float r_up = r + 1.0f, r_dn = r - 1.0f;
        r = (up > 0.0f) ? r_up : r;
        r = (dn <= 0.0f) ? r_dn : r;
    }
    return clampf(r, k.lo_f, k.hi_f);
}

// Weights of the band (up to one common factor) and their power sums in the offset j.
template <int W>
struct Band {
    float cf;          // anchor level as a float
    float u;           // theta - c*delta
    float ctr;         // weight of the anchor level
    float up[W > 0 ? W : 1];   // weight of level c+j at [j-1]
    float dn[W > 0 ? W : 1];   // weight of level c-j at [j-1]
    float Z, S1, S2, S3;
};

// NMOM: how many of S1, S2, S3 are needed.
template <int W, bool EXACT, int NMOM>
__device__ __forceinline__ void band_weights(float th, const QConst &k, Band<W> &b)
{
    const float cf = anchor_level<EXACT>(th, k);
    b.cf = cf;
    if (W == 2) {
        // t = exp(2 alpha delta u), clamped where the far side has long vanished so that t^4 stays finite.
        // Beyond the clamp (theta more than 30 / (2 kappa log2 e) steps outside the level set) the near
        // neighbour keeps a weight of 2^-30 e^-kappa where the true one goes on falling: harmless by itself,
        // but not once it is multiplied by an offset that goes on growing - the scalar gradients therefore
        // hold u / delta at k.r_clamp there, which bounds that product by 3e-11.
        const float u = fmaf(-cf, k.delta, th);
        b.u = u;
        const float t = fast_exp2(clampf(k.b2 * u, -30.0f, 30.0f));
        const float t2 = t * t, t3 = t2 * t, t4 = t2 * t2;
        const float above = k.hi_f - cf, below = cf - k.lo_f;   // levels that exist on each side
        const float k1u = (above >= 1.0f) ? k.k1 : 0.0f, k4u = (above >= 2.0f) ? k.k4 : 0.0f;
        const float k1d = (below >= 1.0f) ? k.k1 : 0.0f, k4d = (below >= 2.0f) ? k.k4 : 0.0f;
        const float A = k4u * t4, B = k1u * t3, C = k1d * t, D = k4d;   // levels +2, +1, -1, -2 (times t^2)
        const float p = A + D, q = B + C, x = A - D, y = B - C;
        b.ctr = t2;
        b.up[0] = B; b.up[1] = A; b.dn[0] = C; b.dn[1] = D;
        b.Z = (p + q) + t2;
        b.S1 = fmaf(2.0f, x, y);
        b.S2 = (NMOM >= 2) ? fmaf(4.0f, p, q) : 0.0f;
        b.S3 = (NMOM >= 3) ? fmaf(8.0f, x, y) : 0.0f;
        return;
    }
    float two_u, corr;
    if (W == 1) {
        // Sharp regime: the exponent of the neighbour next to a midpoint is a small difference
        // scaled by a large kappa.  c*delta is split into its rounded product and the exact
        // remainder so that 2u -+ delta loses nothing when it cancels.
        const float p_hi = cf * k.delta;
        const float p_lo = fmaf(cf, k.delta, -p_hi);
        const float u_hi = th - p_hi;
        two_u = 2.0f * u_hi;
        corr = 2.0f * p_lo;
        b.u = u_hi - p_lo;
    } else {
        b.u = fmaf(-cf, k.delta, th);
        two_u = 2.0f * b.u;
        corr = 0.0f;
    }
    const float above = k.hi_f - cf, below = cf - k.lo_f;
    float Z = 1.0f, S1 = 0.0f, S2 = 0.0f, S3 = 0.0f;
#pragma unroll
    for (int j = 1; j <= W; ++j) {
        const float jf = (float)j;
        const float cj = k.c1 * jf;
        float xu = fmaf(-jf, k.delta, two_u);   // 2u - j delta
        float xd = fmaf(jf, k.delta, two_u);    // 2u + j delta
        if (W == 1) { xu -= corr; xd -= corr; }
        float wu = fast_exp2(cj * xu);
        float wd = fast_exp2(-cj * xd);
        wu = (above >= jf) ? wu : 0.0f;   // level c+j exists
        wd = (below >= jf) ? wd : 0.0f;   // level c-j exists
        b.up[j - 1] = wu;
        b.dn[j - 1] = wd;
        const float s = wu + wd, d = wu - wd;
        Z += s;
        S1 = fmaf(jf, d, S1);
        if (NMOM >= 2) S2 = fmaf(jf * jf, s, S2);
        if (NMOM >= 3) S3 = fmaf(jf * jf * jf, d, S3);
    }
    b.ctr = 1.0f;
    b.Z = Z; b.S1 = S1; b.S2 = S2; b.S3 = S3;
}

// Generic band of run-time half-width (soft regime, many live levels): one exp per level.
struct GenericSums {
    float cf, u, Z, S1, S2, S3;
    int jlo, jhi;
};

__device__ __forceinline__ float generic_weight(int j, float two_u, const QConst &k)
{
    const float jf = (float)j;
    return fast_exp2(k.c1 * jf * fmaf(-jf, k.delta, two_u));
}

// Offsets (relative to the nearest level c) of the levels the generic kernels visit.  Full CPMF: the band
// c-wgen..c+wgen cut at the ends of the set.  Truncated CPMF (Sec. V-B: the top 2 wgen + 1 values, which are
// the nearest ones): the same band, slid inwards at the ends so that it always holds 2 wgen + 1 levels.
__device__ __forceinline__ void generic_window(int c, const QConst &k, int &jlo, int &jhi)
{
    const int hi = k.lo + k.n_levels - 1;
    if (k.slide) {
        const int centre = min(max(c, k.lo + k.wgen), hi - k.wgen);   // host guarantees n_levels >= 2 wgen + 1
        jlo = centre - k.wgen - c;
        jhi = centre + k.wgen - c;
    } else {
        jlo = max(k.lo - c, -k.wgen);
        jhi = min(hi - c, k.wgen);
    }
}

template <bool EXACT>
__device__ __forceinline__ void generic_sums(float th, const QConst &k, GenericSums &g)
{
    // (with a truncated CPMF the kept levels change at the midpoints, so the nearest level has to be exact)
    const float cf = k.slide ? anchor_level<true>(th, k) : anchor_level<EXACT>(th, k);
    g.cf = cf;
    g.u = fmaf(-cf, k.delta, th);
    const int c = (int)cf;
    generic_window(c, k, g.jlo, g.jhi);
    const float two_u = 2.0f * g.u;
    float Z = 0.0f, S1 = 0.0f, S2 = 0.0f, S3 = 0.0f;
    for (int j = g.jlo; j <= g.jhi; ++j) {
        const float jf = (float)j;
        const float w = generic_weight(j, two_u, k);
        Z += w;
        S1 = fmaf(jf, w, S1);
        S2 = fmaf(jf * jf, w, S2);
        S3 = fmaf(jf * jf * jf, w, S3);
    }
    g.Z = Z; g.S1 = S1; g.S2 = S2; g.S3 = S3;
}

// One entry of the quantizer's backward pass (Lemma 1 in offsets from the anchor level): with mu, var, c3 the mean,
// variance and third central moment of the level offset j under the CPMF and r = u / delta,
//     dQd/dtheta = 2 kappa var,   dQd/ddelta = (c + mu) + 2 kappa ((r - c - 2 mu) var - c3),   dQd/dalpha / delta^3 = 2 (r - mu) var - c3.
// W: band half-width of the unrolled kernels, 0 = the generic loop.  SCALARS: also the last two.
template <int W, bool SCALARS>
__device__ __forceinline__ void quantizer_bwd_terms(float th, const QConst &k, float &d_theta, float &t_d, float &t_a)
{
    float cf, u, Z, S1, S2, S3;
    if (W > 0) {
        Band<W> b;
        band_weights<W, false, SCALARS ? 3 : 2>(th, k, b);
        cf = b.cf; u = b.u; Z = b.Z; S1 = b.S1; S2 = b.S2; S3 = b.S3;
    } else {
        GenericSums s;
        generic_sums<false>(th, k, s);
        cf = s.cf; u = s.u; Z = s.Z; S1 = s.S1; S2 = s.S2; S3 = s.S3;
    }
    const float inv = fast_rcp(Z);
    const float mu = S1 * inv, m2 = S2 * inv;
    const float var = fmaf(-mu, mu, m2);
    d_theta = k.two_kappa * var;
    t_d = 0.0f;
    t_a = 0.0f;
    if (SCALARS) {
        const float m3 = S3 * inv;
        const float c3 = fmaf(-mu, fmaf(-2.0f * mu, mu, 3.0f * m2), m3);   // m3 - 3 mu m2 + 2 mu^3
        const float r = clampf(u * k.inv_delta, -k.r_clamp, k.r_clamp);
        t_d = (cf + mu) + k.two_kappa * fmaf(r - cf - 2.0f * mu, var, -c3);
        t_a = fmaf(2.0f * (r - mu), var, -c3);
    }
}

// Launch constants of a quantizer, and which unrolled band kernel serves them (0: the generic loop).
QConst make_const(const cdl_qparams &p);
int band_template(const QConst &k);

}  // namespace cdl
