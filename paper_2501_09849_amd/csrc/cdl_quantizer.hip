// Probabilistic quantizer of CDL on gfx950: forward (hard index, soft value, marginal PMF,
// entropy) and analytic backward (Lemma 1) as single-pass streaming kernels.
//
// The conditional PMF of one entry theta over the levels i*delta is
//     P_i = softmax_i(-alpha (theta - i delta)^2)                       (eq. CPMF, Sec. III-A).
// Let c be the level nearest to theta (clamped to the set), u = theta - c*delta and
// kappa = alpha*delta^2.  Relative to level c the weight of level c+j is
//     w_j = exp(alpha*delta * j * (2u - j*delta)),          w_0 = 1,
// which is exp(-kappa j^2 + 2 alpha delta u j) written so that nothing large cancels.  For
// |u| <= delta/2 it is at most exp(-kappa |j| (|j|-1)), so only a band of W levels on each side
// of c carries weight above fp32 resolution; W depends on kappa alone and is fixed per launch.
// All moments are taken of the offset j, which keeps fp32 free of the cancellation that raw
// powers of the index would suffer:
//     Q_d = delta (c + mu),  Var = delta^2 var_j,  third central moment = delta^3 c3_j.
// Lemma 1 in these terms (Skew_u = c3 + 2 E Var):
//     dQd/dtheta = 2 kappa var_j
//     dQd/ddelta = (c + mu) + 2 kappa ((r - c - 2 mu) var_j - c3_j),   r = u/delta
//     dQd/dalpha = delta^3 (2 (r - mu) var_j - c3_j)
#include "cdl_internal.h"

#include <math.h>

namespace cdl {

namespace {


struct QConst {
    float delta;
    float inv_delta;
    float c1;         // alpha * delta * log2(e): base-2 exponent per unit of j*(2u - j delta)
    float two_kappa;  // 2 alpha delta^2
    float lo_f;
    float hi_f;
    int lo;
    int n_levels;
    int wgen;         // band half-width of the generic kernel
};

// Nearest level to th, lower index on an exact tie, clamped to [lo, hi].
// rint(th/delta) can be off by one next to a midpoint; the two fused multiply-adds evaluate
// 2 th - (2r +- 1) delta with a single rounding, so their signs are those of the exact values.
__device__ __forceinline__ float nearest_level(float th, const QConst &k)
{
    float r = rintf(th * k.inv_delta);
    r = fminf(fmaxf(r, k.lo_f), k.hi_f);
    const float two_th = 2.0f * th;
    const float up = fmaf(-(2.0f * r + 1.0f), k.delta, two_th);  // > 0: r+1 is strictly closer
    const float dn = fmaf(-(2.0f * r - 1.0f), k.delta, two_th);  // <= 0: r-1 is at least as close
    r = (up > 0.0f) ? r + 1.0f : r;
    r = (dn <= 0.0f) ? r - 1.0f : r;
    return fminf(fmaxf(r, k.lo_f), k.hi_f);
}

// Weights of the band around the nearest level and their power sums in the offset j.
template <int W>
struct Band {
    float cf;          // nearest level as a float
    float u;           // theta - c*delta
    float up[W > 0 ? W : 1];
    float dn[W > 0 ? W : 1];
    float Z, S1, S2, S3;
};

template <int W, bool THIRD>
__device__ __forceinline__ void band_weights(float th, const QConst &k, Band<W> &b)
{
    const float cf = nearest_level(th, k);
    b.cf = cf;
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
    float Z = 1.0f, S1 = 0.0f, S2 = 0.0f, S3 = 0.0f;
#pragma unroll
    for (int j = 1; j <= W; ++j) {
        const float jf = (float)j;
        const float cj = k.c1 * jf;
        float xu = fmaf(-jf, k.delta, two_u);   // 2u - j delta
        float xd = fmaf(jf, k.delta, two_u);    // 2u + j delta
        if (W == 1) { xu -= corr; xd -= corr; }
        float wu = __builtin_amdgcn_exp2f(cj * xu);
        float wd = __builtin_amdgcn_exp2f(-cj * xd);
        wu = (cf + jf <= k.hi_f) ? wu : 0.0f;   // level c+j exists
        wd = (cf - jf >= k.lo_f) ? wd : 0.0f;   // level c-j exists
        b.up[j - 1] = wu;
        b.dn[j - 1] = wd;
        const float s = wu + wd, d = wu - wd;
        Z += s;
        S1 = fmaf(jf, d, S1);
        S2 = fmaf(jf * jf, s, S2);
        if (THIRD) S3 = fmaf(jf * jf * jf, d, S3);
    }
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
    return __builtin_amdgcn_exp2f(k.c1 * jf * fmaf(-jf, k.delta, two_u));
}

__device__ __forceinline__ void generic_sums(float th, const QConst &k, GenericSums &g)
{
    const float cf = nearest_level(th, k);
    g.cf = cf;
    g.u = fmaf(-cf, k.delta, th);
    const int c = (int)cf;
    g.jlo = max(k.lo - c, -k.wgen);
    g.jhi = min(k.lo + k.n_levels - 1 - c, k.wgen);
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

__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

// ------------------------------------------------------------------------------------------
// Forward kernel.  One thread handles four consecutive entries per trip of a grid-stride loop
// (one 16-byte load, one 16-byte store of soft values, one 4-byte store of indices).
// MARG: each wave adds the CPMF of its entries into its own LDS histogram; at the end the block
// sums its waves' histograms in a fixed order and writes one partial histogram to `partial`.
// ------------------------------------------------------------------------------------------
template <int W, bool IDX, bool SOFT, bool MARG>
__global__ __launch_bounds__(kQuantThreads)
void quantize_fwd_kernel(const float *__restrict__ theta, int64_t n, QConst k,
                         int8_t *__restrict__ idx, float *__restrict__ soft,
                         float *__restrict__ partial /* [gridDim.x][n_levels] */)
{
    extern __shared__ float lds_hist[];  // [waves][n_levels] when MARG
    const int lane_wave = threadIdx.x >> 6;
    float *my_hist = lds_hist + lane_wave * k.n_levels;
    if (MARG) {
        for (int i = threadIdx.x; i < (kQuantThreads / 64) * k.n_levels; i += kQuantThreads) lds_hist[i] = 0.0f;
        __syncthreads();
    }

    const int64_t n4 = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * kQuantThreads;
    for (int64_t v = (int64_t)blockIdx.x * kQuantThreads + threadIdx.x; v < n4 + 1; v += stride) {
        float th[4];
        int cnt;
        if (v < n4) {
            const float4 t = reinterpret_cast<const float4 *>(theta)[v];
            th[0] = t.x; th[1] = t.y; th[2] = t.z; th[3] = t.w;
            cnt = 4;
        } else {
            cnt = (int)(n - (n4 << 2));   // ragged tail: 0..3 entries, handled by one thread
            if (cnt == 0) break;
            for (int e = 0; e < 4; ++e) th[e] = (e < cnt) ? theta[(n4 << 2) + e] : 0.0f;
        }
        float sv[4];
        int ci[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (W > 0) {
                Band<W> b;
                band_weights<W, false>(th[e], k, b);
                const float inv = fast_rcp(b.Z);
                sv[e] = fmaf(b.S1 * inv, k.delta, b.cf * k.delta);
                ci[e] = (int)b.cf;
                if (MARG && e < cnt) {
                    const int bin = ci[e] - k.lo;
                    atomicAdd(&my_hist[bin], inv);
#pragma unroll
                    for (int j = 1; j <= W; ++j) {
                        if (b.up[j - 1] > 0.0f) atomicAdd(&my_hist[bin + j], b.up[j - 1] * inv);
                        if (b.dn[j - 1] > 0.0f) atomicAdd(&my_hist[bin - j], b.dn[j - 1] * inv);
                    }
                }
            } else {
                GenericSums g;
                generic_sums(th[e], k, g);
                const float inv = fast_rcp(g.Z);
                sv[e] = fmaf(g.S1 * inv, k.delta, g.cf * k.delta);
                ci[e] = (int)g.cf;
                if (MARG && e < cnt) {
                    const int bin = ci[e] - k.lo;
                    const float two_u = 2.0f * g.u;
                    for (int j = g.jlo; j <= g.jhi; ++j) {
                        const float pj = generic_weight(j, two_u, k) * inv;
                        if (pj > 0.0f) atomicAdd(&my_hist[bin + j], pj);
                    }
                }
            }
        }
        if (v < n4) {
            if (SOFT) reinterpret_cast<float4 *>(soft)[v] = make_float4(sv[0], sv[1], sv[2], sv[3]);
            if (IDX) {
                const uint32_t packed = (uint32_t)(ci[0] & 0xff) | ((uint32_t)(ci[1] & 0xff) << 8) |
                                        ((uint32_t)(ci[2] & 0xff) << 16) | ((uint32_t)(ci[3] & 0xff) << 24);
                reinterpret_cast<uint32_t *>(idx)[v] = packed;
            }
        } else {
            for (int e = 0; e < cnt; ++e) {
                if (SOFT) soft[(n4 << 2) + e] = sv[e];
                if (IDX) idx[(n4 << 2) + e] = (int8_t)ci[e];
            }
        }
    }

    if (MARG) {
        __syncthreads();
        for (int i = threadIdx.x; i < k.n_levels; i += kQuantThreads) {
            float s = 0.0f;
#pragma unroll
            for (int w = 0; w < kQuantThreads / 64; ++w) s += lds_hist[w * k.n_levels + i];
            partial[(size_t)blockIdx.x * k.n_levels + i] = s;
        }
    }
}

// Sums the per-block histograms (fixed order, double), normalises by n and takes the entropy.
__global__ __launch_bounds__(1024)
void marginal_finalize_kernel(const float *__restrict__ partial, int nblocks, int n_levels, double inv_n,
                              float *__restrict__ marg, float *__restrict__ entropy_bits)
{
    __shared__ double acc[1024];
    __shared__ double red[256];
    // thread t: level t % lpad, slice t / lpad; slice s adds blocks s, s+nslices, ...
    int lpad = 1;
    while (lpad < n_levels) lpad <<= 1;
    const int nslices = 1024 / lpad;
    const int level = threadIdx.x % lpad, slice = threadIdx.x / lpad;
    double s = 0.0;
    if (level < n_levels)
        for (int b = slice; b < nblocks; b += nslices) s += (double)partial[(size_t)b * n_levels + level];
    acc[threadIdx.x] = s;
    __syncthreads();
    double h = 0.0;
    if (threadIdx.x < 256) {
        double m = 0.0;
        if ((int)threadIdx.x < n_levels) {
            for (int q = 0; q < nslices; ++q) m += acc[q * lpad + threadIdx.x];
            m *= inv_n;
            if (marg) marg[threadIdx.x] = (float)m;
            if (m > 0.0) h = -m * log2(m);
        }
        red[threadIdx.x] = h;
    }
    __syncthreads();
    if (threadIdx.x == 0 && entropy_bits) {
        double H = 0.0;
        for (int i = 0; i < n_levels; ++i) H += red[i];
        *entropy_bits = (float)H;
    }
}

// ------------------------------------------------------------------------------------------
// Backward kernel: recomputes the band, forms the central moments and multiplies by the
// upstream gradient.  The two scalar sums are accumulated per thread in double, reduced over the
// block in a fixed order and written as one partial pair per block.
// ------------------------------------------------------------------------------------------
template <int W, bool DTHETA, bool SCALARS>
__global__ __launch_bounds__(kQuantThreads)
void quantize_bwd_kernel(const float *__restrict__ theta, const float *__restrict__ g, int64_t n, QConst k,
                         float *__restrict__ dtheta, double *__restrict__ partial /* [gridDim.x][2] */)
{
    double acc_d = 0.0, acc_a = 0.0;
    const int64_t n4 = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * kQuantThreads;
    for (int64_t v = (int64_t)blockIdx.x * kQuantThreads + threadIdx.x; v < n4 + 1; v += stride) {
        float th[4], ge[4];
        int cnt;
        if (v < n4) {
            const float4 t = reinterpret_cast<const float4 *>(theta)[v];
            const float4 q = reinterpret_cast<const float4 *>(g)[v];
            th[0] = t.x; th[1] = t.y; th[2] = t.z; th[3] = t.w;
            ge[0] = q.x; ge[1] = q.y; ge[2] = q.z; ge[3] = q.w;
            cnt = 4;
        } else {
            cnt = (int)(n - (n4 << 2));
            if (cnt == 0) break;
            for (int e = 0; e < 4; ++e) {
                th[e] = (e < cnt) ? theta[(n4 << 2) + e] : 0.0f;
                ge[e] = (e < cnt) ? g[(n4 << 2) + e] : 0.0f;
            }
        }
        float dv[4];
        float sum_d = 0.0f, sum_a = 0.0f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float cf, u, Z, S1, S2, S3;
            if (W > 0) {
                Band<W> b;
                band_weights<W, SCALARS>(th[e], k, b);
                cf = b.cf; u = b.u; Z = b.Z; S1 = b.S1; S2 = b.S2; S3 = b.S3;
            } else {
                GenericSums s;
                generic_sums(th[e], k, s);
                cf = s.cf; u = s.u; Z = s.Z; S1 = s.S1; S2 = s.S2; S3 = s.S3;
            }
            const float inv = fast_rcp(Z);
            const float mu = S1 * inv, m2 = S2 * inv;
            const float var = fmaf(-mu, mu, m2);
            dv[e] = ge[e] * (k.two_kappa * var);
            if (SCALARS) {
                const float m3 = S3 * inv;
                const float c3 = fmaf(-mu, fmaf(-2.0f * mu, mu, 3.0f * m2), m3);   // m3 - 3 mu m2 + 2 mu^3
                const float r = u * k.inv_delta;
                const float t_d = (cf + mu) + k.two_kappa * fmaf(r - cf - 2.0f * mu, var, -c3);
                const float t_a = fmaf(2.0f * (r - mu), var, -c3);
                sum_d = fmaf(ge[e], t_d, sum_d);
                sum_a = fmaf(ge[e], t_a, sum_a);
            }
        }
        if (SCALARS) { acc_d += (double)sum_d; acc_a += (double)sum_a; }
        if (DTHETA) {
            if (v < n4) reinterpret_cast<float4 *>(dtheta)[v] = make_float4(dv[0], dv[1], dv[2], dv[3]);
            else for (int e = 0; e < cnt; ++e) dtheta[(n4 << 2) + e] = dv[e];
        }
    }
    if (SCALARS) {
        __shared__ double red_d[kQuantThreads / 64], red_a[kQuantThreads / 64];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            acc_d += __shfl_down(acc_d, off, 64);
            acc_a += __shfl_down(acc_a, off, 64);
        }
        if ((threadIdx.x & 63) == 0) { red_d[threadIdx.x >> 6] = acc_d; red_a[threadIdx.x >> 6] = acc_a; }
        __syncthreads();
        if (threadIdx.x == 0) {
            double sd = 0.0, sa = 0.0;
            for (int w = 0; w < kQuantThreads / 64; ++w) { sd += red_d[w]; sa += red_a[w]; }
            partial[2 * (size_t)blockIdx.x] = sd;
            partial[2 * (size_t)blockIdx.x + 1] = sa;
        }
    }
}

// d_delta = sum of partials; d_alpha = delta^3 * sum of partials.  Fixed summation order.
__global__ __launch_bounds__(256)
void scalar_finalize_kernel(const double *__restrict__ partial, int nblocks, double delta_cubed,
                            float *__restrict__ d_delta, float *__restrict__ d_alpha)
{
    __shared__ double sd[256], sa[256];
    double a = 0.0, b = 0.0;
    for (int i = threadIdx.x; i < nblocks; i += 256) { a += partial[2 * (size_t)i]; b += partial[2 * (size_t)i + 1]; }
    sd[threadIdx.x] = a; sa[threadIdx.x] = b;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) { sd[threadIdx.x] += sd[threadIdx.x + off]; sa[threadIdx.x] += sa[threadIdx.x + off]; }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        if (d_delta) *d_delta = (float)sd[0];
        if (d_alpha) *d_alpha = (float)(sa[0] * delta_cubed);
    }
}

__global__ void zero_floats_kernel(float *a, int na, float *b, int nb, float *c, int nc)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (a && i < na) a[i] = 0.0f;
    if (b && i < nb) b[i] = 0.0f;
    if (c && i < nc) c[i] = 0.0f;
}

QConst make_const(const cdl_qparams &p)
{
    QConst k;
    const double delta = (double)p.delta, alpha = (double)p.alpha;
    k.delta = p.delta;
    k.inv_delta = (float)(1.0 / delta);
    k.c1 = (float)(alpha * delta * 1.4426950408889634);
    k.two_kappa = (float)(2.0 * alpha * delta * delta);
    k.lo = p.lo;
    k.n_levels = p.n_levels;
    k.lo_f = (float)p.lo;
    k.hi_f = (float)(p.lo + p.n_levels - 1);
    k.wgen = quantizer_window(alpha * delta * delta, p.n_levels);
    return k;
}

int grid_for(int64_t n)
{
    const int64_t vecs = (n >> 2) + 1;
    int64_t blocks = (vecs + kQuantThreads - 1) / kQuantThreads;
    if (blocks > kMaxQuantBlocks) blocks = kMaxQuantBlocks;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

// offsets inside the workspace
size_t hist_bytes(int32_t n_levels) { return align_up((size_t)kMaxQuantBlocks * (size_t)n_levels * sizeof(float), 256); }
size_t scalar_bytes() { return align_up((size_t)kMaxQuantBlocks * 2 * sizeof(double), 256); }

template <int W>
void launch_fwd_w(bool want_idx, bool want_soft, bool want_marg, int grid, size_t lds, hipStream_t s,
                  const float *theta, int64_t n, const QConst &k, int8_t *idx, float *soft, float *partial)
{
#define CDL_FWD(I, S, M) \
    CDL_LAUNCH((I) ? "quantize_fwd_kernel" : "quantize_fwd_kernel(marginal only)", s,                     \
               (quantize_fwd_kernel<W, I, S, M>), dim3(grid), dim3(kQuantThreads), (M) ? lds : 0,         \
               theta, n, k, idx, soft, partial)
    if (want_idx && want_soft && want_marg) CDL_FWD(true, true, true);
    else if (want_idx && want_soft) CDL_FWD(true, true, false);
    else if (want_idx && want_marg) CDL_FWD(true, false, true);
    else if (want_idx) CDL_FWD(true, false, false);
    else CDL_FWD(false, false, true);
#undef CDL_FWD
}

template <int W>
void launch_bwd_w(bool want_dtheta, bool want_scalars, int grid, hipStream_t s, const float *theta,
                  const float *g, int64_t n, const QConst &k, float *dtheta, double *partial)
{
#define CDL_BWD(D, S) \
    CDL_LAUNCH("quantize_bwd_kernel", s, (quantize_bwd_kernel<W, D, S>), dim3(grid), dim3(kQuantThreads), 0, \
               theta, g, n, k, dtheta, partial)
    if (want_dtheta && want_scalars) CDL_BWD(true, true);
    else if (want_dtheta) CDL_BWD(true, false);
    else CDL_BWD(false, true);
#undef CDL_BWD
}

}  // namespace

// Smallest W such that every level m > W away from the nearest one has relative weight
// m^3 exp(-kappa m (m-1)) below 3e-9, i.e. below fp32 resolution of every moment used.
int quantizer_window(double kappa, int n_levels)
{
    int W = 1;
    while (W < n_levels - 1) {
        const double m = (double)(W + 1);
        if (kappa * m * (m - 1.0) > 19.6 + 3.0 * log(m)) break;
        ++W;
    }
    return W;
}

size_t quantize_workspace_bytes(int64_t n, int32_t n_levels)
{
    (void)n;
    return hist_bytes(n_levels) + scalar_bytes();
}

int launch_quantize_fwd(const float *theta, int64_t n, const cdl_qparams &p,
                        int8_t *idx, float *soft, float *marg, float *entropy_bits,
                        void *ws, hipStream_t stream)
{
    const bool want_marg = (marg != nullptr) || (entropy_bits != nullptr);
    if (n == 0) {
        if (want_marg) {
            CDL_LAUNCH("zero_floats_kernel", stream, zero_floats_kernel, dim3(1), dim3(256), 0, marg, marg ? p.n_levels : 0,
                               entropy_bits, entropy_bits ? 1 : 0, (float *)nullptr, 0);
            return check_launch();
        }
        return CDL_OK;
    }
    const QConst k = make_const(p);
    const int grid = grid_for(n);
    float *partial = reinterpret_cast<float *>(ws);
    const size_t lds = (size_t)(kQuantThreads / 64) * (size_t)p.n_levels * sizeof(float);
    const bool want_idx = idx != nullptr, want_soft = soft != nullptr;
    switch (k.wgen <= 4 ? k.wgen : 0) {
        case 1: launch_fwd_w<1>(want_idx, want_soft, want_marg, grid, lds, stream, theta, n, k, idx, soft, partial); break;
        case 2: launch_fwd_w<2>(want_idx, want_soft, want_marg, grid, lds, stream, theta, n, k, idx, soft, partial); break;
        case 3: launch_fwd_w<3>(want_idx, want_soft, want_marg, grid, lds, stream, theta, n, k, idx, soft, partial); break;
        case 4: launch_fwd_w<4>(want_idx, want_soft, want_marg, grid, lds, stream, theta, n, k, idx, soft, partial); break;
        default: launch_fwd_w<0>(want_idx, want_soft, want_marg, grid, lds, stream, theta, n, k, idx, soft, partial); break;
    }
    int rc = check_launch();
    if (rc != CDL_OK) return rc;
    if (want_marg) {
        CDL_LAUNCH("marginal_finalize_kernel", stream, marginal_finalize_kernel, dim3(1), dim3(1024), 0, partial, grid, p.n_levels,
                           1.0 / (double)n, marg, entropy_bits);
        rc = check_launch();
    }
    return rc;
}

int launch_quantize_bwd(const float *theta, const float *g, int64_t n, const cdl_qparams &p,
                        float *dtheta, float *d_delta, float *d_alpha, void *ws, hipStream_t stream)
{
    const bool want_scalars = (d_delta != nullptr) || (d_alpha != nullptr);
    if (n == 0) {
        if (want_scalars) {
            CDL_LAUNCH("zero_floats_kernel", stream, zero_floats_kernel, dim3(1), dim3(64), 0, d_delta, d_delta ? 1 : 0,
                               d_alpha, d_alpha ? 1 : 0, (float *)nullptr, 0);
            return check_launch();
        }
        return CDL_OK;
    }
    const QConst k = make_const(p);
    const int grid = grid_for(n);
    double *partial = reinterpret_cast<double *>(reinterpret_cast<char *>(ws) + hist_bytes(p.n_levels));
    const bool want_dtheta = dtheta != nullptr;
    switch (k.wgen <= 4 ? k.wgen : 0) {
        case 1: launch_bwd_w<1>(want_dtheta, want_scalars, grid, stream, theta, g, n, k, dtheta, partial); break;
        case 2: launch_bwd_w<2>(want_dtheta, want_scalars, grid, stream, theta, g, n, k, dtheta, partial); break;
        case 3: launch_bwd_w<3>(want_dtheta, want_scalars, grid, stream, theta, g, n, k, dtheta, partial); break;
        case 4: launch_bwd_w<4>(want_dtheta, want_scalars, grid, stream, theta, g, n, k, dtheta, partial); break;
        default: launch_bwd_w<0>(want_dtheta, want_scalars, grid, stream, theta, g, n, k, dtheta, partial); break;
    }
    int rc = check_launch();
    if (rc != CDL_OK) return rc;
    if (want_scalars) {
        const double d = (double)p.delta;
        CDL_LAUNCH("scalar_finalize_kernel", stream, scalar_finalize_kernel, dim3(1), dim3(256), 0, partial, grid, d * d * d,
                           d_delta, d_alpha);
        rc = check_launch();
    }
    return rc;
}

}  // namespace cdl
