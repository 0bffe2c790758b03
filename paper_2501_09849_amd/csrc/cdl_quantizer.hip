// Probabilistic quantizer of CDL on gfx950: forward (hard index, soft value, marginal PMF,
// entropy) and analytic backward (Lemma 1) as single-pass streaming kernels.
//
// The conditional PMF of one entry theta over the levels i*delta is
//     P_i = softmax_i(-alpha (theta - i delta)^2)                       (eq. CPMF, Sec. III-A).
// Let c be a level next to theta (the nearest one, clamped to the set), u = theta - c*delta and
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
//
// These kernels are bound by plain fp32 ALU work as much as by HBM (one wave instruction costs
// four cycles, exp and rcp sixteen), so the band is evaluated with as few instructions as the
// accuracy allows:
//   W = 1 (kappa > 10.9): two exponentials whose arguments are formed without rounding error;
//   W = 2 (3.8 < kappa <= 10.9): one exponential t = exp(2 alpha delta u); the five weights are
//          t^(j) exp(-kappa j^2), all multiplied by t^2 so that they are a polynomial in t;
//   W = 3, 4: one exponential per level;  larger W: a loop over the band (soft regime).
#include "cdl_internal.h"
#include "cdl_quantizer_math.h"

#include <math.h>

#include <mutex>

namespace cdl {

namespace {

constexpr int kPad = 4;   // spare histogram bins on each side, so that band offsets never leave the array

// Fixed-point histogram: a block of kMargThreads threads (8 waves) makes at most kMaxHistTrips trips of
// its loop, each lane adds 4 entries per trip, and the 2 * 8 lanes with the same lane % 32 share one
// copy of a bin: at most 16 * 4 * 16 = 2^10 adds of at most 2^s each reach one cell, so s = 21 keeps
// every cell at or below 2^31.
constexpr int kMaxHistTrips = 16;
constexpr int kMargThreads = 512;   // threads of a block that builds a histogram
constexpr int kHistScaleBits = 21;

// ------------------------------------------------------------------------------------------
// Forward kernel.  One thread handles four consecutive entries per trip of a grid-stride loop
// (one 16-byte load, one 16-byte store of soft values, one 4-byte store of indices).
//
// MARG: the CPMF of every entry is added into a histogram in LDS, in fixed point: a probability
// p is added as the integer floor(p * 2^s + 1/2).  (LDS integer atomics run at ~10 lane updates
// per clock per CU on this chip, fp32 LDS atomics at a thirtieth of that; integer sums are also
// independent of the order of the adds, so the result is reproducible.)  The block keeps 32 copies of
// the histogram, bin-major and copy-minor, and lane l uses copy l mod 32: the copy is the LDS bank, so
// the lanes of one instruction never meet in a bank except lane l with lane l + 32 (measured against
// 4 or 16 copies per wave, where different bins fall into the same bank: -8 % on the whole forward
// kernel at 255 levels, -22 % on the pass that only builds the histogram).  s comes from
// kHistScaleBits: with at most kMaxHistTrips trips of the loop a cell never exceeds 2^31.
// kPad spare bins on each side take the zero weights of levels that do not exist.  At the end
// the block adds the copies into one 64-bit partial histogram row of `partial`; block 0
// also clears the ticket that the finalize kernel uses.
// ------------------------------------------------------------------------------------------
// Quantizes four entries: soft values, level indices, and (MARG) their CPMFs into the histogram.
template <int W, bool IDX, bool MARG>
__device__ __forceinline__ void forward4(const float (&th)[4], int cnt, const QConst &k, unsigned int *my_hist,
                                         float (&sv)[4], int (&ci)[4])
{
    constexpr int R = 32;
    constexpr float kScale = (float)(1u << kHistScaleBits);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (W > 0) {
            Band<W> b;
            band_weights<W, IDX, 1>(th[e], k, b);
            const float inv = fast_rcp(b.Z);
            sv[e] = fmaf(b.S1 * inv, k.delta, b.cf * k.delta);
            ci[e] = (int)b.cf;
            if (MARG && e < cnt) {
                unsigned int *h = my_hist + (ci[e] - k.lo + kPad - W) * R;   // bin of level c-W
                const float invs = inv * kScale;
                atomicAdd(h + W * R, (unsigned int)fmaf(b.ctr, invs, 0.5f));
#pragma unroll
                for (int j = 1; j <= W; ++j) {
                    atomicAdd(h + (W + j) * R, (unsigned int)fmaf(b.up[j - 1], invs, 0.5f));
                    atomicAdd(h + (W - j) * R, (unsigned int)fmaf(b.dn[j - 1], invs, 0.5f));
                }
            }
        } else {
            GenericSums g;
            generic_sums<IDX>(th[e], k, g);
            const float inv = fast_rcp(g.Z);
            sv[e] = fmaf(g.S1 * inv, k.delta, g.cf * k.delta);
            ci[e] = (int)g.cf;
            if (MARG && e < cnt) {
                unsigned int *h = my_hist + (ci[e] - k.lo + kPad) * R;
                const float two_u = 2.0f * g.u, invs = inv * kScale;
                for (int j = g.jlo; j <= g.jhi; ++j)
                    atomicAdd(h + j * R, (unsigned int)fmaf(generic_weight(j, two_u, k), invs, 0.5f));
            }
        }
    }
}

template <int W, bool IDX, bool SOFT, bool MARG>
__global__ __launch_bounds__(MARG ? kMargThreads : kQuantThreads)
void quantize_fwd_kernel(const float *__restrict__ theta, int64_t n, QConst k,
                         int8_t *__restrict__ idx, float *__restrict__ soft,
                         unsigned long long *__restrict__ partial /* [gridDim.x][n_levels] */,
                         unsigned int *__restrict__ ticket)
{
    extern __shared__ unsigned int lds_hist[];  // [n_levels + 2 kPad][32] when MARG
    constexpr int R = 32;
    constexpr int T = MARG ? kMargThreads : kQuantThreads;
    const int bins = k.n_levels + 2 * kPad;
    unsigned int *my_hist = lds_hist + (threadIdx.x & (R - 1));
    if (MARG) {
        for (int i = threadIdx.x; i < bins * R; i += T) lds_hist[i] = 0u;
        if (blockIdx.x == 0 && threadIdx.x == 0) *ticket = 0u;
        __syncthreads();
    }

    const int64_t n4 = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * T;
    float sv[4];
    int ci[4];
    for (int64_t v = (int64_t)blockIdx.x * T + threadIdx.x; v < n4; v += stride) {
        const float4 t = load_stream4(theta + 4 * v, k.stream);
        const float th[4] = {t.x, t.y, t.z, t.w};
        forward4<W, IDX, MARG>(th, 4, k, my_hist, sv, ci);
        if (SOFT) store_stream4(soft + 4 * v, sv[0], sv[1], sv[2], sv[3], k.stream);
        if (IDX) {
            const uint32_t packed = pack_indices(ci[0], ci[1], ci[2], ci[3], k.idx_off);
            reinterpret_cast<uint32_t *>(idx)[v] = packed;   // (ordinary store: the products read the indices next)
        }
    }
    // ragged tail: the last 1..3 entries, one thread of the last block
    const int cnt = (int)(n - (n4 << 2));
    if (cnt > 0 && blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        float th[4];
        for (int e = 0; e < 4; ++e) th[e] = (e < cnt) ? theta[(n4 << 2) + e] : 0.0f;
        forward4<W, IDX, MARG>(th, cnt, k, my_hist, sv, ci);
        for (int e = 0; e < cnt; ++e) {
            if (SOFT) soft[(n4 << 2) + e] = sv[e];
            if (IDX) idx[(n4 << 2) + e] = (int8_t)(ci[e] - k.idx_off);
        }
    }

    if (MARG) {
        __syncthreads();
        for (int i = threadIdx.x; i < k.n_levels; i += T) {
            unsigned long long s = 0ull;
            const unsigned int *row = lds_hist + (i + kPad) * R;
#pragma unroll
            for (int r = 0; r < R; ++r) s += row[(r + i) & (R - 1)];   // rotated start: no bank conflicts
            partial[(size_t)blockIdx.x * k.n_levels + i] = s;
        }
    }
}

// Sums the per-block fixed-point histograms (exact 64-bit integers, so the order does not matter),
// normalises by n * 2^s and adds up the entropy terms.  Grid: (ceil(levels / 8), chunks <= kFinChunks) with
// about 64 blocks in all (every block ends with an atomic on one ticket word, and those serialize at
// roughly 80 ns each); a block sums its share of the rows for eight levels (32 rows at a time, 64 contiguous bytes per row) into
// second[chunk][level]; the block that finishes last (ticket) adds the chunk sums per level,
// writes the marginal PMF and sums the entropy terms in level order.
constexpr int kFinChunks = 16;
constexpr int kFinThreads = 256, kFinGroups = kFinThreads / 8;

__global__ __launch_bounds__(kFinThreads)
void marginal_finalize_kernel(const unsigned long long *__restrict__ partial, int nblocks, int n_levels, double inv_n,
                              float *__restrict__ marg, float *__restrict__ entropy_bits,
                              unsigned long long *second /* [kFinChunks][256] */, unsigned int *ticket)
{
    __shared__ unsigned long long red[kFinGroups][8];
    __shared__ double hsum[256];
    __shared__ bool is_last;
    const int b8 = threadIdx.x & 7, grp = threadIdx.x >> 3;
    const int level = blockIdx.x * 8 + b8;
    const int chunks = gridDim.y;
    const int rows_per = (nblocks + chunks - 1) / chunks;
    const int r0 = blockIdx.y * rows_per, r1 = min(nblocks, r0 + rows_per);
    unsigned long long s = 0ull;
    if (level < n_levels) {
#pragma unroll 8
        for (int row = r0 + grp; row < r1; row += kFinGroups) s += partial[(size_t)row * n_levels + level];
    }
    red[grp][b8] = s;
    __syncthreads();
    if (threadIdx.x < 8 && level < n_levels) {
        unsigned long long tot = 0ull;
        for (int q = 0; q < kFinGroups; ++q) tot += red[q][threadIdx.x];
        __hip_atomic_store(&second[blockIdx.y * 256 + level], tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // The chunk sums are device-scope atomic stores, which go through the L2 of this XCD; once the wave's
    // store counter is zero they have arrived, and only then does the block take its ticket.  (A device-scope
    // fence would do the same by writing back the whole L2: 4 us more on a kernel of 10.)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int t = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        is_last = (t == gridDim.x * gridDim.y - 1);
    }
    __syncthreads();
    if (!is_last) return;
    asm volatile("" ::: "memory");        // the loads below are device-scope atomic loads: they do not read a stale line
    double h = 0.0;
    if ((int)threadIdx.x < n_levels) {
        unsigned long long tot = 0ull;
        for (int c = 0; c < chunks; ++c)
            tot += __hip_atomic_load(&second[c * 256 + threadIdx.x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const double m = (double)tot * inv_n;
        if (marg) marg[threadIdx.x] = (float)m;
        h = m > 0.0 ? -m * log2(m) : 0.0;
    }
    if (threadIdx.x < 256) hsum[threadIdx.x] = h;
    __syncthreads();
    if (threadIdx.x == 0 && entropy_bits) {
        double H = 0.0;
        for (int i = 0; i < n_levels; ++i) H += hsum[i];
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
            const float4 t = load_stream4(theta + 4 * v, k.stream);
            const float4 q = load_stream4(g + 4 * v, k.stream);
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
            float d_th, t_d, t_a;
            quantizer_bwd_terms<W, SCALARS>(th[e], k, d_th, t_d, t_a);
            dv[e] = ge[e] * d_th;
            if (SCALARS) {
                sum_d = fmaf(ge[e], t_d, sum_d);
                sum_a = fmaf(ge[e], t_a, sum_a);
            }
        }
        if (SCALARS) { acc_d += (double)sum_d; acc_a += (double)sum_a; }
        if (DTHETA) {
            if (v < n4) store_stream4(dtheta + 4 * v, dv[0], dv[1], dv[2], dv[3], k.stream);
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

// ------------------------------------------------------------------------------------------
// Soft regime on a small level set (at most 33 levels, kappa small enough that every level carries weight:
// the paper starts training at alpha = 500, Sec. V-B, where kappa is 0.01 - 0.5 for 2 - 5 bit weights).
// Here the band is the whole set for every entry, so nothing is gained by anchoring at the nearest level, and
// a common centre makes the loop over the levels the same for every lane.  With c0 the centre of the set
// (a level for an odd number of levels, a midpoint for an even one), r = theta / delta - c0 and offsets
// o_j = j - eps (eps = 0 or 1/2), the weight of the level at c0 +- o_j is
//     exp(-kappa o_j^2) T^(+-o_j),      T = exp(2 kappa r),
// a launch constant times a power of one exponential per entry.  The even and odd parts
//     s_j = T^o_j + T^-o_j,   d_j = T^o_j - T^-o_j
// obey s_(j+1) = (T + 1/T) s_j - s_(j-1) (the same for d): one fused multiply-add each per pair of levels,
// and the power sums take one more each (Z += E_j s_j, S1 += o_j E_j d_j, S2 += o_j^2 E_j s_j, S3 += o_j^3 E_j d_j)
// against an exponential and five instructions per single level in the generic loop.
// Everything is in double: an error of T is raised to the power o_j and hits all levels alike (it acts like a
// shift of theta by var_j * eps * delta, 5e-6 delta for fp32 with 31 live levels - too much next to the
// tolerance), moments about a centre that may be 16 levels away from the mean would cancel in fp32, and with
// packed fp32 arithmetic switched off a double fused multiply-add issues at the same rate as a single one.
// theta far outside the set: r is held at +-r_safe = JH + 15 / kappa, beyond which the CPMF is one level to
// 1e-13, so that T^JH stays finite.  The host uses these kernels when kappa * JH^2 <= 72.
// Marginal PMF: sum_e P = sum_e (E_j / 2Z_e)(s_j +- d_j): every thread keeps sum_e s_j / Z_e and sum_e d_j / Z_e
// for all j in registers (the loop is unrolled, JH is a template parameter, level sets in between are padded
// with E_j = 0), the block adds them up in a fixed order through LDS and writes one fixed-point row like the
// histogram kernels do - no atomics at all, where the generic kernel issues one per entry and level.
// ------------------------------------------------------------------------------------------
constexpr int kUniMaxJH = 16;
constexpr int kUniThreads = 256;

struct UniConst {
    double delta, c0;          // step; centre of the level set in units of the step
    double inv_delta;
    double x_per_r;            // log2(e) * kappa: T^(1/2) = exp2(x_per_r * r)
    double two_kappa;
    double r_safe;
    double e[kUniMaxJH][4];    // E_j, o_j E_j, o_j^2 E_j, o_j^3 E_j (zero for offsets beyond the set)
    int odd;                   // number of levels is odd: offsets are integers and the centre is a level
    int pairs;                 // pairs of levels: n_levels / 2
};

template <int JH>
struct UniSums {
    double Z, S1, S2, S3, r;
};

// 1 / a for a positive normal double well inside the exponent range: the hardware's reciprocal estimate and two
// Newton steps (each squares the relative error: full precision), without the scaling and fix-up code that a
// general division carries for subnormal and infinite operands - a fifth of its instructions.
__device__ __forceinline__ double uni_rcp(double a)
{
    double y = __builtin_amdgcn_rcp(a);
    y = fma(fma(-a, y, 1.0), y, y);
    y = fma(fma(-a, y, 1.0), y, y);
    return y;
}

// 2^x for |x| < 1000: x = n + f with |f| <= 1/2, e^(f ln 2) by its Taylor polynomial of degree 12 (remainder
// (ln 2 / 2)^13 / 13! = 1.7e-16) in Horner form, scaled by 2^n.  No special cases: the callers clamp x.
__device__ __forceinline__ double uni_exp2(double x)
{
    const double n = rint(x);
    const double t = (x - n) * 0.6931471805599453094;
    double p = 1.0 / 479001600.0;
    p = fma(p, t, 1.0 / 39916800.0);
    p = fma(p, t, 1.0 / 3628800.0);
    p = fma(p, t, 1.0 / 362880.0);
    p = fma(p, t, 1.0 / 40320.0);
    p = fma(p, t, 1.0 / 5040.0);
    p = fma(p, t, 1.0 / 720.0);
    p = fma(p, t, 1.0 / 120.0);
    p = fma(p, t, 1.0 / 24.0);
    p = fma(p, t, 1.0 / 6.0);
    p = fma(p, t, 0.5);
    p = fma(p, t, 1.0);
    p = fma(p, t, 1.0);
    return ldexp(p, (int)n);
}

// NMOM: how many of S1, S2, S3 are needed.  HIST: also adds s_j / Z and d_j / Z (and 1 / Z for the centre) to acc.
template <int JH, int NMOM, bool HIST>
__device__ __forceinline__ void uni_sums(float th, const UniConst &u, UniSums<JH> &o, double (&acc_s)[JH], double (&acc_d)[JH], double &acc_0)
{
    double r = fma((double)th, u.inv_delta, -u.c0);
    r = fmin(fmax(r, -u.r_safe), u.r_safe);
    o.r = r;
    const double half = uni_exp2(u.x_per_r * r);      // T^(1/2)
    const double half_inv = uni_rcp(half);
    const double T = half * half, Tinv = half_inv * half_inv;
    const double c = T + Tinv;
    const double a = u.odd ? T : half, b = u.odd ? Tinv : half_inv;
    const double s1 = a + b, d1 = a - b;
    double s_prev = u.odd ? 2.0 : s1, d_prev = u.odd ? 0.0 : -d1;
    double s = s1, d = d1;
    double Z = u.odd ? 1.0 : 0.0, S1 = 0.0, S2 = 0.0, S3 = 0.0;
#pragma unroll
    for (int j = 0; j < JH; ++j) {
        Z = fma(u.e[j][0], s, Z);
        S1 = fma(u.e[j][1], d, S1);
        if (NMOM >= 2) S2 = fma(u.e[j][2], s, S2);
        if (NMOM >= 3) S3 = fma(u.e[j][3], d, S3);
        const double s_next = fma(c, s, -s_prev), d_next = fma(c, d, -d_prev);
        s_prev = s; d_prev = d; s = s_next; d = d_next;
    }
    o.Z = Z; o.S1 = S1; o.S2 = S2; o.S3 = S3;
    if (HIST) {
        const double inv = uni_rcp(Z);
        acc_0 += inv;
        s_prev = u.odd ? 2.0 : s1; d_prev = u.odd ? 0.0 : -d1;
        s = s1 * inv; d = d1 * inv;
        s_prev *= inv; d_prev *= inv;
#pragma unroll
        for (int j = 0; j < JH; ++j) {
            acc_s[j] += s;
            acc_d[j] += d;
            const double s_next = fma(c, s, -s_prev), d_next = fma(c, d, -d_prev);
            s_prev = s; d_prev = d; s = s_next; d = d_next;
        }
    }
}

// The same sums for the backward pass, which needs all four.  Four launch constants per offset would be 128
// scalar registers at JH = 16, more than a wave has (the compiler then parks them in vector registers and
// fetches each with two extra instructions: measured twice the time).  So only E_j comes from the table and the
// powers of o_j = j - eps are literals, which costs two more multiplications per pair of levels; ODD (the
// number of levels is odd, eps = 0) is a template parameter for that reason.
template <int JH, int NMOM, bool ODD>
__device__ __forceinline__ void uni_sums_literal(float th, const UniConst &u, UniSums<JH> &o)
{
    double r = fma((double)th, u.inv_delta, -u.c0);
    r = fmin(fmax(r, -u.r_safe), u.r_safe);
    o.r = r;
    const double half = uni_exp2(u.x_per_r * r);      // T^(1/2)
    const double half_inv = uni_rcp(half);
    const double T = half * half, Tinv = half_inv * half_inv;
    const double c = T + Tinv;
    const double a = ODD ? T : half, b = ODD ? Tinv : half_inv;
    const double s1 = a + b, d1 = a - b;
    double s_prev = ODD ? 2.0 : s1, d_prev = ODD ? 0.0 : -d1;
    double s = s1, d = d1;
    double Z = ODD ? 1.0 : 0.0, S1 = 0.0, S2 = 0.0, S3 = 0.0;
#pragma unroll
    for (int j = 0; j < JH; ++j) {
        constexpr double kEps = ODD ? 0.0 : 0.5;
        const double off = (double)(j + 1) - kEps;
        const double es = u.e[j][0] * s, ed = u.e[j][0] * d;
        Z += es;
        S1 = fma(off, ed, S1);
        if (NMOM >= 2) S2 = fma(off * off, es, S2);
        if (NMOM >= 3) S3 = fma(off * off * off, ed, S3);
        const double s_next = fma(c, s, -s_prev), d_next = fma(c, d, -d_prev);
        s_prev = s; d_prev = d; s = s_next; d = d_next;
    }
    o.Z = Z; o.S1 = S1; o.S2 = S2; o.S3 = S3;
}

template <int JH, bool IDX, bool SOFT, bool MARG>
__global__ __launch_bounds__(kUniThreads)
void quantize_fwd_uniform_kernel(const float *__restrict__ theta, int64_t n, QConst k, UniConst u,
                                 int8_t *__restrict__ idx, float *__restrict__ soft,
                                 unsigned long long *__restrict__ partial /* [gridDim.x][n_levels] */,
                                 unsigned int *__restrict__ ticket)
{
    extern __shared__ double uni_lds[];   // [kUniThreads][2 JH + 1] when MARG
    double acc_s[JH], acc_d[JH], acc_0 = 0.0;
#pragma unroll
    for (int j = 0; j < JH; ++j) { acc_s[j] = 0.0; acc_d[j] = 0.0; }
    if (MARG && blockIdx.x == 0 && threadIdx.x == 0) *ticket = 0u;

    const int64_t n4 = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * kUniThreads;
    const int tail = (int)(n - (n4 << 2));
    for (int64_t v = (int64_t)blockIdx.x * kUniThreads + threadIdx.x; v < n4 + (tail ? 1 : 0); v += stride) {
        float th[4];
        int cnt = 4;
        if (v < n4) {
            const float4 t = load_stream4(theta + 4 * v, k.stream);
            th[0] = t.x; th[1] = t.y; th[2] = t.z; th[3] = t.w;
        } else {
            cnt = tail;
            for (int e = 0; e < 4; ++e) th[e] = (e < cnt) ? theta[(n4 << 2) + e] : 0.0f;
        }
        float sv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        int ci[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (IDX) ci[e] = (int)anchor_level<true>(th[e], k);
        if (MARG) {
            // (one entry after the other in a loop that stays a loop, see the backward kernel; entries past the end
            // of the tensor are not visited)
#pragma unroll 1
            for (int e = 0; e < cnt; ++e) {
                const float th_e = e == 0 ? th[0] : (e == 1 ? th[1] : (e == 2 ? th[2] : th[3]));
                UniSums<JH> q;
                uni_sums<JH, 1, true>(th_e, u, q, acc_s, acc_d, acc_0);
                const float sv_e = (float)(u.delta * (u.c0 + q.S1 * uni_rcp(q.Z)));
                sv[0] = e == 0 ? sv_e : sv[0]; sv[1] = e == 1 ? sv_e : sv[1];
                sv[2] = e == 2 ? sv_e : sv[2]; sv[3] = e == 3 ? sv_e : sv[3];
            }
        } else if (SOFT) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                UniSums<JH> q;
                uni_sums<JH, 1, false>(th[e], u, q, acc_s, acc_d, acc_0);
                sv[e] = (float)(u.delta * (u.c0 + q.S1 * uni_rcp(q.Z)));
            }
        }
        if (v < n4) {
            if (SOFT) store_stream4(soft + 4 * v, sv[0], sv[1], sv[2], sv[3], k.stream);
            if (IDX) reinterpret_cast<uint32_t *>(idx)[v] = pack_indices(ci[0], ci[1], ci[2], ci[3], k.idx_off);
        } else {
            for (int e = 0; e < cnt; ++e) {
                if (SOFT) soft[(n4 << 2) + e] = sv[e];
                if (IDX) idx[(n4 << 2) + e] = (int8_t)(ci[e] - k.idx_off);
            }
        }
    }

    if (MARG) {
        // per thread: the sums over its entries of P(level) for every level; row stride 2 JH + 1 doubles
        constexpr int LS = 2 * JH + 1;
        double *mine = uni_lds + (size_t)threadIdx.x * LS;
        // level index (from the lowest level) of the offsets +o_j and -o_j: odd sets pairs + j and pairs - j around the
        // centre level `pairs`; even sets pairs - 1 + j and pairs - j
        if (u.odd) mine[u.pairs] = acc_0;
#pragma unroll
        for (int j = 1; j <= JH; ++j) {
            if (j <= u.pairs) {
                const double up = 0.5 * u.e[j - 1][0] * (acc_s[j - 1] + acc_d[j - 1]);
                const double dn = 0.5 * u.e[j - 1][0] * (acc_s[j - 1] - acc_d[j - 1]);
                mine[u.odd ? u.pairs + j : u.pairs - 1 + j] = up;
                mine[u.pairs - j] = dn;
            }
        }
        __syncthreads();
        if ((int)threadIdx.x < k.n_levels) {
            double tot = 0.0;
            for (int t = 0; t < kUniThreads; ++t) tot += uni_lds[(size_t)t * LS + threadIdx.x];
            partial[(size_t)blockIdx.x * k.n_levels + threadIdx.x] =
                (unsigned long long)__double2ll_rn(tot * (double)(1u << kHistScaleBits));
        }
    }
}

template <int JH, bool ODD, bool DTHETA, bool SCALARS>
__global__ __launch_bounds__(kUniThreads)
void quantize_bwd_uniform_kernel(const float *__restrict__ theta, const float *__restrict__ g, int64_t n, QConst k, UniConst u,
                                 float *__restrict__ dtheta, double *__restrict__ partial /* [gridDim.x][2] */)
{
    double acc_d = 0.0, acc_a = 0.0;
    const int64_t n4 = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * kUniThreads;
    const int tail = (int)(n - (n4 << 2));
    for (int64_t v = (int64_t)blockIdx.x * kUniThreads + threadIdx.x; v < n4 + (tail ? 1 : 0); v += stride) {
        float th[4], ge[4];
        int cnt = 4;
        if (v < n4) {
            const float4 t = load_stream4(theta + 4 * v, k.stream);
            const float4 q = load_stream4(g + 4 * v, k.stream);
            th[0] = t.x; th[1] = t.y; th[2] = t.z; th[3] = t.w;
            ge[0] = q.x; ge[1] = q.y; ge[2] = q.z; ge[3] = q.w;
        } else {
            cnt = tail;
            for (int e = 0; e < 4; ++e) {
                th[e] = (e < cnt) ? theta[(n4 << 2) + e] : 0.0f;
                ge[e] = (e < cnt) ? g[(n4 << 2) + e] : 0.0f;
            }
        }
        float dv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        // One entry after the other, in a loop that stays a loop: four interleaved entries of this much double
        // arithmetic need more registers than four waves per SIMD leave (the compiler took 234, or spilled).
        // th_e, g_e and the outputs move through selects on the loop counter, which is uniform.
#pragma unroll 1
        for (int e = 0; e < 4; ++e) {
            const float th_e = e == 0 ? th[0] : (e == 1 ? th[1] : (e == 2 ? th[2] : th[3]));
            const float g_e = e == 0 ? ge[0] : (e == 1 ? ge[1] : (e == 2 ? ge[2] : ge[3]));
            UniSums<JH> q;
            uni_sums_literal<JH, SCALARS ? 3 : 2, ODD>(th_e, u, q);
            const double inv = uni_rcp(q.Z);
            const double mu = q.S1 * inv, m2 = q.S2 * inv;
            const double var = fma(-mu, mu, m2);
            const double gd = (double)g_e;
            const float dv_e = (float)(gd * (u.two_kappa * var));
            dv[0] = e == 0 ? dv_e : dv[0]; dv[1] = e == 1 ? dv_e : dv[1];
            dv[2] = e == 2 ? dv_e : dv[2]; dv[3] = e == 3 ? dv_e : dv[3];
            if (SCALARS) {
                const double m3 = q.S3 * inv;
                const double c3 = fma(-mu, fma(-2.0 * mu, mu, 3.0 * m2), m3);   // m3 - 3 mu m2 + 2 mu^3
                // Lemma 1 in offsets from the centre c0 (the derivation holds for any origin of the level index)
                const double t_d = (u.c0 + mu) + u.two_kappa * fma(q.r - u.c0 - 2.0 * mu, var, -c3);
                const double t_a = fma(2.0 * (q.r - mu), var, -c3);
                acc_d = fma(gd, t_d, acc_d);
                acc_a = fma(gd, t_a, acc_a);
            }
        }
        if (DTHETA) {
            if (v < n4) store_stream4(dtheta + 4 * v, dv[0], dv[1], dv[2], dv[3], k.stream);
            else for (int e = 0; e < cnt; ++e) dtheta[(n4 << 2) + e] = dv[e];
        }
    }
    if (SCALARS) {
        __shared__ double red_d[kUniThreads / 64], red_a[kUniThreads / 64];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            acc_d += __shfl_down(acc_d, off, 64);
            acc_a += __shfl_down(acc_a, off, 64);
        }
        if ((threadIdx.x & 63) == 0) { red_d[threadIdx.x >> 6] = acc_d; red_a[threadIdx.x >> 6] = acc_a; }
        __syncthreads();
        if (threadIdx.x == 0) {
            double sd = 0.0, sa = 0.0;
            for (int w = 0; w < kUniThreads / 64; ++w) { sd += red_d[w]; sa += red_a[w]; }
            partial[2 * (size_t)blockIdx.x] = sd;
            partial[2 * (size_t)blockIdx.x + 1] = sa;
        }
    }
}

// d_delta = mul_d * sum of partials; d_alpha = mul_a * sum of partials.  Fixed summation order: thread t adds the
// pairs t, t + T, t + 2T, ... (four independent chains, so that four loads are in flight: with a few thousand pairs
// one chain per thread is nothing but memory latency), then the threads are added up by halving.
constexpr int kScalarFinThreads = 1024;

__global__ __launch_bounds__(kScalarFinThreads)
void scalar_finalize_kernel(const double *__restrict__ partial, int nblocks, double mul_d, double mul_a,
                            float *__restrict__ d_delta, float *__restrict__ d_alpha)
{
    constexpr int T = kScalarFinThreads;
    __shared__ double sd[T], sa[T];
    const double2 *pairs = reinterpret_cast<const double2 *>(partial);
    double a[4] = {0.0, 0.0, 0.0, 0.0}, b[4] = {0.0, 0.0, 0.0, 0.0};
    int i = threadIdx.x;
    for (; i + 3 * T < nblocks; i += 4 * T) {
#pragma unroll
        for (int u = 0; u < 4; ++u) { const double2 v = pairs[i + u * T]; a[u] += v.x; b[u] += v.y; }
    }
    for (int u = 0; i < nblocks; i += T, ++u) { const double2 v = pairs[i]; a[u] += v.x; b[u] += v.y; }
    sd[threadIdx.x] = (a[0] + a[1]) + (a[2] + a[3]);
    sa[threadIdx.x] = (b[0] + b[1]) + (b[2] + b[3]);
    __syncthreads();
    for (int off = T / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) { sd[threadIdx.x] += sd[threadIdx.x + off]; sa[threadIdx.x] += sa[threadIdx.x + off]; }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        if (d_delta) *d_delta = (float)(sd[0] * mul_d);
        if (d_alpha) *d_alpha = (float)(sa[0] * mul_a);
    }
}

// ------------------------------------------------------------------------------------------
// The probabilistic quantizer Q_p (eq. Qprob, Sec. III-A) by inversion: with one uniform number
// u in [0,1) per entry the draw is the first level, in increasing order, whose cumulative
// probability exceeds u.  The comparison is made on un-normalised weights (cumulative weight against
// u * Z), which spares the division.  Reads theta and u, writes one index byte per entry.
// ------------------------------------------------------------------------------------------
template <int W>
__device__ __forceinline__ int draw_one(float th, float u, const QConst &k)
{
    if (W > 0) {
        Band<W> b;
        band_weights<W, false, 1>(th, k, b);
        const float target = u * b.Z;
        float cum = 0.0f;
        int pick = -W - 1, last = 0;
#pragma unroll
        for (int i = 0; i <= 2 * W; ++i) {
            const int j = i - W;
            const float w = j < 0 ? b.dn[-j - 1] : (j == 0 ? b.ctr : b.up[j - 1]);
            cum += w;
            if (w > 0.0f) last = j;
            if (pick < -W && cum > target) pick = j;
        }
        if (pick < -W) pick = last;
        return (int)b.cf + pick;
    } else {
        GenericSums g;
        generic_sums<false>(th, k, g);
        const float target = u * g.Z, two_u = 2.0f * g.u;
        float cum = 0.0f;
        int pick = g.jlo - 1, last = g.jlo;
        for (int j = g.jlo; j <= g.jhi; ++j) {
            const float w = generic_weight(j, two_u, k);
            cum += w;
            if (w > 0.0f) last = j;
            if (pick < g.jlo && cum > target) pick = j;
        }
        if (pick < g.jlo) pick = last;
        return (int)g.cf + pick;
    }
}

template <int W>
__global__ __launch_bounds__(kQuantThreads)
void quantize_draw_kernel(const float *__restrict__ theta, const float *__restrict__ u, int64_t n, QConst k,
                          int8_t *__restrict__ idx)
{
    const int64_t n4 = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * kQuantThreads;
    for (int64_t v = (int64_t)blockIdx.x * kQuantThreads + threadIdx.x; v < n4; v += stride) {
        const float4 t = load_stream4(theta + 4 * v, k.stream);
        const float4 r = load_stream4(u + 4 * v, k.stream);
        const int c0 = draw_one<W>(t.x, r.x, k), c1 = draw_one<W>(t.y, r.y, k);
        const int c2 = draw_one<W>(t.z, r.z, k), c3 = draw_one<W>(t.w, r.w, k);
        reinterpret_cast<uint32_t *>(idx)[v] = pack_indices(c0, c1, c2, c3, k.idx_off);
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0)
        for (int64_t e = n4 << 2; e < n; ++e) idx[e] = (int8_t)(draw_one<W>(theta[e], u[e], k) - k.idx_off);
}

// ------------------------------------------------------------------------------------------
// Gradient of the entropy term (Sec. IV-D; Algorithm 1, the step that forms the partials of H).
// With l_k = log2 of the marginal PMF (0 where the marginal is 0), for one entry
//     dH/dtheta = -(2 alpha delta / n) Cov_P(k, l_k)
//     dH/dq     = -(2 alpha / n) (theta Cov_P(k, l) - delta Cov_P(k^2, l))
//     dH/dalpha =  (1 / n) (-2 theta delta Cov_P(k, l) + delta^2 Cov_P(k^2, l))
// (differentiate H = -sum m log2 m through m_k = mean of P_k, with the CPMF derivatives of App. B).
// In band offsets j = k - c, lam_j = l_(c+j) - l_c:  C1 = Cov(j, lam),  C2 = Cov(j^2, lam),
// Cov(k^2, l) = 2 c C1 + C2, so with r = u / delta
//     dH/dq     = -(2 alpha delta / n) sum_e ((r - c) C1 - C2)
//     dH/dalpha =  (delta^2 / n)       sum_e (C2 - 2 r C1)
// The table of l_k sits in LDS with kPad zeros on both sides.  dtheta = g_in + scale * dH/dtheta.
// ------------------------------------------------------------------------------------------
template <int W, bool DTHETA, bool SCALARS, bool ADD>
__global__ __launch_bounds__(kQuantThreads)
void entropy_bwd_kernel(const float *__restrict__ theta, const float *__restrict__ marg, const float *__restrict__ g_in,
                        int64_t n, QConst k, float dtheta_mul /* scale * (-2 alpha delta / n) */,
                        float *__restrict__ dtheta, double *__restrict__ partial /* [gridDim.x][2] */)
{
    // l_k as a sum of two floats: only differences of l enter, between levels a few apart, and the scalar
    // sums multiply them by the anchor index - with a level set around index 100 the 2^-24 of a single float
    // l_k (about -5) showed as 2e-4 of dH/dq
    __shared__ float ell[256 + 2 * kPad], ell_fine[256 + 2 * kPad];
    for (int i = threadIdx.x; i < k.n_levels + 2 * kPad; i += kQuantThreads) {
        const int lv = i - kPad;
        double v = 0.0;
        if (lv >= 0 && lv < k.n_levels) { const float m = marg[lv]; v = m > 0.0f ? log2((double)m) : 0.0; }
        const float hi = (float)v;
        ell[i] = hi;
        ell_fine[i] = (float)(v - (double)hi);
    }
    __syncthreads();
    const float *ell0 = ell + kPad - k.lo;    // ell0[level] for level in [lo - kPad, hi + kPad]
    const float *fine0 = ell_fine + kPad - k.lo;

    double acc_d = 0.0, acc_a = 0.0;
    const int64_t n4 = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * kQuantThreads;
    for (int64_t v = (int64_t)blockIdx.x * kQuantThreads + threadIdx.x; v < n4 + 1; v += stride) {
        float th[4], ge[4];
        int cnt;
        if (v < n4) {
            const float4 t = load_stream4(theta + 4 * v, k.stream);
            th[0] = t.x; th[1] = t.y; th[2] = t.z; th[3] = t.w;
            if (ADD) { const float4 q = load_stream4(g_in + 4 * v, k.stream); ge[0] = q.x; ge[1] = q.y; ge[2] = q.z; ge[3] = q.w; }
            cnt = 4;
        } else {
            cnt = (int)(n - (n4 << 2));
            if (cnt == 0) break;
            for (int e = 0; e < 4; ++e) {
                th[e] = (e < cnt) ? theta[(n4 << 2) + e] : 0.0f;
                if (ADD) ge[e] = (e < cnt) ? g_in[(n4 << 2) + e] : 0.0f;
            }
        }
        float dv[4];
        float sum_d = 0.0f, sum_a = 0.0f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float cf, u, Z, S1, S2, B0 = 0.0f, B1 = 0.0f, B2 = 0.0f;
            if (W > 0) {
                Band<W> b;
                band_weights<W, false, 2>(th[e], k, b);
                cf = b.cf; u = b.u; Z = b.Z; S1 = b.S1; S2 = b.S2;
                const float *lp = ell0 + (int)cf, *fp = fine0 + (int)cf;
                const float l0 = lp[0], f0 = fp[0];
#pragma unroll
                for (int j = 1; j <= W; ++j) {
                    const float jf = (float)j;
                    const float xu = b.up[j - 1] * ((lp[j] - l0) + (fp[j] - f0)), xd = b.dn[j - 1] * ((lp[-j] - l0) + (fp[-j] - f0));
                    B0 += xu + xd;
                    B1 = fmaf(jf, xu - xd, B1);
                    B2 = fmaf(jf * jf, xu + xd, B2);
                }
            } else {
                GenericSums s;
                generic_sums<false>(th[e], k, s);
                cf = s.cf; u = s.u; Z = s.Z; S1 = s.S1; S2 = s.S2;
                const float *lp = ell0 + (int)cf, *fp = fine0 + (int)cf;
                const float l0 = lp[0], f0 = fp[0], two_u = 2.0f * u;
                for (int j = s.jlo; j <= s.jhi; ++j) {
                    const float jf = (float)j;
                    const float x = generic_weight(j, two_u, k) * ((lp[j] - l0) + (fp[j] - f0));
                    B0 += x;
                    B1 = fmaf(jf, x, B1);
                    B2 = fmaf(jf * jf, x, B2);
                }
            }
            const float inv = fast_rcp(Z);
            const float mu = S1 * inv, m2 = S2 * inv, b0 = B0 * inv;
            const float C1 = fmaf(-mu, b0, B1 * inv), C2 = fmaf(-m2, b0, B2 * inv);
            dv[e] = ADD ? fmaf(dtheta_mul, C1, ge[e]) : dtheta_mul * C1;
            if (SCALARS && e < cnt) {
                const float r = clampf(u * k.inv_delta, -k.r_clamp, k.r_clamp);
                sum_d += fmaf(r - cf, C1, -C2);
                sum_a += fmaf(-2.0f * r, C1, C2);
            }
        }
        if (SCALARS) { acc_d += (double)sum_d; acc_a += (double)sum_a; }
        if (DTHETA) {
            if (v < n4) store_stream4(dtheta + 4 * v, dv[0], dv[1], dv[2], dv[3], k.stream);
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

__global__ void zero_floats_kernel(float *a, int na, float *b, int nb, float *c, int nc)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (a && i < na) a[i] = 0.0f;
    if (b && i < nb) b[i] = 0.0f;
    if (c && i < nc) c[i] = 0.0f;
}

}  // namespace

// Which unrolled band kernel serves these parameters (0: the generic loop).
int band_template(const QConst &k) { return (!k.slide && k.wgen <= 4) ? k.wgen : 0; }

QConst make_const(const cdl_qparams &p)
{
    QConst k;
    const double delta = (double)p.delta, alpha = (double)p.alpha;
    const double kappa = alpha * delta * delta;
    k.delta = p.delta;
    k.inv_delta = (float)(1.0 / delta);
    k.c1 = (float)(alpha * delta * 1.4426950408889634);
    k.b2 = (float)(2.0 * alpha * delta * 1.4426950408889634);
    k.k1 = (float)exp(-kappa);
    k.k4 = (float)exp(-4.0 * kappa);
    k.two_kappa = (float)(2.0 * kappa);
    k.lo = p.lo;
    k.idx_off = index_offset(p);
    k.n_levels = p.n_levels;
    k.lo_f = (float)p.lo;
    k.hi_f = (float)(p.lo + p.n_levels - 1);
    k.wgen = quantizer_window(kappa, p.n_levels);
    k.slide = 0;
    k.stream = 0;
    k.r_clamp = INFINITY;
    if (p.top_k > 0 && p.top_k < p.n_levels) {
        // Truncated CPMF.  Where the band that kappa asks for is no wider than the top_k nearest levels the
        // truncation drops nothing above fp32 resolution and the ordinary kernels serve; otherwise the generic
        // kernels run on exactly the top_k nearest levels.
        const int wt = (p.top_k - 1) / 2;
        if (k.wgen > wt) { k.wgen = wt; k.slide = 1; }
    }
    if (band_template(k) == 2) k.r_clamp = (float)(30.0 / (2.0 * kappa * 1.4426950408889634));
    return k;
}

namespace {

int grid_for(int64_t n)
{
    const int64_t vecs = (n >> 2) + 1;
    int64_t blocks = (vecs + kQuantThreads - 1) / kQuantThreads;
    if (blocks > kMaxQuantBlocks) blocks = kMaxQuantBlocks;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

// Grid of the histogram kernels: as above, but never more than kMaxHistTrips trips per block, and - once
// the chip is full - a whole number of rounds: 256 CUs hold four 512-thread blocks each (2048 threads; the
// histogram of 256 levels takes 33 KB of the 160 KB of LDS), and a last round that fills half of them
// cost 10-18 % on 50 M entries.
constexpr int64_t kHistResident = 256 * 4;

int64_t hist_grid_for(int64_t n)
{
    const int64_t vecs = (n >> 2) + 1;
    const int64_t need = (vecs + (int64_t)kMargThreads * kMaxHistTrips - 1) / ((int64_t)kMargThreads * kMaxHistTrips);
    int64_t g = (grid_for(n) + 1) / 2;
    if (need > g) g = need;
    if (g > kHistResident) g = (g + kHistResident - 1) / kHistResident * kHistResident;
    return g;
}

// workspace layout: [per-block histograms][entropy terms + ticket][per-block scalar partials]
size_t hist_bytes(int64_t n, int32_t n_levels)
{
    return align_up((size_t)hist_grid_for(n) * (size_t)n_levels * sizeof(unsigned long long), 256);
}
size_t aux_bytes() { return align_up((size_t)kFinChunks * 256 * sizeof(unsigned long long) + sizeof(unsigned int), 256); }
size_t scalar_bytes() { return align_up((size_t)kMaxQuantBlocks * 2 * sizeof(double), 256); }

template <int W>
void launch_fwd_w(bool want_idx, bool want_soft, bool want_marg, int grid, hipStream_t s,
                  const float *theta, int64_t n, const QConst &k, int8_t *idx, float *soft,
                  unsigned long long *partial, unsigned int *ticket)
{
    const size_t lds = (size_t)(k.n_levels + 2 * kPad) * sizeof(float) * 32;
#define CDL_FWD(I, S, M)                                                                                  \
    CDL_LAUNCH((I) ? "quantize_fwd_kernel" : "quantize_fwd_kernel(marginal only)", s,                     \
               (quantize_fwd_kernel<W, I, S, M>), dim3(grid), dim3((M) ? kMargThreads : kQuantThreads), (M) ? lds : 0, \
               theta, n, k, idx, soft, partial, ticket)
    if (want_idx && want_soft && want_marg) CDL_FWD(true, true, true);
    else if (want_idx && want_soft) CDL_FWD(true, true, false);
    else if (want_idx && want_marg) CDL_FWD(true, false, true);
    else if (want_idx) CDL_FWD(true, false, false);
    else CDL_FWD(false, false, true);
#undef CDL_FWD
}

template <int W>
void launch_fwd(bool want_idx, bool want_soft, bool want_marg, int grid, hipStream_t s,
                const float *theta, int64_t n, const QConst &k, int8_t *idx, float *soft,
                unsigned long long *partial, unsigned int *ticket)
{
    launch_fwd_w<W>(want_idx, want_soft, want_marg, grid, s, theta, n, k, idx, soft, partial, ticket);
}

// The soft-regime kernels on a common centre serve: the full CPMF, 6 to 33 levels (smaller sets always fall to
// the unrolled band kernels), and kappa * JH^2 <= 72 with JH the padded half-width, so that T^JH stays finite
// at +-r_safe.  Returns the padded half-width (4, 8 or 16), or 0 when the other kernels serve.
int uniform_half_width(const cdl_qparams &p, const QConst &k)
{
    if (k.slide || band_template(k) != 0) return 0;
    if (p.n_levels < 6 || p.n_levels > 2 * kUniMaxJH + 1) return 0;
    const int pairs = p.n_levels / 2;
    const int jh = pairs <= 4 ? 4 : (pairs <= 8 ? 8 : 16);
    const double kappa = (double)p.alpha * (double)p.delta * (double)p.delta;
    // only where (nearly) every level is live anyway: a band much narrower than the set is cheaper in the generic loop
    if (2 * k.wgen + 1 < p.n_levels - 2) return 0;
    if (kappa * jh * jh > 72.0) return 0;
    return jh;
}

UniConst make_uniform(const cdl_qparams &p, int jh)
{
    UniConst u{};
    const double delta = (double)p.delta, alpha = (double)p.alpha;
    const double kappa = alpha * delta * delta;
    u.delta = delta;
    u.inv_delta = 1.0 / delta;
    u.odd = p.n_levels & 1;
    u.pairs = p.n_levels / 2;
    u.c0 = (double)p.lo + 0.5 * (double)(p.n_levels - 1);
    u.x_per_r = kappa * 1.4426950408889634;
    u.two_kappa = 2.0 * kappa;
    u.r_safe = (double)jh + 15.0 / kappa;
    for (int j = 1; j <= kUniMaxJH; ++j) {
        const double o = u.odd ? (double)j : (double)j - 0.5;
        const double E = j <= u.pairs ? exp(-kappa * o * o) : 0.0;
        u.e[j - 1][0] = E;
        u.e[j - 1][1] = o * E;
        u.e[j - 1][2] = o * o * E;
        u.e[j - 1][3] = o * o * o * E;
    }
    return u;
}

template <int JH>
int launch_fwd_uniform(bool want_idx, bool want_soft, bool want_marg, int grid, hipStream_t s, const float *theta, int64_t n,
                       const QConst &k, const UniConst &u, int8_t *idx, float *soft, unsigned long long *partial, unsigned int *ticket)
{
    const size_t lds = want_marg ? (size_t)kUniThreads * (2 * JH + 1) * sizeof(double) : 0;
#define CDL_UNI(I, S, M)                                                                                        \
    do {                                                                                                        \
        if (lds > 65536) {                                                                                      \
            const hipError_t e_ = hipFuncSetAttribute((const void *)quantize_fwd_uniform_kernel<JH, I, S, M>,   \
                                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);    \
            if (e_ != hipSuccess) return hip_failed(e_);                                                        \
        }                                                                                                       \
        CDL_LAUNCH((I) ? "quantize_fwd_kernel" : "quantize_fwd_kernel(marginal only)", s,                       \
                   (quantize_fwd_uniform_kernel<JH, I, S, M>), dim3(grid), dim3(kUniThreads), lds,              \
                   theta, n, k, u, idx, soft, partial, ticket);                                                 \
    } while (0)
    if (want_idx && want_soft && want_marg) CDL_UNI(true, true, true);
    else if (want_idx && want_soft) CDL_UNI(true, true, false);
    else if (want_idx && want_marg) CDL_UNI(true, false, true);
    else CDL_UNI(false, false, true);
#undef CDL_UNI
    return CDL_OK;
}

template <int JH>
void launch_bwd_uniform(bool want_dtheta, bool want_scalars, int grid, hipStream_t s, const float *theta, const float *g,
                        int64_t n, const QConst &k, const UniConst &u, float *dtheta, double *partial)
{
#define CDL_UNIB(D, S)                                                                                                          \
    do {                                                                                                                        \
        if (u.odd) CDL_LAUNCH("quantize_bwd_kernel", s, (quantize_bwd_uniform_kernel<JH, true, D, S>), dim3(grid), dim3(kUniThreads), 0, \
                              theta, g, n, k, u, dtheta, partial);                                                              \
        else CDL_LAUNCH("quantize_bwd_kernel", s, (quantize_bwd_uniform_kernel<JH, false, D, S>), dim3(grid), dim3(kUniThreads), 0,      \
                        theta, g, n, k, u, dtheta, partial);                                                                    \
    } while (0)
    if (want_dtheta && want_scalars) CDL_UNIB(true, true);
    else if (want_dtheta) CDL_UNIB(true, false);
    else CDL_UNIB(false, true);
#undef CDL_UNIB
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

// Level sets that reach beyond 127 (the paper's unsigned 8-bit alphabet {0, ..., 255}, eq. repo_alphabet) are
// stored as index - 128, which fits an int8 because such sets start at 0 or above.
int index_offset(const cdl_qparams &p) { return (int64_t)p.lo + p.n_levels - 1 > 127 ? 128 : 0; }

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
    return hist_bytes(n, n_levels) + aux_bytes() + scalar_bytes();
}

// ---- built-in scratch for callers that cannot allocate ---------------------------------------
// One array per GPU the library runs on, held until the process ends.  In host code the array's name is only a
// stand-in: the device address comes from hipGetSymbolAddress, looked up once per device (with that device
// current) and kept; kernels and copies are always handed that address.
namespace {
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};
}  // namespace

int quantizer_static_scratch(void **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_failed(e);
    if (dev < 0 || dev >= kMaxDevices) return CDL_ERR_PARAM;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_failed(e);
        if (!p) return hip_failed(hipErrorInvalidSymbol);
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return CDL_OK;
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
    QConst k = make_const(p);
    k.stream = n >= kStreamFrom;
    const int64_t grid64 = want_marg ? hist_grid_for(n) : grid_for(n);
    if (grid64 > 2147483647LL) return CDL_ERR_PARAM;
    int grid = (int)grid64;
    unsigned long long *partial = reinterpret_cast<unsigned long long *>(ws);
    unsigned long long *second = want_marg
        ? reinterpret_cast<unsigned long long *>(reinterpret_cast<char *>(ws) + hist_bytes(n, p.n_levels)) : nullptr;
    unsigned int *ticket = want_marg ? reinterpret_cast<unsigned int *>(second + kFinChunks * 256) : nullptr;
    const bool want_idx = idx != nullptr, want_soft = soft != nullptr;
    const int jh = (want_soft || want_marg) ? uniform_half_width(p, k) : 0;
    if (jh) {
        const UniConst u = make_uniform(p, jh);
        const int ugrid = grid < kMaxQuantBlocks ? grid : kMaxQuantBlocks;   // (any grid serves: the loop strides over the tensor)
        int rcu = CDL_OK;
        if (jh == 4) rcu = launch_fwd_uniform<4>(want_idx, want_soft, want_marg, ugrid, stream, theta, n, k, u, idx, soft, partial, ticket);
        else if (jh == 8) rcu = launch_fwd_uniform<8>(want_idx, want_soft, want_marg, ugrid, stream, theta, n, k, u, idx, soft, partial, ticket);
        else rcu = launch_fwd_uniform<16>(want_idx, want_soft, want_marg, ugrid, stream, theta, n, k, u, idx, soft, partial, ticket);
        if (rcu != CDL_OK) return rcu;
        grid = ugrid;
    } else
    switch (band_template(k)) {
        case 1: launch_fwd<1>(want_idx, want_soft, want_marg, grid, stream, theta, n, k, idx, soft, partial, ticket); break;
        case 2: launch_fwd<2>(want_idx, want_soft, want_marg, grid, stream, theta, n, k, idx, soft, partial, ticket); break;
        case 3: launch_fwd<3>(want_idx, want_soft, want_marg, grid, stream, theta, n, k, idx, soft, partial, ticket); break;
        case 4: launch_fwd<4>(want_idx, want_soft, want_marg, grid, stream, theta, n, k, idx, soft, partial, ticket); break;
        default: launch_fwd<0>(want_idx, want_soft, want_marg, grid, stream, theta, n, k, idx, soft, partial, ticket); break;
    }
    int rc = check_launch();
    if (rc != CDL_OK) return rc;
    if (want_marg) {
        const int level_blocks = (p.n_levels + 7) / 8;
        const int chunks = level_blocks >= 64 ? 1 : (64 / level_blocks < kFinChunks ? 64 / level_blocks : kFinChunks);
        CDL_LAUNCH("marginal_finalize_kernel", stream, marginal_finalize_kernel, dim3(level_blocks, chunks), dim3(kFinThreads), 0,
                   partial, grid, p.n_levels, 1.0 / ((double)n * (double)(1u << kHistScaleBits)), marg, entropy_bits,
                   second, ticket);
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
    QConst k = make_const(p);
    k.stream = n >= kStreamFrom;
    const int grid = grid_for(n);
    double *partial = want_scalars
        ? reinterpret_cast<double *>(reinterpret_cast<char *>(ws) + hist_bytes(n, p.n_levels) + aux_bytes()) : nullptr;
    const bool want_dtheta = dtheta != nullptr;
    const int jh = uniform_half_width(p, k);
    if (jh) {
        const UniConst u = make_uniform(p, jh);
        if (jh == 4) launch_bwd_uniform<4>(want_dtheta, want_scalars, grid, stream, theta, g, n, k, u, dtheta, partial);
        else if (jh == 8) launch_bwd_uniform<8>(want_dtheta, want_scalars, grid, stream, theta, g, n, k, u, dtheta, partial);
        else launch_bwd_uniform<16>(want_dtheta, want_scalars, grid, stream, theta, g, n, k, u, dtheta, partial);
    } else
    switch (band_template(k)) {
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
        CDL_LAUNCH("scalar_finalize_kernel", stream, scalar_finalize_kernel, dim3(1), dim3(kScalarFinThreads), 0, partial, grid, 1.0, d * d * d,
                   d_delta, d_alpha);
        rc = check_launch();
    }
    return rc;
}

int launch_scalar_finalize(const double *partial, int n, double mul_d, double mul_a, float *d_delta, float *d_alpha, hipStream_t stream)
{
    CDL_LAUNCH("scalar_finalize_kernel", stream, scalar_finalize_kernel, dim3(1), dim3(kScalarFinThreads), 0, partial, n, mul_d, mul_a, d_delta, d_alpha);
    return check_launch();
}

int launch_quantize_draw(const float *theta, const float *u, int64_t n, const cdl_qparams &p, int8_t *idx, hipStream_t stream)
{
    if (n == 0) return CDL_OK;
    QConst k = make_const(p);
    k.stream = n >= kStreamFrom;
    const int grid = grid_for(n);
#define CDL_DRAW(WW) CDL_LAUNCH("quantize_draw_kernel", stream, (quantize_draw_kernel<WW>), dim3(grid), dim3(kQuantThreads), 0, theta, u, n, k, idx)
    switch (band_template(k)) {
        case 1: CDL_DRAW(1); break;
        case 2: CDL_DRAW(2); break;
        case 3: CDL_DRAW(3); break;
        case 4: CDL_DRAW(4); break;
        default: CDL_DRAW(0); break;
    }
#undef CDL_DRAW
    return check_launch();
}

namespace {
template <int W>
void launch_entropy_bwd_w(bool want_dtheta, bool want_scalars, bool add, int grid, hipStream_t s, const float *theta,
                          const float *marg, const float *g_in, int64_t n, const QConst &k, float mul,
                          float *dtheta, double *partial)
{
#define CDL_EB(D, S, A) \
    CDL_LAUNCH("entropy_bwd_kernel", s, (entropy_bwd_kernel<W, D, S, A>), dim3(grid), dim3(kQuantThreads), 0, \
               theta, marg, g_in, n, k, mul, dtheta, partial)
    if (want_dtheta && want_scalars && add) CDL_EB(true, true, true);
    else if (want_dtheta && want_scalars) CDL_EB(true, true, false);
    else if (want_dtheta && add) CDL_EB(true, false, true);
    else if (want_dtheta) CDL_EB(true, false, false);
    else CDL_EB(false, true, false);
#undef CDL_EB
}
}  // namespace

int launch_entropy_bwd(const float *theta, const float *marg, const float *g_in, int64_t n, const cdl_qparams &p,
                       float scale, float *dtheta, float *d_delta, float *d_alpha, void *ws, hipStream_t stream)
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
    QConst k = make_const(p);
    k.stream = n >= kStreamFrom;
    const int grid = grid_for(n);
    double *partial = want_scalars
        ? reinterpret_cast<double *>(reinterpret_cast<char *>(ws) + hist_bytes(n, p.n_levels) + aux_bytes()) : nullptr;
    const bool want_dtheta = dtheta != nullptr;
    const double alpha = (double)p.alpha, delta = (double)p.delta;
    const double mul_theta = (double)scale * (-2.0 * alpha * delta / (double)n);
    switch (band_template(k)) {
        case 1: launch_entropy_bwd_w<1>(want_dtheta, want_scalars, g_in != nullptr, grid, stream, theta, marg, g_in, n, k, (float)mul_theta, dtheta, partial); break;
        case 2: launch_entropy_bwd_w<2>(want_dtheta, want_scalars, g_in != nullptr, grid, stream, theta, marg, g_in, n, k, (float)mul_theta, dtheta, partial); break;
        case 3: launch_entropy_bwd_w<3>(want_dtheta, want_scalars, g_in != nullptr, grid, stream, theta, marg, g_in, n, k, (float)mul_theta, dtheta, partial); break;
        case 4: launch_entropy_bwd_w<4>(want_dtheta, want_scalars, g_in != nullptr, grid, stream, theta, marg, g_in, n, k, (float)mul_theta, dtheta, partial); break;
        default: launch_entropy_bwd_w<0>(want_dtheta, want_scalars, g_in != nullptr, grid, stream, theta, marg, g_in, n, k, (float)mul_theta, dtheta, partial); break;
    }
    int rc = check_launch();
    if (rc != CDL_OK) return rc;
    if (want_scalars) {
        CDL_LAUNCH("scalar_finalize_kernel", stream, scalar_finalize_kernel, dim3(1), dim3(kScalarFinThreads), 0, partial, grid,
                   mul_theta, (double)scale * delta * delta / (double)n, d_delta, d_alpha);
        rc = check_launch();
    }
    return rc;
}

}  // namespace cdl
