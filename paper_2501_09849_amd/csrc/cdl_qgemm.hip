// Layer products over quantized operands on the int8 matrix cores of gfx950
// (v_mfma_i32_32x32x32_i8, int32 accumulation), rescaled by the step sizes only in the epilogue.
//
// One tiled kernel computes C[r, s] = sum_k A[r, k] * B[s, k] for two int8 matrices that both
// have the contraction index contiguous.  The forward product uses it directly on the index
// tensors (Sec. IV-A; Algorithm 1, forward step).  The two backward products contract the fp32
// upstream gradient with an index matrix; the gradient is first written as a short sum of int8
// "limbs" times powers of 2^-7 relative to one power-of-two scale (every step of that split is
// exact in fp32), the limb products are exact in int32, and the limbs are recombined in double in
// the epilogue.  The number of limbs is chosen on the device from the data so that what is cut
// off stays below the parity tolerance.
#include "cdl_internal.h"

#include <math.h>

namespace cdl {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kGemmThreads = 256;
constexpr int kKT = 64;          // contraction bytes staged per pipeline step
constexpr int kMaxLimbs = 6;
constexpr int kLimbBits = 7;     // limbs are integers in [-64, 64]

// Device-side plan of one backward call: scale of the gradient and limb counts.
struct BwdPlan {
    unsigned int absmax_bits;        // max |g| as fp32 bits (non-negative floats order like unsigned ints)
    int scale_exp;                   // sigma = 2^scale_exp, with max|g| <= sigma/2
    int limbs_da, limbs_db;          // limbs used for d_a_hat / d_b_hat
    unsigned long long sumsq_a;      // sum of a_idx^2 (all entries)
    unsigned long long sumsq_b;      // sum of b_idx^2
    double out_scale_da, out_scale_db;  // delta_b * sigma * 2^-7, delta_a * sigma * 2^-7
};

struct GemmArgs {
    const int8_t *A;      // [rowsA][lda] (limb mode: planes of that shape, a_plane bytes apart)
    const int8_t *B;      // [rowsB][ldb]
    int64_t lda, ldb, a_plane;
    int rowsA, rowsB, Kc;  // Kc: contraction length in bytes, multiple of 16
    int tiles_m, tiles_n;
    int32_t *acc_out;     // [rowsA][ldc] or null
    float *y_out;         // [rowsA][ldc] or null
    int64_t ldc;
    float scale;          // forward: delta_a * delta_b
    const BwdPlan *plan;  // limb mode
    int which;            // limb mode: 0 = d_a_hat, 1 = d_b_hat
};

__device__ __forceinline__ int swz(int row, int q) { return q ^ ((row >> 1) & 3); }

// TM x TN: 32x32 MFMA tiles per wave; the block's four waves form a 2 x 2 grid.
template <int TM, int TN, bool LIMBS>
__global__ __launch_bounds__(kGemmThreads, LIMBS ? 1 : 2)
void qgemm_kernel(GemmArgs a)
{
    constexpr int BM = 2 * TM * 32, BN = 2 * TN * 32;
    constexpr int LA = BM / 64, LB = BN / 64;   // 16-byte chunks each thread stages per step
    __shared__ __attribute__((aligned(16))) int8_t lds[2][(BM + BN) * kKT];

    // Workgroups are handed to the eight XCDs round-robin; give each XCD a contiguous run of
    // tiles so that tiles sharing an A row-block meet in one L2.
    const int total = a.tiles_m * a.tiles_n;
    const int per_xcd = (int)gridDim.x >> 3;
    const int logical = ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);
    if (logical >= total) return;
    const int tile_m = logical / a.tiles_n, tile_n = logical % a.tiles_n;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // staging assignment: chunk s = tid + 256 i  ->  LDS byte offset 16 s; row s/4, physical chunk s%4
    const int8_t *ga[LA];
    const int8_t *gb[LB];
    int qa[LA], qb[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int s = tid + kGemmThreads * i, row = s >> 2;
        qa[i] = swz(row, s & 3) * 16;
        const int grow = min(tile_m * BM + row, a.rowsA - 1);
        ga[i] = a.A + (int64_t)grow * a.lda + qa[i];
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int s = tid + kGemmThreads * i, row = s >> 2;
        qb[i] = swz(row, s & 3) * 16;
        const int grow = min(tile_n * BN + row, a.rowsB - 1);
        gb[i] = a.B + (int64_t)grow * a.ldb + qb[i];
    }

    // fragment read offsets (bytes inside one stage), per k-step ks: chunk q = 2 ks + lane/32
    int ra[TM][2], rb[TN][2];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int row = wm * TM * 32 + i * 32 + (lane & 31);
            ra[i][ks] = row * kKT + swz(row, 2 * ks + (lane >> 5)) * 16;
        }
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int row = wn * TN * 32 + j * 32 + (lane & 31);
            rb[j][ks] = BM * kKT + row * kKT + swz(row, 2 * ks + (lane >> 5)) * 16;
        }

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    double run[LIMBS ? TM : 1][LIMBS ? TN : 1][LIMBS ? 16 : 1];
    int n_limbs = 1;
    if (LIMBS) {
        n_limbs = a.which == 0 ? a.plan->limbs_da : a.plan->limbs_db;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) run[i][j][r] = 0.0;
    }

    const int nk = (a.Kc + kKT - 1) / kKT;
    const int steps = nk * n_limbs;
    const v4i zero4 = {0, 0, 0, 0};

    v4i pa[LA], pb[LB];
    auto fetch = [&](int step) {
        const int limb = LIMBS ? (n_limbs - 1 - step / nk) : 0;   // least significant limb first
        const int kt = LIMBS ? (step % nk) : step;
        const int64_t aoff = (int64_t)limb * a.a_plane + (int64_t)kt * kKT;
        const int64_t boff = (int64_t)kt * kKT;
#pragma unroll
        for (int i = 0; i < LA; ++i)
            pa[i] = (kt * kKT + qa[i] < a.Kc) ? *reinterpret_cast<const v4i *>(ga[i] + aoff) : zero4;
#pragma unroll
        for (int i = 0; i < LB; ++i)
            pb[i] = (kt * kKT + qb[i] < a.Kc) ? *reinterpret_cast<const v4i *>(gb[i] + boff) : zero4;
    };
    auto stash = [&](int stage) {
#pragma unroll
        for (int i = 0; i < LA; ++i)
            *reinterpret_cast<v4i *>(&lds[stage][(tid + kGemmThreads * i) * 16]) = pa[i];
#pragma unroll
        for (int i = 0; i < LB; ++i)
            *reinterpret_cast<v4i *>(&lds[stage][BM * kKT + (tid + kGemmThreads * i) * 16]) = pb[i];
    };

    if (steps > 0) {
        fetch(0);
        stash(0);
    }
    __syncthreads();

    for (int step = 0; step < steps; ++step) {
        const int stage = step & 1;
        if (step + 1 < steps) fetch(step + 1);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v4i fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const v4i *>(&lds[stage][ra[i][ks]]);
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[j] = *reinterpret_cast<const v4i *>(&lds[stage][rb[j][ks]]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (LIMBS && ((step + 1) % nk == 0)) {
            // one limb finished: run = run / 128 + acc, exact integers into a double
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        run[i][j][r] = fma(run[i][j][r], 1.0 / 128.0, (double)acc[i][j][r]);
                        acc[i][j][r] = 0;
                    }
        }
        if (step + 1 < steps) stash(stage ^ 1);
        __syncthreads();
    }

    // epilogue: lane holds column (lane%32) of each 32x32 tile; register r holds row 8(r/4) + 4(lane/32) + r%4
    const double out_scale = LIMBS ? (a.which == 0 ? a.plan->out_scale_da : a.plan->out_scale_db) : 0.0;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = tile_n * BN + wn * TN * 32 + j * 32 + (lane & 31);
            if (col >= a.rowsB) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = tile_m * BM + wm * TM * 32 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row >= a.rowsA) continue;
                const int64_t o = (int64_t)row * a.ldc + col;
                if (LIMBS) {
                    a.y_out[o] = (float)(run[i][j][r] * out_scale);
                } else {
                    if (a.acc_out) a.acc_out[o] = acc[i][j][r];
                    if (a.y_out) a.y_out[o] = a.scale * (float)acc[i][j][r];
                }
            }
        }
}

template <int TM, int TN, bool LIMBS>
int launch_gemm(GemmArgs a, hipStream_t stream)
{
    constexpr int BM = 2 * TM * 32, BN = 2 * TN * 32;
    a.tiles_m = (a.rowsA + BM - 1) / BM;
    a.tiles_n = (a.rowsB + BN - 1) / BN;
    const int64_t total = (int64_t)a.tiles_m * a.tiles_n;
    if (total == 0) return CDL_OK;
    const int64_t grid = (total + 7) / 8 * 8;
    CDL_LAUNCH(a.plan ? (a.which ? "qgemm_kernel(limbs, d_b_hat)" : "qgemm_kernel(limbs, d_a_hat)") : "qgemm_kernel(fwd)", stream, (qgemm_kernel<TM, TN, LIMBS>), dim3((unsigned)grid), dim3(kGemmThreads), 0, a);
    return check_launch();
}

// ---- helpers -------------------------------------------------------------------------------

// dst[r][0..ldd) = src[r][0..cols) followed by zeros.
__global__ void pad_rows_kernel(const int8_t *__restrict__ src, int64_t rows, int cols, int8_t *__restrict__ dst, int ldd)
{
    const int64_t total = rows * (int64_t)ldd;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = i / ldd;
        const int c = (int)(i - r * ldd);
        dst[i] = c < cols ? src[r * cols + c] : (int8_t)0;
    }
}

__global__ void plan_init_kernel(BwdPlan *plan)
{
    plan->absmax_bits = 0u;
    plan->sumsq_a = 0ull;
    plan->sumsq_b = 0ull;
}

__global__ __launch_bounds__(256) void absmax_kernel(const float *__restrict__ g, int64_t n, BwdPlan *plan)
{
    unsigned int m = 0u;
    const int64_t n4 = n >> 2;
    for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < n4; v += (int64_t)gridDim.x * 256) {
        const float4 t = reinterpret_cast<const float4 *>(g)[v];
        m = max(m, __float_as_uint(fabsf(t.x)));
        m = max(m, __float_as_uint(fabsf(t.y)));
        m = max(m, __float_as_uint(fabsf(t.z)));
        m = max(m, __float_as_uint(fabsf(t.w)));
    }
    if (blockIdx.x == 0 && threadIdx.x == 0)
        for (int64_t e = n4 << 2; e < n; ++e) m = max(m, __float_as_uint(fabsf(g[e])));
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = max(m, (unsigned int)__shfl_down((int)m, off, 64));
    if ((threadIdx.x & 63) == 0 && m != 0u) atomicMax(&plan->absmax_bits, m);
}

// dst[c][r] = src[r][c] for an int8 matrix [rows][cols]; dst rows are ldd long, zero-filled past
// `rows`.  Also adds sum(src^2) to *sumsq.  64 x 64 tiles through LDS.
__global__ __launch_bounds__(256) void transpose_i8_kernel(const int8_t *__restrict__ src, int rows, int cols,
                                                           int8_t *__restrict__ dst, int ldd,
                                                           unsigned long long *sumsq)
{
    __shared__ int8_t tile[64][65];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    unsigned int ss = 0u;
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int r = i >> 6, c = i & 63;
        int8_t v = 0;
        if (r0 + r < rows && c0 + c < cols) v = src[(int64_t)(r0 + r) * cols + c0 + c];
        tile[r][c] = v;
        ss += (unsigned int)((int)v * (int)v);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int c = i >> 6, r = i & 63;
        if (c0 + c < cols && r0 + r < ldd) dst[(int64_t)(c0 + c) * ldd + r0 + r] = tile[r][c];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += (unsigned int)__shfl_down((int)ss, off, 64);
    if ((threadIdx.x & 63) == 0 && ss != 0u) atomicAdd(sumsq, (unsigned long long)ss);
}

// Chooses the power-of-two scale of g and, for each backward product, the number of limbs:
// after L limbs each entry of g is known to within sigma*2^(-7L)/2 (uniformly distributed), so a
// contraction over n_c index entries of mean square q has a random error of about
// delta * sigma * 2^(-7L) * sqrt(n_c q / 12); L is the smallest count that brings it under 1.5e-7.
__global__ void plan_kernel(BwdPlan *plan, int M, int N, int K, float delta_a, float delta_b)
{
    const float amax = __uint_as_float(plan->absmax_bits);
    int e = 0;
    if (amax > 0.0f) {
        frexpf(amax, &e);   // amax = f * 2^e, f in [0.5, 1)  ->  amax < 2^e
        e += 1;             // sigma = 2^(e+1) > 2 amax
    }
    e = max(min(e, 126), -100);
    plan->scale_exp = e;
    const double sigma = ldexp(1.0, e);
    const double msq_a = (double)plan->sumsq_a / fmax(1.0, (double)M * (double)K);
    const double msq_b = (double)plan->sumsq_b / fmax(1.0, (double)N * (double)K);
    const double target = 1.5e-7;
    int la = 2, lb = 2;
    while (la < kMaxLimbs && (double)delta_b * sigma * ldexp(1.0, -kLimbBits * la) * sqrt((double)N * msq_b / 12.0) > target) ++la;
    while (lb < kMaxLimbs && (double)delta_a * sigma * ldexp(1.0, -kLimbBits * lb) * sqrt((double)M * msq_a / 12.0) > target) ++lb;
    plan->limbs_da = la;
    plan->limbs_db = lb;
    plan->out_scale_da = (double)delta_b * sigma / 128.0;
    plan->out_scale_db = (double)delta_a * sigma / 128.0;
}

// Limb l (1-based) of x = g/sigma, |x| <= 1/2:  v_1 = 128 x, limb_l = rint(v_l), v_(l+1) = 128 (v_l - limb_l).
// Every operation is exact in fp32 (scaling by a power of two; v - rint(v) needs no rounding).
__device__ __forceinline__ void split_limbs(float gval, float inv_sigma, int n_limbs, int8_t *out)
{
    float v = gval * inv_sigma * 128.0f;
#pragma unroll
    for (int l = 0; l < kMaxLimbs; ++l) {
        const float q = rintf(v);
        out[l] = (l < n_limbs) ? (int8_t)(int)q : (int8_t)0;
        v = (v - q) * 128.0f;
    }
}

// Row-major limb planes for d_a_hat: plane l, [M][ldn] with zero padding past N.
__global__ __launch_bounds__(256) void split_rows_kernel(const float *__restrict__ g, int M, int N, int ldn,
                                                         int8_t *__restrict__ planes, int64_t plane_bytes,
                                                         const BwdPlan *plan)
{
    const int n_limbs = plan->limbs_da;
    const float inv_sigma = ldexpf(1.0f, -plan->scale_exp);
    const int64_t total = (int64_t)M * ldn;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t m = i / ldn;
        const int n = (int)(i - m * ldn);
        int8_t limb[kMaxLimbs];
        split_limbs(n < N ? g[m * N + n] : 0.0f, inv_sigma, n_limbs, limb);
        for (int l = 0; l < n_limbs; ++l) planes[(int64_t)l * plane_bytes + i] = limb[l];
    }
}

// Transposed limb planes for d_b_hat: plane l, [N][ldm] with zero padding past M.
__global__ __launch_bounds__(256) void split_cols_kernel(const float *__restrict__ g, int M, int N, int ldm,
                                                         int8_t *__restrict__ planes, int64_t plane_bytes,
                                                         const BwdPlan *plan)
{
    __shared__ float tile[64][65];
    const int n_limbs = plan->limbs_db;
    const float inv_sigma = ldexpf(1.0f, -plan->scale_exp);
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int m = i >> 6, n = i & 63;
        tile[m][n] = (m0 + m < M && n0 + n < N) ? g[(int64_t)(m0 + m) * N + n0 + n] : 0.0f;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int n = i >> 6, m = i & 63;
        if (n0 + n < N && m0 + m < ldm) {
            int8_t limb[kMaxLimbs];
            split_limbs(tile[m][n], inv_sigma, n_limbs, limb);
            for (int l = 0; l < n_limbs; ++l)
                planes[(int64_t)l * plane_bytes + (int64_t)(n0 + n) * ldm + m0 + m] = limb[l];
        }
    }
}

__global__ void zero_f32_kernel(float *p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0.0f;
}

__global__ void zero_i32_kernel(int32_t *p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}

inline int64_t pad_to(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

inline unsigned blocks_for(int64_t n, int per_block, int cap = 65536)
{
    int64_t b = (n + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return (unsigned)b;
}

// workspace layout of a backward call
struct BwdLayout {
    size_t plan, bt, at, la, lb, total;
    int64_t ldn, ldm;             // padded contraction lengths
    int64_t la_plane, lb_plane;
};

BwdLayout bwd_layout(int32_t M, int32_t N, int32_t K)
{
    BwdLayout L;
    L.ldn = pad_to(N, 64);
    L.ldm = pad_to(M, 64);
    L.la_plane = (int64_t)M * L.ldn;
    L.lb_plane = (int64_t)N * L.ldm;
    size_t off = 0;
    L.plan = off; off += align_up(sizeof(BwdPlan), 256);
    L.bt = off;   off += align_up((size_t)K * (size_t)L.ldn, 256);           // b_idx^T: [K][ldn]
    L.at = off;   off += align_up((size_t)K * (size_t)L.ldm, 256);           // a_idx^T: [K][ldm]
    L.la = off;   off += align_up((size_t)kMaxLimbs * (size_t)L.la_plane, 256);
    L.lb = off;   off += align_up((size_t)kMaxLimbs * (size_t)L.lb_plane, 256);
    L.total = off;
    return L;
}

}  // namespace

size_t qgemm_fwd_workspace_bytes(int32_t M, int32_t N, int32_t K)
{
    if (K % 16 == 0) return 0;
    const int64_t kp = pad_to(K, 16);
    return align_up((size_t)M * (size_t)kp, 256) + align_up((size_t)N * (size_t)kp, 256);
}

size_t qgemm_bwd_workspace_bytes(int32_t M, int32_t N, int32_t K)
{
    if ((int64_t)M * N * K == 0) return 0;
    return bwd_layout(M, N, K).total;
}

int launch_qgemm_fwd(const int8_t *a_idx, const int8_t *b_idx, int32_t M, int32_t N, int32_t K,
                     float delta_a, float delta_b, int32_t *acc, float *y, void *ws, hipStream_t stream)
{
    if ((int64_t)M * N == 0) return CDL_OK;
    if (K == 0) {
        if (acc) CDL_LAUNCH("zero_i32_kernel", stream, zero_i32_kernel, dim3(blocks_for((int64_t)M * N, 256, 4096)), dim3(256), 0, acc, (int64_t)M * N);
        if (y) CDL_LAUNCH("zero_f32_kernel", stream, zero_f32_kernel, dim3(blocks_for((int64_t)M * N, 256, 4096)), dim3(256), 0, y, (int64_t)M * N);
        return check_launch();
    }
    GemmArgs g{};
    g.A = a_idx; g.B = b_idx; g.lda = K; g.ldb = K; g.a_plane = 0;
    g.rowsA = M; g.rowsB = N; g.Kc = K;
    if (K % 16 != 0) {
        // rows would not start on 16-byte boundaries: stage zero-padded copies
        const int kp = (int)pad_to(K, 16);
        int8_t *ap = reinterpret_cast<int8_t *>(ws);
        int8_t *bp = ap + align_up((size_t)M * (size_t)kp, 256);
        CDL_LAUNCH("pad_rows_kernel", stream, pad_rows_kernel, dim3(blocks_for((int64_t)M * kp, 256, 8192)), dim3(256), 0, a_idx, (int64_t)M, K, ap, kp);
        CDL_LAUNCH("pad_rows_kernel", stream, pad_rows_kernel, dim3(blocks_for((int64_t)N * kp, 256, 8192)), dim3(256), 0, b_idx, (int64_t)N, K, bp, kp);
        int rc = check_launch();
        if (rc != CDL_OK) return rc;
        g.A = ap; g.B = bp; g.lda = kp; g.ldb = kp; g.Kc = kp;
    }
    g.acc_out = acc; g.y_out = y; g.ldc = N;
    g.scale = delta_a * delta_b;
    g.plan = nullptr; g.which = 0;
    return launch_gemm<4, 2, false>(g, stream);
}

int launch_qgemm_bwd(const float *gr, const int8_t *a_idx, const int8_t *b_idx,
                     int32_t M, int32_t N, int32_t K, float delta_a, float delta_b,
                     float *d_a_hat, float *d_b_hat, void *ws, hipStream_t stream)
{
    if (d_a_hat && ((int64_t)M * K > 0) && N == 0)
        CDL_LAUNCH("zero_f32_kernel", stream, zero_f32_kernel, dim3(blocks_for((int64_t)M * K, 256, 4096)), dim3(256), 0, d_a_hat, (int64_t)M * K);
    if (d_b_hat && ((int64_t)N * K > 0) && M == 0)
        CDL_LAUNCH("zero_f32_kernel", stream, zero_f32_kernel, dim3(blocks_for((int64_t)N * K, 256, 4096)), dim3(256), 0, d_b_hat, (int64_t)N * K);
    if ((int64_t)M * N * K == 0) return check_launch();

    const BwdLayout L = bwd_layout(M, N, K);
    char *base = reinterpret_cast<char *>(ws);
    BwdPlan *plan = reinterpret_cast<BwdPlan *>(base + L.plan);
    int8_t *bt = reinterpret_cast<int8_t *>(base + L.bt);
    int8_t *at = reinterpret_cast<int8_t *>(base + L.at);
    int8_t *la = reinterpret_cast<int8_t *>(base + L.la);
    int8_t *lb = reinterpret_cast<int8_t *>(base + L.lb);

    CDL_LAUNCH("plan_init_kernel", stream, plan_init_kernel, dim3(1), dim3(1), 0, plan);
    CDL_LAUNCH("absmax_kernel", stream, absmax_kernel, dim3(blocks_for(((int64_t)M * N) >> 2, 256, 2048)), dim3(256), 0, gr, (int64_t)M * N, plan);
    if (d_a_hat)
        CDL_LAUNCH("transpose_i8_kernel", stream, transpose_i8_kernel, dim3((K + 63) / 64, (unsigned)(L.ldn / 64)), dim3(256), 0,
                           b_idx, N, K, bt, (int)L.ldn, &plan->sumsq_b);
    if (d_b_hat)
        CDL_LAUNCH("transpose_i8_kernel", stream, transpose_i8_kernel, dim3((K + 63) / 64, (unsigned)(L.ldm / 64)), dim3(256), 0,
                           a_idx, M, K, at, (int)L.ldm, &plan->sumsq_a);
    CDL_LAUNCH("plan_kernel", stream, plan_kernel, dim3(1), dim3(1), 0, plan, M, N, K, delta_a, delta_b);
    int rc = check_launch();
    if (rc != CDL_OK) return rc;

    if (d_a_hat) {
        CDL_LAUNCH("split_rows_kernel", stream, split_rows_kernel, dim3(blocks_for(L.la_plane, 256, 16384)), dim3(256), 0,
                           gr, M, N, (int)L.ldn, la, L.la_plane, plan);
        GemmArgs g{};
        g.A = la; g.lda = L.ldn; g.a_plane = L.la_plane;
        g.B = bt; g.ldb = L.ldn;
        g.rowsA = M; g.rowsB = K; g.Kc = (int)L.ldn;
        g.acc_out = nullptr; g.y_out = d_a_hat; g.ldc = K;
        g.plan = plan; g.which = 0;
        rc = launch_gemm<2, 2, true>(g, stream);
        if (rc != CDL_OK) return rc;
    }
    if (d_b_hat) {
        CDL_LAUNCH("split_cols_kernel", stream, split_cols_kernel, dim3((N + 63) / 64, (unsigned)(L.ldm / 64)), dim3(256), 0,
                           gr, M, N, (int)L.ldm, lb, L.lb_plane, plan);
        GemmArgs g{};
        g.A = lb; g.lda = L.ldm; g.a_plane = L.lb_plane;
        g.B = at; g.ldb = L.ldm;
        g.rowsA = N; g.rowsB = K; g.Kc = (int)L.ldm;
        g.acc_out = nullptr; g.y_out = d_b_hat; g.ldc = K;
        g.plan = plan; g.which = 1;
        rc = launch_gemm<2, 2, true>(g, stream);
        if (rc != CDL_OK) return rc;
    }
    return CDL_OK;
}

}  // namespace cdl
