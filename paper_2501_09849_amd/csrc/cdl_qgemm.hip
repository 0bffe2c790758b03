// Layer products over quantized operands on the int8 matrix cores of gfx950
// (v_mfma_i32_32x32x32_i8, int32 accumulation), rescaled by the step sizes only in the epilogue.
//
// Forward (Sec. IV-A; Algorithm 1, forward step): C[r, s] = sum_k A[r, k] * B[s, k] on the index
// tensors, both with the contraction index contiguous.
//
// Backward (Algorithm 1, backward step): the fp32 upstream gradient G is contracted with an index
// matrix.  The entries of G are written, inside the GEMM kernel, as L balanced base-256 digits
// ("limbs") of q = rint(g * 2^(8L-1) / sigma) for one power-of-two sigma > max|g|: the product
// g * 2^k is exact, so every entry is represented to within sigma * 2^-8L.  Each limb plane is an
// int8 matrix; the limb planes of 32 output rows form L x 32 rows of one int8 MFMA tile, the limb
// products are exact in int32 and are recombined in double in the epilogue.  L (3..6) is chosen on
// the device so that the rounding of q stays well below the parity tolerance.
#include "cdl_internal.h"

#include <mutex>
#include "cdl_quantizer_math.h"

#include <math.h>

#include <type_traits>

namespace cdl {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef const void __attribute__((address_space(1))) *gptr_t;
typedef void __attribute__((address_space(3))) *lptr_t;

constexpr int kGemmThreads = 256;
constexpr int kKT = 64;          // forward: contraction bytes staged per pipeline step

// Device-side plan of one backward call: scale of the gradient and limb counts.
struct BwdPlan {
    int limbs_da, limbs_db;          // limbs used for d_a_hat / d_b_hat
    float gscale_da, gscale_db;      // 2^(8L-1) / sigma
    double out_scale_da, out_scale_db;  // delta_b * sigma / 2^(8L-1), delta_a * sigma / 2^(8L-1)
    double bound_da, bound_db;          // what the rounding of g can change in one entry of d_a_hat / d_b_hat, at most
};

struct GemmArgs {
    const int8_t *A;      // [rowsA][lda]
    const int8_t *B;      // [rowsB][ldb]
    int64_t lda, ldb;
    int rowsA, rowsB, Kc;  // Kc: contraction length in bytes, multiple of 16
    int tiles_m, tiles_n;
    int32_t *acc_out;     // [rowsA][ldc] or null
    float *y_out;         // [rowsA][ldc] or null
    int64_t ldc;
    float scale;          // delta_a * delta_b
    // Operands stored as index - offset (level sets that reach beyond 127): what the stored product lacks,
    //   sum_k (a' + oa)(b' + ob) - sum_k a' b' = oa sum_k b'[s,k] + ob sum_k a'[r,k] + K oa ob,
    // as one int32 per output column (corr_col, includes the constant) and one per output row (corr_row); null = 0.
    const int32_t *corr_col;
    const int32_t *corr_row;
};

__device__ __forceinline__ int swz(int row, int q) { return q ^ ((row >> 1) & 3); }

// TM x TN: 32x32 MFMA tiles per wave; the block's four waves form a 2 x 2 grid.
template <int TM, int TN>
__global__ __launch_bounds__(kGemmThreads, 2)
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

    const int steps = (a.Kc + kKT - 1) / kKT;
    const v4i zero4 = {0, 0, 0, 0};

    v4i pa[LA], pb[LB];
    auto fetch = [&](int kt) {
        const int64_t off = (int64_t)kt * kKT;
#pragma unroll
        for (int i = 0; i < LA; ++i)
            pa[i] = (kt * kKT + qa[i] < a.Kc) ? *reinterpret_cast<const v4i *>(ga[i] + off) : zero4;
#pragma unroll
        for (int i = 0; i < LB; ++i)
            pb[i] = (kt * kKT + qb[i] < a.Kc) ? *reinterpret_cast<const v4i *>(gb[i] + off) : zero4;
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
        if (step + 1 < steps) stash(stage ^ 1);
        __syncthreads();
    }

    // epilogue: lane holds column (lane%32) of each 32x32 tile; register r holds row 8(r/4) + 4(lane/32) + r%4.
    // CORR: operands stored with an offset, corrections per column and row (a branch of its own: a test per
    // element in the common path cost a third of the kernel's time)
    auto epilogue = [&](auto corr_c) {
        constexpr bool CORR = decltype(corr_c)::value;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = tile_n * BN + wn * TN * 32 + j * 32 + (lane & 31);
                if (col >= a.rowsB) continue;
                const int cc = (CORR && a.corr_col) ? a.corr_col[col] : 0;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = tile_m * BM + wm * TM * 32 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    if (row >= a.rowsA) continue;
                    const int64_t o = (int64_t)row * a.ldc + col;
                    const int v = CORR ? acc[i][j][r] + cc + (a.corr_row ? a.corr_row[row] : 0) : acc[i][j][r];
                    if (a.acc_out) a.acc_out[o] = v;
                    if (a.y_out) a.y_out[o] = a.scale * (float)v;
                }
            }
    };
    if (a.corr_col || a.corr_row) epilogue(std::true_type{});
    else epilogue(std::false_type{});
}

template <int TM, int TN>
int launch_gemm(GemmArgs a, hipStream_t stream)
{
    constexpr int BM = 2 * TM * 32, BN = 2 * TN * 32;
    a.tiles_m = (a.rowsA + BM - 1) / BM;
    a.tiles_n = (a.rowsB + BN - 1) / BN;
    const int64_t total = (int64_t)a.tiles_m * a.tiles_n;
    if (total == 0) return CDL_OK;
    const int64_t grid = (total + 7) / 8 * 8;
    CDL_LAUNCH("qgemm_kernel(fwd)", stream, (qgemm_kernel<TM, TN>), dim3((unsigned)grid), dim3(kGemmThreads), 0, a);
    return check_launch();
}

// ---- backward: limb GEMM ---------------------------------------------------------------------

struct LimbArgs {
    const float *G;       // [M][N] fp32 upstream gradient
    int M, N;
    const int8_t *Bt;     // [cols][ldb] int8 index matrix, contraction index contiguous, zero-filled up to nk * kLBK
    int64_t ldb;          // row stride in bytes: an odd multiple of kLBK, so that rows start in different memory channels
    int nk;               // K-tiles covering the contraction: ceil(kc / kLBK)
    int rows, cols, kc;   // output rows / columns, contraction length
    int tiles_r, splits, kt_per_split;
    int units_per_block;  // consecutive row tiles one block works through
    const BwdPlan *plan;
    int which;            // 0 = d_a_hat, 1 = d_b_hat
    float *out;           // [rows][cols] (splits == 1)
    double *partial;      // [splits][rows][cols] (splits > 1, or to_partial)
    int to_partial;       // 1: the unscaled sums go to `partial` as doubles even with one split (a reduction kernel follows)
    // d_a_hat only: the quantizer's backward pass applied to the tile before it leaves the chip (fq_theta != null):
    // out receives dL/dtheta instead of dL/dQ(theta), fq_partial one pair of partial scalar gradients per block
    const float *fq_theta;    // [rows][cols] the tensor that was quantized into the index operand of the forward product
    double *fq_partial;       // [work items][2]
    QConst fq_k;
    int fq_wsel;              // band_template(fq_k)
    float fq_scale;           // forward product with the quantizer in its prologue: delta_a * delta_b
    // activation gradient of a convolution (CONVG): the rows of the fp32 operand are gathered.  Output row m is pixel
    // (b, i, j) of a grid of cg_H x cg_W pixels per image; contraction entry k = (tap (r, s) of cg_R' x cg_S taps, output
    // channel n) is read from G[b, p, q, n] with p = i + pad_h - r, q = j + pad_w - s where those are inside the output
    // image, else 0.  A thread's four consecutive entries share a tap (N % 4 == 0).  Stride 1: the grid is the input
    // image.  Stride 2: one launch per parity class (a, c) of the input pixels, whose grid holds the pixels
    // (2 i + a, 2 j + c) and whose taps are those of the same parity as (a + pad, c + pad) - the only ones that reach
    // such a pixel -, renumbered; the output rows then lie scattered in the tensor (cg_ostep = 2).
    int cg_H, cg_W, cg_P, cg_Q, cg_S, cg_pad_h, cg_pad_w;
    float cg_inv_n, cg_inv_s;     // 1 / N, 1 / S
    int cg_ostep, cg_oa, cg_oc, cg_oH, cg_oW;   // output pixel of grid pixel (b, i, j): (b, ostep i + oa, ostep j + oc) of oH x oW
    uint32_t cg_mul_hw, cg_mul_w;               // m / (cg_H cg_W) and m / cg_W as multiplications (div_by)
    int cg_sh_hw, cg_sh_w;
    int tn;                       // 32-column tiles per wave (1..3; with six limbs at most 2)
    const double *row_corr;   // [rows] or null: added to every entry of an output row (the index operand is stored with an offset:
                              // the missing part of the product is offset * step * sum of g over the contraction); splits == 1 only
};

constexpr int kLBK = 128;     // contraction bytes per K-tile
constexpr int kLRows = 32;    // output rows per block
constexpr int kLPlane = kLRows * kLBK;
constexpr int kLThreads = 256;
constexpr int kMinLimbs = 3, kMaxLimbs = 6;

constexpr int limb_tn(int L) { return L <= 5 ? 3 : 2; }          // 32-column tiles per wave
constexpr int limb_cols(int L) { return 4 * limb_tn(L) * 32; }   // output columns per block
constexpr int limb_stage_bytes(int L) { return L * kLPlane + limb_cols(L) * kLBK; }
constexpr int kLimbLdsBytes = 2 * limb_stage_bytes(5);
static_assert(limb_stage_bytes(3) <= limb_stage_bytes(5) && limb_stage_bytes(4) <= limb_stage_bytes(5) &&
              limb_stage_bytes(6) <= limb_stage_bytes(5), "LDS sized for five limbs");

__device__ __forceinline__ int lswz(int row) { return (row >> 1) & 7; }
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0f70; }   // s_waitcnt vmcnt(n) only
constexpr int kLgkmcnt0 = 0xc07f;                                                   // s_waitcnt lgkmcnt(0) only

__device__ __forceinline__ uint32_t bperm(uint32_t hi, uint32_t lo, uint32_t sel) { return __builtin_amdgcn_perm(hi, lo, sel); }

// Forward product, fast path for contraction lengths that are multiples of 128: 512 threads = 2 x 4 waves,
// 256 x 256 block tile (wave tile 128 x 64: eight 32x32 accumulators), K-tiles of 128 bytes brought in by
// direct global->LDS loads (no staging registers) into two LDS stages of 64 KiB, 16-byte chunks XOR-swizzled
// over the eight chunks of a row so that the fragment reads are free of bank conflicts.  The barrier is a
// bare s_barrier with the one wait it needs written out: the loads of the next tile are issued right after
// it and have the whole K-tile of MFMAs to land.
constexpr int kFBK = 128;
constexpr int kFThreads = 512;
constexpr int kFTile = 256;
constexpr int kFStage = 2 * kFTile * kFBK;
constexpr int kFLdsBytes = 2 * kFStage;

__global__ __launch_bounds__(kFThreads, 1)
void qgemm_dma_kernel(GemmArgs a)
{
    constexpr int WN = 4, TM = 4, TN = 2, CH = kFBK / 16, KS = kFBK / 32;
    constexpr int WL = kFTile * CH / 64 / 8;      // wave-level loads per wave, per operand and K-tile: 4
    extern __shared__ __attribute__((aligned(16))) int8_t flds[];

    const int total = a.tiles_m * a.tiles_n;
    const int per_xcd = (int)gridDim.x >> 3;
    const int logical = ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);
    if (logical >= total) return;
    const int tile_m = logical / a.tiles_n, tile_n = logical % a.tiles_n;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // wave-level load i of this wave fills LDS slots (wave * WL + i) * 64 + lane: row slot / 8, chunk slot % 8
    const int8_t *ga[WL];
    const int8_t *gb[WL];
#pragma unroll
    for (int i = 0; i < WL; ++i) {
        const int sidx = (wave * WL + i) * 64 + lane, row = sidx / CH;
        const int q = (sidx % CH) ^ lswz(row);
        ga[i] = a.A + (int64_t)min(tile_m * kFTile + row, a.rowsA - 1) * a.lda + q * 16;
        gb[i] = a.B + (int64_t)min(tile_n * kFTile + row, a.rowsB - 1) * a.ldb + q * 16;
    }
    int ra[TM], rb[TN], sa[TM], sb[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int row = (wm * TM + i) * 32 + (lane & 31);
        ra[i] = row * kFBK;
        sa[i] = lswz(row);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int row = (wn * TN + j) * 32 + (lane & 31);
        rb[j] = kFTile * kFBK + row * kFBK;
        sb[j] = lswz(row);
    }

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    const int nk = a.Kc / kFBK;
    auto issue = [&](int kt) {
        int8_t *base = flds + (kt & 1) * kFStage;
        const int64_t off = (int64_t)kt * kFBK;
#pragma unroll
        for (int i = 0; i < WL; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t)(ga[i] + off), (lptr_t)(base + (wave * WL + i) * 1024), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < WL; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t)(gb[i] + off), (lptr_t)(base + kFTile * kFBK + (wave * WL + i) * 1024), 16, 0, 0);
    };

    issue(0);
    for (int kt = 0; kt < nk; ++kt) {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // tile kt has landed (nothing younger is in flight)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();               // ... for every wave, and every wave has left the other stage
        asm volatile("" ::: "memory");
        if (kt + 1 < nk) issue(kt + 1);
        const int8_t *base = flds + (kt & 1) * kFStage;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            v4i fa[TM], fb[TN];
            const int q = 2 * ks + (lane >> 5);
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const v4i *>(base + ra[i] + ((q ^ sa[i]) << 4));
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[j] = *reinterpret_cast<const v4i *>(base + rb[j] + ((q ^ sb[j]) << 4));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }

    const bool full = (tile_m + 1) * kFTile <= a.rowsA && (tile_n + 1) * kFTile <= a.rowsB;
    // (CORR: operands stored with an offset; kept out of the common path, see qgemm_kernel)
    auto epilogue = [&](auto corr_c) {
        constexpr bool CORR = decltype(corr_c)::value;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = tile_n * kFTile + (wn * TN + j) * 32 + (lane & 31);
                const int cc = (CORR && a.corr_col && col < a.rowsB) ? a.corr_col[col] : 0;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = tile_m * kFTile + (wm * TM + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    if (full || (row < a.rowsA && col < a.rowsB)) {
                        const int64_t o = (int64_t)row * a.ldc + col;
                        const int v = CORR ? acc[i][j][r] + cc + (a.corr_row ? a.corr_row[row] : 0) : acc[i][j][r];
                        if (a.acc_out) a.acc_out[o] = v;
                        if (a.y_out) a.y_out[o] = a.scale * (float)v;
                    }
                }
            }
    };
    if (a.corr_col || a.corr_row) epilogue(std::true_type{});
    else epilogue(std::false_type{});
}

int launch_gemm_dma(GemmArgs a, hipStream_t stream)
{
    a.tiles_m = (a.rowsA + kFTile - 1) / kFTile;
    a.tiles_n = (a.rowsB + kFTile - 1) / kFTile;
    const int64_t total = (int64_t)a.tiles_m * a.tiles_n;
    if (total == 0) return CDL_OK;
    const int64_t grid = (total + 7) / 8 * 8;
    const hipError_t e = hipFuncSetAttribute((const void *)qgemm_dma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kFLdsBytes);
    if (e != hipSuccess) return hip_failed(e);
    CDL_LAUNCH("qgemm_kernel(fwd)", stream, qgemm_dma_kernel, dim3((unsigned)grid), dim3(kFThreads), kFLdsBytes, a);
    return check_launch();
}

// ---- forward product of a convolutional layer, without an im2col matrix ---------------------------------
//
// acc[b,p,q,n] = sum_{r,s,c} x[b, p*stride + r - pad, q*stride + s - pad, c] * w[n,r,s,c]  (Sec. IV-A for a
// convolutional layer): the product of the [B*P*Q, R*S*C] matrix of input windows with w^T, where row m of that
// matrix is never stored - its 16-byte chunks are read from the NHWC tensor where they lie (C is a multiple of
// 16, so a chunk lies inside one tap), and chunks of taps that fall outside the image come from a page of
// padding bytes (the stored value of level index 0).
struct ConvArgs {
    const int8_t *X;       // [B][H][W][C]
    const int8_t *Wt;      // [N][R*S*C]
    const int8_t *pad_page;   // 128 bytes of the padding value (direct-load kernel)
    int pad_word;          // the padding value in all four bytes (register-staged kernel)
    int B, H, W, C, N, R, S, stride, pad, P, Q;
    int M, Kc;             // B*P*Q, R*S*C
    int tiles_m, tiles_n;
    int32_t *acc_out;      // [M][N] or null
    float *y_out;          // [M][N] or null
    float scale;
    const int32_t *corr_col;   // [N] or null: x stored with an offset, x_offset * sum over the window of w[n]
};

// where output pixel m looks: first input row and column of its window, and the offset of that (possibly
// virtual) pixel in X
struct ConvRow { int h0, w0; int64_t off; };
__device__ __forceinline__ ConvRow conv_row(const ConvArgs &a, int m)
{
    const int pq = a.P * a.Q;
    const int b = m / pq, rem = m - b * pq, p = rem / a.Q, q = rem - p * a.Q;
    ConvRow r;
    r.h0 = p * a.stride - a.pad;
    r.w0 = q * a.stride - a.pad;
    r.off = (((int64_t)b * a.H + r.h0) * a.W + r.w0) * a.C;
    return r;
}

__device__ __forceinline__ void conv_store(const ConvArgs &a, int row, int col, int v)
{
    const int64_t o = (int64_t)row * a.N + col;
    if (a.acc_out) a.acc_out[o] = v;
    if (a.y_out) a.y_out[o] = a.scale * (float)v;
}

// C a multiple of 128: the structure of qgemm_dma_kernel (256 x 256 tile, K-tiles of 128 bytes by direct
// global->LDS loads, two stages), a K-tile being 128 channels of one tap.
__global__ __launch_bounds__(kFThreads, 1)
void qconv_dma_kernel(ConvArgs a)
{
    constexpr int WN = 4, TM = 4, TN = 2, CH = kFBK / 16, KS = kFBK / 32;
    constexpr int WL = kFTile * CH / 64 / 8;
    extern __shared__ __attribute__((aligned(16))) int8_t flds[];

    const int total = a.tiles_m * a.tiles_n;
    const int per_xcd = (int)gridDim.x >> 3;
    const int logical = ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);
    if (logical >= total) return;
    const int tile_m = logical / a.tiles_n, tile_n = logical % a.tiles_n;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    ConvRow xr[WL];
    const int8_t *gb[WL];
#pragma unroll
    for (int i = 0; i < WL; ++i) {
        const int sidx = (wave * WL + i) * 64 + lane, row = sidx / CH;
        const int q = (sidx % CH) ^ lswz(row);
        xr[i] = conv_row(a, min(tile_m * kFTile + row, a.M - 1));
        xr[i].off += q * 16;
        gb[i] = a.Wt + (int64_t)min(tile_n * kFTile + row, a.N - 1) * a.Kc + q * 16;
    }
    int ra[TM], rb[TN], sa[TM], sb[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int row = (wm * TM + i) * 32 + (lane & 31);
        ra[i] = row * kFBK;
        sa[i] = lswz(row);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int row = (wn * TN + j) * 32 + (lane & 31);
        rb[j] = kFTile * kFBK + row * kFBK;
        sb[j] = lswz(row);
    }

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    const int nk = a.Kc / kFBK;
    // tap (tr, ts) and first channel tc of the K-tile that `issue` is called with next (called with 0, 1, 2, ...)
    int tr = 0, ts = 0, tc = 0;
    // where the rows of the next K-tile are read from: worked out while the MFMAs of the current one run, so that the
    // loads go out right behind the barrier
    const int8_t *srcA[WL];
    auto prepare = [&]() {
        const int64_t tap_off = ((int64_t)tr * a.W + ts) * a.C + tc;
#pragma unroll
        for (int i = 0; i < WL; ++i) {
            const bool inside = (unsigned)(xr[i].h0 + tr) < (unsigned)a.H && (unsigned)(xr[i].w0 + ts) < (unsigned)a.W;
            srcA[i] = inside ? a.X + (xr[i].off + tap_off) : a.pad_page;
        }
        tc += kFBK;
        if (tc == a.C) { tc = 0; if (++ts == a.S) { ts = 0; ++tr; } }
    };
    auto issue = [&](int kt) {
        int8_t *base = flds + (kt & 1) * kFStage;
#pragma unroll
        for (int i = 0; i < WL; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t)srcA[i], (lptr_t)(base + (wave * WL + i) * 1024), 16, 0, 0);
        const int64_t off = (int64_t)kt * kFBK;
#pragma unroll
        for (int i = 0; i < WL; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t)(gb[i] + off), (lptr_t)(base + kFTile * kFBK + (wave * WL + i) * 1024), 16, 0, 0);
    };

    prepare();
    issue(0);
    if (nk > 1) prepare();
    for (int kt = 0; kt < nk; ++kt) {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (kt + 1 < nk) issue(kt + 1);
        if (kt + 2 < nk) prepare();
        const int8_t *base = flds + (kt & 1) * kFStage;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            v4i fa[TM], fb[TN];
            const int q = 2 * ks + (lane >> 5);
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const v4i *>(base + ra[i] + ((q ^ sa[i]) << 4));
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[j] = *reinterpret_cast<const v4i *>(base + rb[j] + ((q ^ sb[j]) << 4));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }

    const bool full = (tile_m + 1) * kFTile <= a.M && (tile_n + 1) * kFTile <= a.N;
    // (the corrections of an operand stored with an offset are loaded before the first store and live in a copy of the
    // epilogue of their own: a load between the stores makes every store wait for the one before it - loads and stores
    // share one counter - which cost 10 us per round of blocks)
    auto epilogue = [&](auto corr_c) {
        constexpr bool CORR = decltype(corr_c)::value;
        int cc[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = tile_n * kFTile + (wn * TN + j) * 32 + (lane & 31);
            cc[j] = (CORR && col < a.N) ? a.corr_col[col] : 0;
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = tile_n * kFTile + (wn * TN + j) * 32 + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = tile_m * kFTile + (wm * TM + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    if (full || (row < a.M && col < a.N)) conv_store(a, row, col, CORR ? acc[i][j][r] + cc[j] : acc[i][j][r]);
                }
            }
    };
    if (a.corr_col) epilogue(std::true_type{});
    else epilogue(std::false_type{});
}

// Any C that is a multiple of 16: the structure of qgemm_kernel (256 x 128 tile, 64-byte K steps staged through
// registers), every 16-byte chunk of the window matrix looked up on its own: a table in LDS gives, per chunk of the
// contraction, its tap and its offset from the window's first pixel.
constexpr int kConvMaxChunks = 2048;     // contraction lengths up to 32768

template <int TM, int TN>
__global__ __launch_bounds__(kGemmThreads, 2)
void qconv_kernel(ConvArgs a)
{
    constexpr int BM = 2 * TM * 32, BN = 2 * TN * 32;
    constexpr int LA = BM / 64, LB = BN / 64;
    __shared__ __attribute__((aligned(16))) int8_t lds[2][(BM + BN) * kKT];
    __shared__ int2 taps[kConvMaxChunks];    // .x: offset of the chunk from the window's first pixel, .y: tap row << 16 | tap column

    const int total = a.tiles_m * a.tiles_n;
    const int per_xcd = (int)gridDim.x >> 3;
    const int logical = ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);
    if (logical >= total) return;
    const int tile_m = logical / a.tiles_n, tile_n = logical % a.tiles_n;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    for (int c16 = tid; c16 < a.Kc / 16; c16 += kGemmThreads) {
        const int k = c16 * 16, tap = k / a.C, c = k - tap * a.C, r = tap / a.S, s = tap - r * a.S;
        taps[c16] = make_int2((r * a.W + s) * a.C + c, (r << 16) | s);
    }

    ConvRow xr[LA];
    const int8_t *gb[LB];
    int qa[LA], qb[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int s = tid + kGemmThreads * i, row = s >> 2;
        qa[i] = swz(row, s & 3);
        xr[i] = conv_row(a, min(tile_m * BM + row, a.M - 1));
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int s = tid + kGemmThreads * i, row = s >> 2;
        qb[i] = swz(row, s & 3) * 16;
        const int grow = min(tile_n * BN + row, a.N - 1);
        gb[i] = a.Wt + (int64_t)grow * a.Kc + qb[i];
    }

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

    const int steps = (a.Kc + kKT - 1) / kKT;
    const int chunks = a.Kc / 16;
    const v4i zero4 = {0, 0, 0, 0};
    const v4i pad4 = {a.pad_word, a.pad_word, a.pad_word, a.pad_word};
    __syncthreads();        // the tap table is complete

    v4i pa[LA], pb[LB];
    auto fetch = [&](int kt) {
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int c16 = kt * (kKT / 16) + qa[i];
            v4i v = zero4;                       // beyond the contraction: multiplies zeros of the other operand as well
            if (c16 < chunks) {
                const int2 t = taps[c16];
                const bool inside = (unsigned)(xr[i].h0 + (t.y >> 16)) < (unsigned)a.H && (unsigned)(xr[i].w0 + (t.y & 0xffff)) < (unsigned)a.W;
                v = inside ? *reinterpret_cast<const v4i *>(a.X + (xr[i].off + t.x)) : pad4;
            }
            pa[i] = v;
        }
        const int64_t off = (int64_t)kt * kKT;
#pragma unroll
        for (int i = 0; i < LB; ++i)
            pb[i] = (kt * kKT + qb[i] < a.Kc) ? *reinterpret_cast<const v4i *>(gb[i] + off) : zero4;
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
        if (step + 1 < steps) stash(stage ^ 1);
        __syncthreads();
    }

    auto epilogue = [&](auto corr_c) {
        constexpr bool CORR = decltype(corr_c)::value;
        int cc[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = tile_n * BN + wn * TN * 32 + j * 32 + (lane & 31);
            cc[j] = (CORR && col < a.N) ? a.corr_col[col] : 0;
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = tile_n * BN + wn * TN * 32 + j * 32 + (lane & 31);
                if (col >= a.N) continue;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = tile_m * BM + wm * TM * 32 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    if (row < a.M) conv_store(a, row, col, CORR ? acc[i][j][r] + cc[j] : acc[i][j][r]);
                }
            }
    };
    if (a.corr_col) epilogue(std::true_type{});
    else epilogue(std::false_type{});
}

// 128 bytes that read as level index 0 of an operand stored with offset `off`, and (with an offset) the
// correction per output channel: off * sum of w[n] over the whole window (a padded tap holds -off + off = 0)
__global__ __launch_bounds__(256)
void conv_prep_kernel(int8_t *page, int off, const int8_t *w, int N, int Kc, int32_t *corr)
{
    if (blockIdx.x == 0 && threadIdx.x < 128) page[threadIdx.x] = (int8_t)(-off);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int n = blockIdx.x * 4 + wave; n < N; n += gridDim.x * 4) {
        int s = 0;
        for (int k = lane; k < Kc; k += 64) s += (int)w[(int64_t)n * Kc + k];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) s += __shfl_down(s, o, 64);
        if (lane == 0) corr[n] = off * s;
    }
}

// a page of zeros that belongs to the library's device code (one copy per GPU): the padding of operands stored
// without an offset, so that such calls need no workspace
static __device__ __align__(256) int8_t conv_zero_page[256];

// n / d for 0 <= n < 2^31 by one multiplication: with s = ceil(log2 d) and mul = ceil(2^(31 + s) / d) (below 2^32) the
// quotient is (n * mul) >> (31 + s), exactly (the excess mul * d - 2^(31 + s) is below d <= 2^s, so it adds less than
// one unit of the quotient over the whole range of n); sh = s - 1, or -1 for d = 1.
struct DivBy { uint32_t mul; int sh; };
inline DivBy make_div_by(uint32_t d)
{
    if (d <= 1) return DivBy{0u, -1};
    int s = 0;
    while ((1ull << s) < d) ++s;
    const unsigned long long mul = ((1ull << (31 + s)) + d - 1) / d;
    return DivBy{(uint32_t)mul, s - 1};
}
__device__ __forceinline__ int div_by(int n, uint32_t mul, int sh)
{
    return sh < 0 ? n : (int)(__umulhi((uint32_t)n, mul) >> sh);
}

// Digits of four values: out[l] holds digit l (a signed byte, l = 0 least significant) of g[0..3] in
// its bytes 0..3.  x = g * gscale is exact (gscale is a power of two) and |x| < 0.99 * 2^(8L-1);
// q = rint(x) = sum_l d_l 256^l with d_l in [-128, 127]: the bytes of (q + 0x80..80) ^ 0x80..80.
template <int L>
__device__ __forceinline__ void limbs_of4(const float (&g)[4], float gscale, uint32_t (&out)[L])
{
    if (L <= 4) {
        constexpr uint32_t off = L == 4 ? 0x80808080u : 0x00808080u;
        uint32_t d[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int q = (int)rintf(g[e] * gscale);
            d[e] = ((uint32_t)q + off) ^ off;
        }
        const uint32_t t0 = bperm(d[1], d[0], 0x05010400u), t2 = bperm(d[3], d[2], 0x05010400u);
        out[0] = bperm(t2, t0, 0x05040100u);
        out[1] = bperm(t2, t0, 0x07060302u);
        const uint32_t t1 = bperm(d[1], d[0], 0x07030602u), t3 = bperm(d[3], d[2], 0x07030602u);
        out[2] = bperm(t3, t1, 0x05040100u);
        if (L == 4) out[L - 1] = bperm(t3, t1, 0x07060302u);
    } else {
        // q has up to 48 bits: the low 16 (digits 0, 1) and the rest are rounded separately
        constexpr uint32_t offh = L == 6 ? 0x80808080u : 0x00808080u;
        uint32_t lo[4], hi[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float x = g[e] * gscale;
            const float H = rintf(x * (1.0f / 65536.0f));
            const float r = fmaf(-H, 65536.0f, x);          // exact, |r| <= 32768
            // r + 1.5 * 2^23 has unit spacing: its mantissa bits are those of the constant plus rint(r), ties to even
            const int t = (int)(__float_as_uint(r + 12582912.0f) + (0x8080u - 0x4B400000u));   // rint(r) + 0x8080, in [0x80, 0x10080]
            lo[e] = (uint32_t)t ^ 0x8080u;                  // bytes 0, 1: digits 0, 1
            const int h = (int)H + (t >> 16);               // carry out of the low two digits
            hi[e] = ((uint32_t)h + offh) ^ offh;
        }
        const uint32_t a0 = bperm(lo[1], lo[0], 0x05010400u), a2 = bperm(lo[3], lo[2], 0x05010400u);
        out[0] = bperm(a2, a0, 0x05040100u);
        out[1] = bperm(a2, a0, 0x07060302u);
        const uint32_t t0 = bperm(hi[1], hi[0], 0x05010400u), t2 = bperm(hi[3], hi[2], 0x05010400u);
        out[2] = bperm(t2, t0, 0x05040100u);
        out[3] = bperm(t2, t0, 0x07060302u);
        const uint32_t t1 = bperm(hi[1], hi[0], 0x07030602u), t3 = bperm(hi[3], hi[2], 0x07030602u);
        out[4] = bperm(t3, t1, 0x05040100u);
        if (L == 6) out[L - 1] = bperm(t3, t1, 0x07060302u);
    }
}

// One output tile is 32 rows x (4 waves x TN x 32) columns; every wave holds all L limb tiles of the
// 32 rows for its TN column tiles (one wave per SIMD, accumulators in the AGPRs).  A block takes
// `units_per_block` consecutive row tiles of one column tile (and one piece of the contraction) and
// runs them as ONE sequence of K-tile steps: the loads and conversions for the first K-tiles of the
// next row tile are already under way while the last K-tile of the current one is multiplied, so the
// start-up of a block (plan and argument loads, first G latency from HBM, LDS fill: about 9 us,
// measured) is paid once per block instead of once per output tile.  Per K-tile of 128 contraction
// entries:
//   A side: 16 entries of G per thread -> registers -> digits -> L planes [32][128] int8 in LDS;
//   B side: direct global->LDS loads of the index matrix rows (16-byte chunks, XOR-swizzled).
// Two LDS stages and two register sets for G.  While the MFMAs of step s run (four k-steps of L*TN
// MFMAs), the same wave
//   k-steps 0, 1: turns G(s+1), loaded two steps ago, into digit words (VALU only) and issues the second
//                 half of the direct loads of B(s+1),
//   k-step 2:     writes the digits to the other stage and issues the loads of G(s+3),
//   barrier       (step s+1 complete in LDS for everyone, every read of step s issued and done),
//   k-step 3:     reads the first fragments of step s+1 and issues the first half of the direct loads of
//                 B(s+2) into the stage step s has just left;
//   after the last K-tile of a row tile: recombination of the limbs and the stores of that tile.
// A wave runs its instructions in order: an MFMA occupies the matrix pipe for 32 cycles and about seven
// VALU or LDS instructions issued behind it are free (measured), more are not.  Hence the recipe per
// k-step below, which hands the scheduler the numbers of LDS, memory and VALU instructions per MFMA.
// Every k-step is one basic block: loads never branch (addresses are clamped, the index matrix is
// zero beyond the contraction length, so whatever G value is read there multiplies a zero), which
// lets the scheduler put the VALU and LDS work into the shadow of the MFMAs.
// TRANS: G is read transposed (rows of the product are columns of G).  VEC: 16-byte loads of G
// (N % 4 == 0).
template <int L, int TN, bool TRANS, bool VEC, bool LONG_RUNS, bool FUSED = false, bool QUANT = false, bool CONVG = false>
__device__ __forceinline__ void limb_gemm_body(const LimbArgs &a, int8_t *lds, float gscale, double out_scale)
{
    constexpr int NB = 4 * TN * 32;
    constexpr int STAGE = L * kLPlane + NB * kLBK;
    constexpr int WLB = NB / 32;          // direct loads per wave per K-tile
    constexpr int GL = VEC ? 4 : 16;      // G load instructions per thread per K-tile
    constexpr int NM = L * TN;            // MFMAs per k-step

    // RUNS: a block takes `units_per_block` consecutive row tiles and, for each of them, every column tile
    // in turn (the rows of G just read for one column tile are still in L2 for the next).  With five or six
    // limbs the accumulators fill the AGPRs and a write-out inside the loop makes the register allocator
    // spill in the k-steps: then, and when the launcher does not ask for runs, a block takes one row tile
    // and one column tile and writes it after the loop.
    constexpr bool RUNS = LONG_RUNS && L <= 4;
    const int tiles_c = (a.cols + NB - 1) / NB;
    const int R = RUNS ? a.units_per_block : 1;
    const int runs = (a.tiles_r + R - 1) / R;        // runs of row tiles per contraction piece
    const int c_per_block = RUNS ? tiles_c : 1;
    // Workgroups go to the eight XCDs round-robin: XCD x takes the x-th eighth of the work items, so that
    // neighbouring items (neighbouring rows of G, same K-tiles of the index matrix) share an L2.  The grid
    // may hold more blocks than items (it is sized before the limb count is known).
    const int64_t items = (int64_t)runs * (tiles_c / c_per_block) * a.splits;
    const int64_t per_xcd = (items + 7) >> 3;
    const int64_t slot = (int64_t)((int)blockIdx.x >> 3);
    const int64_t logical = (int64_t)((int)blockIdx.x & 7) * per_xcd + slot;
    if (slot >= per_xcd || logical >= items) return;
    const int c_begin = RUNS ? 0 : (int)(logical % tiles_c);
    const int64_t rest = RUNS ? logical : logical / tiles_c;
    const int run = (int)(rest % runs);
    const int split = (int)(rest / runs);
    const int nk_total = a.nk;
    const int kt0 = split * a.kt_per_split;
    const int nk = min(nk_total, kt0 + a.kt_per_split) - kt0;   // K-tiles per output tile (at least one)
    const int tile_r0 = run * R;
    const int U = min(R, a.tiles_r - tile_r0);                   // row tiles of this block
    const int S = U * c_per_block * nk;                          // steps

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- A side ----
    // Each thread owns four groups q = 0..3 of four consecutive contraction entries (one float4 of G, or
    // one column of a 4 x 4 patch of G^T), laid out so that one load instruction of a wave covers whole
    // 128-byte lines of G:
    // !TRANS: group q is row 8 q + tid / 32, entries 4 (tid % 32) .. +3
    //  TRANS: the patch is rows 4 t .. +3 by entries 4 j .. +3 with t = 0..7 and j = 0..7 inside the wave, j + 8 * wave in the
    //         block; group q is its row q.  t takes tid bits 0, 1 and 5, j bits 2..4: a half-wave then holds four values of
    //         t (four different swizzles) and all eight j (two chunks x four words), i.e. 32 different LDS banks when the
    //         digits are stored (with t in bits 0..2 rows t and t + 4 met in every bank: 19 % conflict cycles, measured).
    float gbuf[2][16];
    const int tr_t = (tid & 3) | ((tid >> 3) & 4), tr_j = ((tid >> 2) & 7) + 8 * (tid >> 6);
    const int ar = TRANS ? 4 * tr_t : (tid >> 5);            // row of group 0
    const int ak = TRANS ? 4 * tr_j : 4 * (tid & 31);        // first contraction entry inside the K-tile
    // (every address inside a tile is clamped to the matrix)
    // (r, kt): row tile inside the block and K-tile inside the contraction piece, both valid
    // CONVG (one row tile per block): the input pixel of each of the thread's four rows, as b * P * Q, h, w
    int cg_base[4] = {0, 0, 0, 0}, cg_h[4] = {0, 0, 0, 0}, cg_w[4] = {0, 0, 0, 0};
    if (CONVG) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int m = min(tile_r0 * kLRows + ar + 8 * q, a.rows - 1), hw = a.cg_H * a.cg_W;
            const int b = div_by(m, a.cg_mul_hw, a.cg_sh_hw), rem = m - b * hw;
            cg_h[q] = div_by(rem, a.cg_mul_w, a.cg_sh_w);
            cg_w[q] = rem - cg_h[q] * a.cg_W;
            cg_base[q] = b * a.cg_P * a.cg_Q;
        }
    }
    auto load_g = [&](float (&g)[16], int r, int kt) {
        const int row0 = (tile_r0 + r) * kLRows;
        const int k0 = (kt0 + kt) * kLBK + ak;
        if (CONVG) {
            // tap and channel of this thread's entries: k0 = tap * N + n0 (k0 < 2^17, so (k0 + 1/2) / N in fp32 is far
            // from a whole number on either side and truncates to the quotient; likewise tap / S)
            const int tap = (int)(((float)k0 + 0.5f) * a.cg_inv_n), n0 = k0 - tap * a.N;
            const int tr = (int)(((float)tap + 0.5f) * a.cg_inv_s), ts = tap - tr * a.cg_S;
            const int dh = a.cg_pad_h - tr, dw = a.cg_pad_w - ts;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int hh = cg_h[q] + dh, ww = cg_w[q] + dw;
                const bool ok = (unsigned)hh < (unsigned)a.cg_P && (unsigned)ww < (unsigned)a.cg_Q;
                const int64_t o = ok ? (int64_t)(cg_base[q] + hh * a.cg_Q + ww) * a.N + n0 : 0;
                const float4 v = *reinterpret_cast<const float4 *>(a.G + o);
                g[4 * q] = ok ? v.x : 0.0f; g[4 * q + 1] = ok ? v.y : 0.0f; g[4 * q + 2] = ok ? v.z : 0.0f; g[4 * q + 3] = ok ? v.w : 0.0f;
            }
        } else if (!TRANS) {
            // g[4 q + e] = G[row0 + ar + 8 q][k0 + e]
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float *p = a.G + (int64_t)min(row0 + ar + 8 * q, a.rows - 1) * a.N;
                if (VEC) {
                    const float4 v = *reinterpret_cast<const float4 *>(p + min(k0, a.kc - 4));
                    g[4 * q] = v.x; g[4 * q + 1] = v.y; g[4 * q + 2] = v.z; g[4 * q + 3] = v.w;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) g[4 * q + e] = p[min(k0 + e, a.kc - 1)];
                }
            }
        } else {
            // g[4 e + q] = G[k0 + e][row0 + ar + q]
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float *p = a.G + (int64_t)min(k0 + e, a.kc - 1) * a.N;
                if (VEC) {
                    const float4 v = *reinterpret_cast<const float4 *>(p + min(row0 + ar, a.rows - 4));
                    g[4 * e] = v.x; g[4 * e + 1] = v.y; g[4 * e + 2] = v.z; g[4 * e + 3] = v.w;
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q) g[4 * e + q] = p[min(row0 + ar + q, a.rows - 1)];
                }
            }
        }
    };
    // digit words of the four groups, w[q][l] = digit l of the group's four entries; two groups at a time
    uint32_t w[4][L];
    auto convert_half = [&](const float (&g)[16], int h) {
#pragma unroll
        for (int q = 2 * h; q < 2 * h + 2; ++q) {
            if constexpr (QUANT) {
                // the "digits" are the level indices of the quantizer (one plane): the forward product with the
                // quantizer in its prologue
                w[q][0] = pack_indices((int)anchor_level<true>(g[4 * q], a.fq_k), (int)anchor_level<true>(g[4 * q + 1], a.fq_k),
                                       (int)anchor_level<true>(g[4 * q + 2], a.fq_k), (int)anchor_level<true>(g[4 * q + 3], a.fq_k),
                                       a.fq_k.idx_off);
            } else if constexpr (!TRANS) {
                const float g4[4] = {g[4 * q], g[4 * q + 1], g[4 * q + 2], g[4 * q + 3]};
                limbs_of4<L>(g4, gscale, w[q]);
            } else {
                const float g4[4] = {g[q], g[4 + q], g[8 + q], g[12 + q]};
                limbs_of4<L>(g4, gscale, w[q]);
            }
        }
    };
    // where the word of group q goes inside a plane: row * 128 + (swizzled 16-byte chunk) + word in chunk.
    // The rows of a thread's groups are 8 apart from a row below 8 (!TRANS: the swizzle of rows +8, +24 is
    // that of row +0 with bit 2 flipped) or consecutive from a multiple of 4 (TRANS: rows +2, +3 flip bit 0).
    const int aw_row = ar * kLBK + ((ak >> 2) & 3) * 4;
    const int aw_chunk = ((ak >> 4) ^ lswz(ar)) << 4;
    auto store_digits = [&](int stage) {
        int8_t *base = lds + stage * STAGE + aw_row;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            int8_t *d = TRANS ? base + (q >> 1 ? aw_chunk ^ 16 : aw_chunk) + q * kLBK
                              : base + (q & 1 ? aw_chunk ^ 64 : aw_chunk) + q * 8 * kLBK;
#pragma unroll
            for (int l = 0; l < L; ++l) *reinterpret_cast<uint32_t *>(d + l * kLPlane) = w[q][l];
        }
    };

    // ---- B side: a uniform base per (column tile, K-tile) and a 32-bit offset per lane.  Load i of a wave
    // covers rows brow + 8 i of the column tile (clamped to the matrix), lane % 8 picks the 16-byte chunk,
    // XOR-swizzled with the row: the swizzle of row brow + 8 i is that of brow with bit 2 flipped for odd i. ----
    const int brow = wave * (WLB * 8) + (lane >> 3);
    const int bq16 = ((lane & 7) ^ lswz(brow)) << 4;
    const uint32_t ldb32 = (uint32_t)a.ldb;
    // half h of the direct loads of K-tile kt of column tile c: a wave that issues all of them back to back
    // outruns the address unit (1 KiB per instruction, 64 bytes per cycle per CU) and stalls behind its own loads
    auto issue_b = [&](int stage, int c, int kt, int h) {
        int8_t *base = lds + stage * STAGE + L * kLPlane + wave * (WLB * 1024);
        const int col0 = (c_begin + c) * NB;
        const int8_t *src = a.Bt + (int64_t)col0 * a.ldb + (int64_t)(kt0 + kt) * kLBK;
        const int lim = a.cols - 1 - col0;
#pragma unroll
        for (int i = h * (WLB / 2); i < (h + 1) * (WLB / 2); ++i) {
            const uint32_t off = (uint32_t)min(brow + 8 * i, lim) * ldb32 + (uint32_t)(i & 1 ? bq16 ^ 64 : bq16);
            __builtin_amdgcn_global_load_lds((gptr_t)(src + off), (lptr_t)(base + i * 1024), 16, 0, 0);
        }
    };

    // ---- fragments ----
    const int frow = lane & 31;
    const int fsw = lswz(frow);
    const int fa_off = frow * kLBK;
    const int fb_off = L * kLPlane + (wave * TN * 32 + frow) * kLBK;   // row 32 t + frow swizzles like frow
    int fc[4];                                                         // the 32-byte slice of k-step ks, per lane half
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) fc[ks] = ((2 * ks + (lane >> 5)) ^ fsw) << 4;

    v4i fa[2][L], fb[2][TN];
    auto read_frags = [&](int buf, int stage, int ks) {
        const int8_t *base = lds + stage * STAGE + fc[ks];
#pragma unroll
        for (int l = 0; l < L; ++l) fa[buf][l] = *reinterpret_cast<const v4i *>(base + l * kLPlane + fa_off);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[buf][j] = *reinterpret_cast<const v4i *>(base + fb_off + j * 32 * kLBK);
    };

    v16i acc[L][TN];
#pragma unroll
    for (int l = 0; l < L; ++l)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[l][j][r] = 0;
    auto mfma_all = [&](int buf) {
#pragma unroll
        for (int l = 0; l < L; ++l)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[l][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[buf][l], fb[buf][j], acc[l][j], 0, 0, 0);
    };

    // a bare s_barrier: the waits it needs are spelled out next to it, so that loads of later tiles stay in flight
    auto barrier = [&]() {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    // Scheduling recipe for one k-step: after every MFMA, up to `ds` LDS accesses, `vm` memory loads and
    // `va` VALU instructions go into its shadow.
#define CDL_INTERLEAVE(ds, vm, va)                                                          \
    _Pragma("unroll") for (int i_ = 0; i_ < NM; ++i_) {                                     \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                  \
        if ((ds) > 0) __builtin_amdgcn_sched_group_barrier(0x080, (ds), 0);                 \
        if ((vm) > 0) __builtin_amdgcn_sched_group_barrier(0x020, (vm), 0);                 \
        if ((va) > 0) __builtin_amdgcn_sched_group_barrier(0x002, (va), 0);                 \
    }
    constexpr int kDs2 = (L + TN + 4 * L + NM - 1) / NM;    // k-step 2: fragment reads + digit writes
    constexpr int kVm2 = (GL + NM - 1) / NM;
    // VALU instructions per MFMA: enough slots for the k-step's conversion work, spread as evenly as the
    // count allows (12 MFMAs and about 30 VALU instructions with up to four limbs: three each measured 2-3 %
    // faster than five, two slower; 15 MFMAs and the longer conversion of five limbs: five, four in the
    // k-steps that convert nothing)
    constexpr int kVaConv = L <= 4 ? 3 : 5, kVaRest = L <= 4 ? 3 : 4;

    // ---- recombination of the limbs of row tile u: the integers are exact, the Horner steps round at
    // 2^-53 relative.  (The lane index passes through an empty asm so that the output addresses are formed
    // here instead of being kept in registers all the way through the loop.) ----
    auto write_tile = [&](int r, int c) {
        int elane = lane;
        asm volatile("" : "+v"(elane));
        const int row0 = (tile_r0 + r) * kLRows, col0 = (c_begin + c) * NB;
        const int erow = row0 + 4 * (elane >> 5), ecol = col0 + wave * TN * 32 + (elane & 31);
        const bool full = row0 + kLRows <= a.rows && col0 + NB <= a.cols;
        // register rr of an accumulator is row 8 (rr / 4) + rr % 4 (+ 4 for the upper half of the lanes)
        auto combined = [&](int j, int rr) {
            double run = (double)acc[L - 1][j][rr];
#pragma unroll
            for (int l = L - 2; l >= 0; --l) run = __builtin_fma(run, 256.0, (double)acc[l][j][rr]);   // run * 256 is exact
            return run;
        };
        // one address per row, the TN column tiles of a wave at fixed distances from it; tiles that do not reach
        // the edge of the matrix (FULL) store without a test
        const int64_t first = (int64_t)erow * a.cols + ecol;
        const bool direct = a.splits == 1 && !a.to_partial;      // the block writes the finished fp32 output itself
        const bool corr = a.row_corr != nullptr && direct;
        // CORR: row corrections of an operand stored with an offset, in a copy of the write-out of their own.  A load
        // between the stores - even one that a branch skips - makes the compiler wait for every earlier store at each
        // row (loads and stores share one counter) and a store takes microseconds to complete: the common path must
        // not contain one (it cost dL/dQ(x) 5 %).  The copy with corrections loads one per row and pays for it; holding
        // all sixteen in registers instead pushed the five-limb kernels into spilling.
        auto emit = [&](auto full_c, auto corr_c, auto *base) {
            constexpr bool FULL = decltype(full_c)::value;
            constexpr bool CORR = decltype(corr_c)::value;
            using T = std::remove_pointer_t<decltype(base)>;
#pragma unroll
            for (int rr = 0; rr < 16; ++rr) {
                const int dr = 8 * (rr >> 2) + (rr & 3);
                T *p = base + (int64_t)dr * a.cols;
                const bool row_ok = FULL || erow + dr < a.rows;
                const double rc = (CORR && row_ok) ? a.row_corr[erow + dr] : 0.0;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if (FULL || (row_ok && ecol + j * 32 < a.cols)) {
                        if (QUANT) p[j * 32] = (T)(a.fq_scale * (float)acc[0][j][rr]);      // as the forward product rounds
                        else if (std::is_same<T, float>::value) p[j * 32] = (T)__builtin_fma(combined(j, rr), out_scale, rc);
                        else p[j * 32] = (T)combined(j, rr);
                    }
                }
            }
        };
        if (CONVG && a.cg_ostep != 1) {
            // the rows of a parity class lie scattered in the tensor: one address per row (no loads between the stores)
#pragma unroll
            for (int rr = 0; rr < 16; ++rr) {
                const int m = erow + 8 * (rr >> 2) + (rr & 3);
                if (m >= a.rows) continue;
                const int b = div_by(m, a.cg_mul_hw, a.cg_sh_hw), rem = m - b * (a.cg_H * a.cg_W);
                const int i = div_by(rem, a.cg_mul_w, a.cg_sh_w), jj = rem - i * a.cg_W;
                const int64_t pix = ((int64_t)b * a.cg_oH + a.cg_ostep * i + a.cg_oa) * a.cg_oW + a.cg_ostep * jj + a.cg_oc;
                float *p = a.out + pix * a.cols + ecol;
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    if (ecol + j * 32 < a.cols) p[j * 32] = (float)__builtin_fma(combined(j, rr), out_scale, 0.0);
            }
            return;
        }
        if (direct) {
            if (corr) {
                if (full) emit(std::true_type{}, std::true_type{}, a.out + first);
                else emit(std::false_type{}, std::true_type{}, a.out + first);
            } else {
                if (full) emit(std::true_type{}, std::false_type{}, a.out + first);
                else emit(std::false_type{}, std::false_type{}, a.out + first);
            }
        } else {
            double *base = a.partial + (int64_t)split * a.rows * a.cols + first;
            if (full) emit(std::true_type{}, std::false_type{}, base);
            else emit(std::false_type{}, std::false_type{}, base);
        }
    };


    // ---- the quantizer's backward pass in the epilogue (eq. partialX3, Jgradqx, Jgrad_alpha_q applied to the
    // tile of dL/dQ(x) while it is still on the chip): the recombined tile goes to LDS as fp32 (the stages are free
    // by now), then all threads walk it four entries at a time, load the matching entries of theta, evaluate the
    // band of the CPMF as the stand-alone kernel does, and store dL/dtheta; dL/dQ(x) itself is never written. ----
    auto fused_tile = [&]() {
        constexpr int NBP = NB + 4;           // row pitch in floats: the two half-waves of a store land 16 banks apart
        float *tile = reinterpret_cast<float *>(lds);
        const int row0 = tile_r0 * kLRows, col0 = c_begin * NB;
        constexpr int Q = NB / 4;             // groups of four columns per row
        const QConst &k = a.fq_k;
        // every thread takes T groups of four entries; all loads of theta are issued here, before the tile is
        // recombined and written to LDS (with one wave per SIMD nothing else hides their latency)
        constexpr int T = kLRows * Q / kLThreads;
        static_assert(T * kLThreads == kLRows * Q, "whole trips");
        // (row corrections of a weight operand stored with an offset: loaded first, in a branch of their own, so that the
        // common path has no load whose wait would also be a wait for the theta loads below)
        double rcs[16];
#pragma unroll
        for (int rr = 0; rr < 16; ++rr) rcs[rr] = 0.0;
        if (a.row_corr) {
            const int lrow0 = tile_r0 * kLRows + 4 * (lane >> 5);
#pragma unroll
            for (int rr = 0; rr < 16; ++rr) {
                const int dr = 8 * (rr >> 2) + (rr & 3);
                rcs[rr] = lrow0 + dr < a.rows ? a.row_corr[lrow0 + dr] : 0.0;
            }
        }
        float4 th4[T];
        bool ok[T];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int e4 = tid + t * kLThreads, row = e4 / Q, c4 = e4 - row * Q;
            const int grow = row0 + row, gcol = col0 + 4 * c4;
            ok[t] = grow < a.rows && gcol < a.cols;          // (cols % 4 == 0: a group is inside or outside)
            const int64_t o = (int64_t)min(grow, a.rows - 1) * a.cols + min(gcol, a.cols - 4);
            th4[t] = load_stream4(a.fq_theta + o, k.stream);
        }
        __builtin_amdgcn_s_waitcnt(kLgkmcnt0);
        barrier();                            // every wave has read its last fragments
        {
            const int lrow = 4 * (lane >> 5), lcol = wave * TN * 32 + (lane & 31);
#pragma unroll
            for (int rr = 0; rr < 16; ++rr) {
                const int dr = 8 * (rr >> 2) + (rr & 3);
                const double rc = rcs[rr];
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    double run = (double)acc[L - 1][j][rr];
#pragma unroll
                    for (int l = L - 2; l >= 0; --l) run = __builtin_fma(run, 256.0, (double)acc[l][j][rr]);
                    tile[(lrow + dr) * NBP + lcol + j * 32] = (float)__builtin_fma(run, out_scale, rc);
                }
            }
        }
        __syncthreads();
        double acc_d = 0.0, acc_a = 0.0;
        auto walk = [&](auto w_c) {
            constexpr int W = decltype(w_c)::value;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const int e4 = tid + t * kLThreads, row = e4 / Q, c4 = e4 - row * Q;
                const int grow = row0 + row, gcol = col0 + 4 * c4;
                const float4 v = *reinterpret_cast<const float4 *>(tile + row * NBP + 4 * c4);
                const float ge[4] = {v.x, v.y, v.z, v.w}, th[4] = {th4[t].x, th4[t].y, th4[t].z, th4[t].w};
                float dv[4], sum_d = 0.0f, sum_a = 0.0f;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float d_th, t_d, t_a;
                    quantizer_bwd_terms<W, true>(th[e], k, d_th, t_d, t_a);
                    dv[e] = ge[e] * d_th;
                    sum_d = fmaf(ge[e], t_d, sum_d);
                    sum_a = fmaf(ge[e], t_a, sum_a);
                }
                if (ok[t]) {
                    acc_d += (double)sum_d;
                    acc_a += (double)sum_a;
                    store_stream4(a.out + ((int64_t)grow * a.cols + gcol), dv[0], dv[1], dv[2], dv[3], k.stream);
                }
            }
        };
        switch (a.fq_wsel) {
            case 1: walk(std::integral_constant<int, 1>{}); break;
            case 2: walk(std::integral_constant<int, 2>{}); break;
            case 3: walk(std::integral_constant<int, 3>{}); break;
            case 4: walk(std::integral_constant<int, 4>{}); break;
            default: walk(std::integral_constant<int, 0>{}); break;
        }
        // partial sums of the block, in a fixed order
        __syncthreads();
        double *red = reinterpret_cast<double *>(lds);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            acc_d += __shfl_down(acc_d, off, 64);
            acc_a += __shfl_down(acc_a, off, 64);
        }
        if (lane == 0) { red[2 * wave] = acc_d; red[2 * wave + 1] = acc_a; }
        __syncthreads();
        if (tid == 0) {
            a.fq_partial[2 * logical] = (red[0] + red[2]) + (red[4] + red[6]);
            a.fq_partial[2 * logical + 1] = (red[1] + red[3]) + (red[5] + red[7]);
        }
    };

    // positions of the steps s, s+1, s+2, s+3 in the block's sequence: (row tile, column tile, K-tile), the
    // K-tile running fastest; past the end they stay on the last valid step (such loads go to registers or
    // to an LDS stage nobody reads)
    struct Pos { int r, c, kt; };
    auto advance = [&](Pos &q) {
        if (q.kt < nk - 1) { ++q.kt; }
        else if (q.c < c_per_block - 1) { q.kt = 0; ++q.c; }
        else if (q.r < U - 1) { q.kt = 0; q.c = 0; ++q.r; }
    };
    Pos p0{0, 0, 0}, p1 = p0;
    advance(p1);
    Pos p2 = p1;
    advance(p2);
    Pos p3 = p2;
    advance(p3);

    // k-step 0 of a step; FIRST: the first K-tile of a row tile starts from zero accumulators
    auto kstep0 = [&](auto parity, auto first) {
        constexpr int P = decltype(parity)::value;
        constexpr bool FIRST = decltype(first)::value;
        read_frags(1, P, 1);
        issue_b(P ^ 1, p1.c, p1.kt, 1);
        convert_half(gbuf[P ^ 1], 0);
        if (FIRST) {
            const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int l = 0; l < L; ++l)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[l][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[0][l], fb[0][j], zero, 0, 0, 0);
        } else {
            mfma_all(0);
        }
        CDL_INTERLEAVE(1, 1, kVaConv)
        __builtin_amdgcn_sched_barrier(0);
    };
    // one step (its parity P picks the LDS stage and the register set of G) under the schedule above
    auto step = [&](auto parity) {
        constexpr int P = decltype(parity)::value;
        // k-step 0
        if (RUNS && p0.kt == 0) kstep0(parity, std::true_type{});
        else kstep0(parity, std::false_type{});
        // k-step 1
        read_frags(0, P, 2);
        convert_half(gbuf[P ^ 1], 1);
        mfma_all(1);
        CDL_INTERLEAVE(1, 0, kVaConv)
        __builtin_amdgcn_sched_barrier(0);
        // k-step 2
        store_digits(P ^ 1);
        read_frags(1, P, 3);
        load_g(gbuf[P ^ 1], p3.r, p3.kt);
        mfma_all(0);
        CDL_INTERLEAVE(kDs2, kVm2, kVaRest)
        __builtin_amdgcn_sched_barrier(0);
        // B(s+1) has landed (younger loads: G(s+3)); own LDS writes and fragment reads are done
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(GL));
        __builtin_amdgcn_s_waitcnt(kLgkmcnt0);
        barrier();
        // k-step 3
        read_frags(0, P ^ 1, 0);
        issue_b(P, p2.c, p2.kt, 0);
        mfma_all(1);
        CDL_INTERLEAVE(1, 1, kVaRest)
        __builtin_amdgcn_sched_barrier(0);
        if (RUNS && p0.kt == nk - 1) write_tile(p0.r, p0.c);
        advance(p0);
        advance(p1);
        advance(p2);
        advance(p3);
    };

    load_g(gbuf[0], p0.r, p0.kt);
    load_g(gbuf[1], p1.r, p1.kt);
    issue_b(0, p0.c, p0.kt, 0);
    issue_b(0, p0.c, p0.kt, 1);
    convert_half(gbuf[0], 0);
    convert_half(gbuf[0], 1);
    store_digits(0);
    asm volatile("" ::: "memory");
    load_g(gbuf[0], p2.r, p2.kt);
    issue_b(1, p1.c, p1.kt, 0);
    asm volatile("" ::: "memory");
    // B(0) has landed (younger loads: G(2), the first half of B(1)); own LDS writes are done
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(GL + WLB / 2));
    __builtin_amdgcn_s_waitcnt(kLgkmcnt0);
    barrier();
    read_frags(0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    int st = 0;
    for (; st + 1 < S; st += 2) {
        step(std::integral_constant<int, 0>{});
        step(std::integral_constant<int, 1>{});
    }
    if (st < S) step(std::integral_constant<int, 0>{});
    // the loads issued for steps past the end write LDS: they must be done before this wave ends
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
#undef CDL_INTERLEAVE
    if (!RUNS) {
        if (FUSED) fused_tile();
        else write_tile(0, 0);
    }
}

template <bool TRANS, bool LONG_RUNS, bool FUSED = false>
__global__ __launch_bounds__(kLThreads, 1)
void limb_gemm_kernel(LimbArgs a)
{
    extern __shared__ __attribute__((aligned(16))) int8_t limb_lds[];
    const bool vec = (a.N & 3) == 0;
    const int limbs = a.which == 0 ? a.plan->limbs_da : a.plan->limbs_db;
    const float gscale = a.which == 0 ? a.plan->gscale_da : a.plan->gscale_db;
    const double out_scale = a.which == 0 ? a.plan->out_scale_da : a.plan->out_scale_db;
    switch (limbs) {
        case 3: if (vec) limb_gemm_body<3, 3, TRANS, true, LONG_RUNS, FUSED>(a, limb_lds, gscale, out_scale); else limb_gemm_body<3, 3, TRANS, false, LONG_RUNS, FUSED>(a, limb_lds, gscale, out_scale); break;
        case 4: if (vec) limb_gemm_body<4, 3, TRANS, true, LONG_RUNS, FUSED>(a, limb_lds, gscale, out_scale); else limb_gemm_body<4, 3, TRANS, false, LONG_RUNS, FUSED>(a, limb_lds, gscale, out_scale); break;
        case 5: if (vec) limb_gemm_body<5, 3, TRANS, true, false, FUSED>(a, limb_lds, gscale, out_scale); else limb_gemm_body<5, 3, TRANS, false, false, FUSED>(a, limb_lds, gscale, out_scale); break;
        default: if (vec) limb_gemm_body<6, 2, TRANS, true, false, FUSED>(a, limb_lds, gscale, out_scale); else limb_gemm_body<6, 2, TRANS, false, false, FUSED>(a, limb_lds, gscale, out_scale); break;
    }
}

// dL/dQ(x) of a convolutional layer: the activation-gradient product with the rows of g gathered by taps (CONVG),
// one row tile of 32 input pixels per block.  TN = column tiles per wave, chosen by the launcher: channel counts are
// powers of two, and 256 or 512 output columns in tiles of 384 would spend a third of the MFMAs on padding.  With one
// column tile per wave (up to 128 channels: the first stages of a network) a K-tile has only 4 L MFMAs per wave, fewer
// cycles than a load takes to come back, and the loop runs at one memory round trip per K-tile: that kernel is held to
// 256 registers and asks for 80 KiB of LDS, so that two blocks share a compute unit and fill each other's waits.
constexpr int conv_dx_lds_bytes(int tn)
{
    return tn == 3 ? kLimbLdsBytes : 2 * (kMaxLimbs * kLPlane + 4 * tn * 32 * kLBK);
}

template <int TN>
__global__ __launch_bounds__(kLThreads, TN == 1 ? 2 : 1)
void limb_conv_dx_kernel(LimbArgs a)
{
    extern __shared__ __attribute__((aligned(16))) int8_t limb_lds[];
    const int limbs = a.plan->limbs_da;
    const float gscale = a.plan->gscale_da;
    const double out_scale = a.plan->out_scale_da;
#define CDL_CONV_DX(L, T) limb_gemm_body<L, T, false, true, false, false, false, true>(a, limb_lds, gscale, out_scale)
    switch (limbs) {
        case 3: CDL_CONV_DX(3, TN); break;
        case 4: CDL_CONV_DX(4, TN); break;
        case 5: CDL_CONV_DX(5, TN); break;
        default: CDL_CONV_DX(6, (TN < 2 ? TN : 2)); break;
    }
#undef CDL_CONV_DX
}

// dL/dQ(x) of a convolutional layer with few channels on both sides (the first stages of a small CNN: 16 -> 16 channels,
// 3 x 3: a contraction of 144 entries and 16 output columns, of which the limb kernel's 32 x 384 tiles would be nine
// tenths padding): one thread per output entry (input pixel, channel c), the weights as doubles in LDS ([tap][n][c], so
// that the lanes of a pixel read neighbouring words), every output a chain of at most R*S*N fused multiply-adds in
// double - products of a float and an int8 are exact there, the additions round at 2^-53 relative.  CC: channels per
// pixel padded to 16 or 32 lanes.
template <int CC>
__global__ __launch_bounds__(256)
void conv_dx_direct_kernel(const float *__restrict__ g, const int8_t *__restrict__ w, int B, int H, int W, int C, int N,
                           int R, int S, int stride, int pad, int P, int Q, double delta_w, float *__restrict__ out)
{
    extern __shared__ double conv_wl[];      // [R*S*N][CC]
    const int kc = R * S * N;
    for (int i = threadIdx.x; i < kc * CC; i += 256) {
        const int k = i / CC, c = i - k * CC, tap = k / N, n = k - tap * N;
        conv_wl[i] = c < C ? (double)w[((int64_t)n * R * S + tap) * C + c] : 0.0;
    }
    __syncthreads();
    // a thread takes one channel of kPer consecutive pixels: every weight it reads from LDS serves kPer outputs
    constexpr int kPer = 4;
    constexpr int PIX = 256 / CC * kPer;
    const int c = threadIdx.x % CC, pl = threadIdx.x / CC;
    const int64_t pixels = (int64_t)B * H * W;
    const int hw = H * W;
    for (int64_t pix0 = (int64_t)blockIdx.x * PIX + pl * kPer; pix0 < pixels; pix0 += (int64_t)gridDim.x * PIX) {
        int pb[kPer], ph[kPer], px[kPer];
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int64_t pix = min(pix0 + i, pixels - 1);
            pb[i] = (int)(pix / hw);
            const int rem = (int)(pix - (int64_t)pb[i] * hw);
            ph[i] = rem / W;
            px[i] = rem - ph[i] * W;
        }
        double acc[kPer] = {0.0, 0.0, 0.0, 0.0};
        for (int r = 0; r < R; ++r) {
            for (int t = 0; t < S; ++t) {
                const float4 *gp[kPer];
                bool ok[kPer];
                bool any = false;
#pragma unroll
                for (int i = 0; i < kPer; ++i) {
                    int hh = ph[i] + pad - r, ww = px[i] + pad - t;
                    ok[i] = hh >= 0 && ww >= 0;
                    if (stride == 2) { ok[i] = ok[i] && ((hh | ww) & 1) == 0; hh >>= 1; ww >>= 1; }
                    ok[i] = ok[i] && hh < P && ww < Q;
                    gp[i] = reinterpret_cast<const float4 *>(g + (ok[i] ? (((int64_t)pb[i] * P + hh) * Q + ww) * N : 0));
                    any = any || ok[i];
                }
                if (!any) continue;
                const double *wp = conv_wl + (int64_t)((r * S + t) * N) * CC + c;
                for (int n4 = 0; n4 < N / 4; ++n4) {
                    float4 v[kPer];
#pragma unroll
                    for (int i = 0; i < kPer; ++i) {
                        v[i] = gp[i][n4];
                        if (!ok[i]) v[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                    }
                    const double w0 = wp[(4 * n4) * CC], w1 = wp[(4 * n4 + 1) * CC], w2 = wp[(4 * n4 + 2) * CC], w3 = wp[(4 * n4 + 3) * CC];
#pragma unroll
                    for (int i = 0; i < kPer; ++i) {
                        acc[i] = fma((double)v[i].x, w0, acc[i]);
                        acc[i] = fma((double)v[i].y, w1, acc[i]);
                        acc[i] = fma((double)v[i].z, w2, acc[i]);
                        acc[i] = fma((double)v[i].w, w3, acc[i]);
                    }
                }
            }
        }
        if (c < C) {
#pragma unroll
            for (int i = 0; i < kPer; ++i)
                if (pix0 + i < pixels) out[(pix0 + i) * C + c] = (float)(acc[i] * delta_w);
        }
    }
}

// For that product: the weights [N][R][S][C] rearranged as its index operand Wr[c][(r', s', n)] (contraction index
// contiguous, rows ld bytes apart, zero beyond the contraction length) and the sum of |w| over the contraction per
// channel c (the limb rule's column sums).  One rearrangement per class of taps (blockIdx.y): the taps
// (r0 + tstep r', s0 + tstep s') with r' < Rc, s' < Sc - all of them for stride 1 (one class, tstep = 1), those of one
// parity for stride 2.
struct ConvDxClass { int r0, s0, Rc, Sc; };
struct ConvDxClasses { ConvDxClass c[4]; int tstep; };

__global__ __launch_bounds__(256)
void conv_dx_prep_kernel(const int8_t *__restrict__ w, int N, int R, int S, int C, ConvDxClasses cls, int8_t *__restrict__ wr, int64_t ld,
                         unsigned int *__restrict__ col_abs)
{
    // one block per input channel c and class; four entries per thread and trip (one 4-byte store): the byte loads are a
    // stride of C apart and nothing but latency, so as many of them as possible are in flight
    __shared__ unsigned int red[4];
    const ConvDxClass k_ = cls.c[blockIdx.y];
    const int kc = k_.Rc * k_.Sc * N;
    const int c = blockIdx.x;
    int8_t *dst = wr + ((int64_t)blockIdx.y * C + c) * ld;
    unsigned int s_abs = 0u;
    for (int k4 = threadIdx.x * 4; k4 < (int)ld; k4 += 1024) {
        int v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int k = k4 + e, kk = min(k, kc - 1), tap = kk / N, n = kk - tap * N;
            const int tr = tap / k_.Sc, ts = tap - tr * k_.Sc;
            const int r = k_.r0 + cls.tstep * tr, sx = k_.s0 + cls.tstep * ts;
            const int x = (int)w[(((int64_t)n * R + r) * S + sx) * C + c];
            v[e] = k < kc ? x : 0;
        }
        *reinterpret_cast<uint32_t *>(dst + k4) =
            (uint32_t)(v[0] & 0xff) | ((uint32_t)(v[1] & 0xff) << 8) | ((uint32_t)(v[2] & 0xff) << 16) | ((uint32_t)(v[3] & 0xff) << 24);
#pragma unroll
        for (int e = 0; e < 4; ++e) s_abs += (unsigned int)(v[e] < 0 ? -v[e] : v[e]);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s_abs += (unsigned int)__shfl_down((int)s_abs, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s_abs;
    __syncthreads();
    if (threadIdx.x == 0) col_abs[blockIdx.y * C + c] = (red[0] + red[1]) + (red[2] + red[3]);
}

// The forward product with the quantizer of the activations in its prologue: y = delta_a delta_b (Q_idx(X) . Wi^T)
// where Q_idx(X) - the level indices cdl_quantize_fwd would store - exists only as one int8 plane per K-tile in LDS.
// The limb kernel's loop with the conversion to digits replaced by the nearest-level rule, one plane, four column
// tiles per wave (512 columns per block), runs of row tiles per block.
constexpr int kQuantFwdTN = 4;
static_assert(2 * (kLPlane + 4 * kQuantFwdTN * 32 * kLBK) <= kLimbLdsBytes, "LDS of the limb kernels serves");

__global__ __launch_bounds__(kLThreads, 1)
void qgemm_quantize_fwd_kernel(LimbArgs a)
{
    extern __shared__ __attribute__((aligned(16))) int8_t limb_lds[];
    limb_gemm_body<1, kQuantFwdTN, false, true, true, false, true>(a, limb_lds, 0.0f, 0.0);
}

// out = out_scale * sum over the contraction splits.  Four partial sums per lane, combined in a fixed order,
// keep four loads in flight: with a few hundred splits a single dependent chain is all latency.  LANES lanes
// share one output (lane j takes the splits j, j + LANES, ...; butterfly over the lanes at the end): used
// when there are few outputs and many splits, where one lane per output leaves most of the chip idle.
template <int LANES>
__global__ __launch_bounds__(256)
void limb_reduce_kernel(const double *__restrict__ partial, int splits, int64_t n, const BwdPlan *plan, float *__restrict__ out,
                        const double *__restrict__ row_corr /* [n / cols] or null */, int cols)
{
    const double out_scale = plan->out_scale_db;
    const int sub = threadIdx.x % LANES;
    const int64_t per_block = 256 / LANES;
    // whole groups of LANES run every trip (the index is clamped), so that the shuffles see all their lanes
    const int64_t n_round = (n + per_block - 1) / per_block * per_block;
    for (int64_t i = (int64_t)blockIdx.x * per_block + threadIdx.x / LANES; i < n_round; i += (int64_t)gridDim.x * per_block) {
        const int64_t ii = i < n ? i : n - 1;
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
        int p = sub;
        for (; p + 3 * LANES < splits; p += 4 * LANES) {
            s0 += partial[(int64_t)p * n + ii];
            s1 += partial[(int64_t)(p + LANES) * n + ii];
            s2 += partial[(int64_t)(p + 2 * LANES) * n + ii];
            s3 += partial[(int64_t)(p + 3 * LANES) * n + ii];
        }
        for (; p < splits; p += LANES) s0 += partial[(int64_t)p * n + ii];
        double s = (s0 + s1) + (s2 + s3);
#pragma unroll
        for (int off = LANES / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
        if (sub == 0 && i < n) out[i] = (float)__builtin_fma(s, out_scale, row_corr ? row_corr[i / cols] : 0.0);
    }
}

// limb_reduce_kernel<1> followed by the quantizer's backward pass on its output (Lemma 1; eq. partialW3, Jgradqw,
// Jgradq_alpha_w): an entry of dL/dQ(w) is formed exactly as above, rounded to fp32 as above, optionally stored, and
// multiplied by the partials of the quantizer at the matching entry of theta - the arithmetic of the stand-alone
// backward kernel, on the same fp32 value it would have read back.  Partial scalar gradients: one pair per block.
template <int W>
__global__ __launch_bounds__(256)
void limb_reduce_quantize_bwd_kernel(const double *__restrict__ partial, int splits, int64_t n, const BwdPlan *plan,
                                     float *__restrict__ d_hat /* nullable */, const double *__restrict__ row_corr, int cols,
                                     const float *__restrict__ theta, QConst k, float *__restrict__ d_theta,
                                     double *__restrict__ fq_partial /* [gridDim.x][2] */)
{
    const double out_scale = plan->out_scale_db;
    double acc_d = 0.0, acc_a = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
        int p = 0;
        for (; p + 3 < splits; p += 4) {
            s0 += partial[(int64_t)p * n + i];
            s1 += partial[(int64_t)(p + 1) * n + i];
            s2 += partial[(int64_t)(p + 2) * n + i];
            s3 += partial[(int64_t)(p + 3) * n + i];
        }
        for (; p < splits; ++p) s0 += partial[(int64_t)p * n + i];
        const double s = (s0 + s1) + (s2 + s3);
        const float ge = (float)__builtin_fma(s, out_scale, row_corr ? row_corr[i / cols] : 0.0);
        if (d_hat) d_hat[i] = ge;
        float d_th, t_d, t_a;
        quantizer_bwd_terms<W, true>(theta[i], k, d_th, t_d, t_a);
        d_theta[i] = ge * d_th;
        acc_d += (double)(ge * t_d);
        acc_a += (double)(ge * t_a);
    }
    __shared__ double red[8];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        acc_d += __shfl_down(acc_d, off, 64);
        acc_a += __shfl_down(acc_a, off, 64);
    }
    if ((threadIdx.x & 63) == 0) { red[2 * (threadIdx.x >> 6)] = acc_d; red[2 * (threadIdx.x >> 6) + 1] = acc_a; }
    __syncthreads();
    if (threadIdx.x == 0) {
        fq_partial[2 * (size_t)blockIdx.x] = (red[0] + red[2]) + (red[4] + red[6]);
        fq_partial[2 * (size_t)blockIdx.x + 1] = (red[1] + red[3]) + (red[5] + red[7]);
    }
}

// dL/dQ(a) for a very short contraction (N <= 32: the first stages of a small CNN have 16 or 32 output
// channels): d_a_hat[m][k] = delta_b * sum_n g[m][n] * b_idx[n][k].  One K-tile of the limb kernel would be
// at least three quarters padding there; here a block takes 128 or 64 rows of g (kept in LDS as doubles), a thread
// C neighbouring output columns, whose N index values each it keeps in registers as doubles, and every output
// is a chain of N fused multiply-adds in double: products of a float and an int8 are exact in double and N <= 32
// additions round at 2^-53 relative.  The threads of a block are spread over (group of C columns, row group):
// with one column per thread and 256 columns per block, 144 columns (workload 2) left 112 threads of every
// block idle (35 us; 28 us now); C columns per thread use each value read from LDS C times and load the C index
// bytes of a row of b_idx as one word.
constexpr int kDirectMaxN = 32;
constexpr int direct_rows(int nn) { return 2048 / nn; }     // rows of g per block: 16 KiB of LDS as doubles

template <int NN, int C>
__global__ __launch_bounds__(256)
void da_direct_kernel(const float *__restrict__ g, const int8_t *__restrict__ b_idx, int M, int N, int K,
                      double delta_b, double b_offset, float *__restrict__ out, int vec_store)
{
    constexpr int kRows = direct_rows(NN);
    __shared__ double gs[kRows][NN];
    const int row0 = blockIdx.x * kRows;
    const int rows = min(kRows, M - row0);
    const int groups_total = (K + C - 1) / C;              // groups of C columns
    const int gpb = min(groups_total, 256);                // of them per block
    const int row_groups = 256 / gpb;
    const int cg = blockIdx.y * gpb + (int)threadIdx.x % gpb, rg = (int)threadIdx.x / gpb;
    for (int i = threadIdx.x; i < kRows * NN; i += 256) {
        const int r = i / NN, n = i - r * NN;
        gs[r][n] = (r < rows && n < N) ? (double)g[(int64_t)(row0 + r) * N + n] : 0.0;
    }
    const bool active = cg < groups_total && rg < row_groups;
    double b[C][NN];
    if (C == 4 && vec_store) {
        // (K % 4 == 0: the four index bytes of a row of b_idx in one load)
#pragma unroll
        for (int n = 0; n < NN; ++n) {
            const uint32_t w4 = (active && n < N) ? *reinterpret_cast<const uint32_t *>(b_idx + (int64_t)n * K + cg * C) : 0u;
#pragma unroll
            for (int c = 0; c < C; ++c) b[c][n] = (active && n < N) ? (double)(int8_t)(w4 >> (8 * c)) + b_offset : 0.0;
        }
    } else {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const int k = cg * C + c;
#pragma unroll
            for (int n = 0; n < NN; ++n) b[c][n] = (active && n < N && k < K) ? (double)b_idx[(int64_t)n * K + k] + b_offset : 0.0;   // (the level index itself)
        }
    }
    __syncthreads();
    if (!active) return;
    const int k0 = cg * C;
    for (int r = rg; r < rows; r += row_groups) {
        double acc[C];
#pragma unroll
        for (int c = 0; c < C; ++c) acc[c] = 0.0;
#pragma unroll
        for (int n = 0; n < NN; ++n) {
            const double gv = gs[r][n];
#pragma unroll
            for (int c = 0; c < C; ++c) acc[c] = fma(gv, b[c][n], acc[c]);
        }
        float *o = out + (int64_t)(row0 + r) * K + k0;
        if (C == 4 && vec_store) {
            *reinterpret_cast<float4 *>(o) = make_float4((float)(acc[0] * delta_b), (float)(acc[1] * delta_b), (float)(acc[2] * delta_b), (float)(acc[3] * delta_b));
        } else {
#pragma unroll
            for (int c = 0; c < C; ++c)
                if (k0 + c < K) o[c] = (float)(acc[c] * delta_b);
        }
    }
}

// out[r] = mult * sum_k idx[r][k] + add for an int8 matrix [rows][K]: the corrections of a product whose
// other operand is stored with an offset.  One wave per row, 4 bytes per lane and trip.
__global__ __launch_bounds__(256) void index_rowsum_kernel(const int8_t *__restrict__ idx, int rows, int K, int mult, int add,
                                                           int32_t *__restrict__ out)
{
    const int lane = threadIdx.x & 63;
    for (int r = blockIdx.x * 4 + (threadIdx.x >> 6); r < rows; r += gridDim.x * 4) {
        const int8_t *p = idx + (int64_t)r * K;
        int s = 0;
        for (int k = lane; k < K; k += 64) s += (int)p[k];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
        if (lane == 0) out[r] = mult * s + add;
    }
}

// Row sums of the fp32 gradient g [M][N] in double, times `mult`: out[m] = mult * sum_n g[m][n].  One wave per row.
__global__ __launch_bounds__(256) void g_rowsum_kernel(const float *__restrict__ g, int M, int N, double mult, double *__restrict__ out)
{
    const int lane = threadIdx.x & 63;
    for (int m = blockIdx.x * 4 + (threadIdx.x >> 6); m < M; m += gridDim.x * 4) {
        const float *p = g + (int64_t)m * N;
        double s = 0.0;
        for (int n = lane; n < N; n += 64) s += (double)p[n];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
        if (lane == 0) out[m] = mult * s;
    }
}

// Column sums of g [M][N]: block b adds rows b * rows_per .. of every column into partial[b][N] (a thread walks its
// columns down the rows, neighbouring threads read neighbouring columns); g_colsum_finish adds the blocks in a
// fixed order and multiplies by `mult`.
constexpr int kColsumBlocks = 512;

__global__ __launch_bounds__(256) void g_colsum_kernel(const float *__restrict__ g, int M, int N, int rows_per, double *__restrict__ partial)
{
    const int m0 = blockIdx.x * rows_per, m1 = min(M, m0 + rows_per);
    for (int n = threadIdx.x; n < N; n += 256) {
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
        int m = m0;
        for (; m + 3 < m1; m += 4) {
            s0 += (double)g[(int64_t)m * N + n];
            s1 += (double)g[(int64_t)(m + 1) * N + n];
            s2 += (double)g[(int64_t)(m + 2) * N + n];
            s3 += (double)g[(int64_t)(m + 3) * N + n];
        }
        for (; m < m1; ++m) s0 += (double)g[(int64_t)m * N + n];
        partial[(int64_t)blockIdx.x * N + n] = (s0 + s1) + (s2 + s3);
    }
}

__global__ __launch_bounds__(256) void g_colsum_finish_kernel(const double *__restrict__ partial, int blocks, int N, double mult, double *__restrict__ out)
{
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    double s = 0.0;
    for (int b = 0; b < blocks; ++b) s += partial[(int64_t)b * N + n];
    out[n] = mult * s;
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

// max |g| per block (as fp32 bits: non-negative floats order like unsigned ints): each block streams
// contiguous pieces, eight independent 16-byte loads per thread and trip.  One plain store per block -
// thousands of atomics on one address would take longer than the pass itself.
__global__ __launch_bounds__(256) void absmax_kernel(const float *__restrict__ g, int64_t n, unsigned int *__restrict__ block_max,
                                                     unsigned int *__restrict__ clear, int n_clear)
{
    // (the transposition kernels that follow on the stream add into these words)
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i < n_clear; i += 256) clear[i] = 0u;
    __shared__ unsigned int wave_max[4];
    unsigned int m = 0u;
    const int64_t n4 = n >> 2;
    const float4 *g4 = reinterpret_cast<const float4 *>(g);
    for (int64_t base = (int64_t)blockIdx.x * 2048; base < n4; base += (int64_t)gridDim.x * 2048) {
        float4 t[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int64_t v = base + j * 256 + threadIdx.x;
            t[j] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (v < n4) {
                // streaming loads (183 -> 122 us on 805 MB): g is far larger than the last-level cache, and the
                // index matrices that the products read next should stay there
                t[j] = load_stream4(reinterpret_cast<const float *>(g4 + v));
            }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            m = max(m, __float_as_uint(fabsf(t[j].x)));
            m = max(m, __float_as_uint(fabsf(t[j].y)));
            m = max(m, __float_as_uint(fabsf(t[j].z)));
            m = max(m, __float_as_uint(fabsf(t[j].w)));
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0)
        for (int64_t e = n4 << 2; e < n; ++e) m = max(m, __float_as_uint(fabsf(g[e])));
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = max(m, (unsigned int)__shfl_down((int)m, off, 64));
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) block_max[blockIdx.x] = max(max(wave_max[0], wave_max[1]), max(wave_max[2], wave_max[3]));
}

// dst[c][r] = src[r][c] for an int8 matrix [rows][cols]; dst rows are ldd bytes apart and are
// zero-filled from `rows` up to the next multiple of 128.  Also adds, for every column c of src, the sum of
// |src[r][c]| over the block's rows to col_abs[c] (one atomic per column and block; the array is cleared by the
// max|g| kernel that runs first): the largest of these sums bounds what the rounding of g can do to one output of
// the product that contracts over r, see plan_kernel.  One block moves a tile of 128 rows x
// 64 columns: 4-byte loads along the rows into LDS (row stride 17 words), then every thread takes a
// 4 x 4 byte block, transposes it in registers and stores 4 bytes of four output rows, so that 32
// lanes write 128 contiguous bytes.  VEC: cols % 4 == 0 (aligned 4-byte loads).
// CONV: src is not a matrix but the activations of a convolutional layer, [B][H][W][C] with C a multiple of 16, and
// "src[r][c]" is entry c = (tap row, tap column, channel) of the window of output pixel r = (b, p, q) - the matrix of
// input windows, which is never stored the right way round: only its transpose is written, as the product that
// contracts over the pixels needs it.  Taps outside the image read as geom.pad_word (the stored byte of level index 0).
struct ConvGeom {
    int B, H, W, C, R, S, stride, pad, P, Q;
    int pad_word;
};

template <bool VEC, bool CONV = false>
__global__ __launch_bounds__(256) void transpose_i8_kernel(const int8_t *__restrict__ src, int rows, int cols,
                                                           int8_t *__restrict__ dst, int64_t ldd,
                                                           unsigned int *__restrict__ col_abs, int tiles_per_block, ConvGeom geom)
{
    __shared__ uint32_t tile[128 * 17];
    __shared__ unsigned int abs_s[64];
    __shared__ int row_h0[128], row_w0[128], row_off[128];     // CONV: window origin of the tile's rows
    const int c0 = blockIdx.y * 64;   // neighbouring blocks write neighbouring 128-byte pieces
    const int tid = threadIdx.x;
    if (tid < 64) abs_s[tid] = 0u;
    // A block takes `tiles_per_block` consecutive row tiles of its 64 columns and keeps the column sums of |x| in
    // registers across them: one atomic per column and BLOCK on col_abs (with one per tile the 512 row tiles of
    // workload 5's activations queued 512 atomics on every address and doubled the kernel's time).
    unsigned int part[2][4] = {};
    const int row_tiles = (rows + 127) / 128;
    const int t_end = min(row_tiles, ((int)blockIdx.x + 1) * tiles_per_block);
    // CONV: the thread's column (the same in all its loads) as a tap and an offset from the window's origin
    int tap_r = 0, tap_s = 0, tap_off = 0;
    if (CONV) {
        const int c = min(c0 + 4 * (tid & 15), cols - 4);
        const int tap = c / geom.C;
        tap_r = tap / geom.S;
        tap_s = tap - tap_r * geom.S;
        tap_off = (tap_r * geom.W + tap_s) * geom.C + (c - tap * geom.C);
    }
    for (int rt = (int)blockIdx.x * tiles_per_block; rt < t_end; ++rt) {
        const int r0 = rt * 128;
        if (CONV) {
            if (tid < 128) {
                const int m = min(r0 + tid, rows - 1), pq = geom.P * geom.Q;
                const int b = m / pq, rem = m - b * pq, p = rem / geom.Q, q = rem - p * geom.Q;
                const int h0 = p * geom.stride - geom.pad, w0 = q * geom.stride - geom.pad;
                row_h0[tid] = h0;
                row_w0[tid] = w0;
                row_off[tid] = ((b * geom.H + h0) * geom.W + w0) * geom.C;      // (host: B*H*W*C < 2^31)
            }
            __syncthreads();
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int i = tid + 256 * j, row = i >> 4, cd = i & 15;
            uint32_t w = 0u;
            const int r = r0 + row, c = c0 + 4 * cd;
            if (CONV) {
                if (r < rows && c < cols) {
                    const bool inside = (unsigned)(row_h0[row] + tap_r) < (unsigned)geom.H && (unsigned)(row_w0[row] + tap_s) < (unsigned)geom.W;
                    w = inside ? *reinterpret_cast<const uint32_t *>(src + ((int64_t)row_off[row] + tap_off)) : (uint32_t)geom.pad_word;
                }
            } else if (r < rows) {
                const int8_t *p = src + (int64_t)r * cols + c;
                if (VEC) {
                    if (c < cols) w = *reinterpret_cast<const uint32_t *>(p);
                } else {
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        if (c + b < cols) w |= (uint32_t)(uint8_t)p[b] << (8 * b);
                }
            }
            tile[row * 17 + cd] = w;
        }
        __syncthreads();
        const int rg = tid & 31;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int cg = (tid >> 5) + 8 * p;
            const uint32_t d0 = tile[(4 * rg) * 17 + cg], d1 = tile[(4 * rg + 1) * 17 + cg];
            const uint32_t d2 = tile[(4 * rg + 2) * 17 + cg], d3 = tile[(4 * rg + 3) * 17 + cg];
            const uint32_t t0 = bperm(d1, d0, 0x05010400u), t2 = bperm(d3, d2, 0x05010400u);
            const uint32_t t1 = bperm(d1, d0, 0x07030602u), t3 = bperm(d3, d2, 0x07030602u);
            const uint32_t o[4] = {bperm(t2, t0, 0x05040100u), bperm(t2, t0, 0x07060302u),
                                   bperm(t3, t1, 0x05040100u), bperm(t3, t1, 0x07060302u)};
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int c = c0 + 4 * cg + b;
                if (c < cols) *reinterpret_cast<uint32_t *>(dst + (int64_t)c * ldd + r0 + 4 * rg) = o[b];
                // sum of |x| over the four int8 of the word: |x| = |(x + 128) - 128| on the biased bytes
                part[p][b] += __builtin_amdgcn_sad_u8(o[b] ^ 0x80808080u, 0x80808080u, 0u);
            }
        }
        __syncthreads();   // the tile is overwritten by the next trip
    }
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            // the 32 lanes of a half-wave hold the same column: add them up, one LDS atomic per half-wave
            unsigned int v = part[p][b];
#pragma unroll
            for (int off = 16; off > 0; off >>= 1) v += (unsigned int)__shfl_xor((int)v, off, 32);
            if ((tid & 31) == 0) atomicAdd(&abs_s[4 * ((tid >> 5) + 8 * p) + b], v);
        }
    __syncthreads();
    if (tid < 64 && c0 + tid < cols && abs_s[tid] != 0u) atomicAdd(&col_abs[c0 + tid], abs_s[tid]);
}

// Chooses the power-of-two scale of g and, for each backward product, the number of limbs.  With
// sigma = 2^e > 1.01 max|g| and L limbs, q = rint(g 2^(8L-1)/sigma) is off by at most half a unit, i.e. every
// entry of g is represented to within sigma 2^-8L, so one output of a product, delta * sum_c g_c idx_c, is off by
// at most delta sigma 2^-8L sum_c |idx_c| whatever the signs and values of g: a bound, not an estimate.  The
// largest sum of |idx| over the contraction (one per output column: col_abs, from the transposition kernels)
// goes in, and L is the smallest count (3..6) that brings the bound under 9e-7 - the absolute part of the
// parity tolerance, less a margin for the roundings of the recombination and of the fp32 result, which are
// relative (1e-7) and covered by its relative part.  If six limbs do not reach it (contractions of many
// millions of large indices) six are used and the bound, stored in the plan, says what was reached.
constexpr double kLimbBoundTarget = 9e-7;

__global__ __launch_bounds__(1024)
void plan_kernel(BwdPlan *plan, const unsigned int *__restrict__ block_max, int n_max,
                 const unsigned int *__restrict__ col_abs_a, int n_abs_a, const unsigned int *__restrict__ col_abs_b, int n_abs_b,
                 float delta_a, float delta_b)
{
    __shared__ unsigned int red_m[1024], red_a[1024], red_b[1024];
    // one block of 1024 threads, four independent loads per thread and trip (the first array holds up to a few
    // thousand per-block results; a single dependent chain per thread is all latency)
    const int t = threadIdx.x;
    unsigned int m = 0u, sa = 0u, sb = 0u;
    for (int i = t; i < n_max; i += 4096) {
        const unsigned int v0 = block_max[i], v1 = i + 1024 < n_max ? block_max[i + 1024] : 0u;
        const unsigned int v2 = i + 2048 < n_max ? block_max[i + 2048] : 0u, v3 = i + 3072 < n_max ? block_max[i + 3072] : 0u;
        m = max(max(m, v0), max(max(v1, v2), v3));
    }
    for (int i = t; i < n_abs_a; i += 1024) sa = max(sa, col_abs_a[i]);
    for (int i = t; i < n_abs_b; i += 1024) sb = max(sb, col_abs_b[i]);
    red_m[t] = m; red_a[t] = sa; red_b[t] = sb;
    __syncthreads();
    for (int off = 512; off > 0; off >>= 1) {
        if (t < off) {
            red_m[t] = max(red_m[t], red_m[t + off]);
            red_a[t] = max(red_a[t], red_a[t + off]);
            red_b[t] = max(red_b[t], red_b[t + off]);
        }
        __syncthreads();
    }
    if (threadIdx.x != 0) return;
    const float amax = __uint_as_float(red_m[0]);
    int e = 0;
    if (amax > 0.0f) frexpf(amax * 1.01f, &e);   // amax * 1.01 = f 2^e with f in [0.5, 1)
    e = max(min(e, 127), -80);                   // keeps 2^(8L-1-e) a normal float for every L
    // d_a_hat contracts g with b_idx (step delta_b), d_b_hat with a_idx (step delta_a)
    const double unit_da = (double)delta_b * (double)red_b[0], unit_db = (double)delta_a * (double)red_a[0];
    int la = kMinLimbs, lb = kMinLimbs;
    while (la < kMaxLimbs && unit_da * ldexp(1.0, e - 8 * la) > kLimbBoundTarget) ++la;
    while (lb < kMaxLimbs && unit_db * ldexp(1.0, e - 8 * lb) > kLimbBoundTarget) ++lb;
    plan->bound_da = unit_da * ldexp(1.0, e - 8 * la);
    plan->bound_db = unit_db * ldexp(1.0, e - 8 * lb);
    plan->limbs_da = la;
    plan->limbs_db = lb;
    plan->gscale_da = ldexpf(1.0f, 8 * la - 1 - e);
    plan->gscale_db = ldexpf(1.0f, 8 * lb - 1 - e);
    plan->out_scale_da = (double)delta_b * ldexp(1.0, e + 1 - 8 * la);
    plan->out_scale_db = (double)delta_a * ldexp(1.0, e + 1 - 8 * lb);
}

__global__ void zero_f32_kernel(float *p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0.0f;
}

__global__ void zero_i32_kernel(int32_t *p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}

// ---- measurement aid: register-resident int8 MFMA issue rate ----------------------------------
// Eight independent accumulators per wave, no memory traffic.  random_operands = 0: the two operand
// registers never change (the least switching activity the matrix cores can see); 1: every MFMA of
// the body gets its own pseudo-random operand bits, as dense random int8 data would present them.
__global__ __launch_bounds__(256)
void mfma_probe_kernel(int iters, int random_operands, int *sink)
{
    v4i xs[8], ys[8];
    unsigned h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            h = h * 1664525u + 1013904223u;
            xs[t][c] = random_operands ? (int)h : 0x01020304;
            h = h * 1664525u + 1013904223u;
            ys[t][c] = random_operands ? (int)h : 0x04030201;
        }
    v16i acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(xs[t], ys[t], acc[t], 0, 0, 0);
    }
    int x = 0;
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) x ^= acc[t][r];
    if (x == 0x7fffffff) *sink = x;   // keeps the MFMAs alive; practically never true
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
constexpr int kFusedReduceBlocks = 2048;   // most blocks of limb_reduce_quantize_bwd_kernel

struct BwdLayout {
    size_t plan, block_max, ss_a, ss_b, fq_partial, fqb_partial, bt, at, partial, corr_da, corr_db, colsum_partial, total;
    int fq_items;                 // most work items the fused activation-gradient product can have
    int n_max;                    // per-block partial results of the absmax launch
    int64_t ldn, ldm;             // row strides of the transposed index copies (odd multiples of kLBK)
    int nk_n, nk_m;               // K-tiles of the two contractions
    int splits, kt_per_split;     // d_b_hat: splits of the contraction over M
};

BwdLayout bwd_layout(int32_t M, int32_t N, int32_t K)
{
    BwdLayout L;
    L.nk_n = (int)((N + kLBK - 1) / kLBK);
    L.nk_m = (int)((M + kLBK - 1) / kLBK);
    L.ldn = (int64_t)(L.nk_n | 1) * kLBK;
    L.ldm = (int64_t)(L.nk_m | 1) * kLBK;
    // d_b_hat has few output tiles and a long contraction: cut the contraction so that about three
    // blocks per compute unit exist, each with at least four K-tiles and (int32 accumulators of
    // products up to 2^14) at most 1023 of them.
    const int64_t base = (int64_t)((N + kLRows - 1) / kLRows) * ((K + limb_cols(5) - 1) / limb_cols(5));
    const int64_t nk = L.nk_m;
    int64_t splits = (768 + base - 1) / base;
    if (splits > nk / 4) splits = nk / 4;
    if (splits < 1) splits = 1;
    int64_t per = (nk + splits - 1) / splits;
    if (per > 1023) per = 1023;
    splits = (nk + per - 1) / per;
    L.splits = (int)splits;
    L.kt_per_split = (int)per;
    L.n_max = (int)blocks_for(((int64_t)M * N) >> 2, 2048, 2048);
    size_t off = 0;
    L.plan = off;    off += align_up(sizeof(BwdPlan), 256);
    L.block_max = off; off += align_up((size_t)L.n_max * sizeof(unsigned int), 256);
    L.ss_a = off;    off += align_up((size_t)K * sizeof(unsigned int), 256);   // sums of |a_idx| per column, directly followed by
    L.ss_b = off;    off += align_up((size_t)K * sizeof(unsigned int), 256);   // sums of |b_idx| per column (cleared together)
    // fused quantizer backward: one pair of partial scalar gradients per work item of the narrowest column tile (cleared with the above)
    L.fq_items = (int)((((int64_t)M + kLRows - 1) / kLRows) * ((K + limb_cols(6) - 1) / limb_cols(6)));
    L.fq_partial = off; off += align_up((size_t)L.fq_items * 2 * sizeof(double), 256);
    L.fqb_partial = off; off += align_up((size_t)kFusedReduceBlocks * 2 * sizeof(double), 256);   // same for the weight-gradient side: one pair per block
    L.bt = off;      off += align_up((size_t)K * (size_t)L.ldn, 256);           // b_idx^T: [K][ldn]
    L.at = off;      off += align_up((size_t)K * (size_t)L.ldm, 256);           // a_idx^T: [K][ldm]
    // (one split: used only when a reduction kernel with the quantizer's backward pass follows)
    L.partial = off; off += align_up((size_t)L.splits * (size_t)N * (size_t)K * sizeof(double), 256);
    // operands stored with an offset: one correction per output row of either product, and the per-block column sums of g
    L.corr_da = off; off += align_up((size_t)M * sizeof(double), 256);
    L.corr_db = off; off += align_up((size_t)N * sizeof(double), 256);
    L.colsum_partial = off; off += align_up((size_t)kColsumBlocks * (size_t)N * sizeof(double), 256);
    L.total = off;
    return L;
}

int launch_limb_gemm(LimbArgs a, bool trans, hipStream_t stream)
{
    // About one block per compute unit: each works through a run of consecutive row tiles.  The limb count,
    // hence the column tile, is only known on the device: the run length is chosen for the wide tile, the
    // grid is sized for the narrowest.
    if (a.tiles_r <= 0 || a.cols <= 0) return CDL_OK;
    int dev = 0, n_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0)
        n_cu = 256;
    const int64_t runs_wanted = n_cu / a.splits > 0 ? n_cu / a.splits : 1;
    a.units_per_block = (int)((a.tiles_r + runs_wanted - 1) / runs_wanted);
    // (five and six limbs: one row tile per block, and six limbs have the narrower column tile)
    const int64_t items = (int64_t)a.tiles_r * ((a.cols + limb_cols(6) - 1) / limb_cols(6)) * a.splits;
    if (items > 2147483640LL) return CDL_ERR_PARAM;
    // the kernel addresses the rows of one column tile of the index matrix with 32-bit offsets
    if ((int64_t)limb_cols(3) * a.ldb > 0xffffffffLL) return CDL_ERR_RANGE;
    const unsigned grid = (unsigned)((items + 7) / 8 * 8);
    // Runs pay off for short contractions (measured against one tile per block: -12 % at two K-tiles, -20 % at
    // one, +10 % at 24, where the start-up they save is small and the blocks, all in the same phase for the
    // whole launch, ask L2 for the same lines at the same moments).
    const bool fused = a.fq_theta != nullptr;      // (one tile per block: the epilogue needs the LDS of the stages)
    const bool long_runs = a.kt_per_split <= 4 && !fused;
    const void *fn = fused ? (const void *)limb_gemm_kernel<false, false, true>
                   : trans ? (long_runs ? (const void *)limb_gemm_kernel<true, true> : (const void *)limb_gemm_kernel<true, false>)
                           : (long_runs ? (const void *)limb_gemm_kernel<false, true> : (const void *)limb_gemm_kernel<false, false>);
    // more than 64 KiB of dynamic LDS has to be allowed per function (and per device: set it every time)
    const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kLimbLdsBytes);
    if (e != hipSuccess) return hip_failed(e);
    const char *name = trans ? "limb_gemm_kernel(d_b_hat)" : "limb_gemm_kernel(d_a_hat)";
    if (fused) CDL_LAUNCH("limb_gemm_kernel(d_a_hat + quantize_bwd)", stream, (limb_gemm_kernel<false, false, true>), dim3(grid), dim3(kLThreads), kLimbLdsBytes, a);
    else if (trans && long_runs) CDL_LAUNCH(name, stream, (limb_gemm_kernel<true, true>), dim3(grid), dim3(kLThreads), kLimbLdsBytes, a);
    else if (trans) CDL_LAUNCH(name, stream, (limb_gemm_kernel<true, false>), dim3(grid), dim3(kLThreads), kLimbLdsBytes, a);
    else if (long_runs) CDL_LAUNCH(name, stream, (limb_gemm_kernel<false, true>), dim3(grid), dim3(kLThreads), kLimbLdsBytes, a);
    else CDL_LAUNCH(name, stream, (limb_gemm_kernel<false, false>), dim3(grid), dim3(kLThreads), kLimbLdsBytes, a);
    return check_launch();
}

void launch_transpose(const int8_t *src, int rows, int cols, int8_t *dst, int64_t ldd, unsigned int *col_abs, hipStream_t stream)
{
    // about a thousand blocks where the matrix has that many tiles, each with up to 16 row tiles of its columns
    const int row_tiles = (rows + 127) / 128, col_tiles = (cols + 63) / 64;
    int per = (int)(((int64_t)row_tiles * col_tiles + 1023) / 1024);
    per = per < 1 ? 1 : (per > 16 ? 16 : per);
    const dim3 grid((row_tiles + per - 1) / per, col_tiles);
    if (cols % 4 == 0) CDL_LAUNCH("transpose_i8_kernel", stream, transpose_i8_kernel<true>, grid, dim3(256), 0, src, rows, cols, dst, ldd, col_abs, per, ConvGeom{});
    else CDL_LAUNCH("transpose_i8_kernel", stream, transpose_i8_kernel<false>, grid, dim3(256), 0, src, rows, cols, dst, ldd, col_abs, per, ConvGeom{});
}

// the transposed matrix of input windows of a convolution, straight from the activations (rows = B*P*Q, cols = R*S*C)
void launch_transpose_windows(const int8_t *x, const ConvGeom &g, int8_t *dst, int64_t ldd, unsigned int *col_abs, hipStream_t stream)
{
    const int rows = g.B * g.P * g.Q, cols = g.R * g.S * g.C;
    const int row_tiles = (rows + 127) / 128, col_tiles = (cols + 63) / 64;
    int per = (int)(((int64_t)row_tiles * col_tiles + 1023) / 1024);
    per = per < 1 ? 1 : (per > 16 ? 16 : per);
    const dim3 grid((row_tiles + per - 1) / per, col_tiles);
    CDL_LAUNCH("transpose_i8_kernel(windows)", stream, (transpose_i8_kernel<true, true>), grid, dim3(256), 0, x, rows, cols, dst, ldd, col_abs, per, g);
}

}  // namespace

int launch_mfma_probe(int iters, int random_operands, int blocks, int *sink, hipStream_t stream)
{
    CDL_LAUNCH("mfma_probe_kernel", stream, mfma_probe_kernel, dim3(blocks), dim3(256), 0, iters, random_operands, sink);
    return check_launch();
}

// forward workspace: [zero-padded operand copies when K % 16 != 0][with offsets: corrections per output column: int32 N][per output row: int32 M]
size_t qgemm_fwd_workspace_bytes(int32_t M, int32_t N, int32_t K, bool with_offsets)
{
    size_t b = 0;
    if (K % 16 != 0) {
        const int64_t kp = pad_to(K, 16);
        b += align_up((size_t)M * (size_t)kp, 256) + align_up((size_t)N * (size_t)kp, 256);
    }
    if (with_offsets) b += align_up((size_t)N * sizeof(int32_t), 256) + align_up((size_t)M * sizeof(int32_t), 256);
    return b;
}

size_t qgemm_bwd_workspace_bytes(int32_t M, int32_t N, int32_t K)
{
    if ((int64_t)M * N * K == 0) return 0;
    return bwd_layout(M, N, K).total;
}

int launch_qgemm_fwd(const int8_t *a_idx, const int8_t *b_idx, int32_t M, int32_t N, int32_t K,
                     float delta_a, float delta_b, int32_t a_offset, int32_t b_offset,
                     int32_t *acc, float *y, void *ws, hipStream_t stream)
{
    if ((int64_t)M * N == 0) return CDL_OK;
    if (K == 0) {
        if (acc) CDL_LAUNCH("zero_i32_kernel", stream, zero_i32_kernel, dim3(blocks_for((int64_t)M * N, 256, 4096)), dim3(256), 0, acc, (int64_t)M * N);
        if (y) CDL_LAUNCH("zero_f32_kernel", stream, zero_f32_kernel, dim3(blocks_for((int64_t)M * N, 256, 4096)), dim3(256), 0, y, (int64_t)M * N);
        return check_launch();
    }
    GemmArgs g{};
    g.A = a_idx; g.B = b_idx; g.lda = K; g.ldb = K;
    g.rowsA = M; g.rowsB = N; g.Kc = K;
    char *corr_base = reinterpret_cast<char *>(ws) + qgemm_fwd_workspace_bytes(M, N, K, false);
    int32_t *corr_col = reinterpret_cast<int32_t *>(corr_base);
    int32_t *corr_row = reinterpret_cast<int32_t *>(corr_base + align_up((size_t)N * sizeof(int32_t), 256));
    if (a_offset != 0) {
        // per output column s: oa * sum_k b'[s][k] + K oa ob
        CDL_LAUNCH("index_rowsum_kernel", stream, index_rowsum_kernel, dim3(blocks_for(N, 4, 4096)), dim3(256), 0, b_idx, N, K, a_offset,
                   K * a_offset * b_offset, corr_col);
        g.corr_col = corr_col;
    }
    if (b_offset != 0) {
        // per output row r: ob * sum_k a'[r][k] (plus the constant if no column correction carries it)
        CDL_LAUNCH("index_rowsum_kernel", stream, index_rowsum_kernel, dim3(blocks_for(M, 4, 4096)), dim3(256), 0, a_idx, M, K, b_offset,
                   a_offset != 0 ? 0 : K * a_offset * b_offset, corr_row);
        g.corr_row = corr_row;
    }
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
    // contraction lengths that are whole 128-byte K-tiles take the direct-load kernel (a tile grid of 256 x 256
    // needs enough rows to be worth it)
    // (up to 128 output columns would leave half of its 256-column tile empty)
    if (g.Kc % kFBK == 0 && (int64_t)M * N >= (int64_t)kFTile * kFTile * 64 && N > 128) return launch_gemm_dma(g, stream);
    // (up to 64 output columns: tiles 64 columns wide, so that half of a wider one is not padding; fewer tiles of 256
    // rows than compute units: tiles of 128 rows, twice as many blocks)
    const bool few = (int64_t)((M + 255) / 256) * ((N + (N <= 64 ? 63 : 127)) / (N <= 64 ? 64 : 128)) < 256 && M > 128;
    if (N <= 64) return few ? launch_gemm<2, 1>(g, stream) : launch_gemm<4, 1>(g, stream);
    return few ? launch_gemm<2, 2>(g, stream) : launch_gemm<4, 2>(g, stream);
}

int launch_qgemm_quantize_fwd(const float *x, const cdl_qparams &p, const int8_t *b_idx, int32_t M, int32_t N, int32_t K,
                              float delta_b, float *y, hipStream_t stream)
{
    if ((int64_t)M * N == 0) return CDL_OK;
    LimbArgs a{};
    a.G = x; a.M = M; a.N = K;            // the fp32 operand: [M][K], contraction along its rows
    a.Bt = b_idx; a.ldb = K;              // [N][K]: the contraction index is contiguous as it is
    a.rows = M; a.cols = N; a.kc = K;
    a.nk = K / kLBK;
    a.tiles_r = (M + kLRows - 1) / kLRows; a.splits = 1; a.kt_per_split = a.nk;
    a.out = y;
    a.fq_k = make_const(p);
    a.fq_scale = p.delta * delta_b;
    constexpr int NB = 4 * kQuantFwdTN * 32;
    if ((int64_t)NB * a.ldb > 0xffffffffLL) return CDL_ERR_RANGE;
    int dev = 0, n_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0)
        n_cu = 256;
    a.units_per_block = (a.tiles_r + n_cu - 1) / n_cu;
    const int64_t items = (a.tiles_r + a.units_per_block - 1) / a.units_per_block;      // runs; each takes every column tile
    const unsigned grid = (unsigned)((items + 7) / 8 * 8);
    const hipError_t e = hipFuncSetAttribute((const void *)qgemm_quantize_fwd_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLimbLdsBytes);
    if (e != hipSuccess) return hip_failed(e);
    CDL_LAUNCH("qgemm_kernel(quantize + fwd)", stream, qgemm_quantize_fwd_kernel, dim3(grid), dim3(kLThreads), kLimbLdsBytes, a);
    return check_launch();
}

// few channels on both sides: the direct kernel (its weights in at most 48 KiB of LDS)
bool conv_dx_is_direct(int32_t N, int32_t C, int32_t R, int32_t S)
{
    return C <= 32 && (int64_t)R * S * N <= 288 && (int64_t)R * S * N * (C <= 16 ? 16 : 32) * 8 <= 49152;
}

// workspace of the activation gradient of a convolution: [plan][per-block max|g|][col sums][Wr]
struct ConvDxLayout {
    size_t plan, block_max, ss_b, wr, total;
    int n_max, nk, classes;
    int64_t ld;
};

ConvDxLayout conv_dx_layout(int64_t M_out, int32_t N, int32_t C, int32_t R, int32_t S, int32_t stride)
{
    ConvDxLayout L;
    // stride 2: four classes of taps, each with at most ceil(R / 2) x ceil(S / 2) of them
    L.classes = stride == 2 ? 4 : 1;
    const int64_t kc = stride == 2 ? (int64_t)((R + 1) / 2) * ((S + 1) / 2) * N : (int64_t)R * S * N;
    L.nk = (int)((kc + kLBK - 1) / kLBK);
    L.ld = (int64_t)(L.nk | 1) * kLBK;
    L.n_max = (int)blocks_for((M_out * N) >> 2, 2048, 2048);
    size_t off = 0;
    L.plan = off;      off += align_up(sizeof(BwdPlan), 256);
    L.block_max = off; off += align_up((size_t)L.n_max * sizeof(unsigned int), 256);
    L.ss_b = off;      off += align_up((size_t)L.classes * C * sizeof(unsigned int), 256);
    L.wr = off;        off += align_up((size_t)L.classes * C * (size_t)L.ld, 256);
    L.total = off;
    return L;
}

size_t qconv_bwd_activations_workspace_bytes(int64_t M_out, int32_t N, int32_t C, int32_t R, int32_t S, int32_t stride)
{
    return conv_dx_layout(M_out, N, C, R, S, stride).total;
}

int launch_qconv_bwd_activations(const float *g, const int8_t *w_idx, int32_t B, int32_t H, int32_t W, int32_t C, int32_t N,
                                 int32_t R, int32_t S, int32_t stride, int32_t pad, float delta_w, float *d_x_hat, void *ws,
                                 hipStream_t stream)
{
    const int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    const int64_t M_out = (int64_t)B * P * Q;
    if (conv_dx_is_direct(N, C, R, S)) {
        const int cc = C <= 16 ? 16 : 32;
        const size_t lds = (size_t)R * S * N * cc * sizeof(double);
        const unsigned grid = blocks_for((int64_t)B * H * W, 256 / cc * 4, 16384);
        if (cc == 16) CDL_LAUNCH("conv_dx_direct_kernel", stream, conv_dx_direct_kernel<16>, dim3(grid), dim3(256), lds, g, w_idx, B, H, W, C, N, R, S, stride, pad, P, Q, (double)delta_w, d_x_hat);
        else CDL_LAUNCH("conv_dx_direct_kernel", stream, conv_dx_direct_kernel<32>, dim3(grid), dim3(256), lds, g, w_idx, B, H, W, C, N, R, S, stride, pad, P, Q, (double)delta_w, d_x_hat);
        return check_launch();
    }
    const ConvDxLayout L = conv_dx_layout(M_out, N, C, R, S, stride);
    char *base = reinterpret_cast<char *>(ws);
    BwdPlan *plan = reinterpret_cast<BwdPlan *>(base + L.plan);
    unsigned int *block_max = reinterpret_cast<unsigned int *>(base + L.block_max);
    unsigned int *ss_b = reinterpret_cast<unsigned int *>(base + L.ss_b);
    int8_t *wr = reinterpret_cast<int8_t *>(base + L.wr);

    // The classes of input pixels.  Stride 1: all of them, every tap.  Stride 2: input pixel (h, w) is reached only by the
    // taps r = h + pad, s = w + pad (mod 2) - with all R x S taps three products in four would multiply zeros -, so the
    // pixels (2 i + a, 2 j + c) of each parity (a, c) form a product of their own over the taps r = r0 + 2 r',
    // s = s0 + 2 s' (r0 = (a + pad) mod 2, likewise s0), in which g is read at p = i + (a + pad - r0) / 2 - r'.
    struct Cls { int oa, oc, Hc, Wc, pad_h, pad_w, Rc, Sc; };
    Cls cl[4];
    ConvDxClasses taps{};
    taps.tstep = stride;
    int n_cls = 0;
    bool zero_first = false;
    if (stride == 1) {
        cl[n_cls] = Cls{0, 0, H, W, pad, pad, R, S};
        taps.c[n_cls++] = ConvDxClass{0, 0, R, S};
    } else {
        for (int pa = 0; pa < 2; ++pa)
            for (int pc = 0; pc < 2; ++pc) {
                const int Hc = (H - pa + 1) / 2, Wc = (W - pc + 1) / 2;
                if (Hc <= 0 || Wc <= 0) continue;
                const int r0 = (pa + pad) & 1, s0 = (pc + pad) & 1;
                const int Rc = r0 < R ? (R - r0 + 1) / 2 : 0, Sc = s0 < S ? (S - s0 + 1) / 2 : 0;
                if (Rc == 0 || Sc == 0) { zero_first = true; continue; }     // no tap reaches these pixels
                cl[n_cls] = Cls{pa, pc, Hc, Wc, (pa + pad - r0) / 2, (pc + pad - s0) / 2, Rc, Sc};
                taps.c[n_cls++] = ConvDxClass{r0, s0, Rc, Sc};
            }
    }
    if (zero_first)
        CDL_LAUNCH("zero_f32_kernel", stream, zero_f32_kernel, dim3(blocks_for((int64_t)B * H * W * C, 256, 4096)), dim3(256), 0, d_x_hat, (int64_t)B * H * W * C);
    if (n_cls == 0) return check_launch();
    CDL_LAUNCH("absmax_kernel", stream, absmax_kernel, dim3(L.n_max), dim3(256), 0, g, M_out * N, block_max, ss_b, 0);
    CDL_LAUNCH("conv_dx_prep_kernel", stream, conv_dx_prep_kernel, dim3((unsigned)C, (unsigned)n_cls), dim3(256), 0,
               w_idx, N, R, S, C, taps, wr, L.ld, ss_b);
    // (one limb count for all classes: the largest column sum of any of them)
    CDL_LAUNCH("plan_kernel", stream, plan_kernel, dim3(1), dim3(1024), 0, plan, block_max, L.n_max,
               (const unsigned int *)nullptr, 0, ss_b, n_cls * C, 1.0f, delta_w);
    int rc = check_launch();
    if (rc != CDL_OK) return rc;
    LimbArgs a{};
    a.G = g; a.M = (int)M_out; a.N = N;
    a.ldb = L.ld;
    a.cols = C;
    a.splits = 1;
    a.units_per_block = 1;
    a.plan = plan; a.which = 0;
    a.out = d_x_hat;
    a.cg_P = P; a.cg_Q = Q;
    a.cg_inv_n = 1.0f / (float)N;
    a.cg_ostep = stride; a.cg_oH = H; a.cg_oW = W;
    // the tile width (128, 256 or 384 columns) that pads the channels least; the widest of those that pad equally
    a.tn = 3;
    for (int tn = 2; tn >= 1; --tn) {
        const int w = 128 * tn, wbest = 128 * a.tn;
        if ((C + w - 1) / w * w < (C + wbest - 1) / wbest * wbest) a.tn = tn;
    }
    if ((int64_t)limb_cols(3) * a.ldb > 0xffffffffLL) return CDL_ERR_RANGE;
    const void *fn = a.tn == 1 ? (const void *)limb_conv_dx_kernel<1> : a.tn == 2 ? (const void *)limb_conv_dx_kernel<2> : (const void *)limb_conv_dx_kernel<3>;
    const int lds_bytes = conv_dx_lds_bytes(a.tn);
    const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return hip_failed(e);
    for (int ci = 0; ci < n_cls; ++ci) {
        const Cls &k = cl[ci];
        a.Bt = wr + (int64_t)ci * C * L.ld;
        a.rows = B * k.Hc * k.Wc;
        a.kc = k.Rc * k.Sc * N;
        a.nk = (a.kc + kLBK - 1) / kLBK;
        a.kt_per_split = a.nk;
        a.tiles_r = (a.rows + kLRows - 1) / kLRows;
        a.cg_H = k.Hc; a.cg_W = k.Wc; a.cg_S = k.Sc; a.cg_pad_h = k.pad_h; a.cg_pad_w = k.pad_w;
        a.cg_inv_s = 1.0f / (float)k.Sc;
        a.cg_oa = k.oa; a.cg_oc = k.oc;
        const DivBy by_hw = make_div_by((uint32_t)k.Hc * (uint32_t)k.Wc), by_w = make_div_by((uint32_t)k.Wc);
        a.cg_mul_hw = by_hw.mul; a.cg_sh_hw = by_hw.sh; a.cg_mul_w = by_w.mul; a.cg_sh_w = by_w.sh;
        // (the grid is sized before the limb count is known: six limbs take tiles of at most 256 columns)
        const int narrow = 128 * (a.tn < 2 ? a.tn : 2);
        const int64_t items = (int64_t)a.tiles_r * ((a.cols + narrow - 1) / narrow);
        if (items > 2147483640LL) return CDL_ERR_PARAM;
        const unsigned grid = (unsigned)((items + 7) / 8 * 8);
        if (a.tn == 1) CDL_LAUNCH("limb_gemm_kernel(conv d_x_hat)", stream, limb_conv_dx_kernel<1>, dim3(grid), dim3(kLThreads), lds_bytes, a);
        else if (a.tn == 2) CDL_LAUNCH("limb_gemm_kernel(conv d_x_hat)", stream, limb_conv_dx_kernel<2>, dim3(grid), dim3(kLThreads), lds_bytes, a);
        else CDL_LAUNCH("limb_gemm_kernel(conv d_x_hat)", stream, limb_conv_dx_kernel<3>, dim3(grid), dim3(kLThreads), lds_bytes, a);
    }
    return check_launch();
}

size_t qconv_fwd_workspace_bytes(int32_t N, int32_t x_offset)
{
    return x_offset != 0 ? 256 + align_up((size_t)N * sizeof(int32_t), 256) : 0;
}

namespace {
// address of conv_zero_page on the current device (taken once per device)
int conv_zero_page_ptr(const int8_t **ptr)
{
    constexpr int kMaxDevices = 64;
    static const int8_t *cached[kMaxDevices];
    static std::mutex mu;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_failed(e);
    if (dev < 0 || dev >= kMaxDevices) return CDL_ERR_PARAM;
    std::lock_guard<std::mutex> lock(mu);
    if (!cached[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(conv_zero_page));
        if (e != hipSuccess) return hip_failed(e);
        if (!p) return hip_failed(hipErrorInvalidSymbol);
        cached[dev] = reinterpret_cast<const int8_t *>(p);
    }
    *ptr = cached[dev];
    return CDL_OK;
}
}  // namespace

int launch_qconv_fwd(const int8_t *x_idx, const int8_t *w_idx, int32_t B, int32_t H, int32_t W, int32_t C, int32_t N,
                     int32_t R, int32_t S, int32_t stride, int32_t pad, float delta_x, float delta_w, int32_t x_offset,
                     int32_t *acc, float *y, void *ws, hipStream_t stream)
{
    ConvArgs a{};
    a.X = x_idx; a.Wt = w_idx;
    a.B = B; a.H = H; a.W = W; a.C = C; a.N = N; a.R = R; a.S = S; a.stride = stride; a.pad = pad;
    a.P = (H + 2 * pad - R) / stride + 1;
    a.Q = (W + 2 * pad - S) / stride + 1;
    a.M = B * a.P * a.Q;
    a.Kc = R * S * C;
    a.acc_out = acc; a.y_out = y;
    a.scale = delta_x * delta_w;
    if ((int64_t)a.M * N == 0) return CDL_OK;
    if (x_offset != 0) {
        int8_t *page = reinterpret_cast<int8_t *>(ws);
        int32_t *corr = reinterpret_cast<int32_t *>(page + 256);
        CDL_LAUNCH("conv_prep_kernel", stream, conv_prep_kernel, dim3((unsigned)blocks_for(N, 4, 1024)), dim3(256), 0, page, x_offset, w_idx, N, a.Kc, corr);
        int rc = check_launch();
        if (rc != CDL_OK) return rc;
        a.pad_page = page;
        a.corr_col = corr;
    } else {
        int rc = conv_zero_page_ptr(&a.pad_page);
        if (rc != CDL_OK) return rc;
    }
    const uint32_t pb = (uint32_t)(uint8_t)(int8_t)(-x_offset);
    a.pad_word = (int)(pb | (pb << 8) | (pb << 16) | (pb << 24));
    if (C % kFBK == 0 && (int64_t)a.M * N >= (int64_t)kFTile * kFTile * 64 && N > 128) {
        a.tiles_m = (a.M + kFTile - 1) / kFTile;
        a.tiles_n = (N + kFTile - 1) / kFTile;
        const int64_t grid = ((int64_t)a.tiles_m * a.tiles_n + 7) / 8 * 8;
        const hipError_t e = hipFuncSetAttribute((const void *)qconv_dma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kFLdsBytes);
        if (e != hipSuccess) return hip_failed(e);
        CDL_LAUNCH("qconv_kernel(fwd)", stream, qconv_dma_kernel, dim3((unsigned)grid), dim3(kFThreads), kFLdsBytes, a);
        return check_launch();
    }
    // (tiles of 256 x 128, or 256 x 64 for up to 64 output channels)
    // (fewer such tiles than compute units: 128 rows per tile, twice as many blocks)
    const int BN = N <= 64 ? 64 : 128;
    const bool few = (int64_t)((a.M + 255) / 256) * ((N + BN - 1) / BN) < 256 && a.M > 128;
    const int BM = few ? 128 : 256;
    a.tiles_m = (a.M + BM - 1) / BM;
    a.tiles_n = (N + BN - 1) / BN;
    const int64_t grid = ((int64_t)a.tiles_m * a.tiles_n + 7) / 8 * 8;
    if (N <= 64 && few) CDL_LAUNCH("qconv_kernel(fwd)", stream, (qconv_kernel<2, 1>), dim3((unsigned)grid), dim3(kGemmThreads), 0, a);
    else if (N <= 64) CDL_LAUNCH("qconv_kernel(fwd)", stream, (qconv_kernel<4, 1>), dim3((unsigned)grid), dim3(kGemmThreads), 0, a);
    else if (few) CDL_LAUNCH("qconv_kernel(fwd)", stream, (qconv_kernel<2, 2>), dim3((unsigned)grid), dim3(kGemmThreads), 0, a);
    else CDL_LAUNCH("qconv_kernel(fwd)", stream, (qconv_kernel<4, 2>), dim3((unsigned)grid), dim3(kGemmThreads), 0, a);
    return check_launch();
}

int qconv_max_chunks() { return kConvMaxChunks; }

int launch_qgemm_bwd(const float *gr, const int8_t *a_idx, const int8_t *b_idx,
                     int32_t M, int32_t N, int32_t K, float delta_a, float delta_b, int32_t a_offset, int32_t b_offset,
                     float *d_a_hat, float *d_b_hat, void *ws, hipStream_t stream, const FusedQuantBwd *fq, const FusedQuantBwd *fqb,
                     const ConvWindows *cw)
{
    const bool want_db = d_b_hat != nullptr || fqb != nullptr;     // the weight-gradient product runs
    if (cw && d_a_hat) return CDL_ERR_PARAM;                       // (windows: a_idx is not a matrix; only the product over its rows is served)
    if (d_a_hat && ((int64_t)M * K > 0) && N == 0)
        CDL_LAUNCH("zero_f32_kernel", stream, zero_f32_kernel, dim3(blocks_for((int64_t)M * K, 256, 4096)), dim3(256), 0, d_a_hat, (int64_t)M * K);
    if (d_b_hat && ((int64_t)N * K > 0) && M == 0)
        CDL_LAUNCH("zero_f32_kernel", stream, zero_f32_kernel, dim3(blocks_for((int64_t)N * K, 256, 4096)), dim3(256), 0, d_b_hat, (int64_t)N * K);
    if ((int64_t)M * N * K == 0) return check_launch();

    if (d_a_hat && N <= kDirectMaxN) {
        // four columns per thread (two where 32 index values per column would not leave registers for four)
        const int c_per = N <= 16 ? 4 : 2;
        const int col_groups = (K + c_per - 1) / c_per;
        const int rows_per = direct_rows(N <= 16 ? 16 : 32);
        const dim3 grid((M + rows_per - 1) / rows_per, (col_groups + 255) / 256);
        const int vec_store = K % 4 == 0 && (reinterpret_cast<uintptr_t>(d_a_hat) & 15) == 0 && (reinterpret_cast<uintptr_t>(b_idx) & 3) == 0;
        if (N <= 16) CDL_LAUNCH("da_direct_kernel", stream, (da_direct_kernel<16, 4>), grid, dim3(256), 0, gr, b_idx, M, N, K, (double)delta_b, (double)b_offset, d_a_hat, vec_store);
        else CDL_LAUNCH("da_direct_kernel", stream, (da_direct_kernel<32, 2>), grid, dim3(256), 0, gr, b_idx, M, N, K, (double)delta_b, (double)b_offset, d_a_hat, vec_store);
        d_a_hat = nullptr;           // done; what follows is for the other product only
        if (!want_db) return check_launch();
    }

    const BwdLayout L = bwd_layout(M, N, K);
    char *base = reinterpret_cast<char *>(ws);
    BwdPlan *plan = reinterpret_cast<BwdPlan *>(base + L.plan);
    int8_t *bt = reinterpret_cast<int8_t *>(base + L.bt);
    int8_t *at = reinterpret_cast<int8_t *>(base + L.at);
    double *partial = reinterpret_cast<double *>(base + L.partial);

    unsigned int *block_max = reinterpret_cast<unsigned int *>(base + L.block_max);
    unsigned int *ss_a = reinterpret_cast<unsigned int *>(base + L.ss_a);
    unsigned int *ss_b = reinterpret_cast<unsigned int *>(base + L.ss_b);
    CDL_LAUNCH("absmax_kernel", stream, absmax_kernel, dim3(L.n_max), dim3(256), 0, gr, (int64_t)M * N, block_max,
               ss_a, fq ? (int)((L.fq_partial - L.ss_a) / sizeof(unsigned int)) + L.fq_items * 4
                        : (int)((L.ss_b - L.ss_a) / sizeof(unsigned int)) + K);
    if (d_a_hat) launch_transpose(b_idx, N, K, bt, L.ldn, ss_b, stream);
    if (want_db && cw) {
        ConvGeom g{cw->B, cw->H, cw->W, cw->C, cw->R, cw->S, cw->stride, cw->pad, cw->P, cw->Q, 0};
        const uint32_t pb = (uint32_t)(uint8_t)(int8_t)(-a_offset);
        g.pad_word = (int)(pb | (pb << 8) | (pb << 16) | (pb << 24));
        launch_transpose_windows(a_idx, g, at, L.ldm, ss_a, stream);
    } else if (want_db) launch_transpose(a_idx, M, K, at, L.ldm, ss_a, stream);
    CDL_LAUNCH("plan_kernel", stream, plan_kernel, dim3(1), dim3(1024), 0, plan, block_max, L.n_max,
               ss_a, want_db ? K : 0, ss_b, d_a_hat ? K : 0, delta_a, delta_b);
    // operands stored as index - offset: d_a_hat lacks delta_b * ob * sum_n g[m][n] in row m, d_b_hat lacks
    // delta_a * oa * sum_m g[m][n] in row n; both sums are taken of the unrounded g, in double
    double *corr_da = nullptr, *corr_db = nullptr;
    if (d_a_hat && b_offset != 0) {
        corr_da = reinterpret_cast<double *>(base + L.corr_da);
        CDL_LAUNCH("g_rowsum_kernel", stream, g_rowsum_kernel, dim3(blocks_for(M, 4, 8192)), dim3(256), 0, gr, M, N,
                   (double)delta_b * (double)b_offset, corr_da);
    }
    if (want_db && a_offset != 0) {
        corr_db = reinterpret_cast<double *>(base + L.corr_db);
        double *cp = reinterpret_cast<double *>(base + L.colsum_partial);
        const int rows_per = (M + kColsumBlocks - 1) / kColsumBlocks;
        const int blocks = (M + rows_per - 1) / rows_per;
        CDL_LAUNCH("g_colsum_kernel", stream, g_colsum_kernel, dim3(blocks), dim3(256), 0, gr, M, N, rows_per, cp);
        CDL_LAUNCH("g_colsum_finish_kernel", stream, g_colsum_finish_kernel, dim3((N + 255) / 256), dim3(256), 0, cp, blocks, N,
                   (double)delta_a * (double)a_offset, corr_db);
    }
    int rc = check_launch();
    if (rc != CDL_OK) return rc;

    if (d_a_hat) {
        LimbArgs a{};
        a.G = gr; a.M = M; a.N = N;
        a.Bt = bt; a.ldb = L.ldn;
        a.rows = M; a.cols = K; a.kc = N;
        a.nk = L.nk_n;
        a.tiles_r = (M + kLRows - 1) / kLRows; a.splits = 1; a.kt_per_split = L.nk_n;
        a.plan = plan; a.which = 0;
        a.out = d_a_hat; a.partial = nullptr;
        a.row_corr = corr_da;
        if (fq) {
            a.fq_theta = fq->theta;
            a.fq_partial = reinterpret_cast<double *>(base + L.fq_partial);
            a.fq_k = make_const(*fq->p);
            a.fq_k.stream = (int64_t)M * K >= kStreamFrom;
            a.fq_wsel = band_template(a.fq_k);
        }
        rc = launch_limb_gemm(a, false, stream);
        if (rc != CDL_OK) return rc;
        if (fq && (fq->d_delta || fq->d_alpha)) {
            const double d = (double)fq->p->delta;
            rc = launch_scalar_finalize(a.fq_partial, L.fq_items, 1.0, d * d * d, fq->d_delta, fq->d_alpha, stream);
            if (rc != CDL_OK) return rc;
        }
    }
    if (want_db) {
        LimbArgs a{};
        a.G = gr; a.M = M; a.N = N;
        a.Bt = at; a.ldb = L.ldm;
        a.rows = N; a.cols = K; a.kc = M;
        a.nk = L.nk_m;
        a.tiles_r = (N + kLRows - 1) / kLRows; a.splits = L.splits; a.kt_per_split = L.kt_per_split;
        a.plan = plan; a.which = 1;
        a.out = d_b_hat; a.partial = partial;
        a.to_partial = fqb ? 1 : 0;
        a.row_corr = corr_db;
        rc = launch_limb_gemm(a, true, stream);
        if (rc != CDL_OK) return rc;
        if (fqb) {
            // the sum over the splits (one or more) and the quantizer's backward pass on the weights in one kernel
            QConst k = make_const(*fqb->p);
            k.stream = 0;
            double *fp = reinterpret_cast<double *>(base + L.fqb_partial);
            const int blocks = (int)blocks_for((int64_t)N * K, 256, kFusedReduceBlocks);
#define CDL_RQ(WW) CDL_LAUNCH("limb_reduce_kernel(+ quantize_bwd)", stream, (limb_reduce_quantize_bwd_kernel<WW>), dim3(blocks), dim3(256), 0, \
                              partial, L.splits, (int64_t)N * K, plan, d_b_hat, corr_db, K, fqb->theta, k, fqb->d_theta, fp)
            switch (band_template(k)) {
                case 1: CDL_RQ(1); break;
                case 2: CDL_RQ(2); break;
                case 3: CDL_RQ(3); break;
                case 4: CDL_RQ(4); break;
                default: CDL_RQ(0); break;
            }
#undef CDL_RQ
            rc = check_launch();
            if (rc != CDL_OK) return rc;
            if (fqb->d_delta || fqb->d_alpha) {
                const double d = (double)fqb->p->delta;
                rc = launch_scalar_finalize(fp, blocks, 1.0, d * d * d, fqb->d_delta, fqb->d_alpha, stream);
            }
        } else if (L.splits > 1) {
            if ((int64_t)N * K <= 65536 && L.splits >= 32)
                CDL_LAUNCH("limb_reduce_kernel", stream, limb_reduce_kernel<16>, dim3(blocks_for((int64_t)N * K * 16, 256, 4096)), dim3(256), 0,
                           partial, L.splits, (int64_t)N * K, plan, d_b_hat, corr_db, K);
            else
                CDL_LAUNCH("limb_reduce_kernel", stream, limb_reduce_kernel<1>, dim3(blocks_for((int64_t)N * K, 256, 4096)), dim3(256), 0,
                           partial, L.splits, (int64_t)N * K, plan, d_b_hat, corr_db, K);
            rc = check_launch();
        }
    }
    return rc;
}

}  // namespace cdl
