// Internal declarations shared by the translation units of libcdl (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "cdl.h"

namespace cdl {

// Most blocks any quantizer kernel is launched with; also the number of per-block partial
// results the workspace holds.  256 CUs x 8 resident blocks of 256 threads.
constexpr int kMaxQuantBlocks = 2048;
constexpr int kQuantThreads = 256;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Record a failed HIP call; returns CDL_ERR_HIP.
int hip_failed(hipError_t e);

// Returns CDL_ERR_HIP (and records the code) when the most recent launch failed.
int check_launch();

// Brackets the kernels launched during its lifetime with two HIP events when profiling is on.
class ProfileScope {
public:
    ProfileScope(const char *name, hipStream_t stream);
    ~ProfileScope();
    ProfileScope(const ProfileScope &) = delete;
    ProfileScope &operator=(const ProfileScope &) = delete;
private:
    int slot_;
    hipStream_t stream_;
};

// Launch KERNEL on STREAM, timed under NAME when profiling is on.
#define CDL_LAUNCH(NAME, STREAM, KERNEL, GRID, BLOCK, LDS, ...)                       \
    do {                                                                              \
        ::cdl::ProfileScope cdl_ps_(NAME, STREAM);                                    \
        hipLaunchKernelGGL(KERNEL, GRID, BLOCK, LDS, STREAM, __VA_ARGS__);            \
    } while (0)

// ---- streaming loads and stores ------------------------------------------------------------
// Large tensors that a pass reads or writes exactly once go through non-temporal accesses: they are not
// kept in the caches, and a pass over data that is not cached anyway runs faster that way (a reduction over
// 805 MB: 183 us with ordinary loads, 122 us with these; quantizer forward and backward on 50 M entries:
// -10 %).  A tensor that fits the 256 MB last-level cache and is visited again soon is better off with
// ordinary accesses (25.6 M entries back to back: +7 % with these), hence the flag.
#if defined(__HIPCC__)
typedef float cdl_v4f __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream4(const float *p, bool stream = true)
{
    if (!stream) return *reinterpret_cast<const float4 *>(p);
    const cdl_v4f v = __builtin_nontemporal_load(reinterpret_cast<const cdl_v4f *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream4(float *p, float a, float b, float c, float d, bool stream = true)
{
    if (!stream) { *reinterpret_cast<float4 *>(p) = make_float4(a, b, c, d); return; }
    const cdl_v4f v = {a, b, c, d};
    __builtin_nontemporal_store(v, reinterpret_cast<cdl_v4f *>(p));
}
// entries from which a tensor counts as large (32 MiB of fp32)
constexpr long long kStreamFrom = 1ll << 23;
__device__ __forceinline__ void store_stream_u32(void *p, unsigned int v)
{
    __builtin_nontemporal_store(v, reinterpret_cast<unsigned int *>(p));
}
#endif

// ---- quantizer (cdl_quantizer.hip) -------------------------------------------------------
size_t quantize_workspace_bytes(int64_t n, int32_t n_levels);

int launch_quantize_fwd(const float *theta, int64_t n, const cdl_qparams &p,
                        int8_t *idx, float *soft, float *marg, float *entropy_bits,
                        void *ws, hipStream_t stream);

int launch_quantize_bwd(const float *theta, const float *g, int64_t n, const cdl_qparams &p,
                        float *dtheta, float *d_delta, float *d_alpha,
                        void *ws, hipStream_t stream);

int launch_quantize_draw(const float *theta, const float *u, int64_t n, const cdl_qparams &p, int8_t *idx, hipStream_t stream);

int launch_entropy_bwd(const float *theta, const float *marg, const float *g_in, int64_t n, const cdl_qparams &p,
                       float scale, float *dtheta, float *d_delta, float *d_alpha, void *ws, hipStream_t stream);

// Scratch that lives inside the library (one file-scope device array per GPU) for the entry point that takes
// no workspace: its size, and its device address on the current device (looked up on first use).
constexpr size_t kStaticScratchBytes = 8u << 20;
int quantizer_static_scratch(void **ptr);

// 0, or 128 for level sets that reach beyond 127: what the kernels subtract from a level index before storing it.
int index_offset(const cdl_qparams &p);

// Half-width of the band of levels around the nearest one that the kernels visit for a given
// kappa = alpha*delta^2 (levels further out carry less than fp32 resolution of the result).
int quantizer_window(double kappa, int n_levels);

// ---- index GEMMs (cdl_qgemm.hip) ---------------------------------------------------------
size_t qgemm_fwd_workspace_bytes(int32_t M, int32_t N, int32_t K, bool with_offsets);
size_t qgemm_bwd_workspace_bytes(int32_t M, int32_t N, int32_t K);

// a_offset / b_offset: what was subtracted from the level indices of that operand before they were stored (0 or 128)
int launch_qgemm_fwd(const int8_t *a_idx, const int8_t *b_idx, int32_t M, int32_t N, int32_t K,
                     float delta_a, float delta_b, int32_t a_offset, int32_t b_offset, int32_t *acc, float *y,
                     void *ws, hipStream_t stream);

// fq != null: d_a_hat receives dL/dtheta of the activations (the quantizer's backward pass applied in the epilogue
// of the product) and the two scalar gradients go to fq->d_delta / fq->d_alpha.
// fqb != null: the same for the weights, applied where the splits of the weight-gradient product are added up:
// fqb->d_theta receives dL/dtheta of the weights; d_b_hat (nullable then) still receives dL/dQ(w) when given.
struct FusedQuantBwd {
    const float *theta;       // the tensor the operand was quantized from, in the operand's layout
    const cdl_qparams *p;     // its quantizer
    float *d_delta, *d_alpha; // DEVICE fp32[1], nullable
    float *d_theta;           // weight side only: where dL/dtheta goes
};

// cw != null: a_idx is not an [M][K] matrix but the activations [B][H][W][C] of a convolutional layer, whose matrix of
// input windows (M = B*P*Q rows, K = R*S*C columns) is the operand; only d_b_hat (the weight gradient) is served.
struct ConvWindows {
    int B, H, W, C, R, S, stride, pad, P, Q;
};

int launch_qgemm_bwd(const float *g, const int8_t *a_idx, const int8_t *b_idx,
                     int32_t M, int32_t N, int32_t K, float delta_a, float delta_b, int32_t a_offset, int32_t b_offset,
                     float *d_a_hat, float *d_b_hat, void *ws, hipStream_t stream, const FusedQuantBwd *fq = nullptr,
                     const FusedQuantBwd *fqb = nullptr, const ConvWindows *cw = nullptr);

// Forward product with the quantizer of the activations in its prologue (K % 128 == 0, indices stored without an offset).
int launch_qgemm_quantize_fwd(const float *x, const cdl_qparams &p, const int8_t *b_idx, int32_t M, int32_t N, int32_t K,
                              float delta_b, float *y, hipStream_t stream);

// Forward product of a convolutional layer over level indices, without an im2col matrix (C % 16 == 0).
size_t qconv_fwd_workspace_bytes(int32_t N, int32_t x_offset);
int qconv_max_chunks();   // most 16-byte chunks of the contraction R*S*C the kernels index
int launch_qconv_fwd(const int8_t *x_idx, const int8_t *w_idx, int32_t B, int32_t H, int32_t W, int32_t C, int32_t N,
                     int32_t R, int32_t S, int32_t stride, int32_t pad, float delta_x, float delta_w, int32_t x_offset,
                     int32_t *acc, float *y, void *ws, hipStream_t stream);

// Activation gradient of a convolutional layer (N % 128 == 0, stride 1 or 2): d_x_hat [B][H][W][C].
size_t qconv_bwd_activations_workspace_bytes(int64_t M_out, int32_t N, int32_t C, int32_t R, int32_t S, int32_t stride);
int launch_qconv_bwd_activations(const float *g, const int8_t *w_idx, int32_t B, int32_t H, int32_t W, int32_t C, int32_t N,
                                 int32_t R, int32_t S, int32_t stride, int32_t pad, float delta_w, float *d_x_hat, void *ws,
                                 hipStream_t stream);

// d_delta = mul_d * sum of partial[2 i], d_alpha = mul_a * sum of partial[2 i + 1], i < n, in a fixed order.
int launch_scalar_finalize(const double *partial, int n, double mul_d, double mul_a, float *d_delta, float *d_alpha, hipStream_t stream);

// ---- Huffman-coded size (cdl_huffman.hip) --------------------------------------------------
size_t huffman_workspace_bytes(int64_t n);

int launch_huffman_bits(const int8_t *idx, int64_t n, int lo, int n_levels, unsigned long long *counts,
                        unsigned long long *total_bits, float *bits_per_entry, void *ws, hipStream_t stream);

int launch_mfma_probe(int iters, int random_operands, int blocks, int *sink, hipStream_t stream);

}  // namespace cdl
