// The C boundary of libcdl: argument validation (host only, before any GPU call) and dispatch.
#include "cdl_internal.h"

#include <atomic>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

namespace cdl {

namespace {
std::atomic<int> g_last_hip_error{0};
}

int hip_failed(hipError_t e)
{
    g_last_hip_error.store((int)e);
    return CDL_ERR_HIP;
}

int check_launch()
{
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? (int)CDL_OK : hip_failed(e);
}

// ---- per-kernel timing ---------------------------------------------------------------------
namespace {
struct ProfileRec {
    const char *name;
    hipEvent_t start, stop;
};
std::atomic<bool> g_profile_on{false};
std::mutex g_profile_mutex;
char g_profile_only[56] = "";                // when not empty: only launches recorded under this name are bracketed
std::vector<ProfileRec> g_profile_recs;      // recorded, not yet collected
std::vector<hipEvent_t> g_profile_free;      // events ready for reuse

hipEvent_t profile_event()
{
    if (!g_profile_free.empty()) {
        hipEvent_t e = g_profile_free.back();
        g_profile_free.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

ProfileScope::ProfileScope(const char *name, hipStream_t stream) : slot_(-1), stream_(stream)
{
    if (!g_profile_on.load(std::memory_order_relaxed)) return;
    std::lock_guard<std::mutex> lock(g_profile_mutex);
    if (g_profile_only[0] != '\0' && std::strcmp(g_profile_only, name) != 0) return;
    ProfileRec r{name, profile_event(), profile_event()};
    if (!r.start || !r.stop) return;
    (void)hipEventRecord(r.start, stream);
    g_profile_recs.push_back(r);
    slot_ = (int)g_profile_recs.size() - 1;
}

ProfileScope::~ProfileScope()
{
    if (slot_ < 0) return;
    std::lock_guard<std::mutex> lock(g_profile_mutex);
    if (slot_ < (int)g_profile_recs.size()) (void)hipEventRecord(g_profile_recs[slot_].stop, stream_);
}

namespace {

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int check_qparams(const cdl_qparams *p)
{
    if (!p) return CDL_ERR_NULL;
    if (p->n_levels < 2) return CDL_ERR_PARAM;
    if (!(std::isfinite(p->delta) && p->delta > 0.0f)) return CDL_ERR_PARAM;
    if (!(std::isfinite(p->alpha) && p->alpha > 0.0f)) return CDL_ERR_PARAM;
    const int64_t hi = (int64_t)p->lo + (int64_t)p->n_levels - 1;
    // stored as int8: sets inside [-128, 127] as they are, sets that reach beyond 127 (up to 255) minus 128
    if (p->lo < -128 || hi > 255 || (hi > 127 && p->lo < 0)) return CDL_ERR_RANGE;
    if (!(p->top_k == 0 || (p->top_k >= 1 && p->top_k <= 9 && (p->top_k & 1)))) return CDL_ERR_PARAM;
    // derived constants must stay finite in fp32
    const double kappa = (double)p->alpha * (double)p->delta * (double)p->delta;
    if (!(kappa < 1e30) || !((double)p->alpha * (double)p->delta < 1e30) || !(1.0 / (double)p->delta < 1e30))
        return CDL_ERR_PARAM;
    return CDL_OK;
}

int check_ws(const void *ws, size_t have, size_t need)
{
    if (need == 0) return CDL_OK;
    if (!ws || have < need) return CDL_ERR_WORKSPACE;
    if (!aligned(ws, 256)) return CDL_ERR_ALIGN;
    return CDL_OK;
}

}  // namespace
}  // namespace cdl

using namespace cdl;

extern "C" {

size_t cdl_quantize_workspace_bytes(int64_t n, int32_t n_levels)
{
    if (n < 0 || n_levels < 2 || n_levels > 256) return 0;
    return quantize_workspace_bytes(n, n_levels);
}

size_t cdl_qgemm_fwd_workspace_bytes(int32_t M, int32_t N, int32_t K)
{
    if (M < 0 || N < 0 || K < 0) return 0;
    return qgemm_fwd_workspace_bytes(M, N, K, false);
}

size_t cdl_qgemm_fwd_offset_workspace_bytes(int32_t M, int32_t N, int32_t K)
{
    if (M < 0 || N < 0 || K < 0) return 0;
    return qgemm_fwd_workspace_bytes(M, N, K, true);
}

int32_t cdl_index_offset(const cdl_qparams *p)
{
    const int rc = check_qparams(p);
    return rc != CDL_OK ? rc : index_offset(*p);
}

size_t cdl_qgemm_bwd_workspace_bytes(int32_t M, int32_t N, int32_t K)
{
    if (M < 0 || N < 0 || K < 0) return 0;
    return qgemm_bwd_workspace_bytes(M, N, K);
}

int cdl_quantize_fwd(const float *theta, int64_t n, const cdl_qparams *p,
                     int8_t *idx, float *soft, float *marg, float *entropy_bits,
                     void *ws, size_t ws_bytes, void *hip_stream)
{
    int rc = check_qparams(p);
    if (rc != CDL_OK) return rc;
    if (n < 0) return CDL_ERR_PARAM;
    if (n > 0 && (!theta || !idx)) return CDL_ERR_NULL;
    if (!aligned(theta, 16) || !aligned(soft, 16) || !aligned(idx, 4) || !aligned(marg, 4) || !aligned(entropy_bits, 4))
        return CDL_ERR_ALIGN;
    if (marg || entropy_bits) {
        rc = check_ws(ws, ws_bytes, quantize_workspace_bytes(n, p->n_levels));
        if (rc != CDL_OK) return rc;
    }
    return launch_quantize_fwd(theta, n, *p, idx, soft, marg, entropy_bits, ws, (hipStream_t)hip_stream);
}

size_t cdl_static_scratch_bytes(void) { return kStaticScratchBytes; }

int cdl_quantize_fwd_static(const float *theta, int64_t n, const cdl_qparams *p,
                            int8_t *idx, float *soft, float *marg, float *entropy_bits, void *hip_stream)
{
    int rc = check_qparams(p);
    if (rc != CDL_OK) return rc;
    if (n < 0) return CDL_ERR_PARAM;
    if (n > 0 && (!theta || !idx)) return CDL_ERR_NULL;
    if (!aligned(theta, 16) || !aligned(soft, 16) || !aligned(idx, 4) || !aligned(marg, 4) || !aligned(entropy_bits, 4))
        return CDL_ERR_ALIGN;
    void *ws = nullptr;
    if (marg || entropy_bits) {
        if (quantize_workspace_bytes(n, p->n_levels) > kStaticScratchBytes) return CDL_ERR_TOO_LARGE;
        rc = quantizer_static_scratch(&ws);
        if (rc != CDL_OK) return rc;
    }
    return launch_quantize_fwd(theta, n, *p, idx, soft, marg, entropy_bits, ws, (hipStream_t)hip_stream);
}

int cdl_quantize_bwd(const float *theta, const float *g, int64_t n, const cdl_qparams *p,
                     float *dtheta, float *d_delta, float *d_alpha,
                     void *ws, size_t ws_bytes, void *hip_stream)
{
    int rc = check_qparams(p);
    if (rc != CDL_OK) return rc;
    if (n < 0) return CDL_ERR_PARAM;
    if (!dtheta && !d_delta && !d_alpha) return CDL_ERR_NULL;
    if (n > 0 && (!theta || !g)) return CDL_ERR_NULL;
    if (!aligned(theta, 16) || !aligned(g, 16) || !aligned(dtheta, 16) || !aligned(d_delta, 4) || !aligned(d_alpha, 4))
        return CDL_ERR_ALIGN;
    if (d_delta || d_alpha) {
        rc = check_ws(ws, ws_bytes, quantize_workspace_bytes(n, p->n_levels));
        if (rc != CDL_OK) return rc;
    }
    return launch_quantize_bwd(theta, g, n, *p, dtheta, d_delta, d_alpha, ws, (hipStream_t)hip_stream);
}

int cdl_marginal_entropy(const float *theta, int64_t n, const cdl_qparams *p,
                         float *marg, float *entropy_bits,
                         void *ws, size_t ws_bytes, void *hip_stream)
{
    int rc = check_qparams(p);
    if (rc != CDL_OK) return rc;
    if (n < 0) return CDL_ERR_PARAM;
    if (!marg && !entropy_bits) return CDL_ERR_NULL;
    if (n > 0 && !theta) return CDL_ERR_NULL;
    if (!aligned(theta, 16) || !aligned(marg, 4) || !aligned(entropy_bits, 4)) return CDL_ERR_ALIGN;
    rc = check_ws(ws, ws_bytes, quantize_workspace_bytes(n, p->n_levels));
    if (rc != CDL_OK) return rc;
    return launch_quantize_fwd(theta, n, *p, nullptr, nullptr, marg, entropy_bits, ws, (hipStream_t)hip_stream);
}

int cdl_quantize_draw(const float *theta, const float *u, int64_t n, const cdl_qparams *p, int8_t *idx, void *hip_stream)
{
    int rc = check_qparams(p);
    if (rc != CDL_OK) return rc;
    if (n < 0) return CDL_ERR_PARAM;
    if (n > 0 && (!theta || !u || !idx)) return CDL_ERR_NULL;
    if (!aligned(theta, 16) || !aligned(u, 16) || !aligned(idx, 4)) return CDL_ERR_ALIGN;
    return launch_quantize_draw(theta, u, n, *p, idx, (hipStream_t)hip_stream);
}

int cdl_entropy_bwd(const float *theta, const float *marg, const float *g_in, int64_t n, const cdl_qparams *p, float scale,
                    float *dtheta, float *d_delta, float *d_alpha, void *ws, size_t ws_bytes, void *hip_stream)
{
    int rc = check_qparams(p);
    if (rc != CDL_OK) return rc;
    if (n < 0 || !std::isfinite(scale)) return CDL_ERR_PARAM;
    if (!dtheta && !d_delta && !d_alpha) return CDL_ERR_NULL;
    if (n > 0 && (!theta || !marg)) return CDL_ERR_NULL;
    if (!aligned(theta, 16) || !aligned(g_in, 16) || !aligned(dtheta, 16) || !aligned(marg, 4) || !aligned(d_delta, 4) || !aligned(d_alpha, 4))
        return CDL_ERR_ALIGN;
    if (d_delta || d_alpha) {
        rc = check_ws(ws, ws_bytes, quantize_workspace_bytes(n, p->n_levels));
        if (rc != CDL_OK) return rc;
    }
    return launch_entropy_bwd(theta, marg, g_in, n, *p, scale, dtheta, d_delta, d_alpha, ws, (hipStream_t)hip_stream);
}

size_t cdl_huffman_workspace_bytes(int64_t n)
{
    if (n < 0) return 0;
    return huffman_workspace_bytes(n);
}

int cdl_huffman_bits(const int8_t *idx, int64_t n, int32_t lo, int32_t n_levels,
                     unsigned long long *counts, unsigned long long *total_bits, float *bits_per_entry,
                     void *ws, size_t ws_bytes, void *hip_stream)
{
    if (n < 0 || n_levels < 1) return CDL_ERR_PARAM;
    const int64_t hi = (int64_t)lo + n_levels - 1;
    if (lo < -128 || hi > 255 || (hi > 127 && lo < 0)) return CDL_ERR_RANGE;
    if (hi > 127) lo -= 128;      // such sets are stored as index - 128
    if (!counts && !total_bits && !bits_per_entry) return CDL_ERR_NULL;
    if (n > 0 && !idx) return CDL_ERR_NULL;
    if (!aligned(idx, 16) || !aligned(counts, 8) || !aligned(total_bits, 8) || !aligned(bits_per_entry, 4)) return CDL_ERR_ALIGN;
    const int rc = check_ws(ws, ws_bytes, huffman_workspace_bytes(n));
    if (rc != CDL_OK) return rc;
    return launch_huffman_bits(idx, n, lo, n_levels, counts, total_bits, bits_per_entry, ws, (hipStream_t)hip_stream);
}

namespace {
bool offset_ok(int32_t o) { return o == 0 || o == 128; }
}

int cdl_qgemm_fwd_offset(const int8_t *a_idx, const int8_t *b_idx, int32_t M, int32_t N, int32_t K,
                         float delta_a, float delta_b, int32_t a_offset, int32_t b_offset, int32_t *acc, float *y,
                         void *ws, size_t ws_bytes, void *hip_stream)
{
    if (M < 0 || N < 0 || K < 0 || !offset_ok(a_offset) || !offset_ok(b_offset)) return CDL_ERR_PARAM;
    if (!(std::isfinite(delta_a) && delta_a > 0.0f) || !(std::isfinite(delta_b) && delta_b > 0.0f)) return CDL_ERR_PARAM;
    if (!acc && !y) return CDL_ERR_NULL;
    // the int32 result holds K products of level indices of magnitude up to 128, or 255 for an operand stored with an offset
    if ((int64_t)K * (a_offset ? 255 : 128) * (b_offset ? 255 : 128) > 2147483647LL) return CDL_ERR_RANGE;
    if ((int64_t)M * N > 0 && K > 0 && (!a_idx || !b_idx)) return CDL_ERR_NULL;
    if (!aligned(a_idx, 16) || !aligned(b_idx, 16) || !aligned(acc, 16) || !aligned(y, 16)) return CDL_ERR_ALIGN;
    int rc = check_ws(ws, ws_bytes, qgemm_fwd_workspace_bytes(M, N, K, a_offset != 0 || b_offset != 0));
    if (rc != CDL_OK) return rc;
    return launch_qgemm_fwd(a_idx, b_idx, M, N, K, delta_a, delta_b, a_offset, b_offset, acc, y, ws, (hipStream_t)hip_stream);
}

int cdl_qgemm_fwd(const int8_t *a_idx, const int8_t *b_idx, int32_t M, int32_t N, int32_t K,
                  float delta_a, float delta_b, int32_t *acc, float *y,
                  void *ws, size_t ws_bytes, void *hip_stream)
{
    return cdl_qgemm_fwd_offset(a_idx, b_idx, M, N, K, delta_a, delta_b, 0, 0, acc, y, ws, ws_bytes, hip_stream);
}

int cdl_qgemm_bwd_offset(const float *g, const int8_t *a_idx, const int8_t *b_idx,
                         int32_t M, int32_t N, int32_t K, float delta_a, float delta_b, int32_t a_offset, int32_t b_offset,
                         float *d_a_hat, float *d_b_hat,
                         void *ws, size_t ws_bytes, void *hip_stream)
{
    if (M < 0 || N < 0 || K < 0 || !offset_ok(a_offset) || !offset_ok(b_offset)) return CDL_ERR_PARAM;
    if (!(std::isfinite(delta_a) && delta_a > 0.0f) || !(std::isfinite(delta_b) && delta_b > 0.0f)) return CDL_ERR_PARAM;
    if (!d_a_hat && !d_b_hat) return CDL_ERR_NULL;
    // int32 accumulators hold limb (<= 128) x stored index (<= 128) products over the contraction length; the
    // contraction over M is cut into pieces by the library, the one over N is not
    if (d_a_hat && (int64_t)N * 128 * 128 > 2147483647LL) return CDL_ERR_RANGE;
    // the kernels address 384 rows of the transposed copy of a_idx (row length M, padded) with 32-bit offsets
    if (d_b_hat && (int64_t)M > 11000000LL) return CDL_ERR_RANGE;
    if ((int64_t)M * N * K > 0 && (!g || (d_a_hat && !b_idx) || (d_b_hat && !a_idx))) return CDL_ERR_NULL;
    if (!aligned(g, 16) || !aligned(a_idx, 16) || !aligned(b_idx, 16) || !aligned(d_a_hat, 16) || !aligned(d_b_hat, 16))
        return CDL_ERR_ALIGN;
    int rc = check_ws(ws, ws_bytes, qgemm_bwd_workspace_bytes(M, N, K));
    if (rc != CDL_OK) return rc;
    return launch_qgemm_bwd(g, a_idx, b_idx, M, N, K, delta_a, delta_b, a_offset, b_offset, d_a_hat, d_b_hat, ws, (hipStream_t)hip_stream);
}

int cdl_qgemm_fwd_quantize(const float *x, const cdl_qparams *p_a, const int8_t *b_idx, int32_t M, int32_t N, int32_t K,
                           float delta_b, float *y, void *hip_stream)
{
    const int rc = check_qparams(p_a);
    if (rc != CDL_OK) return rc;
    if (M < 0 || N < 0 || K <= 0) return CDL_ERR_PARAM;
    if (!(std::isfinite(delta_b) && delta_b > 0.0f)) return CDL_ERR_PARAM;
    // whole K-tiles of 128 entries; activations whose indices are stored as they are
    if (K % 128 != 0 || index_offset(*p_a) != 0) return CDL_ERR_PARAM;
    if ((int64_t)K * 128 * 128 > 2147483647LL) return CDL_ERR_RANGE;
    if ((int64_t)M * N > 0 && (!x || !b_idx || !y)) return CDL_ERR_NULL;
    if (!aligned(x, 16) || !aligned(b_idx, 16) || !aligned(y, 4)) return CDL_ERR_ALIGN;
    return launch_qgemm_quantize_fwd(x, *p_a, b_idx, M, N, K, delta_b, y, (hipStream_t)hip_stream);
}

size_t cdl_qconv_fwd_workspace_bytes(int32_t N, int32_t x_offset)
{
    if (N < 0 || !offset_ok(x_offset)) return 0;
    return qconv_fwd_workspace_bytes(N, x_offset);
}

int cdl_qconv_fwd(const int8_t *x_idx, const int8_t *w_idx, int32_t B, int32_t H, int32_t W, int32_t C, int32_t N,
                  int32_t R, int32_t S, int32_t stride, int32_t pad, float delta_x, float delta_w, int32_t x_offset,
                  int32_t *acc, float *y, void *ws, size_t ws_bytes, void *hip_stream)
{
    if (B < 0 || H <= 0 || W <= 0 || C <= 0 || N < 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0 || !offset_ok(x_offset)) return CDL_ERR_PARAM;
    if (!(std::isfinite(delta_x) && delta_x > 0.0f && std::isfinite(delta_w) && delta_w > 0.0f)) return CDL_ERR_PARAM;
    // a 16-byte chunk of the window matrix must lie inside one tap; padding wider than the kernel makes no sense
    if (C % 16 != 0 || pad >= R || pad >= S) return CDL_ERR_PARAM;
    if (H + 2 * pad < R || W + 2 * pad < S) return CDL_ERR_PARAM;
    if (!acc && !y) return CDL_ERR_NULL;
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    const int64_t M = (int64_t)B * P * Q, K = (int64_t)R * S * C;
    // int32 row index and offsets inside one image, the tap table, and accumulators of products up to 2^14 (2^15 with an offset)
    if (M > 2147483647LL - 256 || (int64_t)H * W * C > 2147483647LL || K / 16 > qconv_max_chunks()) return CDL_ERR_RANGE;
    if (K * (x_offset ? 32768 : 16384) > 2147483647LL) return CDL_ERR_RANGE;
    if (M * N > 0 && (!x_idx || !w_idx)) return CDL_ERR_NULL;
    if (!aligned(x_idx, 16) || !aligned(w_idx, 16) || !aligned(acc, 4) || !aligned(y, 4)) return CDL_ERR_ALIGN;
    const int rc = check_ws(ws, ws_bytes, qconv_fwd_workspace_bytes(N, x_offset));
    if (rc != CDL_OK) return rc;
    return launch_qconv_fwd(x_idx, w_idx, B, H, W, C, N, R, S, stride, pad, delta_x, delta_w, x_offset, acc, y, ws, (hipStream_t)hip_stream);
}

size_t cdl_qconv_bwd_weights_workspace_bytes(int32_t B, int32_t H, int32_t W, int32_t C, int32_t N, int32_t R, int32_t S,
                                             int32_t stride, int32_t pad)
{
    if (B <= 0 || H <= 0 || W <= 0 || C <= 0 || N <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0) return 0;
    if (H + 2 * pad < R || W + 2 * pad < S) return 0;
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    const int64_t M = (int64_t)B * P * Q, K = (int64_t)R * S * C;
    if (M > 11000000LL || K > 2147483647LL) return 0;
    return qgemm_bwd_workspace_bytes((int32_t)M, N, (int32_t)K);
}

int cdl_qconv_bwd_weights(const float *g, const int8_t *x_idx, int32_t B, int32_t H, int32_t W, int32_t C, int32_t N,
                          int32_t R, int32_t S, int32_t stride, int32_t pad, float delta_x, int32_t x_offset,
                          float *d_w_hat, void *ws, size_t ws_bytes, void *hip_stream)
{
    if (B <= 0 || H <= 0 || W <= 0 || C <= 0 || N <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0 || !offset_ok(x_offset)) return CDL_ERR_PARAM;
    if (!(std::isfinite(delta_x) && delta_x > 0.0f)) return CDL_ERR_PARAM;
    if (C % 16 != 0 || pad >= R || pad >= S) return CDL_ERR_PARAM;
    if (H + 2 * pad < R || W + 2 * pad < S) return CDL_ERR_PARAM;
    if (!g || !x_idx || !d_w_hat) return CDL_ERR_NULL;
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    const int64_t M = (int64_t)B * P * Q, K = (int64_t)R * S * C;
    // 32-bit offsets into the activations and into the transposed window matrix
    if ((int64_t)B * H * W * C > 2147483647LL || M > 11000000LL || K > 2147483647LL / 2) return CDL_ERR_RANGE;
    if (!aligned(g, 16) || !aligned(x_idx, 16) || !aligned(d_w_hat, 16)) return CDL_ERR_ALIGN;
    const int rc = check_ws(ws, ws_bytes, qgemm_bwd_workspace_bytes((int32_t)M, N, (int32_t)K));
    if (rc != CDL_OK) return rc;
    const ConvWindows cw{B, H, W, C, R, S, stride, pad, (int)P, (int)Q};
    return launch_qgemm_bwd(g, x_idx, nullptr, (int32_t)M, N, (int32_t)K, delta_x, 1.0f, x_offset, 0, nullptr, d_w_hat, ws,
                            (hipStream_t)hip_stream, nullptr, nullptr, &cw);
}

namespace {
// shared checks of the activation gradient of a convolution; M_out = B*P*Q on success
int conv_dx_geometry(int32_t B, int32_t H, int32_t W, int32_t C, int32_t N, int32_t R, int32_t S, int32_t stride, int32_t pad, int64_t *M_out)
{
    if (B <= 0 || H <= 0 || W <= 0 || C <= 0 || N <= 0 || R <= 0 || S <= 0 || pad < 0) return CDL_ERR_PARAM;
    // four consecutive entries of the contraction over (tap, output channel) share a tap; strides as the ResNets use them
    if (N % 4 != 0 || C % 4 != 0 || (stride != 1 && stride != 2) || pad >= R || pad >= S) return CDL_ERR_PARAM;
    if (H + 2 * pad < R || W + 2 * pad < S) return CDL_ERR_PARAM;
    const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    *M_out = (int64_t)B * P * Q;
    if ((int64_t)R * S * N > 131071 || *M_out > 2147483647LL / 2 || (int64_t)B * H * W > 2147483647LL / 2) return CDL_ERR_RANGE;
    return CDL_OK;
}
}  // namespace

size_t cdl_qconv_bwd_activations_workspace_bytes(int32_t B, int32_t H, int32_t W, int32_t C, int32_t N, int32_t R, int32_t S,
                                                 int32_t stride, int32_t pad)
{
    int64_t M_out = 0;
    if (conv_dx_geometry(B, H, W, C, N, R, S, stride, pad, &M_out) != CDL_OK) return 0;
    return qconv_bwd_activations_workspace_bytes(M_out, N, C, R, S, stride);
}

int cdl_qconv_bwd_activations(const float *g, const int8_t *w_idx, int32_t B, int32_t H, int32_t W, int32_t C, int32_t N,
                              int32_t R, int32_t S, int32_t stride, int32_t pad, float delta_w,
                              float *d_x_hat, void *ws, size_t ws_bytes, void *hip_stream)
{
    int64_t M_out = 0;
    int rc = conv_dx_geometry(B, H, W, C, N, R, S, stride, pad, &M_out);
    if (rc != CDL_OK) return rc;
    if (!(std::isfinite(delta_w) && delta_w > 0.0f)) return CDL_ERR_PARAM;
    if (!g || !w_idx || !d_x_hat) return CDL_ERR_NULL;
    if (!aligned(g, 16) || !aligned(w_idx, 16) || !aligned(d_x_hat, 16)) return CDL_ERR_ALIGN;
    rc = check_ws(ws, ws_bytes, qconv_bwd_activations_workspace_bytes(M_out, N, C, R, S, stride));
    if (rc != CDL_OK) return rc;
    return launch_qconv_bwd_activations(g, w_idx, B, H, W, C, N, R, S, stride, pad, delta_w, d_x_hat, ws, (hipStream_t)hip_stream);
}

int cdl_qgemm_bwd_quantize_bwd(const float *g, const int8_t *a_idx, const int8_t *b_idx, int32_t M, int32_t N, int32_t K,
                               const float *theta_a, const cdl_qparams *p_a, float delta_b, int32_t b_offset,
                               float *d_theta_a, float *d_delta_a, float *d_alpha_a, float *d_b_hat,
                               const float *theta_b, const cdl_qparams *p_b, float *d_theta_b, float *d_delta_b, float *d_alpha_b,
                               void *ws, size_t ws_bytes, void *hip_stream)
{
    int rc = check_qparams(p_a);
    if (rc != CDL_OK) return rc;
    if (M <= 0 || N <= 0 || K <= 0 || !offset_ok(b_offset)) return CDL_ERR_PARAM;
    if (!(std::isfinite(delta_b) && delta_b > 0.0f)) return CDL_ERR_PARAM;
    // the fused epilogue walks the tile four columns at a time, and very short contractions take a kernel without it
    if (K % 4 != 0 || N <= 32) return CDL_ERR_PARAM;
    if (!d_theta_a) return CDL_ERR_NULL;
    const bool weights = theta_b || p_b || d_theta_b || d_delta_b || d_alpha_b;
    if (weights) {
        rc = check_qparams(p_b);
        if (rc != CDL_OK) return rc;
        if (!theta_b || !d_theta_b) return CDL_ERR_NULL;
        // the weight quantizer is the one b_idx was stored with
        if (p_b->delta != delta_b || index_offset(*p_b) != b_offset) return CDL_ERR_PARAM;
    }
    const bool want_db = d_b_hat || weights;
    if ((int64_t)N * 128 * 128 > 2147483647LL) return CDL_ERR_RANGE;
    if (want_db && (int64_t)M > 11000000LL) return CDL_ERR_RANGE;
    if (!g || !b_idx || !theta_a || (want_db && !a_idx)) return CDL_ERR_NULL;
    if (!aligned(g, 16) || !aligned(a_idx, 16) || !aligned(b_idx, 16) || !aligned(theta_a, 16) || !aligned(d_theta_a, 16) ||
        !aligned(d_b_hat, 16) || !aligned(d_delta_a, 4) || !aligned(d_alpha_a, 4) || !aligned(theta_b, 16) || !aligned(d_theta_b, 16) ||
        !aligned(d_delta_b, 4) || !aligned(d_alpha_b, 4))
        return CDL_ERR_ALIGN;
    rc = check_ws(ws, ws_bytes, qgemm_bwd_workspace_bytes(M, N, K));
    if (rc != CDL_OK) return rc;
    const FusedQuantBwd fq{theta_a, p_a, d_delta_a, d_alpha_a, nullptr};
    const FusedQuantBwd fqb{theta_b, p_b, d_delta_b, d_alpha_b, d_theta_b};
    return launch_qgemm_bwd(g, a_idx, b_idx, M, N, K, p_a->delta, delta_b, index_offset(*p_a), b_offset, d_theta_a, d_b_hat, ws,
                            (hipStream_t)hip_stream, &fq, weights ? &fqb : nullptr);
}

int cdl_qgemm_bwd(const float *g, const int8_t *a_idx, const int8_t *b_idx,
                  int32_t M, int32_t N, int32_t K, float delta_a, float delta_b,
                  float *d_a_hat, float *d_b_hat,
                  void *ws, size_t ws_bytes, void *hip_stream)
{
    return cdl_qgemm_bwd_offset(g, a_idx, b_idx, M, N, K, delta_a, delta_b, 0, 0, d_a_hat, d_b_hat, ws, ws_bytes, hip_stream);
}

int cdl_probe_mfma_int8(int32_t iters, int32_t random_operands, int32_t blocks, void *sink, double *ops, void *hip_stream)
{
    if (iters < 1 || blocks < 1 || !sink) return iters < 1 || blocks < 1 ? CDL_ERR_PARAM : CDL_ERR_NULL;
    if (!aligned(sink, 4)) return CDL_ERR_ALIGN;
    // 4 waves per block, 8 MFMAs of 32 x 32 x 32 multiply-adds per wave and trip
    if (ops) *ops = (double)blocks * 4.0 * (double)iters * 8.0 * 2.0 * 32.0 * 32.0 * 32.0;
    return launch_mfma_probe(iters, random_operands != 0, blocks, reinterpret_cast<int *>(sink), (hipStream_t)hip_stream);
}

int cdl_profile_enable(int enable)
{
    cdl::g_profile_on.store(enable != 0);
    return CDL_OK;
}

int cdl_profile_only(const char *kernel)
{
    std::lock_guard<std::mutex> lock(cdl::g_profile_mutex);
    std::memset(cdl::g_profile_only, 0, sizeof(cdl::g_profile_only));
    if (kernel) std::strncpy(cdl::g_profile_only, kernel, sizeof(cdl::g_profile_only) - 1);
    return CDL_OK;
}

int cdl_profile_collect(cdl_profile_record *out, int max_records)
{
    if (max_records < 0 || (max_records > 0 && !out)) return CDL_ERR_PARAM;
    std::lock_guard<std::mutex> lock(cdl::g_profile_mutex);
    int n = 0;
    for (const cdl::ProfileRec &r : cdl::g_profile_recs) {
        float ms = 0.0f;
        hipError_t e = hipEventSynchronize(r.stop);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.start, r.stop);
        if (e != hipSuccess) {
            cdl::g_profile_recs.clear();
            return hip_failed(e);
        }
        if (n < max_records) {
            std::memset(&out[n], 0, sizeof(out[n]));
            std::strncpy(out[n].kernel, r.name, sizeof(out[n].kernel) - 1);
            out[n].ms = ms;
            ++n;
        }
        cdl::g_profile_free.push_back(r.start);
        cdl::g_profile_free.push_back(r.stop);
    }
    cdl::g_profile_recs.clear();
    return n;
}

const char *cdl_status_string(int status)
{
    switch (status) {
        case CDL_OK: return "ok";
        case CDL_ERR_NULL: return "a required pointer is NULL";
        case CDL_ERR_PARAM: return "invalid size or quantizer parameter";
        case CDL_ERR_RANGE: return "level set outside int8 or int32 accumulator overflow possible";
        case CDL_ERR_ALIGN: return "pointer not sufficiently aligned";
        case CDL_ERR_WORKSPACE: return "workspace missing or too small";
        case CDL_ERR_HIP: return "a HIP call failed (see cdl_last_hip_error)";
        case CDL_ERR_TOO_LARGE: return "tensor needs more scratch than the library's built-in buffer holds (see cdl_static_scratch_bytes)";
        default: return "unknown status";
    }
}

int cdl_last_hip_error(void) { return cdl::g_last_hip_error.load(); }

int cdl_version(void) { return 100; }

}  // extern "C"
