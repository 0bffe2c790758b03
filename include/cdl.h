/*
 * libcdl - the quantized layer step of Coded Deep Learning (CDL) on AMD MI355X (gfx950).
 *
 * One layer, one minibatch, in the order of Algorithm 1 of the paper:
 *
 *   quantize weights        cdl_quantize_fwd(W)            -> level indices, soft values, marginal PMF / entropy
 *   quantize activations    cdl_quantize_fwd(X)
 *   forward over indices    cdl_qgemm_fwd(Xi, Wi)          -> Y = dx*dw * (Xi . Wi^T)
 *   backward over indices   cdl_qgemm_bwd(G, Xi, Wi)       -> dL/dQ(X), dL/dQ(W)
 *   quantizer backward      cdl_quantize_bwd(X, dL/dQ(X))  -> dL/dX, dL/d(step), dL/d(sharpness); same for W
 *
 * Other forms of the same steps: cdl_qgemm_fwd_offset / cdl_qgemm_bwd_offset (operands of the unsigned 8-bit
 * alphabet), cdl_qgemm_bwd_quantize_bwd (the last two steps in one call), cdl_qgemm_fwd_quantize (the second and
 * third), cdl_qconv_fwd / cdl_qconv_bwd_weights / cdl_qconv_bwd_activations (a convolutional layer on [B,H,W,C]
 * activations), cdl_quantize_fwd_static (no workspace); next to the path: cdl_marginal_entropy, cdl_entropy_bwd,
 * cdl_quantize_draw, cdl_huffman_bits.
 *
 * Conventions for every entry point
 *   - All tensor and scalar-output pointers are DEVICE pointers owned by the caller; tensors are
 *     contiguous, row-major.  fp32 tensors must be 16-byte aligned, int8 index tensors 4-byte
 *     aligned (16-byte for the GEMMs), else CDL_ERR_ALIGN.
 *   - Step size and sharpness are HOST scalars.
 *   - `ws` is caller-owned device scratch of at least the size the matching *_workspace_bytes()
 *     query returns (256-byte aligned); the library allocates and frees nothing and keeps no state
 *     between calls except the last HIP error code.  Two calls may share `ws` only if they are
 *     ordered on one stream.
 *   - `hip_stream` is a hipStream_t (NULL = the default stream).  Calls enqueue kernels and return
 *     without synchronising.  Outputs are overwritten, never accumulated into.
 *   - Return value: CDL_OK or a negative cdl_status.  Arguments are validated on the host before
 *     any GPU call; on error nothing is launched.  Inputs must be finite; the result for NaN or
 *     infinite tensor entries is unspecified.
 *   - n == 0 (or an empty GEMM dimension of an output) is CDL_OK: scalar outputs and the marginal
 *     PMF are set to 0.
 */
#ifndef CDL_H
#define CDL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * A uniform quantizer of the paper (Sec. III-A, Sec. IV-A): index set {lo, ..., lo+n_levels-1},
 * reproduction value of index i is i*delta (the paper's q_l for weights, s_l for activations),
 * sharpness alpha (the paper's alpha_l / beta_l).  The paper's signed b-bit set is
 * lo = -2^(b-1), n_levels = 2^b; its unsigned set (eq. repo_alphabet) is lo = 0, n_levels = 2^b.
 * Accepted: any contiguous set inside [-128, 127], and any contiguous set inside [0, 255] - which
 * includes the unsigned 8-bit set the paper keeps for the first and last layer (Sec. V-B).
 * Level indices are stored as int8: as they are for sets inside [-128, 127], and as index - 128 for
 * sets that reach beyond 127; cdl_index_offset() returns that offset (0 or 128) for a quantizer, and
 * the *_offset forms of the layer products take it for each operand.
 * top_k = 0: the CPMF of eq. CPMF over all levels.  top_k = 1, 3, 5, 7 or 9: the CPMF truncated to its
 * top_k most probable values (Sec. V-B, where the paper uses five for activations):
 * the top_k most probable levels - the nearest ones, lower index first on a tie - keep their
 * probabilities renormalised to sum 1, all others get 0; every entry point then works with that
 * truncated CPMF.  A top_k of n_levels or more is the full CPMF.
 */
typedef struct cdl_qparams {
    int32_t lo;
    int32_t n_levels;
    float   delta;
    float   alpha;
    int32_t top_k;
} cdl_qparams;

typedef enum cdl_status {
    CDL_OK            =  0,
    CDL_ERR_NULL      = -1,   /* a required pointer is NULL */
    CDL_ERR_PARAM     = -2,   /* negative size, n_levels < 2, delta/alpha not finite and positive, ... */
    CDL_ERR_RANGE     = -3,   /* level set inside neither [-128,127] nor [0,255], or an int32 accumulator could overflow */
    CDL_ERR_ALIGN     = -4,   /* pointer alignment, see above */
    CDL_ERR_WORKSPACE = -5,   /* ws is NULL or smaller than the query says */
    CDL_ERR_HIP       = -6,   /* a HIP call failed; see cdl_last_hip_error() */
    CDL_ERR_TOO_LARGE = -7    /* cdl_quantize_fwd_static: the tensor needs more scratch than the built-in buffer holds */
} cdl_status;

/* Scratch needed by cdl_quantize_fwd / cdl_quantize_bwd / cdl_marginal_entropy for n elements. */
size_t cdl_quantize_workspace_bytes(int64_t n, int32_t n_levels);

/* Scratch needed by cdl_qgemm_fwd (staging copies when K is not a multiple of 16). */
size_t cdl_qgemm_fwd_workspace_bytes(int32_t M, int32_t N, int32_t K);

/* Scratch needed by cdl_qgemm_fwd_offset (the above plus one int32 per output row and column). */
size_t cdl_qgemm_fwd_offset_workspace_bytes(int32_t M, int32_t N, int32_t K);

/*
 * What the library subtracts from the level indices of this quantizer before storing them as int8:
 * 0 for level sets inside [-128, 127], 128 for sets that reach beyond 127 (eq. repo_alphabet with b = 8:
 * {0, ..., 255} is stored as -128 ... 127).  A negative cdl_status for invalid parameters.
 */
int32_t cdl_index_offset(const cdl_qparams *p);

/* Scratch needed by cdl_qgemm_bwd (transposed index copies, partial sums of the split contraction). */
size_t cdl_qgemm_bwd_workspace_bytes(int32_t M, int32_t N, int32_t K);

/*
 * Forward quantizer over a flat tensor (eq. CPMF, eq. softQ; per-layer forms eq. PMFw / PMFa and
 * eq. softboth).  For each entry theta[e] the conditional PMF over the levels is
 * softmax_i(-alpha (theta[e] - i delta)^2).  Outputs:
 *   idx[e]   the level index at the mode of that PMF, i.e. the nearest level, clamped to the set;
 *            an exact tie between two levels goes to the lower index; stored minus
 *            cdl_index_offset(p)                                               (int8[n], required)
 *   soft[e]  Q_d(theta[e]) = sum_i P_i * i * delta                            (fp32[n], nullable)
 *   marg[k]  (1/n) sum_e P(level lo+k | theta[e]), the marginal PMF of eq. approx1/n
 *                                                                      (fp32[n_levels], nullable)
 *   entropy_bits   -sum_k marg[k] log2 marg[k], bits per entry (Sec. IV-C) (fp32[1], nullable)
 * marg may be NULL while entropy_bits is not.
 */
int cdl_quantize_fwd(const float *theta, int64_t n, const cdl_qparams *p,
                     int8_t *idx, float *soft, float *marg, float *entropy_bits,
                     void *ws, size_t ws_bytes, void *hip_stream);

/*
 * cdl_quantize_fwd for callers that cannot allocate device memory or have no workspace to hand over: code
 * running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * outputs and kernels as cdl_quantize_fwd, minus `ws`: the per-block histograms, the second-level sums and the
 * ticket word of the marginal PMF live in a buffer that is part of the library's device code
 * (cdl_static_scratch_bytes() = 8 MiB on every GPU the library runs on, held until the process ends).  The call
 * allocates and frees nothing, on the host or on the device, as long as cdl_profile_enable is off.
 * CDL_ERR_TOO_LARGE when marg or entropy_bits is requested and cdl_quantize_workspace_bytes(n, n_levels)
 * exceeds cdl_static_scratch_bytes() (with 255 levels: beyond about 10^8 entries); nothing is launched then.
 * Without marg and entropy_bits no scratch is used and any n is accepted.
 * All calls on one GPU share that GPU's buffer, which keeps the last call's contents (every call overwrites
 * what it reads): two calls that overlap in time on one GPU - different streams, different host threads -
 * race.  Calls ordered on one stream are safe.  The first call on a GPU that asks for marg or entropy_bits looks
 * the buffer's address up (hipGetSymbolAddress, once per GPU): make that call before a capture begins.
 */
size_t cdl_static_scratch_bytes(void);
int cdl_quantize_fwd_static(const float *theta, int64_t n, const cdl_qparams *p,
                            int8_t *idx, float *soft, float *marg, float *entropy_bits, void *hip_stream);

/*
 * Backward of the quantizer through its soft proxy Q_d (Lemma 1; chain rule of Sec. IV-B,
 * eq. partialX3, partialW3, Jgradqw, Jgradqx, Jgradq_alpha_w, Jgrad_alpha_q).
 * g[e] is dL/dQ_p(theta[e]) as produced by cdl_qgemm_bwd.  Outputs:
 *   dtheta[e] = g[e] * 2 alpha Var{Q_p | theta[e]}                              (fp32[n], nullable)
 *   d_delta   = sum_e g[e] * (E + 2 alpha theta Var - 2 alpha Skew_u) / delta  (fp32[1], nullable)
 *   d_alpha   = sum_e g[e] * (2 theta Var - Skew_u)                           (fp32[1], nullable)
 * The last formula is not printed in the paper (Sec. IV-B only notes that it has an analytic form):
 * dQ_d/dalpha = -Cov(Q_p, (theta - Q_p)^2).  At least one output must be non-NULL.
 * The two sums are reproducible: same inputs, same bits.
 */
int cdl_quantize_bwd(const float *theta, const float *g, int64_t n, const cdl_qparams *p,
                     float *dtheta, float *d_delta, float *d_alpha,
                     void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Marginal PMF of the quantized tensor and its entropy (Sec. IV-C, eq. approx1/n and the
 * definition of H(W^)), without the per-entry outputs.  marg: fp32[n_levels] (nullable),
 * entropy_bits: fp32[1] (nullable); at least one non-NULL.  Total bits of the tensor = n * entropy.
 */
int cdl_marginal_entropy(const float *theta, int64_t n, const cdl_qparams *p,
                         float *marg, float *entropy_bits,
                         void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The probabilistic quantizer Q_p itself (eq. Qprob, Sec. III-A; Algorithm 1 quantizes with it):
 * theta[e] is mapped to level i with probability P(i delta | theta[e]).  The draw is made by
 * inversion with the caller's uniform numbers u[e] in [0,1): idx[e] is the first level, in
 * increasing order, whose cumulative probability exceeds u[e].  theta, u: DEVICE fp32[n], 16-byte
 * aligned; idx: DEVICE int8[n], 4-byte aligned.  Entries whose u lies within fp32 rounding
 * (about 1e-6) of a boundary of the cumulative distribution may come out one level off.
 */
int cdl_quantize_draw(const float *theta, const float *u, int64_t n, const cdl_qparams *p,
                      int8_t *idx, void *hip_stream);

/*
 * Gradient of the entropy term of the objective (eq. obj, eq. opt4, Sec. IV-D; Algorithm 1, the
 * step that forms the partials of H(w) and H(x)).  With H = -sum_k m_k log2 m_k the entropy in
 * bits of the marginal PMF m (eq. approx1/n) of the tensor theta,
 *   dtheta[e] = g_in[e] + scale * dH/dtheta[e]     (fp32[n], nullable; g_in nullable = 0)
 *   d_delta   = scale * dH/d delta,  d_alpha = scale * dH/d alpha   (DEVICE fp32[1], nullable)
 * marg: DEVICE fp32[n_levels], the marginal PMF the forward pass produced for this tensor and
 * these parameters (levels with marg = 0 contribute nothing).  scale: e.g. lambda * n for the
 * total-bits term lambda * n * H added to a loss whose gradient is g_in.  The paper does not print
 * these partials (Sec. IV-D only notes that they have an analytic form); they follow from
 * dH = -sum_k log2(m_k) dm_k and the CPMF derivatives of Appendix B.  Workspace as for
 * cdl_quantize_bwd when a scalar output is requested.  At least one output non-NULL.
 */
int cdl_entropy_bwd(const float *theta, const float *marg, const float *g_in, int64_t n,
                    const cdl_qparams *p, float scale,
                    float *dtheta, float *d_delta, float *d_alpha,
                    void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Size of a quantized tensor under Huffman coding of its level indices (Sec. V-A, eq. Nofbits: the
 * paper reports bits per weight and per activation as average Huffman code lengths).
 *   counts[k]      = number of entries equal to level lo + k       (DEVICE uint64[n_levels], nullable)
 *   total_bits     = total code length of an optimal prefix code   (DEVICE uint64[1], nullable)
 *   bits_per_entry = total_bits / n                                (DEVICE fp32[1], nullable)
 * idx: DEVICE int8[n], 16-byte aligned (the hard indices or the draws of the quantizer, stored as the
 * quantizer stores them: minus 128 for a level set that reaches beyond 127); entries outside
 * [lo, lo + n_levels) are ignored.  The total is the same for every Huffman tree of the
 * counts.  A tensor in which a single level occurs costs one bit per entry (the paper does not
 * treat the case); n = 0 gives zeros.  Scratch: cdl_huffman_workspace_bytes(n), 256-byte aligned.
 */
size_t cdl_huffman_workspace_bytes(int64_t n);
int cdl_huffman_bits(const int8_t *idx, int64_t n, int32_t lo, int32_t n_levels,
                     unsigned long long *counts, unsigned long long *total_bits, float *bits_per_entry,
                     void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Forward layer product over quantized operands (Sec. IV-A; Algorithm 1, forward step):
 *   acc[m,n] = sum_k a_idx[m,k] * b_idx[n,k]        exact int32             (int32[M,N], nullable)
 *   y[m,n]   = (delta_a * delta_b) * acc[m,n]       one fp32 multiply       (fp32[M,N],  nullable)
 * a_idx: int8[M,K] (activations), b_idx: int8[N,K] (weights, one row per output feature); the
 * contraction index is contiguous in both.  At least one of acc / y must be non-NULL.
 * CDL_ERR_RANGE if K * 128 * 128 could overflow int32 (K > 131071).
 */
int cdl_qgemm_fwd(const int8_t *a_idx, const int8_t *b_idx, int32_t M, int32_t N, int32_t K,
                  float delta_a, float delta_b, int32_t *acc, float *y,
                  void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The same product for operands stored with an offset (Sec. IV-A on the unsigned 8-bit alphabet of
 * eq. repo_alphabet; first and last layer in Sec. V-B): a_idx holds level index - a_offset, b_idx holds
 * level index - b_offset (each offset 0 or 128, as cdl_index_offset reports for the operand's quantizer), and
 *   acc[m,n] = sum_k (a_idx[m,k] + a_offset) * (b_idx[n,k] + b_offset),
 * the product of the level indices themselves: the matrix cores multiply the stored int8 values, and the
 * epilogue adds a_offset * sum_k b_idx[n,k] + b_offset * sum_k a_idx[m,k] + K * a_offset * b_offset from row
 * sums that a small kernel forms first.  CDL_ERR_RANGE if K products of indices up to 255 (operand with offset)
 * or 128 could overflow int32; CDL_ERR_PARAM for other offsets.  Scratch: cdl_qgemm_fwd_offset_workspace_bytes.
 */
int cdl_qgemm_fwd_offset(const int8_t *a_idx, const int8_t *b_idx, int32_t M, int32_t N, int32_t K,
                         float delta_a, float delta_b, int32_t a_offset, int32_t b_offset,
                         int32_t *acc, float *y, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Backward of that product with respect to the two quantized operands (Algorithm 1, backward
 * step; these are the dL/dQ_p factors of eq. partialX3 / partialW3).  g: fp32[M,N] = dL/dy.
 *   d_a_hat[m,k] = delta_b * sum_n g[m,n] * b_idx[n,k]                       (fp32[M,K], nullable)
 *   d_b_hat[n,k] = delta_a * sum_m g[m,n] * a_idx[m,k]                       (fp32[N,K], nullable)
 * The gradient stays fp32 (the paper quantizes weights and activations only).  Internally every
 * g is rounded to q = rint(g * 2^(8L-1) / sigma) for one power-of-two sigma > max|g|, q is written
 * in L balanced base-256 digits (int8 limbs), each limb product is accumulated exactly in int32 on
 * the int8 matrix cores and the limbs are recombined in double.  Every g is thereby represented to
 * within sigma * 2^-8L, so an output differs from the exact contraction of the fp32 g by at most
 *   step * sigma * 2^-8L * (largest sum of |index| over the contraction, one sum per output column)
 * whatever the values and signs of g; L (3..6) is chosen on the device as the smallest count for
 * which this bound is at most 9e-7.  (Only if six limbs do not reach that - contractions over many
 * millions of large indices - is the bound larger; it is reported, see below.)
 * At least one output non-NULL.  CDL_ERR_RANGE if d_a_hat is requested and N > 131071 (int32
 * accumulators over the contraction; the contraction over M is cut into pieces internally), or if
 * d_b_hat is requested and M > 11 000 000 (32-bit offsets into the transposed copy of a_idx).
 * Diagnostics: once the call has run, the first two int32 of ws hold the limb counts the device
 * chose for d_a_hat and for d_b_hat, and the two doubles at byte offsets 32 and 40 of ws the bounds
 * above for the two products (meaningful for a product that was requested; d_a_hat with N <= 32 is
 * formed directly in double, without limbs).
 */
int cdl_qgemm_bwd(const float *g, const int8_t *a_idx, const int8_t *b_idx,
                  int32_t M, int32_t N, int32_t K, float delta_a, float delta_b,
                  float *d_a_hat, float *d_b_hat,
                  void *ws, size_t ws_bytes, void *hip_stream);

/*
 * cdl_qgemm_bwd for operands stored with an offset (see cdl_qgemm_fwd_offset): the gradients with respect to
 * the quantized operands whose level indices are a_idx + a_offset and b_idx + b_offset,
 *   d_a_hat[m,k] = delta_b * sum_n g[m,n] * (b_idx[n,k] + b_offset)
 *   d_b_hat[n,k] = delta_a * sum_m g[m,n] * (a_idx[m,k] + a_offset).
 * The offset parts, b_offset * delta_b * sum_n g[m,n] and a_offset * delta_a * sum_m g[m,n], are sums of the
 * unrounded fp32 gradient taken in double by separate passes over g.  Scratch: cdl_qgemm_bwd_workspace_bytes.
 */
int cdl_qgemm_bwd_offset(const float *g, const int8_t *a_idx, const int8_t *b_idx,
                         int32_t M, int32_t N, int32_t K, float delta_a, float delta_b,
                         int32_t a_offset, int32_t b_offset, float *d_a_hat, float *d_b_hat,
                         void *ws, size_t ws_bytes, void *hip_stream);

/*
 * cdl_quantize_fwd (hard index only) and cdl_qgemm_fwd in one kernel: y = delta_a * delta_b * (Q_idx(x) . b_idx^T),
 * where Q_idx(x)[m,k], the level index nearest to x[m,k] (ties: the lower one) under the quantizer *p_a, is formed
 * tile by tile on the chip and never written to memory (Sec. III-A, the mode of the CPMF; Sec. IV-A).
 *   x DEVICE fp32[M,K], b_idx DEVICE int8[N,K], y DEVICE fp32[M,N] (all required when M*N > 0)
 * y is bit for bit what the two calls give.  The fp32 activations are read once per 512 output columns instead of
 * their int8 indices once per 256: for wide layers this moves more data and costs the nearest-level rule N / 512
 * times per entry - it pays where the indices are not needed again (inference), not inside a training step, whose
 * backward products read them.  Restrictions: K a multiple of 128, K <= 131071, a level set stored without an
 * offset (cdl_index_offset(p_a) == 0), else CDL_ERR_PARAM / CDL_ERR_RANGE.  No scratch.
 */
int cdl_qgemm_fwd_quantize(const float *x, const cdl_qparams *p_a, const int8_t *b_idx, int32_t M, int32_t N, int32_t K,
                           float delta_b, float *y, void *hip_stream);

/*
 * The forward product of a convolutional layer over level indices (Sec. IV-A, the forward pass over quantized
 * weights and activations, for the convolutional layers of Sec. II), without forming the matrix of input windows:
 *   acc[b,p,q,n] = sum_{r,s,c} X[b, p*stride + r - pad, q*stride + s - pad, c] * w_idx[n,r,s,c],
 *   y = delta_x * delta_w * acc,          P = (H + 2 pad - R) / stride + 1, Q = (W + 2 pad - S) / stride + 1,
 * where X is the level index of the activation, x_idx + x_offset, inside the image and 0 (the quantized value 0)
 * outside it.
 *   x_idx  DEVICE int8[B,H,W,C] (channels contiguous), stored minus x_offset (0, or 128 for the unsigned 8-bit
 *          alphabet: cdl_index_offset); w_idx DEVICE int8[N,R,S,C], level indices as they are
 *   acc    DEVICE int32[B,P,Q,N] (nullable), y DEVICE fp32[B,P,Q,N] (nullable), at least one of them
 * The result is bit for bit what cdl_qgemm_fwd(_offset) gives on the [B*P*Q, R*S*C] matrix of windows; the
 * activations are read where they lie, each about R*S/stride^2 times from cache instead of once from a matrix
 * R*S/stride^2 times their size.  Restrictions: C a multiple of 16, pad < R and pad < S, R*S*C <= 32768
 * (CDL_ERR_PARAM / CDL_ERR_RANGE otherwise: form the matrix and call cdl_qgemm_fwd there).  Both pointers 16-byte
 * aligned.  Scratch: cdl_qconv_fwd_workspace_bytes(N, x_offset), which is 0 when x_offset is 0 (the padding then
 * comes from a page of zeros inside the library's device code; the first such call on a GPU looks its address up
 * with hipGetSymbolAddress, so make one call on each GPU before capturing this entry point into a HIP graph).
 */
size_t cdl_qconv_fwd_workspace_bytes(int32_t N, int32_t x_offset);
int cdl_qconv_fwd(const int8_t *x_idx, const int8_t *w_idx, int32_t B, int32_t H, int32_t W, int32_t C, int32_t N,
                  int32_t R, int32_t S, int32_t stride, int32_t pad, float delta_x, float delta_w, int32_t x_offset,
                  int32_t *acc, float *y, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The weight gradient of that convolutional layer (Algorithm 1, backward step), again without the caller forming
 * the matrix of input windows:
 *   d_w_hat[n,r,s,c] = delta_x * sum over (b,p,q) of g[b,p,q,n] * X[b, p*stride + r - pad, q*stride + s - pad, c]
 * with X as in cdl_qconv_fwd (level index x_idx + x_offset inside the image, 0 outside).  It is cdl_qgemm_bwd's
 * d_b_hat on the window matrix - same limbs, same exactness - whose transposed copy (which that product needs
 * anyway) is gathered straight from the activations.
 *   g DEVICE fp32[B,P,Q,N], x_idx DEVICE int8[B,H,W,C], d_w_hat DEVICE fp32[N,R,S,C]
 * Restrictions as for cdl_qconv_fwd, and B*P*Q <= 11 000 000.  Scratch: cdl_qconv_bwd_weights_workspace_bytes
 * (it holds the transposed window matrix: R*S*C * B*P*Q bytes).
 */
size_t cdl_qconv_bwd_weights_workspace_bytes(int32_t B, int32_t H, int32_t W, int32_t C, int32_t N, int32_t R, int32_t S,
                                             int32_t stride, int32_t pad);
int cdl_qconv_bwd_weights(const float *g, const int8_t *x_idx, int32_t B, int32_t H, int32_t W, int32_t C, int32_t N,
                          int32_t R, int32_t S, int32_t stride, int32_t pad, float delta_x, int32_t x_offset,
                          float *d_w_hat, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The gradient with respect to the quantized activations of that convolutional layer (Algorithm 1, backward step):
 *   d_x_hat[b,h,w,c] = delta_w * sum over (p,q,r,s,n) with p*stride + r - pad = h, q*stride + s - pad = w of
 *                      g[b,p,q,n] * w_idx[n,r,s,c],
 * an exact real contraction over (r,s,n) rounded once, as cdl_qgemm_bwd's d_a_hat is: the same limb product, whose
 * fp32 operand is gathered from g tap by tap (a transposed convolution) instead of read row by row.
 *   g DEVICE fp32[B,P,Q,N], w_idx DEVICE int8[N,R,S,C] (level indices as they are), d_x_hat DEVICE fp32[B,H,W,C]
 * Restrictions: N and C multiples of 4, stride 1 or 2, pad < R and pad < S, R*S*N <= 131071
 * (CDL_ERR_PARAM / CDL_ERR_RANGE otherwise).  Pointers 16-byte aligned.  Scratch:
 * cdl_qconv_bwd_activations_workspace_bytes (a rearranged copy of the weights and small tables).
 */
size_t cdl_qconv_bwd_activations_workspace_bytes(int32_t B, int32_t H, int32_t W, int32_t C, int32_t N, int32_t R, int32_t S,
                                                 int32_t stride, int32_t pad);
int cdl_qconv_bwd_activations(const float *g, const int8_t *w_idx, int32_t B, int32_t H, int32_t W, int32_t C, int32_t N,
                              int32_t R, int32_t S, int32_t stride, int32_t pad, float delta_w,
                              float *d_x_hat, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The backward step of Algorithm 1 for a layer in one call: cdl_qgemm_bwd followed by cdl_quantize_bwd on its
 * d_a_hat (and, optionally, on its d_b_hat), with the quantizer's backward pass (Lemma 1; eq. partialX3, Jgradqx,
 * Jgrad_alpha_q) applied to each tile of dL/dQ(x) in the epilogue of the product, while the tile is still on the
 * chip.  dL/dQ(x) itself is never written to memory or read back (on a transformer-sized layer that is a fifth of the
 * backward pass's traffic).  Arguments as for the two calls it replaces:
 *   theta_a   fp32[M,K], the activations that were quantized into a_idx with the quantizer *p_a
 *   a_idx     int8[M,K] as cdl_quantize_fwd stored it (needed for d_b_hat only), b_idx int8[N,K] stored minus b_offset
 *   d_theta_a fp32[M,K]  = (delta_b * sum_n g[m,n] * level index of b[n,k]) * dQ_d/dtheta(theta_a[m,k])   (required)
 *   d_delta_a, d_alpha_a  the two scalar gradients of the activation quantizer       (DEVICE fp32[1], nullable)
 *   d_b_hat   fp32[N,K] as in cdl_qgemm_bwd(_offset), with a_offset = cdl_index_offset(p_a)              (nullable)
 * The weight operand likewise, if theta_b is given (all five of its arguments may be NULL instead): the quantizer's
 * backward pass on the weights (eq. partialW3, Jgradqw, Jgradq_alpha_w) is applied where the pieces of the
 * contraction over M are added up, so dL/dQ(w) is not read back either:
 *   theta_b   fp32[N,K], the weights that were quantized into b_idx with *p_b; p_b->delta must equal delta_b and
 *             cdl_index_offset(p_b) must equal b_offset, else CDL_ERR_PARAM
 *   d_theta_b fp32[N,K]  = (delta_a * sum_m g[m,n] * level index of a[m,k]) * dQ_d/dtheta(theta_b[n,k])   (required then)
 *   d_delta_b, d_alpha_b  the two scalar gradients of the weight quantizer              (DEVICE fp32[1], nullable)
 *   d_b_hat   may still be requested and is written by the same kernel.
 * Results equal those of the separate calls (the same arithmetic on the same fp32 intermediate; the scalar
 * sums are added up in a different, fixed order).  Restrictions: M, N, K > 0, K a multiple of 4 and N > 32, else
 * CDL_ERR_PARAM - use the separate calls there.  Scratch: cdl_qgemm_bwd_workspace_bytes(M, N, K).
 */
int cdl_qgemm_bwd_quantize_bwd(const float *g, const int8_t *a_idx, const int8_t *b_idx, int32_t M, int32_t N, int32_t K,
                               const float *theta_a, const cdl_qparams *p_a, float delta_b, int32_t b_offset,
                               float *d_theta_a, float *d_delta_a, float *d_alpha_a, float *d_b_hat,
                               const float *theta_b, const cdl_qparams *p_b, float *d_theta_b, float *d_delta_b, float *d_alpha_b,
                               void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Optional per-kernel timing (a measurement aid, not part of the method).  While enabled, every
 * kernel the library enqueues is bracketed by a pair of HIP events recorded on the caller's
 * stream.  cdl_profile_collect waits for the recorded events, writes up to max_records entries
 * (launch order) into `out` (HOST memory), forgets them and returns how many it wrote, or a
 * negative cdl_status.  Enabling creates HIP events, which is the only place the library
 * allocates anything; it is off by default.
 */
typedef struct cdl_profile_record {
    char  kernel[56];   /* name of the kernel, NUL-terminated */
    float ms;           /* elapsed time between its two events */
} cdl_profile_record;

/*
 * Measurement aid, not part of the method: enqueues a kernel that only issues int8 matrix-core
 * instructions on register-resident operands (`blocks` workgroups of four waves, `iters` trips of
 * eight 32x32x32 MFMAs per wave) and writes the number of integer operations it performs to *ops
 * (HOST double, nullable).  random_operands = 0 keeps the operand bits constant, 1 gives every MFMA
 * pseudo-random operand bits.  Timed with cdl_profile_* it yields the matrix-core rate the chip
 * sustains at its power limit, which is what the GEMM kernels' fractions should be read against.
 * sink: DEVICE int[1], never written in practice.
 */
int cdl_probe_mfma_int8(int32_t iters, int32_t random_operands, int32_t blocks, void *sink, double *ops, void *hip_stream);

int cdl_profile_enable(int enable);
int cdl_profile_collect(cdl_profile_record *out, int max_records);
/*
 * Restricts the timing to launches recorded under exactly this kernel name (as cdl_profile_collect reports it);
 * NULL or "" = every launch again.  An event pair costs a few microseconds of stream time per launch, so a
 * caller that times a whole step and wants one kernel's duration from inside it brackets that kernel only.
 */
int cdl_profile_only(const char *kernel);

/* Text for a cdl_status. */
const char *cdl_status_string(int status);

/* hipError_t of the most recent failed HIP call made by this library in this process (0 = none). */
int cdl_last_hip_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int cdl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CDL_H */
