/*
 * mesa.h -- C ABI of libmesa: Mesa's activation-compression hot path on one MI355X (gfx950).
 *
 * Forward half: 8-bit quantization of the activations a Transformer layer saves, head-wise for
 * multi-head self-attention and channel-group-wise elsewhere, with the clipping range alpha and
 * the offset beta kept as running estimates.  Backward half: de-quantization fused into the
 * gradients of softmax, GELU, LayerNorm and the Linear weight gradient.
 * (Mesa, arXiv 2111.11124: Sec. 3.1 Eq. 1-2; Sec. 3.2 Eq. 3-7; Fig. "bucketing"; Sec. 3.3.)
 *
 * Common conventions
 *   Pointers    Every data pointer is a DEVICE pointer owned by the caller.  The library never
 *               allocates, frees or keeps one.  x, q, dy, dx, x_hat, dW and ws must be 16-byte
 *               aligned; alpha, beta, mean, rstd, gamma, dgamma, dbeta, db 4-byte aligned.
 *   Layout      A tensor is contiguous and viewed as (outer, groups, inner): element (o, g, i) is
 *               at flat index (o*groups + g)*inner + i and uses alpha[g], beta[g].
 *                 head-wise (q, k, v, attention):  (B, N_h, N, D_h) -> outer=B, groups=N_h, inner=N*D_h
 *                 channel groups (token matrices): (B*N, D)        -> outer=B*N, groups=G, inner=D/G
 *   Codes       int8, q = x_bar - 128 with x_bar in [0, 255] from Eq. (3); Eq. (5) adds 128 back.
 *   Parameters  alpha[g], beta[g]: binary32 on the device, 2*groups values per tensor.
 *   dtype       storage type of activations and gradients; all arithmetic is binary32
 *               (the matrix-core contraction multiplies in the storage type, accumulates binary32).
 *   stream      a hipStream_t (NULL = the default stream).  Every call only enqueues kernels and
 *               returns; there is no host synchronisation and no host read of device data.
 *   ws          caller-provided device scratch of at least mesa_workspace_bytes(...) bytes; its
 *               contents are undefined before and after a call.
 *   Errors      Arguments are checked on the host before anything is enqueued.  On an argument,
 *               shape or workspace error nothing is written.  MESA_ERR_LAUNCH is what the HIP runtime
 *               reports after a launch (a call of several kernels stops at the first that fails, so a
 *               later kernel never consumes scratch nobody wrote); it may also be an error that an
 *               earlier HIP call of the calling thread left unread.  Zero elements is MESA_OK and a no-op.
 *   Threads     No global mutable state; calls on distinct streams may run concurrently provided
 *               they use distinct ws and outputs.
 *   Limits      groups <= 8192; for groups > 1, inner < 2^30.  Outside them: MESA_ERR_UNSUPPORTED.
 */
#ifndef MESA_H
#define MESA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MESA_OK = 0,
    MESA_ERR_INVALID_ARG = 1,  /* null pointer, negative extent, misaligned pointer, bad enum, lambda outside [0,1] */
    MESA_ERR_UNSUPPORTED = 2,  /* a shape outside the limits stated with each call */
    MESA_ERR_WORKSPACE = 3,    /* ws is null or ws_bytes is too small */
    MESA_ERR_LAUNCH = 4        /* the HIP runtime reported an error at launch */
} mesa_status;

/* Storage type of activations and gradients.  The paper trains with binary16 mixed precision; bfloat16
 * (upper half of a binary32 word, round to nearest even on store) is accepted wherever binary16 is.
 * Codes and parameters are decided in binary32 from the
 * stored value whatever its type. */
typedef enum { MESA_F32 = 0, MESA_F16 = 1, MESA_BF16 = 2 } mesa_dtype;

typedef enum {
    MESA_ROUND_NEAREST_EVEN = 0, /* ablation "nearest rounding"; ties to even */
    MESA_ROUND_STOCHASTIC = 1    /* Eq. (4), the method's default */
} mesa_round;

typedef struct { int64_t outer, groups, inner; } mesa_layout;

typedef enum {
    MESA_OP_UPDATE_RUNNING_PARAMS = 0, /* d0,d1,d2 = outer, groups, inner */
    MESA_OP_LAYERNORM_BWD_Q = 1,       /* d0,d1,d2 = M, D, G */
    MESA_OP_LINEAR_DW_Q = 2,           /* d0,d1,d2 = M, K, N_out */
    MESA_OP_SOFTMAX_FWD_Q = 3,         /* d0,d1,d2 = B*H*rows, H, cols */
    MESA_OP_LAYERNORM_FWD_Q = 4        /* d0,d1,d2 = M, D, G */
} mesa_op;

/*
 * Running estimates, Sec. 3.2 Eq. (6)-(7); initialisation from the first iteration's min-max
 * (Sec. 5.1, implementation details).
 *   mn_g, mx_g = min / max over every element of group g in x (all samples: the parameters are
 *   shared across samples).
 *   first_call != 0:  alpha_g = mx_g - mn_g,  beta_g = mn_g
 *   otherwise:        alpha_g = lambda*alpha_g + (1-lambda)*(mx_g - mn_g)
 *                     beta_g  = lambda*beta_g  + (1-lambda)*mn_g
 * in binary32, each product, difference and sum rounded separately (no fused multiply-add), so the
 * result is reproducible bit for bit.  A minimum of -0.0 is returned as +0.0.
 * x: [outer*groups*inner] of dt (in).  alpha, beta: [groups] binary32 (in/out).
 * ws: MESA_OP_UPDATE_RUNNING_PARAMS bytes.
 */
mesa_status mesa_update_running_params(const void *x, mesa_dtype dt, mesa_layout L,
                                       float *alpha, float *beta, float lambda, int first_call,
                                       void *ws, size_t ws_bytes, void *stream);

/*
 * Symmetric RANGE (a second, milder reading of the ablation of Sec. 5.2; the scale-only scheme proper is
 * mesa_quantize_sym below): one scale from m_g = max |x| over group g, no free offset, but the codes and
 * every other call stay the asymmetric ones.  The clipping range is [-m_g, +m_g]: the call above with mn_g := -m_g and mx_g := +m_g, so that alpha_g
 * moves towards 2 m_g and beta_g towards -m_g.  Quantizer, dequantizer and the backward calls take
 * the resulting alpha, beta unchanged.  Arguments, workspace and errors: as for the call above.
 */
mesa_status mesa_update_running_params_sym(const void *x, mesa_dtype dt, mesa_layout L,
                                           float *alpha, float *beta, float lambda, int first_call,
                                           void *ws, size_t ws_bytes, void *stream);

/*
 * Scale-only symmetric quantization, the scheme the ablation of Sec. 5.2 ("asymmetric vs. symmetric quantization")
 * compares the method with: the input is quantized by a scale factor only -- no offset, zero is a code.  The paper
 * prints the scale as (2^b - 1) / max|X|; with signed b-bit codes that would need b + 1 bits, so the signed reading is
 * taken: 127 steps on each side of zero.  Three calls:
 *   mesa_update_running_scale_sym   m_g <- lambda*m_g + (1-lambda)*max|x| over group g  (first_call: m_g = max|x|)
 *   mesa_quantize_sym               q = clip(round(x * (127 / m_g)), -127, 127);  round: nearest-even or Eq. (4)
 *   mesa_dequantize_sym             x_hat = q * (m_g / 127)
 * binary32, every operation rounded on its own; random source, layouts, workspace and errors as for the asymmetric
 * calls.  m: [groups] binary32 on the device.  The fused backward calls take these codes as well, with
 * alpha_g = m_g * 255/127 and beta_g = -m_g * 128/127 (the same x_hat up to rounding).
 */
mesa_status mesa_update_running_scale_sym(const void *x, mesa_dtype dt, mesa_layout L, float *m, float lambda,
                                          int first_call, void *ws, size_t ws_bytes, void *stream);
mesa_status mesa_quantize_sym(const void *x, mesa_dtype dt, mesa_layout L, const float *m, int8_t *q,
                              mesa_round mode, uint64_t seed, uint64_t offset, void *stream);
mesa_status mesa_dequantize_sym(const int8_t *q, mesa_layout L, const float *m, void *x_hat, mesa_dtype dt,
                                void *stream);

/*
 * Fixed offset, Sec. 6 (evolution of alpha and beta in FFN layers): the offset of the second FFN
 * layer's input settles at the minimum of GELU, about -0.17, so it need not be estimated.  beta_g = beta_fixed for
 * every group; alpha_g is the running estimate of mx_g - beta_fixed (Eq. (6) with the minimum
 * replaced by beta_fixed; first_call != 0: alpha_g = mx_g - beta_fixed).  Values below beta_fixed
 * saturate at the lowest code.  beta: [groups] (out).  beta_fixed must be finite.
 * Other arguments, workspace and errors: as for mesa_update_running_params.
 */
mesa_status mesa_update_running_params_fixed_beta(const void *x, mesa_dtype dt, mesa_layout L,
                                                  float *alpha, float *beta, float lambda,
                                                  int first_call, float beta_fixed,
                                                  void *ws, size_t ws_bytes, void *stream);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture, serving loops,
 * harnesses that forbid hipMalloc): mesa_update_running_params with the partial extrema in a
 * device array that the library owns (mesa_static_scratch_bytes() = 1 MiB per GPU, held until the
 * process ends) instead of a caller's workspace.  Same kernels, same results bit for bit.  The call
 * allocates nothing and frees nothing; its first use on a device looks the array's address up once.
 * Limit: groups <= 4096 (the array holds the partial extrema, 8 bytes per group, of at least 32
 * workgroups), else MESA_ERR_UNSUPPORTED; with many groups the scan runs on as many workgroups as
 * the array has room for (fewer than with a caller's workspace: slower, same results).  Every call on a GPU shares that GPU's array: two calls that overlap
 * in time on one GPU (distinct streams, or threads) race; calls on one stream do not.
 */
mesa_status mesa_update_running_params_static(const void *x, mesa_dtype dt, mesa_layout L,
                                              float *alpha, float *beta, float lambda, int first_call,
                                              void *stream);
size_t mesa_static_scratch_bytes(void);

/*
 * Quantizer, Sec. 3.2 Eq. (3)-(4):  x_bar = clip(round((x - beta_g) * (255 / alpha_g)), 0, 255).
 * binary32, separately rounded: r = 255/alpha_g (0 when alpha_g <= 0), t = x - beta_g, v = t*r,
 *   nearest:     w = v rounded to the nearest integer, ties to even
 *   stochastic:  w = floor(v + u), u in [0,1) -- rounds up with probability frac(v)
 * then w is clipped to [0, 255] and stored as q = w - 128.
 * Random source (the paper names none): Philox-4x32-10 keyed by `seed`; the counter is
 * offset + e/8 for flat element index e (64-bit, counter words 0-1), and element e takes 16 bits of
 * the 128-bit output: word (e%8)/2, low half for even e, high half for odd e; u = bits * 2^-16.
 * A caller advances `offset` by ceil(numel/8) between calls so that streams never repeat.
 * x: [numel] of dt (in).  q: [numel] int8 (out).  alpha, beta: [groups] (in).
 */
mesa_status mesa_quantize_headwise(const void *x, mesa_dtype dt, mesa_layout L,
                                   const float *alpha, const float *beta, int8_t *q,
                                   mesa_round mode, uint64_t seed, uint64_t offset, void *stream);

/*
 * Single-pass forward: Sec. 3.2 Eq. (3)-(4) and Eq. (6)-(7) in ONE read of x.  The codes are taken
 * with alpha, beta as they are on entry; the same pass gathers this batch's per-group extrema, and
 * the running estimates are then moved by Eq. (6)-(7) (never the first-call form) for the next call.
 * This is a variant, not the order Sec. 5.1 implies: there the first iteration's statistics
 * initialise the parameters it quantizes with, so a training run starts with
 * mesa_update_running_params(first_call = 1) + mesa_quantize_headwise and may use this call from
 * the second iteration on; its parameters then lag the two-call order by exactly one step.
 * Arithmetic, rounding modes, random source and layouts: as in the two calls it combines, bit for bit.
 * x: [numel] of dt (in).  alpha, beta: [groups] (in/out).  q: [numel] int8 (out).
 * ws: MESA_OP_UPDATE_RUNNING_PARAMS bytes.  Limits: the layout's (groups <= 8192; beyond 4096 groups the kernel's
 * tables take more than half of a compute unit's local memory: one workgroup per unit, slower).
 */
mesa_status mesa_quantize_update_fused(const void *x, mesa_dtype dt, mesa_layout L,
                                       float *alpha, float *beta, float lambda, int8_t *q,
                                       mesa_round mode, uint64_t seed, uint64_t offset,
                                       void *ws, size_t ws_bytes, void *stream);

/*
 * A Mesa GELU layer's forward in one pass over x (Sec. 3.1: the forward output is computed from the
 * exact input, the input is what is saved, compressed): y = gelu(x) (exact, erf form), and for the
 * saved input x exactly what mesa_quantize_update_fused does -- codes q with alpha, beta as they are
 * on entry, Eq. (3)-(4), then the running estimates moved by this batch's extrema, Eq. (6)-(7).
 * x is read once; per binary16 element 2 bytes in, 2 + 1 bytes out.
 * x: [numel] of dt (in).  y: [numel] of dt (out), not aliasing x.  q: [numel] int8 (out).
 * alpha, beta: [groups] (in/out).  ws: MESA_OP_UPDATE_RUNNING_PARAMS bytes.
 */
mesa_status mesa_gelu_fwd_q(const void *x, mesa_dtype dt, mesa_layout L,
                            float *alpha, float *beta, float lambda, void *y, int8_t *q,
                            mesa_round mode, uint64_t seed, uint64_t offset,
                            void *ws, size_t ws_bytes, void *stream);

/*
 * A Mesa softmax layer's forward in one pass over the logits s (B, H, rows, cols) (Sec. 3.1: the
 * forward output is computed exactly; the output -- the attention map -- is what is saved, compressed):
 *   y = softmax(s) over the last axis (max-subtracted, binary32 arithmetic), stored as dt;
 *   q = codes of the STORED y, head-wise, with alpha, beta as they are on entry, Eq. (3)-(4);
 *   alpha, beta then moved by the per-head extrema of the stored y, Eq. (6)-(7).
 * I.e. mesa_quantize_update_fused applied to y with the layout {B, H, rows*cols}, without the pass
 * that reads y back.  Logits of -infinity (a mask) get probability 0; every row needs one finite logit.  Per binary16 element 2 bytes in, 2 + 1 bytes out.
 * s: [B*H*rows*cols] of dt (in).  y: same (out), not aliasing s.  q: int8 (out).
 * alpha, beta: [H] (in/out).  ws: MESA_OP_SOFTMAX_FWD_Q bytes.  Limits: rows, cols and B*H*rows below 2^31, else
 * MESA_ERR_UNSUPPORTED.  One pass over s for H <= 1024 and rows of up to 256 elements (any length), rows of 8k elements
 * up to 4096, and other rows of at least 8 elements as long as 8 / gcd(cols, 8) of them fit a tile of 8192 elements
 * (odd lengths up to 1024, even ones up to 2048, ...).  Every other shape takes two steps inside the call -- y by a
 * plain kernel, one workgroup per row, then mesa_quantize_update_fused on y (which reads y back) -- and that step's
 * limits: H <= 8192, rows*cols < 2^30.
 */
mesa_status mesa_softmax_fwd_q(const void *s, int64_t B, int64_t H, int64_t rows, int64_t cols,
                               float *alpha, float *beta, float lambda, void *y, int8_t *q,
                               mesa_round mode, uint64_t seed, uint64_t offset,
                               void *ws, size_t ws_bytes, mesa_dtype dt, void *stream);

/*
 * A Mesa LayerNorm layer's forward in one pass over x (M, D) (Sec. 3.1; the saved tensor is the input):
 *   mean_m = sum_j x_mj / D,  rstd_m = 1/sqrt(sum_j (x_mj - mean_m)^2 / D + eps)     (binary32, out: what
 *   y = (x - mean)*rstd*gamma + bias, stored as dt;                                   mesa_layernorm_bwd_q takes)
 *   q = codes of x in G channel groups of D/G columns with alpha, beta as they are on entry, Eq. (3)-(4);
 *   alpha, beta then moved by this batch's per-group extrema of x, Eq. (6)-(7)  (as mesa_quantize_update_fused).
 * x: (M, D) of dt (in).  gamma, bias: [D] of dt.  y: (M, D) of dt (out), not aliasing x.  mean, rstd: [M] binary32
 * (out).  q: int8 (out).  alpha, beta: [G] (in/out).  ws: MESA_OP_LAYERNORM_FWD_Q bytes.
 * One pass over x for D % 8 == 0, (D/G) % 8 == 0, D <= 2048, G <= 1024.  Every other shape takes two steps inside the
 * call -- mesa_quantize_update_fused on x, then mean, rstd and y by a plain kernel, one workgroup per row -- with that
 * step's limit G <= 8192.  D >= 2^31 or M >= 2^40: MESA_ERR_UNSUPPORTED.
 */
mesa_status mesa_layernorm_fwd_q(const void *x, int64_t M, int64_t D, int64_t G,
                                 const void *gamma, const void *bias, float eps,
                                 float *alpha, float *beta, float lambda,
                                 void *y, float *mean, float *rstd, int8_t *q,
                                 mesa_round mode, uint64_t seed, uint64_t offset,
                                 void *ws, size_t ws_bytes, mesa_dtype dt, void *stream);

/*
 * De-quantizer, Sec. 3.2 Eq. (5):  x_hat = (q + 128) * (alpha_g / 255) + beta_g, binary32 with the
 * quotient, product and sum rounded separately, then rounded to dt (nearest even).
 * q: [numel] int8 (in).  x_hat: [numel] of dt (out).
 */
mesa_status mesa_dequantize(const int8_t *q, mesa_layout L, const float *alpha, const float *beta,
                            void *x_hat, mesa_dtype dt, void *stream);

/*
 * Four-bit codes (Sec. 4.2 names lower bit widths as the step beyond the method's fixed eight bits): Eq. (3)-(5)
 * with 2^4 - 1 = 15 steps across the clipping range,
 *   x_bar = clip(round((x - beta_g) * (15 / alpha_g)), 0, 15),     x_hat = x_bar * (alpha_g / 15) + beta_g,
 * same binary32 operation sequence, rounding modes and random source as mesa_quantize_headwise, same running
 * estimates (mesa_update_running_params).  Two codes per byte: element e in byte e/2, the low four bits for even e;
 * q4 holds (numel + 1) / 2 bytes (16-byte aligned; with an odd numel the last byte's high bits are zero).
 * mesa_gelu_bwd_q_b4: dx = dy * gelu'(x_hat) at that reconstruction; dx may alias dy.
 */
mesa_status mesa_quantize_headwise_b4(const void *x, mesa_dtype dt, mesa_layout L,
                                      const float *alpha, const float *beta, uint8_t *q4,
                                      mesa_round mode, uint64_t seed, uint64_t offset, void *stream);
mesa_status mesa_dequantize_b4(const uint8_t *q4, mesa_layout L, const float *alpha, const float *beta,
                               void *x_hat, mesa_dtype dt, void *stream);
mesa_status mesa_gelu_bwd_q_b4(const uint8_t *q4, mesa_layout L, const float *alpha, const float *beta,
                               const void *dy, void *dx, mesa_dtype dt, void *stream);

/*
 * Softmax backward at the de-quantized output, Sec. 3.1 Eq. (2) with G_l = softmax's gradient.
 * The saved tensor is the softmax OUTPUT y (the attention map), shape (B, H, rows, cols),
 * head-wise parameters alpha[H], beta[H].  Per row:  d = sum_j dy_j*y_hat_j,
 * dx_j = y_hat_j * (dy_j - d), accumulated in binary32.
 * yq: int8 (in); dy, dx: [B*H*rows*cols] of dt (in / out); dx may alias dy.
 * Limits: rows, cols, H and B*H*rows below 2^31, else MESA_ERR_UNSUPPORTED.  The tiled kernels take rows of up
 * to 256 elements of any length, and longer rows with R*cols <= 8192 for R = 8/gcd(cols, 8) (cols <= 8192 when
 * cols % 8 == 0, cols <= 1024 when cols is odd), at H <= 1024; every other shape runs a plain kernel, one
 * workgroup per row (rows of 1025 elements: two thirds of the rate of rows of 1024; 4097: 0.96 of 4096).
 */
mesa_status mesa_softmax_bwd_q(const int8_t *yq, int64_t B, int64_t H, int64_t rows, int64_t cols,
                               const float *alpha, const float *beta, const void *dy, void *dx,
                               mesa_dtype dt, void *stream);

/*
 * GELU backward at the de-quantized input, Eq. (2) with the exact (erf) GELU:
 *   dx = dy * (Phi(x_hat) + x_hat*phi(x_hat)),  Phi / phi the standard normal cdf / pdf.
 * xq: int8 (in), channel-group layout L; dy, dx: [numel] of dt; dx may alias dy.
 */
mesa_status mesa_gelu_bwd_q(const int8_t *xq, mesa_layout L, const float *alpha, const float *beta,
                            const void *dy, void *dx, mesa_dtype dt, void *stream);

/*
 * ReLU backward at the de-quantized input (ReLU is among the CNN layers Sec. 3.3 covers, quantized
 * group-wise: for an (N, C, H, W) activation in G channel groups use L = {N, G, (C/G)*H*W}):
 *   dx = dy where x_hat > 0, else 0     (x_hat as mesa_dequantize returns it; 0 at x_hat == 0).
 * Arguments as for mesa_gelu_bwd_q.
 */
mesa_status mesa_relu_bwd_q(const int8_t *xq, mesa_layout L, const float *alpha, const float *beta,
                            const void *dy, void *dx, mesa_dtype dt, void *stream);

/*
 * LayerNorm backward at the de-quantized input, Eq. (2).  Saved: codes of the input x (M, D) in G
 * channel groups of D/G columns, plus the forward's per-row mean and 1/sqrt(var+eps) (binary32).
 *   xn = (x_hat - mean)*rstd,  g = dy*gamma,
 *   dx = rstd * (g - mean_j(g) - xn*mean_j(g*xn)),
 *   dgamma_j = sum_rows dy*xn,  dbeta_j = sum_rows dy        (binary32, fixed summation order)
 * gamma: [D] of dt.  dx: (M, D) of dt, may alias dy.  dgamma, dbeta: [D] binary32 (overwritten).
 * ws: MESA_OP_LAYERNORM_BWD_Q bytes.
 * Limit: D < 2^31, else MESA_ERR_UNSUPPORTED.  The vector kernels take D % 8 == 0, (D/G) % 8 == 0, D <= 4096;
 * every other row length runs two plain kernels (element by element, no workspace needed; the column sums
 * with one lane per column), far below their rate.
 */
mesa_status mesa_layernorm_bwd_q(const int8_t *xq, int64_t M, int64_t D, int64_t G,
                                 const float *alpha, const float *beta,
                                 const float *mean, const float *rstd, const void *gamma,
                                 const void *dy, void *dx, float *dgamma, float *dbeta, mesa_dtype dt,
                                 void *ws, size_t ws_bytes, void *stream);

/*
 * Linear weight gradient at the de-quantized input, Eq. (2) for y = x W^T, W of shape (N_out, K):
 *   dW[n, k] = sum_m dy[m, n] * x_hat[m, k],   db[n] = sum_m dy[m, n]
 * evaluated as  s_g(k) * sum_m dy[m,n]*(q[m,k]+128+c)  +  (beta_g(k) - c*s_g(k)) * db[n]  on the matrix cores
 * (binary16 products for MESA_F16, bfloat16 products for MESA_BF16, binary32 accumulation; fixed summation order;
 * c = 1024 for MESA_F16, where 1024 + code is the cheapest exact binary16 operand, c = 0 otherwise: the binary32
 * sums then carry a term c*db[n] that cancels in the result, which costs accuracy when dy has a large mean --
 * about 3e-4 of max|dW| at a mean of half a standard deviation over 50000 rows, 1e-5 at mean zero).
 * xq: (M, K) int8, K in G channel groups.  dy: (M, N_out) of dt.  dW: (N_out, K) binary32, row-major,
 * overwritten.  db: [N_out] binary32 or NULL.  ws: MESA_OP_LINEAR_DW_Q bytes.
 * K % G == 0.  Widths with K % 16 != 0 or N_out % 8 != 0 (and binary32 tensors) run a plain, slow kernel.
 * Limits: K * N_out < 2^31, else MESA_ERR_UNSUPPORTED.
 */
mesa_status mesa_linear_dw_q(const int8_t *xq, int64_t M, int64_t K, int64_t G,
                             const float *alpha, const float *beta,
                             const void *dy, int64_t N_out, mesa_dtype dt,
                             float *dW, float *db, void *ws, size_t ws_bytes, void *stream);

/*
 * Weight gradient of a two-dimensional convolution at the de-quantized input, Eq. (2) with the gradient of a
 * convolution as G_l (Sec. 3.3: convolutional layers take the group-wise scheme; the input's C_in channels form G
 * groups of C_in / G consecutive channels, one (alpha, beta) pair each).  Contiguous channels-first tensors:
 *   xq (B, C_in, H, W) int8,  dy (B, C_out, OH, OW) of dt,  dW (C_out, C_in, KH, KW) binary32,  db [C_out] binary32 or NULL
 *   OH = (H + 2*pad_h - dil_h*(KH-1) - 1) / stride_h + 1,  OW likewise
 *   dW[co,ci,kh,kw] = sum_{b,oh,ow} dy[b,co,oh,ow] * x_hat[b,ci, oh*stride_h - pad_h + kh*dil_h, ow*stride_w - pad_w + kw*dil_w]
 *   db[co]          = sum_{b,oh,ow} dy[b,co,oh,ow]
 * A position outside the image contributes nothing (the forward pads with zeros, not with de-quantized codes).
 * dW and db are overwritten.  Fixed summation order.  ws: mesa_conv2d_dw_q_workspace_bytes(cv, dt) bytes.
 * 16-bit tensors with a 3x3 kernel and pad_w = 1, or a 1x1 kernel and pad_w = 0, stride_w = dil_w = 1 (any row stride,
 * dilation and padding) run on the matrix cores (binary16 / bfloat16 products, binary32 sums, the contracted operand
 * as in mesa_linear_dw_q; widths that are multiples of 8 with aligned vector loads, other widths with unaligned ones,
 * widths below 8 from copies with rows of eight elements in the workspace); every other case runs a plain kernel, one
 * workgroup per (output, input) channel pair, summed in binary64.
 * Errors: a kernel larger than the padded image, a zero stride or dilation, C_in % G != 0 -> MESA_ERR_INVALID_ARG;
 * C_out*C_in*KH*KW, H*W or OH*OW >= 2^31 -> MESA_ERR_UNSUPPORTED.
 */
typedef struct mesa_conv2d {
    int64_t B, C_in, H, W, C_out, KH, KW;
    int64_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
} mesa_conv2d;
size_t mesa_conv2d_dw_q_workspace_bytes(mesa_conv2d cv, mesa_dtype dt);
mesa_status mesa_conv2d_dw_q(const int8_t *xq, mesa_conv2d cv, int64_t G, const float *alpha, const float *beta,
                             const void *dy, mesa_dtype dt, float *dW, float *db,
                             void *ws, size_t ws_bytes, void *stream);

/*
 * Backward of the two matrix products of self-attention at head-wise de-quantized operands, Sec. 3.1
 * Eq. (2) with G_l = the gradient of a matrix product (the "MatMul" rows of the paper's overhead table;
 * Sec. 3.2: the operands are saved as codes with one (alpha, beta) pair per head).  All tensors are
 * (B, H, N, .) contiguous, upstream gradients and results of dt (binary32 tensors run one plain, slow
 * kernel, as do extents below 8), accumulation in binary32; any N and Dh (nothing needs to be aligned).
 *
 * O = A V with A the attention map (B,H,N,N) and V (B,H,N,Dh):
 *   dA[i,j] = sum_d dO[i,d] * V_hat[j,d],    dV[j,d] = sum_i A_hat[i,j] * dO[i,d]
 * aq, vq: codes (in).  alpha_*, beta_*: [H] (in).  dO: [B,H,N,Dh] (in).  dA: [B,H,N,N], dV: [B,H,N,Dh] (out).
 */
mesa_status mesa_attn_av_bwd_q(const int8_t *aq, const int8_t *vq, int64_t B, int64_t H, int64_t N, int64_t Dh,
                               const float *alpha_a, const float *beta_a, const float *alpha_v, const float *beta_v,
                               const void *dO, void *dA, void *dV, mesa_dtype dt, void *stream);

/*
 * S = scale * Q K^T with Q, K (B,H,N,Dh):
 *   dQ[i,d] = scale * sum_j dS[i,j] * K_hat[j,d],    dK[j,d] = scale * sum_i dS[i,j] * Q_hat[i,d]
 * qq, kq: codes (in).  dS: [B,H,N,N] (in; e.g. the output of mesa_softmax_bwd_q).  dQ, dK: [B,H,N,Dh] (out).
 */
mesa_status mesa_attn_qk_bwd_q(const int8_t *qq, const int8_t *kq, int64_t B, int64_t H, int64_t N, int64_t Dh,
                               const float *alpha_q, const float *beta_q, const float *alpha_k, const float *beta_k,
                               const void *dS, float scale, void *dQ, void *dK, mesa_dtype dt, void *stream);

/* Scratch size in bytes for `op` at the given extents (see mesa_op); 0 for unknown ops. */
size_t mesa_workspace_bytes(mesa_op op, int64_t d0, int64_t d1, int64_t d2, mesa_dtype dt);

const char *mesa_status_string(mesa_status s);
int mesa_version(void);

/*
 * Measurement helpers (not part of the method).
 * mesa_stream_copy: plain device-to-device copy kernel of `bytes` bytes (both pointers 16-byte
 * aligned, bytes % 16 == 0): the known-traffic kernel that bandwidth counters are scaled against.
 * mesa_event_*: HIP events recorded on the stream the kernels are launched on; elapsed_ms waits
 * for `stop` on the host.
 */
mesa_status mesa_stream_copy(const void *src, void *dst, size_t bytes, void *stream);
/* mesa_stream_read: reads `bytes` bytes and writes nothing (sink: one device word, left as it is unless
 * the data fold to one particular value); mesa_stream_fill: writes `word` over `bytes` bytes and reads
 * nothing.  The bandwidth of one direction alone, next to the copy's.  Alignment as for the copy. */
mesa_status mesa_stream_read(const void *src, size_t bytes, void *sink, void *stream);
mesa_status mesa_stream_fill(void *dst, size_t bytes, uint32_t word, void *stream);
/* mesa_mfma_probe: the matrix-core instruction stream of the weight gradient alone -- 256 workgroups of four
 * waves, each wave `steps` times sixteen v_mfma_f32_32x32x16_f16 on a 128 x 128 tile of accumulators
 * (flops of a launch: 256 * 4 * steps * 16 * 32768).  form 0: operands in registers; form 1: operands read
 * from LDS every step; form 2: form 1 plus 12 KB per workgroup and step loaded from `feed` (device memory,
 * 16-byte aligned, 2 MiB <= feed_bytes <= 16 GiB, a multiple of 16; read cyclically) and stored to
 * LDS; form 3: form 2's work shared out among eight waves per workgroup (two per SIMD, a 128 x 64 tile
 * each).  feed is ignored by forms 0 and 1.  sink: 65536 floats of device memory, overwritten (one sum per
 * thread; zeros for steps == 0).  0 <= steps <= 2^20. */
mesa_status mesa_mfma_probe(int form, int64_t steps, const void *feed, size_t feed_bytes, float *sink, void *stream);
mesa_status mesa_event_create(void **event);
mesa_status mesa_event_record(void *event, void *stream);
mesa_status mesa_event_elapsed_ms(void *start, void *stop, float *ms);
mesa_status mesa_event_destroy(void *event);

#ifdef __cplusplus
}
#endif
#endif /* MESA_H */
