/*
 * lbt.h -- C ABI of the INT4 fixed-point backward pass for gfx950 (MI355X).
 *
 * Implements the hot path of "Toward INT4 Fixed-Point Training via Exploring
 * Quantization Error for Gradients" (Kim et al.): per layer, the gradient
 * quantizer whose interval is gamma * max|dY| (Sec. 3.1), with gamma moved by
 * the clipping-factor update of Sec. 3.3 (Eq. 15-16, Alg. 1), then the two
 * integer contractions of the backward pass on the 4-bit codes and the
 * denormalisation of Eq. (4).  Also: the quantized forward product of the same
 * layers (Sec. 3.1), bit-widths 2..8 (Sec. 4.2 uses 4, 5, 6 and 8), two options of
 * the backward calls (interval update inside the call; single-sweep quantizer), a forward
 * call that keeps the quantized operands for a backward call that reads them, and the
 * gradient through the weight / activation quantizers for learned clip values.
 *
 * A layer's calls may be issued on any stream; calls that share a workspace or a state must
 * be ordered (same stream, or the caller's events).  Calls on different streams with
 * workspaces and states of their own may overlap.  A buffer of kept operand codes is written
 * by the forward call and only read by backward calls, which must be ordered after it.
 * A call may be captured into a HIP graph and replayed (it enqueues kernels only: no
 * allocation, no memset, no host synchronisation; the state advances on every replay); make one
 * call of the same shape outside the capture first (the first launch of a kernel variant sets
 * a function attribute).
 *
 * Conventions for every entry point
 *   - Returns LBT_OK (0) or a negative LBT_ERR_* code.  Nothing throws.
 *   - Tensor pointers, state pointers and workspaces are DEVICE pointers owned
 *     by the caller; the library never allocates, frees or retains them.
 *     fp32 tensors must be 16-byte aligned, code buffers 4-byte aligned,
 *     workspaces 256-byte aligned.
 *   - A workspace needs no initialisation and can be reused from call to call
 *     and between layers, by one stream at a time.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; they do not synchronise with the host, except
 *     lbt_state_read which waits for its copy.
 *   - Conditions found on the device (non-finite or all-zero gradient) are
 *     written to lbt_grad_state.status and read back with lbt_state_read.
 *   - All tensors are dense, row-major, fp32.
 *   - Bit-width b (Eq. 1-3): 2..8, the same for the weights, activations and gradients of a
 *     call; 4 unless LBT_BITS(b) is OR-ed into the call's `rounding` word.  A gradient
 *     quantization records its b in st->bits (used by the update, Eq. 16).
 *   - Flat code format (lbt_quantize_grad, lbt_quantize_operand): for b <= 4, ceil(n/2)
 *     bytes, element 2j in the low nibble of byte j and 2j+1 in the high nibble (signed
 *     codes as 4-bit two's complement, a trailing pad nibble is 0); for b > 4, n bytes, one
 *     code each (int8 two's complement or uint8), and `codes` must be 8-byte aligned.
 */
#ifndef LBT_H_
#define LBT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LBT_OK 0
#define LBT_ERR_NULL (-1)        /* a required pointer is NULL                     */
#define LBT_ERR_SHAPE (-2)       /* a size is <= 0 or inconsistent                 */
#define LBT_ERR_UNSUPPORTED (-3) /* bits outside 2..8, unknown flag, size beyond a documented limit */
#define LBT_ERR_WORKSPACE (-4)   /* workspace smaller than lbt_workspace_bytes_*   */
#define LBT_ERR_OVERFLOW (-5)    /* a contraction could exceed int32 accumulators  */
#define LBT_ERR_HIP (-6)         /* a HIP runtime call failed                      */
#define LBT_ERR_ALIGN (-7)       /* a pointer is not aligned as required           */
#define LBT_ERR_TOO_LARGE (-8)   /* lbt_quantize_grad_static: n above LBT_QUANTIZE_STATIC_MAX_N */

#define LBT_STATUS_OK 0
#define LBT_STATUS_NONFINITE 1   /* NaN or Inf seen in a tensor whose maximum was taken */
#define LBT_STATUS_ZERO_GRAD 2   /* max|dY| == 0, or c_g so small (below about q * 2.9e-39) that q / c_g
                                    is not a finite fp32 number: codes 0, clip 0, scale 0, gamma
                                    not updated                                          */

#define LBT_ROUND_NEAREST 0      /* round half to even                              */
#define LBT_ROUND_STOCHASTIC 1   /* (floor(x_n*2^16) + r16) >> 16, r16 from Philox  */
/*
 * May be OR-ed into `rounding`: take the interval from the maximum of the PREVIOUS gradient
 * tensor of this layer (st->gmax as left by the last call) instead of this tensor's own, so
 * that the tensor is swept once; this tensor's maximum is recorded in st->gmax for the next
 * call.  NOT the quantizer of Sec. 3.1 (which uses the tensor's own maximum): a separate,
 * explicitly requested mode.  With st->gmax == 0 (no previous call) all codes are 0 and the
 * status is LBT_STATUS_ZERO_GRAD; a non-finite value in this tensor gives
 * LBT_STATUS_NONFINITE, leaves st->gmax unchanged, and the codes are unspecified.
 */
#define LBT_HINDSIGHT_MAX 2
/*
 * May be OR-ed into `rounding`: the call itself applies the interval update (Alg. 1) to *st
 * once its quantizers have finished, exactly as lbt_update_interval(st) right after the call
 * would (same arithmetic, same conditions: only when the status is LBT_STATUS_OK); saves that
 * call's kernel launch.  Do not call lbt_update_interval for the same tensor again.
 */
#define LBT_FUSED_UPDATE 4
/* May be OR-ed into `rounding`: bit-width b in 2..8 (the paper's experiments: 4, 5, 6, 8). */
#define LBT_BITS(b) (((b) & 15) << 8)

/*
 * Per-layer state of the gradient quantizer: the scalars of Alg. 1 plus the
 * statistics of the last quantized gradient tensor.  Lives in device memory
 * (sizeof = 96).  It is the whole persistent state of the method: saving and
 * restoring it (lbt_state_read / lbt_state_write) resumes a run bit for bit,
 * since the stochastic-rounding stream is a pure function of (seed, step,
 * element index).
 */
typedef struct lbt_grad_state {
  double gamma;      /* clipping factor, Sec. 3.1; c_g = gamma * g_max              */
  double alpha;      /* ratio of large gradients N(G_L)/N(G), Sec. 3.2              */
  double beta;       /* step of the update, Eq. (15)                                */
  double gamma_min;  /* gamma is clamped to [gamma_min, gamma_max] after the update */
  double gamma_max;
  int32_t bits;      /* b                                                           */
  int32_t status;    /* LBT_STATUS_* of the last quantized gradient                 */
  uint64_t step;     /* number of updates done; also the RNG's iteration word       */
  uint64_t n_total;  /* N(G) of the last quantized gradient                         */
  uint64_t n_out;    /* N(G_out): number of |g| > c_g (strict)                      */
  uint64_t sync_word; /* internal: count + arrival ticket of the running quantizer;
                         zero between calls                                         */
  float gmax;        /* g_max = max|G|                                              */
  float clip;        /* c_g = (float)(gamma * (double)g_max)                        */
  float scale;       /* s = c_g / (2^(b-1) - 1), Eq. (2)                            */
  uint32_t sync_max; /* internal: running maximum of the hindsight mode; zero between calls */
} lbt_grad_state;

const char* lbt_version(void);
const char* lbt_strerror(int code);
size_t lbt_state_sizeof(void);

/* Initialise a device-resident state: gamma0 (the paper starts from the full
 * range, gamma = 1), alpha and beta (1e-3 each in the paper's experiments,
 * Sec. 4.1 and supplement S4), clamp range, bit-width.  step = 0. */
int lbt_state_init(lbt_grad_state* st, double gamma0, double alpha, double beta,
                   double gamma_min, double gamma_max, int bits, void* stream);
/* Copy a state device -> host (waits for the stream) / host -> device. */
int lbt_state_read(const lbt_grad_state* st, lbt_grad_state* host_out, void* stream);
int lbt_state_write(lbt_grad_state* st, const lbt_grad_state* host_in, void* stream);

/*
 * Clipping-factor update, Eq. (15)-(16) / Alg. 1:
 *   gamma <- clamp(gamma + beta * sign(N(G_out)/N(G) - alpha/(2^b - 1))), step <- step + 1
 * using n_out, n_total left in *st by the last gradient quantization (which
 * used the gamma being replaced).  sign(0) = 0.  No-op if status != OK.
 */
int lbt_update_interval(lbt_grad_state* st, void* stream);

/*
 * Gradient quantizer of one layer (Sec. 3.1, Eq. 1, 2, 4).
 *   g[n] fp32  ->  codes in the flat format above, values in [-q, q] with
 *   q = 2^(b-1) - 1 ([-7, 7] for b = 4; the most negative code never occurs).
 * Computes g_max, c_g = gamma * g_max, the codes, and N(G_out); writes gmax,
 * clip, scale, n_total, n_out, status to *st.  Does not change gamma or step.
 * The code is decided in fp32: x_n = clip(g) * fl32(q / c_g), one multiply.
 * rounding = LBT_ROUND_STOCHASTIC draws 16 bits per element from
 * Philox4x32-10 with key = seed and counter = (element/8, st->step); element
 * e uses 16-bit lane e%8 of the four output words, low half first.
 * ws: lbt_workspace_bytes_quantize(n) bytes.
 */
int lbt_quantize_grad(const float* g, int64_t n, lbt_grad_state* st, uint64_t seed,
                      int rounding, uint8_t* codes, void* ws, size_t ws_bytes, void* stream);
size_t lbt_workspace_bytes_quantize(int64_t n);

/*
 * lbt_quantize_grad for callers that cannot allocate device memory and have no workspace to
 * pass (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * same arguments, kernels and results, but the scratch (partial maxima and arrival counters,
 * 33 024 bytes) is a static array in the library's device image, one copy per GPU, held until
 * the process ends.  The call allocates nothing (no hipMalloc / hipFree, no allocating library
 * routine).  n up to LBT_QUANTIZE_STATIC_MAX_N elements; above that LBT_ERR_TOO_LARGE and
 * nothing is enqueued.  All calls on one GPU share that GPU's array: calls that overlap on one
 * GPU (different streams or threads) race; order them.  The array needs no clearing between
 * calls (every call resets the counters it uses before it reads them), so a call may follow
 * one of any other size.  The first call on a device looks up the array's address; make that
 * call outside a graph capture.
 */
#define LBT_QUANTIZE_STATIC_MAX_N ((int64_t)1 << 30)
int lbt_quantize_grad_static(const float* g, int64_t n, lbt_grad_state* st, uint64_t seed,
                             int rounding, uint8_t* codes, void* stream);

/*
 * Weight / activation quantizer (Eq. 2 for zero-centred inputs, Eq. 3 for
 * inputs after a ReLU), nearest rounding, same code format as above (unsigned
 * codes are 0..2^b - 1).  c > 0 is the clipping value (learned by the caller in the
 * paper, Sec. 3.1); c <= 0 selects the tensor's own maximum (max|x| signed,
 * max x unsigned).  clip_scale_out (device, 2 floats, may be NULL) receives
 * the clip value and the scale s.  ws: lbt_workspace_bytes_quantize(n).
 * A clip value so small that q / c is not a finite fp32 number (below about q * 2.9e-39) gives
 * all-zero codes, like c = 0 (an all-zero tensor).
 */
int lbt_quantize_operand(const float* x, int64_t n, float c, int is_unsigned, int bits,
                         uint8_t* codes, float* clip_scale_out, void* ws, size_t ws_bytes,
                         void* stream);

/*
 * Gradient of a loss through the operand quantizer, for callers that learn the clip values of
 * weights and activations (Sec. 3.1 learns them end to end and gives no formula; this is the
 * derivative of Eq. 1-4 with the rounding passed straight through, i.e. the step-size gradient
 * of the learned-step-size quantizers the section cites, over q).  With grad_q = dL/dQ(x) (the
 * dW, for a layer's weights, and the dX, for its input activations, that lbt_backward_* returns
 * for that layer):
 *   grad_x[i] = grad_q[i] if lo < x[i] < c, else 0            (lo = -c signed, 0 unsigned)
 *   grad_c    = sum_i grad_q[i] * d_i,   d_i = (round(u_i) - u_i) / q inside the interval,
 *               +1 for x[i] >= c, -1 for x[i] <= -c (signed), 0 for x[i] <= 0 (unsigned),
 *               u_i = clip(x[i], c) / s as the quantizer computes it, q = c / s
 * x, grad_q, grad_x: device, n floats, 16-byte aligned; grad_x may be NULL and may be grad_q
 * (in place).  grad_c: device, one float, may be NULL; products and the sum are taken in fp64
 * in a fixed order (the same inputs give the same bits).  c must be > 0 and finite
 * (LBT_ERR_UNSUPPORTED otherwise: an interval taken from the tensor's maximum has no learned
 * parameter), and large enough that q / c is a finite fp32 number.
 * ws: lbt_workspace_bytes_quantize(n).
 */
int lbt_ste_backward(const float* x, int64_t n, float c, int is_unsigned, int bits,
                     const float* grad_q, float* grad_x, float* grad_c, void* ws, size_t ws_bytes,
                     void* stream);

/*
 * Backward pass of a linear layer Y = X W with row-major X[M,K_in],
 * W[K_in,N_out], dY[M,N_out]:
 *   dX = Q(dY) . Q(W)^T   [M,K_in]      dW = Q(X)^T . Q(dY)   [K_in,N_out]
 * dY goes through the gradient quantizer (as lbt_quantize_grad; statistics
 * are left in *st, gamma is not changed: call lbt_update_interval afterwards);
 * X and W through the operand quantizer with clip values c_x, c_w (<= 0: the
 * tensor's maximum); x_unsigned selects Eq. (3) for X.  The sums run on int8
 * matrix cores with int32 accumulators and are exact; outputs are
 * acc * (s_a * s_b) in fp32.  dX or dW may be NULL to skip that product.
 * Exactness is checked on the host against the worst case: with q = 2^(b-1) - 1 and
 * q_x = 2^b - 1 for unsigned X, the dX contraction needs N_out * q * q < 2^31, and every
 * int32 accumulator of dW (the contraction over M is cut into slices of at most 131072
 * terms, added in 64 bits) needs slice * q * q_x < 2^31: LBT_ERR_OVERFLOW otherwise.
 * Unsigned X with b = 8 (codes 0..255) does not fit the signed int8 operands of the
 * matrix cores: LBT_ERR_UNSUPPORTED when dW is asked for.
 */
int lbt_backward_linear(const float* X, const float* W, const float* dY, int64_t M,
                        int64_t K_in, int64_t N_out, float c_x, int x_unsigned, float c_w,
                        lbt_grad_state* st, uint64_t seed, int rounding, float* dX, float* dW,
                        void* ws, size_t ws_bytes, void* stream);
size_t lbt_workspace_bytes_linear(int64_t M, int64_t K_in, int64_t N_out);

/*
 * Backward pass of a 2-D convolution (cross-correlation, NCHW, no dilation,
 * no groups): X[N,C,H,Wd], W[K,C,R,S], dY[N,K,P,Q], P = (H+2*pad-R)/stride+1:
 *   dX[n,c,h,w]  = s_g s_w * sum_{k,r,s} qG[n,k,p,q] qW[k,c,r,s],  h = p*stride-pad+r, ...
 *   dW[k,c,r,s]  = s_x s_g * sum_{n,p,q} qG[n,k,p,q] qX[n,c,h,w]   (zero outside the image)
 * Same quantizers, state handling and NULL-output rule as the linear call.
 */
int lbt_backward_conv2d(const float* X, const float* W, const float* dY, int64_t N, int64_t C,
                        int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t stride,
                        int64_t pad, float c_x, int x_unsigned, float c_w, lbt_grad_state* st,
                        uint64_t seed, int rounding, float* dX, float* dW, void* ws,
                        size_t ws_bytes, void* stream);
size_t lbt_workspace_bytes_conv2d(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K,
                                  int64_t R, int64_t S, int64_t stride, int64_t pad);

/*
 * Quantized forward pass of the same layers (Sec. 3.1: weights and activations go through
 * Eq. 2 / Eq. 3 before the product, Eq. 4 after it):
 *   linear: Y[M,N_out] = s_x s_w * sum_k qX[m,k] qW[k,n]       X[M,K_in], W[K_in,N_out]
 *   conv:   Y[n,k,p,q] = s_x s_w * sum_{c,r,s} qW[k,c,r,s] qX[n,c,p*stride-pad+r,q*stride-pad+s]
 *           (zero outside the image; X[N,C,H,Wd], W[K,C,R,S], Y[N,K,P,Q])
 * X and W through the operand quantizer (nearest rounding) with clip values c_x, c_w (<= 0:
 * the tensor's maximum); x_unsigned selects Eq. (3) for X.  `flags`: 0 or LBT_BITS(b).
 * acc_Y (may be NULL, shaped like Y): the raw int32 sums.  status (device, may be NULL)
 * receives LBT_STATUS_OK, or LBT_STATUS_NONFINITE when a tensor whose maximum was taken
 * holds NaN / Inf (its codes are then all 0, so Y is 0).  The sums are exact:
 * LBT_ERR_OVERFLOW if K_in (C*R*S) * q * q_x could reach 2^31; LBT_ERR_UNSUPPORTED for
 * unsigned X at b = 8.  The codes stay in the workspace only; lbt_forward_*_save below keeps
 * them for the backward call.
 */
int lbt_forward_linear(const float* X, const float* W, int64_t M, int64_t K_in, int64_t N_out,
                       float c_x, int x_unsigned, float c_w, int flags, float* Y, int32_t* acc_Y,
                       int32_t* status, void* ws, size_t ws_bytes, void* stream);
size_t lbt_workspace_bytes_forward_linear(int64_t M, int64_t K_in, int64_t N_out);
int lbt_forward_conv2d(const float* X, const float* W, int64_t N, int64_t C, int64_t H, int64_t Wd,
                       int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad, float c_x,
                       int x_unsigned, float c_w, int flags, float* Y, int32_t* acc_Y,
                       int32_t* status, void* ws, size_t ws_bytes, void* stream);
size_t lbt_workspace_bytes_forward_conv2d(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K,
                                          int64_t R, int64_t S, int64_t stride, int64_t pad);

/*
 * Forward pass that keeps the quantized operands for the layer's backward pass (Sec. 3.1: the
 * weights and activations are quantized once, in the forward pass; the backward products of
 * the layer read the same quantized tensors).  As lbt_forward_linear / lbt_forward_conv2d, and
 * in the same quantize launch the codes of X in the layout dW reads and of W in the layout dX
 * reads go to `saved` (device memory of the caller, lbt_saved_bytes_*(same shape) bytes,
 * 256-byte aligned, opaque; it also holds the two clip values and the non-finite flags).
 * Y may be NULL: then only the codes are produced (no product; acc_Y and status must be NULL,
 * ws may be NULL).
 *
 * lbt_backward_*_saved: the backward call without X and W: dY goes through the gradient
 * quantizer exactly as in lbt_backward_*, the products read `saved`.  Same geometry, bit-width
 * (LBT_BITS in `rounding` = the `flags` of the saving call) and x_unsigned as the call that
 * wrote `saved`; results are identical to lbt_backward_* on the same X, W, c_x, c_w.  A
 * non-finite X or W seen while saving gives LBT_STATUS_NONFINITE in *st here.  acc_dX / acc_dW
 * (may be NULL) as in lbt_backward_*_acc.  ws: lbt_workspace_bytes_linear / _conv2d.
 * `saved` is only read: several backward calls may use it.
 */
size_t lbt_saved_bytes_linear(int64_t M, int64_t K_in, int64_t N_out);
size_t lbt_saved_bytes_conv2d(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R,
                              int64_t S, int64_t stride, int64_t pad);
int lbt_forward_linear_save(const float* X, const float* W, int64_t M, int64_t K_in,
                            int64_t N_out, float c_x, int x_unsigned, float c_w, int flags,
                            float* Y, int32_t* acc_Y, int32_t* status, void* saved,
                            size_t saved_bytes, void* ws, size_t ws_bytes, void* stream);
int lbt_forward_conv2d_save(const float* X, const float* W, int64_t N, int64_t C, int64_t H,
                            int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t stride,
                            int64_t pad, float c_x, int x_unsigned, float c_w, int flags,
                            float* Y, int32_t* acc_Y, int32_t* status, void* saved,
                            size_t saved_bytes, void* ws, size_t ws_bytes, void* stream);
int lbt_backward_linear_saved(const void* saved, size_t saved_bytes, const float* dY, int64_t M,
                              int64_t K_in, int64_t N_out, int x_unsigned, lbt_grad_state* st,
                              uint64_t seed, int rounding, float* dX, float* dW, int32_t* acc_dX,
                              int32_t* acc_dW, void* ws, size_t ws_bytes, void* stream);
int lbt_backward_conv2d_saved(const void* saved, size_t saved_bytes, const float* dY, int64_t N,
                              int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                              int64_t stride, int64_t pad, int x_unsigned, lbt_grad_state* st,
                              uint64_t seed, int rounding, float* dX, float* dW, int32_t* acc_dX,
                              int32_t* acc_dW, void* ws, size_t ws_bytes, void* stream);

/*
 * Backward pass of a layer whose clip values c_x, c_w are learned (both > 0 and finite where
 * their product is asked for: LBT_ERR_UNSUPPORTED otherwise): lbt_backward_linear /
 * lbt_backward_conv2d followed by lbt_ste_backward on (W, dW) and on (X, dX) in one call, on
 * the call's own workspace.  dW and dX come out masked; grad_c (device, 2 floats) receives dL/dc_w in [0] (when dW is
 * asked for) and dL/dc_x in [1] (when dX is).
 */
int lbt_backward_linear_learned(const float* X, const float* W, const float* dY, int64_t M,
                                int64_t K_in, int64_t N_out, float c_x, int x_unsigned,
                                float c_w, lbt_grad_state* st, uint64_t seed, int rounding,
                                float* dX, float* dW, float* grad_c, void* ws, size_t ws_bytes,
                                void* stream);
int lbt_backward_conv2d_learned(const float* X, const float* W, const float* dY, int64_t N,
                                int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R,
                                int64_t S, int64_t stride, int64_t pad, float c_x,
                                int x_unsigned, float c_w, lbt_grad_state* st, uint64_t seed,
                                int rounding, float* dX, float* dW, float* grad_c, void* ws,
                                size_t ws_bytes, void* stream);

/*
 * lbt_backward_linear and lbt_backward_conv2d with the raw int32 accumulators also written out
 * (acc_dX shaped like dX, acc_dW like dW; either may be NULL).  For checking
 * the integer sums bit for bit.  LBT_ERR_OVERFLOW if the worst case of a whole sum (not
 * only of a slice) does not fit 32 bits.
 */
int lbt_backward_linear_acc(const float* X, const float* W, const float* dY, int64_t M,
                            int64_t K_in, int64_t N_out, float c_x, int x_unsigned, float c_w,
                            lbt_grad_state* st, uint64_t seed, int rounding, float* dX,
                            float* dW, int32_t* acc_dX, int32_t* acc_dW, void* ws,
                            size_t ws_bytes, void* stream);
int lbt_backward_conv2d_acc(const float* X, const float* W, const float* dY, int64_t N,
                            int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                            int64_t stride, int64_t pad, float c_x, int x_unsigned, float c_w,
                            lbt_grad_state* st, uint64_t seed, int rounding, float* dX,
                            float* dW, int32_t* acc_dX, int32_t* acc_dW, void* ws,
                            size_t ws_bytes, void* stream);

/*
 * Optional per-kernel timing (off by default).  While enabled, each kernel the
 * library launches is bracketed by HIP events on the caller's stream.
 * lbt_profile_read waits for the recorded launches and returns, per kernel
 * class 0 .. lbt_profile_kernel_count()-1, the number of launches, their
 * summed duration in ms and their summed algorithmic work (elements for the
 * element-wise kernels, integer operations for the contractions, counted as
 * 2*N*P*Q*K*C*R*S per product); it then clears the records.  Host arrays of
 * `capacity` >= kernel count entries.  lbt_profile_enable also clears.
 * Process-wide; not meant for concurrent use from several threads' streams.
 *
 * lbt_profile_skeleton(1): a measurement aid, never for production: until switched off again the
 * product launches (dX, dW, forward) run their launch, prologue and epilogue but skip the
 * contraction loop, so that every output is 0 and their duration is what a product costs before
 * its first multiply (launch, set-up, writing the result).  Process-wide.
 */
int lbt_profile_skeleton(int on);
int lbt_profile_enable(int on);
int lbt_profile_kernel_count(void);
const char* lbt_profile_kernel_name(int kernel_class);
int lbt_profile_read(int64_t* launches, double* total_ms, double* total_work, int capacity);

#ifdef __cplusplus
}
#endif
#endif /* LBT_H_ */
