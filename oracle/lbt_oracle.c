/*
 * lbt_oracle.c -- CPU oracle for the INT4 fixed-point backward pass
 * (Kim et al., "Toward INT4 Fixed-Point Training via Exploring Quantization
 * Error for Gradients").
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * obviously-correct implementation in double / int64_t that the GPU library is
 * compared against.  It shares no code with the HIP path and must never be
 * called from it.  Only the tests, the smoke entry and the benchmark's
 * cpu_baseline leg use it.
 *
 * What follows the paper, step by step, in the paper's notation:
 *   g_max, c_g = gamma * g_max                     Sec. 3.1 (text after Eq. 4)
 *   clip / scale / round (signed and unsigned)     Eq. (1)-(4)
 *   clip-out count N(G_out, gamma)                 Sec. 3.3 "ULG", Alg. 1 step 5
 *   clipping-factor update                         Eq. (15), (16), Alg. 1
 * What the paper only implies (integer arithmetic for the backward pass,
 * Sec. 1) and is written here as the plain definition:
 *   dX = Q(dY) . Q(W)^T,  dW = Q(X)^T . Q(dY)      integer sums in int64_t
 *   denormalisation by the two scale factors       Eq. (4)
 *
 * Readings taken where the paper is silent (kept identical in the GPU path
 * by independent code):
 *   - the clip value is held in fp32: c = (float)(gamma * (double)g_max);
 *   - the integer code is decided in fp32, the precision of the tensors the
 *     paper quantizes (Sec. 1: full-precision gradients are 32-bit floats):
 *     normalisation x_n = clip(x,c)/s is ONE fp32 multiply by
 *     inv_s = (float)(q / c), no fused multiply-add (-ffp-contract=off);
 *     scales, denormalisation and every diagnostic stay in double;
 *   - the rounding bracket of Eq. (4) is round-half-to-even;
 *   - stochastic rounding (Sec. 4.1 says it is used for gradients, without a
 *     generator) keeps 16 fractional bits: code = floor((floor(x_n * 2^16) +
 *     r16) / 2^16), i.e. x_n rounds up with probability floor(frac * 2^16) /
 *     2^16; r16 are 16 bits from Philox4x32-10 (Salmon et al., SC'11) keyed by
 *     the seed and indexed by (element, step);
 *   - G_out is counted over the whole tensor: |g| > c, strictly;
 *   - sign(0) = 0; gamma is clamped to [gamma_min, gamma_max].
 *
 * Parity status: the tie rule, the precision of c, the generator and the
 * order "quantize with gamma_{i-1}, then update" are fixed by this file, not
 * by the paper ("parity unpinned" for those four choices); everything else is
 * pinned by tests/test_oracle_*.py against closed forms, invariants, brute
 * force in exact rational arithmetic and library routines.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_NONFINITE 1
#define ORC_ZERO_GRAD 2

int orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Philox4x32-10, written from the definition in Salmon et al. (2011): */
/* a 4-word counter, a 2-word key, ten rounds; each round multiplies   */
/* words 0 and 2 by fixed constants, mixes the high halves with words  */
/* 1 and 3 and the round key, and the key is bumped by the Weyl        */
/* constants between rounds.                                           */
/* ------------------------------------------------------------------ */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    uint32_t n0 = hi1 ^ c1 ^ k0;
    uint32_t n1 = lo1;
    uint32_t n2 = hi0 ^ c3 ^ k1;
    uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 16 random bits used for element e at iteration `step`: one Philox call
 * serves 8 consecutive elements; element e takes 16-bit lane (e mod 8),
 * lanes numbered from the low half of word 0 to the high half of word 3. */
static uint32_t r16_for_element(uint64_t e, uint64_t seed, uint64_t step) {
  uint64_t blk = e / 8u;
  uint32_t ctr[4] = {(uint32_t)blk, (uint32_t)(blk >> 32), (uint32_t)step, (uint32_t)(step >> 32)};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t out[4];
  orc_philox4x32_10(ctr, key, out);
  unsigned lane = (unsigned)(e % 8u);
  return (out[lane / 2u] >> (16u * (lane % 2u))) & 0xFFFFu;
}

uint32_t orc_r16(uint64_t e, uint64_t seed, uint64_t step) { return r16_for_element(e, seed, step); }

/* ------------------------------------------------------------------ */
/* g_max = max |g| over one layer's gradient tensor (Sec. 3.1).        */
/* For activations after a ReLU the interval is [0, c]; the max-abs    */
/* fallback for c uses the plain maximum (use_abs = 0).                */
/* ------------------------------------------------------------------ */
int orc_max(const float* x, int64_t n, int use_abs, float* out) {
  float m = 0.0f;
  int bad = 0;
#pragma omp parallel for reduction(max : m) reduction(| : bad) schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    float v = x[i];
    if (!isfinite(v)) { bad = 1; continue; }
    float a = use_abs ? fabsf(v) : v;
    if (a > m) m = a;
  }
  *out = m;
  if (bad) return ORC_NONFINITE;
  if (m == 0.0f) return ORC_ZERO_GRAD;
  return ORC_OK;
}

/* c_g = gamma * g_max, held in fp32 (Sec. 3.1). */
float orc_clip_value(double gamma, float gmax) { return (float)(gamma * (double)gmax); }

/* Number of positive levels: 2^(b-1)-1 for the signed quantizer (Eq. 2),
 * 2^b-1 for the unsigned one (Eq. 3). */
int orc_levels(int bits, int is_unsigned) {
  return is_unsigned ? ((1 << bits) - 1) : ((1 << (bits - 1)) - 1);
}

/* Eq. (1) divides by s = c / q; the code decision multiplies by fl32(q / c).  An
 * interval so small that this factor is not a finite fp32 number (c below about
 * q * 2.9e-39, i.e. subnormal-scale tensors) cannot be normalised by and is
 * treated like c = 0: every code is zero. */
int orc_interval_usable(float c, int bits, int is_unsigned) {
  if (!(c > 0.0f)) return 0;
  float inv_s = (float)((double)orc_levels(bits, is_unsigned) / (double)c);
  return isfinite(inv_s) ? 1 : 0;
}

/* s = c / q (Eq. 2, 3). */
double orc_scale(float c, int bits, int is_unsigned) {
  if (!(c > 0.0f)) return 0.0;
  return (double)c / (double)orc_levels(bits, is_unsigned);
}

/* ------------------------------------------------------------------ */
/* Uniform quantizer, Eq. (1)-(4): clip to the interval, normalise by  */
/* s, round.  Returns the integer code round(x_n); Q(x) = s * code.    */
/* rounding: 0 = nearest (ties to even), 1 = stochastic.               */
/* Also returns through n_out the clip-out count #{ |x| > c }          */
/* (signed) used by Alg. 1.  code[] is int32 so any b in [2,8] fits.   */
/* ------------------------------------------------------------------ */
void orc_quantize(const float* x, int64_t n, float c, int bits, int is_unsigned, int rounding,
                  uint64_t seed, uint64_t step, int32_t* code, uint64_t* n_out) {
  uint64_t cnt = 0;
  if (!orc_interval_usable(c, bits, is_unsigned)) { /* degenerate interval: every code is zero */
    for (int64_t i = 0; i < n; ++i) code[i] = 0;
    if (n_out) *n_out = 0;
    return;
  }
  const int q = orc_levels(bits, is_unsigned);
  const float inv_s = (float)((double)q / (double)c);
  const float lo = is_unsigned ? 0.0f : -c;
#pragma omp parallel for reduction(+ : cnt) schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    float v = x[i];
    /* clip(x, c) = min(max(x, lo), c) */
    float xc = v;
    if (xc < lo) xc = lo;
    if (xc > c) xc = c;
    /* x_n = clip(x, c) / s, as one fp32 multiply by q / c */
    float t = xc * inv_s;
    int32_t k;
    if (rounding == 0) {
      k = (int32_t)rintf(t); /* default rounding mode: ties to even */
    } else {
      /* x_n in units of 2^-16 (the scaling is exact), truncated downwards */
      int64_t fixed = (int64_t)floorf(t * 65536.0f);
      fixed += (int64_t)r16_for_element((uint64_t)i, seed, step);
      /* floor division by 2^16 */
      int64_t d = fixed / 65536;
      if (fixed % 65536 < 0) d -= 1;
      k = (int32_t)d;
    }
    /* t can exceed q by one ulp; keep the code in range */
    int32_t kmin = is_unsigned ? 0 : -q;
    if (k > q) k = q;
    if (k < kmin) k = kmin;
    code[i] = k;
    if (fabsf(v) > c) cnt += 1; /* clip-out gradient, strict inequality */
  }
  if (n_out) *n_out = cnt;
}

/* Two 4-bit codes per byte: element 2j in the low nibble, 2j+1 in the high
 * nibble, two's complement; a trailing pad nibble is zero. */
void orc_pack_nibbles(const int32_t* code, int64_t n, uint8_t* out) {
  int64_t nb = (n + 1) / 2;
  for (int64_t j = 0; j < nb; ++j) {
    uint32_t lo = (uint32_t)code[2 * j] & 0xFu;
    uint32_t hi = (2 * j + 1 < n) ? ((uint32_t)code[2 * j + 1] & 0xFu) : 0u;
    out[j] = (uint8_t)(lo | (hi << 4));
  }
}

/* ------------------------------------------------------------------ */
/* Alg. 1 / Eq. (15)-(16): gamma_i = gamma_{i-1} + beta * sign(T),      */
/* T = R(G_out, gamma_{i-1}) - alpha / (2^b - 1),  R = N(G_out)/N(G).   */
/* The sign is taken on (2^b-1) * N(G_out) vs alpha * N(G) in double    */
/* (same sign as T, no division).  Returns the sign used.               */
/* ------------------------------------------------------------------ */
int orc_update_interval(double* gamma, double alpha, double beta, double gamma_min,
                        double gamma_max, int bits, uint64_t n_out, uint64_t n_total) {
  double lhs = (double)n_out * (double)((1 << bits) - 1);
  double rhs = alpha * (double)n_total;
  int sg = (lhs > rhs) - (lhs < rhs);
  double g = *gamma + beta * (double)sg;
  if (g < gamma_min) g = gamma_min;
  if (g > gamma_max) g = gamma_max;
  *gamma = g;
  return sg;
}

/* ------------------------------------------------------------------ */
/* Linear layer, row-major X[M,K], W[K,N], dY[M,N]:                     */
/*   acc_dX[m,k] = sum_n qG[m,n] * qW[k,n]      (dX = Q(dY) . Q(W)^T)   */
/*   acc_dW[k,n] = sum_m qX[m,k] * qG[m,n]      (dW = Q(X)^T . Q(dY))   */
/* ------------------------------------------------------------------ */
void orc_linear_dx(const int32_t* qG, const int32_t* qW, int64_t M, int64_t K, int64_t N,
                   int64_t* acc) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t k = 0; k < K; ++k) {
      int64_t s = 0;
      for (int64_t n = 0; n < N; ++n) s += (int64_t)qG[m * N + n] * (int64_t)qW[k * N + n];
      acc[m * K + k] = s;
    }
}

void orc_linear_dw(const int32_t* qX, const int32_t* qG, int64_t M, int64_t K, int64_t N,
                   int64_t* acc) {
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < K; ++k)
    for (int64_t n = 0; n < N; ++n) {
      int64_t s = 0;
      for (int64_t m = 0; m < M; ++m) s += (int64_t)qX[m * K + k] * (int64_t)qG[m * N + n];
      acc[k * N + n] = s;
    }
}

/* ------------------------------------------------------------------ */
/* 2-D convolution (cross-correlation, no dilation, no groups), NCHW:   */
/*   Y[n,k,p,q] = sum_{c,r,s} X[n,c,p*st-pad+r,q*st-pad+s] W[k,c,r,s]   */
/* Its two gradients, on integer codes:                                 */
/*   acc_dX[n,c,h,w] = sum over (k,r,s,p,q) with h = p*st-pad+r,        */
/*                     w = q*st-pad+s of qG[n,k,p,q] * qW[k,c,r,s]      */
/*   acc_dW[k,c,r,s] = sum_{n,p,q} qG[n,k,p,q] * qX[n,c,h,w], zero      */
/*                     outside the image                                */
/* P = (H + 2*pad - R)/st + 1, Q likewise.                              */
/* ------------------------------------------------------------------ */
void orc_conv2d_dx(const int32_t* qG, const int32_t* qW, int64_t N, int64_t C, int64_t H,
                   int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t st, int64_t pad,
                   int64_t* acc) {
  const int64_t P = (H + 2 * pad - R) / st + 1, Q = (Wd + 2 * pad - S) / st + 1;
  memset(acc, 0, sizeof(int64_t) * (size_t)(N * C * H * Wd));
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t c = 0; c < C; ++c)
      for (int64_t k = 0; k < K; ++k)
        for (int64_t r = 0; r < R; ++r)
          for (int64_t s = 0; s < S; ++s)
            for (int64_t p = 0; p < P; ++p)
              for (int64_t q = 0; q < Q; ++q) {
                int64_t h = p * st - pad + r, w = q * st - pad + s;
                if (h < 0 || h >= H || w < 0 || w >= Wd) continue;
                acc[((n * C + c) * H + h) * Wd + w] +=
                    (int64_t)qG[((n * K + k) * P + p) * Q + q] *
                    (int64_t)qW[((k * C + c) * R + r) * S + s];
              }
}

void orc_conv2d_dw(const int32_t* qG, const int32_t* qX, int64_t N, int64_t C, int64_t H,
                   int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t st, int64_t pad,
                   int64_t* acc) {
  const int64_t P = (H + 2 * pad - R) / st + 1, Q = (Wd + 2 * pad - S) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t k = 0; k < K; ++k)
    for (int64_t c = 0; c < C; ++c)
      for (int64_t r = 0; r < R; ++r)
        for (int64_t s = 0; s < S; ++s) {
          int64_t sum = 0;
          for (int64_t n = 0; n < N; ++n)
            for (int64_t p = 0; p < P; ++p)
              for (int64_t q = 0; q < Q; ++q) {
                int64_t h = p * st - pad + r, w = q * st - pad + s;
                if (h < 0 || h >= H || w < 0 || w >= Wd) continue;
                sum += (int64_t)qG[((n * K + k) * P + p) * Q + q] *
                       (int64_t)qX[((n * C + c) * H + h) * Wd + w];
              }
          acc[((k * C + c) * R + r) * S + s] = sum;
        }
}

/* The same two sums evaluated at chosen output positions only (flat indices
 * into dX / dW), so that full-size layers can be spot-checked.  dX is written
 * here as a gather over the taps that reach (h,w); tests check it against the
 * scatter form above. */
void orc_conv2d_dx_at(const int32_t* qG, const int32_t* qW, int64_t N, int64_t C, int64_t H,
                      int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t st, int64_t pad,
                      const int64_t* idx, int64_t n_idx, int64_t* acc) {
  const int64_t P = (H + 2 * pad - R) / st + 1, Q = (Wd + 2 * pad - S) / st + 1;
  (void)N;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t i = 0; i < n_idx; ++i) {
    int64_t f = idx[i];
    int64_t w = f % Wd, h = (f / Wd) % H, c = (f / (Wd * H)) % C, n = f / (Wd * H * C);
    int64_t sum = 0;
    for (int64_t k = 0; k < K; ++k)
      for (int64_t r = 0; r < R; ++r)
        for (int64_t s = 0; s < S; ++s) {
          int64_t hp = h + pad - r, wq = w + pad - s;
          if (hp < 0 || wq < 0 || hp % st != 0 || wq % st != 0) continue;
          int64_t p = hp / st, q = wq / st;
          if (p >= P || q >= Q) continue;
          sum += (int64_t)qG[((n * K + k) * P + p) * Q + q] *
                 (int64_t)qW[((k * C + c) * R + r) * S + s];
        }
    acc[i] = sum;
  }
}

void orc_conv2d_dw_at(const int32_t* qG, const int32_t* qX, int64_t N, int64_t C, int64_t H,
                      int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t st, int64_t pad,
                      const int64_t* idx, int64_t n_idx, int64_t* acc) {
  const int64_t P = (H + 2 * pad - R) / st + 1, Q = (Wd + 2 * pad - S) / st + 1;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t i = 0; i < n_idx; ++i) {
    int64_t f = idx[i];
    int64_t s = f % S, r = (f / S) % R, c = (f / (S * R)) % C, k = f / (S * R * C);
    int64_t sum = 0;
    for (int64_t n = 0; n < N; ++n)
      for (int64_t p = 0; p < P; ++p)
        for (int64_t q = 0; q < Q; ++q) {
          int64_t h = p * st - pad + r, w = q * st - pad + s;
          if (h < 0 || h >= H || w < 0 || w >= Wd) continue;
          sum += (int64_t)qG[((n * K + k) * P + p) * Q + q] *
                 (int64_t)qX[((n * C + c) * H + h) * Wd + w];
        }
    acc[i] = sum;
  }
}

/* Denormalisation, Eq. (4) applied to a product of two quantized values:
 * out = acc * (s_a * s_b), evaluated in double, stored as fp32. */
void orc_dequant(const int64_t* acc, int64_t n, double s_a, double s_b, float* out) {
  const double ss = s_a * s_b;
  for (int64_t i = 0; i < n; ++i) out[i] = (float)((double)acc[i] * ss);
}
