// Quantizer kernels: tensor maximum, uniform b=4 quantizer (Eq. 1-4 of the paper)
// with nearest or stochastic rounding, clip-out count (Sec. 3.3, Alg. 1 step 5),
// nibble packing in the flat format of the C ABI and in the two GEMM layouts,
// and the one-thread clipping-factor update (Eq. 15-16).
//
// Arithmetic contract (decides integer codes, so it is fixed to the last bit):
//   c      = (float)(gamma * (double)g_max)
//   inv_s  = (double)q / (double)c,  q = 7 (signed) or 15 (unsigned)
//   t      = (double)clip(x) * inv_s          -- one double multiply, no FMA
//   code   = rint(t)  |  floor(t + r16 / 65536)
//   code   = clamp(code, -q or 0, q)
#include "lbt_internal.h"

namespace lbt {
namespace {

constexpr int kThreads = 256;
constexpr uint32_t kInfBits = 0x7f800000u;

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11): counter-based generator, 10 rounds.
// ---------------------------------------------------------------------------
struct Philox4 {
  uint32_t w[4];
};

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2,
                                                 uint32_t c3, uint32_t k0, uint32_t k1) {
  constexpr uint32_t kMulA = 0xD2511F53u, kMulB = 0xCD9E8D57u;
  constexpr uint32_t kWeylA = 0x9E3779B9u, kWeylB = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t a_hi = __umulhi(kMulA, c0), a_lo = kMulA * c0;
    const uint32_t b_hi = __umulhi(kMulB, c2), b_lo = kMulB * c2;
    c0 = b_hi ^ c1 ^ k0;
    c1 = b_lo;
    c2 = a_hi ^ c3 ^ k1;
    c3 = a_lo;
    k0 += kWeylA;
    k1 += kWeylB;
  }
  return Philox4{{c0, c1, c2, c3}};
}

// 16 random bits for flat element e: lane e%8 of block e/8.
__device__ __forceinline__ uint32_t r16_of(const Philox4& p, uint32_t lane) {
  return (p.w[lane >> 1] >> ((lane & 1u) * 16u)) & 0xFFFFu;
}

// ---------------------------------------------------------------------------
// Per-call quantizer constants, uniform across the grid.
// ---------------------------------------------------------------------------
struct QConst {
  float c;       // clip value; <= 0 means "all codes zero"
  float lo;      // lower clip bound: -c or 0
  double inv_s;  // q / c
  int q;         // largest code
  int kmin;      // smallest code
};

__device__ __forceinline__ QConst make_qconst(float c, bool is_unsigned) {
  QConst k;
  k.c = c;
  k.q = is_unsigned ? 15 : 7;
  k.kmin = is_unsigned ? 0 : -7;
  k.lo = is_unsigned ? 0.0f : -c;
  k.inv_s = (c > 0.0f) ? (double)k.q / (double)c : 0.0;
  return k;
}

__device__ __forceinline__ double normalised(float v, const QConst& k) {
  const float xc = fminf(fmaxf(v, k.lo), k.c);
  return __dmul_rn((double)xc, k.inv_s);
}

__device__ __forceinline__ int code_nearest(float v, const QConst& k) {
  const int r = (int)rint(normalised(v, k));
  return min(max(r, k.kmin), k.q);
}

__device__ __forceinline__ int code_stochastic(float v, const QConst& k, uint32_t r16) {
  const double u = (double)r16 * (1.0 / 65536.0);
  const int r = (int)floor(__dadd_rn(normalised(v, k), u));
  return min(max(r, k.kmin), k.q);
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__device__ __forceinline__ uint32_t wave_max(uint32_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = max(v, __shfl_xor(v, off, 64));
  return v;
}

// Block-wide sum of per-thread counts, then ONE atomic per block.
__device__ __forceinline__ void block_count_add(uint32_t cnt, unsigned long long* target) {
  __shared__ uint32_t part[kThreads / 64];
  cnt = wave_sum(cnt);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = cnt;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t tot = 0;
#pragma unroll
    for (int i = 0; i < kThreads / 64; ++i) tot += part[i];
    if (tot) atomicAdd(target, (unsigned long long)tot);
  }
}

// ---------------------------------------------------------------------------
// small one-thread kernels
// ---------------------------------------------------------------------------
__global__ void k_begin(lbt_grad_state* st, OperandScalars* sc) {
  if (st) {
    st->gmax = 0.0f;
    st->n_out = 0;
    st->status = LBT_STATUS_OK;
  }
  if (sc) {
    sc->xmax_bits = 0;
    sc->wmax_bits = 0;
    sc->c_x = 0.0f;
    sc->c_w = 0.0f;
    sc->nonfinite = 0;
  }
}

__global__ void k_grad_prepare(lbt_grad_state* st, unsigned long long n) {
  const uint32_t bits = __float_as_uint(st->gmax);
  st->n_total = n;
  st->n_out = 0;
  if (bits >= kInfBits) {
    st->status = LBT_STATUS_NONFINITE;
    st->clip = 0.0f;
    st->scale = 0.0f;
  } else if (bits == 0) {
    st->status = LBT_STATUS_ZERO_GRAD;
    st->clip = 0.0f;
    st->scale = 0.0f;
  } else {
    st->status = LBT_STATUS_OK;
    const float c = (float)__dmul_rn(st->gamma, (double)st->gmax);
    st->clip = c;
    st->scale = (c > 0.0f) ? (float)((double)c / 7.0) : 0.0f;
  }
}

__global__ void k_operand_prepare(OperandScalars* sc, lbt_grad_state* st, float c_x, float c_w) {
  uint32_t bad = 0;
  float cx = c_x, cw = c_w;
  if (!(cx > 0.0f)) {
    if (sc->xmax_bits >= kInfBits) { bad = 1; cx = 0.0f; }
    else cx = __uint_as_float(sc->xmax_bits);
  }
  if (!(cw > 0.0f)) {
    if (sc->wmax_bits >= kInfBits) { bad = 1; cw = 0.0f; }
    else cw = __uint_as_float(sc->wmax_bits);
  }
  sc->c_x = cx;
  sc->c_w = cw;
  sc->nonfinite = bad;
  if (bad && st) st->status = LBT_STATUS_NONFINITE;
}

__global__ void k_update_interval(lbt_grad_state* st) {
  if (st->status != LBT_STATUS_OK) return;
  const double lhs = (double)st->n_out * (double)((1 << st->bits) - 1);
  const double rhs = __dmul_rn(st->alpha, (double)st->n_total);
  const int sg = (lhs > rhs) - (lhs < rhs);
  double g = __dadd_rn(st->gamma, __dmul_rn(st->beta, (double)sg));
  g = fmax(g, st->gamma_min);
  g = fmin(g, st->gamma_max);
  st->gamma = g;
  st->step += 1;
}

__global__ void k_state_set(lbt_grad_state* st, lbt_grad_state v) { *st = v; }

// ---------------------------------------------------------------------------
// tensor maximum: max |x| (use_abs) or max(x, 0) as an unsigned compare of the
// fp32 bit patterns (monotone for non-negative floats; NaN/Inf sort on top).
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t max_key(float v, int use_abs) {
  const uint32_t b = __float_as_uint(v);
  const uint32_t mag = b & 0x7fffffffu;
  if (use_abs) return mag;
  // signed maximum clipped at 0: negatives contribute 0, but keep NaN/Inf visible
  if (mag >= kInfBits) return mag;
  return (b >> 31) ? 0u : b;
}

__global__ __launch_bounds__(kThreads) void k_absmax(const float* __restrict__ x, long long n,
                                                      int use_abs, uint32_t* max_bits) {
  const long long n4 = n / 4;
  const float4* x4 = reinterpret_cast<const float4*>(x);
  uint32_t m = 0;
  const long long stride = (long long)gridDim.x * kThreads;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < n4; i += stride) {
    const float4 v = x4[i];
    m = max(m, max(max(max_key(v.x, use_abs), max_key(v.y, use_abs)),
                   max(max_key(v.z, use_abs), max_key(v.w, use_abs))));
  }
  if (blockIdx.x == 0 && threadIdx.x < (n - n4 * 4)) m = max(m, max_key(x[n4 * 4 + threadIdx.x], use_abs));
  m = wave_max(m);
  __shared__ uint32_t part[kThreads / 64];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t t = part[0];
#pragma unroll
    for (int i = 1; i < kThreads / 64; ++i) t = max(t, part[i]);
    if (t) atomicMax(max_bits, t);
  }
}

// ---------------------------------------------------------------------------
// flat quantizer: 8 consecutive elements per thread -> one 32-bit word of codes
// MODE 0: signed nearest, 1: unsigned nearest, 2: signed nearest + count,
//      3: signed stochastic + count
// ---------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(kThreads) void k_quantize_flat(
    const float* __restrict__ x, long long n, const float* clip_ptr, lbt_grad_state* st,
    unsigned long long seed, uint8_t* __restrict__ codes, float* clip_scale_out) {
  constexpr bool kUnsigned = (MODE == 1);
  constexpr bool kCount = (MODE >= 2);
  constexpr bool kStoch = (MODE == 3);
  const float c = kCount ? st->clip : *clip_ptr;
  const QConst qc = make_qconst(c, kUnsigned);
  const bool live = c > 0.0f;
  const unsigned long long step = kStoch ? st->step : 0ull;
  if (!kCount && clip_scale_out && blockIdx.x == 0 && threadIdx.x == 0) {
    clip_scale_out[0] = c;
    clip_scale_out[1] = live ? (float)((double)c / (double)qc.q) : 0.0f;
  }
  const long long groups = (n + 7) / 8;
  const long long stride = (long long)gridDim.x * kThreads;
  uint32_t cnt = 0;
  for (long long gi = (long long)blockIdx.x * kThreads + threadIdx.x; gi < groups; gi += stride) {
    const long long e0 = gi * 8;
    const int valid = (int)min(8ll, n - e0);
    float v[8];
    if (valid == 8) {
      const float4 a = reinterpret_cast<const float4*>(x)[2 * gi];
      const float4 b = reinterpret_cast<const float4*>(x)[2 * gi + 1];
      v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
      v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = (j < valid) ? x[e0 + j] : 0.0f;
    }
    uint32_t word = 0;
    if (live) {
      Philox4 rnd;
      if (kStoch)
        rnd = philox4x32_10((uint32_t)gi, (uint32_t)((unsigned long long)gi >> 32), (uint32_t)step,
                            (uint32_t)(step >> 32), (uint32_t)seed, (uint32_t)(seed >> 32));
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        int k;
        if (kStoch) k = code_stochastic(v[j], qc, r16_of(rnd, j));
        else k = code_nearest(v[j], qc);
        if (j >= valid) k = 0;
        word |= ((uint32_t)k & 0xFu) << (4 * j);
        if (kCount) cnt += (fabsf(v[j]) > c) ? 1u : 0u;
      }
    }
    if (valid == 8) {
      reinterpret_cast<uint32_t*>(codes)[gi] = word;
    } else {
      const int nbytes = (valid + 1) / 2;
      for (int j = 0; j < nbytes; ++j) codes[gi * 4 + j] = (uint8_t)(word >> (8 * j));
    }
  }
  if (kCount) block_count_add(cnt, reinterpret_cast<unsigned long long*>(&st->n_out));
}

// ---------------------------------------------------------------------------
// quantize + re-layout: T[A][B][L] -> out_b [A][L][Bp] and/or out_a [B][L][Ap],
// nibbles packed along the innermost axis, zero padded to Bp / Ap.
// A workgroup quantizes a TA x TB x TL tile into LDS (one byte per code), then
// gathers eight codes along B (or A) into each 32-bit output word.
// ---------------------------------------------------------------------------
template <int TA, int TB, int TL, int MODE>
__global__ __launch_bounds__(kThreads) void k_quantize_relayout(
    const float* __restrict__ x, int A, int B, int L, int Ap, int Bp, const float* clip_ptr,
    lbt_grad_state* st, unsigned long long seed, uint32_t* __restrict__ out_b,
    uint32_t* __restrict__ out_a) {
  constexpr bool kUnsigned = (MODE == 1);
  constexpr bool kCount = (MODE >= 2);
  constexpr bool kStoch = (MODE == 3);
  constexpr int TLP = TL + 1;  // odd byte pitch spreads the strided gathers over banks
  __shared__ uint8_t tile[TA * TB * TLP];

  const float c = kCount ? st->clip : *clip_ptr;
  const QConst qc = make_qconst(c, kUnsigned);
  const bool live = c > 0.0f;
  const unsigned long long step = kStoch ? st->step : 0ull;
  const int l0 = blockIdx.x * TL, b0 = blockIdx.y * TB, a0 = blockIdx.z * TA;

  uint32_t cnt = 0;
  for (int idx = threadIdx.x; idx < TA * TB * TL; idx += kThreads) {
    const int l = idx % TL, b = (idx / TL) % TB, a = idx / (TL * TB);
    const int ga = a0 + a, gb = b0 + b, gl = l0 + l;
    int k = 0;
    if (ga < A && gb < B && gl < L) {
      const long long e = ((long long)ga * B + gb) * L + gl;
      const float v = x[e];
      if (live) {
        if (kStoch) {
          const unsigned long long blk = (unsigned long long)e >> 3;
          const Philox4 rnd = philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), (uint32_t)step,
                                            (uint32_t)(step >> 32), (uint32_t)seed,
                                            (uint32_t)(seed >> 32));
          k = code_stochastic(v, qc, r16_of(rnd, (uint32_t)e & 7u));
        } else {
          k = code_nearest(v, qc);
        }
        if (kCount) cnt += (fabsf(v) > c) ? 1u : 0u;
      }
    }
    tile[(a * TB + b) * TLP + l] = (uint8_t)(k & 0xF);
  }
  __syncthreads();

  if (out_b) {
    constexpr int GB = TB / 8;
    for (int idx = threadIdx.x; idx < TA * TL * GB; idx += kThreads) {
      const int bg = idx % GB, l = (idx / GB) % TL, a = idx / (GB * TL);
      const int ga = a0 + a, gl = l0 + l, gb = b0 + 8 * bg;
      if (ga < A && gl < L && gb < Bp) {
        uint32_t word = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) word |= (uint32_t)tile[(a * TB + 8 * bg + j) * TLP + l] << (4 * j);
        out_b[(((long long)ga * L + gl) * Bp + gb) >> 3] = word;
      }
    }
  }
  if (out_a) {
    constexpr int GA = TA / 8;
    for (int idx = threadIdx.x; idx < TB * TL * GA; idx += kThreads) {
      const int ag = idx % GA, l = (idx / GA) % TL, b = idx / (GA * TL);
      const int gb = b0 + b, gl = l0 + l, ga = a0 + 8 * ag;
      if (gb < B && gl < L && ga < Ap) {
        uint32_t word = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) word |= (uint32_t)tile[((8 * ag + j) * TB + b) * TLP + l] << (4 * j);
        out_a[(((long long)gb * L + gl) * Ap + ga) >> 3] = word;
      }
    }
  }
  if (kCount) block_count_add(cnt, reinterpret_cast<unsigned long long*>(&st->n_out));
}

inline int flat_grid(long long work_items) {
  long long blocks = (work_items + kThreads - 1) / kThreads;
  const long long cap = 256 * 16;  // 256 compute units, several workgroups each
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return (int)blocks;
}

template <int MODE>
int relayout_dispatch(const float* x, int64_t A, int64_t B, int64_t L, const float* clip_ptr,
                      lbt_grad_state* st, uint64_t seed, uint8_t* out_b, uint8_t* out_a,
                      hipStream_t s) {
  const int Ap = (int)round_up(A, kGranule), Bp = (int)round_up(B, kGranule);
  auto ob = reinterpret_cast<uint32_t*>(out_b);
  auto oa = reinterpret_cast<uint32_t*>(out_a);
#define LBT_RELAYOUT(TA, TB, TL)                                                              \
  do {                                                                                        \
    dim3 grid((unsigned)((L + TL - 1) / TL), (unsigned)((Bp + TB - 1) / TB),                  \
              (unsigned)((Ap + TA - 1) / TA));                                                \
    if (grid.y > 65535u || grid.z > 65535u) return LBT_ERR_UNSUPPORTED;                       \
    hipLaunchKernelGGL((k_quantize_relayout<TA, TB, TL, MODE>), grid, dim3(kThreads), 0, s, x, \
                       (int)A, (int)B, (int)L, Ap, Bp, clip_ptr, st, seed, ob, oa);           \
  } while (0)
  if (L == 1) {
    LBT_RELAYOUT(64, 64, 1);
  } else if (!out_b) {
    LBT_RELAYOUT(64, 16, 32);
  } else {
    LBT_RELAYOUT(32, 32, 32);
  }
#undef LBT_RELAYOUT
  LBT_LAUNCH_CHECK();
  return LBT_OK;
}

}  // namespace

int launch_begin(lbt_grad_state* st, OperandScalars* sc, hipStream_t s) {
  ProfScope prof(KID_BEGIN, 0.0, s);
  hipLaunchKernelGGL(k_begin, dim3(1), dim3(1), 0, s, st, sc);
  LBT_LAUNCH_CHECK();
  return LBT_OK;
}

int launch_absmax(const float* x, int64_t n, int use_abs, uint32_t* max_bits, hipStream_t s) {
  ProfScope prof(KID_ABSMAX, (double)n, s);
  hipLaunchKernelGGL(k_absmax, dim3(flat_grid((n / 4 + 3) / 4)), dim3(kThreads), 0, s, x,
                     (long long)n, use_abs, max_bits);
  LBT_LAUNCH_CHECK();
  return LBT_OK;
}

int launch_grad_prepare(lbt_grad_state* st, int64_t n, hipStream_t s) {
  ProfScope prof(KID_GRAD_PREPARE, 0.0, s);
  hipLaunchKernelGGL(k_grad_prepare, dim3(1), dim3(1), 0, s, st, (unsigned long long)n);
  LBT_LAUNCH_CHECK();
  return LBT_OK;
}

int launch_operand_prepare(OperandScalars* sc, lbt_grad_state* st, float c_x, float c_w,
                           hipStream_t s) {
  ProfScope prof(KID_OPERAND_PREPARE, 0.0, s);
  hipLaunchKernelGGL(k_operand_prepare, dim3(1), dim3(1), 0, s, sc, st, c_x, c_w);
  LBT_LAUNCH_CHECK();
  return LBT_OK;
}

int launch_quantize_flat_grad(const float* g, int64_t n, lbt_grad_state* st, uint64_t seed,
                              int rounding, uint8_t* codes, hipStream_t s) {
  ProfScope prof(KID_FLAT_GRAD, (double)n, s);
  const int grid = flat_grid((n + 7) / 8);
  if (rounding == LBT_ROUND_STOCHASTIC)
    hipLaunchKernelGGL(k_quantize_flat<3>, dim3(grid), dim3(kThreads), 0, s, g, (long long)n,
                       (const float*)nullptr, st, (unsigned long long)seed, codes, (float*)nullptr);
  else
    hipLaunchKernelGGL(k_quantize_flat<2>, dim3(grid), dim3(kThreads), 0, s, g, (long long)n,
                       (const float*)nullptr, st, (unsigned long long)seed, codes, (float*)nullptr);
  LBT_LAUNCH_CHECK();
  return LBT_OK;
}

int launch_quantize_flat_operand(const float* x, int64_t n, const float* clip_ptr, int is_unsigned,
                                 uint8_t* codes, float* clip_scale_out, hipStream_t s) {
  ProfScope prof(KID_FLAT_OPERAND, (double)n, s);
  const int grid = flat_grid((n + 7) / 8);
  if (is_unsigned)
    hipLaunchKernelGGL(k_quantize_flat<1>, dim3(grid), dim3(kThreads), 0, s, x, (long long)n,
                       clip_ptr, (lbt_grad_state*)nullptr, 0ull, codes, clip_scale_out);
  else
    hipLaunchKernelGGL(k_quantize_flat<0>, dim3(grid), dim3(kThreads), 0, s, x, (long long)n,
                       clip_ptr, (lbt_grad_state*)nullptr, 0ull, codes, clip_scale_out);
  LBT_LAUNCH_CHECK();
  return LBT_OK;
}

int launch_quantize_relayout_grad(const float* g, int64_t A, int64_t B, int64_t L,
                                  lbt_grad_state* st, uint64_t seed, int rounding, uint8_t* out_b,
                                  uint8_t* out_a, hipStream_t s) {
  ProfScope prof(KID_RELAYOUT_GRAD, (double)A * (double)B * (double)L, s);
  if (rounding == LBT_ROUND_STOCHASTIC)
    return relayout_dispatch<3>(g, A, B, L, nullptr, st, seed, out_b, out_a, s);
  return relayout_dispatch<2>(g, A, B, L, nullptr, st, seed, out_b, out_a, s);
}

int launch_quantize_relayout_operand(const float* x, int64_t A, int64_t B, int64_t L,
                                     const float* clip_ptr, int is_unsigned, uint8_t* out_b,
                                     uint8_t* out_a, hipStream_t s) {
  ProfScope prof(KID_RELAYOUT_OPERAND, (double)A * (double)B * (double)L, s);
  if (is_unsigned) return relayout_dispatch<1>(x, A, B, L, clip_ptr, nullptr, 0, out_b, out_a, s);
  return relayout_dispatch<0>(x, A, B, L, clip_ptr, nullptr, 0, out_b, out_a, s);
}

int launch_update_interval(lbt_grad_state* st, hipStream_t s) {
  ProfScope prof(KID_UPDATE, 0.0, s);
  hipLaunchKernelGGL(k_update_interval, dim3(1), dim3(1), 0, s, st);
  LBT_LAUNCH_CHECK();
  return LBT_OK;
}

int launch_state_init(lbt_grad_state* st, const lbt_grad_state& v, hipStream_t s) {
  ProfScope prof(KID_STATE, 0.0, s);
  hipLaunchKernelGGL(k_state_set, dim3(1), dim3(1), 0, s, st, v);
  LBT_LAUNCH_CHECK();
  return LBT_OK;
}

}  // namespace lbt
