// Integer contractions of the backward pass on int8 matrix cores (gfx950).
//
// Both gradients of a convolution (and of a linear layer, which is the 1x1 case
// on a 1x1 image) are computed by one implicit-GEMM kernel
//     D[m][j] = sum_k A[m][k] * B[j][k]
// whose operands are 4-bit codes packed two per byte along the contraction axis:
//   dX: A = weights  [C][R*S][Kp]  (dense rows),  B row j = output pixel (n,h,w),
//       gathered from the gradient codes [N][P*Q][Kp] tap by tap;
//   dW: A = gradient [K][P*Q][Np]  (dense rows),  B row j = (c,r,s), gathered
//       from the activation codes [C][H*W][Np] with the tap's shift.
// The contraction axis is cut into chunks of 16 codes (8 bytes); a chunk is
// either wholly inside the image or wholly padding, so the gather works on
// whole chunks.  Codes are widened to int8 in registers: a signed nibble is
// moved to the top of its byte (value * 16, exact two's complement), an unsigned
// nibble is masked in place; the accumulators therefore carry a factor 256 or 16
// that the epilogue shifts out exactly.  Accumulation is int32 and exact.
#include "lbt_internal.h"

namespace lbt {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int BM = 128, BN = 128;   // workgroup tile
constexpr int BKC = 8;              // chunks (of 16 codes) per K step: 128 codes = 64 bytes per row
constexpr int PITCH = BKC * 8 + 8;  // LDS row pitch in bytes (72: conflict-free 8-byte reads)
constexpr int WM = 64, WN = 64;     // wave tile (2 x 2 waves)

struct GemmArgs {
  const uint8_t* A;
  const uint8_t* B;
  long long lda;      // bytes per A row
  int M, NJ;          // rows of A, rows of B
  int chunks;         // total K chunks
  int chunks_per_split;
  int mode;           // gather of B rows: 0 = conv dX (pixel rows), 1 = conv dW ((c,r,s) rows)
  int epi;            // 0 = scaled store to NCHW dX, 1 = int32 atomic add row-major,
                      // 2 = scaled store row-major
  int N, C, H, W, K, R, S, P, Q, stride, pad;
  int inner_chunks;   // chunks per tap (dX: Kp/16) or per output position (dW: Np/16)
  int shift;          // log2 of the factor carried by the accumulators
  const lbt_grad_state* st;
  const OperandScalars* sc;
  int x_unsigned;
  float* out;         // dX: fp32 result; dW: int32 accumulation buffer (same storage as the result)
  int32_t* acc;       // optional raw accumulators (dX only; dW takes them in the finalize pass)
};

// Signed nibbles -> int8 values 16*code (nibble placed in the high half of each byte).
__device__ __forceinline__ void widen_signed(uint32_t p, int& even, int& odd) {
  odd = (int)(p & 0xF0F0F0F0u);
  even = (int)((p << 4) & 0xF0F0F0F0u);
}
// Unsigned nibbles -> int8 values code.
__device__ __forceinline__ void widen_unsigned(uint32_t p, int& even, int& odd) {
  even = (int)(p & 0x0F0F0F0Fu);
  odd = (int)((p >> 4) & 0x0F0F0F0Fu);
}

template <bool UNS>
__device__ __forceinline__ v4i widen(uint2 p) {
  v4i r;
  int a, b, c, d;
  if (UNS) { widen_unsigned(p.x, a, b); widen_unsigned(p.y, c, d); }
  else { widen_signed(p.x, a, b); widen_signed(p.y, c, d); }
  r[0] = a; r[1] = b; r[2] = c; r[3] = d;
  return r;
}

// Location of chunk t of B row j, or -1 when the chunk lies in the padding.
struct RowInfo {
  int i0, i1, i2;  // dX: n, h, w     dW: c, r, s
  bool valid;
};

__device__ __forceinline__ RowInfo decode_row(const GemmArgs& g, int j) {
  RowInfo r;
  r.valid = j < g.NJ;
  if (g.mode == 0) {
    r.i2 = j % g.W;
    r.i1 = (j / g.W) % g.H;
    r.i0 = j / (g.W * g.H);
  } else {
    r.i2 = j % g.S;
    r.i1 = (j / g.S) % g.R;
    r.i0 = j / (g.S * g.R);
  }
  return r;
}

__device__ __forceinline__ long long chunk_offset(const GemmArgs& g, const RowInfo& r, int t) {
  if (!r.valid || t >= g.chunks) return -1;
  const int outer = t / g.inner_chunks, inner = t - outer * g.inner_chunks;
  if (g.mode == 0) {
    // outer = tap (r,s); the pixel (h,w) receives from p = (h + pad - r)/stride when integral
    const int fr = outer / g.S, fs = outer - fr * g.S;
    const int hp = r.i1 + g.pad - fr, wq = r.i2 + g.pad - fs;
    if (hp < 0 || wq < 0) return -1;
    const int p = hp / g.stride, q = wq / g.stride;
    if (p * g.stride != hp || q * g.stride != wq || p >= g.P || q >= g.Q) return -1;
    return ((((long long)r.i0 * g.P + p) * g.Q + q) * g.inner_chunks + inner) * 8;
  } else {
    // outer = output position (p,q); row (c,r,s) reads x at h = p*stride - pad + r
    const int p = outer / g.Q, q = outer - p * g.Q;
    const int h = p * g.stride - g.pad + r.i1, w = q * g.stride - g.pad + r.i2;
    if (h < 0 || h >= g.H || w < 0 || w >= g.W) return -1;
    return ((((long long)r.i0 * g.H + h) * g.W + w) * g.inner_chunks + inner) * 8;
  }
}

template <bool A_UNSIGNED, bool B_UNSIGNED>
__global__ __launch_bounds__(kThreads) void k_implicit_gemm(const GemmArgs g) {
  __shared__ __attribute__((aligned(16))) uint8_t sA[BM * PITCH];
  __shared__ __attribute__((aligned(16))) uint8_t sB[BN * PITCH];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * WM, wn = (wave & 1) * WN;
  const int m0 = blockIdx.y * BM, j0 = blockIdx.x * BN;
  const int t_begin = blockIdx.z * g.chunks_per_split;
  const int t_end = min(t_begin + g.chunks_per_split, g.chunks);

  // each thread stages 4 chunks of A and 4 of B per K step: chunk id = tid + 256*i
  // -> row = id / BKC, chunk-in-step = id % BKC
  RowInfo brow[4];
  int arow[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int id = tid + kThreads * i;
    arow[i] = m0 + id / BKC;
    brow[i] = decode_row(g, j0 + id / BKC);
  }
  const int cpos = tid % BKC;  // kThreads is a multiple of BKC: same chunk column for all i

  v4i acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = v4i{0, 0, 0, 0};

  for (int t0 = t_begin; t0 < t_end; t0 += BKC) {
    uint2 ra[4], rb[4];
    const int t = t0 + cpos;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ra[i] = make_uint2(0, 0);
      rb[i] = make_uint2(0, 0);
      if (arow[i] < g.M && t < t_end)
        ra[i] = *reinterpret_cast<const uint2*>(g.A + (long long)arow[i] * g.lda + (long long)t * 8);
      const long long off = (t < t_end) ? chunk_offset(g, brow[i], t) : -1;
      if (off >= 0) rb[i] = *reinterpret_cast<const uint2*>(g.B + off);
    }
    __syncthreads();  // previous step's fragments have been read
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + kThreads * i;
      *reinterpret_cast<uint2*>(sA + (id / BKC) * PITCH + cpos * 8) = ra[i];
      *reinterpret_cast<uint2*>(sB + (id / BKC) * PITCH + cpos * 8) = rb[i];
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BKC / 4; ++kk) {
      // one 16x16x64 step: lane holds row (lane % 16), K group (lane / 16) = chunk kk*4 + lane/16
      const int coff = (kk * 4 + (lane >> 4)) * 8;
      v4i fa[4], fb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint2 pa = *reinterpret_cast<const uint2*>(sA + (wm + i * 16 + (lane & 15)) * PITCH + coff);
        const uint2 pb = *reinterpret_cast<const uint2*>(sB + (wn + i * 16 + (lane & 15)) * PITCH + coff);
        fa[i] = widen<A_UNSIGNED>(pa);
        fb[i] = widen<B_UNSIGNED>(pb);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  }

  // epilogue.  Accumulator layout of the 16x16 tile: lane holds column (lane % 16),
  // rows 4*(lane/16) .. +3.
  const int shift = g.shift;
  const double s_g = (double)g.st->clip / 7.0;
  const double s_w = (double)g.sc->c_w / 7.0;
  const float scale = (float)(s_g * s_w);
  if (g.epi == 0) {
    const int HW = g.H * g.W;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = j0 + wn + j * 16 + (lane & 15);
      if (col >= g.NJ) continue;
      const int n = col / HW, hw = col - n * HW;
      const long long base = (long long)n * g.C * HW + hw;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = m0 + wm + i * 16 + (lane >> 4) * 4 + r;
          if (row >= g.M) continue;
          const int v = acc[i][j][r] >> shift;
          const long long o = base + (long long)row * HW;
          g.out[o] = (float)v * scale;
          if (g.acc) g.acc[o] = v;
        }
    }
  } else {
    int32_t* out = reinterpret_cast<int32_t*>(g.out);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = j0 + wn + j * 16 + (lane & 15);
      if (col >= g.NJ) continue;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = m0 + wm + i * 16 + (lane >> 4) * 4 + r;
          if (row >= g.M) continue;
          const int v = acc[i][j][r] >> shift;
          const long long o = (long long)row * g.NJ + col;
          if (g.epi == 1) {
            if (v) atomicAdd(out + o, v);
          } else {
            g.out[o] = (float)v * scale;
            if (g.acc) g.acc[o] = v;
          }
        }
    }
  }
}

__global__ __launch_bounds__(kThreads) void k_zero_i32(int32_t* p, long long n) {
  const long long stride = (long long)gridDim.x * kThreads;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) p[i] = 0;
}

// dW: int32 sums -> fp32 in place, out = acc * (s_x * s_g)
__global__ __launch_bounds__(kThreads) void k_finalize_dw(float* out, int32_t* acc, long long n,
                                                           const lbt_grad_state* st,
                                                           const OperandScalars* sc, int x_unsigned) {
  const double s_g = (double)st->clip / 7.0;
  const double s_x = (double)sc->c_x / (x_unsigned ? 15.0 : 7.0);
  const float scale = (float)(s_x * s_g);
  const long long stride = (long long)gridDim.x * kThreads;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
    const int v = reinterpret_cast<const int32_t*>(out)[i];
    if (acc) acc[i] = v;
    out[i] = (float)v * scale;
  }
}

inline int small_grid(long long n) {
  long long b = (n + kThreads - 1) / kThreads;
  if (b > 2048) b = 2048;
  if (b < 1) b = 1;
  return (int)b;
}

}  // namespace

static void fill_geom(GemmArgs& g, const ConvGeom& c) {
  g.N = c.N; g.C = c.C; g.H = c.H; g.W = c.W; g.K = c.K; g.R = c.R; g.S = c.S;
  g.P = c.P; g.Q = c.Q; g.stride = c.stride; g.pad = c.pad;
}

static int run_gemm(const GemmArgs& g, bool a_uns, bool b_uns, int splits, hipStream_t s) {
  // algorithmic work: the convolution's multiply-adds, padding taps included
  const double work = 2.0 * g.N * g.P * g.Q * (double)g.K * g.C * g.R * g.S;
  ProfScope prof(g.epi == 1 ? KID_GEMM_DW : KID_GEMM_DX, work, s);
  dim3 grid((unsigned)((g.NJ + BN - 1) / BN), (unsigned)((g.M + BM - 1) / BM), (unsigned)splits);
  if (grid.y > 65535u || grid.z > 65535u) return LBT_ERR_UNSUPPORTED;
  if (a_uns && b_uns) return LBT_ERR_UNSUPPORTED;
  if (a_uns) hipLaunchKernelGGL((k_implicit_gemm<true, false>), grid, dim3(kThreads), 0, s, g);
  else if (b_uns) hipLaunchKernelGGL((k_implicit_gemm<false, true>), grid, dim3(kThreads), 0, s, g);
  else hipLaunchKernelGGL((k_implicit_gemm<false, false>), grid, dim3(kThreads), 0, s, g);
  LBT_LAUNCH_CHECK();
  return LBT_OK;
}

// Direct (no split) product with signed operands: |sum| <= chunks*16 * 112 * 112 < 2^31.
static int run_dx(GemmArgs& g, hipStream_t s) {
  g.chunks_per_split = g.chunks;
  g.shift = 8;
  g.x_unsigned = 0;
  if ((long long)g.chunks * 16 * 12544 >= (1ll << 31)) return LBT_ERR_OVERFLOW;
  return run_gemm(g, false, false, 1, s);
}

// Split-K product accumulated with int32 atomics into `out`, then scaled in place.
static int run_dw(GemmArgs& g, bool a_uns, bool b_uns, long long true_k, int32_t* acc,
                  hipStream_t s) {
  const int x_unsigned = (a_uns || b_uns) ? 1 : 0;
  g.epi = 1;
  g.shift = x_unsigned ? 4 : 8;
  g.x_unsigned = x_unsigned;
  g.acc = nullptr;
  // the exact sum must fit int32
  if (true_k * (x_unsigned ? 105 : 49) >= (1ll << 31)) return LBT_ERR_OVERFLOW;
  const int tiles = ((g.NJ + BN - 1) / BN) * ((g.M + BM - 1) / BM);
  // split K so that about 1024 workgroups exist, each split a multiple of the K step and
  // short enough that the widened partial sum (factor 256) stays inside int32
  int splits = (1024 + tiles - 1) / tiles;
  int per = (g.chunks + splits - 1) / splits;
  per = (per + BKC - 1) / BKC * BKC;
  const int max_per = 8192;  // 8192 chunks * 16 codes * 112 * 112 < 2^31
  if (per > max_per) per = max_per;
  if (per < BKC) per = BKC;
  splits = (g.chunks + per - 1) / per;
  g.chunks_per_split = per;
  const long long n_out = (long long)g.M * g.NJ;
  {
    ProfScope prof(KID_ZERO, (double)n_out, s);
    hipLaunchKernelGGL(k_zero_i32, dim3(small_grid(n_out)), dim3(kThreads), 0, s,
                       reinterpret_cast<int32_t*>(g.out), n_out);
  }
  int rc = run_gemm(g, a_uns, b_uns, splits, s);
  if (rc) return rc;
  {
    ProfScope prof(KID_FINALIZE, (double)n_out, s);
    hipLaunchKernelGGL(k_finalize_dw, dim3(small_grid(n_out)), dim3(kThreads), 0, s, g.out, acc,
                       n_out, g.st, g.sc, x_unsigned);
  }
  LBT_LAUNCH_CHECK();
  return LBT_OK;
}

int launch_conv_dx(const ConvGeom& c, const uint8_t* w_crsk, const uint8_t* g_npqk,
                   const lbt_grad_state* st, const OperandScalars* sc, float* dX, int32_t* acc,
                   hipStream_t s) {
  GemmArgs g{};
  fill_geom(g, c);
  g.A = w_crsk;
  g.B = g_npqk;
  g.inner_chunks = c.Kp / kGranule;
  g.chunks = c.R * c.S * g.inner_chunks;
  g.lda = (long long)g.chunks * 8;
  g.M = c.C;
  const long long nj = (long long)c.N * c.H * c.W;
  if (nj > 0x7fffffffll) return LBT_ERR_UNSUPPORTED;
  g.NJ = (int)nj;
  g.mode = 0;
  g.epi = 0;
  g.st = st; g.sc = sc;
  g.out = dX; g.acc = acc;
  return run_dx(g, s);
}

int launch_conv_dw(const ConvGeom& c, const uint8_t* g_kpqn, const uint8_t* x_chwn,
                   const lbt_grad_state* st, const OperandScalars* sc, int x_unsigned, float* dW,
                   int32_t* acc, hipStream_t s) {
  GemmArgs g{};
  fill_geom(g, c);
  g.A = g_kpqn;
  g.B = x_chwn;
  g.inner_chunks = c.Np / kGranule;
  const long long chunks = (long long)c.P * c.Q * g.inner_chunks;
  if (chunks > 0x7fffffffll / 16) return LBT_ERR_UNSUPPORTED;
  g.chunks = (int)chunks;
  g.lda = chunks * 8;
  g.M = c.K;
  g.NJ = c.C * c.R * c.S;
  g.mode = 1;
  g.st = st; g.sc = sc;
  g.out = dW;
  return run_dw(g, false, x_unsigned != 0, (long long)c.N * c.P * c.Q, acc, s);
}

// Linear layer (1x1 image): operands swap roles so that the row-major outputs
// dX[M][K_in] and dW[K_in][N_out] have their contiguous axis on the lanes.
int launch_linear_dx(const ConvGeom& c, const uint8_t* w_ck, const uint8_t* g_nk,
                     const lbt_grad_state* st, const OperandScalars* sc, float* dX, int32_t* acc,
                     hipStream_t s) {
  GemmArgs g{};
  fill_geom(g, c);
  g.A = g_nk;   // [N][Kp] gradient rows
  g.B = w_ck;   // [C][Kp] weight rows, read with the (c,r,s)-row gather on a 1x1 image
  g.inner_chunks = c.Kp / kGranule;
  g.chunks = g.inner_chunks;
  g.lda = (long long)g.chunks * 8;
  g.M = c.N;
  g.NJ = c.C;
  g.mode = 1;
  g.epi = 2;
  g.st = st; g.sc = sc;
  g.out = dX; g.acc = acc;
  return run_dx(g, s);
}

int launch_linear_dw(const ConvGeom& c, const uint8_t* g_kn, const uint8_t* x_cn,
                     const lbt_grad_state* st, const OperandScalars* sc, int x_unsigned, float* dW,
                     int32_t* acc, hipStream_t s) {
  GemmArgs g{};
  fill_geom(g, c);
  g.A = x_cn;   // [C][Np] activation rows
  g.B = g_kn;   // [K][Np] gradient rows
  g.inner_chunks = c.Np / kGranule;
  g.chunks = g.inner_chunks;
  g.lda = (long long)g.chunks * 8;
  g.M = c.C;
  g.NJ = c.K;
  g.mode = 1;
  g.st = st; g.sc = sc;
  g.out = dW;
  return run_dw(g, x_unsigned != 0, false, (long long)c.N, acc, s);
}

}  // namespace lbt
