// Integer contractions of the backward pass on int8 matrix cores (gfx950).
//
// Both gradients of a convolution (and of a linear layer, which is the 1x1 case
// on a 1x1 image) are computed by one implicit-GEMM kernel
//     D[m][j] = sum_k A[m][k] * B[j][k]
// whose operands are 4-bit codes packed two per byte along the contraction axis:
//   dX: A = weights  [C][Kp/16][R*S][16] (dense rows), B row j = output pixel (n,h,w),
//       gathered from the gradient codes [N][Kp/16][P*Q][16] tap by tap;
//   dW: A = gradient [K][Np/16][P*Q][16] (dense rows), B row j = (c,r,s), gathered
//       from the activation codes [C][Np/16][H*W][16] with the tap's shift.
// The contraction axis is cut into chunks of 16 codes (8 bytes), numbered
// t = group * inner + position (group: which sixteen channels / samples; position:
// tap for dX, output pixel for dW); a chunk is either wholly inside the image or
// wholly padding, so the gather works on whole chunks.
//
// A workgroup (4 waves) owns a BM x 128 tile of D.  Per K step of 8 chunks it stages
// the packed operand tiles in LDS (double buffered; the global loads of step i+1 are
// in flight while step i runs on the matrix cores).  Codes are widened to int8 in
// registers after the LDS read: a signed nibble is moved to the top of its byte
// (value * 16, exact two's complement), an unsigned nibble is masked in place; the
// accumulators therefore carry a factor 256 or 16 that the epilogue shifts out
// exactly.  v_mfma_i32_32x32x32_i8, int32 accumulation, exact.
//
// dW has a small output and a very long contraction: the contraction is split
// over workgroups, each writes its partial tile with plain stores, and a second
// kernel sums the partials and applies the scale (no atomics: the result does not
// depend on data sparsity or arrival order).
#include "lbt_internal.h"

namespace lbt {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int BN = 128;             // columns of D per workgroup
constexpr int BKC = 8;              // chunks (of 16 codes) per K step: 128 codes = 64 bytes per row
constexpr int PITCH = BKC * 8 + 8;  // LDS row pitch in bytes (72: conflict-free 8-byte reads)
constexpr int kXcds = 8;            // workgroups are dealt round-robin to 8 dies, each with its own L2

struct GemmArgs {
  const uint8_t* A;
  const uint8_t* B;
  long long lda;      // bytes per A row
  int M, NJ;          // rows of A, rows of B
  int chunks;         // total K chunks
  int chunks_per_split;
  int tiles_m, tiles_n, total_blocks;
  int epi;            // 0 = scaled store to NCHW dX, 1 = int32 partial tile (split K),
                      // 2 = scaled store row-major
  int scale_kind;     // 0: s_g*s_w   1: s_x*s_g (signed x)   2: s_x*s_g (unsigned x)
  int N, C, H, W, K, R, S, P, Q, stride, pad;
  int inner;          // chunk t = group * inner + pos; inner = R*S (dX) or P*Q (dW)
  int groups;         // granule groups per row of the gathered tensor (Kp/16 or Np/16)
  int shift;          // log2 of the factor carried by the accumulators
  const lbt_grad_state* st;
  const OperandScalars* sc;
  float* out;
  int32_t* acc;       // optional raw accumulators (direct epilogues only)
  int32_t* partial;   // [splits][M][NJ] for epi 1
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

__device__ __forceinline__ float output_scale(const GemmArgs& g) {
  const double s_g = (double)g.st->clip / 7.0;
  double other;
  if (g.scale_kind == 0) other = (double)g.sc->c_w / 7.0;
  else other = (double)g.sc->c_x / (g.scale_kind == 2 ? 15.0 : 7.0);
  return (float)(s_g * other);
}

// MODE 0: B rows are output pixels (dX of a convolution)
// MODE 1: B rows are (c,r,s) triples read with the tap's shift (dW; also every
//         linear-layer product, where the image is 1x1)
template <int BM, bool A_UNSIGNED, bool B_UNSIGNED, int MODE>
__global__ __launch_bounds__(kThreads) void k_implicit_gemm(const GemmArgs g) {
  constexpr int WGM = (BM == 128) ? 2 : 1;     // wave grid: WGM x WGN
  constexpr int WGN = 4 / WGM;
  constexpr int WM = BM / WGM, WN = BN / WGN;  // wave tile
  constexpr int TM = WM / 32, TN = WN / 32;    // 32x32 MFMA blocks per wave
  constexpr int NA = BM * BKC / kThreads, NB = BN * BKC / kThreads;
  __shared__ __attribute__((aligned(16))) uint8_t sA[2][BM * PITCH];
  __shared__ __attribute__((aligned(16))) uint8_t sB[2][BN * PITCH];
  extern __shared__ int s_tap[];  // MODE 0: [BN][R*S] pixel offset of each tap, or -1

  // workgroup id -> tile, so that the workgroups sharing a B tile run on one die
  const int per_xcd = gridDim.x / kXcds;
  const int lid = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
  if (lid >= g.total_blocks) return;
  const int m_tile = lid % g.tiles_m;
  const int n_tile = (lid / g.tiles_m) % g.tiles_n;
  const int split = lid / (g.tiles_m * g.tiles_n);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;
  const int m0 = m_tile * BM, j0 = n_tile * BN;
  const int t_begin = split * g.chunks_per_split;
  const int t_end = min(t_begin + g.chunks_per_split, g.chunks);
  const int HW = g.H * g.W, PQ = g.P * g.Q, RS = g.R * g.S;

  // ---- A staging: chunk-fastest, thread owns chunk column (tid & 7) of NA rows ----------
  const uint8_t* a_ptr[NA];
  bool a_ok[NA];
  const int a_cpos = tid & 7;
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    const int row = m0 + ((tid + kThreads * i) >> 3);
    a_ok[i] = row < g.M;
    a_ptr[i] = g.A + (long long)row * g.lda + (long long)(t_begin + a_cpos) * 8;
  }
  int a_t = t_begin + a_cpos;

  // ---- B staging ---------------------------------------------------------------------------
  // MODE 1: chunk-fastest like A; per row (c,r,s); thread-level running (group, p, q).
  int b_base[NB], b_dh[NB], b_dw[NB];
  bool b_ok[NB];
  int b_t = 0, b_grp = 0, b_p = 0, b_q = 0;
  // MODE 0: row-fastest; thread owns ONE pixel row and NB chunk columns.
  int x_row = 0, x_base = 0;
  bool x_ok = false;
  int x_t[NB], x_grp[NB], x_tap[NB];
  if (MODE == 1) {
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int j = j0 + ((tid + kThreads * i) >> 3);
      b_ok[i] = j < g.NJ;
      const int s_ = j % g.S, r_ = (j / g.S) % g.R, c_ = j / RS;
      b_base[i] = c_ * g.groups * HW;
      b_dh[i] = r_ - g.pad;
      b_dw[i] = s_ - g.pad;
    }
    b_t = t_begin + (tid & 7);
    b_grp = b_t / g.inner;
    const int pos = b_t - b_grp * g.inner;
    b_p = pos / g.Q;
    b_q = pos - b_p * g.Q;
  } else {
    x_row = tid % BN;
    const int j = j0 + x_row;
    x_ok = j < g.NJ;
    const int n_ = j / HW, hw = j - n_ * HW;
    const int h_ = hw / g.W, w_ = hw - h_ * g.W;
    x_base = n_ * g.groups * PQ;
    // tap table of this row; the 256 / BN threads that share the row split the taps
    for (int tap = tid / BN; tap < RS; tap += kThreads / BN) {
      const int fr = tap / g.S, fs = tap - fr * g.S;
      const int hp = h_ + g.pad - fr, wq = w_ + g.pad - fs;
      int off = -1;
      if (x_ok && hp >= 0 && wq >= 0) {
        const int p = hp / g.stride, q = wq / g.stride;
        if (p * g.stride == hp && q * g.stride == wq && p < g.P && q < g.Q) off = p * g.Q + q;
      }
      s_tap[x_row * RS + tap] = off;
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      x_t[i] = t_begin + tid / BN + i * (kThreads / BN);
      x_grp[i] = x_t[i] / g.inner;
      x_tap[i] = x_t[i] - x_grp[i] * g.inner;
    }
    __syncthreads();
  }

  uint2 ra[NA], rb[NB];
  auto load_tiles = [&]() {
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      ra[i] = make_uint2(0, 0);
      if (a_ok[i] && a_t < t_end) ra[i] = *reinterpret_cast<const uint2*>(a_ptr[i]);
      a_ptr[i] += BKC * 8;
    }
    a_t += BKC;
    if (MODE == 1) {
      const bool in_k = b_t < t_end;
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        rb[i] = make_uint2(0, 0);
        const int h = b_p * g.stride + b_dh[i], w = b_q * g.stride + b_dw[i];
        if (in_k && b_ok[i] && (unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W)
          rb[i] = *reinterpret_cast<const uint2*>(
              g.B + ((long long)b_base[i] + (long long)b_grp * HW + h * g.W + w) * 8);
      }
      b_t += BKC;
      if (g.inner == 1) {
        b_grp += BKC;
      } else {
        b_q += BKC;
        while (b_q >= g.Q) { b_q -= g.Q; ++b_p; }
        while (b_p >= g.P) { b_p -= g.P; ++b_grp; }
      }
    } else {
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        rb[i] = make_uint2(0, 0);
        if (x_t[i] < t_end) {
          const int off = s_tap[x_row * RS + x_tap[i]];
          if (off >= 0)
            rb[i] = *reinterpret_cast<const uint2*>(
                g.B + ((long long)x_base + (long long)x_grp[i] * PQ + off) * 8);
        }
        x_t[i] += BKC;
        if (g.inner == 1) {
          x_grp[i] += BKC;
        } else {
          x_tap[i] += BKC;
          while (x_tap[i] >= RS) { x_tap[i] -= RS; ++x_grp[i]; }
        }
      }
    }
  };
  auto store_tiles = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NA; ++i)
      *reinterpret_cast<uint2*>(&sA[buf][((tid + kThreads * i) >> 3) * PITCH + a_cpos * 8]) = ra[i];
    if (MODE == 1) {
#pragma unroll
      for (int i = 0; i < NB; ++i)
        *reinterpret_cast<uint2*>(&sB[buf][((tid + kThreads * i) >> 3) * PITCH + (tid & 7) * 8]) = rb[i];
    } else {
#pragma unroll
      for (int i = 0; i < NB; ++i)
        *reinterpret_cast<uint2*>(
            &sB[buf][x_row * PITCH + (tid / BN + i * (kThreads / BN)) * 8]) = rb[i];
    }
  };

  v16i acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  if (t_begin < t_end) {
    load_tiles();
    store_tiles(0);
  }
  __syncthreads();
  int buf = 0;
  for (int t0 = t_begin; t0 < t_end; t0 += BKC) {
    const bool more = t0 + BKC < t_end;
    if (more) load_tiles();
#pragma unroll
    for (int kk = 0; kk < BKC / 2; ++kk) {
      // one 32x32x32 step: lane holds row (lane % 32) and chunk 2*kk + lane/32
      const int coff = (2 * kk + (lane >> 5)) * 8;
      v4i fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[i] = widen<A_UNSIGNED>(*reinterpret_cast<const uint2*>(
            &sA[buf][(wm + i * 32 + (lane & 31)) * PITCH + coff]));
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[j] = widen<B_UNSIGNED>(*reinterpret_cast<const uint2*>(
            &sB[buf][(wn + j * 32 + (lane & 31)) * PITCH + coff]));
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (more) store_tiles(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }

  // ---- epilogue.  32x32 accumulator block: lane holds column (lane % 32) and rows
  // 8*(r/4) + 4*(lane/32) + r%4 for r = 0..15, so 32 lanes store 32 consecutive columns.
  const int shift = g.shift;
  const float scale = (g.epi == 1) ? 0.0f : output_scale(g);
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int col = j0 + wn + j * 32 + (lane & 31);
    if (col >= g.NJ) continue;
    long long base;
    long long row_stride;
    if (g.epi == 0) {
      const int n_ = col / HW, hw = col - n_ * HW;
      base = (long long)n_ * g.C * HW + hw;
      row_stride = HW;
    } else {
      base = col;
      row_stride = g.NJ;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row >= g.M) continue;
        const int v = acc[i][j][r] >> shift;
        const long long o = base + (long long)row * row_stride;
        if (g.epi == 1) {
          g.partial[(long long)split * g.M * g.NJ + o] = v;
        } else {
          g.out[o] = (float)v * scale;
          if (g.acc) g.acc[o] = v;
        }
      }
  }
}

// Sum the split-K partial tiles and apply the scale: out = (sum_s partial[s]) * s_a * s_b.
__global__ __launch_bounds__(kThreads) void k_splitk_reduce(const int32_t* __restrict__ partial,
                                                             int splits, long long n, GemmArgs g) {
  const float scale = output_scale(g);
  const long long stride = (long long)gridDim.x * kThreads;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
    int sum = 0;
    int s = 0;
    for (; s + 4 <= splits; s += 4) {
      const int v0 = partial[(long long)s * n + i], v1 = partial[(long long)(s + 1) * n + i];
      const int v2 = partial[(long long)(s + 2) * n + i], v3 = partial[(long long)(s + 3) * n + i];
      sum += (v0 + v1) + (v2 + v3);
    }
    for (; s < splits; ++s) sum += partial[(long long)s * n + i];
    g.out[i] = (float)sum * scale;
    if (g.acc) g.acc[i] = sum;
  }
}

void fill_geom(GemmArgs& g, const ConvGeom& c) {
  g.N = c.N; g.C = c.C; g.H = c.H; g.W = c.W; g.K = c.K; g.R = c.R; g.S = c.S;
  g.P = c.P; g.Q = c.Q; g.stride = c.stride; g.pad = c.pad;
}

template <int BM, int MODE>
void launch_variant(const GemmArgs& g, bool a_uns, bool b_uns, unsigned grid, size_t dyn,
                    hipStream_t s) {
  if (a_uns)
    LBT_LAUNCH((k_implicit_gemm<BM, true, false, MODE>), dim3(grid), dim3(kThreads), dyn, s, g);
  else if (b_uns)
    LBT_LAUNCH((k_implicit_gemm<BM, false, true, MODE>), dim3(grid), dim3(kThreads), dyn, s, g);
  else
    LBT_LAUNCH((k_implicit_gemm<BM, false, false, MODE>), dim3(grid), dim3(kThreads), dyn, s, g);
}

int run_gemm(GemmArgs& g, int mode, bool a_uns, bool b_uns, int bm, int splits, int kid,
             hipStream_t s) {
  // algorithmic work: the convolution's multiply-adds, padding taps included
  const double work = 2.0 * g.N * g.P * g.Q * (double)g.K * g.C * g.R * g.S;
  ProfScope prof(kid, work, s);
  if (a_uns && b_uns) return LBT_ERR_UNSUPPORTED;
  g.tiles_m = (g.M + bm - 1) / bm;
  g.tiles_n = (g.NJ + BN - 1) / BN;
  const long long total = (long long)g.tiles_m * g.tiles_n * splits;
  if (total > (1ll << 30)) return LBT_ERR_UNSUPPORTED;
  g.total_blocks = (int)total;
  const unsigned grid = (unsigned)((total + kXcds - 1) / kXcds * kXcds);
  size_t dyn = 0;
  if (mode == 0) {
    dyn = (size_t)BN * g.R * g.S * sizeof(int);
    if (dyn > 25 * 1024) return LBT_ERR_UNSUPPORTED;  // filter windows up to 7x7
    if (bm == 64) launch_variant<64, 0>(g, false, false, grid, dyn, s);
    else launch_variant<128, 0>(g, false, false, grid, dyn, s);
  } else {
    if (bm == 64) launch_variant<64, 1>(g, a_uns, b_uns, grid, dyn, s);
    else launch_variant<128, 1>(g, a_uns, b_uns, grid, dyn, s);
  }
  LBT_LAUNCH_CHECK();
  return LBT_OK;
}

// Direct (no split) product with signed operands: |sum| <= chunks*16 * 112 * 112 < 2^31.
int run_direct(GemmArgs& g, int mode, hipStream_t s) {
  g.chunks_per_split = g.chunks;
  g.shift = 8;
  g.scale_kind = 0;
  if ((long long)g.chunks * 16 * 12544 >= (1ll << 31)) return LBT_ERR_OVERFLOW;
  return run_gemm(g, mode, false, false, g.M <= 64 ? 64 : 128, 1, KID_GEMM_DX, s);
}

int run_splitk(GemmArgs& g, bool a_uns, bool b_uns, long long true_k, int32_t* acc, int32_t* partial,
               hipStream_t s) {
  const bool x_unsigned = a_uns || b_uns;
  g.shift = x_unsigned ? 4 : 8;
  g.scale_kind = x_unsigned ? 2 : 1;
  // the exact sum must fit int32
  if (true_k * (x_unsigned ? 105 : 49) >= (1ll << 31)) return LBT_ERR_OVERFLOW;
  const SplitPlan plan = plan_split_k(g.M, g.NJ, g.chunks);
  g.chunks_per_split = plan.chunks_per_split;
  int rc;
  if (plan.splits == 1) {
    g.epi = 2;
    g.acc = acc;
    return run_gemm(g, 1, a_uns, b_uns, plan.bm, 1, KID_GEMM_DW, s);
  }
  g.epi = 1;
  g.acc = nullptr;
  g.partial = partial;
  if ((rc = run_gemm(g, 1, a_uns, b_uns, plan.bm, plan.splits, KID_GEMM_DW, s))) return rc;
  const long long n_out = (long long)g.M * g.NJ;
  ProfScope prof(KID_FINALIZE, (double)n_out, s);
  g.acc = acc;
  long long blocks = (n_out + kThreads - 1) / kThreads;
  if (blocks > 4096) blocks = 4096;
  LBT_LAUNCH(k_splitk_reduce, dim3((unsigned)blocks), dim3(kThreads), 0, s, partial,
                     plan.splits, n_out, g);
  LBT_LAUNCH_CHECK();
  return LBT_OK;
}

}  // namespace

SplitPlan plan_split_k(int M, int NJ, int chunks) {
  SplitPlan p;
  p.bm = M <= 64 ? 64 : 128;
  const long long tiles = (long long)((M + p.bm - 1) / p.bm) * ((NJ + BN - 1) / BN);
  const int iters = (chunks + BKC - 1) / BKC;
  long long splits = 512 / tiles;           // aim at about two workgroups per compute unit
  if (splits < 1) splits = 1;
  if (splits > iters) splits = iters;
  const long long out_bytes = (long long)M * NJ * 4;
  while (splits > 1 && splits * out_bytes > (48ll << 20)) --splits;
  int per = (int)((iters + splits - 1) / splits) * BKC;
  if (per > 8192) per = 8192;               // 8192 chunks * 16 codes * 112 * 112 < 2^31
  p.chunks_per_split = per;
  p.splits = (chunks + per - 1) / per;
  p.partial_bytes = p.splits > 1 ? (size_t)p.splits * (size_t)out_bytes : 0;
  return p;
}

int launch_conv_dx(const ConvGeom& c, const uint8_t* w_codes, const uint8_t* g_codes,
                   const lbt_grad_state* st, const OperandScalars* sc, float* dX, int32_t* acc,
                   hipStream_t s) {
  GemmArgs g{};
  fill_geom(g, c);
  g.A = w_codes;
  g.B = g_codes;
  g.groups = c.Kp / kGranule;
  g.inner = c.R * c.S;
  g.chunks = g.groups * g.inner;
  g.lda = (long long)g.chunks * 8;
  g.M = c.C;
  const long long nj = (long long)c.N * c.H * c.W;
  if (nj > 0x7fffffffll) return LBT_ERR_UNSUPPORTED;
  g.NJ = (int)nj;
  g.epi = 0;
  g.st = st; g.sc = sc;
  g.out = dX; g.acc = acc;
  return run_direct(g, 0, s);
}

int launch_conv_dw(const ConvGeom& c, const uint8_t* g_codes, const uint8_t* x_codes,
                   const lbt_grad_state* st, const OperandScalars* sc, int x_unsigned, float* dW,
                   int32_t* acc, int32_t* partial, hipStream_t s) {
  GemmArgs g{};
  fill_geom(g, c);
  g.A = g_codes;
  g.B = x_codes;
  g.groups = c.Np / kGranule;
  g.inner = c.P * c.Q;
  const long long chunks = (long long)g.inner * g.groups;
  if (chunks > 0x7fffffffll / 16) return LBT_ERR_UNSUPPORTED;
  g.chunks = (int)chunks;
  g.lda = chunks * 8;
  g.M = c.K;
  g.NJ = c.C * c.R * c.S;
  g.st = st; g.sc = sc;
  g.out = dW;
  return run_splitk(g, false, x_unsigned != 0, (long long)c.N * c.P * c.Q, acc, partial, s);
}

// Linear layer (1x1 image): operands swap roles so that the row-major outputs
// dX[M][K_in] and dW[K_in][N_out] have their contiguous axis on the lanes.
int launch_linear_dx(const ConvGeom& c, const uint8_t* w_codes, const uint8_t* g_codes,
                     const lbt_grad_state* st, const OperandScalars* sc, float* dX, int32_t* acc,
                     hipStream_t s) {
  GemmArgs g{};
  fill_geom(g, c);
  g.A = g_codes;   // [N][Kp/16][16] gradient rows
  g.B = w_codes;   // [C][Kp/16][16] weight rows, read with the (c,r,s)-row gather on a 1x1 image
  g.groups = c.Kp / kGranule;
  g.inner = 1;
  g.chunks = g.groups;
  g.lda = (long long)g.chunks * 8;
  g.M = c.N;
  g.NJ = c.C;
  g.epi = 2;
  g.st = st; g.sc = sc;
  g.out = dX; g.acc = acc;
  return run_direct(g, 1, s);
}

int launch_linear_dw(const ConvGeom& c, const uint8_t* g_codes, const uint8_t* x_codes,
                     const lbt_grad_state* st, const OperandScalars* sc, int x_unsigned, float* dW,
                     int32_t* acc, int32_t* partial, hipStream_t s) {
  GemmArgs g{};
  fill_geom(g, c);
  g.A = x_codes;   // [C][Np/16][16] activation rows
  g.B = g_codes;   // [K][Np/16][16] gradient rows
  g.groups = c.Np / kGranule;
  g.inner = 1;
  g.chunks = g.groups;
  g.lda = (long long)g.chunks * 8;
  g.M = c.C;
  g.NJ = c.K;
  g.st = st; g.sc = sc;
  g.out = dW;
  return run_splitk(g, x_unsigned != 0, false, (long long)c.N, acc, partial, s);
}

}  // namespace lbt
