// Integer contractions of the backward pass on int8 matrix cores (gfx950).
//
// Both gradients of a convolution (and of a linear layer, which is the 1x1 case
// on a 1x1 image) are computed by one implicit-GEMM kernel
//     D[m][j] = sum_k A[m][k] * B[j][k]
// whose operands are 4-bit codes held one per int8 byte, in granules ("chunks") of 16
// codes = 16 bytes along the contraction axis:
//   dX: A = weights  [C][R*S][Kp/16][16] (dense rows, tap-major), B row j = input pixel
//       (n,h,w), gathered from the gradient codes [N][Kp/16][P*Q][16] tap by tap;
//   dW: A = gradient [K][Np/16][P*Q][16] (dense rows), B row j = (c,r,s), gathered
//       from the activation codes [C][Np/16][H*W][16] with the tap's shift.
// A chunk is either wholly inside the image or wholly padding, so the gather works on
// whole chunks.  dX runs over the contraction tap by tap (all channel groups of one tap,
// then the next tap; the group count is padded to 1, 2, 4 or a multiple of 8 with
// zero chunks so that a K step of 8 chunks never straddles taps unevenly); dW runs
// over t = sample_group * P*Q + output pixel.
//
// A workgroup (4 waves) owns a BM x BN tile of D (64 or 128 each; smaller tiles when the
// problem would otherwise not fill the chip).  Per K step of 8 chunks (128 codes) the
// operand tiles go from global memory straight into LDS (buffer loads with the LDS
// destination, 16 bytes per lane, no registers and no ALU work in between; an offset
// outside the tensor writes zeros, which is how padding, ragged edges and the K tail
// are masked).  A wave's load lands as 1 KiB of consecutive LDS bytes in lane order, so
// the lane -> (row, chunk) assignment fixes the tile layout:
//   dense rows (A; B of dW): [row][8 chunks], eight lanes read 128 consecutive bytes of
//       one row; chunk c of row r sits in slot c ^ ((r >> 1) & 7) so that the 32 rows a
//       fragment read touches fall into different banks;
//   gathered pixels (B of dX): [chunk][row], 64 lanes read the granules of 64
//       consecutive pixels (consecutive in memory) and a fragment read is contiguous.
// Two to four LDS stages: while the matrix cores work on step s (fragments already in
// registers), the loads of the following steps are in flight.  v_mfma_i32_32x32x32_i8, int32
// accumulation, exact.  The forward product of a convolution is the dX kernel with another
// tap table (output pixel -> input pixel under the tap); that of a linear layer the dense-row
// mode with the operands' roles exchanged.
//
// dW has a small output and a very long contraction: the contraction is split
// over workgroups, each writes its partial tile with plain stores, and a second
// kernel sums the partials and applies the scale (no atomics: the result does not
// depend on data sparsity or arrival order).
#include <atomic>

#include "lbt_internal.h"
#include <type_traits>

namespace lbt {
int launch_pending_reduce(const PendingReduce& r, lbt_grad_state* update_st, hipStream_t s);
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;

constexpr int kThreads = 256;
constexpr int BKC = 8;             // chunks (of 16 codes) per K step
constexpr int ROWB = BKC * 16;     // bytes of one tile row per K step
constexpr int kXcds = 8;           // workgroups are dealt round-robin to 8 dies, each with its own L2

struct GemmArgs {
  const uint8_t* A;
  const uint8_t* B;
  unsigned a_bytes, b_bytes;  // sizes of the two code tensors (buffer bounds)
  unsigned lda;       // bytes per A row
  int M, NJ;          // rows of A, rows of B
  int chunks;         // MODE 1: K chunks; MODE 0: padded chunk count R*S*Gp
  int steps, steps_per_split;
  int tiles_m, tiles_n, total_blocks;
  int epi;            // 0 = scaled store to NCHW dX, 1 = int32 partial tile (split K),
                      // 2 = scaled store row-major, 3 = NCHW dX of a strided 1x1 convolution:
                      //     the columns are the P x Q output pixels of the forward layer, each
                      //     owning a cell of up x up input pixels of which only the corner
                      //     receives a sum (out_h x out_w = the input image, up = the stride)
  int out_h, out_w, up;
  int scale_kind;     // 0: s_g*s_w   1: s_x*s_g (signed x)   2: s_x*s_g (unsigned x)
                      // 3: s_x*s_w (signed x)   4: s_x*s_w (unsigned x): forward product
  int fwd;            // MODE 0 gathers input pixels of a forward convolution (see the tap table)
  int32_t* status_out;  // forward product: receives LBT_STATUS_OK / NONFINITE of its operands
  int bits;           // b: the codes' scales are c / levels(b)
  int N, C, H, W, K, R, S, P, Q, stride, pad;
  int inner;          // MODE 1: chunk t = group * inner + pos, inner = P*Q (1 for linear)
  int groups;         // granule groups per row of the gathered tensor (Kp/16 or Np/16)
  int gp, gp_log2;    // MODE 0: padded group count; gp_log2 >= 0 when gp is 1, 2 or 4, else -1
  const lbt_grad_state* st;
  lbt_grad_state* update_st;  // not null: this launch also applies Alg. 1 to the state
  const OperandScalars* sc;
  float* out;
  int32_t* acc;       // optional raw accumulators (direct epilogues only)
  int32_t* partial;   // [splits][M][NJ] for epi 1
  // A split contraction left pending by the launch before this one (dW's int32 partial tiles):
  // workgroups gemm_grid .. gemm_grid + red.blocks - 1 of this launch add its slices and apply
  // its scale, beside the workgroups of this launch's own product.
  PendingReduce red;
  unsigned gemm_grid; // workgroups of the product itself (a multiple of the die count)
};

// 16 bytes per lane from a buffer straight into LDS: lane l of the wave writes LDS byte
// dst + 16 * l (dst uniform across the wave); an offset outside the buffer writes zeros.
// Issued as an instruction the compiler does not track, so that the kernel can wait for
// the loads of one K step while those of later steps stay in flight (wait_loads below);
// every read of the tile is ordered after such a wait and a workgroup barrier.
__device__ __forceinline__ void load16_to_lds(__amdgpu_buffer_rsrc_t rsrc, unsigned dst,
                                              unsigned offset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "s"(dst), "v"(offset), "s"(rsrc) : "memory", "m0");
}
// Wait until at most N of this wave's buffer loads are outstanding.
template <int N>
__device__ __forceinline__ void wait_loads() {
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

__device__ __forceinline__ float output_scale(int scale_kind, int bits, const lbt_grad_state* st,
                                              const OperandScalars* sc) {
  const double q_signed = (double)levels(bits, false);
  if (scale_kind >= 3)
    return (float)(((double)sc->c_x / (scale_kind == 4 ? (double)levels(bits, true) : q_signed)) *
                   ((double)sc->c_w / q_signed));
  const double s_g = (double)st->clip / q_signed;
  double other;
  if (scale_kind == 0) other = (double)sc->c_w / q_signed;
  else other = (double)sc->c_x / (scale_kind == 2 ? (double)levels(bits, true) : q_signed);
  return (float)(s_g * other);
}
__device__ __forceinline__ float output_scale(const GemmArgs& g) {
  return output_scale(g.scale_kind, g.bits, g.st, g.sc);
}

// Sum the split-K partial tiles and apply the scale: out = (sum_s partial[s]) * s_a * s_b.
// A workgroup takes 256 / SL consecutive outputs at a time; SL groups of threads share the
// slices (group w sums slices w, w + SL, ..., eight loads in flight per thread) and meet in
// LDS.  SL = 4 for many slices of a small output, SL = 1 for few slices of a large one.
// Integer adds: the result does not depend on how the slices are grouped.
// WIDE: the slices are added in 64 bits (their sum may exceed 32 bits; each slice fits).
// Workgroup `blk` of `nblk`.
template <int SL, bool WIDE>
__device__ __forceinline__ void reduce_slices(const PendingReduce& r, unsigned blk, unsigned nblk) {
  constexpr int OUTS = kThreads / SL;
  using sum_t = typename std::conditional<WIDE, long long, int>::type;
  __shared__ sum_t red[SL][OUTS];
  const float scale = output_scale(r.scale_kind, r.bits, r.st, r.sc);
  const int32_t* __restrict__ partial = r.partial;
  const long long n = r.n;
  const int splits = r.splits;
  const int io = threadIdx.x % OUTS, sl = threadIdx.x / OUTS;
  for (long long base = (long long)blk * OUTS; base < n; base += (long long)nblk * OUTS) {
    const long long i = base + io;
    sum_t sum = 0;
    if (i < n) {
      for (int s0 = sl; s0 < splits; s0 += 8 * SL) {
        int v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int sp = s0 + SL * u;
          v[u] = sp < splits ? partial[(long long)sp * n + i] : 0;
        }
        sum += (((sum_t)v[0] + v[1]) + ((sum_t)v[2] + v[3])) + (((sum_t)v[4] + v[5]) + ((sum_t)v[6] + v[7]));
      }
    }
    if (SL > 1) {
      red[sl][io] = sum;
      __syncthreads();
      if (sl == 0) {
        sum = 0;
#pragma unroll
        for (int w = 0; w < SL; ++w) sum += red[w][io];
      }
    }
    if (sl == 0 && i < n) {
      r.out[i] = (float)sum * scale;
      if (r.acc) r.acc[i] = (int)sum;   // the host has checked that it fits
    }
    if (SL > 1) __syncthreads();
  }
}

// MODE 0: B rows are input pixels (dX of a convolution)
// MODE 1: B rows are (c,r,s) triples read with the tap's shift (dW; also every
//         linear-layer product, where the image is 1x1)
template <int BM, int BN, int MODE, int STAGES, bool STREAM>
__global__ __launch_bounds__(kThreads) void k_implicit_gemm(const GemmArgs g) {
  // wave grid WGM x WGN: 128x128 -> 2x2, 64x128 -> 1x4, 128x64 -> 4x1, 64x64 -> 2x2
  constexpr int WGM = (BM == BN) ? 2 : (BM > BN ? 4 : 1);
  constexpr int WGN = 4 / WGM;
  constexpr int WM = BM / WGM, WN = BN / WGN;  // wave tile
  constexpr int TM = WM / 32, TN = WN / 32;    // 32x32 MFMA blocks per wave
  constexpr int NA = BM * BKC / kThreads, NB = BN * BKC / kThreads;  // loads per thread per step
  constexpr int STAGE = (BM + BN) * ROWB;      // bytes of one LDS stage (A tile, then B tile)
  constexpr int LPS = NA + NB;                 // buffer loads of a wave per K step
  // dynamic LDS: STAGES stages, then (MODE 0) the tap table
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  int* const s_tap = reinterpret_cast<int*>(lds + STAGES * STAGE);  // [BN][R*S]
  const unsigned lds_base = (unsigned)(uintptr_t)(lds_ptr_t)lds;    // LDS byte address of lds[0]

  // the workgroups behind the product's own carry out a pending split-K sum (measured: placed
  // in front of them instead, they delay the product more than they gain: 5.36 against
  // 5.31 ms per ResNet-50 step)
  if (blockIdx.x >= g.gemm_grid) {
    if (g.red.many) reduce_slices<4, false>(g.red, blockIdx.x - g.gemm_grid, g.red.blocks);
    else reduce_slices<1, false>(g.red, blockIdx.x - g.gemm_grid, g.red.blocks);
    return;
  }
  // workgroup id -> tile, so that the workgroups sharing a B tile run on one die
  const unsigned bid = blockIdx.x;
  const int per_xcd = g.gemm_grid / kXcds;
  const int lid = (bid % kXcds) * per_xcd + bid / kXcds;
  if (lid >= g.total_blocks) return;
  // (the products read only the clip value from the state: no order to keep with this)
  if (g.update_st && bid == 0 && threadIdx.x == 0) interval_update(g.update_st);
  if (g.status_out && bid == 0 && threadIdx.x == 0)
    *g.status_out = (g.sc->bad_x | g.sc->bad_w) ? LBT_STATUS_NONFINITE : LBT_STATUS_OK;
  const int m_tile = lid % g.tiles_m;
  const int n_tile = (lid / g.tiles_m) % g.tiles_n;
  const int split = lid / (g.tiles_m * g.tiles_n);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;
  const int m0 = m_tile * BM, j0 = n_tile * BN;
  const int s_begin = split * g.steps_per_split;
  const int n_steps = min(s_begin + g.steps_per_split, g.steps) - s_begin;
  const int HW = g.H * g.W, PQ = g.P * g.Q, RS = g.R * g.S;

  // Raw buffer views of the code tensors: a load whose offset is >= the size returns 0.
  const __amdgpu_buffer_rsrc_t rsrc_a =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(g.A), 0, g.a_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_b =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(g.B), 0, g.b_bytes, 0x00020000);
  const unsigned oob_a = g.a_bytes, oob_b = g.b_bytes;

  // ---- dense-row staging ([row][slot] tiles): load i of a wave covers tile rows
  // (4 i + wave) * 8 .. + 8; lane -> row (lane / 8) of them and slot (lane % 8), which
  // holds chunk slot ^ ((row >> 1) & 7): sixteen consecutive rows of one chunk then fall into
  // sixteen different 16-byte bank groups (a row is 128 bytes = 8 groups, so rows r and r + 1
  // differ by 8 groups and the slot permutation has to change every second row; with
  // slot ^ (row & 7) fragment reads met two-way conflicts: measured, up to one conflict cycle
  // per active LDS cycle).  The chunk is the same for all loads of a thread:
  // row = (4 i + wave) * 8 + lane / 8, so (row >> 1) & 7 = 4 (wave & 1) + lane / 16.
  const int col = (lane & 7) ^ ((4 * (wave & 1) + (lane >> 4)) & 7);
  const int sub = lane >> 3;
  unsigned a_row[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) a_row[i] = (unsigned)(m0 + (4 * i + wave) * 8 + sub) * g.lda;
  // MODE 0 walks (tap, group); all threads of the workgroup share (tap_base, kg_base)
  const bool small = g.gp_log2 >= 0;
  int tap_base = 0, kg_base = 0;
  int a_dt = 0, a_kgo = col;
  // MODE 1 walks chunk t = 8 * step + col
  int t_cur = s_begin * BKC + col;

  // ---- B staging ---------------------------------------------------------------------------
  // MODE 1: dense-row scheme like A; row i is a (c,r,s) triple; the thread's running output
  // position (group, p, q) belongs to its chunk.
  unsigned b_row[NB];
  int b_dh[NB], b_dw[NB];
  int b_grp = 0, b_p = 0, b_q = 0;
  // MODE 0: [chunk][row] tile; load i of a wave covers chunk x_chunk(i) and 64 consecutive
  // pixel rows, lane -> pixel row x_row (the same for all loads of a thread).
  constexpr int HALVES = BN / 64;
  const int x_row = (wave % HALVES) * 64 + lane;
  unsigned x_const = 0;
  if (MODE == 1) {
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int j = j0 + (4 * i + wave) * 8 + sub;
      const int c_ = j / RS, rs = j - c_ * RS;
      const int r_ = rs / g.S, s_ = rs - r_ * g.S;
      b_dh[i] = r_ - g.pad;
      b_dw[i] = s_ - g.pad;
      b_row[i] = j < g.NJ ? (unsigned)(c_ * g.groups * HW + b_dh[i] * g.W + b_dw[i]) * 16u : oob_b;
    }
    b_grp = t_cur / g.inner;
    const int pos = t_cur - b_grp * g.inner;
    b_p = pos / g.Q;
    b_q = pos - b_p * g.Q;
  } else {
    const int t0 = s_begin * BKC;
    if (small) {
      tap_base = t0 >> g.gp_log2;
      a_dt = col >> g.gp_log2;
      a_kgo = col & (g.gp - 1);
    } else {
      tap_base = t0 / g.gp;
      kg_base = t0 - tap_base * g.gp;
    }
    // tap table: byte offset of output pixel (p,q) inside one channel group, or -1 when
    // the tap falls outside the output / between strides.  Row tid % BN; the 256 / BN
    // threads that share a row split its taps.
    {
      constexpr int SUB = kThreads / BN;
      const int t_row = tid % BN;
      const int j = j0 + t_row;
      const bool ok = j < g.NJ;
      const int n_ = j / HW, hw = j - n_ * HW;
      const int h_ = hw / g.W, w_ = hw - h_ * g.W;
      int fr = 0, fs = tid / BN;
      while (fs >= g.S) { fs -= g.S; ++fr; }
      for (int tap = tid / BN; tap < RS; tap += SUB) {
        int hp = h_ + g.pad - fr, wq = w_ + g.pad - fs;
        int off = -1;
        if (g.fwd) {
          // forward: column (h_, w_) is an OUTPUT pixel, the table points at the input pixel
          // under tap (fr, fs); g.P x g.Q is the input image here
          hp = h_ * g.stride - g.pad + fr;
          wq = w_ * g.stride - g.pad + fs;
          if (ok && hp >= 0 && wq >= 0 && hp < g.P && wq < g.Q) off = (hp * g.Q + wq) * 16;
        } else if (ok && hp >= 0 && wq >= 0) {
          int p, q;
          bool on_grid;
          if (g.stride == 1) {
            p = hp; q = wq; on_grid = true;
          } else if (g.stride == 2) {
            p = hp >> 1; q = wq >> 1; on_grid = ((hp | wq) & 1) == 0;
          } else {
            p = hp / g.stride; q = wq / g.stride;
            on_grid = p * g.stride == hp && q * g.stride == wq;
          }
          if (on_grid && p < g.P && q < g.Q) off = (p * g.Q + q) * 16;
        }
        s_tap[t_row * RS + tap] = off;
        fs += SUB;
        while (fs >= g.S) { fs -= g.S; ++fr; }
      }
    }
    {
      const int j = j0 + x_row;
      const int n_ = j / HW;
      x_const = (unsigned)(n_ * g.groups * PQ) * 16u;   // rows past the end have no valid tap
    }
    __syncthreads();
  }

  // MODE 0, group count >= 8: every K step lies inside one tap; x_cur holds the byte offset
  // of this lane's pixel at the current tap (x_const + table entry), or an offset beyond
  // every buffer when the tap does not reach the pixel.
  constexpr unsigned kNoTap = 0x80000000u;
  unsigned x_cur = kNoTap;
  auto load_tap = [&](int tap) {
    const int off = s_tap[x_row * RS + min(tap, RS - 1)];
    x_cur = off >= 0 ? x_const + (unsigned)off : kNoTap;
  };
  if (MODE == 0 && !small) load_tap(tap_base);
  const unsigned pq16 = (unsigned)PQ * 16u;

  // Issue the loads of the next K step into LDS stage `st` and advance the walk.  A step
  // past the end of this workgroup's K range loads zero A chunks (its tile is never read).
  int ld_step = 0;
  auto issue = [&](int st) {
    const unsigned sa = lds_base + st * STAGE;
    const unsigned sb = sa + BM * ROWB;
    const bool live = ld_step < n_steps;
    ++ld_step;
    if (MODE == 1) {
      const unsigned a_col = (live && t_cur < g.chunks) ? (unsigned)t_cur * 16u : oob_a;
#pragma unroll
      for (int i = 0; i < NA; ++i)
        load16_to_lds(rsrc_a, sa + (4 * i + wave) * 1024, min(a_row[i] + a_col, oob_a));
      const int ph = b_p * g.stride, qw = b_q * g.stride;
      const unsigned pos = (unsigned)(b_grp * HW + ph * g.W + qw) * 16u;
      if (g.pad == 0) {
#pragma unroll
        for (int i = 0; i < NB; ++i) load16_to_lds(rsrc_b, sb + (4 * i + wave) * 1024, b_row[i] + pos);
      } else {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
          const bool in = (unsigned)(ph + b_dh[i]) < (unsigned)g.H &&
                          (unsigned)(qw + b_dw[i]) < (unsigned)g.W;
          load16_to_lds(rsrc_b, sb + (4 * i + wave) * 1024, in ? b_row[i] + pos : oob_b);
        }
      }
      t_cur += BKC;
      if (g.inner == 1) {
        b_grp += BKC;
      } else {
        b_q += BKC;
        while (b_q >= g.Q) { b_q -= g.Q; ++b_p; }
        while (b_p >= g.P) { b_p -= g.P; ++b_grp; }
      }
    } else {
      const int tap_a = tap_base + a_dt, kg_a = kg_base + a_kgo;
      const unsigned a_col = (live && tap_a < RS && kg_a < g.groups)
                                 ? (unsigned)(tap_a * g.groups + kg_a) * 16u : oob_a;
#pragma unroll
      for (int i = 0; i < NA; ++i)
        load16_to_lds(rsrc_a, sa + (4 * i + wave) * 1024, min(a_row[i] + a_col, oob_a));
      if (small) {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
          // load i of this wave: chunk (4 i + wave) / HALVES of the step, all lanes alike
          const int c = (4 * i + wave) / HALVES;
          const int kg = c & (g.gp - 1);
          // chunks past the last tap or group meet zero A chunks: any in-table tap will do
          const int tap = min(tap_base + (c >> g.gp_log2), RS - 1);
          const int off = s_tap[x_row * RS + tap];
          load16_to_lds(rsrc_b, sb + (4 * i + wave) * 1024,
                        off >= 0 ? x_const + (unsigned)kg * pq16 + (unsigned)off : oob_b);
        }
        tap_base += BKC >> g.gp_log2;
      } else {
        const unsigned k0 = (unsigned)(kg_base + wave / HALVES) * pq16;   // uniform
#pragma unroll
        for (int i = 0; i < NB; ++i)
          load16_to_lds(rsrc_b, sb + (4 * i + wave) * 1024, x_cur + k0 + (unsigned)(4 * i / HALVES) * pq16);
        kg_base += BKC;
        if (kg_base >= g.gp) {
          kg_base = 0;
          ++tap_base;
          load_tap(tap_base);
        }
      }
    }
  };

  // the output scale's inputs are fetched now, long before the epilogue needs them
  const float scale = (g.epi == 1) ? 0.0f : output_scale(g);

  v16i acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  // Fragment addresses inside a stage: one 32x32x32 product takes, per lane, row (lane % 32)
  // and chunk 2*kk + lane/32 of each operand.
  unsigned fa_off[BKC / 2][TM], fb_off[BKC / 2][TN];
#pragma unroll
  for (int kk = 0; kk < BKC / 2; ++kk) {
    const int c = 2 * kk + (lane >> 5);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int r = wm + i * 32 + (lane & 31);
      fa_off[kk][i] = (unsigned)(r * ROWB + ((c ^ ((r >> 1) & 7)) * 16));
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int r = wn + j * 32 + (lane & 31);
      fb_off[kk][j] = (unsigned)(BM * ROWB) +
                      (MODE == 1 ? (unsigned)(r * ROWB + ((c ^ ((r >> 1) & 7)) * 16)) : (unsigned)((c * BN + r) * 16));
    }
  }

  // Pipeline with STAGES LDS stages.  Every step issues the loads of step s + STAGES - 1
  // (zero tiles past the end), so exactly STAGES - 2 later steps are in flight whenever a
  // step is waited for.  After the barrier every wave pulls the step's fragments into
  // registers, then the new loads go into the stage that step s - 1 used (all waves have
  // read it: they passed this barrier), then the matrix cores run on the fragments.
  constexpr int AHEAD = STAGES - 1;
#pragma unroll
  for (int d = 0; d < AHEAD; ++d) issue(d);
  int st_read = 0, st_load = AHEAD % STAGES;
  for (int s = 0; s < n_steps; ++s) {
    wait_loads<(AHEAD - 1) * LPS>();
    __syncthreads();
    const uint8_t* const stage = lds + st_read * STAGE;
    v4i fa[BKC / 2][TM], fb[BKC / 2][TN];
#pragma unroll
    for (int kk = 0; kk < BKC / 2; ++kk) {
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[kk][i] = *reinterpret_cast<const v4i*>(stage + fa_off[kk][i]);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[kk][j] = *reinterpret_cast<const v4i*>(stage + fb_off[kk][j]);
    }
    issue(st_load);
    st_read = st_read + 1 == STAGES ? 0 : st_read + 1;
    st_load = st_load + 1 == STAGES ? 0 : st_load + 1;
#pragma unroll
    for (int kk = 0; kk < BKC / 2; ++kk)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[kk][i], fb[kk][j], acc[i][j], 0, 0, 0);
  }
  // the zero tiles requested past the end must have landed before the LDS is given back
  wait_loads<0>();

  // ---- epilogue.  32x32 accumulator block: lane holds column (lane % 32) and rows
  // 8*(r/4) + 4*(lane/32) + r%4 for r = 0..15, so 32 lanes store 32 consecutive columns.
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int col_j = j0 + wn + j * 32 + (lane & 31);
    if (col_j >= g.NJ) continue;
    long long base;
    long long row_stride;
    // (the gather mode only ever has the two NCHW epilogues, the dense-row mode the other two:
    // each kernel compiles its own pair)
    if (MODE == 0 && g.epi == 3) {
      // column = (n, p, q); the cell's corner is input pixel (p * up, q * up); the rest of
      // the cell gets zeros (no output position of the layer reads those pixels with a tap)
      const int n_ = col_j / HW, pq = col_j - n_ * HW;
      const int p_ = pq / g.W, q_ = pq - p_ * g.W;
      const int h0 = p_ * g.up, w0 = q_ * g.up;
      const long long plane = (long long)g.out_h * g.out_w;
      const long long cell = (long long)n_ * g.C * plane + (long long)h0 * g.out_w + w0;
      const bool pair = g.up == 2 && (g.out_w & 1) == 0;   // (value, 0) as one 8-byte store
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = m0 + wm + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (row >= g.M) continue;
          const int v = acc[i][j][r];
          const float f = (float)v * scale;
          const long long o = cell + (long long)row * plane;
          if (pair) {
            *reinterpret_cast<float2*>(g.out + o) = make_float2(f, 0.0f);
            if (g.acc) *reinterpret_cast<int2*>(g.acc + o) = make_int2(v, 0);
            if (h0 + 1 < g.out_h) {
              *reinterpret_cast<float2*>(g.out + o + g.out_w) = make_float2(0.0f, 0.0f);
              if (g.acc) *reinterpret_cast<int2*>(g.acc + o + g.out_w) = make_int2(0, 0);
            }
          } else {
            for (int dy = 0; dy < g.up && h0 + dy < g.out_h; ++dy)
              for (int dx = 0; dx < g.up && w0 + dx < g.out_w; ++dx) {
                const bool corner = (dy | dx) == 0;
                g.out[o + (long long)dy * g.out_w + dx] = corner ? f : 0.0f;
                if (g.acc) g.acc[o + (long long)dy * g.out_w + dx] = corner ? v : 0;
              }
          }
        }
      continue;
    }
    if (MODE == 0) {
      const int n_ = col_j / HW, hw = col_j - n_ * HW;
      base = (long long)n_ * g.C * HW + hw;
      row_stride = HW;
    } else {
      base = col_j;
      row_stride = g.NJ;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row >= g.M) continue;
        const int v = acc[i][j][r];
        const long long o = base + (long long)row * row_stride;
        if (MODE == 1 && g.epi == 1) {
          g.partial[(long long)split * g.M * g.NJ + o] = v;
        } else {
          if (STREAM) __builtin_nontemporal_store((float)v * scale, &g.out[o]);
          else g.out[o] = (float)v * scale;
          if (g.acc) g.acc[o] = v;
        }
      }
  }
}

// The same sum as a launch of its own (no product launch follows that could carry it).
template <int SL, bool WIDE>
__global__ __launch_bounds__(kThreads) void k_splitk_reduce(const PendingReduce r, lbt_grad_state* update_st) {
  if (update_st && blockIdx.x == 0 && threadIdx.x == 0) interval_update(update_st);
  reduce_slices<SL, WIDE>(r, blockIdx.x, gridDim.x);
}

void fill_geom(GemmArgs& g, const ConvGeom& c) {
  g.N = c.N; g.C = c.C; g.H = c.H; g.W = c.W; g.K = c.K; g.R = c.R; g.S = c.S;
  g.P = c.P; g.Q = c.Q; g.stride = c.stride; g.pad = c.pad;
  g.bits = c.bits;
}

constexpr size_t kMaxDynLds = 128 * 1024;
constexpr int kMaxDevices = 64;

template <int BM, int BN, int MODE, int STAGES, bool STREAM>
int launch_one(const GemmArgs& g, unsigned grid, size_t tap_bytes, hipStream_t s) {
  void (*kernel)(const GemmArgs) = &k_implicit_gemm<BM, BN, MODE, STAGES, STREAM>;
  const size_t dyn = (size_t)STAGES * (BM + BN) * ROWB + tap_bytes;
  if (dyn > kMaxDynLds) return LBT_ERR_UNSUPPORTED;
  // more than 64 KiB of dynamic LDS has to be allowed once per kernel and device (callers on
  // several threads may arrive here together: setting the attribute twice is harmless)
  static std::atomic<bool> raised[kMaxDevices];
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess) return LBT_ERR_HIP;
  const bool tracked = device >= 0 && device < kMaxDevices;
  if (!tracked || !raised[device].load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)kMaxDynLds) != hipSuccess)
      return LBT_ERR_HIP;
    if (tracked) raised[device].store(true, std::memory_order_release);
  }
  LBT_LAUNCH(kernel, dim3(grid + g.red.blocks), dim3(kThreads), dyn, s, g);
  return LBT_OK;
}

int run_gemm(GemmArgs& g, int mode, int bm, int bn, int splits, int kid, hipStream_t s) {
  // algorithmic work: the convolution's multiply-adds, padding taps included
  // (the convolution's output image is P x Q, except in the forward product's geometry)
  const double out_px = g.fwd ? (double)g.H * g.W : (double)g.P * g.Q;
  const double work = 2.0 * g.N * out_px * (double)g.K * g.C * g.R * g.S;
  ProfScope prof(kid, work, s);
  // 32-bit buffer offsets: both code tensors below 2 GiB, with room for the rows of a
  // ragged last tile
  if ((unsigned long long)g.a_bytes >= (1ull << 31) || (unsigned long long)g.b_bytes >= (1ull << 31) ||
      (unsigned long long)(g.M + 128) * g.lda + g.a_bytes >= (1ull << 32))
    return LBT_ERR_UNSUPPORTED;
  // measurement aid: launch, prologue and epilogue only (the outputs are then all zero)
  if (profile_skeleton()) g.steps = g.steps_per_split = 0;
  g.tiles_m = (g.M + bm - 1) / bm;
  g.tiles_n = (g.NJ + bn - 1) / bn;
  const long long total = (long long)g.tiles_m * g.tiles_n * splits;
  if (total > (1ll << 30)) return LBT_ERR_UNSUPPORTED;
  g.total_blocks = (int)total;
  const unsigned grid = (unsigned)((total + kXcds - 1) / kXcds * kXcds);
  g.gemm_grid = grid;
  size_t tap_bytes = 0;
  if (mode == 0) {
    if ((size_t)128 * g.R * g.S * sizeof(int) > 25 * 1024) return LBT_ERR_UNSUPPORTED;  // up to 7x7
    tap_bytes = (size_t)bn * g.R * g.S * sizeof(int);
  }
  // LDS stages (= K steps of loads in flight + 1).  Measured on the ResNet-50 shapes:
  // workgroups sharing a compute unit hide each other's latency better than a deeper
  // pipeline does, so the deep variants (3 stages, 4 for 64x64) are used only when the
  // whole grid still fits the chip in one go with their larger LDS footprint.
  const int deep_stages = (bm == 64 && bn == 64) ? 4 : 3;
  const size_t deep_lds = (size_t)deep_stages * (bm + bn) * ROWB + tap_bytes;
  const long long deep_capacity = 256ll * (long long)((160 * 1024) / deep_lds);
  const bool deep = total <= deep_capacity;
  // Direct epilogues write the fp32 result with streaming (non-temporal) stores where a wave's
  // 32-column segments start on 64-byte boundaries (rows of a multiple of 16 floats): the
  // result then leaves for HBM while the product runs, instead of sitting dirty in the cache
  // until the next layer's sweeps evict it (measured on the ResNet-50 sweep: -0.4 ms in the
  // maximum kernel against +0.1 ms here).  Rows that start inside a line (14x14 and 7x7 maps)
  // keep ordinary stores: the cache merges their partial lines, streaming stores do not.
  const bool stream_out = (g.epi == 0) ? (g.H * g.W) % 16 == 0 : (g.epi == 2 && g.NJ % 16 == 0);
  int rc = LBT_ERR_UNSUPPORTED;
#define LBT_GEMM_CASE(BM_, BN_, ST_)                                                        \
  if (bm == BM_ && bn == BN_) {                                                             \
    if (stream_out)                                                                         \
      rc = (mode == 0) ? launch_one<BM_, BN_, 0, ST_, true>(g, grid, tap_bytes, s)          \
                       : launch_one<BM_, BN_, 1, ST_, true>(g, grid, tap_bytes, s);         \
    else                                                                                    \
      rc = (mode == 0) ? launch_one<BM_, BN_, 0, ST_, false>(g, grid, tap_bytes, s)         \
                       : launch_one<BM_, BN_, 1, ST_, false>(g, grid, tap_bytes, s);        \
  }
  if (deep) {
    LBT_GEMM_CASE(128, 128, 3)
    LBT_GEMM_CASE(64, 128, 3)
    LBT_GEMM_CASE(128, 64, 3)
    LBT_GEMM_CASE(64, 64, 4)
  } else {
    LBT_GEMM_CASE(128, 128, 2)
    LBT_GEMM_CASE(64, 128, 2)
    LBT_GEMM_CASE(128, 64, 2)
    LBT_GEMM_CASE(64, 64, 2)
  }
#undef LBT_GEMM_CASE
  if (rc) return rc;
  return LBT_OK;
}

// Tile shape: the largest of 128x128, 64x128 / 128x64, 64x64 that still yields one
// workgroup per compute unit (measured on the ResNet-50 shapes: below that the smaller
// tile wins, above it the larger one does).
void pick_tile(int M, int NJ, int splits, int* bm, int* bn) {
  const int cand[4][2] = {{128, 128}, {64, 128}, {128, 64}, {64, 64}};
  for (int i = 0; i < 4; ++i) {
    const int m = cand[i][0], n = cand[i][1];
    if (M <= 64 && m == 128) continue;
    if (NJ <= 64 && n == 128) continue;
    const long long blocks = (long long)((M + m - 1) / m) * ((NJ + n - 1) / n) * splits;
    *bm = m;
    *bn = n;
    if (blocks >= 256) return;
  }
}

// Direct (no split) product: |sum| <= chunks * 16 * q * q' < 2^31 (q' = the unsigned range
// when the forward product reads unsigned activations).
int run_direct(GemmArgs& g, int mode, int scale_kind, int kid, hipStream_t s) {
  g.steps = (g.chunks + BKC - 1) / BKC;
  g.steps_per_split = g.steps;
  g.scale_kind = scale_kind;
  const long long q = levels(g.bits, false), q2 = levels(g.bits, scale_kind == 4);
  if ((long long)g.chunks * 16 * q * q2 >= (1ll << 31)) return LBT_ERR_OVERFLOW;
  int bm, bn;
  pick_tile(g.M, g.NJ, 1, &bm, &bn);
  return run_gemm(g, mode, bm, bn, 1, kid, s);
}

// defer (may be null): where to leave the sum of the slices for the call's next product
// launch to carry out, instead of launching it here.
int run_splitk(GemmArgs& g, bool x_unsigned, long long true_k, int32_t* acc, int32_t* partial,
               PendingReduce* defer, hipStream_t s) {
  g.scale_kind = x_unsigned ? 2 : 1;
  const SplitPlan plan = plan_split_k(g.M, g.NJ, g.chunks);
  // Every int32 accumulator (one slice of the contraction) must hold its exact sum; the
  // slices are added in 64 bits.  The raw int32 sums can be handed out only if the whole
  // sum fits as well.
  const long long term = (long long)levels(g.bits, false) * levels(g.bits, x_unsigned);
  const long long slice_k = plan.splits == 1 ? true_k
                                             : (true_k < (long long)plan.chunks_per_split * 16
                                                    ? true_k : (long long)plan.chunks_per_split * 16);
  if (slice_k * term >= (1ll << 31)) return LBT_ERR_OVERFLOW;
  const bool wide = true_k * term >= (1ll << 31);
  if (acc && wide) return LBT_ERR_OVERFLOW;
  g.steps = (g.chunks + BKC - 1) / BKC;
  g.steps_per_split = plan.chunks_per_split / BKC;
  int rc;
  if (plan.splits == 1) {
    g.epi = 2;
    g.acc = acc;
    return run_gemm(g, 1, plan.bm, plan.bn, 1, KID_GEMM_DW, s);
  }
  g.epi = 1;
  g.acc = nullptr;
  g.partial = partial;
  lbt_grad_state* const update_st = g.update_st;   // left to the launch that ends the call
  g.update_st = nullptr;
  if ((rc = run_gemm(g, 1, plan.bm, plan.bn, plan.splits, KID_GEMM_DW, s))) return rc;
  const long long n_out = (long long)g.M * g.NJ;
  PendingReduce r{};
  r.partial = partial;
  r.splits = plan.splits;
  r.n = n_out;
  r.out = g.out;
  r.acc = acc;
  r.st = g.st;
  r.sc = g.sc;
  r.scale_kind = g.scale_kind;
  r.bits = g.bits;
  r.many = plan.splits >= 8;
  r.wide = wide;
  long long blocks = (n_out + (r.many ? 63 : 255)) / (r.many ? 64 : 256);
  if (blocks > 4096) blocks = 4096;
  r.blocks = (unsigned)blocks;
  if (defer && !wide) {
    // a carried sum shares the chip with the product that carries it: fewer workgroups, each
    // walking more outputs
    if (r.blocks > 512) r.blocks = 512;
    *defer = r;
    return LBT_OK;
  }
  return launch_pending_reduce(r, update_st, s);
}

}  // namespace

int launch_pending_reduce(const PendingReduce& r, lbt_grad_state* update_st, hipStream_t s) {
  if (!r.blocks) return LBT_OK;
  ProfScope prof(KID_FINALIZE, (double)r.n, s);
#define LBT_REDUCE_CASE(SL_, WIDE_)                                                             \
  LBT_LAUNCH((k_splitk_reduce<SL_, WIDE_>), dim3(r.blocks), dim3(kThreads), 0, s, r, update_st)
  if (r.many && r.wide) LBT_REDUCE_CASE(4, true);
  else if (r.many) LBT_REDUCE_CASE(4, false);
  else if (r.wide) LBT_REDUCE_CASE(1, true);
  else LBT_REDUCE_CASE(1, false);
#undef LBT_REDUCE_CASE
  return LBT_OK;
}

// Measured on the ResNet-50 shapes (every variant of tile and slice count per layer): a dW
// launch costs 11 us or more whatever its size, and each slice adds its int32 tile twice to
// the traffic (written here, read by the reduce).  Long contractions over a small output
// want many slices of 128-wide tiles; short ones (<= 32 K steps) over an output of 256 or
// more 64x64 tiles run fastest unsplit, with no reduce launch at all; in between, 64x64
// tiles cut four ways.
SplitPlan plan_split_k(int M, int NJ, int chunks) {
  SplitPlan p;
  const int iters = (chunks + BKC - 1) / BKC;
  const long long tiles64 = (long long)((M + 63) / 64) * ((NJ + 63) / 64);
  long long splits;
  if (iters <= 32 && tiles64 >= 256) {
    p.bm = (tiles64 >= 512 && M >= 128) ? 128 : 64;
    p.bn = 64;
    splits = 1;
  } else if (iters <= 128 && tiles64 >= 64 && tiles64 <= 256) {
    p.bm = 64;
    p.bn = 64;
    splits = 4;
  } else {
    p.bm = M <= 64 ? 64 : 128;
    p.bn = 128;
    const long long tiles = (long long)((M + p.bm - 1) / p.bm) * ((NJ + p.bn - 1) / p.bn);
    splits = 512 / tiles;           // aim at about two workgroups per compute unit
  }
  if (splits < 1) splits = 1;
  // a slice of at most 1024 K steps keeps the int32 accumulators exact at every bit-width
  // (131072 terms of at most 127 * 127)
  if (splits < (iters + 1023) / 1024) splits = (iters + 1023) / 1024;
  if (splits > iters) splits = iters;
  const long long out_bytes = (long long)M * NJ * 4;
  while (splits > 1 && splits * out_bytes > (48ll << 20)) --splits;
  int per = (int)((iters + splits - 1) / splits) * BKC;
  p.chunks_per_split = per;
  p.splits = (chunks + per - 1) / per;
  p.partial_bytes = p.splits > 1 ? (size_t)p.splits * (size_t)out_bytes : 0;
  return p;
}

int launch_conv_dx(const ConvGeom& c, const uint8_t* w_codes, const uint8_t* g_codes,
                   const lbt_grad_state* st, const OperandScalars* sc, float* dX, int32_t* acc,
                   lbt_grad_state* update_st, const PendingReduce* carry, hipStream_t s) {
  GemmArgs g{};
  if (carry) g.red = *carry;
  fill_geom(g, c);
  g.A = w_codes;
  g.B = g_codes;
  g.groups = c.Kp / kGranule;
  g.inner = c.R * c.S;
  // group count padded so that a K step of 8 chunks covers whole taps or part of one tap
  if (g.groups <= 4) {
    g.gp = g.groups == 3 ? 4 : g.groups;
    g.gp_log2 = g.gp == 1 ? 0 : (g.gp == 2 ? 1 : 2);
  } else {
    g.gp = (g.groups + BKC - 1) / BKC * BKC;
    g.gp_log2 = -1;
  }
  const long long padded = (long long)g.gp * g.inner;
  const long long a_bytes = (long long)c.C * g.groups * g.inner * 16;
  const long long b_bytes = (long long)c.N * g.groups * c.P * c.Q * 16;
  const long long nj = (long long)c.N * c.H * c.W;
  if (nj > 0x7fffffffll || padded > 0x7fffffffll / 16 || a_bytes >= (1ll << 31) ||
      b_bytes >= (1ll << 31))
    return LBT_ERR_UNSUPPORTED;
  g.chunks = (int)padded;
  g.lda = (unsigned)(g.groups * g.inner * 16);
  g.a_bytes = (unsigned)a_bytes;
  g.b_bytes = (unsigned)b_bytes;
  g.M = c.C;
  g.NJ = (int)nj;
  g.epi = 0;
  if (c.R == 1 && c.S == 1 && c.pad == 0 && c.stride > 1) {
    // strided 1x1 layer: only input pixels (p * stride, q * stride) receive a sum.  The
    // product runs over the P x Q grid as an unstrided 1x1 layer and the epilogue fills each
    // stride x stride cell (the corner's value, zeros elsewhere).
    g.H = c.P; g.W = c.Q; g.stride = 1;
    g.NJ = c.N * c.P * c.Q;
    g.epi = 3;
    g.out_h = c.H; g.out_w = c.W; g.up = c.stride;
  }
  g.st = st; g.sc = sc; g.update_st = update_st;
  g.out = dX; g.acc = acc;
  return run_direct(g, 0, 0, KID_GEMM_DX, s);
}

// Forward convolution through the same gather kernel: rows are output channels, columns
// output pixels (n, p, q), the contraction walks (tap, input-channel group).
//   A = W codes [K][R*S][Cp/16][16], B = X codes [N][Cp/16][H*W][16]; out/acc [N][K][P][Q].
int launch_conv_fwd(const ConvGeom& c, const uint8_t* w_codes, const uint8_t* x_codes,
                    const OperandScalars* sc, int x_unsigned, float* Y, int32_t* acc,
                    int32_t* status_out, hipStream_t s) {
  GemmArgs g{};
  g.N = c.N; g.R = c.R; g.S = c.S; g.stride = c.stride; g.pad = c.pad; g.bits = c.bits;
  g.C = c.K;            // rows of the output
  g.K = c.C;            // contraction channels
  g.H = c.P; g.W = c.Q;  // the columns' image: the output
  g.P = c.H; g.Q = c.W;  // the gathered image: the input
  g.fwd = 1;
  g.A = w_codes;
  g.B = x_codes;
  g.groups = (int)(round_up(c.C, kGranule) / kGranule);
  g.inner = c.R * c.S;
  if (g.groups <= 4) {
    g.gp = g.groups == 3 ? 4 : g.groups;
    g.gp_log2 = g.gp == 1 ? 0 : (g.gp == 2 ? 1 : 2);
  } else {
    g.gp = (g.groups + BKC - 1) / BKC * BKC;
    g.gp_log2 = -1;
  }
  const long long padded = (long long)g.gp * g.inner;
  const long long a_bytes = (long long)c.K * g.groups * g.inner * 16;
  const long long b_bytes = (long long)c.N * g.groups * c.H * c.W * 16;
  const long long nj = (long long)c.N * c.P * c.Q;
  if (nj > 0x7fffffffll || padded > 0x7fffffffll / 16 || a_bytes >= (1ll << 31) ||
      b_bytes >= (1ll << 31))
    return LBT_ERR_UNSUPPORTED;
  g.chunks = (int)padded;
  g.lda = (unsigned)(g.groups * g.inner * 16);
  g.a_bytes = (unsigned)a_bytes;
  g.b_bytes = (unsigned)b_bytes;
  g.M = c.K;
  g.NJ = (int)nj;
  g.epi = 0;
  g.sc = sc;
  g.status_out = status_out;
  g.out = Y; g.acc = acc;
  return run_direct(g, 0, x_unsigned ? 4 : 3, KID_GEMM_FWD, s);
}

// Forward product of a linear layer, Y[M][N_out] = X . W: rows of X against rows of W^T.
//   A = X codes [M][Kin_p/16][16], B = W codes [N_out][Kin_p/16][16].
int launch_linear_fwd(int M, int K_in, int N_out, int bits, const uint8_t* x_codes,
                      const uint8_t* w_codes, const OperandScalars* sc, int x_unsigned, float* Y,
                      int32_t* acc, int32_t* status_out, hipStream_t s) {
  GemmArgs g{};
  g.N = M; g.C = N_out; g.K = K_in; g.H = g.W = g.P = g.Q = g.R = g.S = 1; g.stride = 1; g.pad = 0;
  g.bits = bits;
  g.A = x_codes;
  g.B = w_codes;
  g.groups = (int)(round_up(K_in, kGranule) / kGranule);
  g.inner = 1;
  g.chunks = g.groups;
  if ((long long)g.chunks * 16 * M >= (1ll << 31) || (long long)g.chunks * 16 * N_out >= (1ll << 31))
    return LBT_ERR_UNSUPPORTED;
  g.lda = (unsigned)(g.chunks * 16);
  g.a_bytes = g.lda * (unsigned)M;
  g.b_bytes = g.lda * (unsigned)N_out;
  g.M = M;
  g.NJ = N_out;
  g.epi = 2;
  g.sc = sc;
  g.status_out = status_out;
  g.out = Y; g.acc = acc;
  return run_direct(g, 1, x_unsigned ? 4 : 3, KID_GEMM_FWD, s);
}

int launch_conv_dw(const ConvGeom& c, const uint8_t* g_codes, const uint8_t* x_codes,
                   const lbt_grad_state* st, const OperandScalars* sc, int x_unsigned, float* dW,
                   int32_t* acc, int32_t* partial, lbt_grad_state* update_st, PendingReduce* defer,
                   hipStream_t s) {
  GemmArgs g{};
  fill_geom(g, c);
  g.A = g_codes;
  g.B = x_codes;
  g.groups = c.Np / kGranule;
  g.inner = c.P * c.Q;
  const long long chunks = (long long)g.inner * g.groups;
  const long long a_bytes = chunks * 16 * c.K;
  const long long b_bytes = (long long)c.C * g.groups * c.H * c.W * 16;
  if (chunks > 0x7fffffffll / 16 || a_bytes >= (1ll << 31) || b_bytes >= (1ll << 31))
    return LBT_ERR_UNSUPPORTED;
  g.chunks = (int)chunks;
  g.lda = (unsigned)(chunks * 16);
  g.a_bytes = (unsigned)a_bytes;
  g.b_bytes = (unsigned)b_bytes;
  g.M = c.K;
  g.NJ = c.C * c.R * c.S;
  g.st = st; g.sc = sc; g.update_st = update_st;
  g.out = dW;
  return run_splitk(g, x_unsigned != 0, (long long)c.N * c.P * c.Q, acc, partial, defer, s);
}

// Linear layer (1x1 image): operands swap roles so that the row-major outputs
// dX[M][K_in] and dW[K_in][N_out] have their contiguous axis on the lanes.
int launch_linear_dx(const ConvGeom& c, const uint8_t* w_codes, const uint8_t* g_codes,
                     const lbt_grad_state* st, const OperandScalars* sc, float* dX, int32_t* acc,
                     lbt_grad_state* update_st, const PendingReduce* carry, hipStream_t s) {
  GemmArgs g{};
  if (carry) g.red = *carry;
  fill_geom(g, c);
  g.A = g_codes;   // [N][Kp/16][16] gradient rows
  g.B = w_codes;   // [C][Kp/16][16] weight rows, read with the (c,r,s)-row gather on a 1x1 image
  g.groups = c.Kp / kGranule;
  g.inner = 1;
  g.chunks = g.groups;
  if ((long long)g.chunks * 16 * c.N >= (1ll << 31) || (long long)g.chunks * 16 * c.C >= (1ll << 31))
    return LBT_ERR_UNSUPPORTED;
  g.lda = (unsigned)(g.chunks * 16);
  g.a_bytes = g.lda * (unsigned)c.N;
  g.b_bytes = g.lda * (unsigned)c.C;
  g.M = c.N;
  g.NJ = c.C;
  g.epi = 2;
  g.st = st; g.sc = sc; g.update_st = update_st;
  g.out = dX; g.acc = acc;
  return run_direct(g, 1, 0, KID_GEMM_DX, s);
}

int launch_linear_dw(const ConvGeom& c, const uint8_t* g_codes, const uint8_t* x_codes,
                     const lbt_grad_state* st, const OperandScalars* sc, int x_unsigned, float* dW,
                     int32_t* acc, int32_t* partial, lbt_grad_state* update_st, PendingReduce* defer,
                     hipStream_t s) {
  GemmArgs g{};
  fill_geom(g, c);
  g.A = x_codes;   // [C][Np/16][16] activation rows
  g.B = g_codes;   // [K][Np/16][16] gradient rows
  g.groups = c.Np / kGranule;
  g.inner = 1;
  g.chunks = g.groups;
  if ((long long)g.chunks * 16 * c.C >= (1ll << 31) || (long long)g.chunks * 16 * c.K >= (1ll << 31))
    return LBT_ERR_UNSUPPORTED;
  g.lda = (unsigned)(g.chunks * 16);
  g.a_bytes = g.lda * (unsigned)c.C;
  g.b_bytes = g.lda * (unsigned)c.K;
  g.M = c.C;
  g.NJ = c.K;
  g.st = st; g.sc = sc; g.update_st = update_st;
  g.out = dW;
  return run_splitk(g, x_unsigned != 0, (long long)c.N, acc, partial, defer, s);
}

}  // namespace lbt
