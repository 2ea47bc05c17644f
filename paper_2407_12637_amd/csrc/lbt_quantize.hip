// Quantizer kernels: tensor maximum, uniform b-bit quantizer (Eq. 1-4 of the paper, b = 2..8,
// 4 by default) with nearest or stochastic rounding, clip-out count (Sec. 3.3, Alg. 1 step 5),
// the flat code format of the C ABI (nibbles up to 4 bits, bytes above), byte-per-code granules
// in the GEMM layouts, and the one-thread clipping-factor update (Eq. 15-16).
//
// Arithmetic contract (decides integer codes, so it is fixed to the last bit):
//   c      = (float)(gamma * (double)g_max)
//   inv_s  = (float)((double)q / (double)c),  q = 2^(b-1) - 1 (signed) or 2^b - 1 (unsigned)
//   t      = clip(x) * inv_s                  -- one fp32 multiply, no FMA
//   code   = rint(t)  |  (floor(t * 2^16) + r16) >> 16   (16 fractional bits)
//   code   = clamp(code, -q or 0, q)
//
// A tensor is swept twice: k_absmax3 takes the maxima of up to three tensors in one
// launch (one partial maximum per workgroup, no atomics), then a quantizer kernel
// re-reduces those partials in its prologue and streams the tensor once more.  (With the
// single-sweep flag the interval comes from the previous tensor's maximum instead and this
// tensor's maximum is gathered during the one sweep.)  The clip-out count travels in one
// 64-bit atomic per workgroup (count in the low 40 bits, arrival ticket above) on one of
// 16 counters in the workspace, whose sums meet in a word of the layer state; k_absmax3
// zeroes the counters and the last workgroup clears the word, so no scratch memory has to
// be zero-initialised by the caller.
#include "lbt_internal.h"

namespace lbt {
namespace {

constexpr int kThreads = 256;
constexpr uint32_t kInfBits = 0x7f800000u;
constexpr unsigned long long kTicket = 1ull << 40;
constexpr unsigned long long kCountMask = kTicket - 1;

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
  // each round needs both halves of two 32 x 32 -> 64 bit products: one multiply
  // instruction apiece when written as a 64-bit product
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const unsigned long long pa = (unsigned long long)kMulA * c0;
    const unsigned long long pb = (unsigned long long)kMulB * c2;
    c0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
    c1 = (uint32_t)pb;
    c2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
    c3 = (uint32_t)pa;
    k0 += kWeylA;
    k1 += kWeylB;
  }
  return Philox4{{c0, c1, c2, c3}};
}

// Random words of the block of 8 elements number `blk` (= flat element index / 8).
__device__ __forceinline__ Philox4 philox_block(unsigned long long blk, unsigned long long step,
                                                unsigned long long seed) {
  return philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), (uint32_t)step,
                       (uint32_t)(step >> 32), (uint32_t)seed, (uint32_t)(seed >> 32));
}

// 16 random bits for flat element e: lane e%8 of block e/8.
__device__ __forceinline__ uint32_t r16_of(const Philox4& p, uint32_t lane) {
  return (p.w[lane >> 1] >> ((lane & 1u) * 16u)) & 0xFFFFu;
}

// floor(x) as an integer in one instruction (the conversion that rounds towards minus infinity)
__device__ __forceinline__ int floor_to_int(float x) {
  int r;
  asm("v_cvt_flr_i32_f32_e32 %0, %1" : "=v"(r) : "v"(x));
  return r;
}

__device__ __forceinline__ int clamp_code(int r, const QConst& k) {
  int m;
  asm("v_med3_i32 %0, %1, %2, %3" : "=v"(m) : "v"(r), "v"(k.kmin), "v"(k.q));
  return m;
}

// |x_n| <= q (1 + 2^-23) < q + 1/2, so the nearest integer is already inside [-q, q]
__device__ __forceinline__ int code_nearest(float v, const QConst& k) {
  return (int)rintf(normalised(v, k));
}

__device__ __forceinline__ int code_stochastic(float v, const QConst& k, uint32_t r16) {
  // x_n in units of 2^-16 (exact scaling), truncated downwards, plus 16 random bits;
  // x_n may exceed q by an ulp and floor(-q - ulp) is -q - 1: the code is clamped
  const int fixed = floor_to_int(__fmul_rn(normalised(v, k), 65536.0f)) + (int)r16;
  return clamp_code(fixed >> 16, k);  // arithmetic shift: floor division
}

// MODE 0: signed nearest, 1: unsigned nearest, 2: signed nearest + count,
//      3: signed stochastic + count   (2 and 3 are the gradient quantizer)
template <int MODE>
__device__ __forceinline__ int quantize_one(float v, const QConst& qc, const Philox4& rnd,
                                            uint32_t lane, uint32_t& cnt) {
  int k;
  if (MODE == 3) k = code_stochastic(v, qc, r16_of(rnd, lane));
  else k = code_nearest(v, qc);
  if (MODE >= 2) cnt += (fabsf(v) > qc.c) ? 1u : 0u;
  return k;
}

// Eight consecutive elements (one generator block) -> two words of four code bytes each.
// ok0 / ok1: whether the first / second four elements belong to the tile (a half that does
// not gives a zero word and is not counted; its values are whatever a harmless load of valid
// memory returned).  The clip-out count is taken per WAVE: each compare's lane mask is counted
// by the scalar unit, so cnt_wave holds the same running total in every lane.
template <int MODE>
__device__ __forceinline__ void quantize8(const float v[8], bool ok0, bool ok1, const QConst& qc,
                                          const Philox4& rnd, uint32_t& w0, uint32_t& w1,
                                          uint32_t& cnt_wave) {
  w0 = 0;
  w1 = 0;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    int k;
    if (MODE == 3) k = code_stochastic(v[u], qc, r16_of(rnd, u));
    else k = code_nearest(v[u], qc);
    const uint32_t byte = ((uint32_t)k & 0xFFu) << (8 * (u & 3));
    if (u < 4) w0 |= byte; else w1 |= byte;
  }
  w0 = ok0 ? w0 : 0u;
  w1 = ok1 ? w1 : 0u;
  if (MODE >= 2) {
    const unsigned long long m0 = __ballot(ok0), m1 = __ballot(ok1);
#pragma unroll
    for (int u = 0; u < 8; ++u)
      cnt_wave += (uint32_t)__popcll(__ballot(fabsf(v[u]) > qc.c) & (u < 4 ? m0 : m1));
  }
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

// Block-wide reductions; every thread receives the result.
__device__ __forceinline__ uint32_t block_max(uint32_t m) {
  __shared__ uint32_t part[16];
  const int nw = blockDim.x >> 6;
  m = wave_max(m);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
  __syncthreads();
  uint32_t t = part[0];
  for (int i = 1; i < nw; ++i) t = max(t, part[i]);
  return t;
}

__device__ __forceinline__ uint32_t block_sum(uint32_t v) {
  __shared__ uint32_t part[16];
  const int nw = blockDim.x >> 6;
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
  __syncthreads();
  uint32_t t = 0;
  for (int i = 0; i < nw; ++i) t += part[i];
  return t;
}

// Maximum of column `col` of the partial maxima left by k_absmax3.
__device__ __forceinline__ uint32_t reduce_partials(const uint32_t* pmax, int nblocks, int col) {
  uint32_t m = 0;
  for (int i = threadIdx.x; i < nblocks; i += blockDim.x) m = max(m, pmax[i * 4 + col]);
  return block_max(m);
}

// ---------------------------------------------------------------------------
// Gradient quantizer prologue / epilogue shared by the flat and the tiled kernels
// ---------------------------------------------------------------------------
struct GradSetup {
  float gmax, c;
  int status;
  int bits;
  bool hindsight;
  bool fused_update;  // the workgroup that publishes the statistics also applies Alg. 1
};

// hindsight: the interval comes from the maximum the previous call left in the state; this
// tensor's own maximum is gathered during the sweep (grad_finish).
__device__ __forceinline__ GradSetup grad_setup(const lbt_grad_state* st, const uint32_t* pmax,
                                                int nblocks, int bits, bool hindsight = false) {
  GradSetup g;
  g.bits = bits;
  g.hindsight = hindsight;
  g.fused_update = false;
  uint32_t mx;
  if (hindsight) {
    mx = __float_as_uint(st->gmax) & 0x7fffffffu;
    if (mx >= kInfBits) mx = 0;      // unusable: treated like "no previous maximum"
  } else {
    mx = reduce_partials(pmax, nblocks, 0);
  }
  g.gmax = __uint_as_float(mx);
  g.c = 0.0f;
  if (mx >= kInfBits) g.status = LBT_STATUS_NONFINITE;
  else if (mx == 0) g.status = LBT_STATUS_ZERO_GRAD;
  else {
    g.status = LBT_STATUS_OK;
    g.c = (float)__dmul_rn(st->gamma, (double)g.gmax);
    // an interval too small to normalise by (subnormal-scale gradients) counts as all-zero
    if (!interval_usable(g.c, levels(bits, false))) {
      g.status = LBT_STATUS_ZERO_GRAD;
      g.c = 0.0f;
    }
  }
  return g;
}

// One atomic per workgroup carries the clip-out count and the arrival ticket.  Workgroup
// `id` reports to counter id % 16 (atomics on one address complete at about 16 ns each;
// with thousands of workgroups one counter would be the longest chain of the kernel); the
// workgroup that completes a counter forwards its sum to the state's word, and the one
// that completes that word publishes the statistics and clears it.  The 16 counters are
// zeroed by k_absmax3, which runs before every gradient quantizer.
__device__ __forceinline__ void grad_finish(lbt_grad_state* st, const GradSetup& g, uint32_t cnt,
                                            unsigned long long n_total, unsigned nblk, unsigned id,
                                            unsigned long long* slots, uint32_t my_max = 0) {
  const uint32_t tot = block_sum(cnt);
  uint32_t blk_max = 0;
  if (g.hindsight) blk_max = block_max(my_max);
  if (threadIdx.x == 0) {
    const unsigned slot = id % kTicketSlots;
    const unsigned in_slot = (nblk - slot + kTicketSlots - 1) / kTicketSlots;
    uint32_t* const max_slots = reinterpret_cast<uint32_t*>(slots + kTicketSlots);
    // Single-sweep mode: a workgroup's maximum must be in its counter before the ticket that
    // announces it.  Both are device-scope atomics that return a value, executed at the one
    // point of coherence of the device; the ticket is made to depend on the value the first
    // atomic returned, so it cannot be issued before that atomic has been performed.  (The
    // textbook form, an agent-scope release fence between the two and an acquire fence on the
    // collector's side, was measured: the fence writes the workgroup's freshly stored codes
    // back through L2 before the ticket may go out, one workgroup after the other, and the
    // ResNet-50 step in this mode went from 5.06 to 7.84 ms.  The dependency carries no data
    // other than the atomics' own, which is all this exchange needs.)
    unsigned long long carry = 0;
    if (g.hindsight) {
      uint32_t seen = atomicMax(&max_slots[slot], blk_max), copy = seen;
      asm volatile("" : "+v"(copy));
      carry = seen ^ copy;
    }
    const unsigned long long old = atomicAdd(&slots[slot], kTicket + tot + carry);
    if ((old >> 40) != in_slot - 1) return;
    const unsigned long long sub = (old + tot) & kCountMask;
    const unsigned n_slots = nblk < (unsigned)kTicketSlots ? nblk : (unsigned)kTicketSlots;
    carry = 0;
    if (g.hindsight) {
      const uint32_t slot_max = atomicMax(&max_slots[slot], 0u);   // every member has reported
      uint32_t seen = atomicMax(&st->sync_max, slot_max), copy = seen;
      asm volatile("" : "+v"(copy));
      carry = seen ^ copy;
    }
    const unsigned long long old2 =
        atomicAdd(reinterpret_cast<unsigned long long*>(&st->sync_word), kTicket + sub + carry);
    if ((old2 >> 40) == n_slots - 1) {
      int status = g.status;
      st->n_out = (old2 + sub) & kCountMask;
      st->n_total = n_total;
      if (g.hindsight) {
        const uint32_t now = atomicMax(&st->sync_max, 0u);
        if (now >= kInfBits) status = LBT_STATUS_NONFINITE;   // and the recorded maximum stays
        else st->gmax = __uint_as_float(now);
        st->sync_max = 0;
      } else {
        st->gmax = g.gmax;
      }
      st->clip = g.c;
      st->scale = (g.c > 0.0f) ? (float)((double)g.c / (double)levels(g.bits, false)) : 0.0f;
      st->bits = g.bits;
      // k_absmax3 has reset the status to OK; an operand quantizer of the same launch
      // may already have flagged a non-finite operand, which must stay
      if (status != LBT_STATUS_OK) atomicCAS(&st->status, LBT_STATUS_OK, status);
      else if (g.fused_update) interval_update_with(st, (old2 + sub) & kCountMask, n_total);
      st->sync_word = 0;
    }
  }
}

// Operand clip value: the caller's, or the tensor maximum from the partials.
__device__ __forceinline__ float operand_setup(float c_given, const uint32_t* pmax, int nblocks,
                                               int col, bool is_unsigned, float* c_out,
                                               uint32_t* bad_out, lbt_grad_state* st,
                                               float* clip_scale_out, bool first_block, int bits) {
  float c = c_given;
  bool bad = false;
  if (!(c > 0.0f)) {
    const uint32_t bits = reduce_partials(pmax, nblocks, col);
    if (bits >= kInfBits) { bad = true; c = 0.0f; }
    else c = __uint_as_float(bits);
  }
  if (first_block && threadIdx.x == 0) {
    if (c_out) *c_out = c;
    if (bad_out) *bad_out = bad ? 1u : 0u;
    if (bad && st) st->status = LBT_STATUS_NONFINITE;
    if (clip_scale_out) {
      clip_scale_out[0] = c;
      clip_scale_out[1] = (c > 0.0f) ? (float)((double)c / (double)levels(bits, is_unsigned)) : 0.0f;
    }
  }
  return c;
}

// ---------------------------------------------------------------------------
// one-thread kernels
// ---------------------------------------------------------------------------
__global__ void k_update_interval(lbt_grad_state* st) { interval_update(st); }

__global__ void k_state_set(lbt_grad_state* st, lbt_grad_state v) { *st = v; }

// ---------------------------------------------------------------------------
// tensor maxima of up to three tensors in one launch: max |x| (use_abs) or
// max(x, 0), as unsigned compares of fp32 bit patterns (monotone for
// non-negative floats; NaN/Inf sort on top).  Workgroup i writes its partial
// maximum to pmax[i][tensor] and zeros to the other columns.
// ---------------------------------------------------------------------------
struct MaxSeg {
  const float* p;
  long long n;
  int use_abs;
  int first_block;  // first workgroup of this tensor
};

// The tensors are read with streaming (non-temporal) loads.  Measured on the ResNet-50 sweep:
// the maximum sweep then runs at 5.7 TB/s instead of 4.8; the quantizer's second sweep loses
// the few cache hits it had (+0.1 ms per step against -0.16 ms here), at every tensor size.
__global__ __launch_bounds__(kThreads) void k_absmax3(MaxSeg s0, MaxSeg s1, MaxSeg s2,
                                                       long long per_block, uint32_t* pmax,
                                                       unsigned long long* tickets,
                                                       lbt_grad_state* st,
                                                       const OperandScalars* kept, int kept_mask) {
  const int blk = blockIdx.x;
  // every quantizer launch that follows reports into a fresh status and fresh counters;
  // operands quantized by an earlier call (kept: bit 0 of the mask X, bit 1 W) bring the
  // non-finite flag of that call with them
  if (blk == 0) {
    if (st && threadIdx.x == 0) {
      const bool bad = kept && (((kept_mask & 1) && kept->bad_x) || ((kept_mask & 2) && kept->bad_w));
      st->status = bad ? LBT_STATUS_NONFINITE : LBT_STATUS_OK;
    }
    if (threadIdx.x < kTicketSlots) {
      tickets[threadIdx.x] = 0ull;
      reinterpret_cast<uint32_t*>(tickets + kTicketSlots)[threadIdx.x] = 0u;
    }
  }
  int t = 0;
  MaxSeg s = s0;
  if (blk >= s2.first_block) { s = s2; t = 2; }
  else if (blk >= s1.first_block) { s = s1; t = 1; }
  const long long start = (long long)(blk - s.first_block) * per_block;
  const long long count = min(per_block, s.n - start);
  const float4* p4 = reinterpret_cast<const float4*>(s.p + start);
  const long long n4 = count / 4;
  // Two running maxima, three operations per element: of the magnitudes' bit patterns (unsigned
  // compare: NaN / Inf of either sign end up on top) and of the bit patterns as signed integers
  // (= max(x, 0) for finite values: negatives are negative integers).
  uint32_t mag = 0;
  int pos = 0;
  auto take = [&](const float4& v) __attribute__((always_inline)) {
    const uint32_t b0 = __float_as_uint(v.x), b1 = __float_as_uint(v.y), b2 = __float_as_uint(v.z),
                   b3 = __float_as_uint(v.w);
    mag = max(max(mag, b0 & 0x7fffffffu), max(b1 & 0x7fffffffu, max(b2 & 0x7fffffffu, b3 & 0x7fffffffu)));
    pos = max(max(pos, (int)b0), max((int)b1, max((int)b2, (int)b3)));
  };
  long long i = threadIdx.x;
  for (; i + 7 * kThreads < n4; i += 8 * kThreads) {
    float4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      typedef float f4n __attribute__((ext_vector_type(4)));
      const f4n t = __builtin_nontemporal_load(reinterpret_cast<const f4n*>(p4 + i + u * kThreads));
      v[u] = make_float4(t.x, t.y, t.z, t.w);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) take(v[u]);
  }
  for (; i < n4; i += kThreads) take(p4[i]);
  if ((long long)threadIdx.x < count - n4 * 4) {
    const float x = s.p[start + n4 * 4 + threadIdx.x];
    take(make_float4(x, 0.0f, 0.0f, 0.0f));
  }
  // max |x|, or max(x, 0) with a non-finite value of either sign kept visible
  uint32_t m = (s.use_abs || mag >= kInfBits) ? mag : (uint32_t)pos;
  m = block_max(m);
  if (threadIdx.x < 4) pmax[blk * 4 + threadIdx.x] = ((int)threadIdx.x == t) ? m : 0u;
}

// ---------------------------------------------------------------------------
// Gradient through an operand quantizer (Sec. 3.1 learns the clip values of weights and
// activations; Eq. 1-4 with the rounding passed straight through):
//   grad_x = grad_q inside the interval (lo < x < c), 0 outside;
//   grad_c = sum grad_q * d,  d = (round(u) - u) / q inside, +1 for x >= c, -1 for x <= -c
//            (signed), 0 for x <= 0 (unsigned);  u = clip(x) * (q / c) as the quantizer takes it.
// Products and sums in fp64 (of grad_q * q d; one division by q per workgroup, none per
// element); one partial sum per workgroup, added in a fixed order by
// k_ste_finish, so the result does not depend on how the workgroups were scheduled.
// ---------------------------------------------------------------------------
// grad_x may be null, and may be grad_q itself (every element is read before it is written).
// Streaming (non-temporal) loads and stores: nothing is read twice, and the masked gradient
// leaves for HBM at once instead of being written back under the next kernel (measured on the
// ResNet-50 sweep with this pass after every layer: 7.19 -> 6.85 ms per step).
__global__ __launch_bounds__(kThreads) void k_ste_backward(const float* x, const float* grad_q,
                                                            long long n, float c, int is_unsigned,
                                                            int bits, float* grad_x, double* partial) {
  const QConst k = make_qconst(c, is_unsigned != 0, bits);
  const float below = is_unsigned ? 0.0f : -(float)k.q;
  const float4* x4 = reinterpret_cast<const float4*>(x);
  const float4* g4 = reinterpret_cast<const float4*>(grad_q);
  float4* o4 = reinterpret_cast<float4*>(grad_x);
  const long long n4 = n >> 2, stride = (long long)gridDim.x * kThreads;
  double acc = 0.0;
  typedef float f4n __attribute__((ext_vector_type(4)));
  auto ld = [](const float4* p) __attribute__((always_inline)) {
    const f4n t = __builtin_nontemporal_load(reinterpret_cast<const f4n*>(p));
    return make_float4(t.x, t.y, t.z, t.w);
  };
  auto stv = [](float4* p, const float4& v) __attribute__((always_inline)) {
    f4n t; t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
    __builtin_nontemporal_store(t, reinterpret_cast<f4n*>(p));
  };
  long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
  // two float4 pairs per thread in flight
  for (; i + stride < n4; i += 2 * stride) {
    const float4 xa = ld(x4 + i), ga = ld(g4 + i), xb = ld(x4 + i + stride), gb = ld(g4 + i + stride);
    float4 oa, ob;
    oa.x = ste_one(xa.x, ga.x, k, below, acc); oa.y = ste_one(xa.y, ga.y, k, below, acc);
    oa.z = ste_one(xa.z, ga.z, k, below, acc); oa.w = ste_one(xa.w, ga.w, k, below, acc);
    ob.x = ste_one(xb.x, gb.x, k, below, acc); ob.y = ste_one(xb.y, gb.y, k, below, acc);
    ob.z = ste_one(xb.z, gb.z, k, below, acc); ob.w = ste_one(xb.w, gb.w, k, below, acc);
    if (grad_x) { stv(o4 + i, oa); stv(o4 + i + stride, ob); }
  }
  if (i < n4) {
    const float4 xa = x4[i], ga = g4[i];
    float4 oa;
    oa.x = ste_one(xa.x, ga.x, k, below, acc); oa.y = ste_one(xa.y, ga.y, k, below, acc);
    oa.z = ste_one(xa.z, ga.z, k, below, acc); oa.w = ste_one(xa.w, ga.w, k, below, acc);
    if (grad_x) o4[i] = oa;
  }
  if (blockIdx.x == 0 && (long long)threadIdx.x < n - n4 * 4) {   // the last n % 4 elements
    const long long e = n4 * 4 + threadIdx.x;
    const float o = ste_one(x[e], grad_q[e], k, below, acc);
    if (grad_x) grad_x[e] = o;
  }
  const double tot = block_sum_f64(acc);
  if (partial && threadIdx.x == 0) partial[blockIdx.x] = tot / (double)k.q;
}

// Workgroup j adds the partial sums of pass j (one or two passes per launch).
struct SteSums {
  const double* partial[2];
  int nblocks[2];
  float* grad_c[2];
};
__global__ __launch_bounds__(kThreads) void k_ste_finish(const SteSums f) {
  const int j = blockIdx.x;
  const double* partial = j ? f.partial[1] : f.partial[0];
  const int nblocks = j ? f.nblocks[1] : f.nblocks[0];
  double acc = 0.0;
  for (int i = threadIdx.x; i < nblocks; i += kThreads) acc += partial[i];
  const double tot = block_sum_f64(acc);
  if (threadIdx.x == 0) *(j ? f.grad_c[1] : f.grad_c[0]) = (float)tot;
}

// Largest |v| of eight values as an fp32 bit pattern (NaN/Inf sort on top).
__device__ __forceinline__ uint32_t max_abs_bits8(const float v[8]) {
  uint32_t m = 0;
#pragma unroll
  for (int u = 0; u < 8; ++u) m = max(m, __float_as_uint(v[u]) & 0x7fffffffu);
  return m;
}

// ---------------------------------------------------------------------------
// flat quantizer (C-ABI code format): 8 consecutive elements per thread -> one
// 32-bit word of codes
// ---------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(kThreads) void k_quantize_flat(
    const float* __restrict__ x, long long n, float c_given, const uint32_t* pmax, int nblocks,
    unsigned long long* tickets, lbt_grad_state* st, unsigned long long seed, uint8_t* __restrict__ codes, float* c_out,
    float* clip_scale_out, int hindsight, int fused_update, int bits) {
  constexpr bool kGrad = (MODE >= 2);
  GradSetup gs{};
  float c;
  if (kGrad) {
    gs = grad_setup(st, pmax, nblocks, bits, hindsight != 0);
    gs.fused_update = fused_update != 0;
    c = gs.c;
  } else {
    c = operand_setup(c_given, pmax, nblocks, 1, MODE == 1, c_out, nullptr, nullptr, clip_scale_out,
                      blockIdx.x == 0, bits);
  }
  const QConst qc = make_qconst(c, MODE == 1, bits);
  const bool bytes = bits > 4;   // one byte per code instead of one nibble
  const bool live = qc.live;
  const unsigned long long step = (MODE == 3) ? st->step : 0ull;
  const long long groups = (n + 7) / 8;
  const long long stride = (long long)gridDim.x * kThreads;
  uint32_t cnt_wave = 0, seen_max = 0;
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
    if (kGrad && gs.hindsight) seen_max = max(seen_max, max_abs_bits8(v));
    // byte format: elements 0-3 in lo, 4-7 in hi; nibble format: the low nibbles of those
    // bytes.  Elements past the end were loaded as 0.0: code 0, never counted.
    uint32_t word = 0, lo = 0, hi = 0;
    if (live) {
      Philox4 rnd{};
      if (MODE == 3) rnd = philox_block((unsigned long long)gi, step, seed);
      quantize8<MODE>(v, true, true, qc, rnd, lo, hi, cnt_wave);
      // gather the low nibble of each byte: 0x0d0c0b0a -> 0xdcba
      const uint32_t l4 = lo & 0x0F0F0F0Fu, h4 = hi & 0x0F0F0F0Fu;
      const uint32_t l2 = (l4 | (l4 >> 4)) & 0x00FF00FFu, h2 = (h4 | (h4 >> 4)) & 0x00FF00FFu;
      word = ((l2 | (l2 >> 8)) & 0xFFFFu) | (((h2 | (h2 >> 8)) & 0xFFFFu) << 16);
    }
    if (bytes) {
      if (valid == 8) {
        reinterpret_cast<uint2*>(codes)[gi] = make_uint2(lo, hi);
      } else {
        for (int j = 0; j < valid; ++j)
          codes[gi * 8 + j] = (uint8_t)((j < 4 ? lo >> (8 * j) : hi >> (8 * (j - 4))) & 0xFFu);
      }
    } else if (valid == 8) {
      reinterpret_cast<uint32_t*>(codes)[gi] = word;
    } else {
      const int nbytes = (valid + 1) / 2;
      for (int j = 0; j < nbytes; ++j) codes[gi * 4 + j] = (uint8_t)(word >> (8 * j));
    }
  }
  if (kGrad) grad_finish(st, gs, (threadIdx.x & 63) == 0 ? cnt_wave : 0u, (unsigned long long)n, gridDim.x,
                         blockIdx.x, tickets, seen_max);
}

// ---------------------------------------------------------------------------
// quantize + re-layout of T[A][B][L] (L contiguous) into the GEMM layouts
//   out_b [A][BG][L][16]  sixteen consecutive b per 16-byte granule (BG = Bp/16)
//   out_a [B][AG][L][16]  sixteen consecutive a per 16-byte granule (AG = Ap/16);
//         [B][L][AG][16] when a_lmajor is set (the dX kernel reads weights tap by tap);
//         likewise out_b as [A][L][BG][16] when b_lmajor is set (forward product)
// zero padded in the last granule.  A workgroup owns a 16(a) x 16(b) x TL(l)
// tile: it quantizes into LDS (one byte per code, [a][b][l]), then each thread
// gathers the sixteen codes of one granule and stores its 16 bytes; consecutive
// threads store consecutive l, so the stores are contiguous.
// ---------------------------------------------------------------------------
struct TileArgs {
  const float* x;
  int A, B, L;
  int AG, BG;
  // clip value: c_given if > 0, else *c_ptr if c_ptr, else the tensor maximum (pmax)
  float c_given;
  const float* c_ptr;
  const uint32_t* pmax;  // partial maxima left by k_absmax3
  int nblocks;
  int pmax_col;
  unsigned long long* tickets;  // gradient only: arrival counters and running maxima
  lbt_grad_state* st;
  unsigned long long seed;
  float* c_out;
  uint32_t* bad_out;
  uint4* out_b;
  uint4* out_a;
  int a_lmajor;
  int b_lmajor;   // out_b as [A][L][BG][16]
  int hindsight;  // gradient only: interval from the previous call's maximum
  int bits;       // b of Eq. (2)/(3)
  int is_unsigned;  // operand only: Eq. (3) instead of Eq. (2)
};

// Phase B: gather granules out of the LDS tile.  `pitch` = bytes per (a,b) row.  A granule
// is sixteen int8 codes (16 bytes), element j in byte j.
// Byte-wise version (any tile length): one LDS byte read per code.
__device__ __forceinline__ void store_granules(const TileArgs& t, const uint8_t* tile, int pitch,
                                               int tl, int a0, int b0, int l0) {
  const int n_items = 16 * tl;
  if (t.out_b) {
    const int bg = b0 >> 4;
    for (int it = threadIdx.x; it < n_items; it += blockDim.x) {
      const int a = it / tl, l = it - a * tl;
      if (a0 + a >= t.A || l0 + l >= t.L) continue;
      uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
      for (int j = 0; j < 16; ++j) w[j >> 2] |= (uint32_t)tile[(a * 16 + j) * pitch + l] << (8 * (j & 3));
      const long long o = t.b_lmajor ? ((long long)(a0 + a) * t.L + l0 + l) * t.BG + bg
                                     : ((long long)(a0 + a) * t.BG + bg) * t.L + l0 + l;
      t.out_b[o] = make_uint4(w[0], w[1], w[2], w[3]);
    }
  }
  if (t.out_a) {
    const int ag = a0 >> 4;
    for (int it = threadIdx.x; it < n_items; it += blockDim.x) {
      const int b = it / tl, l = it - b * tl;
      if (b0 + b >= t.B || l0 + l >= t.L) continue;
      uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
      for (int j = 0; j < 16; ++j) w[j >> 2] |= (uint32_t)tile[(j * 16 + b) * pitch + l] << (8 * (j & 3));
      const long long o = t.a_lmajor ? ((long long)(b0 + b) * t.L + l0 + l) * t.AG + ag
                                     : ((long long)(b0 + b) * t.AG + ag) * t.L + l0 + l;
      t.out_a[o] = make_uint4(w[0], w[1], w[2], w[3]);
    }
  }
}

// Word-wise version for tile lengths that are multiples of 4: a thread takes the 16 LDS
// words that hold four consecutive l of the sixteen rows of one granule column and
// transposes 16 x 4 bytes with byte permutes, producing the four granules l .. l+3
// (64 contiguous bytes of output).
//   base: LDS byte offset of row 0 of the group; stride: bytes between its rows
__device__ __forceinline__ void granules4(const uint8_t* tile, int base, int stride, uint4 out[4]) {
  // __builtin_amdgcn_perm(hi, lo, sel): result byte k = byte sel[k] of the 8-byte {hi:lo}
  uint32_t q[4][4];  // q[g][l]: rows 4g .. 4g+3 at position l
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    uint32_t d[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
      d[j] = *reinterpret_cast<const uint32_t*>(tile + base + (4 * g + j) * stride);
    const uint32_t p01l = __builtin_amdgcn_perm(d[1], d[0], 0x05010400u);  // [d0.b0, d1.b0, d0.b1, d1.b1]
    const uint32_t p01h = __builtin_amdgcn_perm(d[1], d[0], 0x07030602u);  // [d0.b2, d1.b2, d0.b3, d1.b3]
    const uint32_t p23l = __builtin_amdgcn_perm(d[3], d[2], 0x05010400u);
    const uint32_t p23h = __builtin_amdgcn_perm(d[3], d[2], 0x07030602u);
    q[g][0] = __builtin_amdgcn_perm(p23l, p01l, 0x05040100u);  // [d0.b0, d1.b0, d2.b0, d3.b0]
    q[g][1] = __builtin_amdgcn_perm(p23l, p01l, 0x07060302u);
    q[g][2] = __builtin_amdgcn_perm(p23h, p01h, 0x05040100u);
    q[g][3] = __builtin_amdgcn_perm(p23h, p01h, 0x07060302u);
  }
#pragma unroll
  for (int l = 0; l < 4; ++l) out[l] = make_uint4(q[0][l], q[1][l], q[2][l], q[3][l]);
}

__device__ __forceinline__ void store_granules_w4(const TileArgs& t, const uint8_t* tile, int pitch,
                                                  int tl, int a0, int b0, int l0) {
  const int quads = tl >> 2, n_items = 16 * quads;
  if (t.out_b) {
    const int bg = b0 >> 4;
    for (int it = threadIdx.x; it < n_items; it += blockDim.x) {
      const int a = it / quads, l = (it - a * quads) * 4;
      if (a0 + a >= t.A) continue;
      uint4 g4[4];
      granules4(tile, (a * 16) * pitch + l, pitch, g4);
      const long long o = t.b_lmajor ? ((long long)(a0 + a) * t.L + l0 + l) * t.BG + bg
                                     : ((long long)(a0 + a) * t.BG + bg) * t.L + l0 + l;
      const int step = t.b_lmajor ? t.BG : 1;
#pragma unroll
      for (int i = 0; i < 4; ++i) t.out_b[o + (long long)i * step] = g4[i];
    }
  }
  if (t.out_a) {
    const int ag = a0 >> 4;
    for (int it = threadIdx.x; it < n_items; it += blockDim.x) {
      const int b = it / quads, l = (it - b * quads) * 4;
      if (b0 + b >= t.B) continue;
      uint4 g4[4];
      granules4(tile, b * pitch + l, 16 * pitch, g4);
      const long long o = t.a_lmajor ? ((long long)(b0 + b) * t.L + l0 + l) * t.AG + ag
                                     : ((long long)(b0 + b) * t.AG + ag) * t.L + l0 + l;
      const int step = t.a_lmajor ? t.AG : 1;
#pragma unroll
      for (int i = 0; i < 4; ++i) t.out_a[o + (long long)i * step] = g4[i];
    }
  }
}

// ---------------------------------------------------------------------------
// Streaming tile quantizer: one 16(a) x 16(b) x window(l) tile per workgroup.
//   windowed tiles (SMALL = false): L % 4 == 0, window_len(L) <= 64 elements of l;
//   whole-row tiles (SMALL = true): 16 x 16 x L with B % 16 == 0 and (B*L) % 8 == 0;
//     for one a the sixteen rows are contiguous (16*L floats) and are read as
//     8-element groups that may straddle rows.
// One work item = one aligned block of 8 consecutive elements (the unit of the random
// number generator), as two halves of 4.  In a windowed tile a half can fall outside
// the window or the row; such a half is not read and not written.
// ---------------------------------------------------------------------------
struct ItemPos {
  long long e0;    // flat index of the block's first element (a multiple of 8)
  int row;         // windowed: LDS row a*16+b; whole-row: a
  int off;         // windowed: LDS byte offset of the first half inside the row (may be < 0
                   //           when that half is invalid); whole-row: group index j
  bool v0, v1;     // halves to read and quantize
  bool z0, z1;     // halves to zero-fill in LDS (padding rows)
};

template <bool SMALL>
__device__ __forceinline__ ItemPos item_pos(const TileArgs& t, int a0, int b0, int l0, int tl,
                                            int it) {
  ItemPos p;
  if (SMALL) {
    const int octs = 2 * t.L;
    const int a = it / octs, j = it - a * octs;
    p.row = a;
    p.off = j;
    p.v0 = p.v1 = (a < 16) && (a0 + a < t.A);
    p.z0 = p.z1 = (a < 16) && !p.v0;
    p.e0 = ((long long)(a0 + a) * t.B + b0) * t.L + 8 * j;
  } else {
    const int row = it >> 3, j = it & 7;
    const int ga = a0 + (row >> 4), gb = b0 + (row & 15);
    const bool row_ok = ga < t.A && gb < t.B;
    // padding rows are zero-filled with the block pattern of a row that starts at 0
    const long long e_row = row_ok ? ((long long)ga * t.B + gb) * t.L : 0;
    const int l_end = min(l0 + tl, t.L);
    p.e0 = (((e_row + l0) >> 3) + j) << 3;
    const int lq0 = (int)(p.e0 - e_row), lq1 = lq0 + 4;
    const bool in0 = lq0 >= l0 && lq0 + 4 <= l_end, in1 = lq1 >= l0 && lq1 + 4 <= l_end;
    p.row = row;
    p.off = lq0 - l0;
    p.v0 = row_ok && in0;
    p.v1 = row_ok && in1;
    p.z0 = !row_ok && in0;
    p.z1 = !row_ok && in1;
  }
  return p;
}

// Both halves are always loaded (an invalid half reads elements 0..3 and is ignored), so
// that no branch separates the loads of different items.
__device__ __forceinline__ void load8(const float* x, const ItemPos& p, float v[8]) {
  const float4 lo = *reinterpret_cast<const float4*>(x + (p.v0 ? p.e0 : 0));
  const float4 hi = *reinterpret_cast<const float4*>(x + (p.v1 ? p.e0 + 4 : 0));
  v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w;
  v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
}

// Window length along l of the windowed tiles: a multiple of 4 (of 8 when rows start on
// multiples of 8) such that a row window overlaps at most 8 generator blocks.
__host__ __device__ inline int window_len(int L) {
  const int cap = (L % 8 == 0) ? 64 : 56;
  const int nw = (L + cap - 1) / cap;
  const int per = (L + nw - 1) / nw;
  return (L % 8 == 0) ? (per + 7) / 8 * 8 : (per + 3) / 4 * 4;
}

// Where a workgroup stands inside its tensor's grid of tiles.
struct TileCoord {
  int x, y, z;          // tile index along l, b, a
  unsigned n_blocks;    // workgroups that work on this tensor
  unsigned id;          // this workgroup's index among them
  bool first;           // the tensor's first workgroup
  unsigned gx, tiles;   // matrix tiles: tiles along b and in all; workgroup id takes tiles
                        // id, id + n_blocks, ...
};

template <int MODE, bool SMALL>
__device__ __forceinline__ void stream_body(const TileArgs& t, int pitch, int tl, const TileCoord& bc,
                                            uint8_t* dyn_tile) {
  constexpr bool kGrad = MODE >= 2;
  GradSetup gs{};
  float c;
  if (kGrad) {
    gs = grad_setup(t.st, t.pmax, t.nblocks, t.bits, t.hindsight != 0);
    c = gs.c;
  } else if (!(t.c_given > 0.0f) && t.c_ptr) {
    c = *t.c_ptr;
  } else {
    c = operand_setup(t.c_given, t.pmax, t.nblocks, t.pmax_col, t.is_unsigned != 0, t.c_out, t.bad_out,
                      t.st, nullptr, bc.first, t.bits);
  }
  const QConst qc = make_qconst(c, MODE < 2 && t.is_unsigned != 0, t.bits);
  const bool live = qc.live;
  const unsigned long long step = (MODE == 3) ? t.st->step : 0ull;
  const int l0 = bc.x * tl, b0 = bc.y * 16, a0 = bc.z * 16;

  uint32_t cnt = 0, cnt_wave = 0, seen_max = 0;
  auto quantize_item = [&](const ItemPos& p, const float v[8]) __attribute__((always_inline)) {
    // eight codes of one generator block -> LDS bytes
    Philox4 rnd{};
    if (MODE == 3 && live) rnd = philox_block((unsigned long long)p.e0 >> 3, step, t.seed);
    if (SMALL) {
      if (p.row >= 16) return;  // beyond the tile's groups
      int b = (8 * p.off) / t.L, l = 8 * p.off - b * t.L;
      const bool have = p.v0 && live;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        int k = 0;
        if (have) k = quantize_one<MODE>(v[u], qc, rnd, u, cnt);
        dyn_tile[(p.row * 16 + b) * pitch + l] = (uint8_t)k;
        if (++l == t.L) { l = 0; ++b; }
      }
    } else {
      uint32_t w0 = 0, w1 = 0;
      if (live) quantize8<MODE>(v, p.v0, p.v1, qc, rnd, w0, w1, cnt_wave);
      uint8_t* dst = dyn_tile + p.row * pitch + p.off;
      if (p.v0 || p.z0) *reinterpret_cast<uint32_t*>(dst) = w0;
      if (p.v1 || p.z1) *reinterpret_cast<uint32_t*>(dst + 4) = w1;
    }
  };
  // items in batches of four: the eight loads of a batch are in flight together
  const int n_items = SMALL ? 32 * t.L : 8 * kThreads;
  for (int base = 0; base < n_items; base += 4 * kThreads) {
    float v[4][8];
    ItemPos p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      p[i] = item_pos<SMALL>(t, a0, b0, l0, tl, base + i * kThreads + threadIdx.x);
      load8(t.x, p[i], v[i]);  // unconditional (also when every code is 0): no branch between loads
    }
    // keep the eight loads together ahead of the arithmetic that consumes them
    __builtin_amdgcn_sched_barrier(0);
    if (kGrad && gs.hindsight) {
      // a load outside the tile has fetched the tensor's first elements: harmless for a maximum
#pragma unroll
      for (int i = 0; i < 4; ++i) seen_max = max(seen_max, max_abs_bits8(v[i]));
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) quantize_item(p[i], v[i]);
  }
  __syncthreads();
  if (SMALL) store_granules(t, dyn_tile, pitch, t.L, a0, b0, 0);
  else store_granules_w4(t, dyn_tile, pitch, min(tl, t.L - l0), a0, b0, l0);
  if (kGrad) grad_finish(t.st, gs, cnt + ((threadIdx.x & 63) == 0 ? cnt_wave : 0u),
                         (unsigned long long)t.A * t.B * t.L, bc.n_blocks, bc.id, t.tickets, seen_max);
}

// ---------------------------------------------------------------------------
// Any shape, two kernels (k_absmax3 first, or a clip value from the caller):
// tile 16 x 16 x TL with one scalar load per element.  TL = 1 serves matrices.
// ---------------------------------------------------------------------------
template <int MODE, int TL>
__device__ __forceinline__ void generic_body(const TileArgs& t, const TileCoord& bc, uint8_t* tile) {
  constexpr int PITCH = (TL == 1) ? 1 : TL + 4;
  GradSetup gs{};
  float c;
  if (MODE >= 2) {
    gs = grad_setup(t.st, t.pmax, t.nblocks, t.bits, t.hindsight != 0);
    c = gs.c;
  } else if (!(t.c_given > 0.0f) && t.c_ptr) {
    c = *t.c_ptr;
  } else {
    c = operand_setup(t.c_given, t.pmax, t.nblocks, t.pmax_col, t.is_unsigned != 0, t.c_out, t.bad_out,
                      t.st, nullptr, bc.first, t.bits);
  }
  const QConst qc = make_qconst(c, MODE < 2 && t.is_unsigned != 0, t.bits);
  const bool live = qc.live;
  const unsigned long long step = (MODE == 3) ? t.st->step : 0ull;
  const int l0 = bc.x * TL, b0 = bc.y * 16, a0 = bc.z * 16;
  uint32_t cnt = 0, seen_max = 0;
  const bool scan = live || (MODE >= 2 && gs.hindsight);
  for (int idx = threadIdx.x; idx < 256 * TL; idx += kThreads) {
    const int l = idx % TL, row = idx / TL;
    const int ga = a0 + (row >> 4), gb = b0 + (row & 15), gl = l0 + l;
    int k = 0;
    if (scan && ga < t.A && gb < t.B && gl < t.L) {
      const long long e = ((long long)ga * t.B + gb) * t.L + gl;
      const float v = t.x[e];
      seen_max = max(seen_max, __float_as_uint(v) & 0x7fffffffu);
      if (live) {
        Philox4 rnd{};
        if (MODE == 3) rnd = philox_block((unsigned long long)e >> 3, step, t.seed);
        k = quantize_one<MODE>(v, qc, rnd, (uint32_t)e & 7u, cnt);
      }
    }
    tile[row * PITCH + l] = (uint8_t)k;
  }
  __syncthreads();
  store_granules(t, tile, PITCH, TL, a0, b0, l0);
  if (MODE >= 2) grad_finish(t.st, gs, cnt, (unsigned long long)t.A * t.B * t.L, bc.n_blocks, bc.id,
                             t.tickets, seen_max);
}

// ---------------------------------------------------------------------------
// Matrices (L = 1, B % 8 == 0, 16-byte aligned): one 64(a) x 64(b) tile per workgroup.
// A thread quantizes two runs of 8 consecutive b (one generator block each) into an [a][b]
// LDS tile.  Granules along b are 16 consecutive tile bytes (one per thread); granules along a
// come out of the 16 x 4 byte transpose also used by the streaming tiles (64 threads, four
// granules each).  Four neighbouring threads store 64 contiguous bytes.  A workgroup walks
// several tiles when the matrix has more than the grid's cap, so that the prologue (the
// re-reduction of the partial maxima) and the ticket are paid once per workgroup.
// ---------------------------------------------------------------------------
template <int MODE>
__device__ __forceinline__ void matrix_body(const TileArgs& t, const TileCoord& bc, uint8_t* lds) {
  constexpr int PITCH = 80;
  uint8_t* const tile = lds;                 // [64 a][PITCH]
  GradSetup gs{};
  float c;
  if (MODE >= 2) {
    gs = grad_setup(t.st, t.pmax, t.nblocks, t.bits, t.hindsight != 0);
    c = gs.c;
  } else if (!(t.c_given > 0.0f) && t.c_ptr) {
    c = *t.c_ptr;
  } else {
    c = operand_setup(t.c_given, t.pmax, t.nblocks, t.pmax_col, t.is_unsigned != 0, t.c_out, t.bad_out,
                      t.st, nullptr, bc.first, t.bits);
  }
  const QConst qc = make_qconst(c, MODE < 2 && t.is_unsigned != 0, t.bits);
  const bool live = qc.live;
  const unsigned long long step = (MODE == 3) ? t.st->step : 0ull;
  uint32_t cnt_wave = 0, seen_max = 0;
  for (unsigned tile_id = bc.id; tile_id < bc.tiles; tile_id += bc.n_blocks) {
  const int b0 = (int)(tile_id % bc.gx) * 64, a0 = (int)(tile_id / bc.gx) * 64;
  float v[2][8];
  bool ok[2];
  long long e0[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int it = threadIdx.x + kThreads * i;
    const int row = it >> 3, col = (it & 7) * 8;
    ok[i] = a0 + row < t.A && b0 + col < t.B;
    e0[i] = ok[i] ? (long long)(a0 + row) * t.B + b0 + col : 0;
    const float4 lo = *reinterpret_cast<const float4*>(t.x + e0[i]);
    const float4 hi = *reinterpret_cast<const float4*>(t.x + e0[i] + 4);
    v[i][0] = lo.x; v[i][1] = lo.y; v[i][2] = lo.z; v[i][3] = lo.w;
    v[i][4] = hi.x; v[i][5] = hi.y; v[i][6] = hi.z; v[i][7] = hi.w;
  }
  // (a run outside the matrix has fetched the tensor's first elements: harmless for a maximum)
  if (MODE >= 2 && gs.hindsight) seen_max = max(seen_max, max(max_abs_bits8(v[0]), max_abs_bits8(v[1])));
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int it = threadIdx.x + kThreads * i;
    const int row = it >> 3, col = (it & 7) * 8;
    Philox4 rnd{};
    if (MODE == 3 && live && ok[i]) rnd = philox_block((unsigned long long)e0[i] >> 3, step, t.seed);
    uint32_t w0 = 0, w1 = 0;
    if (live) quantize8<MODE>(v[i], ok[i], ok[i], qc, rnd, w0, w1, cnt_wave);
    *reinterpret_cast<uint2*>(tile + row * PITCH + col) = make_uint2(w0, w1);
  }
  __syncthreads();
  const int r = threadIdx.x >> 2, gl = threadIdx.x & 3;
  if (t.out_b && a0 + r < t.A && (b0 >> 4) + gl < t.BG)
    t.out_b[(long long)(a0 + r) * t.BG + (b0 >> 4) + gl] =
        *reinterpret_cast<const uint4*>(tile + r * PITCH + 16 * gl);
  if (t.out_a && threadIdx.x < 64 && (a0 >> 4) + gl < t.AG) {
    uint4 g4[4];
    granules4(tile, (16 * gl) * PITCH + 4 * r, PITCH, g4);   // b = 4 r .. 4 r + 3, a = 16 gl .. + 15
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (b0 + 4 * r + i < t.B) t.out_a[(long long)(b0 + 4 * r + i) * t.AG + (a0 >> 4) + gl] = g4[i];
  }
  __syncthreads();   // the tile is free for the workgroup's next one
  }
  if (MODE >= 2) grad_finish(t.st, gs, (threadIdx.x & 63) == 0 ? cnt_wave : 0u,
                             (unsigned long long)t.A * t.B * t.L, bc.n_blocks, bc.id, t.tickets, seen_max);
}

// ---------------------------------------------------------------------------
// One launch quantizes up to three tensors of a layer (output gradient, activations,
// weights): workgroups [first, first + n_blocks) belong to a tensor and walk its tiles in
// the order l fastest, then b, then a (matrix tiles: in the order of their indices).
// ---------------------------------------------------------------------------
enum TileKind { kGenericTile = 0, kGenericColumn, kWindowed, kWholeRow, kMatrix };

struct Segment {
  TileArgs t;
  int kind;             // TileKind
  int pitch, tl;        // LDS row pitch and tile length along l (streaming kinds)
  unsigned gx, gy, gz;  // tiles along l, b and a
  unsigned first, n_blocks;
};

template <int MODE>
__device__ __forceinline__ void run_segment(const Segment& sg, unsigned blk, uint8_t* lds) {
  const unsigned local = blk - sg.first;
  // Workgroups are dealt to the eight dies round-robin by their index, and each die has its own
  // L2.  Neighbouring windows of a row share the cache lines at their common edge whenever the
  // rows do not start on line boundaries (28 x 28 and 14 x 14 maps), so a die is given a
  // contiguous run of tiles: workgroups j, j + 8, j + 16, ... take consecutive tiles.
  const unsigned per_die = sg.n_blocks >> 3, extra = sg.n_blocks & 7u, die = local & 7u;
  const unsigned tile = die * per_die + min(die, extra) + (local >> 3);
  TileCoord bc;
  bc.x = (int)(tile % sg.gx);
  const unsigned rest = tile / sg.gx;
  bc.y = (int)(rest % sg.gy);
  bc.z = (int)(rest / sg.gy);
  bc.n_blocks = sg.n_blocks;
  bc.id = local;
  bc.first = local == 0;
  bc.gx = sg.gx;
  bc.tiles = sg.gx * sg.gy * sg.gz;
  switch (sg.kind) {
    case kWindowed: stream_body<MODE, false>(sg.t, sg.pitch, sg.tl, bc, lds); break;
    case kWholeRow: stream_body<MODE, true>(sg.t, sg.pitch, sg.tl, bc, lds); break;
    case kGenericColumn: generic_body<MODE, 1>(sg.t, bc, lds); break;
    case kMatrix: matrix_body<MODE>(sg.t, bc, lds); break;
    default: generic_body<MODE, 32>(sg.t, bc, lds);
  }
}

// GMODE: 2 nearest / 3 stochastic gradient quantizer.  Activations and weights share ONE copy
// of the operand code (signed or unsigned is a run-time field of the tensor): the kernel's
// size counts, its workgroups run three different bodies side by side on a compute unit.
// A tensor with n_blocks == 0 is absent.
template <int GMODE>
__global__ __launch_bounds__(kThreads, 6) void k_quantize_layer(const Segment sg, const Segment sx,
                                                              const Segment sw) {
  extern __shared__ __attribute__((aligned(16))) uint8_t dyn_tile[];
  const unsigned blk = blockIdx.x;
  if (blk < sx.first) run_segment<GMODE>(sg, blk, dyn_tile);
  else run_segment<0>(blk < sw.first ? sx : sw, blk, dyn_tile);
}

inline int flat_grid(long long work_items) {
  long long blocks = (work_items + kThreads - 1) / kThreads;
  const long long cap = 256 * 16;  // 256 compute units, several workgroups each
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return (int)blocks;
}

// Matrix tiles: workgroups per tensor above which a workgroup takes more than one tile.
constexpr unsigned long long kMatrixGridCap = 2048;

TileKind tile_kind(const float* x, long long B, long long L) {
  if (reinterpret_cast<uintptr_t>(x) % 16 == 0) {
    if (L == 1 && B % 8 == 0) return kMatrix;
    if (L >= 16 && L % 4 == 0) return kWindowed;
    if (L >= 2 && L <= 248 && B % 16 == 0 && (B * L) % 8 == 0) return kWholeRow;
  }
  return L == 1 ? kGenericColumn : kGenericTile;
}

// Tile grid, LDS need and kernel variant of one tensor; returns the dynamic LDS bytes.
size_t plan_segment(Segment& sg) {
  const TileArgs& t = sg.t;
  sg.kind = tile_kind(t.x, t.B, t.L);
  sg.gy = (unsigned)t.BG;
  sg.gz = (unsigned)t.AG;
  size_t lds;
  switch (sg.kind) {
    case kWindowed:
      sg.tl = window_len(t.L);
      sg.pitch = 72;
      sg.gx = (unsigned)((t.L + sg.tl - 1) / sg.tl);
      lds = (size_t)256 * sg.pitch;
      break;
    case kWholeRow:
      sg.tl = t.L;
      sg.pitch = (t.L + 3) / 4 * 4 + 4;
      sg.gx = 1;
      lds = (size_t)256 * sg.pitch;
      break;
    case kGenericColumn:
      sg.tl = 1; sg.pitch = 1; sg.gx = 1;
      lds = 256;
      break;
    case kMatrix:
      sg.tl = 1; sg.pitch = 80;
      sg.gx = (unsigned)((t.B + 63) / 64);
      sg.gy = 1;
      sg.gz = (unsigned)((t.A + 63) / 64);
      lds = (size_t)64 * 80;
      break;
    default:
      sg.tl = 32; sg.pitch = 36;
      sg.gx = (unsigned)((t.L + 31) / 32);
      lds = (size_t)256 * 36;
  }
  return lds;
}

}  // namespace

int launch_absmax3(const float* p0, int64_t n0, int abs0, const float* p1, int64_t n1, int abs1,
                   const float* p2, int64_t n2, int abs2, uint32_t* pmax,
                   unsigned long long* tickets, int* nblocks_out, lbt_grad_state* st, hipStream_t s,
                   const OperandScalars* kept, int kept_mask) {
  if (!p0) n0 = 0;
  if (!p1) n1 = 0;
  if (!p2) n2 = 0;
  ProfScope prof(KID_ABSMAX, (double)(n0 + n1 + n2), s);
  const long long total = n0 + n1 + n2;
  // at most ~512 partial rows (two workgroups per compute unit on a large layer), so that a
  // consumer's prologue reads 2 per thread
  long long per = (total + 511) / 512;
  per = (per + 8191) / 8192 * 8192;  // 256 threads x 8 float4
  if (per < 8192) per = 8192;
  const long long nb0 = (n0 + per - 1) / per, nb1 = (n1 + per - 1) / per, nb2 = (n2 + per - 1) / per;
  long long nb = nb0 + nb1 + nb2;
  if (nb == 0 && !st) { *nblocks_out = 0; return LBT_OK; }
  if (nb == 0) nb = 1;  // the state and the counters are still reset; the one partial row is zero
  *nblocks_out = (int)nb;
  if (nb > kMaxPartialBlocks) return LBT_ERR_UNSUPPORTED;
  MaxSeg s0{p0, n0, abs0, 0}, s1{p1, n1, abs1, (int)nb0}, s2{p2, n2, abs2, (int)(nb0 + nb1)};
  LBT_LAUNCH(k_absmax3, dim3((unsigned)nb), dim3(kThreads), 0, s, s0, s1, s2, per, pmax, tickets, st,
             kept, kept_mask);
  return LBT_OK;
}

int ste_blocks(int64_t n) {
  long long blocks = ((n >> 2) + 2 * kThreads - 1) / (2 * kThreads);
  if (blocks > kStePartials) blocks = kStePartials;
  return blocks < 1 ? 1 : (int)blocks;
}

// finish = false: the partial sums stay in `partial` for a later launch_ste_finish.
int launch_ste_backward(const float* x, const float* grad_q, int64_t n, float c, int is_unsigned,
                        int bits, float* grad_x, float* grad_c, double* partial, hipStream_t s,
                        bool finish) {
  ProfScope prof(KID_STE, (double)n, s);
  const int blocks = ste_blocks(n);
  LBT_LAUNCH(k_ste_backward, dim3((unsigned)blocks), dim3(kThreads), 0, s, x, grad_q, (long long)n, c,
             is_unsigned, bits, grad_x, (grad_c || !finish) ? partial : (double*)nullptr);
  if (grad_c && finish) {
    SteSums f{{partial, nullptr}, {blocks, 0}, {grad_c, nullptr}};
    LBT_LAUNCH(k_ste_finish, dim3(1), dim3(kThreads), 0, s, f);
  }
  return LBT_OK;
}

// The sums of one or two passes of n0 (and n1 > 0) elements whose partial sums were left in
// partial0 (and partial1), in one launch.
int launch_ste_finish(const double* partial0, int64_t n0, float* grad_c0, const double* partial1,
                      int64_t n1, float* grad_c1, hipStream_t s) {
  ProfScope prof(KID_STE, 0.0, s);
  SteSums f{{partial0, partial1}, {ste_blocks(n0), n1 > 0 ? ste_blocks(n1) : 0}, {grad_c0, grad_c1}};
  LBT_LAUNCH(k_ste_finish, dim3(n1 > 0 ? 2 : 1), dim3(kThreads), 0, s, f);
  return LBT_OK;
}

int launch_quantize_flat_grad(const float* g, int64_t n, const uint32_t* pmax, int nblocks,
                              unsigned long long* tickets, lbt_grad_state* st, uint64_t seed, int rounding, int hindsight,
                              int fused_update, int bits, uint8_t* codes, hipStream_t s) {
  ProfScope prof(KID_FLAT_GRAD, (double)n, s);
  const int grid = flat_grid((n + 7) / 8);
  if (rounding == LBT_ROUND_STOCHASTIC)
    LBT_LAUNCH(k_quantize_flat<3>, dim3(grid), dim3(kThreads), 0, s, g, (long long)n, 0.0f,
                       pmax, nblocks, tickets, st, (unsigned long long)seed, codes, (float*)nullptr,
                       (float*)nullptr, hindsight, fused_update, bits);
  else
    LBT_LAUNCH(k_quantize_flat<2>, dim3(grid), dim3(kThreads), 0, s, g, (long long)n, 0.0f,
                       pmax, nblocks, tickets, st, (unsigned long long)seed, codes, (float*)nullptr,
                       (float*)nullptr, hindsight, fused_update, bits);
  return LBT_OK;
}

int launch_quantize_flat_operand(const float* x, int64_t n, float c_given, const uint32_t* pmax,
                                 int nblocks, int is_unsigned, int bits, uint8_t* codes, float* c_out,
                                 float* clip_scale_out, hipStream_t s) {
  ProfScope prof(KID_FLAT_OPERAND, (double)n, s);
  const int grid = flat_grid((n + 7) / 8);
  if (is_unsigned)
    LBT_LAUNCH(k_quantize_flat<1>, dim3(grid), dim3(kThreads), 0, s, x, (long long)n,
                       c_given, pmax, nblocks, (unsigned long long*)nullptr, (lbt_grad_state*)nullptr, 0ull, codes, c_out,
                       clip_scale_out, 0, 0, bits);
  else
    LBT_LAUNCH(k_quantize_flat<0>, dim3(grid), dim3(kThreads), 0, s, x, (long long)n,
                       c_given, pmax, nblocks, (unsigned long long*)nullptr, (lbt_grad_state*)nullptr, 0ull, codes, c_out,
                       clip_scale_out, 0, 0, bits);
  return LBT_OK;
}

static void fill_tile_args(TileArgs& t, const float* x, int64_t A, int64_t B, int64_t L,
                           const RelayoutIo& io) {
  t.x = x; t.A = (int)A; t.B = (int)B; t.L = (int)L;
  t.AG = (int)(round_up(A, kGranule) / kGranule);
  t.BG = (int)(round_up(B, kGranule) / kGranule);
  t.pmax = io.pmax; t.nblocks = io.nblocks; t.pmax_col = io.pmax_col;
  t.tickets = io.tickets;
  t.st = io.st;
  t.out_b = reinterpret_cast<uint4*>(io.out_b);
  t.out_a = reinterpret_cast<uint4*>(io.out_a);
  t.a_lmajor = io.a_lmajor;
  t.b_lmajor = io.b_lmajor;
}

int launch_quantize_layer(const LayerTensors& q, hipStream_t s) {
  double work = 0.0;
  Segment seg[3] = {};
  size_t lds = 0;
  unsigned long long next = 0;
  for (int i = 0; i < 3; ++i) {
    const LayerTensors::One& o = q.tensor[i];
    Segment& sg = seg[i];
    sg.first = (unsigned)next;
    if (!o.x) continue;
    fill_tile_args(sg.t, o.x, o.A, o.B, o.L, o.io);
    sg.t.seed = q.seed;
    sg.t.hindsight = (i == 0) ? q.hindsight : 0;
    sg.t.bits = q.bits;
    sg.t.is_unsigned = (i == 1) ? q.x_unsigned : 0;
    sg.t.c_given = o.c_given;
    sg.t.c_out = o.c_out;
    sg.t.bad_out = o.bad_out;
    const size_t need = plan_segment(sg);
    if (need > lds) lds = need;
    unsigned long long nb = (unsigned long long)sg.gx * sg.gy * sg.gz;
    if (nb == 0 || nb > 0x7fffffffull || next + nb > 0x7fffffffull) return LBT_ERR_UNSUPPORTED;
    if (sg.kind == kMatrix && nb > kMatrixGridCap) {   // several tiles per workgroup
      const unsigned long long per = (nb + kMatrixGridCap - 1) / kMatrixGridCap;
      nb = (nb + per - 1) / per;
    }
    sg.n_blocks = (unsigned)nb;
    next += nb;
    work += (double)o.A * (double)o.B * (double)o.L;
  }
  if (next == 0) return LBT_OK;
  const dim3 block(kThreads);
  const bool sr = q.rounding == LBT_ROUND_STOCHASTIC;
  ProfScope prof(KID_QUANTIZE_LAYER, work, s);
  const dim3 grid((unsigned)next);
  if (sr) LBT_LAUNCH((k_quantize_layer<3>), grid, block, lds, s, seg[0], seg[1], seg[2]);
  else LBT_LAUNCH((k_quantize_layer<2>), grid, block, lds, s, seg[0], seg[1], seg[2]);
  return LBT_OK;
}

int launch_update_interval(lbt_grad_state* st, hipStream_t s) {
  ProfScope prof(KID_UPDATE, 0.0, s);
  LBT_LAUNCH(k_update_interval, dim3(1), dim3(1), 0, s, st);
  return LBT_OK;
}

int launch_state_init(lbt_grad_state* st, const lbt_grad_state& v, hipStream_t s) {
  ProfScope prof(KID_STATE, 0.0, s);
  LBT_LAUNCH(k_state_set, dim3(1), dim3(1), 0, s, st, v);
  return LBT_OK;
}

}  // namespace lbt
