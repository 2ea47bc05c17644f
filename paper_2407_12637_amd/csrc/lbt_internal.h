// Internal declarations shared by the HIP translation units of liblbt.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <type_traits>
#include <utility>

#include "lbt.h"

#define LBT_HIP_CHECK(expr)                       \
  do {                                            \
    hipError_t lbt_e_ = (expr);                   \
    if (lbt_e_ != hipSuccess) return LBT_ERR_HIP; \
  } while (0)


namespace lbt {

constexpr int kGranule = 16;  // contraction-axis padding of the GEMM code layouts, in codes

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// Largest code of a b-bit quantizer: 2^(b-1) - 1 signed (Eq. 2), 2^b - 1 unsigned (Eq. 3).
__host__ __device__ inline int levels(int bits, bool is_unsigned) {
  return is_unsigned ? (1 << bits) - 1 : (1 << (bits - 1)) - 1;
}

// Scalars shared between the kernels of one backward call; lives at the start
// of the caller's workspace.
struct OperandScalars {
  float c_x;       // clip value actually used for X
  float c_w;       // ... for W
  uint32_t bad_x;  // operand maximum was Inf/NaN
  uint32_t bad_w;
};

// Alg. 1 (Eq. 15-16) for a quantization that ended with status OK, clip-out count n_out of
// n_total elements: one thread.
__device__ __forceinline__ void interval_update_with(lbt_grad_state* st, unsigned long long n_out,
                                                     unsigned long long n_total) {
  const double lhs = (double)n_out * (double)((1 << st->bits) - 1);
  const double rhs = __dmul_rn(st->alpha, (double)n_total);
  const int sg = (lhs > rhs) - (lhs < rhs);
  double g = __dadd_rn(st->gamma, __dmul_rn(st->beta, (double)sg));
  g = fmax(g, st->gamma_min);
  g = fmin(g, st->gamma_max);
  st->gamma = g;
  st->step += 1;
}
// ... on the statistics the last gradient quantization left in the state.
__device__ __forceinline__ void interval_update(lbt_grad_state* st) {
  if (st->status != LBT_STATUS_OK) return;
  interval_update_with(st, st->n_out, st->n_total);
}


// ---- device helpers shared by the element-wise kernels and the products' epilogues -------
// Per-call quantizer constants, uniform across the grid.
struct QConst {
  float c;       // clip value; <= 0 means "all codes zero"
  float lo;      // lower clip bound: -c or 0
  float inv_s;   // q / c
  int q;         // largest code
  int kmin;      // smallest code
  bool live;     // false: degenerate interval (c <= 0, or so small that q / c is not a finite
                 // fp32 number): every code is 0
};

// Eq. (1) needs q / c as a finite fp32 number; below c ~ q * 2.9e-39 it is not.
__host__ __device__ inline bool interval_usable(float c, int q) {
  return c > 0.0f && (float)((double)q / (double)c) < INFINITY;
}

__device__ __forceinline__ QConst make_qconst(float c, bool is_unsigned, int bits) {
  QConst k;
  k.c = c;
  k.q = levels(bits, is_unsigned);
  k.kmin = is_unsigned ? 0 : -k.q;
  k.lo = is_unsigned ? 0.0f : -c;
  k.live = interval_usable(c, k.q);
  k.inv_s = k.live ? (float)((double)k.q / (double)c) : 0.0f;
  return k;
}

// x_n of Eq. (1): clip to [lo, c] (the median of the three: one instruction), then one fp32
// multiply by q / c.
__device__ __forceinline__ float normalised(float v, const QConst& k) {
  const float xc = __builtin_amdgcn_fmed3f(v, k.lo, k.c);
  return __fmul_rn(xc, k.inv_s);
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__device__ __forceinline__ double block_sum_f64(double v) {
  __shared__ double part[16];
  const int nw = blockDim.x >> 6;
  v = wave_sum_f64(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
  __syncthreads();
  double t = 0.0;
  for (int i = 0; i < nw; ++i) t += part[i];
  return t;
}

// One element of the gradient through an operand quantizer: returns the masked gradient and
// adds g * (q * dQ/dc) to acc (the caller divides the sum by q once): q * dQ/dc is
// round(u) - u inside the interval (exact in fp32: both are within 1/2 of each other), +q for
// v >= c, below_q (-q signed, 0 unsigned) for v <= lo.
__device__ __forceinline__ float ste_one(float v, float g, const QConst& k, float below_q, double& acc) {
  const bool inside = v > k.lo && v < k.c;
  const float u = normalised(v, k);
  const float w = inside ? rintf(u) - u : (v >= k.c ? (float)k.q : (v <= k.lo ? below_q : 0.0f));
  acc += (double)g * (double)w;
  return inside ? g : 0.0f;
}

// ---- profile.hip: optional event timing of every launch ------------------------
enum KernelId {
  KID_ABSMAX = 0, KID_FLAT_GRAD, KID_FLAT_OPERAND, KID_QUANTIZE_LAYER, KID_GEMM_DX,
  KID_GEMM_DW, KID_GEMM_FWD,
  KID_FINALIZE, KID_UPDATE, KID_STATE, KID_STE, KID_COUNT
};
// Records a start event now and a stop event when it goes out of scope (after the
// launch it brackets).  `work` is the algorithmic work of the launch: elements for
// the element-wise kernels, integer operations (2 per multiply-add) for the GEMMs.
class ProfScope {
 public:
  ProfScope(int kid, double work, hipStream_t s);
  ~ProfScope();
  ProfScope(const ProfScope&) = delete;
  ProfScope& operator=(const ProfScope&) = delete;

 private:
  long long idx_;
  hipStream_t s_;
};

// Measurement aid (lbt_profile_skeleton): the product launches skip their contraction loop.
bool profile_skeleton();

// Every kernel of the library is launched through launch_kernel, which hands back the error
// of THIS launch (the runtime's "last error" may stem from an earlier call of the caller's).
template <typename... KArgs, size_t... I>
inline hipError_t launch_tuple(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t shmem,
                               hipStream_t s, std::tuple<std::decay_t<KArgs>...>& vals,
                               std::index_sequence<I...>) {
  void* ptrs[] = {static_cast<void*>(&std::get<I>(vals))...};
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, shmem, s);
}
template <typename... KArgs, typename... Args>
inline hipError_t launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t shmem,
                                hipStream_t s, Args&&... args) {
  static_assert(sizeof...(KArgs) == sizeof...(Args), "kernel argument count");
  std::tuple<std::decay_t<KArgs>...> vals(std::forward<Args>(args)...);
  return launch_tuple(kernel, grid, block, shmem, s, vals, std::index_sequence_for<KArgs...>{});
}
// Launch, and leave the enclosing function with LBT_ERR_HIP if the launch was refused.
#define LBT_LAUNCH(kernel, grid, block, shmem, stream, ...)                                       \
  do {                                                                                            \
    if (lbt::launch_kernel(kernel, grid, block, shmem, stream, __VA_ARGS__) != hipSuccess)        \
      return LBT_ERR_HIP;                                                                         \
  } while (0)

// ---- quantize.hip -------------------------------------------------------------
constexpr int kMaxPartialBlocks = 2048;  // partial-maximum slots in the workspace header
// Workspace header: OperandScalars (256 bytes), then pmax[kMaxPartialBlocks][4] uint32.
constexpr size_t kWsScalarsBytes = 256;
// Inside the scalars: 16 arrival counters (8 bytes each) of the gradient quantizer's
// two-level ticket, then 16 running maxima (4 bytes each) of its hindsight mode; all zeroed
// by every launch of the maximum kernel.
constexpr size_t kWsTicketOffset = 64;
constexpr int kTicketSlots = 16;
constexpr size_t kWsHeaderBytes = kWsScalarsBytes + (size_t)kMaxPartialBlocks * 16;

// Views of a workspace header.
inline uint32_t* header_pmax(void* header) {
  return reinterpret_cast<uint32_t*>(static_cast<uint8_t*>(header) + kWsScalarsBytes);
}
inline unsigned long long* header_tickets(void* header) {
  return reinterpret_cast<unsigned long long*>(static_cast<uint8_t*>(header) + kWsTicketOffset);
}

// One launch for the maxima of up to three tensors (null pointer = absent); partial
// maxima go to pmax[block][tensor]; tickets: the header's counters, zeroed by this launch.  *nblocks_out = number of partial rows written.
// st (may be null): its status is reset to OK for the quantizer launches that follow; with a
// state the kernel is launched even when every tensor is absent.
int launch_absmax3(const float* p0, int64_t n0, int abs0, const float* p1, int64_t n1, int abs1,
                   const float* p2, int64_t n2, int abs2, uint32_t* pmax,
                   unsigned long long* tickets, int* nblocks_out, lbt_grad_state* st, hipStream_t s,
                   const OperandScalars* kept = nullptr, int kept_mask = 0);
int launch_quantize_flat_grad(const float* g, int64_t n, const uint32_t* pmax, int nblocks,
                              unsigned long long* tickets, lbt_grad_state* st, uint64_t seed, int rounding, int hindsight,
                              int fused_update, int bits, uint8_t* codes, hipStream_t s);
int launch_quantize_flat_operand(const float* x, int64_t n, float c_given, const uint32_t* pmax,
                                 int nblocks, int is_unsigned, int bits, uint8_t* codes,
                                 float* c_out, float* clip_scale_out, hipStream_t s);
// Quantize T[A][B][L] (L contiguous) into GEMM layouts of 16-byte granules (16 int8 codes):
// out_b [A][ceil(B/16)][L][16] and out_a [B][ceil(A/16)][L][16] (either may be null).
// The tensor maximum, where needed, comes from the partial maxima of launch_absmax3.
struct RelayoutIo {
  const uint32_t* pmax;
  int nblocks;
  int pmax_col;
  unsigned long long* tickets;  // the header's arrival counters (used by the gradient tensor)
  lbt_grad_state* st;
  uint8_t* out_b;
  uint8_t* out_a;
  int a_lmajor;  // out_a as [B][L][A/16][16] instead of [B][A/16][L][16]
  int b_lmajor;  // out_b as [A][L][B/16][16] instead of [A][B/16][L][16]
};
// The tensors of one layer, quantized by ONE launch: [0] the output gradient (clip value
// from gamma in *st and the maximum; statistics go to *st), [1] the activations, [2] the
// weights (clip value c_given if > 0, else the tensor maximum; written to *c_out).  A null
// x marks an absent tensor.
struct LayerTensors {
  struct One {
    const float* x;
    int64_t A, B, L;
    RelayoutIo io;
    float c_given;
    float* c_out;
    uint32_t* bad_out;
  } tensor[3];
  uint64_t seed;
  int rounding;
  int hindsight;  // gradient interval from the maximum left in *st by the previous call
  int x_unsigned;
  int bits;       // b for all three tensors
};
int launch_quantize_layer(const LayerTensors& q, hipStream_t s);
// Gradient through an operand quantizer; partial: kStePartials doubles of scratch (the
// partial-maxima area of a workspace header is large enough).
constexpr int kStePartials = 2048;
int launch_ste_backward(const float* x, const float* grad_q, int64_t n, float c, int is_unsigned,
                        int bits, float* grad_x, float* grad_c, double* partial, hipStream_t s,
                        bool finish = true);
int launch_ste_finish(const double* partial0, int64_t n0, float* grad_c0, const double* partial1,
                      int64_t n1, float* grad_c1, hipStream_t s);
int launch_update_interval(lbt_grad_state* st, hipStream_t s);
int launch_state_init(lbt_grad_state* st, const lbt_grad_state& v, hipStream_t s);

// ---- gemm.hip -----------------------------------------------------------------
struct ConvGeom {
  int N, C, H, W, K, R, S, P, Q, stride, pad;
  int Np, Kp;  // N and K rounded up to kGranule
  int bits;    // b of all three code tensors
};
// How the long contraction of dW is cut over workgroups.
struct SplitPlan {
  int bm;                // rows of the workgroup tile (64 or 128)
  int bn;                // columns of the workgroup tile (64 or 128)
  int splits;            // number of K slices
  int chunks_per_split;  // chunks (16 codes) per slice
  size_t partial_bytes;  // int32 partial tiles [splits][M][NJ]; 0 when splits == 1
};
SplitPlan plan_split_k(int M, int NJ, int chunks);

// The sum of a split contraction's int32 slices, with its scale: left pending by a dW launch
// (defer), carried out by extra workgroups of the call's next product launch (carry) or by a
// launch of its own (launch_pending_reduce).  blocks == 0: nothing pending.
struct PendingReduce {
  const int32_t* partial;     // [splits][n]
  int splits;
  long long n;                // outputs
  float* out;
  int32_t* acc;               // optional raw sums
  const lbt_grad_state* st;   // scale inputs, as for the products
  const OperandScalars* sc;
  int scale_kind, bits;
  int many;                   // >= 8 slices: four thread groups share the slices of an output
  int wide;                   // slices added in 64 bits (never carried)
  unsigned blocks;            // workgroups that carry it out
};
int launch_pending_reduce(const PendingReduce& r, lbt_grad_state* update_st, hipStream_t s);

// dX: A = W codes [C][R*S][Kp/16][16], B = dY codes [N][Kp/16][P*Q][16]; out/acc [N][C][H][W].
int launch_conv_dx(const ConvGeom& g, const uint8_t* w_codes, const uint8_t* g_codes,
                   const lbt_grad_state* st, const OperandScalars* sc, float* dX, int32_t* acc,
                   lbt_grad_state* update_st, const PendingReduce* carry, hipStream_t s);
// dW: A = dY codes [K][Np/16][P*Q][16], B = X codes [C][Np/16][H*W][16]; out/acc [K][C][R][S].
int launch_conv_dw(const ConvGeom& g, const uint8_t* g_codes, const uint8_t* x_codes,
                   const lbt_grad_state* st, const OperandScalars* sc, int x_unsigned, float* dW,
                   int32_t* acc, int32_t* partial, lbt_grad_state* update_st, PendingReduce* defer,
                   hipStream_t s);
// Forward products Y = Q(X) . Q(W) (no gradient state: the scale comes from the operand
// scalars; status_out, may be null, receives the operands' status).
int launch_conv_fwd(const ConvGeom& g, const uint8_t* w_codes, const uint8_t* x_codes,
                    const OperandScalars* sc, int x_unsigned, float* Y, int32_t* acc,
                    int32_t* status_out, hipStream_t s);
int launch_linear_fwd(int M, int K_in, int N_out, int bits, const uint8_t* x_codes,
                      const uint8_t* w_codes, const OperandScalars* sc, int x_unsigned, float* Y,
                      int32_t* acc, int32_t* status_out, hipStream_t s);
// Linear layer: A/B roles swapped so both outputs are written along their rows.
// update_st (all four; may be null): the launch that ends the product also applies Alg. 1 to
// that state (the products read only the scale from it, so the order inside does not matter).
int launch_linear_dx(const ConvGeom& g, const uint8_t* w_codes, const uint8_t* g_codes,
                     const lbt_grad_state* st, const OperandScalars* sc, float* dX, int32_t* acc,
                     lbt_grad_state* update_st, const PendingReduce* carry, hipStream_t s);
int launch_linear_dw(const ConvGeom& g, const uint8_t* g_codes, const uint8_t* x_codes,
                     const lbt_grad_state* st, const OperandScalars* sc, int x_unsigned, float* dW,
                     int32_t* acc, int32_t* partial, lbt_grad_state* update_st, PendingReduce* defer,
                     hipStream_t s);

}  // namespace lbt
