// Internal declarations shared by the HIP translation units of liblbt.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lbt.h"

#define LBT_HIP_CHECK(expr)                       \
  do {                                            \
    hipError_t lbt_e_ = (expr);                   \
    if (lbt_e_ != hipSuccess) return LBT_ERR_HIP; \
  } while (0)

#define LBT_LAUNCH_CHECK()                              \
  do {                                                  \
    if (hipGetLastError() != hipSuccess) return LBT_ERR_HIP; \
  } while (0)

namespace lbt {

constexpr int kGranule = 16;  // contraction-axis padding of the GEMM code layouts, in codes

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// Scalars shared between the kernels of one backward call; lives at the start
// of the caller's workspace.
struct OperandScalars {
  uint32_t xmax_bits;  // atomicMax target: bits of max x (or max|x|)
  uint32_t wmax_bits;
  float c_x;           // clip value actually used for X
  float c_w;
  uint32_t nonfinite;  // set when an operand maximum is Inf/NaN
  uint32_t pad[3];
};

// ---- profile.hip: optional event timing of every launch ------------------------
enum KernelId {
  KID_BEGIN = 0, KID_ABSMAX, KID_GRAD_PREPARE, KID_OPERAND_PREPARE, KID_FLAT_GRAD, KID_FLAT_OPERAND,
  KID_RELAYOUT_GRAD, KID_RELAYOUT_OPERAND, KID_GEMM_DX, KID_GEMM_DW, KID_ZERO, KID_FINALIZE,
  KID_UPDATE, KID_STATE, KID_COUNT
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

// ---- quantize.hip -------------------------------------------------------------
int launch_begin(lbt_grad_state* st, OperandScalars* sc, hipStream_t s);
int launch_absmax(const float* x, int64_t n, int use_abs, uint32_t* max_bits, hipStream_t s);
int launch_grad_prepare(lbt_grad_state* st, int64_t n, hipStream_t s);
int launch_operand_prepare(OperandScalars* sc, lbt_grad_state* st, float c_x, float c_w, hipStream_t s);
int launch_quantize_flat_grad(const float* g, int64_t n, lbt_grad_state* st, uint64_t seed,
                              int rounding, uint8_t* codes, hipStream_t s);
int launch_quantize_flat_operand(const float* x, int64_t n, const float* clip_ptr, int is_unsigned,
                                 uint8_t* codes, float* clip_scale_out, hipStream_t s);
// Quantize T[A][B][L] (L contiguous) into GEMM layouts: out_b [A][L][Bp] with the
// B axis innermost, out_a [B][L][Ap] with the A axis innermost (either may be null).
// Gradient flavour reads its clip value from *st and counts clip-outs; operand
// flavour reads the clip value from *clip_ptr.
int launch_quantize_relayout_grad(const float* g, int64_t A, int64_t B, int64_t L,
                                  lbt_grad_state* st, uint64_t seed, int rounding, uint8_t* out_b,
                                  uint8_t* out_a, hipStream_t s);
int launch_quantize_relayout_operand(const float* x, int64_t A, int64_t B, int64_t L,
                                     const float* clip_ptr, int is_unsigned, uint8_t* out_b,
                                     uint8_t* out_a, hipStream_t s);
int launch_update_interval(lbt_grad_state* st, hipStream_t s);
int launch_state_init(lbt_grad_state* st, const lbt_grad_state& v, hipStream_t s);

// ---- gemm.hip -----------------------------------------------------------------
struct ConvGeom {
  int N, C, H, W, K, R, S, P, Q, stride, pad;
  int Np, Kp;  // N and K rounded up to kGranule
};
// dX: A = W codes [C][R*S][Kp], B = dY codes [N][P*Q][Kp]; out/acc [N][C][H][W].
int launch_conv_dx(const ConvGeom& g, const uint8_t* w_crsk, const uint8_t* g_npqk,
                   const lbt_grad_state* st, const OperandScalars* sc, float* dX, int32_t* acc,
                   hipStream_t s);
// dW: A = dY codes [K][P*Q][Np], B = X codes [C][H*W][Np]; out/acc [K][C][R][S].
// out doubles as the int32 split-K accumulation buffer before the final scaling.
int launch_conv_dw(const ConvGeom& g, const uint8_t* g_kpqn, const uint8_t* x_chwn,
                   const lbt_grad_state* st, const OperandScalars* sc, int x_unsigned, float* dW,
                   int32_t* acc, hipStream_t s);

// Linear layer: A/B roles swapped so both outputs are written along their rows.
int launch_linear_dx(const ConvGeom& g, const uint8_t* w_ck, const uint8_t* g_nk,
                     const lbt_grad_state* st, const OperandScalars* sc, float* dX, int32_t* acc,
                     hipStream_t s);
int launch_linear_dw(const ConvGeom& g, const uint8_t* g_kn, const uint8_t* x_cn,
                     const lbt_grad_state* st, const OperandScalars* sc, int x_unsigned, float* dW,
                     int32_t* acc, hipStream_t s);

}  // namespace lbt
