// C ABI of liblbt.so: argument validation, workspace carving, kernel sequencing.
// Every call only enqueues work on the caller's stream (lbt_state_read excepted).
#include <mutex>

#include "lbt_internal.h"

using namespace lbt;

// Scratch of lbt_quantize_grad_static (the partial maxima and arrival counters that the other
// entry points keep in the caller's workspace): one copy per GPU, held until the process ends.
// The name is only a host-side handle: host code uses the address hipGetSymbolAddress returns.
static __device__ __align__(256) unsigned char scratch[kWsHeaderBytes];

namespace {

// Device address of `scratch` on the current device, looked up once per device.
int static_scratch(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr[kMaxDevices];
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess) return LBT_ERR_HIP;
  if (device < 0 || device >= kMaxDevices) return LBT_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[device]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LBT_ERR_HIP;
    ptr[device] = p;
  }
  *out = ptr[device];
  return LBT_OK;
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline size_t pad256(size_t b) { return (b + 255) / 256 * 256; }

struct ConvWorkspace {
  size_t off_scalars, off_g_npqk, off_g_kpqn, off_x_chwn, off_w_crsk, off_partial, total;
};

ConvWorkspace conv_workspace(const ConvGeom& g, bool is_linear) {
  ConvWorkspace w{};
  size_t o = 0;
  w.off_scalars = o;
  o += kWsHeaderBytes;
  w.off_g_npqk = o;
  o += pad256((size_t)g.N * g.P * g.Q * g.Kp);
  w.off_g_kpqn = o;
  o += pad256((size_t)g.K * g.P * g.Q * g.Np);
  w.off_x_chwn = o;
  o += pad256((size_t)g.C * g.H * g.W * g.Np);
  w.off_w_crsk = o;
  o += pad256((size_t)g.C * g.R * g.S * g.Kp);
  w.off_partial = o;
  const SplitPlan plan = is_linear
      ? plan_split_k(g.C, g.K, g.Np / kGranule)
      : plan_split_k(g.K, g.C * g.R * g.S, g.P * g.Q * (g.Np / kGranule));
  o += pad256(plan.partial_bytes);
  w.total = o;
  return w;
}

// Operand codes kept from the forward pass for the layer's backward call: a header like the
// workspace's (clip values and non-finite flags of X and W; partial maxima while saving),
// then X in the layout dW reads and W in the layout dX reads.
struct SavedLayout {
  size_t off_x, off_w, total;
};
SavedLayout saved_layout(const ConvGeom& g) {
  SavedLayout w{};
  size_t o = kWsHeaderBytes;
  w.off_x = o;
  o += pad256((size_t)g.C * g.H * g.W * g.Np);
  w.off_w = o;
  o += pad256((size_t)g.C * g.R * g.S * g.Kp);
  w.total = o;
  return w;
}

int make_geom(int64_t N, int64_t C, int64_t H, int64_t W, int64_t K, int64_t R, int64_t S,
              int64_t stride, int64_t pad, ConvGeom* out) {
  if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0)
    return LBT_ERR_SHAPE;
  if (H + 2 * pad < R || W + 2 * pad < S) return LBT_ERR_SHAPE;
  const int64_t P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
  const int64_t lim = 0x7fffffffll;
  if (N * C * H * W > lim || N * K * P * Q > lim || K * C * R * S > lim) return LBT_ERR_UNSUPPORTED;
  ConvGeom g;
  g.N = (int)N; g.C = (int)C; g.H = (int)H; g.W = (int)W; g.K = (int)K; g.R = (int)R; g.S = (int)S;
  g.P = (int)P; g.Q = (int)Q; g.stride = (int)stride; g.pad = (int)pad;
  g.Np = (int)round_up(N, kGranule);
  g.Kp = (int)round_up(K, kGranule);
  g.bits = 4;
  *out = g;
  return LBT_OK;
}

// Splits the flag word `rounding`: checks it, returns the bit-width (LBT_BITS field, 0 = 4).
bool split_flags(int rounding, int* bits) {
  const int known = LBT_ROUND_STOCHASTIC | LBT_HINDSIGHT_MAX | LBT_FUSED_UPDATE | LBT_BITS(15);
  if (rounding & ~known) return false;
  const int b = (rounding >> 8) & 15;
  *bits = b ? b : 4;
  return *bits >= 2 && *bits <= 8;
}

// w_is_ck: W is stored [C][K] (linear layer, [in][out]) instead of [K][C][R][S].
int backward_common(const float* X, const float* W, const float* dY, ConvGeom g,
                    bool w_is_ck, float c_x, int x_unsigned, float c_w, lbt_grad_state* st,
                    uint64_t seed, int rounding, float* dX, float* dW, int32_t* acc_dX,
                    int32_t* acc_dW, void* ws, size_t ws_bytes, void* stream,
                    const void* saved = nullptr, size_t saved_bytes = 0, float* grad_c = nullptr) {
  // grad_c (2 floats, may be null): the clip values are learned - dW and dX are masked with the
  // intervals of the weight / activation quantizers and grad_c receives dL/dc_w, dL/dc_x
  if (grad_c) {
    if (saved || !X || !W) return LBT_ERR_NULL;
    if (!aligned(grad_c, 4)) return LBT_ERR_ALIGN;
    if ((dW && !(c_w > 0.0f && c_w < INFINITY)) || (dX && !(c_x > 0.0f && c_x < INFINITY)))
      return LBT_ERR_UNSUPPORTED;
    // (bit-widths 2..8: an interval usable at the largest q is usable at every q)
    if ((dW && !interval_usable(c_w, 255)) || (dX && !interval_usable(c_x, 255)))
      return LBT_ERR_UNSUPPORTED;
  }
  // saved: X and W were quantized by a forward call (lbt_forward_*_save); X, W, c_x, c_w unused
  if (!dY || !st || !ws) return LBT_ERR_NULL;
  if (!saved && (!W || (dW && !X))) return LBT_ERR_NULL;
  if ((acc_dX && !dX) || (acc_dW && !dW)) return LBT_ERR_NULL;
  int bits;
  if (!split_flags(rounding, &bits)) return LBT_ERR_UNSUPPORTED;
  // unsigned 8-bit codes (0..255) do not fit the signed int8 operands of the matrix cores
  if (x_unsigned && dW && bits == 8) return LBT_ERR_UNSUPPORTED;
  g.bits = bits;
  const int hindsight = (rounding & LBT_HINDSIGHT_MAX) ? 1 : 0;
  const int fused_update = (rounding & LBT_FUSED_UPDATE) ? 1 : 0;
  rounding &= LBT_ROUND_STOCHASTIC;
  if (!aligned(dY, 16) || (W && !aligned(W, 16)) || (X && !aligned(X, 16)) || !aligned(ws, 256) ||
      (dX && !aligned(dX, 16)) || (dW && !aligned(dW, 16)) || !aligned(st, 8) ||
      (saved && !aligned(saved, 256)))
    return LBT_ERR_ALIGN;
  const ConvWorkspace lay = conv_workspace(g, w_is_ck);
  if (ws_bytes < lay.total) return LBT_ERR_WORKSPACE;
  const SavedLayout kept = saved_layout(g);
  if (saved && saved_bytes < kept.total) return LBT_ERR_WORKSPACE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  uint8_t* base = static_cast<uint8_t*>(ws);
  OperandScalars* sc = reinterpret_cast<OperandScalars*>(base + lay.off_scalars);
  uint8_t* g_npqk = base + lay.off_g_npqk;
  uint8_t* g_kpqn = base + lay.off_g_kpqn;
  uint8_t* x_chwn = base + lay.off_x_chwn;
  uint8_t* w_crsk = base + lay.off_w_crsk;
  int32_t* partial = reinterpret_cast<int32_t*>(base + lay.off_partial);
  if (saved) {
    uint8_t* kept_base = const_cast<uint8_t*>(static_cast<const uint8_t*>(saved));
    sc = reinterpret_cast<OperandScalars*>(kept_base);
    x_chwn = kept_base + kept.off_x;
    w_crsk = kept_base + kept.off_w;
  }

  uint32_t* pmax = header_pmax(base);
  unsigned long long* tickets = header_tickets(base);
  const int64_t n_dy = (int64_t)g.N * g.K * g.P * g.Q;
  const int64_t n_x = (int64_t)g.N * g.C * g.H * g.W;
  const int64_t n_w = (int64_t)g.K * g.C * g.R * g.S;
  const int64_t PQ = (int64_t)g.P * g.Q, HW = (int64_t)g.H * g.W, RS = (int64_t)g.R * g.S;
  int rc, nblocks = 0;
  const bool want_cw = !saved && dX && !(c_w > 0.0f), want_cx = !saved && dW && !(c_x > 0.0f);
  // Tensor shapes as the re-layout sees them: T[A][B][L], L contiguous
  const int64_t wA = w_is_ck ? g.C : g.K, wB = w_is_ck ? g.K : g.C, wL = w_is_ck ? 1 : RS;
  // 1. maxima of dY (unless the previous tensor's maximum is to be used), and of X / W where
  //    no clip value was given, in one launch
  if ((rc = launch_absmax3(hindsight ? nullptr : dY, n_dy, 1, want_cx ? X : nullptr, n_x, x_unsigned ? 0 : 1,
                           want_cw ? W : nullptr, n_w, 1, pmax, tickets, &nblocks, st, s,
                           saved ? sc : nullptr, (dW ? 1 : 0) | (dX ? 2 : 0))))
    return rc;
  // 2. codes of all three tensors in the layouts the two products read, one launch:
  //    gradient for both products, activations for dW, weights for dX (convolution weights
  //    tap-major [C][R*S][Kp/16][16]: the dX kernel walks the contraction tap by tap)
  {
    LayerTensors q{};
    q.seed = seed;
    q.rounding = rounding;
    q.hindsight = hindsight;
    q.bits = bits;
    q.x_unsigned = x_unsigned;
    q.tensor[0] = {dY, g.N, g.K, PQ,
                   RelayoutIo{pmax, nblocks, 0, tickets, st, dX ? g_npqk : nullptr, dW ? g_kpqn : nullptr, 0},
                   0.0f, nullptr, nullptr};
    if (dW && !saved)
      q.tensor[1] = {X, g.N, g.C, HW, RelayoutIo{pmax, nblocks, 1, tickets, st, nullptr, x_chwn, 0},
                     c_x, &sc->c_x, &sc->bad_x};
    if (dX && !saved)
      q.tensor[2] = {W, wA, wB, wL,
                     RelayoutIo{pmax, nblocks, 2, tickets, st, w_is_ck ? w_crsk : nullptr,
                                w_is_ck ? nullptr : w_crsk, 1},
                     c_w, &sc->c_w, &sc->bad_w};
    if ((rc = launch_quantize_layer(q, s))) return rc;
  }
  // 3. the two products, dW first (measured: its operands are then still where the quantizer
  //    left them, and the large streaming write of dX comes last; -0.03 ms per ResNet-50 step);
  //    with LBT_FUSED_UPDATE the last launch also applies Alg. 1 (the quantizers, all of which
  //    can change the status, have finished by then)
  lbt_grad_state* const upd = fused_update ? st : nullptr;
  // partial sums of the two clip-value gradients: the two halves of the partial-maxima area
  static_assert(2 * (size_t)kStePartials * sizeof(double) <= kWsHeaderBytes - kWsScalarsBytes,
                "both passes' partial sums must fit the header");
  double* const ste_w = reinterpret_cast<double*>(pmax);
  double* const ste_x = ste_w + kStePartials;
  // dW's split-K sum is carried out by extra workgroups of the dX launch (one launch and one
  // launch gap less per layer), unless the masked dW is needed before dX (learned clips) or
  // no dX follows
  PendingReduce pending{};
  if (dW) {
    lbt_grad_state* const u = dX ? nullptr : upd;
    PendingReduce* const defer = (dX && !grad_c) ? &pending : nullptr;
    rc = w_is_ck ? launch_linear_dw(g, g_kpqn, x_chwn, st, sc, x_unsigned, dW, acc_dW, partial, u, defer, s)
                 : launch_conv_dw(g, g_kpqn, x_chwn, st, sc, x_unsigned, dW, acc_dW, partial, u, defer, s);
    if (rc) return rc;
    // dW is dL/dQ(W) and has W's layout: its mask and dL/dc_w (the partial-maxima area of the
    // header is free again once the quantizers have run: scratch of the pass's partial sums)
    if (grad_c && (rc = launch_ste_backward(W, dW, n_w, c_w, 0, bits, dW, nullptr, ste_w, s, false)))
      return rc;
  }
  if (dX) {
    const PendingReduce* const carry = pending.blocks ? &pending : nullptr;
    rc = w_is_ck ? launch_linear_dx(g, w_crsk, g_npqk, st, sc, dX, acc_dX, upd, carry, s)
                 : launch_conv_dx(g, w_crsk, g_npqk, st, sc, dX, acc_dX, upd, carry, s);
    if (rc) return rc;
    // dX is dL/dQ(X) and has X's layout.  (The mask applied in the product's epilogue instead
    // was measured: the product then takes 1.5 ms more per ResNet-50 step, this pass 1.3 ms.)
    if (grad_c && (rc = launch_ste_backward(X, dX, n_x, c_x, x_unsigned, bits, dX, nullptr, ste_x, s,
                                            false)))
      return rc;
  }
  // the sums of both passes in one launch
  if (grad_c && dW && dX && (rc = launch_ste_finish(ste_w, n_w, grad_c, ste_x, n_x, grad_c + 1, s)))
    return rc;
  if (grad_c && dW && !dX && (rc = launch_ste_finish(ste_w, n_w, grad_c, nullptr, 0, nullptr, s)))
    return rc;
  if (grad_c && dX && !dW && (rc = launch_ste_finish(ste_x, n_x, grad_c + 1, nullptr, 0, nullptr, s)))
    return rc;
  if (upd && !dX && !dW && (rc = launch_update_interval(st, s))) return rc;
  return LBT_OK;
}

// Forward product: maxima where no clip value is given, both operands quantized in one
// launch into the layouts the product reads, then the product.
//   linear: X as T[M][K_in][1] -> [M][Kin_p/16][16]; W as T[K_in][N_out][1] -> [N_out][Kin_p/16][16]
//   conv:   X as T[N][C][H*W]  -> [N][Cp/16][H*W][16]; W as T[K][C][R*S] -> [K][R*S][Cp/16][16]
struct ForwardWorkspace {
  size_t off_x, off_w, total;
};
ForwardWorkspace forward_workspace(const ConvGeom& g) {
  ForwardWorkspace w;
  const size_t cp = (size_t)round_up(g.C, kGranule);
  size_t o = kWsHeaderBytes;
  w.off_x = o;
  o += pad256((size_t)g.N * g.H * g.W * cp);
  w.off_w = o;
  o += pad256((size_t)g.K * g.R * g.S * cp);
  w.total = o;
  return w;
}

int forward_common(const float* X, const float* W, ConvGeom g, bool is_linear, float c_x,
                   int x_unsigned, float c_w, int flags, float* Y, int32_t* acc_Y, int32_t* status,
                   void* ws, size_t ws_bytes, void* stream, void* saved = nullptr,
                   size_t saved_bytes = 0, bool save_call = false) {
  // save_call: the codes the backward products read are also written to `saved`; Y may then be
  // NULL (no product, no workspace: the maxima go through the header of `saved`)
  const bool product = Y != nullptr;
  if (!X || !W) return LBT_ERR_NULL;
  if (!save_call && (!Y || !ws)) return LBT_ERR_NULL;
  if (save_call && (!saved || (product && !ws) || (!product && (acc_Y || status)))) return LBT_ERR_NULL;
  int bits;
  if ((flags & ~LBT_BITS(15)) || !split_flags(flags, &bits)) return LBT_ERR_UNSUPPORTED;
  if (x_unsigned && bits == 8) return LBT_ERR_UNSUPPORTED;
  g.bits = bits;
  if (!aligned(X, 16) || !aligned(W, 16) || (Y && !aligned(Y, 16)) || (ws && !aligned(ws, 256)) ||
      (acc_Y && !aligned(acc_Y, 16)) || (status && !aligned(status, 4)) ||
      (saved && !aligned(saved, 256)))
    return LBT_ERR_ALIGN;
  const ForwardWorkspace lay = forward_workspace(g);
  if (product && ws_bytes < lay.total) return LBT_ERR_WORKSPACE;
  const SavedLayout kept = saved_layout(g);
  if (saved && saved_bytes < kept.total) return LBT_ERR_WORKSPACE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  // scalars and partial maxima: in the header of `saved` when there is one (the backward call
  // reads the clip values there), else in the workspace
  uint8_t* head = saved ? static_cast<uint8_t*>(saved) : static_cast<uint8_t*>(ws);
  OperandScalars* sc = reinterpret_cast<OperandScalars*>(head);
  uint32_t* pmax = header_pmax(head);
  unsigned long long* tickets = header_tickets(head);
  uint8_t* x_codes = product ? static_cast<uint8_t*>(ws) + lay.off_x : nullptr;
  uint8_t* w_codes = product ? static_cast<uint8_t*>(ws) + lay.off_w : nullptr;
  uint8_t* x_kept = saved ? static_cast<uint8_t*>(saved) + kept.off_x : nullptr;   // [C][Np/16][HW][16]
  uint8_t* w_kept = saved ? static_cast<uint8_t*>(saved) + kept.off_w : nullptr;   // [C][RS][Kp/16][16]
  const int64_t HW = (int64_t)g.H * g.W, RS = (int64_t)g.R * g.S;
  const int64_t n_x = (int64_t)g.N * g.C * HW, n_w = (int64_t)g.K * g.C * RS;
  int rc, nblocks = 0;
  if ((rc = launch_absmax3(nullptr, 0, 0, !(c_x > 0.0f) ? X : nullptr, n_x, x_unsigned ? 0 : 1,
                           !(c_w > 0.0f) ? W : nullptr, n_w, 1, pmax, tickets, &nblocks, nullptr, s)))
    return rc;
  LayerTensors q{};
  q.rounding = LBT_ROUND_NEAREST;
  q.x_unsigned = x_unsigned;
  q.bits = bits;
  q.tensor[1] = {X, g.N, g.C, HW, RelayoutIo{pmax, nblocks, 1, tickets, nullptr, x_codes, x_kept, 0, 0},
                 c_x, &sc->c_x, &sc->bad_x};
  if (is_linear)   // W[K_in][N_out]: rows of W^T, sixteen consecutive k_in per granule;
                   // kept for dX as rows of W, sixteen consecutive n_out per granule
    q.tensor[2] = {W, g.C, g.K, 1, RelayoutIo{pmax, nblocks, 2, tickets, nullptr, w_kept, w_codes, 0, 0},
                   c_w, &sc->c_w, &sc->bad_w};
  else             // W[K][C][R*S]: tap-major rows, sixteen consecutive c per granule;
                   // kept for dX tap-major with sixteen consecutive k per granule
    q.tensor[2] = {W, g.K, g.C, RS, RelayoutIo{pmax, nblocks, 2, tickets, nullptr, w_codes, w_kept, 1, 1},
                   c_w, &sc->c_w, &sc->bad_w};
  if ((rc = launch_quantize_layer(q, s))) return rc;
  if (!product) return LBT_OK;
  return is_linear ? launch_linear_fwd(g.N, g.C, g.K, bits, x_codes, w_codes, sc, x_unsigned, Y, acc_Y,
                                       status, s)
                   : launch_conv_fwd(g, w_codes, x_codes, sc, x_unsigned, Y, acc_Y, status, s);
}

}  // namespace

extern "C" {

const char* lbt_version(void) { return "lbt-gfx950 0.1"; }

const char* lbt_strerror(int code) {
  switch (code) {
    case LBT_OK: return "ok";
    case LBT_ERR_NULL: return "null pointer";
    case LBT_ERR_SHAPE: return "bad shape";
    case LBT_ERR_UNSUPPORTED: return "unsupported configuration";
    case LBT_ERR_WORKSPACE: return "workspace too small";
    case LBT_ERR_OVERFLOW: return "contraction may overflow int32";
    case LBT_ERR_HIP: return "HIP runtime error";
    case LBT_ERR_ALIGN: return "misaligned pointer";
    case LBT_ERR_TOO_LARGE: return "tensor larger than the static scratch serves";
    default: return "unknown error";
  }
}

size_t lbt_state_sizeof(void) { return sizeof(lbt_grad_state); }

int lbt_state_init(lbt_grad_state* st, double gamma0, double alpha, double beta, double gamma_min,
                   double gamma_max, int bits, void* stream) {
  if (!st) return LBT_ERR_NULL;
  if (!aligned(st, 8)) return LBT_ERR_ALIGN;
  if (bits < 2 || bits > 8) return LBT_ERR_UNSUPPORTED;
  if (!(gamma_min > 0.0) || !(gamma_max >= gamma_min) || !(gamma0 >= gamma_min) ||
      !(gamma0 <= gamma_max) || !(alpha > 0.0) || !(beta >= 0.0))
    return LBT_ERR_SHAPE;
  lbt_grad_state v{};  // sync_word = 0: no quantizer in flight
  v.gamma = gamma0; v.alpha = alpha; v.beta = beta;
  v.gamma_min = gamma_min; v.gamma_max = gamma_max;
  v.bits = bits;
  return launch_state_init(st, v, reinterpret_cast<hipStream_t>(stream));
}

int lbt_state_read(const lbt_grad_state* st, lbt_grad_state* host_out, void* stream) {
  if (!st || !host_out) return LBT_ERR_NULL;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  LBT_HIP_CHECK(hipMemcpyAsync(host_out, st, sizeof(lbt_grad_state), hipMemcpyDeviceToHost, s));
  LBT_HIP_CHECK(hipStreamSynchronize(s));
  return LBT_OK;
}

int lbt_state_write(lbt_grad_state* st, const lbt_grad_state* host_in, void* stream) {
  if (!st || !host_in) return LBT_ERR_NULL;
  if (host_in->bits < 2 || host_in->bits > 8) return LBT_ERR_UNSUPPORTED;
  lbt_grad_state v = *host_in;
  v.sync_word = 0;
  v.sync_max = 0;
  return launch_state_init(st, v, reinterpret_cast<hipStream_t>(stream));
}

int lbt_update_interval(lbt_grad_state* st, void* stream) {
  if (!st) return LBT_ERR_NULL;
  return launch_update_interval(st, reinterpret_cast<hipStream_t>(stream));
}

size_t lbt_workspace_bytes_quantize(int64_t n) {
  (void)n;
  return kWsHeaderBytes;
}

int lbt_quantize_grad(const float* g, int64_t n, lbt_grad_state* st, uint64_t seed, int rounding,
                      uint8_t* codes, void* ws, size_t ws_bytes, void* stream) {
  if (!g || !st || !codes || !ws) return LBT_ERR_NULL;
  if (n <= 0) return LBT_ERR_SHAPE;
  int bits;
  if (!split_flags(rounding, &bits)) return LBT_ERR_UNSUPPORTED;
  const int hindsight = (rounding & LBT_HINDSIGHT_MAX) ? 1 : 0;
  const int fused_update = (rounding & LBT_FUSED_UPDATE) ? 1 : 0;
  rounding &= LBT_ROUND_STOCHASTIC;
  if (!aligned(g, 16) || !aligned(codes, bits > 4 ? 8 : 4) || !aligned(st, 8) || !aligned(ws, 256))
    return LBT_ERR_ALIGN;
  if (ws_bytes < lbt_workspace_bytes_quantize(n)) return LBT_ERR_WORKSPACE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  uint32_t* pmax = header_pmax(ws);
  unsigned long long* tickets = header_tickets(ws);
  int rc, nblocks = 0;
  if ((rc = launch_absmax3(hindsight ? nullptr : g, n, 1, nullptr, 0, 0, nullptr, 0, 0, pmax, tickets,
                           &nblocks, st, s)))
    return rc;
  return launch_quantize_flat_grad(g, n, pmax, nblocks, tickets, st, seed, rounding, hindsight, fused_update,
                                   bits, codes, s);
}

int lbt_quantize_grad_static(const float* g, int64_t n, lbt_grad_state* st, uint64_t seed,
                             int rounding, uint8_t* codes, void* stream) {
  if (!g || !st || !codes) return LBT_ERR_NULL;
  if (n <= 0) return LBT_ERR_SHAPE;
  if (n > LBT_QUANTIZE_STATIC_MAX_N) return LBT_ERR_TOO_LARGE;
  static_assert(sizeof(scratch) >= kWsHeaderBytes, "scratch must hold a workspace header");
  void* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc) return rc;
  // the same kernels as lbt_quantize_grad, on this GPU's static scratch; nothing in it has to
  // start at zero (the maximum kernel resets the counters it shares with the quantizer)
  return lbt_quantize_grad(g, n, st, seed, rounding, codes, ws, sizeof(scratch), stream);
}

int lbt_quantize_operand(const float* x, int64_t n, float c, int is_unsigned, int bits,
                         uint8_t* codes, float* clip_scale_out, void* ws, size_t ws_bytes,
                         void* stream) {
  if (!x || !codes || !ws) return LBT_ERR_NULL;
  if (n <= 0) return LBT_ERR_SHAPE;
  if (bits < 2 || bits > 8) return LBT_ERR_UNSUPPORTED;
  if (!aligned(x, 16) || !aligned(codes, bits > 4 ? 8 : 4) || !aligned(ws, 256)) return LBT_ERR_ALIGN;
  if (ws_bytes < lbt_workspace_bytes_quantize(n)) return LBT_ERR_WORKSPACE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  OperandScalars* sc = static_cast<OperandScalars*>(ws);
  uint32_t* pmax = header_pmax(ws);
  int rc, nblocks = 0;
  if (!(c > 0.0f))
    if ((rc = launch_absmax3(nullptr, 0, 0, x, n, is_unsigned ? 0 : 1, nullptr, 0, 0, pmax,
                             header_tickets(ws), &nblocks, nullptr, s)))
      return rc;
  return launch_quantize_flat_operand(x, n, c, pmax, nblocks, is_unsigned, bits, codes, &sc->c_x,
                                      clip_scale_out, s);
}

int lbt_ste_backward(const float* x, int64_t n, float c, int is_unsigned, int bits,
                     const float* grad_q, float* grad_x, float* grad_c, void* ws, size_t ws_bytes,
                     void* stream) {
  if (!x || !grad_q || !ws) return LBT_ERR_NULL;
  if (n <= 0) return LBT_ERR_SHAPE;
  if (bits < 2 || bits > 8 || !(c < INFINITY) || !interval_usable(c, levels(bits, is_unsigned != 0)))
    return LBT_ERR_UNSUPPORTED;
  if (!aligned(x, 16) || !aligned(grad_q, 16) || (grad_x && !aligned(grad_x, 16)) ||
      (grad_c && !aligned(grad_c, 4)) || !aligned(ws, 256))
    return LBT_ERR_ALIGN;
  if (ws_bytes < lbt_workspace_bytes_quantize(n)) return LBT_ERR_WORKSPACE;
  static_assert((size_t)kStePartials * sizeof(double) <= kWsHeaderBytes - kWsScalarsBytes,
                "partial sums must fit the header");
  double* partial = reinterpret_cast<double*>(static_cast<uint8_t*>(ws) + kWsScalarsBytes);
  return launch_ste_backward(x, grad_q, n, c, is_unsigned, bits, grad_x, grad_c, partial,
                             reinterpret_cast<hipStream_t>(stream));
}

size_t lbt_workspace_bytes_conv2d(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R,
                                  int64_t S, int64_t stride, int64_t pad) {
  ConvGeom g;
  if (make_geom(N, C, H, Wd, K, R, S, stride, pad, &g) != LBT_OK) return 0;
  return conv_workspace(g, false).total;
}

size_t lbt_workspace_bytes_linear(int64_t M, int64_t K_in, int64_t N_out) {
  ConvGeom g;
  if (make_geom(M, K_in, 1, 1, N_out, 1, 1, 1, 0, &g) != LBT_OK) return 0;
  return conv_workspace(g, true).total;
}

size_t lbt_workspace_bytes_forward_conv2d(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K,
                                          int64_t R, int64_t S, int64_t stride, int64_t pad) {
  ConvGeom g;
  if (make_geom(N, C, H, Wd, K, R, S, stride, pad, &g) != LBT_OK) return 0;
  return forward_workspace(g).total;
}

size_t lbt_workspace_bytes_forward_linear(int64_t M, int64_t K_in, int64_t N_out) {
  ConvGeom g;
  if (make_geom(M, K_in, 1, 1, N_out, 1, 1, 1, 0, &g) != LBT_OK) return 0;
  return forward_workspace(g).total;
}

int lbt_forward_conv2d(const float* X, const float* W, int64_t N, int64_t C, int64_t H, int64_t Wd,
                       int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad, float c_x,
                       int x_unsigned, float c_w, int flags, float* Y, int32_t* acc_Y,
                       int32_t* status, void* ws, size_t ws_bytes, void* stream) {
  ConvGeom g;
  const int rc = make_geom(N, C, H, Wd, K, R, S, stride, pad, &g);
  if (rc) return rc;
  return forward_common(X, W, g, false, c_x, x_unsigned, c_w, flags, Y, acc_Y, status, ws, ws_bytes,
                        stream);
}

int lbt_forward_linear(const float* X, const float* W, int64_t M, int64_t K_in, int64_t N_out,
                       float c_x, int x_unsigned, float c_w, int flags, float* Y, int32_t* acc_Y,
                       int32_t* status, void* ws, size_t ws_bytes, void* stream) {
  ConvGeom g;
  const int rc = make_geom(M, K_in, 1, 1, N_out, 1, 1, 1, 0, &g);
  if (rc) return rc;
  return forward_common(X, W, g, true, c_x, x_unsigned, c_w, flags, Y, acc_Y, status, ws, ws_bytes,
                        stream);
}

size_t lbt_saved_bytes_conv2d(int64_t N, int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R,
                              int64_t S, int64_t stride, int64_t pad) {
  ConvGeom g;
  if (make_geom(N, C, H, Wd, K, R, S, stride, pad, &g) != LBT_OK) return 0;
  return saved_layout(g).total;
}

size_t lbt_saved_bytes_linear(int64_t M, int64_t K_in, int64_t N_out) {
  ConvGeom g;
  if (make_geom(M, K_in, 1, 1, N_out, 1, 1, 1, 0, &g) != LBT_OK) return 0;
  return saved_layout(g).total;
}

int lbt_forward_conv2d_save(const float* X, const float* W, int64_t N, int64_t C, int64_t H,
                            int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t stride, int64_t pad,
                            float c_x, int x_unsigned, float c_w, int flags, float* Y, int32_t* acc_Y,
                            int32_t* status, void* saved, size_t saved_bytes, void* ws,
                            size_t ws_bytes, void* stream) {
  ConvGeom g;
  const int rc = make_geom(N, C, H, Wd, K, R, S, stride, pad, &g);
  if (rc) return rc;
  return forward_common(X, W, g, false, c_x, x_unsigned, c_w, flags, Y, acc_Y, status, ws, ws_bytes,
                        stream, saved, saved_bytes, true);
}

int lbt_forward_linear_save(const float* X, const float* W, int64_t M, int64_t K_in, int64_t N_out,
                            float c_x, int x_unsigned, float c_w, int flags, float* Y, int32_t* acc_Y,
                            int32_t* status, void* saved, size_t saved_bytes, void* ws,
                            size_t ws_bytes, void* stream) {
  ConvGeom g;
  const int rc = make_geom(M, K_in, 1, 1, N_out, 1, 1, 1, 0, &g);
  if (rc) return rc;
  return forward_common(X, W, g, true, c_x, x_unsigned, c_w, flags, Y, acc_Y, status, ws, ws_bytes,
                        stream, saved, saved_bytes, true);
}

int lbt_backward_conv2d_saved(const void* saved, size_t saved_bytes, const float* dY, int64_t N,
                              int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                              int64_t stride, int64_t pad, int x_unsigned, lbt_grad_state* st,
                              uint64_t seed, int rounding, float* dX, float* dW, int32_t* acc_dX,
                              int32_t* acc_dW, void* ws, size_t ws_bytes, void* stream) {
  if (!saved) return LBT_ERR_NULL;
  ConvGeom g;
  int rc = make_geom(N, C, H, Wd, K, R, S, stride, pad, &g);
  if (rc) return rc;
  return backward_common(nullptr, nullptr, dY, g, false, 0.0f, x_unsigned, 0.0f, st, seed, rounding,
                         dX, dW, acc_dX, acc_dW, ws, ws_bytes, stream, saved, saved_bytes);
}

int lbt_backward_linear_saved(const void* saved, size_t saved_bytes, const float* dY, int64_t M,
                              int64_t K_in, int64_t N_out, int x_unsigned, lbt_grad_state* st,
                              uint64_t seed, int rounding, float* dX, float* dW, int32_t* acc_dX,
                              int32_t* acc_dW, void* ws, size_t ws_bytes, void* stream) {
  if (!saved) return LBT_ERR_NULL;
  ConvGeom g;
  int rc = make_geom(M, K_in, 1, 1, N_out, 1, 1, 1, 0, &g);
  if (rc) return rc;
  return backward_common(nullptr, nullptr, dY, g, true, 0.0f, x_unsigned, 0.0f, st, seed, rounding,
                         dX, dW, acc_dX, acc_dW, ws, ws_bytes, stream, saved, saved_bytes);
}

int lbt_backward_conv2d_learned(const float* X, const float* W, const float* dY, int64_t N,
                                int64_t C, int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S,
                                int64_t stride, int64_t pad, float c_x, int x_unsigned, float c_w,
                                lbt_grad_state* st, uint64_t seed, int rounding, float* dX,
                                float* dW, float* grad_c, void* ws, size_t ws_bytes, void* stream) {
  if (!grad_c) return LBT_ERR_NULL;
  ConvGeom g;
  int rc = make_geom(N, C, H, Wd, K, R, S, stride, pad, &g);
  if (rc) return rc;
  return backward_common(X, W, dY, g, false, c_x, x_unsigned, c_w, st, seed, rounding, dX, dW,
                         nullptr, nullptr, ws, ws_bytes, stream, nullptr, 0, grad_c);
}

int lbt_backward_linear_learned(const float* X, const float* W, const float* dY, int64_t M,
                                int64_t K_in, int64_t N_out, float c_x, int x_unsigned, float c_w,
                                lbt_grad_state* st, uint64_t seed, int rounding, float* dX,
                                float* dW, float* grad_c, void* ws, size_t ws_bytes, void* stream) {
  if (!grad_c) return LBT_ERR_NULL;
  ConvGeom g;
  int rc = make_geom(M, K_in, 1, 1, N_out, 1, 1, 1, 0, &g);
  if (rc) return rc;
  return backward_common(X, W, dY, g, true, c_x, x_unsigned, c_w, st, seed, rounding, dX, dW,
                         nullptr, nullptr, ws, ws_bytes, stream, nullptr, 0, grad_c);
}

int lbt_backward_conv2d_acc(const float* X, const float* W, const float* dY, int64_t N, int64_t C,
                            int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t stride,
                            int64_t pad, float c_x, int x_unsigned, float c_w, lbt_grad_state* st,
                            uint64_t seed, int rounding, float* dX, float* dW, int32_t* acc_dX,
                            int32_t* acc_dW, void* ws, size_t ws_bytes, void* stream) {
  ConvGeom g;
  int rc = make_geom(N, C, H, Wd, K, R, S, stride, pad, &g);
  if (rc) return rc;
  return backward_common(X, W, dY, g, false, c_x, x_unsigned, c_w, st, seed, rounding, dX, dW,
                         acc_dX, acc_dW, ws, ws_bytes, stream);
}

int lbt_backward_conv2d(const float* X, const float* W, const float* dY, int64_t N, int64_t C,
                        int64_t H, int64_t Wd, int64_t K, int64_t R, int64_t S, int64_t stride,
                        int64_t pad, float c_x, int x_unsigned, float c_w, lbt_grad_state* st,
                        uint64_t seed, int rounding, float* dX, float* dW, void* ws, size_t ws_bytes,
                        void* stream) {
  return lbt_backward_conv2d_acc(X, W, dY, N, C, H, Wd, K, R, S, stride, pad, c_x, x_unsigned, c_w,
                                 st, seed, rounding, dX, dW, nullptr, nullptr, ws, ws_bytes, stream);
}

int lbt_backward_linear_acc(const float* X, const float* W, const float* dY, int64_t M, int64_t K_in,
                            int64_t N_out, float c_x, int x_unsigned, float c_w, lbt_grad_state* st,
                            uint64_t seed, int rounding, float* dX, float* dW, int32_t* acc_dX,
                            int32_t* acc_dW, void* ws, size_t ws_bytes, void* stream) {
  // a linear layer is a 1x1 convolution on a 1x1 image: N = M, C = K_in, K = N_out
  ConvGeom g;
  int rc = make_geom(M, K_in, 1, 1, N_out, 1, 1, 1, 0, &g);
  if (rc) return rc;
  return backward_common(X, W, dY, g, true, c_x, x_unsigned, c_w, st, seed, rounding, dX, dW,
                         acc_dX, acc_dW, ws, ws_bytes, stream);
}

int lbt_backward_linear(const float* X, const float* W, const float* dY, int64_t M, int64_t K_in,
                        int64_t N_out, float c_x, int x_unsigned, float c_w, lbt_grad_state* st,
                        uint64_t seed, int rounding, float* dX, float* dW, void* ws, size_t ws_bytes,
                        void* stream) {
  return lbt_backward_linear_acc(X, W, dY, M, K_in, N_out, c_x, x_unsigned, c_w, st, seed, rounding,
                                 dX, dW, nullptr, nullptr, ws, ws_bytes, stream);
}

}  // extern "C"
