// Host-side validation of the C ABI under AddressSanitizer / UndefinedBehaviorSanitizer.
// Linked against a host-only build of the library (no device code): every call below must
// return its error code before anything reaches the GPU runtime.  Exit status 0 = all as
// expected; the sanitizers abort the process on any finding.
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "lbt.h"

static int failures = 0;
#define EXPECT(call, want)                                                      \
  do {                                                                          \
    const long long got_ = (long long)(call);                                   \
    if (got_ != (long long)(want)) {                                            \
      std::printf("%s:%d: %s = %lld, want %lld\n", __FILE__, __LINE__, #call, got_, (long long)(want)); \
      ++failures;                                                               \
    }                                                                           \
  } while (0)

int main() {
  float* p = reinterpret_cast<float*>(4096);            // never dereferenced on the host
  uint8_t* b = reinterpret_cast<uint8_t*>(4096);
  lbt_grad_state* st = reinterpret_cast<lbt_grad_state*>(4096);
  void* ws = reinterpret_cast<void*>(4096);
  const size_t big = (size_t)1 << 40;

  EXPECT(std::strcmp(lbt_strerror(LBT_OK), "ok"), 0);
  for (int code = -12; code <= 1; ++code) EXPECT(lbt_strerror(code) != nullptr, 1);
  EXPECT(lbt_state_sizeof(), 96);
  EXPECT(lbt_update_interval(nullptr, nullptr), LBT_ERR_NULL);
  EXPECT(lbt_state_init(nullptr, 1, 1e-3, 1e-3, 1e-3, 1, 4, nullptr), LBT_ERR_NULL);
  EXPECT(lbt_state_init(st, 1, 1e-3, 1e-3, 1e-3, 1, 9, nullptr), LBT_ERR_UNSUPPORTED);
  EXPECT(lbt_state_init(st, 2, 1e-3, 1e-3, 1e-3, 1, 4, nullptr), LBT_ERR_SHAPE);
  EXPECT(lbt_state_read(nullptr, nullptr, nullptr), LBT_ERR_NULL);
  lbt_grad_state host{};
  host.bits = 11;
  EXPECT(lbt_state_write(st, &host, nullptr), LBT_ERR_UNSUPPORTED);

  EXPECT(lbt_workspace_bytes_quantize(8), 256 + 2048 * 16);
  EXPECT(lbt_quantize_grad(nullptr, 8, st, 0, 0, b, ws, big, nullptr), LBT_ERR_NULL);
  EXPECT(lbt_quantize_grad(p, 0, st, 0, 0, b, ws, big, nullptr), LBT_ERR_SHAPE);
  EXPECT(lbt_quantize_grad(p, -5, st, 0, 0, b, ws, big, nullptr), LBT_ERR_SHAPE);
  EXPECT(lbt_quantize_grad(p, 8, st, 0, 8, b, ws, big, nullptr), LBT_ERR_UNSUPPORTED);
  EXPECT(lbt_quantize_grad(p, 8, st, 0, LBT_BITS(9), b, ws, big, nullptr), LBT_ERR_UNSUPPORTED);
  EXPECT(lbt_quantize_grad(p + 1, 8, st, 0, 0, b, ws, big, nullptr), LBT_ERR_ALIGN);
  EXPECT(lbt_quantize_grad(p, 8, st, 0, 0, b, ws, 16, nullptr), LBT_ERR_WORKSPACE);
  EXPECT(lbt_quantize_grad_static(p, LBT_QUANTIZE_STATIC_MAX_N + 1, st, 0, 0, b, nullptr), LBT_ERR_TOO_LARGE);
  EXPECT(lbt_quantize_grad_static(p, INT64_MAX, st, 0, 0, b, nullptr), LBT_ERR_TOO_LARGE);
  EXPECT(lbt_quantize_grad_static(p, 0, st, 0, 0, b, nullptr), LBT_ERR_SHAPE);
  EXPECT(lbt_quantize_operand(p, 8, 1.0f, 0, 1, b, nullptr, ws, big, nullptr), LBT_ERR_UNSUPPORTED);
  EXPECT(lbt_quantize_operand(p, 8, 1.0f, 0, 4, b, nullptr, ws, 0, nullptr), LBT_ERR_WORKSPACE);
  EXPECT(lbt_ste_backward(p, 8, 0.0f, 0, 4, p, p, p, ws, big, nullptr), LBT_ERR_UNSUPPORTED);
  EXPECT(lbt_ste_backward(p, 8, 1e-41f, 0, 4, p, p, p, ws, big, nullptr), LBT_ERR_UNSUPPORTED);

  // shapes: zero, negative, kernel larger than the padded image, sizes beyond 32 bits
  EXPECT(lbt_workspace_bytes_conv2d(1, 1, 2, 2, 1, 3, 3, 1, 0), 0);
  EXPECT(lbt_workspace_bytes_conv2d(0, 1, 2, 2, 1, 1, 1, 1, 0), 0);
  EXPECT(lbt_workspace_bytes_conv2d((int64_t)1 << 40, 64, 56, 56, 64, 3, 3, 1, 1), 0);
  EXPECT(lbt_workspace_bytes_linear(-1, 4, 4), 0);
  const size_t need = lbt_workspace_bytes_conv2d(4, 16, 12, 12, 32, 3, 3, 1, 1);
  EXPECT(need > 0 && need % 256 == 0, 1);
  EXPECT(lbt_backward_conv2d(p, p, p, 4, 16, 12, 12, 32, 3, 3, 1, 1, 0, 1, 0, st, 0, 0, p, p, ws, need - 1, nullptr),
         LBT_ERR_WORKSPACE);
  EXPECT(lbt_backward_conv2d(p, p, p, 4, 16, 12, 12, 32, 3, 3, 0, 1, 0, 1, 0, st, 0, 0, p, p, ws, need, nullptr),
         LBT_ERR_SHAPE);
  EXPECT(lbt_backward_conv2d(p, p, nullptr, 4, 16, 12, 12, 32, 3, 3, 1, 1, 0, 1, 0, st, 0, 0, p, p, ws, need, nullptr),
         LBT_ERR_NULL);
  EXPECT(lbt_backward_conv2d(p, p, p, 4, 16, 12, 12, 32, 3, 3, 1, 1, 0, 1, 0, st, 0, LBT_BITS(8), p, p, ws, need,
                             nullptr), LBT_ERR_UNSUPPORTED);   // unsigned 8-bit activations for dW
  EXPECT(lbt_backward_conv2d(p, p, p, 4, 16, 12, 12, 32, 3, 3, 1, 1, 0, 1, 0, st, 0, 1 << 14, p, p, ws, need,
                             nullptr), LBT_ERR_UNSUPPORTED);   // unknown flag
  EXPECT(lbt_backward_linear(p, p, p, 0, 4, 4, 0, 0, 0, st, 0, 0, p, p, ws, big, nullptr), LBT_ERR_SHAPE);
  EXPECT(lbt_backward_linear(p, p, p, 8, 8, 8, 0, 0, 0, st, 0, 0, p, p + 1, ws, big, nullptr), LBT_ERR_ALIGN);
  EXPECT(lbt_backward_linear(p, p, p, 8, 8, 8, 0, 0, 0, nullptr, 0, 0, p, p, ws, big, nullptr), LBT_ERR_NULL);
  EXPECT(lbt_backward_linear_learned(p, p, p, 8, 8, 8, 0.0f, 0, 1.0f, st, 0, 0, p, p, p, ws, big, nullptr),
         LBT_ERR_UNSUPPORTED);                                  // learned clip values must be given
  EXPECT(lbt_backward_linear_learned(p, p, p, 8, 8, 8, 1.0f, 0, 1.0f, st, 0, 0, p, p, nullptr, ws, big, nullptr),
         LBT_ERR_NULL);
  EXPECT(lbt_forward_linear(p, p, 8, 8, 8, 0, 1, 0, LBT_BITS(8), p, nullptr, nullptr, ws, big, nullptr),
         LBT_ERR_UNSUPPORTED);
  EXPECT(lbt_forward_conv2d(p, nullptr, 4, 16, 12, 12, 32, 3, 3, 1, 1, 0, 1, 0, 0, p, nullptr, nullptr, ws, big,
                            nullptr), LBT_ERR_NULL);
  EXPECT(lbt_saved_bytes_conv2d(4, 16, 12, 12, 32, 3, 3, 1, 1) > 0, 1);
  EXPECT(lbt_saved_bytes_linear(0, 1, 1), 0);
  EXPECT(lbt_backward_conv2d_saved(nullptr, 0, p, 4, 16, 12, 12, 32, 3, 3, 1, 1, 1, st, 0, 0, p, p, nullptr,
                                   nullptr, ws, need, nullptr), LBT_ERR_NULL);
  EXPECT(lbt_backward_conv2d_saved(ws, 16, p, 4, 16, 12, 12, 32, 3, 3, 1, 1, 1, st, 0, 0, p, p, nullptr, nullptr,
                                   ws, need, nullptr), LBT_ERR_WORKSPACE);
  // an int32 accumulator that could overflow is refused on the host: 8-bit codes over a
  // contraction of 2^17 * 9 terms in dX
  EXPECT(lbt_workspace_bytes_conv2d(1, 8, 8, 8, 1 << 17, 3, 3, 1, 1) > 0, 1);
  EXPECT(lbt_profile_kernel_count() > 0, 1);
  EXPECT(lbt_profile_read(nullptr, nullptr, nullptr, 0), LBT_ERR_NULL);

  if (failures) std::printf("%d expectation(s) failed\n", failures);
  else std::printf("abi refusals under sanitizers: ok\n");
  return failures ? 1 : 0;
}
