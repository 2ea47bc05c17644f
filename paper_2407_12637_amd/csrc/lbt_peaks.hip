// Stand-alone probe of the ceilings the library's kernels are rated against on this GPU:
// HBM read / write / copy bandwidth with plain streaming kernels, LDS 16-byte read bandwidth
// per compute unit, and the issue rate of v_mfma_i32_32x32x32_i8 back to back.  Built beside
// the library (build.py), run by `python bench.py --peaks`; not part of the library itself.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));

#define CK(x)                                                                    \
  do {                                                                           \
    hipError_t e_ = (x);                                                         \
    if (e_ != hipSuccess) {                                                      \
      std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
      return 1;                                                                  \
    }                                                                            \
  } while (0)

constexpr int kCus = 256;
constexpr double kClock = 2.4e9;

// each workgroup reads one contiguous chunk, eight 16-byte loads in flight per thread
__global__ __launch_bounds__(256) void k_read(const f4* __restrict__ p, long long n4, uint32_t* out) {
  const long long per = (n4 + gridDim.x - 1) / gridDim.x;
  long long i = blockIdx.x * per + threadIdx.x;
  const long long end = min(n4, (long long)(blockIdx.x + 1) * per);
  uint32_t m = 0;
  for (; i + 7 * 256 < end; i += 8 * 256) {
    f4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + i + u * 256);
#pragma unroll
    for (int u = 0; u < 8; ++u)
      m = max(max(m, __float_as_uint(v[u].x)), max(__float_as_uint(v[u].y), max(__float_as_uint(v[u].z), __float_as_uint(v[u].w))));
  }
  for (; i < end; i += 256) m = max(m, __float_as_uint(p[i].x));
  if (m == 0x7fc12345u) out[0] = m;   // never true for the zero-filled buffer: keeps the loads
}

__global__ __launch_bounds__(256) void k_write(f4* __restrict__ p, long long n4, float value) {
  const long long stride = (long long)gridDim.x * 256;
  const f4 v = {value, value, value, value};
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) p[i] = v;
}

__global__ __launch_bounds__(256) void k_copy(const f4* __restrict__ src, f4* __restrict__ dst, long long n4) {
  const long long stride = (long long)gridDim.x * 256;
  long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n4; i += 4 * stride) {
    f4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < 4; ++u) dst[i + u * stride] = v[u];
  }
  for (; i < n4; i += stride) dst[i] = src[i];
}

// every lane reads 16 bytes, consecutive lanes consecutive addresses (no bank conflicts);
// eight reads in flight per wave, written as one asm block so that they are issued together
__global__ __launch_bounds__(256) void k_lds_read(int iters, int* out) {
  __shared__ __attribute__((aligned(16))) int buf[8192];
  for (int i = threadIdx.x; i < 8192; i += 256) buf[i] = i;
  __syncthreads();
  const unsigned base = (unsigned)(uintptr_t)buf + (threadIdx.x & 63) * 16 + (threadIdx.x >> 6) * 1024;
  int acc = 0;
  for (int it = 0; it < iters; ++it) {
    v4i v0, v1, v2, v3, v4, v5, v6, v7;
    asm volatile(
        "ds_read_b128 %0, %8\n ds_read_b128 %1, %8 offset:4096\n ds_read_b128 %2, %8 offset:8192\n"
        "ds_read_b128 %3, %8 offset:12288\n ds_read_b128 %4, %8 offset:16384\n"
        "ds_read_b128 %5, %8 offset:20480\n ds_read_b128 %6, %8 offset:24576\n"
        "ds_read_b128 %7, %8 offset:28672\n s_waitcnt lgkmcnt(0)\n"
        : "=v"(v0), "=v"(v1), "=v"(v2), "=v"(v3), "=v"(v4), "=v"(v5), "=v"(v6), "=v"(v7)
        : "v"(base)
        : "memory");
    acc ^= v0[0] ^ v1[1] ^ v2[2] ^ v3[3] ^ v4[0] ^ v5[1] ^ v6[2] ^ v7[3];
  }
  if (acc == 0x12345678) out[0] = acc;
}

// four independent accumulators per wave: the matrix core never waits for a result
__global__ __launch_bounds__(256) void k_mfma(int iters, int* out) {
  v16i acc[4];
  for (int i = 0; i < 4; ++i)
    for (int r = 0; r < 16; ++r) acc[i][r] = 0;
  const v4i a = {(int)threadIdx.x, 1, 2, 3}, b = {4, 5, 6, (int)blockIdx.x};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i], 0, 0, 0);
  }
  int s = 0;
  for (int i = 0; i < 4; ++i)
    for (int r = 0; r < 16; ++r) s ^= acc[i][r];
  if (s == 0x12345678) out[0] = s;
}

template <typename F>
static int timed(F launch, int reps, float* best_ms) {
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  *best_ms = 1e30f;
  for (int r = 0; r < reps; ++r) {
    CK(hipEventRecord(e0, 0));
    launch();
    CK(hipEventRecord(e1, 0));
    CK(hipEventSynchronize(e1));
    float ms = 0.0f;
    CK(hipEventElapsedTime(&ms, e0, e1));
    if (r > 0 && ms < *best_ms) *best_ms = ms;   // the first repetition warms up
  }
  CK(hipEventDestroy(e0));
  CK(hipEventDestroy(e1));
  return 0;
}

int main() {
  const long long bytes = 1ll << 30, n4 = bytes / 16;
  f4 *a = nullptr, *b = nullptr;
  int* out = nullptr;
  CK(hipMalloc(&a, bytes));
  CK(hipMalloc(&b, bytes));
  CK(hipMalloc(&out, 64));
  CK(hipMemset(a, 0, bytes));
  CK(hipMemset(b, 0, bytes));
  float ms;
  std::printf("buffers of 1 GiB (larger than every cache); best of 7 launches after a warm-up; rates against\n"
              "the published peaks 8 TB/s and 5.0 POP/s (256 compute units at 2.4 GHz)\n");
  for (int blocks : {2048, 4096, 8192}) {
    if (timed([&] { hipLaunchKernelGGL(k_read, dim3(blocks), dim3(256), 0, 0, a, n4, (uint32_t*)out); }, 8, &ms)) return 1;
    std::printf("HBM read   %5d workgroups: %7.1f us  %.2f TB/s  (%.0f %% of 8 TB/s)\n", blocks, ms * 1e3,
                bytes / (ms * 1e-3) / 1e12, bytes / (ms * 1e-3) / 8e12 * 100);
  }
  for (int blocks : {2048, 8192}) {
    if (timed([&] { hipLaunchKernelGGL(k_write, dim3(blocks), dim3(256), 0, 0, b, n4, 1.0f); }, 8, &ms)) return 1;
    std::printf("HBM write  %5d workgroups: %7.1f us  %.2f TB/s  (%.0f %%)\n", blocks, ms * 1e3,
                bytes / (ms * 1e-3) / 1e12, bytes / (ms * 1e-3) / 8e12 * 100);
  }
  for (int blocks : {2048, 8192}) {
    if (timed([&] { hipLaunchKernelGGL(k_copy, dim3(blocks), dim3(256), 0, 0, a, b, n4); }, 8, &ms)) return 1;
    std::printf("HBM copy   %5d workgroups: %7.1f us  %.2f TB/s read + %.2f TB/s written  (%.0f %% in total)\n", blocks,
                ms * 1e3, bytes / (ms * 1e-3) / 1e12, bytes / (ms * 1e-3) / 1e12, 2.0 * bytes / (ms * 1e-3) / 8e12 * 100);
  }
  {
    const int iters = 4000, per_cu = 2;
    if (timed([&] { hipLaunchKernelGGL(k_lds_read, dim3(kCus * per_cu), dim3(256), 0, 0, iters, out); }, 4, &ms)) return 1;
    const double total = (double)kCus * per_cu * 256 * iters * 8 * 16;
    std::printf("LDS 16-byte reads, conflict-free: %.1f bytes per clock and compute unit at 2.4 GHz\n",
                total / (ms * 1e-3) / kCus / kClock);
  }
  for (int per_simd = 1; per_simd <= 2; ++per_simd) {
    const int iters = 20000;
    if (timed([&] { hipLaunchKernelGGL(k_mfma, dim3(kCus * per_simd), dim3(256), 0, 0, iters, out); }, 4, &ms)) return 1;
    const double n = (double)iters * 4 * per_simd;   // instructions per SIMD
    std::printf("v_mfma_i32_32x32x32_i8 back to back, %d wave(s) per SIMD: %.1f clocks each at 2.4 GHz, %.2f POP/s (%.0f %% of 5.0)\n",
                per_simd, ms * 1e-3 * kClock / n, (double)kCus * 4 * n * 65536.0 / (ms * 1e-3) / 1e15,
                (double)kCus * 4 * n * 65536.0 / (ms * 1e-3) / 5.0e15 * 100);
  }
  CK(hipFree(a));
  CK(hipFree(b));
  CK(hipFree(out));
  return 0;
}
