/* Runs every function of oracle/lbt_oracle.c on small, exactly sized heap buffers, built with
 * -fsanitize=address,undefined: an out-of-bounds access, a signed overflow, a float-to-integer
 * conversion out of range or a misaligned access aborts the process.  The values are checked
 * elsewhere (tests/test_oracle_*.py); here only a few are, to make sure the calls did run. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int orc_num_threads(void);
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
uint32_t orc_r16(uint64_t e, uint64_t seed, uint64_t step);
int orc_max(const float* x, int64_t n, int use_abs, float* out);
float orc_clip_value(double gamma, float gmax);
int orc_levels(int bits, int is_unsigned);
int orc_interval_usable(float c, int bits, int is_unsigned);
double orc_scale(float c, int bits, int is_unsigned);
void orc_quantize(const float* x, int64_t n, float c, int bits, int is_unsigned, int rounding,
                  uint64_t seed, uint64_t step, int32_t* code, uint64_t* n_out);
void orc_pack_nibbles(const int32_t* code, int64_t n, uint8_t* out);
int orc_update_interval(double* gamma, double alpha, double beta, double gamma_min,
                        double gamma_max, int bits, uint64_t n_out, uint64_t n_total);
void orc_linear_dx(const int32_t* qG, const int32_t* qW, int64_t M, int64_t K, int64_t N, int64_t* acc);
void orc_linear_dw(const int32_t* qX, const int32_t* qG, int64_t M, int64_t K, int64_t N, int64_t* acc);
void orc_conv2d_dx(const int32_t* qG, const int32_t* qW, int64_t N, int64_t C, int64_t H, int64_t Wd,
                   int64_t K, int64_t R, int64_t S, int64_t st, int64_t pad, int64_t* acc);
void orc_conv2d_dw(const int32_t* qG, const int32_t* qX, int64_t N, int64_t C, int64_t H, int64_t Wd,
                   int64_t K, int64_t R, int64_t S, int64_t st, int64_t pad, int64_t* acc);
void orc_conv2d_dx_at(const int32_t* qG, const int32_t* qW, int64_t N, int64_t C, int64_t H, int64_t Wd,
                      int64_t K, int64_t R, int64_t S, int64_t st, int64_t pad, const int64_t* idx,
                      int64_t n_idx, int64_t* acc);
void orc_conv2d_dw_at(const int32_t* qG, const int32_t* qX, int64_t N, int64_t C, int64_t H, int64_t Wd,
                      int64_t K, int64_t R, int64_t S, int64_t st, int64_t pad, const int64_t* idx,
                      int64_t n_idx, int64_t* acc);
void orc_dequant(const int64_t* acc, int64_t n, double s_a, double s_b, float* out);

static int failures = 0;
#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) { printf("%s:%d: %s\n", __FILE__, __LINE__, #cond); ++failures; } \
  } while (0)

static uint64_t lcg = 88172645463325252ull;
static double unit(void) {   /* uniform in [-1, 1) */
  lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
  return (double)(int64_t)(lcg >> 11) / 4503599627370496.0 - 1.0;
}

static void quantizer_cases(void) {
  const float scales[] = {1.0f, 1e-3f, 3e-38f, 1e-40f, 1e30f};
  const int64_t sizes[] = {1, 2, 7, 8, 9, 1001};
  for (unsigned si = 0; si < sizeof(sizes) / sizeof(sizes[0]); ++si)
    for (unsigned sc = 0; sc < sizeof(scales) / sizeof(scales[0]); ++sc) {
      const int64_t n = sizes[si];
      float* x = malloc(sizeof(float) * (size_t)n);
      int32_t* code = malloc(sizeof(int32_t) * (size_t)n);
      uint8_t* packed = malloc((size_t)((n + 1) / 2));
      for (int64_t i = 0; i < n; ++i) x[i] = (float)(unit() * scales[sc]);
      float m = 0.0f;
      const int status = orc_max(x, n, 1, &m);
      CHECK(status == 0 || status == 2);
      for (int bits = 2; bits <= 8; ++bits)
        for (int uns = 0; uns <= 1; ++uns)
          for (int rounding = 0; rounding <= 1; ++rounding) {
            const float c = orc_clip_value(0.37, m);
            uint64_t n_out = 12345;
            orc_quantize(x, n, c, bits, uns, rounding, 0xFFFFFFFFFFFFFFFFull, 0xFFFFFFFF00000001ull,
                         code, &n_out);
            const int q = orc_levels(bits, uns);
            for (int64_t i = 0; i < n; ++i) CHECK(code[i] <= q && code[i] >= (uns ? 0 : -q));
            CHECK(n_out <= (uint64_t)n);
            if (!orc_interval_usable(c, bits, uns)) CHECK(n_out == 0 && code[0] == 0);
            (void)orc_scale(c, bits, uns);
          }
      orc_quantize(x, n, m, 4, 0, 0, 0, 0, code, NULL);
      orc_pack_nibbles(code, n, packed);
      free(x); free(code); free(packed);
    }
  /* non-finite inputs never reach the quantizer through the callers; the maximum flags them */
  float bad[3] = {1.0f, NAN, -INFINITY}, m;
  CHECK(orc_max(bad, 3, 1, &m) == 1);
  CHECK(orc_max(bad, 1, 0, &m) == 0 && m == 1.0f);
  /* the largest finite inputs with the smallest usable interval: the decision variable
   * stays finite because the input is clipped first */
  float big[2] = {3.0e38f, -3.0e38f};
  int32_t code[2];
  orc_quantize(big, 2, 4e-37f, 8, 0, 1, 1, 1, code, NULL);
  CHECK(code[0] == 127 && code[1] == -127);
}

static void update_cases(void) {
  double g = 0.5;
  CHECK(orc_update_interval(&g, 1e-3, 1e-3, 1e-3, 1.0, 4, 0, 1000) == -1);
  CHECK(orc_update_interval(&g, 1e-3, 1e-3, 1e-3, 1.0, 8, UINT64_MAX >> 12, UINT64_MAX >> 8) == 1);
  g = 1.0;
  CHECK(orc_update_interval(&g, 1e-3, 1e-3, 1e-3, 1.0, 4, 1000, 1000) == 1 && g == 1.0);
  uint32_t ctr[4] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu}, key[2] = {0xFFFFFFFFu, 0xFFFFFFFFu};
  uint32_t out[4];
  orc_philox4x32_10(ctr, key, out);
  CHECK(out[0] == 0x408f276du);   /* published known answer for the all-ones input */
  CHECK(orc_r16(UINT64_MAX, UINT64_MAX, UINT64_MAX) <= 0xFFFFu);
  CHECK(orc_num_threads() >= 1);
}

static void fill_codes(int32_t* p, int64_t n, int lo, int hi) {
  for (int64_t i = 0; i < n; ++i) p[i] = lo + (int)((unit() * 0.5 + 0.5) * (hi - lo + 1)) % (hi - lo + 1);
}

static void contraction_cases(void) {
  const int geoms[][7] = {/* N C H K R stride pad */
                          {2, 3, 7, 4, 3, 1, 1}, {1, 2, 9, 3, 3, 2, 1}, {2, 5, 6, 2, 1, 2, 0},
                          {1, 1, 5, 1, 5, 1, 2}, {1, 3, 8, 2, 7, 2, 3}, {3, 2, 4, 2, 2, 1, 0}};
  for (unsigned gi = 0; gi < sizeof(geoms) / sizeof(geoms[0]); ++gi) {
    const int64_t N = geoms[gi][0], C = geoms[gi][1], H = geoms[gi][2], W = H + 1, K = geoms[gi][3],
                  R = geoms[gi][4], S = R, st = geoms[gi][5], pad = geoms[gi][6];
    const int64_t P = (H + 2 * pad - R) / st + 1, Q = (W + 2 * pad - S) / st + 1;
    const int64_t n_g = N * K * P * Q, n_x = N * C * H * W, n_w = K * C * R * S;
    int32_t* qG = malloc(sizeof(int32_t) * (size_t)n_g);
    int32_t* qX = malloc(sizeof(int32_t) * (size_t)n_x);
    int32_t* qW = malloc(sizeof(int32_t) * (size_t)n_w);
    int64_t* ax = malloc(sizeof(int64_t) * (size_t)n_x);
    int64_t* aw = malloc(sizeof(int64_t) * (size_t)n_w);
    fill_codes(qG, n_g, -127, 127);
    fill_codes(qX, n_x, 0, 255);
    fill_codes(qW, n_w, -127, 127);
    orc_conv2d_dx(qG, qW, N, C, H, W, K, R, S, st, pad, ax);
    orc_conv2d_dw(qG, qX, N, C, H, W, K, R, S, st, pad, aw);
    int64_t* idx = malloc(sizeof(int64_t) * (size_t)n_x);
    int64_t* at = malloc(sizeof(int64_t) * (size_t)n_x);
    for (int64_t i = 0; i < n_x; ++i) idx[i] = n_x - 1 - i;
    orc_conv2d_dx_at(qG, qW, N, C, H, W, K, R, S, st, pad, idx, n_x, at);
    for (int64_t i = 0; i < n_x; ++i) CHECK(at[i] == ax[idx[i]]);
    free(idx); free(at);
    idx = malloc(sizeof(int64_t) * (size_t)n_w);
    at = malloc(sizeof(int64_t) * (size_t)n_w);
    for (int64_t i = 0; i < n_w; ++i) idx[i] = i;
    orc_conv2d_dw_at(qG, qX, N, C, H, W, K, R, S, st, pad, idx, n_w, at);
    for (int64_t i = 0; i < n_w; ++i) CHECK(at[i] == aw[i]);
    float* out = malloc(sizeof(float) * (size_t)n_w);
    orc_dequant(aw, n_w, 1e-3 / 7.0, 2.0 / 15.0, out);
    free(idx); free(at); free(out);
    free(qG); free(qX); free(qW); free(ax); free(aw);
  }
  const int64_t M = 5, K = 3, N = 4;
  int32_t* qG = malloc(sizeof(int32_t) * (size_t)(M * N));
  int32_t* qW = malloc(sizeof(int32_t) * (size_t)(K * N));
  int32_t* qX = malloc(sizeof(int32_t) * (size_t)(M * K));
  int64_t* ax = malloc(sizeof(int64_t) * (size_t)(M * K));
  int64_t* aw = malloc(sizeof(int64_t) * (size_t)(K * N));
  fill_codes(qG, M * N, -7, 7);
  fill_codes(qW, K * N, -7, 7);
  fill_codes(qX, M * K, 0, 15);
  orc_linear_dx(qG, qW, M, K, N, ax);
  orc_linear_dw(qX, qG, M, K, N, aw);
  free(qG); free(qW); free(qX); free(ax); free(aw);
}

int main(void) {
  quantizer_cases();
  update_cases();
  contraction_cases();
  if (failures) printf("%d check(s) failed\n", failures);
  else printf("oracle under sanitizers: ok\n");
  return failures ? 1 : 0;
}
