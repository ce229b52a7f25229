/* Brute-force nested loops for the three kernels the paper defines element by
 * element.  TEST INFRASTRUCTURE ONLY: this is the second, independent form of
 * the CPU oracle.  It shares no code with the access-pattern interpreter
 * (oracle/access_pattern.py) or with the HIP library; the tests require all
 * three to agree.
 *
 *   conv2d   : out[n,o,x,y] = sum_{dx,dy,c} A[n,c,S0*x+dx,S1*y+dy] * W[o,c,dx,dy]
 *              (2D-convolution equation, Sec. 5.1), x along H, y along W.
 *   max-pool : out[n,c,x,y] = max_{dx,dy} A[n,c,S0*x+dx,S1*y+dy]
 *              (max-pooling equation, Sec. 5.1).
 *   matmul   : R[i,j] = sum_k P[i,k] * Q[k,j]   (Sec. 3.1).
 *
 * Extension (not in the paper): symmetric spatial padding p0,p1.  A padded
 * position reads `fill` (0 for the sums, the lowest value of the storage type
 * for max), which is what applying the paper's program to an explicitly
 * padded tensor gives.
 *
 * Arithmetic: double in, double accumulate, double out for the real-valued
 * paths; int64 for the integer paths (exact).  Rounding to a storage type is
 * done by the caller.  OpenMP only parallelises the outermost independent
 * loops; the summation order inside one output element is the plain loop
 * order c, dx, dy.
 */
#include <stdint.h>
#include <stddef.h>

#define OUT_DIM(in, pad, k, s) (((in) + 2 * (pad) - (k)) / (s) + 1)

#define DEFINE_CONV2D(NAME, T)                                                        \
  int NAME(const T* A, const T* W, T* out, int64_t N, int64_t C, int64_t H,           \
           int64_t Wd, int64_t O, int64_t Kh, int64_t Kw, int64_t S0, int64_t S1,     \
           int64_t p0, int64_t p1) {                                                  \
    if (H + 2 * p0 < Kh || Wd + 2 * p1 < Kw || S0 < 1 || S1 < 1) return 1;            \
    const int64_t Ho = OUT_DIM(H, p0, Kh, S0), Wo = OUT_DIM(Wd, p1, Kw, S1);          \
    _Pragma("omp parallel for collapse(2) schedule(static)")                          \
    for (int64_t n = 0; n < N; ++n)                                                   \
      for (int64_t o = 0; o < O; ++o)                                                 \
        for (int64_t x = 0; x < Ho; ++x)                                              \
          for (int64_t y = 0; y < Wo; ++y) {                                          \
            T acc = 0;                                                                \
            for (int64_t c = 0; c < C; ++c)                                           \
              for (int64_t dx = 0; dx < Kh; ++dx)                                     \
                for (int64_t dy = 0; dy < Kw; ++dy) {                                 \
                  const int64_t h = S0 * x + dx - p0, w = S1 * y + dy - p1;           \
                  const T a = (h < 0 || h >= H || w < 0 || w >= Wd)                   \
                                  ? (T)0                                              \
                                  : A[((n * C + c) * H + h) * Wd + w];                \
                  acc += a * W[((o * C + c) * Kh + dx) * Kw + dy];                    \
                }                                                                     \
            out[((n * O + o) * Ho + x) * Wo + y] = acc;                               \
          }                                                                           \
    return 0;                                                                         \
  }

DEFINE_CONV2D(brute_conv2d_f64, double)
DEFINE_CONV2D(brute_conv2d_i64, int64_t)

#define DEFINE_MAXPOOL(NAME, T)                                                       \
  int NAME(const T* A, T* out, int64_t N, int64_t C, int64_t H, int64_t Wd,           \
           int64_t Kh, int64_t Kw, int64_t S0, int64_t S1, int64_t p0, int64_t p1,    \
           T fill) {                                                                  \
    if (H + 2 * p0 < Kh || Wd + 2 * p1 < Kw || S0 < 1 || S1 < 1) return 1;            \
    const int64_t Ho = OUT_DIM(H, p0, Kh, S0), Wo = OUT_DIM(Wd, p1, Kw, S1);          \
    _Pragma("omp parallel for collapse(2) schedule(static)")                          \
    for (int64_t n = 0; n < N; ++n)                                                   \
      for (int64_t c = 0; c < C; ++c)                                                 \
        for (int64_t x = 0; x < Ho; ++x)                                              \
          for (int64_t y = 0; y < Wo; ++y) {                                          \
            int first = 1;                                                            \
            T best = fill;                                                            \
            for (int64_t dx = 0; dx < Kh; ++dx)                                       \
              for (int64_t dy = 0; dy < Kw; ++dy) {                                   \
                const int64_t h = S0 * x + dx - p0, w = S1 * y + dy - p1;             \
                const T a = (h < 0 || h >= H || w < 0 || w >= Wd)                     \
                                ? fill                                                \
                                : A[((n * C + c) * H + h) * Wd + w];                  \
                if (first || a > best) best = a;                                      \
                first = 0;                                                            \
              }                                                                       \
            out[((n * C + c) * Ho + x) * Wo + y] = best;                              \
          }                                                                           \
    return 0;                                                                         \
  }

DEFINE_MAXPOOL(brute_maxpool_f64, double)
DEFINE_MAXPOOL(brute_maxpool_i64, int64_t)

/* R[i,j] = sum_k P[i,k] * Q[k,j];  P is I x K, Q is K x J, both row-major. */
#define DEFINE_MATMUL(NAME, T)                                                        \
  int NAME(const T* P, const T* Q, T* R, int64_t I, int64_t K, int64_t J) {           \
    _Pragma("omp parallel for schedule(static)")                                      \
    for (int64_t i = 0; i < I; ++i)                                                   \
      for (int64_t j = 0; j < J; ++j) {                                               \
        T acc = 0;                                                                    \
        for (int64_t k = 0; k < K; ++k) acc += P[i * K + k] * Q[k * J + j];           \
        R[i * J + j] = acc;                                                           \
      }                                                                               \
    return 0;                                                                         \
  }

DEFINE_MATMUL(brute_matmul_f64, double)
DEFINE_MATMUL(brute_matmul_i64, int64_t)

/* Row reductions: out[r] = sum / max over the `cols` values of row r. */
#define DEFINE_ROWREDUCE(NAME, T)                                                     \
  int NAME(const T* in, T* out, int64_t rows, int64_t cols, int is_max) {             \
    if (is_max && cols < 1) return 1;                                                 \
    _Pragma("omp parallel for schedule(static)")                                      \
    for (int64_t r = 0; r < rows; ++r) {                                              \
      T acc = is_max ? in[r * cols] : (T)0;                                           \
      for (int64_t c = is_max ? 1 : 0; c < cols; ++c) {                               \
        const T v = in[r * cols + c];                                                 \
        if (is_max) { if (v > acc) acc = v; } else { acc += v; }                      \
      }                                                                               \
      out[r] = acc;                                                                   \
    }                                                                                 \
    return 0;                                                                         \
  }

DEFINE_ROWREDUCE(brute_rowreduce_f64, double)
DEFINE_ROWREDUCE(brute_rowreduce_i64, int64_t)
