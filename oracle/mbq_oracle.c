/*
 * Plain C oracle (fp64, straight loops) of MoBiQuant's token-routed any-precision linear:
 * encode, route, bucket, routed linear.  TEST AND BENCHMARK INFRASTRUCTURE ONLY: it exists so that
 * the CPU baseline can be timed in full on the Llama-shaped configurations (the numpy oracle
 * needs too much memory there) and it is itself pinned against the numpy oracle in the CPU tests.
 * It shares no code with the HIP library and is never linked into it.
 *
 * Every function takes the paper's steps in the paper's order:
 *   encode : Sec. 4.1 Eq. 2 with the floor-aligned quantiser, scale refinement s_{e+1} = s_e / 4 and
 *            centred residual zero point z_e = 2 of App. B; (s0, z0) from the min/max fit
 *            s0 = (max - min) / 4, z0 = -min / s0 (single fp32 operations, range floored for
 *            constant groups), codes from the fp64 recursion
 *              c_e = clamp(floor(R / s_e + z_e), 0, 3),  R <- R - s_e ((c_e - z_e) + 0.5);
 *   route  : Sec. 4.2 Eq. 4 read as one linear map to four logits, argmax with the first maximum
 *            winning ties, gap = top1 - top2;
 *   bucket : Sec. 4.3, tokens grouped by precision, stable in token order;
 *   linear : Sec. 4.2 Eq. 6 with the prefix mask: Y_i = sum_{e <= p_i} W_e^T X_i, with
 *            W_e = s_e ((c_e - z_e) + 0.5) dequantised row by row, then plain dot products.
 * Threads (OpenMP) split independent output rows / tokens only; no blocking, no reordering inside
 * a dot product.  Build: gcc -O2 -fopenmp -shared -fPIC (see oracle/build.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define GROUP 128
#define N_SLICES 4

static double bf16_to_f64(uint16_t bits) {
  uint32_t u = (uint32_t)bits << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

int mbq_oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void mbq_oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* W fp32 [N][K] -> codes uint8 [4][N][K], s0 fp32 [N][K/128], z0 fp32 [N][K/128] */
void mbq_oracle_encode(const float* W, int64_t N, int64_t K, uint8_t* codes, float* s0, float* z0) {
  const int64_t G = K / GROUP;
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < N; ++n) {
    for (int64_t g = 0; g < G; ++g) {
      const float* w = W + n * K + g * GROUP;
      float lo = w[0], hi = w[0];
      for (int j = 1; j < GROUP; ++j) {
        if (w[j] < lo) lo = w[j];
        if (w[j] > hi) hi = w[j];
      }
      float rng = hi - lo;
      const float mag = fmaxf(fabsf(lo), fabsf(hi));
      const float floor_rng = fmaxf(mag * 0x1p-16f, 0x1p-100f);
      if (rng < floor_rng) rng = floor_rng;
      const float s = rng / 4.0f;
      const float z = (-lo) / s;
      s0[n * G + g] = s;
      z0[n * G + g] = z;
      for (int j = 0; j < GROUP; ++j) {
        double R = (double)w[j];
        for (int e = 0; e < N_SLICES; ++e) {
          const double s_e = (double)s / (double)(1 << (2 * e));
          const double z_e = e == 0 ? (double)z : 2.0;
          double c = floor(R / s_e + z_e);
          if (c < 0.0) c = 0.0;
          if (c > 3.0) c = 3.0;
          codes[((int64_t)e * N + n) * K + g * GROUP + j] = (uint8_t)c;
          R = R - s_e * ((c - z_e) + 0.5);
        }
      }
    }
  }
}

/* X bf16 bits [T][K], Wr fp32 [4][K], br fp32 [4] -> logits fp64 [T][4], prec int32 [T], gap fp64 [T] */
void mbq_oracle_route(const uint16_t* X, int64_t T, int64_t K, const float* Wr, const float* br, double* logits,
                      int32_t* prec, double* gap) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < T; ++i) {
    double s[4];
    for (int q = 0; q < 4; ++q) {
      double acc = 0.0;
      for (int64_t k = 0; k < K; ++k) acc += bf16_to_f64(X[i * K + k]) * (double)Wr[q * K + k];
      s[q] = acc + (double)br[q];
      logits[i * 4 + q] = s[q];
    }
    int arg = 0;
    for (int q = 1; q < 4; ++q)
      if (s[q] > s[arg]) arg = q; /* strict: the first maximum wins */
    double second = -INFINITY;
    for (int q = 0; q < 4; ++q)
      if (q != arg && s[q] > second) second = s[q];
    prec[i] = arg;
    gap[i] = s[arg] - second;
  }
}

/* prec [T] -> perm [T] (token ids by ascending precision, stable), offsets [5] */
void mbq_oracle_bucket(const int32_t* prec, int64_t T, int32_t* perm, int32_t* offsets) {
  int64_t pos = 0;
  for (int q = 0; q < 4; ++q) {
    offsets[q] = (int32_t)pos;
    for (int64_t i = 0; i < T; ++i)
      if (prec[i] == q) perm[pos++] = (int32_t)i;
  }
  offsets[4] = (int32_t)pos;
}

/* Y fp64 [T][N] = routed output; row n of each slice is dequantised (Eq. 3's terms), then dotted with the
 * activation rows that use the slice (Eq. 6). */
void mbq_oracle_linear(const uint16_t* X, int64_t T, int64_t K, const uint8_t* codes, const float* s0, const float* z0,
                       int64_t N, const int32_t* prec, double* Y) {
  const int64_t G = K / GROUP;
  double* Xd = (double*)malloc((size_t)T * (size_t)K * sizeof(double));
  for (int64_t i = 0; i < T * K; ++i) Xd[i] = bf16_to_f64(X[i]);
#pragma omp parallel
  {
    double* We = (double*)malloc((size_t)K * sizeof(double));
#pragma omp for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
      for (int64_t i = 0; i < T; ++i) Y[i * N + n] = 0.0;
      for (int e = 0; e < N_SLICES; ++e) {
        int used = 0;
        for (int64_t i = 0; i < T; ++i) used |= prec[i] >= e;
        if (!used) continue;
        for (int64_t k = 0; k < K; ++k) {
          const double s_e = (double)s0[n * G + k / GROUP] / (double)(1 << (2 * e));
          const double z_e = e == 0 ? (double)z0[n * G + k / GROUP] : 2.0;
          We[k] = s_e * (((double)codes[((int64_t)e * N + n) * K + k] - z_e) + 0.5);
        }
        for (int64_t i = 0; i < T; ++i) {
          if (prec[i] < e) continue;
          double acc = 0.0;
          const double* x = Xd + i * K;
          for (int64_t k = 0; k < K; ++k) acc += x[k] * We[k];
          Y[i * N + n] += acc;
        }
      }
    }
    free(We);
  }
  free(Xd);
}
