// Slow, straightforward routed linear: one thread per output element, fp64
// accumulate.  Kept as an on-device cross-check of the blob addressing and of the
// fast kernels (paper Sec. 4.2 Eq. 6 with the merged-code form of App. B:
// What = (s0/4^p)(I_p - 4^p z0 + 0.5)).
#include "mbq_common.h"

namespace mbq {

__global__ __launch_bounds__(256) void linear_simple_kernel(const uint16_t* __restrict__ X, int64_t T,
                                                            const uint32_t* __restrict__ codes,
                                                            size_t slice_words,
                                                            const float2* __restrict__ meta, int64_t N,
                                                            int64_t K, int NT, int KB,
                                                            const int32_t* __restrict__ prec,
                                                            float* __restrict__ Y, int bit_view, int gshift) {
  // bit_view = 0: prec holds digit precisions (2 (p + 1) bits); 1: bits - 1 (see RouteView), any count from 1 to 8
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= T * N) return;
  const int64_t i = idx / N, n = idx % N;
  int p = prec[i];
  int bits = bit_view ? p + 1 : 2 * (p + 1);
  bits = bits < 1 ? 1 : (bits > 2 * kSlices ? 2 * kSlices : bits);
  const double pw = __builtin_ldexp(1.0, bits - 2);
  double y = 0.0;
  const int group = 1 << gshift;  // 128, or 64 / 32 for the configurations that say so
  for (int g = 0; g < (int)(K >> gshift); ++g) {
    const float2 m = meta[meta_index(KB, n, g, kTileK >> gshift)];
    double dot = 0.0, sx = 0.0;
    for (int kk = 0; kk < group; ++kk) {
      const int64_t k = (int64_t)g * group + kk;
      const size_t w = code_word(NT, KB, n, k);
      int I = 0;
      for (int e = 0; 2 * e < bits; ++e) I = I * 4 + (int)((codes[e * slice_words + w] >> code_bit(e, k)) & 3u);
      I >>= (bits & 1);  // an odd count stops at the high bit of its last digit
      const double x = (double)__uint_as_float((uint32_t)X[i * K + k] << 16);
      dot += x * (double)I;
      sx += x;
    }
    y += ((double)m.x / pw) * (dot + (0.5 - pw * (double)m.y) * sx);
  }
  Y[idx] = (float)y;
}

mbq_status launch_linear_simple(const uint16_t* X, int64_t T, const void* blob, const Shape& sh,
                                const int32_t* prec, float* Y, hipStream_t stream, bool bit_view) {
  const uint32_t* codes = reinterpret_cast<const uint32_t*>(blob);
  const float2* meta = reinterpret_cast<const float2*>(reinterpret_cast<const char*>(blob) + sh.meta_offset);
  const int64_t total = T * sh.N;
  hipLaunchKernelGGL(linear_simple_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, X, T,
                     codes, sh.slice_words, meta, sh.N, sh.K, sh.NT, sh.KB, prec, Y, bit_view ? 1 : 0, sh.gshift);
  return hip_status(hipGetLastError(), "linear_simple_kernel launch");
}

}  // namespace mbq
