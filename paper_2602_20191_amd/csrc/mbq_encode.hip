// Offline side of the layer: recursive residual quantisation into the packed blob
// (paper Sec. 4.1 Eq. 2, quantiser and scale refinement of App. B), and the inverse
// helpers that turn the blob back into canonical arrays.
//
// This translation unit is compiled with -ffp-contract=off: the code recursion is
// specified operation by operation in fp64 and must not be fused.
#include "mbq_common.h"

namespace mbq {

// One workgroup of 256 threads encodes one code tile (16 rows x 256 columns = two
// groups per row).  Thread (lane, d) owns dword d of lane `lane`: row nn = lane%16,
// columns 64*d + 32*step + 8*kq + s for step in {0,1}, s in 0..7 (kq = lane/16).
__global__ __launch_bounds__(256) void encode_kernel(const float* __restrict__ W, int64_t N, int64_t K,
                                                     int NT, int KB, uint32_t* __restrict__ codes,
                                                     size_t slice_words, float2* __restrict__ meta,
                                                     const float* __restrict__ ext_scale,
                                                     const float* __restrict__ ext_zero) {
#pragma clang fp contract(off)
  const int nt = blockIdx.x;
  const int kb = blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = tid >> 2;
  const int d = tid & 3;
  const int nn = lane & 15;
  const int kq = lane >> 4;
  const int64_t n = (int64_t)nt * kTileN + nn;
  const int64_t kbase = (int64_t)kb * kTileK + 64 * d + 8 * kq;
  const int h = d >> 1;  // group of this thread inside the tile
  const int64_t g = 2 * (int64_t)kb + h;
  const bool real = (n < N) && (g * kGroup < K);

  float w[16];
#pragma unroll
  for (int step = 0; step < 2; ++step) {
    if (real) {
      const float4* src = reinterpret_cast<const float4*>(W + n * K + kbase + 32 * step);
      float4 a = src[0], b = src[1];
      w[8 * step + 0] = a.x; w[8 * step + 1] = a.y; w[8 * step + 2] = a.z; w[8 * step + 3] = a.w;
      w[8 * step + 4] = b.x; w[8 * step + 5] = b.y; w[8 * step + 6] = b.z; w[8 * step + 7] = b.w;
    } else {
#pragma unroll
      for (int s = 0; s < 8; ++s) w[8 * step + s] = 0.f;
    }
  }
  float lo = w[0], hi = w[0];
#pragma unroll
  for (int i = 1; i < 16; ++i) {
    lo = fminf(lo, w[i]);
    hi = fmaxf(hi, w[i]);
  }
  // a (row, group) is spread over 8 threads: d in {2h, 2h+1} x kq in 0..3
  __shared__ float s_lo[16][2][8];
  __shared__ float s_hi[16][2][8];
  s_lo[nn][h][(d & 1) * 4 + kq] = lo;
  s_hi[nn][h][(d & 1) * 4 + kq] = hi;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    lo = fminf(lo, s_lo[nn][h][i]);
    hi = fmaxf(hi, s_hi[nn][h][i]);
  }
  // base-slice fit: four floor-aligned bins tile [lo, hi]
  float rng = hi - lo;
  const float mag = fmaxf(fabsf(lo), fabsf(hi));
  const float floor_rng = fmaxf(mag * 0x1p-16f, 0x1p-100f);
  rng = fmaxf(rng, floor_rng);
  float s0 = rng * 0.25f;
  float z0 = (float)((double)(-lo) / (double)s0);  // equals the IEEE fp32 quotient
  // calibrated parameters from outside (e.g. a learned clipping range, Sec. 4.1 / App. B): weights beyond
  // the range they span saturate in the clamp of every slice
  if (ext_scale != nullptr && real) {
    s0 = ext_scale[n * (K / kGroup) + g];
    z0 = ext_zero[n * (K / kGroup) + g];
  }

  uint32_t word[kSlices] = {0u, 0u, 0u, 0u};
  if (real) {
    const double s0d = (double)s0, z0d = (double)z0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int step = i >> 3, s = i & 7;
      const int field = 16 * (s & 1) + 4 * (s >> 1) + 2 * step;
      double R = (double)w[i];
      double se = s0d;
#pragma unroll
      for (int e = 0; e < kSlices; ++e) {
        const double ze = (e == 0) ? z0d : 2.0;
        double q = floor(R / se + ze);
        q = fmin(fmax(q, 0.0), 3.0);
        R = R - se * ((q - ze) + 0.5);
        word[e] |= (uint32_t)q << ((field + 2 - 2 * e) & 31);
        se = se * 0.25;
      }
    }
  }
  const size_t widx = ((size_t)nt * KB + kb) * kTileWords + (size_t)lane * 4 + d;
#pragma unroll
  for (int e = 0; e < kSlices; ++e) codes[e * slice_words + widx] = word[e];
  if ((d & 1) == 0 && kq == 0) {
    float2 m;
    m.x = real ? s0 : 0.f;
    m.y = real ? z0 : 0.f;
    meta[meta_index(KB, n, (int)g)] = m;
  }
}

// Groups of 64 or 32 columns (App. C.1 lists the group size among the settings): the same recursion and the same code
// words; a thread's two runs of eight columns may lie in different groups, and each thread finds the extremes of the
// group(s) it works in by reading them (an offline step: no effort is made to share those reads).
__global__ __launch_bounds__(256) void encode_small_group_kernel(const float* __restrict__ W, int64_t N, int64_t K,
                                                                 int NT, int KB, uint32_t* __restrict__ codes,
                                                                 size_t slice_words, float2* __restrict__ meta,
                                                                 int gshift) {
#pragma clang fp contract(off)
  const int nt = blockIdx.x;
  const int kb = blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = tid >> 2;
  const int d = tid & 3;
  const int nn = lane & 15;
  const int kq = lane >> 4;
  const int64_t n = (int64_t)nt * kTileN + nn;
  const int64_t kbase = (int64_t)kb * kTileK + 64 * d + 8 * kq;
  const int group = 1 << gshift;
  const int per_tile = kTileK >> gshift;
  uint32_t word[kSlices] = {0u, 0u, 0u, 0u};
  for (int step = 0; step < 2; ++step) {
    const int64_t k0 = kbase + 32 * step;      // first of this thread's eight columns of the step
    const int64_t g = k0 >> gshift;
    const int64_t gs = g << gshift;            // first column of their group
    const bool real = (n < N) && (gs < K);
    float s0 = 0.f, z0 = 0.f;
    if (real) {
      const float* row = W + n * K + gs;
      float lo = row[0], hi = row[0];
      for (int j = 1; j < group; ++j) {
        lo = fminf(lo, row[j]);
        hi = fmaxf(hi, row[j]);
      }
      float rng = hi - lo;
      const float mag = fmaxf(fabsf(lo), fabsf(hi));
      rng = fmaxf(rng, fmaxf(mag * 0x1p-16f, 0x1p-100f));
      s0 = rng * 0.25f;
      z0 = (float)((double)(-lo) / (double)s0);
      const double s0d = (double)s0, z0d = (double)z0;
      for (int s = 0; s < 8; ++s) {
        const int field = 16 * (s & 1) + 4 * (s >> 1) + 2 * step;
        double R = (double)W[n * K + k0 + s];
        double se = s0d;
#pragma unroll
        for (int e = 0; e < kSlices; ++e) {
          const double ze = (e == 0) ? z0d : 2.0;
          double q = floor(R / se + ze);
          q = fmin(fmax(q, 0.0), 3.0);
          R = R - se * ((q - ze) + 0.5);
          word[e] |= (uint32_t)q << ((field + 2 - 2 * e) & 31);
          se = se * 0.25;
        }
      }
    }
    // the thread whose run starts the group files its parameters (padding rows and groups: zeros)
    if (k0 == gs && (step == 0 || gshift == 5)) {
      float2 m;
      m.x = s0;
      m.y = z0;
      meta[meta_index(KB, n, (int)g, per_tile)] = m;
    }
  }
  const size_t widx = ((size_t)nt * KB + kb) * kTileWords + (size_t)lane * 4 + d;
#pragma unroll
  for (int e = 0; e < kSlices; ++e) codes[e * slice_words + widx] = word[e];
}

__global__ __launch_bounds__(256) void unpack_kernel(const uint32_t* __restrict__ codes, size_t slice_words,
                                                     const float2* __restrict__ meta, int64_t N, int64_t K,
                                                     int NT, int KB, uint8_t* __restrict__ out_codes,
                                                     float* __restrict__ scale, float* __restrict__ zero) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= N * K) return;
  const int64_t n = idx / K, k = idx % K;
  if (out_codes) {
    const size_t w = code_word(NT, KB, n, k);
#pragma unroll
    for (int e = 0; e < kSlices; ++e)
      out_codes[(size_t)e * N * K + idx] = (uint8_t)((codes[e * slice_words + w] >> code_bit(e, k)) & 3u);
  }
  if ((k % kGroup) == 0) {
    const int g = (int)(k / kGroup);
    const float2 m = meta[meta_index(KB, n, g)];
    if (scale) scale[n * (K / kGroup) + g] = m.x;
    if (zero) zero[n * (K / kGroup) + g] = m.y;
  }
}

// The blob seen through a slice configuration (see RouteView): slice q of the configuration is the run of bits of the
// eight-bit code after those of slice q - 1; its first-slice parameters are the blob's, moved by the power of two
// between a 2-bit and a b_0-bit first slice (exact).
__global__ __launch_bounds__(256) void unpack_view_kernel(const uint32_t* __restrict__ codes, size_t slice_words,
                                                          const float2* __restrict__ meta, int64_t N, int64_t K,
                                                          int NT, int KB, const RouteView view, int gshift,
                                                          uint8_t* __restrict__ out_codes, float* __restrict__ scale,
                                                          float* __restrict__ zero) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= N * K) return;
  const int64_t n = idx / K, k = idx % K;
  if (out_codes) {
    const size_t w = code_word(NT, KB, n, k);
    uint32_t I = 0u;  // the eight-bit code
#pragma unroll
    for (int e = 0; e < kSlices; ++e) I = I * 4u + ((codes[e * slice_words + w] >> code_bit(e, k)) & 3u);
    int before = 0;
    for (int q = 0; q < view.P; ++q) {
      const int width = view.bits[q] - before;
      out_codes[(size_t)q * N * K + idx] = (uint8_t)((I >> (2 * kSlices - view.bits[q])) & ((1u << width) - 1u));
      before = view.bits[q];
    }
  }
  if ((k & ((1 << gshift) - 1)) == 0) {
    const int g = (int)(k >> gshift);
    const float2 m = meta[meta_index(KB, n, g, kTileK >> gshift)];
    if (scale) scale[n * (K >> gshift) + g] = __builtin_ldexpf(m.x, 2 - view.bits[0]);
    if (zero) zero[n * (K >> gshift) + g] = __builtin_ldexpf(m.y, view.bits[0] - 2);
  }
}

__global__ __launch_bounds__(256) void dequant_kernel(const uint32_t* __restrict__ codes, size_t slice_words,
                                                      const float2* __restrict__ meta, int64_t N, int64_t K,
                                                      int NT, int KB, int bits, int gshift,
                                                      float* __restrict__ What) {
  // the first `bits` bits of the eight-bit code: W = s0 / 2^(bits - 2) ((I - 2^(bits - 2) z0) + 0.5)
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= N * K) return;
  const int64_t n = idx / K, k = idx % K;
  const size_t w = code_word(NT, KB, n, k);
  int I = 0;
  for (int e = 0; e < kSlices; ++e) I = I * 4 + (int)((codes[e * slice_words + w] >> code_bit(e, k)) & 3u);
  I >>= 2 * kSlices - bits;
  const float2 m = meta[meta_index(KB, n, (int)(k >> gshift), kTileK >> gshift)];
  const double pw = __builtin_ldexp(1.0, bits - 2);
  What[idx] = (float)(((double)m.x / pw) * (((double)I - pw * (double)m.y) + 0.5));
}

mbq_status launch_encode(const float* W, const Shape& sh, void* blob, const float* ext_scale, const float* ext_zero,
                         hipStream_t stream) {
  uint32_t* codes = reinterpret_cast<uint32_t*>(blob);
  float2* meta = reinterpret_cast<float2*>(reinterpret_cast<char*>(blob) + sh.meta_offset);
  dim3 grid(sh.NT, sh.KB);
  hipLaunchKernelGGL(encode_kernel, grid, dim3(256), 0, stream, W, sh.N, sh.K, sh.NT, sh.KB, codes,
                     sh.slice_words, meta, ext_scale, ext_zero);
  return hip_status(hipGetLastError(), "encode_kernel launch");
}

mbq_status launch_encode_small_group(const float* W, const Shape& sh, void* blob, hipStream_t stream) {
  uint32_t* codes = reinterpret_cast<uint32_t*>(blob);
  float2* meta = reinterpret_cast<float2*>(reinterpret_cast<char*>(blob) + sh.meta_offset);
  dim3 grid(sh.NT, sh.KB);
  hipLaunchKernelGGL(encode_small_group_kernel, grid, dim3(256), 0, stream, W, sh.N, sh.K, sh.NT, sh.KB, codes,
                     sh.slice_words, meta, sh.gshift);
  return hip_status(hipGetLastError(), "encode_small_group_kernel launch");
}

mbq_status launch_unpack(const void* blob, const Shape& sh, uint8_t* out_codes, float* scale, float* zero,
                         hipStream_t stream) {
  const uint32_t* codes = reinterpret_cast<const uint32_t*>(blob);
  const float2* meta = reinterpret_cast<const float2*>(reinterpret_cast<const char*>(blob) + sh.meta_offset);
  const int64_t total = sh.N * sh.K;
  hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, codes,
                     sh.slice_words, meta, sh.N, sh.K, sh.NT, sh.KB, out_codes, scale, zero);
  return hip_status(hipGetLastError(), "unpack_kernel launch");
}

mbq_status launch_unpack_view(const void* blob, const Shape& sh, const RouteView& view, uint8_t* out_codes,
                              float* scale, float* zero, hipStream_t stream) {
  const uint32_t* codes = reinterpret_cast<const uint32_t*>(blob);
  const float2* meta = reinterpret_cast<const float2*>(reinterpret_cast<const char*>(blob) + sh.meta_offset);
  const int64_t total = sh.N * sh.K;
  hipLaunchKernelGGL(unpack_view_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, codes,
                     sh.slice_words, meta, sh.N, sh.K, sh.NT, sh.KB, view, sh.gshift, out_codes, scale, zero);
  return hip_status(hipGetLastError(), "unpack_view_kernel launch");
}

mbq_status launch_dequant(const void* blob, const Shape& sh, int p, float* What, hipStream_t stream) {
  return launch_dequant_bits(blob, sh, 2 * (p + 1), What, stream);
}

mbq_status launch_dequant_bits(const void* blob, const Shape& sh, int bits, float* What, hipStream_t stream) {
  const uint32_t* codes = reinterpret_cast<const uint32_t*>(blob);
  const float2* meta = reinterpret_cast<const float2*>(reinterpret_cast<const char*>(blob) + sh.meta_offset);
  const int64_t total = sh.N * sh.K;
  hipLaunchKernelGGL(dequant_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, codes,
                     sh.slice_words, meta, sh.N, sh.K, sh.NT, sh.KB, bits, sh.gshift, What);
  return hip_status(hipGetLastError(), "dequant_kernel launch");
}

}  // namespace mbq
