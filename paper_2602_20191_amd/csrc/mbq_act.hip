// Activation-quantised variant of the layer (paper App. E.4; `abits` of App. C.1): per-token quantiser of the
// transformed activations X~ = (X - delta) / s, the integers q - zp as the main path's bf16 operand, the router's
// input rebuilt in the original space (X_r = X~ s + delta), and the row scaling that finishes the main path.
//
// This translation unit is compiled with -ffp-contract=off: every step of the quantiser is one fp32 operation
// (the codes must not depend on how the compiler fuses them).
#include "mbq_common.h"

namespace mbq {

__device__ __forceinline__ float bf16_value(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
// round to nearest even; finite inputs
__device__ __forceinline__ uint32_t bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

// One workgroup per token.  Pass 1 finds the row's extremes (zero included), pass 2 writes the codes.  kHold > 0: the
// row fits in kHold chunks of eight values per thread and the transformed values of pass 1 stay in registers;
// kHold = 0: pass 2 re-reads the row (it is in cache) and computes the transformed values again with the same two
// operations.
template <int kThreads, int kHold>
__global__ __launch_bounds__(kThreads) void act_quant_kernel(const uint16_t* __restrict__ X, int64_t K, int abits,
                                                        const float* __restrict__ let_shift,
                                                        const float* __restrict__ let_scale,
                                                        uint16_t* __restrict__ Xint, float* __restrict__ row_scale,
                                                        uint16_t* __restrict__ Xr) {
#pragma clang fp contract(off)
  const int64_t row = blockIdx.x;
  const int tid = threadIdx.x;
  const uint4* x8 = reinterpret_cast<const uint4*>(X + row * K);  // eight bf16 values per load
  const int n8 = (int)(K >> 3);
  const bool let = let_scale != nullptr;

  auto transformed = [&](int j, float t[8]) {
    const uint4 v = x8[j];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      t[2 * h] = bf16_value(w[h] & 0xFFFFu);
      t[2 * h + 1] = bf16_value(w[h] >> 16);
    }
    if (let) {
      const float4 d0 = reinterpret_cast<const float4*>(let_shift)[2 * j];
      const float4 d1 = reinterpret_cast<const float4*>(let_shift)[2 * j + 1];
      const float4 s0 = reinterpret_cast<const float4*>(let_scale)[2 * j];
      const float4 s1 = reinterpret_cast<const float4*>(let_scale)[2 * j + 1];
      const float d[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
      const float s[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
#pragma unroll
      for (int h = 0; h < 8; ++h) t[h] = (t[h] - d[h]) / s[h];
    }
  };

  float lo = 0.f, hi = 0.f;
  float held[kHold > 0 ? kHold : 1][8];
  if constexpr (kHold > 0) {
#pragma unroll
    for (int c = 0; c < kHold; ++c) {
      const int j = tid + c * kThreads;
      if (j < n8) {
        transformed(j, held[c]);
#pragma unroll
        for (int h = 0; h < 8; ++h) {
          lo = fminf(lo, held[c][h]);
          hi = fmaxf(hi, held[c][h]);
        }
      }
    }
  } else {
    for (int j = tid; j < n8; j += kThreads) {
      float t[8];
      transformed(j, t);
#pragma unroll
      for (int h = 0; h < 8; ++h) {
        lo = fminf(lo, t[h]);
        hi = fmaxf(hi, t[h]);
      }
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    lo = fminf(lo, __shfl_xor(lo, off));
    hi = fmaxf(hi, __shfl_xor(hi, off));
  }
  constexpr int kWavefronts = kThreads / 64;
  __shared__ float s_lo[kWavefronts], s_hi[kWavefronts];
  if ((tid & 63) == 0) {
    s_lo[tid >> 6] = lo;
    s_hi[tid >> 6] = hi;
  }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kWavefronts; ++w) {
    lo = fminf(lo, s_lo[w]);
    hi = fmaxf(hi, s_hi[w]);
  }

  const float top = (float)((1 << abits) - 1);
  const float rng = fmaxf(hi - lo, 0x1p-100f);
  const float scale = rng / top;
  const float zp = fminf(fmaxf(rintf((-lo) / scale), 0.f), top);
  if (tid == 0) row_scale[row] = scale;

  uint4* out8 = reinterpret_cast<uint4*>(Xint + row * K);
  uint4* xr8 = Xr ? reinterpret_cast<uint4*>(Xr + row * K) : nullptr;
  auto write_chunk = [&](int j, const float t[8]) {
    float xi[8];
#pragma unroll
    for (int h = 0; h < 8; ++h) {
      const float q = fminf(fmaxf(rintf(t[h] / scale) + zp, 0.f), top);
      xi[h] = q - zp;  // an integer of at most abits bits and a sign: exact in bf16
    }
    uint4 o;
    o.x = bf16_bits(xi[0]) | (bf16_bits(xi[1]) << 16);
    o.y = bf16_bits(xi[2]) | (bf16_bits(xi[3]) << 16);
    o.z = bf16_bits(xi[4]) | (bf16_bits(xi[5]) << 16);
    o.w = bf16_bits(xi[6]) | (bf16_bits(xi[7]) << 16);
    out8[j] = o;
    if (xr8) {
      float r[8];
#pragma unroll
      for (int h = 0; h < 8; ++h) r[h] = xi[h] * scale;
      if (let) {
        const float4 d0 = reinterpret_cast<const float4*>(let_shift)[2 * j];
        const float4 d1 = reinterpret_cast<const float4*>(let_shift)[2 * j + 1];
        const float4 s0 = reinterpret_cast<const float4*>(let_scale)[2 * j];
        const float4 s1 = reinterpret_cast<const float4*>(let_scale)[2 * j + 1];
        const float d[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
        const float s[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
#pragma unroll
        for (int h = 0; h < 8; ++h) r[h] = r[h] * s[h] + d[h];
      }
      uint4 p;
      p.x = bf16_bits(r[0]) | (bf16_bits(r[1]) << 16);
      p.y = bf16_bits(r[2]) | (bf16_bits(r[3]) << 16);
      p.z = bf16_bits(r[4]) | (bf16_bits(r[5]) << 16);
      p.w = bf16_bits(r[6]) | (bf16_bits(r[7]) << 16);
      xr8[j] = p;
    }
  };
  if constexpr (kHold > 0) {
#pragma unroll
    for (int c = 0; c < kHold; ++c) {
      const int j = tid + c * kThreads;
      if (j < n8) write_chunk(j, held[c]);
    }
  } else {
    for (int j = tid; j < n8; j += kThreads) {
      float t[8];
      transformed(j, t);
      write_chunk(j, t);
    }
  }
}

// Y[i][n] = Y[i][n] * row_scale[i] (+ bias[n]): one multiplication and one addition, in place.
__global__ __launch_bounds__(256) void scale_rows_kernel(float* __restrict__ Y, int64_t total, int64_t N,
                                                         const float* __restrict__ row_scale,
                                                         const float* __restrict__ bias) {
#pragma clang fp contract(off)
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int64_t i = idx / N, n = idx - i * N;
  float y = Y[idx] * row_scale[i];
  if (bias) y = y + bias[n];
  Y[idx] = y;
}

struct ScaleList {
  float* Y[MBQ_MAX_GROUP];
  const float* bias[MBQ_MAX_GROUP];
  long long total[MBQ_MAX_GROUP];  // T * N
  int N[MBQ_MAX_GROUP];
};
__global__ __launch_bounds__(256) void scale_rows_group_kernel(const ScaleList list,
                                                               const float* __restrict__ row_scale) {
#pragma clang fp contract(off)
  const int j = blockIdx.y;
  float* __restrict__ Y = list.Y[j];
  const float* __restrict__ bias = list.bias[j];
  const long long total = list.total[j];
  const int N = list.N[j];
  for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long long)gridDim.x * 256) {
    const long long i = idx / N;
    float y = Y[idx] * row_scale[i];
    if (bias) y = y + bias[idx - i * N];
    Y[idx] = y;
  }
}

mbq_status launch_scale_rows_group(int n, float* const* Y, int64_t T, const int64_t* N, const float* row_scale,
                                   const float* const* bias, hipStream_t stream) {
  ScaleList list = {};
  long long most = 0;
  for (int j = 0; j < n; ++j) {
    list.Y[j] = Y[j];
    list.bias[j] = bias ? bias[j] : nullptr;
    list.total[j] = (long long)T * N[j];
    list.N[j] = (int)N[j];
    if (list.total[j] > most) most = list.total[j];
  }
  long long blocks = (most + 255) / 256;
  if (blocks > 65536) blocks = 65536;  // the kernel strides
  hipLaunchKernelGGL(scale_rows_group_kernel, dim3((unsigned)blocks, (unsigned)n), dim3(256), 0, stream, list,
                     row_scale);
  return hip_status(hipGetLastError(), "scale_rows_group_kernel launch");
}

mbq_status launch_act_quant(const uint16_t* X, int64_t T, int64_t K, int abits, const float* let_shift,
                            const float* let_scale, uint16_t* Xint, float* row_scale, uint16_t* Xr,
                            hipStream_t stream) {
  // up to 16384 columns a row is held in registers by 512 threads (four chunks of eight values each)
  if (K <= 512 * 4 * 8)
    hipLaunchKernelGGL((act_quant_kernel<512, 4>), dim3((unsigned)T), dim3(512), 0, stream, X, K, abits, let_shift,
                       let_scale, Xint, row_scale, Xr);
  else
    hipLaunchKernelGGL((act_quant_kernel<256, 0>), dim3((unsigned)T), dim3(256), 0, stream, X, K, abits, let_shift,
                       let_scale, Xint, row_scale, Xr);
  return hip_status(hipGetLastError(), "act_quant_kernel launch");
}

mbq_status launch_scale_rows(float* Y, int64_t T, int64_t N, const float* row_scale, const float* bias,
                             hipStream_t stream) {
  const int64_t total = T * N;
  hipLaunchKernelGGL(scale_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, Y, total, N,
                     row_scale, bias);
  return hip_status(hipGetLastError(), "scale_rows_kernel launch");
}

}  // namespace mbq
