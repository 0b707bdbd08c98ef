// Measurement and diagnostic entry points (include/mbq_bench.h): what the chip itself reaches on a plain
// copy, a read-only stream and an LDS-fed MFMA loop, and the decode linear kernel alone / with a timeline.
#include "mbq_bench.h"
#include "mbq_common.h"

namespace mbq {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

static int bench_compute_units() { return device_compute_units(); }

// four 16-byte loads in flight per lane and round
__global__ __launch_bounds__(512) void bench_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                         size_t n_vec) {
  const size_t stride = (size_t)gridDim.x * 512;
  size_t i = (size_t)blockIdx.x * 512 + threadIdx.x;
  for (; i + 3 * stride < n_vec; i += 4 * stride) {
    const u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride),
                c = __builtin_nontemporal_load(src + i + 2 * stride), d = __builtin_nontemporal_load(src + i + 3 * stride);
    __builtin_nontemporal_store(a, dst + i);
    __builtin_nontemporal_store(b, dst + i + stride);
    __builtin_nontemporal_store(c, dst + i + 2 * stride);
    __builtin_nontemporal_store(d, dst + i + 3 * stride);
  }
  for (; i < n_vec; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

__global__ __launch_bounds__(512) void bench_read_kernel(const u32x4* __restrict__ src, size_t n_vec,
                                                         uint32_t* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * 512;
  size_t i = (size_t)blockIdx.x * 512 + threadIdx.x;
  uint32_t fold = 0u;
  for (; i + 7 * stride < n_vec; i += 8 * stride) {
    u32x4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(src + i + j * stride);
#pragma unroll
    for (int j = 0; j < 8; ++j) fold += v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
  }
  for (; i < n_vec; i += stride) {
    const u32x4 v = __builtin_nontemporal_load(src + i);
    fold += v.x ^ v.y ^ v.z ^ v.w;
  }
  if (fold == 0x9E3779B9u) *sink = fold;
}

// One workgroup = 8 wavefronts as 2 x 4, wavefront tile 128 x 64 = 4 x 2 accumulators of 32 x 32; a step reads the
// A fragments (4 x 16 bytes per lane and k half) and B fragments (2 x 16 bytes) from LDS and issues 16 MFMAs.
template <bool kBarrier>
__global__ __launch_bounds__(512) void bench_mfma_kernel(int steps, float* __restrict__ sink) {
  __shared__ __attribute__((aligned(16))) char smem[2 * 16384 + 2 * 20480];
  for (int i = threadIdx.x; i < (int)sizeof(smem) / 4; i += 512) reinterpret_cast<uint32_t*>(smem)[i] = 0x3C003C00u;
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave >> 2, wn = wave & 3;
  floatx16 acc[4][2];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
  const uint32_t fa = (32 * wm + (lane & 31)) * 64 + (lane >> 5) * 16;                 // 256 rows x 64 bytes
  const uint32_t fb = 2 * 16384 + (64 * wn + (lane & 31)) * 80 + (lane >> 5) * 16;     // 256 rows x 80 bytes
  for (int h = 0; h < steps; ++h) {
    const char* pa = smem + (h & 1) * 16384 + fa;
    const char* pb = smem + (h & 1) * 20480 + fb;
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      u32x4 af[4], bf[2];
#pragma unroll
      for (int a = 0; a < 4; ++a) af[a] = *reinterpret_cast<const u32x4*>(pa + a * 4096 + kk * 32);
#pragma unroll
      for (int b = 0; b < 2; ++b) bf[b] = *reinterpret_cast<const u32x4*>(pb + b * 2560 + kk * 32);
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[a]),
                                                              __builtin_bit_cast(bf16x8, bf[b]), acc[a][b], 0, 0, 0);
    }
    if constexpr (kBarrier) __syncthreads();
  }
  float s = 0.f;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) s += acc[a][b][i];
  if (s == 1234.5f) *sink = s;
}

static bool group_args(const char* who, int64_t T, int64_t K, int n_proj, const void* const* blob_host,
                       const int64_t* N_host, const int32_t* const* prec_host, float* const* Y_host, const void* ws,
                       size_t ws_bytes, Shape* sh, mbq_status* st) {
  *st = MBQ_ERR_INVALID_ARG;
  if (n_proj < 1 || n_proj > MBQ_MAX_GROUP || !blob_host || !N_host || !prec_host || !Y_host || !ws ||
      ((uintptr_t)ws % 256) != 0) {
    set_error("%s: bad projection count, null pointer array or null/misaligned workspace", who);
    return false;
  }
  size_t need = 0;
  for (int i = 0; i < n_proj; ++i) {
    if (!make_shape(N_host[i], K, &sh[i])) {
      *st = MBQ_ERR_BAD_SHAPE;
      return false;
    }
    if (!blob_host[i] || !prec_host[i] || !Y_host[i] || ((uintptr_t)blob_host[i] % 256) != 0) {
      set_error("%s: null or misaligned pointer for projection %d", who, i);
      return false;
    }
    const size_t b = mbq_linear_workspace_bytes(T, N_host[i], K);
    if (b > need) need = b;
  }
  if (!decode_f4_supports(T, sh[0])) {
    set_error("%s: only the one-token-tile decode kernels (1 <= T <= 16), T=%lld", who, (long long)T);
    *st = MBQ_ERR_BAD_SHAPE;
    return false;
  }
  if (ws_bytes < need) {
    set_error("%s: workspace too small (%zu < %zu)", who, ws_bytes, need);
    *st = MBQ_ERR_WORKSPACE;
    return false;
  }
  *st = MBQ_OK;
  return true;
}

}  // namespace mbq

using namespace mbq;

extern "C" {

mbq_status mbq_bench_copy(const void* src, void* dst, size_t bytes, int waves_of_workgroups, void* stream) {
  if (!src || !dst || bytes % 16 != 0 || ((uintptr_t)src % 16) != 0 || ((uintptr_t)dst % 16) != 0 ||
      waves_of_workgroups < 1 || waves_of_workgroups > 64) {
    set_error("mbq_bench_copy: null/misaligned pointer, size not a multiple of 16 or bad launch width");
    return MBQ_ERR_INVALID_ARG;
  }
  if (bytes == 0) return MBQ_OK;
  hipLaunchKernelGGL(bench_copy_kernel, dim3(bench_compute_units() * waves_of_workgroups), dim3(512), 0,
                     (hipStream_t)stream, reinterpret_cast<const u32x4*>(src), reinterpret_cast<u32x4*>(dst),
                     bytes / 16);
  return hip_status(hipGetLastError(), "bench_copy_kernel launch");
}

mbq_status mbq_bench_read(const void* src, size_t bytes, int waves_of_workgroups, void* sink, void* stream) {
  if (!src || !sink || bytes % 16 != 0 || ((uintptr_t)src % 16) != 0 || waves_of_workgroups < 1 ||
      waves_of_workgroups > 64) {
    set_error("mbq_bench_read: null/misaligned pointer, size not a multiple of 16 or bad launch width");
    return MBQ_ERR_INVALID_ARG;
  }
  if (bytes == 0) return MBQ_OK;
  hipLaunchKernelGGL(bench_read_kernel, dim3(bench_compute_units() * waves_of_workgroups), dim3(512), 0,
                     (hipStream_t)stream, reinterpret_cast<const u32x4*>(src), bytes / 16,
                     reinterpret_cast<uint32_t*>(sink));
  return hip_status(hipGetLastError(), "bench_read_kernel launch");
}

mbq_status mbq_bench_mfma_loop(int steps, int with_barrier, void* sink, double* flops_host, void* stream) {
  if (steps < 1 || steps > (1 << 24) || !sink) {
    set_error("mbq_bench_mfma_loop: steps outside 1..2^24 or null sink");
    return MBQ_ERR_INVALID_ARG;
  }
  const int cus = bench_compute_units();
  if (with_barrier)
    hipLaunchKernelGGL(bench_mfma_kernel<true>, dim3(cus), dim3(512), 0, (hipStream_t)stream, steps,
                       reinterpret_cast<float*>(sink));
  else
    hipLaunchKernelGGL(bench_mfma_kernel<false>, dim3(cus), dim3(512), 0, (hipStream_t)stream, steps,
                       reinterpret_cast<float*>(sink));
  if (flops_host) *flops_host = (double)cus * 8.0 * (double)steps * 16.0 * (2.0 * 32 * 32 * 16);
  return hip_status(hipGetLastError(), "bench_mfma_kernel launch");
}

mbq_status mbq_bench_linear_group_prepared(int64_t T, int64_t K, int n_proj, const void* const* blob_host,
                                           const int64_t* N_host, const int32_t* const* prec_host,
                                           float* const* Y_host, const void* ws, size_t ws_bytes, void* stream) {
  ApiScope scope;
  Shape sh[MBQ_MAX_GROUP];
  mbq_status st;
  if (!group_args("mbq_bench_linear_group_prepared", T, K, n_proj, blob_host, N_host, prec_host, Y_host, ws, ws_bytes,
                  sh, &st))
    return st;
  return launch_linear_decode_f4(T, n_proj, blob_host, sh, prec_host, Y_host, ws, (hipStream_t)stream, nullptr,
                                 nullptr);
}

size_t mbq_bench_decode_timeline_bytes(void) {
  return (size_t)decode_f4_timeline_workgroups() * (size_t)decode_f4_timeline_slots() * 8;
}
int mbq_bench_decode_timeline_workgroups(void) { return decode_f4_timeline_workgroups(); }

mbq_status mbq_bench_decode_timeline(int64_t T, int64_t K, int n_proj, const void* const* blob_host,
                                     const int64_t* N_host, const int32_t* const* prec_host, float* const* Y_host,
                                     const void* ws, size_t ws_bytes, unsigned long long* stamps,
                                     size_t stamps_bytes, void* stream) {
  ApiScope scope;
  Shape sh[MBQ_MAX_GROUP];
  mbq_status st;
  if (!group_args("mbq_bench_decode_timeline", T, K, n_proj, blob_host, N_host, prec_host, Y_host, ws, ws_bytes, sh,
                  &st))
    return st;
  if (!stamps || stamps_bytes < mbq_bench_decode_timeline_bytes()) {
    set_error("mbq_bench_decode_timeline: stamps buffer null or smaller than %zu bytes",
              mbq_bench_decode_timeline_bytes());
    return MBQ_ERR_INVALID_ARG;
  }
  return launch_linear_decode_f4(T, n_proj, blob_host, sh, prec_host, Y_host, ws, (hipStream_t)stream, nullptr,
                                 nullptr, stamps);
}

}  // extern "C"
