// Router scores + argmax (paper Sec. 4.2 Eq. 4, read as one linear map to four
// logits) and the token permutation by precision (Sec. 4.3, challenge 3).
#include "mbq_common.h"

namespace mbq {

constexpr int kP = MBQ_N_PRECISIONS;

__device__ inline float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

// Stable counting sort of token ids by precision by ONE workgroup of NW wavefronts
// (Sec. 4.3, token permutation).  Counting and ranking use wavefront ballots: a lane's rank
// inside its wavefront is the population count of the ballot below its lane.
template <int NW>
__device__ inline void bucket_by_workgroup(const int32_t* prec, int64_t T,
                                           int32_t* __restrict__ perm, int32_t* __restrict__ offsets) {
  __shared__ int s_wave[NW][kP];  // per-wavefront counts of the current pass
  __shared__ int s_run[kP];       // running write position of each precision
  constexpr int NT = NW * 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));

  // pass 1: totals
  int cnt[kP] = {0, 0, 0, 0};
  for (int64_t base = 0; base < T; base += NT) {
    const int64_t i = base + tid;
    const int p = (i < T) ? prec[i] : -1;
#pragma unroll
    for (int q = 0; q < kP; ++q) cnt[q] += __popcll(__ballot(p == q));
  }
  if (lane == 0)
#pragma unroll
    for (int q = 0; q < kP; ++q) s_wave[wave][q] = cnt[q];
  __syncthreads();
  if (tid == 0) {
    int pos = 0;
    for (int q = 0; q < kP; ++q) {
      int c = 0;
      for (int w = 0; w < NW; ++w) c += s_wave[w][q];
      s_run[q] = pos;
      offsets[q] = pos;
      pos += c;
    }
    offsets[kP] = pos;
  }
  __syncthreads();

  // pass 2: stable placement, NT tokens at a time in token order
  for (int64_t base = 0; base < T; base += NT) {
    const int64_t i = base + tid;
    const int p = (i < T) ? prec[i] : -1;
    int rank_in_wave = 0;
#pragma unroll
    for (int q = 0; q < kP; ++q) {
      const uint64_t b = __ballot(p == q);
      if (p == q) rank_in_wave = __popcll(b & below);
      if (lane == 0) s_wave[wave][q] = __popcll(b);
    }
    __syncthreads();
    if (p >= 0) {
      int pos = s_run[p] + rank_in_wave;
      for (int w = 0; w < wave; ++w) pos += s_wave[w][p];
      perm[pos] = (int32_t)i;
    }
    __syncthreads();
    if (tid < kP) {
      int c = 0;
      for (int w = 0; w < NW; ++w) c += s_wave[w][tid];
      s_run[tid] += c;
    }
    __syncthreads();
  }
}

// One workgroup of 256 threads scores TPW consecutive tokens (Sec. 4.2 Eq. 4).  The K axis
// is split over the threads in chunks of 8 columns; each thread keeps 4 x TPW fp64 partial
// sums (bf16 x fp32 products are exact in fp64), reduced over the wavefront with shuffles and
// over the four wavefronts through LDS.  The workgroup that finishes last (a ticket counter in
// the workspace, left at zero again) then buckets all tokens, so routing is one launch.
template <int TPW>
__global__ __launch_bounds__(256) void route_kernel(const uint16_t* __restrict__ X, int64_t T, int64_t K,
                                                    const float* __restrict__ Wr, const float* __restrict__ br,
                                                    int32_t* prec, int32_t* __restrict__ perm,
                                                    int32_t* __restrict__ offsets, double* __restrict__ logits,
                                                    unsigned int* __restrict__ ticket) {
  const int64_t tok0 = (int64_t)blockIdx.x * TPW;
  const int tid = threadIdx.x;
  double acc[TPW][kP];
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int q = 0; q < kP; ++q) acc[t][q] = 0.0;

  for (int64_t k = (int64_t)tid * 8; k < K; k += 256 * 8) {
    float w[kP][8];
#pragma unroll
    for (int q = 0; q < kP; ++q) {
      const float4* src = reinterpret_cast<const float4*>(Wr + (int64_t)q * K + k);
      float4 a = src[0], b = src[1];
      w[q][0] = a.x; w[q][1] = a.y; w[q][2] = a.z; w[q][3] = a.w;
      w[q][4] = b.x; w[q][5] = b.y; w[q][6] = b.z; w[q][7] = b.w;
    }
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
      if (tok0 + t < T) {
        const uint4 xv = *reinterpret_cast<const uint4*>(X + (tok0 + t) * K + k);
        const float x[8] = {bf16_lo(xv.x), bf16_hi(xv.x), bf16_lo(xv.y), bf16_hi(xv.y),
                            bf16_lo(xv.z), bf16_hi(xv.z), bf16_lo(xv.w), bf16_hi(xv.w)};
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
          for (int q = 0; q < kP; ++q) acc[t][q] = fma((double)x[j], (double)w[q][j], acc[t][q]);
      }
    }
  }
  __shared__ double red[4][TPW][kP];
  __shared__ unsigned int s_ticket;
  const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int q = 0; q < kP; ++q) {
      double v = acc[t][q];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) v += __shfl_down(v, off, 64);
      if (lane == 0) red[wave][t][q] = v;
    }
  __syncthreads();
  if (tid < TPW && tok0 + tid < T) {
    double best = 0.0;
    int arg = 0;
#pragma unroll
    for (int q = 0; q < kP; ++q) {
      const double s = ((red[0][tid][q] + red[1][tid][q]) + (red[2][tid][q] + red[3][tid][q])) + (double)br[q];
      if (logits) logits[(tok0 + tid) * kP + q] = s;
      if (q == 0 || s > best) {  // strict: the first maximum wins ties
        best = s;
        arg = q;
      }
    }
    prec[tok0 + tid] = arg;
    __threadfence();  // publish this workgroup's choices before taking a ticket
  }
  __syncthreads();
  if (tid == 0) s_ticket = atomicAdd(ticket, 1u);
  __syncthreads();
  if (s_ticket != gridDim.x - 1) return;
  // last workgroup: every token's precision is visible now
  __threadfence();
  bucket_by_workgroup<4>(prec, T, perm, offsets);
  if (tid == 0) *ticket = 0u;  // leave the counter ready for the next call
}

// T = 0: only the (all-zero) offsets have to be written.
__global__ __launch_bounds__(64) void bucket_kernel(const int32_t* __restrict__ prec, int64_t T,
                                                    int32_t* __restrict__ perm, int32_t* __restrict__ offsets) {
  bucket_by_workgroup<1>(prec, T, perm, offsets);
}

mbq_status launch_route(const uint16_t* X, int64_t T, int64_t K, const float* Wr, const float* br,
                        int32_t* prec, int32_t* perm, int32_t* offsets, double* logits, void* ws,
                        hipStream_t stream) {
  unsigned int* ticket = reinterpret_cast<unsigned int*>(ws);
  if (T == 0) {
    hipLaunchKernelGGL(bucket_kernel, dim3(1), dim3(64), 0, stream, prec, T, perm, offsets);
    return hip_status(hipGetLastError(), "bucket_kernel launch");
  }
  if (T <= 256) {
    hipLaunchKernelGGL(route_kernel<1>, dim3((unsigned)T), dim3(256), 0, stream, X, T, K, Wr, br, prec, perm,
                       offsets, logits, ticket);
  } else {
    hipLaunchKernelGGL(route_kernel<4>, dim3((unsigned)((T + 3) / 4)), dim3(256), 0, stream, X, T, K, Wr, br,
                       prec, perm, offsets, logits, ticket);
  }
  return hip_status(hipGetLastError(), "route_kernel launch");
}

}  // namespace mbq
