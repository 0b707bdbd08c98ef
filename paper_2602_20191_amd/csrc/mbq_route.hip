// Router scores + argmax (paper Sec. 4.2 Eq. 4, read as one linear map to four
// logits) and the token permutation by precision (Sec. 4.3, challenge 3).
#include "mbq_common.h"
#include "mbq_f4_prep.h"

namespace mbq {

constexpr int kP = MBQ_N_PRECISIONS;

__device__ inline float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

// Stable counting sort of token ids by precision by ONE workgroup of NW wavefronts
// (Sec. 4.3, token permutation).  Counting and ranking use wavefront ballots: a lane's rank
// inside its wavefront is the population count of the ballot below its lane.
template <int NW>
__device__ inline void bucket_by_workgroup(const int32_t* prec, int64_t T,
                                           int32_t* __restrict__ perm, int32_t* __restrict__ offsets, int shift = 0) {
  __shared__ int s_wave[NW][kP];  // per-wavefront counts of the current pass
  __shared__ int s_run[kP];       // running write position of each precision
  constexpr int NT = NW * 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));

  // pass 1: totals
  int cnt[kP] = {0, 0, 0, 0};
  for (int64_t base = 0; base < T; base += NT) {
    const int64_t i = base + tid;
    const int p = (i < T) ? (prec[i] >> shift) : -1;
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
    const int p = (i < T) ? (prec[i] >> shift) : -1;
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

// Cross-lane moves of a double through the data-parallel-primitive path of the vector ALU (no LDS
// round trip as for a general shuffle): CTRL is a DPP control word, here a permutation inside each
// group of four lanes (quad_perm) or a rotation inside each row of 16 lanes (row_ror).
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
  const long long b = __builtin_bit_cast(long long, v);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(unsigned)(b & 0xFFFFFFFFll), CTRL, 0xF, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, 0xF, 0xF, false);
  return __builtin_bit_cast(double, ((long long)hi << 32) | (long long)(unsigned)lo);
}
constexpr int kDppQuadXor1 = 0xB1, kDppQuadXor2 = 0x4E;  // quad_perm [1,0,3,2], [2,3,0,1]
constexpr int kDppRowRor4 = 0x124, kDppRowRor8 = 0x128;

// Sums four per-lane values over the wavefront.  The first two exchanges halve the number of values a
// lane carries (lanes 1 apart split the four between them, then lanes 2 apart), so that seven moves of
// a double do the work of twenty-four; afterwards lane l holds the total of value wave_sum4_index(l).
__device__ __forceinline__ int wave_sum4_index(int lane) { return 2 * (lane & 1) + ((lane >> 1) & 1); }
__device__ __forceinline__ double wave_sum4(const double (&acc)[4], int lane) {
  const bool odd = (lane & 1) != 0, upper = (lane & 2) != 0;
  double keep0 = odd ? acc[2] : acc[0], keep1 = odd ? acc[3] : acc[1];
  keep0 += dpp_move<kDppQuadXor1>(odd ? acc[0] : acc[2]);
  keep1 += dpp_move<kDppQuadXor1>(odd ? acc[1] : acc[3]);
  double v = upper ? keep1 : keep0;
  v += dpp_move<kDppQuadXor2>(upper ? keep0 : keep1);
  v += dpp_move<kDppRowRor4>(v);
  v += dpp_move<kDppRowRor8>(v);
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  return v;
}

// One workgroup of 256 threads scores TPW consecutive tokens (Sec. 4.2 Eq. 4).  The K axis
// is split over the threads in chunks of 8 columns; each thread keeps 4 x TPW fp64 partial
// sums (bf16 x fp32 products are exact in fp64), reduced over the wavefront (wave_sum4) and
// over the four wavefronts through LDS.  The workgroup that finishes last (a ticket counter in
// the workspace, cleared ahead of the launch) then buckets all tokens.
template <int TPW>
__global__ __launch_bounds__(256) void route_kernel(const uint16_t* __restrict__ X, int64_t T, int64_t K,
                                                    const float* __restrict__ Wr, const float* __restrict__ br,
                                                    int32_t* prec, int32_t* __restrict__ perm,
                                                    int32_t* __restrict__ offsets, double* __restrict__ logits,
                                                    unsigned int* __restrict__ ticket, const RouteView view) {
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
      const float4* src = reinterpret_cast<const float4*>(Wr + (int64_t)min(q, view.P - 1) * K + k);  // rows past P: unused
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
  for (int t = 0; t < TPW; ++t) {
    const double v = wave_sum4(acc[t], lane);
    if (lane < kP) red[wave][t][wave_sum4_index(lane)] = v;
  }
  __syncthreads();
  if (tid < TPW && tok0 + tid < T) {
    double best = 0.0;
    int arg = 0;
#pragma unroll
    for (int q = 0; q < kP; ++q) {
      if (q < view.P) {
        const double s = ((red[0][tid][q] + red[1][tid][q]) + (red[2][tid][q] + red[3][tid][q])) + (double)br[q];
        if (logits) logits[(tok0 + tid) * view.P + q] = s;
        if (q == 0 || s > best) {  // strict: the first maximum wins ties
          best = s;
          arg = q;
        }
      }
    }
    prec[tok0 + tid] = view.value[arg];
    __threadfence();  // publish this workgroup's choices before taking a ticket
  }
  __syncthreads();
  if (tid == 0) s_ticket = atomicAdd(ticket, 1u);
  __syncthreads();
  if (s_ticket != gridDim.x - 1) return;
  // last workgroup: every token's precision is visible now
  __threadfence();
  bucket_by_workgroup<4>(prec, T, perm, offsets, view.shift);
  if (tid == 0) *ticket = 0u;  // leave the counter ready for the next call
}

// Small batches (T <= 128; the packed meeting word below up to kSmallRouteTokens), one or several routers over the same activations
// (the projections of a decoder block that share their input, Sec. 4.3, fused router launch).
// blockIdx.x = token, blockIdx.y = router.  512 threads split the K axis in chunks of 8 columns,
// two chunks in flight per thread.  Workgroups meet through ONE 64-bit atomic add per token: the
// word carries 2 bits per token and an arrival count in its top byte, so the workgroup that
// arrives last holds every token's precision in the returned value and buckets them with
// wavefront ballots, without fences or a second pass over memory.  The word is cleared ahead of the launch.
constexpr int kSmallRouteTokens = 28;
constexpr int kRouteGroupMax = MBQ_MAX_GROUP;

struct RouteOut {
  const float* Wr;
  const float* br;
  int32_t* prec;
  int32_t* perm;
  int32_t* offsets;
  double* logits;
};
struct RouteGroup {
  RouteOut r[kRouteGroupMax];
  RouteView view;
};

//
// The launch can carry the activation preparation of the FP4-operand decode kernel along: plane
// blockIdx.y == n_routers of the grid prepares 256-column block blockIdx.x with its first
// wavefront (prep == nullptr: no such plane).  defer_bucket: only the precisions are written; the linear
// kernel that follows sorts the tokens (it reads every precision anyway), which takes the atomic
// round trip and the sort out of this launch.
__global__ __launch_bounds__(512) void route_small_kernel(const uint16_t* __restrict__ X, int T, int64_t K,
                                                          RouteGroup group, int n_routers,
                                                          unsigned long long* words, char* prep, int prep_blocks,
                                                          const ZeroList zl, int defer_bucket,
                                                          const uint16_t* __restrict__ Xprep) {
  // Xprep: the activations the linear kernel multiplies (X itself, except in the activation-quantised variant,
  // where the routers read the rebuilt activations and the linear kernel the integers)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if ((int)blockIdx.y == n_routers) {
    if (wave == 0) {
      if ((int)blockIdx.x < prep_blocks) f4::prep_block(Xprep, T, K, prep, (int)blockIdx.x, lane);
    } else {
      zero_share(zl, (int)blockIdx.x, (int)gridDim.x, tid - 64, 448);  // outputs a split-K linear kernel adds into
    }
    return;
  }
  if ((int)blockIdx.x >= T) return;
  const RouteOut& out = group.r[blockIdx.y];
  const int tok = blockIdx.x;
  const uint16_t* x = X + (int64_t)tok * K;
  const float* __restrict__ Wr = out.Wr;
  double acc[kP] = {0.0, 0.0, 0.0, 0.0};
  for (int64_t k = (int64_t)tid * 8; k < K; k += 2 * 4096) {
    const bool two = k + 4096 < K;
    const int64_t k2 = two ? k + 4096 : k;  // a valid address either way
    const uint4 xa = *reinterpret_cast<const uint4*>(x + k);
    const uint4 xb = *reinterpret_cast<const uint4*>(x + k2);
    float4 wa[kP][2], wb[kP][2];
#pragma unroll
    for (int q = 0; q < kP; ++q) {
      const int64_t row = min(q, group.view.P - 1);  // rows past P do not exist: re-read the last one, never used
      const float4* sa = reinterpret_cast<const float4*>(Wr + row * K + k);
      const float4* sb = reinterpret_cast<const float4*>(Wr + row * K + k2);
      wa[q][0] = sa[0]; wa[q][1] = sa[1];
      wb[q][0] = sb[0]; wb[q][1] = sb[1];
    }
    auto add = [&](const uint4& xv, const float4 (&w)[kP][2]) {
      const float xs[8] = {bf16_lo(xv.x), bf16_hi(xv.x), bf16_lo(xv.y), bf16_hi(xv.y),
                           bf16_lo(xv.z), bf16_hi(xv.z), bf16_lo(xv.w), bf16_hi(xv.w)};
#pragma unroll
      for (int q = 0; q < kP; ++q) {
        const float ws[8] = {w[q][0].x, w[q][0].y, w[q][0].z, w[q][0].w, w[q][1].x, w[q][1].y, w[q][1].z, w[q][1].w};
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[q] = fma((double)xs[j], (double)ws[j], acc[q]);
      }
    };
    add(xa, wa);
    if (two) add(xb, wb);
  }
  __shared__ double red[8][kP];
  {
    const double v = wave_sum4(acc, lane);
    if (lane < kP) red[wave][wave_sum4_index(lane)] = v;
  }
  __syncthreads();
  if (wave != 0) return;
  // lanes 0..3 finish one logit each; every lane then sees all four
  const int P = group.view.P;
  double mine = 0.0;
  if (lane < P) {
    mine = ((red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane])) +
           ((red[4][lane] + red[5][lane]) + (red[6][lane] + red[7][lane])) + (double)out.br[lane];
    if (out.logits) out.logits[(int64_t)tok * P + lane] = mine;
  }
  double best = __shfl(mine, 0, 64);
  int arg = 0;
#pragma unroll
  for (int q = 1; q < kP; ++q) {
    const double s = __shfl(mine, q, 64);
    if (q < P && s > best) {  // strict: the first maximum wins ties
      best = s;
      arg = q;
    }
  }
  // the router's output q stands for the first bits[q] bits of the code: `value` is what the precision array holds,
  // `arg` from here on the digit count minus one that tokens are sorted by
  const RouteView& vw = group.view;
  const int value = arg == 0 ? vw.value[0] : arg == 1 ? vw.value[1] : arg == 2 ? vw.value[2] : vw.value[3];
  arg = arg == 0 ? vw.digits[0] : arg == 1 ? vw.digits[1] : arg == 2 ? vw.digits[2] : vw.digits[3];
  if (defer_bucket) {  // the consumer of the precisions sorts the tokens itself: no meeting, the workgroup is done
    if (lane == 0) out.prec[tok] = value;
    return;
  }
  if (T > kSmallRouteTokens) {
    // Too many tokens for the packed word: the word only counts arrivals; precisions travel through memory
    // (store, fence, count; the last to arrive fences and reads them back) and one wavefront sorts them.
    unsigned long long arrived = 0ull;
    if (lane == 0) {
      out.prec[tok] = value;
      __threadfence();
      arrived = atomicAdd(words + blockIdx.y, 1ull) + 1ull;
    }
    arrived = __shfl(arrived, 0, 64);
    if ((int)arrived != T) return;
    __threadfence();
    // stable counting sort of up to 128 tokens by one wavefront: lane holds tokens lane and lane + 64
    const int p = (lane < T) ? (__hip_atomic_load(out.prec + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> vw.shift) : -1;
    const int p2 = (lane + 64 < T) ? (__hip_atomic_load(out.prec + lane + 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> vw.shift) : -1;
    const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    int start = 0, my_pos = 0, my_pos2 = 0;
#pragma unroll
    for (int q = 0; q < kP; ++q) {
      const uint64_t b = __ballot(p == q), b2 = __ballot(p2 == q);
      if (p == q) my_pos = start + __popcll(b & below);
      if (p2 == q) my_pos2 = start + __popcll(b) + __popcll(b2 & below);
      if (lane == q) out.offsets[q] = start;
      start += __popcll(b) + __popcll(b2);
    }
    if (lane == kP) out.offsets[kP] = start;
    if (p >= 0) out.perm[my_pos] = lane;
    if (p2 >= 0) out.perm[my_pos2] = lane + 64;
    if (lane == 0) words[blockIdx.y] = 0ull;
    return;
  }
  unsigned long long all = 0ull;
  if (lane == 0) {
    out.prec[tok] = value;
    const unsigned long long inc = ((unsigned long long)arg << (2 * tok)) + (1ull << 56);
    all = atomicAdd(words + blockIdx.y, inc) + inc;
  }
  all = __shfl(all, 0, 64);
  if ((int)(all >> 56) != T) return;
  // last workgroup of this router: stable counting sort of the T tokens by precision
  const int p = (lane < T) ? (int)((all >> (2 * lane)) & 3ull) : -1;
  const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  int start = 0, my_pos = 0;
#pragma unroll
  for (int q = 0; q < kP; ++q) {
    const uint64_t b = __ballot(p == q);
    if (p == q) my_pos = start + __popcll(b & below);
    if (lane == q) out.offsets[q] = start;
    start += __popcll(b);
  }
  if (lane == kP) out.offsets[kP] = start;
  if (p >= 0) out.perm[my_pos] = lane;
  if (lane == 0) words[blockIdx.y] = 0ull;  // ready for the next call
}

// The arrival counters of a workspace (its first 256 bytes), cleared ahead of a launch that meets through them:
// a caller's workspace may hold anything, for instance what a call that was cut short left behind.
__global__ __launch_bounds__(64) void clear_counters_kernel(unsigned int* __restrict__ counters) {
  counters[threadIdx.x] = 0u;
}
static mbq_status clear_counters(void* ws, hipStream_t stream) {
  hipLaunchKernelGGL(clear_counters_kernel, dim3(1), dim3(64), 0, stream, reinterpret_cast<unsigned int*>(ws));
  return hip_status(hipGetLastError(), "clear_counters_kernel launch");
}

// T = 0: only the (all-zero) offsets have to be written.
__global__ __launch_bounds__(64) void bucket_kernel(const int32_t* __restrict__ prec, int64_t T,
                                                    int32_t* __restrict__ perm, int32_t* __restrict__ offsets) {
  bucket_by_workgroup<1>(prec, T, perm, offsets);
}

static mbq_status launch_route_one(const uint16_t* X, int64_t T, int64_t K, const float* Wr, const float* br,
                                   int32_t* prec, int32_t* perm, int32_t* offsets, double* logits,
                                   unsigned int* ticket, hipStream_t stream, const RouteView& view) {
  if (T == 0) {
    hipLaunchKernelGGL(bucket_kernel, dim3(1), dim3(64), 0, stream, prec, T, perm, offsets);
    return hip_status(hipGetLastError(), "bucket_kernel launch");
  }
  if (T <= 256) {
    hipLaunchKernelGGL(route_kernel<1>, dim3((unsigned)T), dim3(256), 0, stream, X, T, K, Wr, br, prec, perm,
                       offsets, logits, ticket, view);
  } else {
    hipLaunchKernelGGL(route_kernel<4>, dim3((unsigned)((T + 3) / 4)), dim3(256), 0, stream, X, T, K, Wr, br,
                       prec, perm, offsets, logits, ticket, view);
  }
  return hip_status(hipGetLastError(), "route_kernel launch");
}

// Workspace: the ticket counter of the general kernels at byte 0, the per-router words of the
// small-batch kernel from byte 64.
bool route_can_carry_prep(int64_t T) { return T >= 1 && T <= kSmallRouteTokens && knob(4) != 1; }
// one launch for all routers of a call: up to two tokens per lane of the sorting wavefront
static bool route_small_supports(int64_t T) { return T >= 1 && T <= 128 && knob(4) != 1; }
// the one-launch kernel can leave the token sort to the consumer of the precisions (defer_bucket below), which
// sorts up to 128 tokens
bool route_defers_sort(int64_t T) { return route_small_supports(T); }

// prep != nullptr (only when route_can_carry_prep(T)): the launch also prepares the activations
// of the FP4-operand decode kernel, prep_blocks 256-column blocks, into prep.
mbq_status launch_route_group(const uint16_t* X, int64_t T, int64_t K, int n, const float* const* Wr,
                              const float* const* br, int32_t* const* prec, int32_t* const* perm,
                              int32_t* const* offsets, double* const* logits, void* ws, hipStream_t stream,
                              void* prep, int prep_blocks, const ZeroList* zl, bool defer_bucket,
                              const RouteView& view, const uint16_t* Xprep) {
  unsigned int* ticket = reinterpret_cast<unsigned int*>(ws);
  if (T > 0 && !(defer_bucket && route_small_supports(T))) {  // a launch that sorts meets through the counters
    mbq_status st = clear_counters(ws, stream);
    if (st != MBQ_OK) return st;
  }
  if (route_small_supports(T)) {
    if (!route_can_carry_prep(T)) prep = nullptr;
    RouteGroup g;
    g.view = view;
    for (int i = 0; i < kRouteGroupMax; ++i) {
      const int j = i < n ? i : 0;
      g.r[i] = RouteOut{Wr[j], br[j], prec[j], perm[j], offsets[j], logits ? logits[j] : nullptr};
    }
    unsigned long long* words = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(ws) + 64);
    bool clears = false;  // outputs to clear also without a preparation: the extra plane then only clears
    if (zl)
      for (int i = 0; i < kRouteGroupMax; ++i) clears = clears || zl->p[i] != nullptr;
    const bool plane = prep != nullptr || clears;
    const unsigned gx = (prep && prep_blocks > (int)T) ? (unsigned)prep_blocks : (unsigned)T;
    hipLaunchKernelGGL(route_small_kernel, dim3(gx, (unsigned)n + (plane ? 1u : 0u)), dim3(512), 0, stream, X, (int)T,
                       K, g, n, words, reinterpret_cast<char*>(prep), prep ? prep_blocks : 0,
                       (plane && zl) ? *zl : ZeroList{}, defer_bucket ? 1 : 0, Xprep ? Xprep : X);
    return hip_status(hipGetLastError(), "route_small_kernel launch");
  }
  for (int i = 0; i < n; ++i) {
    mbq_status st = launch_route_one(X, T, K, Wr[i], br[i], prec[i], perm[i], offsets[i],
                                     logits ? logits[i] : nullptr, ticket, stream, view);
    if (st != MBQ_OK) return st;
  }
  return MBQ_OK;
}

mbq_status launch_route(const uint16_t* X, int64_t T, int64_t K, const float* Wr, const float* br,
                        int32_t* prec, int32_t* perm, int32_t* offsets, double* logits, void* ws,
                        hipStream_t stream, const RouteView& view) {
  double* const lg[1] = {logits};
  return launch_route_group(X, T, K, 1, &Wr, &br, &prec, &perm, &offsets, logits ? lg : nullptr, ws, stream,
                            nullptr, 0, nullptr, false, view);
}

// ---------------------------------------------------------------------------------------------
// The paper's own router (Sec. 4.2 Eq. 4): a 2-layer MLP scores every slice, S = relu(X W1^T + b1)
// W2^T + b2 (the activation is not given in the paper; ReLU is the reading taken), and the
// run-time threshold of Sec. 4.2 turns scores into slice gates, G = 1[(S - delta) > 0].  The base
// slice is always active (shared-expert slice); a token's precision is the number of leading
// active residual slices, so that it names a prefix of slices like every other path here.
//
// Two launches.  Hidden layer: a workgroup of 256 threads produces eight hidden units of TPW consecutive
// tokens (grid = token groups x hidden chunks, so small batches still fill the chip): the K axis is
// split over the threads in chunks of 8 columns (bf16 x fp32 products are exact in fp64, accumulation
// in fp64), partial sums meet through wavefront shuffles and LDS, bias and ReLU are applied and the
// hidden vector goes to the workspace.  Scores: one thread per (token, slice) forms the score in a
// fixed order, one thread per token decides, and the workgroup that finishes last buckets all tokens
// (same ticket scheme as route_kernel).
constexpr int kMlpHiddenChunk = 8;
constexpr int kMlpMaxHidden = 512;

template <int TPW>
__global__ __launch_bounds__(256) void route_mlp_hidden_kernel(const uint16_t* __restrict__ X, int64_t T, int64_t K,
                                                               const float* __restrict__ W1,
                                                               const float* __restrict__ b1, int H,
                                                               double* __restrict__ hidden) {
  constexpr int HC = kMlpHiddenChunk;
  const int64_t tok0 = (int64_t)blockIdx.x * TPW;
  const int h0 = (int)blockIdx.y * HC;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  __shared__ double s_red[4][TPW][HC];
  double acc[TPW][HC];
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int j = 0; j < HC; ++j) acc[t][j] = 0.0;
  for (int64_t k = (int64_t)tid * 8; k < K; k += 256 * 8) {
    double w[HC][8];
#pragma unroll
    for (int j = 0; j < HC; ++j) {
      const int h = (h0 + j < H) ? h0 + j : H - 1;  // a valid row either way; surplus units are dropped below
      const float4* src = reinterpret_cast<const float4*>(W1 + (int64_t)h * K + k);
      const float4 a = src[0], b = src[1];
      w[j][0] = a.x; w[j][1] = a.y; w[j][2] = a.z; w[j][3] = a.w;
      w[j][4] = b.x; w[j][5] = b.y; w[j][6] = b.z; w[j][7] = b.w;
    }
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
      const int64_t tok = (tok0 + t < T) ? tok0 + t : T - 1;  // a valid row either way
      const uint4 xv = *reinterpret_cast<const uint4*>(X + tok * K + k);
      const double x[8] = {bf16_lo(xv.x), bf16_hi(xv.x), bf16_lo(xv.y), bf16_hi(xv.y),
                           bf16_lo(xv.z), bf16_hi(xv.z), bf16_lo(xv.w), bf16_hi(xv.w)};
#pragma unroll
      for (int j = 0; j < HC; ++j)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[t][j] = fma(x[c], w[j][c], acc[t][j]);
    }
  }
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int j = 0; j < HC; ++j) {
      double v = acc[t][j];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) v += __shfl_down(v, off, 64);
      if (lane == 0) s_red[wave][t][j] = v;
    }
  __syncthreads();
  if (tid < TPW * HC) {
    const int t = tid / HC, j = tid % HC;
    if (h0 + j < H && tok0 + t < T) {
      const double pre = ((s_red[0][t][j] + s_red[1][t][j]) + (s_red[2][t][j] + s_red[3][t][j])) + (double)b1[h0 + j];
      hidden[(tok0 + t) * H + h0 + j] = pre > 0.0 ? pre : 0.0;
    }
  }
}

// Hidden layer of larger batches on the fp64 matrix cores.  A workgroup of four wavefronts owns a tile
// of 16 tokens x 16 hidden units; the K axis is dealt to the wavefronts in blocks of 32 columns.  One
// v_mfma_f64_16x16x4 takes A[token i][k] from lane i + 16 k and B[k][unit j] from lane j + 16 k, so a
// lane reads 8 consecutive columns of its token row and of its unit's weight row (16-byte loads) and
// feeds them to 8 MFMAs, column c of every lane quarter forming the K = 4 of MFMA c.  The result lane
// l, register r is D[token 4 r + l / 16][unit l % 16]; the four partial tiles meet in LDS.
typedef double f64x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void route_mlp_hidden_mfma_kernel(const uint16_t* __restrict__ X, int64_t T,
                                                                    int64_t K, const float* __restrict__ W1,
                                                                    const float* __restrict__ b1, int H,
                                                                    double* __restrict__ hidden) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t tok0 = (int64_t)blockIdx.x * 16;
  const int h0 = (int)blockIdx.y * 16;
  const int64_t tok = (tok0 + (lane & 15) < T) ? tok0 + (lane & 15) : T - 1;  // valid rows either way;
  const int h = (h0 + (lane & 15) < H) ? h0 + (lane & 15) : H - 1;            // surplus results are dropped
  const uint16_t* xrow = X + tok * K;
  const float* wrow = W1 + (int64_t)h * K;
  f64x4 acc = {0.0, 0.0, 0.0, 0.0};
  for (int64_t k = (int64_t)wave * 32 + (lane >> 4) * 8; k < K; k += 4 * 32) {
    const uint4 xv = *reinterpret_cast<const uint4*>(xrow + k);
    const float4 wa = *reinterpret_cast<const float4*>(wrow + k);
    const float4 wb = *reinterpret_cast<const float4*>(wrow + k + 4);
    const double x[8] = {bf16_lo(xv.x), bf16_hi(xv.x), bf16_lo(xv.y), bf16_hi(xv.y),
                         bf16_lo(xv.z), bf16_hi(xv.z), bf16_lo(xv.w), bf16_hi(xv.w)};
    const double w[8] = {wa.x, wa.y, wa.z, wa.w, wb.x, wb.y, wb.z, wb.w};
#pragma unroll
    for (int c = 0; c < 8; ++c) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(x[c], w[c], acc, 0, 0, 0);
  }
  __shared__ double s_part[4][64][4];
#pragma unroll
  for (int r = 0; r < 4; ++r) s_part[wave][lane][r] = acc[r];
  __syncthreads();
  {
    const int l = tid >> 2, r = tid & 3;  // one result of the 16 x 16 tile per thread
    const int64_t t = tok0 + 4 * r + (l >> 4);
    const int hu = h0 + (l & 15);
    if (t < T && hu < H) {
      const double pre = ((s_part[0][l][r] + s_part[1][l][r]) + (s_part[2][l][r] + s_part[3][l][r])) + (double)b1[hu];
      hidden[t * H + hu] = pre > 0.0 ? pre : 0.0;
    }
  }
}

// 64 tokens per workgroup: thread (token, slice) forms the score, then one thread per token decides.
__global__ __launch_bounds__(256) void route_mlp_score_kernel(const double* __restrict__ hidden, int64_t T, int H,
                                                              const float* __restrict__ W2,
                                                              const float* __restrict__ b2, double delta,
                                                              int32_t* prec, int32_t* __restrict__ perm,
                                                              int32_t* __restrict__ offsets,
                                                              double* __restrict__ scores,
                                                              unsigned int* __restrict__ ticket) {
  const int tid = threadIdx.x;
  const int64_t tok = (int64_t)blockIdx.x * 64 + (tid >> 2);
  const int e = tid & 3;
  __shared__ double s_score[64][kP];
  __shared__ unsigned int s_ticket;
  if (tok < T) {
    const double* hrow = hidden + tok * H;
    double s = 0.0;
    for (int j = 0; j < H; ++j) s = fma(hrow[j], (double)W2[(int64_t)e * H + j], s);
    s += (double)b2[e];
    s_score[tid >> 2][e] = s;
    if (scores) scores[tok * kP + e] = s;
  }
  __syncthreads();
  if (tid < 64 && (int64_t)blockIdx.x * 64 + tid < T) {
    int p = 0;
#pragma unroll
    for (int q = 1; q < kP; ++q) {
      if (p == q - 1 && (s_score[tid][q] - delta) > 0.0) p = q;  // strict: a score on the threshold is inactive
    }
    prec[(int64_t)blockIdx.x * 64 + tid] = p;
    __threadfence();  // publish this workgroup's choices before taking a ticket
  }
  __syncthreads();
  if (tid == 0) s_ticket = atomicAdd(ticket, 1u);
  __syncthreads();
  if (s_ticket != gridDim.x - 1) return;
  __threadfence();
  bucket_by_workgroup<4>(prec, T, perm, offsets);
  if (tid == 0) *ticket = 0u;
}

// ws: the ticket counter in the first 256 bytes, then the hidden layer, fp64 [T][H]
size_t route_mlp_workspace_bytes(int64_t T, int H) { return 256 + (size_t)T * (size_t)H * sizeof(double); }

mbq_status launch_route_mlp(const uint16_t* X, int64_t T, int64_t K, const float* W1, const float* b1, int H,
                            const float* W2, const float* b2, double delta, int32_t* prec, int32_t* perm,
                            int32_t* offsets, double* scores, void* ws, hipStream_t stream) {
  unsigned int* ticket = reinterpret_cast<unsigned int*>(ws);
  double* hidden = reinterpret_cast<double*>(reinterpret_cast<char*>(ws) + 256);
  if (T == 0) {
    hipLaunchKernelGGL(bucket_kernel, dim3(1), dim3(64), 0, stream, prec, T, perm, offsets);
    return hip_status(hipGetLastError(), "bucket_kernel launch");
  }
  mbq_status st = clear_counters(ws, stream);
  if (st != MBQ_OK) return st;
  const unsigned chunks = (unsigned)((H + kMlpHiddenChunk - 1) / kMlpHiddenChunk);
  if (T <= 256)
    hipLaunchKernelGGL(route_mlp_hidden_kernel<1>, dim3((unsigned)T, chunks), dim3(256), 0, stream, X, T, K, W1, b1,
                       H, hidden);
  else
    hipLaunchKernelGGL(route_mlp_hidden_mfma_kernel, dim3((unsigned)((T + 15) / 16), (unsigned)((H + 15) / 16)),
                       dim3(256), 0, stream, X, T, K, W1, b1, H, hidden);
  st = hip_status(hipGetLastError(), "route_mlp_hidden_kernel launch");
  if (st != MBQ_OK) return st;
  hipLaunchKernelGGL(route_mlp_score_kernel, dim3((unsigned)((T + 63) / 64)), dim3(256), 0, stream, hidden, T, H, W2,
                     b2, delta, prec, perm, offsets, scores, ticket);
  return hip_status(hipGetLastError(), "route_mlp_score_kernel launch");
}
int route_mlp_max_hidden() { return kMlpMaxHidden; }

// Layer-wise threshold calibration (App. C.2): the (k+1)-th largest of the T (E-1) residual-slice
// scores, found by a most-significant-bit-first radix selection on the order-preserving integer
// image of the doubles; one workgroup, 64 passes over the scores (an offline step).
__device__ inline unsigned long long ordered_key(double v) {
  const unsigned long long u = (unsigned long long)__double_as_longlong(v);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}
__global__ __launch_bounds__(1024) void threshold_quantile_kernel(const double* __restrict__ scores, int64_t T,
                                                                   long long k, double* __restrict__ delta_out) {
  const int64_t M = T * (kP - 1);
  __shared__ unsigned long long s_cnt[16];
  __shared__ unsigned long long s_total;
  if (k >= M) {  // every residual score stays active
    if (threadIdx.x == 0) *delta_out = -__builtin_huge_val();
    return;
  }
  unsigned long long prefix = 0ull, mask = 0ull;
  long long want = k;  // rank (0 = largest) among the scores that match the prefix so far
  for (int bit = 63; bit >= 0; --bit) {
    const unsigned long long cand = prefix | (1ull << bit), cmask = mask | (1ull << bit);
    unsigned long long c = 0;
    for (int64_t i = threadIdx.x; i < M; i += 1024) {
      const double v = scores[(i / (kP - 1)) * kP + 1 + (i % (kP - 1))];
      c += ((ordered_key(v) & cmask) == cand) ? 1ull : 0ull;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) c += __shfl_down(c, off, 64);
    if ((threadIdx.x & 63) == 0) s_cnt[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) {
      unsigned long long tot = 0;
      for (int w = 0; w < 16; ++w) tot += s_cnt[w];
      s_total = tot;
    }
    __syncthreads();
    const unsigned long long ones = s_total;  // scores that match the prefix and have this bit set (the larger ones)
    if ((unsigned long long)want < ones) {
      prefix = cand;
    } else {
      want -= (long long)ones;
    }
    mask = cmask;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const unsigned long long u = (prefix >> 63) ? (prefix & 0x7FFFFFFFFFFFFFFFull) : ~prefix;
    *delta_out = __longlong_as_double((long long)u);
  }
}

mbq_status launch_threshold_quantile(const double* scores, int64_t T, long long k, double* delta_out,
                                     hipStream_t stream) {
  hipLaunchKernelGGL(threshold_quantile_kernel, dim3(1), dim3(1024), 0, stream, scores, T, k, delta_out);
  return hip_status(hipGetLastError(), "threshold_quantile_kernel launch");
}

}  // namespace mbq
