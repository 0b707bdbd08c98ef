// Decode-side routed linear (T <= 64): a bandwidth-bound skinny GEMM.
//
// Paper Sec. 4.2 Eq. 6 evaluated slice by slice, Y_i = sum_{e <= p_i} W_e^T X_i, with
// the shared-scale structure of App. B (s_e = s0 / 4^e, z_e = 2 for e >= 1) so that
// only slices 0..max_i p_i are fetched (Sec. 4.3, on-demand slice access).
//
// One wavefront owns a 16-row code tile over a range of 256-column blocks.  A lane
// fetches each slice of a tile with ONE 128-bit load (64 two-bit codes) and turns a
// dword into MFMA B operands with a rotate and an and-or per pair of codes: the
// 2-bit field is OR-ed into the mantissa of the bf16 constant 128.0, giving exactly
// 128 + c (or 128 + 4c, 128 + 16c one field higher).  Tokens are the 16 rows of the
// v_mfma_f32_16x16x32_bf16 A operand, loaded straight from X (8 consecutive bf16 per
// lane); products are exact in fp32.  The 128 offset, the field weights, the slice
// scales 4^-e, the zero points and the per-row slice mask are all applied once per
// group of 128 columns on the 16x16 accumulators, using the group sums of X that
// two extra MFMAs against an all-ones operand deliver in accumulator layout:
//   sum_k x c_e = (Da_e - 128 Sa)/wa_e + (Db_e - 128 Sb)/wb_e
// (a/b = the two field positions of a dword, Sa/Sb = sums of x over their columns).
#include <type_traits>

#include "mbq_common.h"

namespace mbq {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ inline floatx4 mfma16(const uint4& a, const uint4& b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                 c, 0, 0, 0);
}

template <int R>
__device__ inline uint32_t rotr(uint32_t w) {
  if constexpr (R == 0) return w;
  return __builtin_amdgcn_alignbit(w, w, R);
}

constexpr uint32_t kBias = 0x43004300u;  // two bf16 128.0: a 2-bit field OR-ed at mantissa bit m adds c * 2^m

// B operands of the two MFMA k-steps held by one dword of slice E.
// Unrotated field of (step, slot s = 2j + h) is at bit 16h + 4j + 2*step; slice E is
// stored rotated left by 2 - 2E.  Slice 0 keeps its fields one position up (weights
// 4 and 16) so that it needs no extra rotation; the others use weights 1 and 4.
template <int E>
__device__ inline void unpack_dword(uint32_t w, uint4& Ba, uint4& Bb) {
  constexpr int rho = (2 - 2 * E) & 31;
  constexpr int a0 = (E == 0) ? 2 : 0;
  constexpr uint32_t ma = 0x00030003u << a0;
  constexpr uint32_t mb = 0x000C000Cu << a0;
  const uint32_t t0 = rotr<(0 + rho - a0) & 31>(w);
  const uint32_t t1 = rotr<(4 + rho - a0) & 31>(w);
  const uint32_t t2 = rotr<(8 + rho - a0) & 31>(w);
  const uint32_t t3 = rotr<(12 + rho - a0) & 31>(w);
  Ba.x = (t0 & ma) | kBias; Bb.x = (t0 & mb) | kBias;
  Ba.y = (t1 & ma) | kBias; Bb.y = (t1 & mb) | kBias;
  Ba.z = (t2 & ma) | kBias; Bb.z = (t2 & mb) | kBias;
  Ba.w = (t3 & ma) | kBias; Bb.w = (t3 & mb) | kBias;
}

__device__ inline uint32_t dword_of(const uint4& v, int d) {
  return d == 0 ? v.x : d == 1 ? v.y : d == 2 ? v.z : v.w;
}

template <int WAVES, int MT>
__global__ __launch_bounds__(WAVES * 64) void decode_kernel(
    const uint16_t* __restrict__ X, int T, int64_t K, const uint4* __restrict__ codes, size_t slice_vec,
    const float2* __restrict__ meta, int64_t N, int KB, const int32_t* __restrict__ perm,
    const int32_t* __restrict__ offsets, float* __restrict__ Y, float* __restrict__ partial, int kb_per_split,
    int64_t Npad) {
  const int nt = blockIdx.x;
  const int split = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int m = lane & 15;   // token row of the A operand / weight row of the B operand / output column
  const int kq = lane >> 4;  // quarter of the 32-wide k-step held by this lane; output rows 4kq..4kq+3

  const int o1 = offsets[1], o2 = offsets[2], o3 = offsets[3];
  const int pmax = (T > o3) ? 3 : (T > o2) ? 2 : (T > o1) ? 1 : 0;

  // per output row: slice weights ca_e = [e <= p] 4^-e / wa_e and the coefficient of
  // the group sums; wb_e = 4 wa_e for every slice.
  float ca[MT][4][4], alpha_a[MT][4], alpha_b[MT][4];
  int tile_pmax[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    const int last = min(16 * t + 15, T - 1);
    tile_pmax[t] = (16 * t < T) ? ((last >= o1) + (last >= o2) + (last >= o3)) : -1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = 16 * t + 4 * kq + i;
      const bool valid = r < T;
      const int p = (r >= o1) + (r >= o2) + (r >= o3);
      float CA = 0.f, Q = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float inv4e = 1.f / (float)(1 << (2 * e));
        const float wa = (e == 0) ? 4.f : 1.f;
        const bool on = valid && (e <= p);
        ca[t][i][e] = on ? inv4e / wa : 0.f;
        CA += ca[t][i][e];
        Q += on ? inv4e : 0.f;
      }
      alpha_a[t][i] = valid ? (128.f * CA + 1.5f * (Q - 1.f) - 0.5f) : 0.f;
      alpha_b[t][i] = valid ? (32.f * CA + 1.5f * (Q - 1.f) - 0.5f) : 0.f;
    }
  }

  const uint16_t* xrow[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    const int r = 16 * t + m;
    xrow[t] = (r < T) ? (X + (int64_t)perm[r] * K) : nullptr;
  }

  floatx4 acc[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
  const uint4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};

  const int kb_begin = split * kb_per_split;
  const int kb_end = min(KB, kb_begin + kb_per_split);
  for (int kb = kb_begin + wave; kb < kb_end; kb += WAVES) {
    const size_t tile = ((size_t)nt * KB + kb) * 64 + lane;
    uint4 w[4];
    w[0] = codes[tile];
    if (pmax >= 1) w[1] = codes[slice_vec + tile];
    if (pmax >= 2) w[2] = codes[2 * slice_vec + tile];
    if (pmax >= 3) w[3] = codes[3 * slice_vec + tile];
    float2 mt[2];
    mt[0] = meta[((size_t)nt * (2 * KB) + 2 * kb) * kTileN + m];
    mt[1] = meta[((size_t)nt * (2 * KB) + 2 * kb + 1) * kTileN + m];

#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint4 A[MT][4];
#pragma unroll
      for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int64_t k = (int64_t)kb * kTileK + 128 * h + 32 * j + 8 * kq;
          A[t][j] = (xrow[t] != nullptr && k < K) ? *reinterpret_cast<const uint4*>(xrow[t] + k)
                                                  : uint4{0u, 0u, 0u, 0u};
        }
      floatx4 Sa[MT], Sb[MT], V[MT];
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        V[t] = zero4;
        if (tile_pmax[t] >= 0) {
          Sa[t] = mfma16(A[t][0], ones, zero4);
          Sa[t] = mfma16(A[t][2], ones, Sa[t]);
          Sb[t] = mfma16(A[t][1], ones, zero4);
          Sb[t] = mfma16(A[t][3], ones, Sb[t]);
        } else {
          Sa[t] = zero4;
          Sb[t] = zero4;
        }
      }
      auto slice = [&](auto etag) {
        constexpr int E = decltype(etag)::value;
        uint4 Ba0, Bb0, Ba1, Bb1;
        unpack_dword<E>(dword_of(w[E], 2 * h), Ba0, Bb0);
        unpack_dword<E>(dword_of(w[E], 2 * h + 1), Ba1, Bb1);
#pragma unroll
        for (int t = 0; t < MT; ++t) {
          if (tile_pmax[t] >= E) {
            floatx4 Da = mfma16(A[t][0], Ba0, zero4);
            Da = mfma16(A[t][2], Ba1, Da);
            floatx4 Db = mfma16(A[t][1], Bb0, zero4);
            Db = mfma16(A[t][3], Bb1, Db);
#pragma unroll
            for (int i = 0; i < 4; ++i) V[t][i] += ca[t][i][E] * (Da[i] + 0.25f * Db[i]);
          }
        }
      };
      slice(std::integral_constant<int, 0>{});
      if (pmax >= 1) slice(std::integral_constant<int, 1>{});
      if (pmax >= 2) slice(std::integral_constant<int, 2>{});
      if (pmax >= 3) slice(std::integral_constant<int, 3>{});
      const float s0 = mt[h].x, s0z0 = mt[h].x * mt[h].y;
#pragma unroll
      for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float v = V[t][i] - alpha_a[t][i] * Sa[t][i] - alpha_b[t][i] * Sb[t][i];
          acc[t][i] += s0 * v - s0z0 * (Sa[t][i] + Sb[t][i]);
        }
    }
  }

  // sum the wavefronts' partial tiles through LDS, then write rows in token order
  __shared__ float red[WAVES][MT][64][4];
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) red[wave][t][lane][i] = acc[t][i];
  __syncthreads();
  for (int o = threadIdx.x; o < MT * 256; o += WAVES * 64) {
    const int t = o >> 8, r = (o >> 4) & 15, c = o & 15;
    const int row = 16 * t + r;
    const int64_t n = (int64_t)nt * kTileN + c;
    if (row >= T) continue;
    float sum = 0.f;
#pragma unroll
    for (int wv = 0; wv < WAVES; ++wv) sum += red[wv][t][16 * (r >> 2) + c][r & 3];
    if (gridDim.y == 1) {
      if (n < N) Y[(int64_t)perm[row] * N + n] = sum;
    } else {
      partial[((size_t)split * (MT * 16) + row) * Npad + n] = sum;
    }
  }
}

__global__ __launch_bounds__(256) void decode_reduce_kernel(const float* __restrict__ partial, int splits,
                                                            int rows_pad, int T, int64_t N, int64_t Npad,
                                                            const int32_t* __restrict__ perm,
                                                            float* __restrict__ Y) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)T * N) return;
  const int row = (int)(idx / N);
  const int64_t n = idx % N;
  float sum = 0.f;
  for (int s = 0; s < splits; ++s) sum += partial[((size_t)s * rows_pad + row) * Npad + n];
  Y[(int64_t)perm[row] * N + n] = sum;
}

size_t decode_workspace_bytes(int64_t T, const Shape& sh) {
  if (T > kMaxDecodeTokens) return 0;
  const int64_t rows = ((T + 15) / 16) * 16;
  return (size_t)kMaxKSplit * rows * ((size_t)sh.NT * kTileN) * sizeof(float);
}

template <int WAVES, int MT>
static void launch_one(dim3 grid, hipStream_t stream, const uint16_t* X, int T, const Shape& sh,
                       const uint4* codes, const float2* meta, const int32_t* perm, const int32_t* offsets,
                       float* Y, float* partial, int kb_per_split) {
  hipLaunchKernelGGL((decode_kernel<WAVES, MT>), grid, dim3(WAVES * 64), 0, stream, X, T, sh.K, codes,
                     sh.slice_words / 4, meta, sh.N, sh.KB, perm, offsets, Y, partial, kb_per_split,
                     (int64_t)sh.NT * kTileN);
}

mbq_status launch_linear_decode(const uint16_t* X, int64_t T, const void* blob, const Shape& sh,
                                const int32_t* perm, const int32_t* offsets, float* Y, void* ws,
                                hipStream_t stream) {
  const uint4* codes = reinterpret_cast<const uint4*>(blob);
  const float2* meta = reinterpret_cast<const float2*>(reinterpret_cast<const char*>(blob) + sh.meta_offset);
  const int mt = (int)((T + 15) / 16);

  // launch shape: WAVES wavefronts share one row tile and split its column blocks;
  // when the matrix has few row tiles, several workgroups split K further (their
  // partial tiles are summed by a second kernel).  Register budget: 16 wavefronts
  // only with one token tile, 8 with two, 4 beyond.
  const int max_waves = (mt == 1) ? 16 : (mt == 2 ? 8 : 4);
  int ksplit = knob(1);
  if (ksplit <= 0) {
    ksplit = 1;
    while (ksplit < kMaxKSplit && (int64_t)sh.NT * ksplit < 256 && sh.KB / (ksplit * 2) >= 4) ksplit *= 2;
  }
  if (ksplit > kMaxKSplit) ksplit = kMaxKSplit;
  if (ksplit > sh.KB) ksplit = sh.KB;
  const int kb_per_split = (sh.KB + ksplit - 1) / ksplit;
  ksplit = (sh.KB + kb_per_split - 1) / kb_per_split;
  int waves = knob(0);
  if (waves != 4 && waves != 8 && waves != 16) waves = (kb_per_split >= 16) ? 16 : (kb_per_split >= 8 ? 8 : 4);
  if (waves > max_waves) waves = max_waves;
  dim3 grid(sh.NT, ksplit);
  float* partial = reinterpret_cast<float*>(ws);

#define MBQ_DECODE_CASE(WV, MTV)                                                                            \
  if (waves == WV && mt == MTV)                                                                             \
    launch_one<WV, MTV>(grid, stream, X, (int)T, sh, codes, meta, perm, offsets, Y, partial, kb_per_split); \
  else
  MBQ_DECODE_CASE(4, 1) MBQ_DECODE_CASE(8, 1) MBQ_DECODE_CASE(16, 1)
  MBQ_DECODE_CASE(4, 2) MBQ_DECODE_CASE(8, 2)
  MBQ_DECODE_CASE(4, 3) MBQ_DECODE_CASE(4, 4) {
    set_error("decode kernel: no instantiation for %d wavefronts x %d token tiles", waves, mt);
    return MBQ_ERR_INVALID_ARG;
  }
#undef MBQ_DECODE_CASE
  mbq_status st = hip_status(hipGetLastError(), "decode_kernel launch");
  if (st != MBQ_OK) return st;
  if (ksplit > 1) {
    const int64_t total = T * sh.N;
    hipLaunchKernelGGL(decode_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       partial, ksplit, mt * 16, (int)T, sh.N, (int64_t)sh.NT * kTileN, perm, Y);
    st = hip_status(hipGetLastError(), "decode_reduce_kernel launch");
  }
  return st;
}

}  // namespace mbq
