// Prefill-side routed linear: a bf16 MFMA tiled GEMM per precision bucket.
//
// Paper Sec. 4.2 Eq. 6 in the merged-code form of App. B (truncating the merged
// integer code is the coarser quantiser): for a token of precision p,
//   Y[i][n] = sum_g (s0/64) * ( sum_{k in g} x_ik V_nk + (0.5 * 4^(3-p) - 64 z0) * Sx[i][g] )
// with V = I_p * 4^(3-p) the 8-bit code whose unused low digits are zero (an integer
// <= 255, exact in bf16) and Sx the group sums of x.  Tokens arrive sorted by
// precision (Sec. 4.3, token permutation), so a 128-row M tile has one precision and
// reads only slices 0..p.  The integer products are exact in the fp32 MFMA
// accumulator; the group scale is applied to each 128-column partial in fp32.
//
// Workgroup: 256 threads = 2 x 2 wavefronts, tile 128 (tokens) x 128 (outputs),
// K step = one group of 128.  Codes are merged with a rotate + and-or per slice (the
// blob stores slice e rotated so that the four fields of one weight line up as one
// byte), converted with v_cvt_f32_ubyte and written to LDS as bf16.
#include <type_traits>

#include "mbq_common.h"

namespace mbq {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kBN = 128, kBK = 128;

__device__ inline floatx16 mfma32(const uint4& a, const uint4& b, floatx16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                 c, 0, 0, 0);
}

template <int R>
__device__ inline uint32_t rotr_c(uint32_t w) {
  if constexpr (R == 0) return w;
  return __builtin_amdgcn_alignbit(w, w, R);
}

// bf16 pair {byte B0 of m, byte B0+2 of m} as exact small integers.
template <int B0>
__device__ inline uint32_t bf16_pair_from_bytes(uint32_t m) {
  const float lo = (float)((m >> (8 * B0)) & 0xFFu);
  const float hi = (float)((m >> (8 * (B0 + 2))) & 0xFFu);
  return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
}

// Merged bytes of the 16 weights of one dword position, slices 0..p.
// out[r], r = 0..3: byte b holds the code of (step = r & 1, slot 4(b&1) + 2(r>>1) + (b>>1)).
__device__ inline void merge_dword(const uint32_t w[4], int p, uint32_t out[4]) {
  auto part = [&](uint32_t ws, uint32_t mask, uint32_t o[4]) {
    o[0] |= rotr_c<28>(ws) & mask;
    o[1] |= rotr_c<30>(ws) & mask;
    o[2] |= ws & mask;
    o[3] |= rotr_c<2>(ws) & mask;
  };
  out[0] = out[1] = out[2] = out[3] = 0u;
  part(w[0], 0xC0C0C0C0u, out);
  if (p >= 1) part(w[1], 0x30303030u, out);
  if (p >= 2) part(w[2], 0x0C0C0C0Cu, out);
  if (p >= 3) part(w[3], 0x03030303u, out);
}

// Group sums of the activations in sorted-row order: Sx[r][g] = sum_{k in g} X[perm[r]][k].
__global__ __launch_bounds__(256) void prefill_sx_kernel(const uint16_t* __restrict__ X, int64_t T, int64_t K,
                                                         const int32_t* __restrict__ perm,
                                                         float* __restrict__ Sx) {
  const int G = (int)(K / kGroup);
  const int64_t item = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 4;  // (row, group)
  const int sub = threadIdx.x & 15;
  float s = 0.f;
  if (item < T * G) {
    const int64_t r = item / G;
    const int g = (int)(item % G);
    const uint4 v = *reinterpret_cast<const uint4*>(X + (int64_t)perm[r] * K + (int64_t)g * kGroup + 8 * sub);
    const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) s += __uint_as_float(u[j] << 16) + __uint_as_float(u[j] & 0xFFFF0000u);
  }
#pragma unroll
  for (int off = 8; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
  if (item < T * G && sub == 0) Sx[item] = s;
}

// WM = wavefront rows of the workgroup: tile = (64 WM) tokens x 128 outputs, 128 WM threads,
// each wavefront a 64 x 64 sub-tile.  WM = 2: 128-token tiles, two workgroups per compute unit;
// WM = 4: 256-token tiles (the unpacked weight tile feeds twice as many tokens), one workgroup
// of eight wavefronts per compute unit.
//
// The K loop advances in half groups of 64 columns through two LDS buffers: while the matrix
// cores consume half-step h from one buffer, the same wavefronts unpack half-step h+1 into the
// other and the global loads of half-step h+2 are in flight; one barrier per half-step.
constexpr int kHalfK = 64;
constexpr int kHalfStride = kHalfK + 8;  // bf16 per LDS row (144 bytes): conflict-free 128-bit row reads

template <int WM>
__global__ __launch_bounds__(WM * 128, WM == 2 ? 2 : 1) void prefill_kernel(
    const uint16_t* __restrict__ X, int64_t T, int64_t K, const uint32_t* __restrict__ codes, size_t slice_words,
    const float2* __restrict__ meta, int64_t N, int KB, const int32_t* __restrict__ perm,
    const int32_t* __restrict__ offsets, const float* __restrict__ Sx, float* __restrict__ Y) {
  constexpr int BM = 64 * WM;
  constexpr int THREADS = 128 * WM;
  constexpr int A_ITERS = BM * 8 / THREADS;  // 128-bit loads of a half-step of the A tile per thread (= 4)
  constexpr int B_ITERS = 512 / THREADS;     // (code tile, lane) dwords of a half-step of the B tile per thread
  // ---- which (precision bucket, BM-row tile) is this workgroup's ----
  int ty = blockIdx.y, p = -1, row0 = 0, rows = 0;
  {
    int lo = offsets[0];
#pragma unroll
    for (int q = 0; q < MBQ_N_PRECISIONS; ++q) {
      const int hi = offsets[q + 1];
      const int tiles = (hi - lo + BM - 1) / BM;
      if (p < 0) {
        if (ty < tiles) {
          p = q;
          row0 = lo + ty * BM;
          rows = min(BM, hi - row0);
        } else {
          ty -= tiles;
        }
      }
      lo = hi;
    }
  }
  if (p < 0) return;
  const int G = (int)(K / kGroup);
  const int H = 2 * G;  // half-steps
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const bool wave_has_rows = 64 * wm < rows;       // a wavefront whose 64 rows are all padding skips the MFMAs
  const int ntile0 = blockIdx.x * (kBN / kTileN);  // first 16-row code tile of this workgroup
  const int NT = (int)((N + kTileN - 1) / kTileN);

  __shared__ __attribute__((aligned(16))) uint16_t sA[2][BM][kHalfStride];
  __shared__ __attribute__((aligned(16))) uint16_t sB[2][kBN][kHalfStride];
  __shared__ __attribute__((aligned(16))) float sSx[2][BM];

  // ---- global -> register staging of one half-step ----
  // A: thread loads rows (tid/8) + (THREADS/8) i, columns 8 (tid%8) .. +7 of the 64-column half
  const int a_col = 8 * (tid & 7);
  uint32_t a_src[A_ITERS];  // row offsets in units of 8 bf16 (16 bytes); ~0u marks a padding row
  const uint32_t k8 = (uint32_t)(K >> 3);
#pragma unroll
  for (int i = 0; i < A_ITERS; ++i) {
    const int r = (tid >> 3) + (THREADS / 8) * i;
    a_src[i] = (r < rows) ? ((uint32_t)perm[row0 + r] * k8 + (uint32_t)(tid & 7)) : ~0u;
  }
  const uint4* X4 = reinterpret_cast<const uint4*>(X);
  uint4 a_reg[A_ITERS];
  uint32_t b_reg[B_ITERS][4];
  float sx_reg = 0.f;
  auto load_half = [&](int h) {
    const int g = h >> 1, dd = h & 1;
#pragma unroll
    for (int i = 0; i < A_ITERS; ++i)
      a_reg[i] = (a_src[i] != ~0u) ? X4[(size_t)a_src[i] + (size_t)h * (kHalfK / 8)] : uint4{0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < B_ITERS; ++i) {
      const int nt = ntile0 + wave + 2 * WM * i;
      const size_t v = (((size_t)nt * KB + (g >> 1)) * 64 + lane) * 4 + 2 * (g & 1) + dd;
#pragma unroll
      for (int e = 0; e < 4; ++e) b_reg[i][e] = (nt < NT && e <= p) ? codes[e * slice_words + v] : 0u;
    }
    if (dd == 0 && tid < BM) sx_reg = (tid < rows) ? Sx[(int64_t)(row0 + tid) * G + g] : 0.f;
  };
  // registers -> LDS buffer h & 1 (A as is, B merged and converted to exact bf16 integers)
  auto store_half = [&](int h) {
    const int buf = h & 1;
#pragma unroll
    for (int i = 0; i < A_ITERS; ++i)
      *reinterpret_cast<uint4*>(&sA[buf][(tid >> 3) + (THREADS / 8) * i][a_col]) = a_reg[i];
#pragma unroll
    for (int i = 0; i < B_ITERS; ++i) {
      const int nl = 16 * (wave + 2 * WM * i) + (lane & 15);
      const int kq = lane >> 4;
      uint32_t mg[4];
      merge_dword(b_reg[i], p, mg);
#pragma unroll
      for (int step = 0; step < 2; ++step) {
        uint4 v;
        v.x = bf16_pair_from_bytes<0>(mg[step]);
        v.y = bf16_pair_from_bytes<0>(mg[step + 2]);
        v.z = bf16_pair_from_bytes<1>(mg[step]);
        v.w = bf16_pair_from_bytes<1>(mg[step + 2]);
        *reinterpret_cast<uint4*>(&sB[buf][nl][32 * step + 8 * kq]) = v;
      }
    }
    if ((h & 1) == 0 && tid < BM) sSx[(h >> 1) & 1][tid] = sx_reg;
  };

  floatx16 acc[2][2], part[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
  const float half_step = 0.5f * (float)(1 << (2 * (3 - p)));

  // one half-step: stage h+1, fetch h+2, multiply h; the first half of a group starts fresh
  // partial accumulators (zero C operand), the second half ends with the group epilogue
  auto half = [&](int h, auto first_tag, auto rows_tag) {
    constexpr bool kFirst = decltype(first_tag)::value;
    constexpr bool kHasRows = decltype(rows_tag)::value;
    if (h + 1 < H) store_half(h + 1);
    if (h + 2 < H) load_half(h + 2);
    if (kHasRows) {
      const int buf = h & 1;
#pragma unroll
      for (int kk = 0; kk < kHalfK / 16; ++kk) {
        uint4 af[2], bf[2];
#pragma unroll
        for (int a = 0; a < 2; ++a)
          af[a] = *reinterpret_cast<const uint4*>(&sA[buf][64 * wm + 32 * a + (lane & 31)][16 * kk + 8 * (lane >> 5)]);
#pragma unroll
        for (int b = 0; b < 2; ++b)
          bf[b] = *reinterpret_cast<const uint4*>(&sB[buf][64 * wn + 32 * b + (lane & 31)][16 * kk + 8 * (lane >> 5)]);
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int b = 0; b < 2; ++b) {
            if (kFirst && kk == 0) {
              floatx16 z;
#pragma unroll
              for (int i = 0; i < 16; ++i) z[i] = 0.f;
              part[a][b] = mfma32(af[a], bf[b], z);
            } else {
              part[a][b] = mfma32(af[a], bf[b], part[a][b]);
            }
          }
      }
      if (!kFirst) {
        // group finished: scale and zero point in fp32
        const int g = h >> 1;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const int64_t n = (int64_t)blockIdx.x * kBN + 64 * wn + 32 * b + (lane & 31);
          float s3 = 0.f, c = 0.f;
          if (n < (int64_t)NT * kTileN) {
            const float2 mt = meta[((size_t)(n >> 4) * (2 * KB) + g) * kTileN + (n & 15)];
            s3 = mt.x * (1.f / 64.f);
            c = half_step - 64.f * mt.y;
          }
#pragma unroll
          for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int r = 64 * wm + 32 * a + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
              acc[a][b][i] += s3 * (part[a][b][i] + c * sSx[g & 1][r]);
            }
        }
      }
    }
    __syncthreads();
  };

  load_half(0);
  store_half(0);
  load_half(1);
  __syncthreads();
  // the row test is hoisted out of the K loop: a wavefront of padding rows only stages data
  if (wave_has_rows) {
    for (int g = 0; g < G; ++g) {
      half(2 * g, std::true_type{}, std::true_type{});
      half(2 * g + 1, std::false_type{}, std::true_type{});
    }
  } else {
    for (int g = 0; g < G; ++g) {
      half(2 * g, std::true_type{}, std::false_type{});
      half(2 * g + 1, std::false_type{}, std::false_type{});
    }
  }

  // ---- write the tile in original token order ----
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int r = 64 * wm + 32 * a + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
      if (r < rows) {
        const int64_t tok = perm[row0 + r];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const int64_t n = (int64_t)blockIdx.x * kBN + 64 * wn + 32 * b + (lane & 31);
          if (n < N) Y[tok * N + n] = acc[a][b][i];
        }
      }
    }
}

size_t prefill_workspace_bytes(int64_t T, const Shape& sh) { return (size_t)T * sh.G * sizeof(float); }

mbq_status launch_linear_prefill(const uint16_t* X, int64_t T, const void* blob, const Shape& sh,
                                 const int32_t* perm, const int32_t* offsets, float* Y, void* ws,
                                 hipStream_t stream) {
  const uint32_t* codes = reinterpret_cast<const uint32_t*>(blob);
  const float2* meta = reinterpret_cast<const float2*>(reinterpret_cast<const char*>(blob) + sh.meta_offset);
  float* Sx = reinterpret_cast<float*>(ws);
  const int64_t items = T * sh.G * 16;
  hipLaunchKernelGGL(prefill_sx_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, stream, X, T, sh.K,
                     perm, Sx);
  mbq_status st = hip_status(hipGetLastError(), "prefill_sx_kernel launch");
  if (st != MBQ_OK) return st;
  // 256-token tiles halve the unpack work per token once buckets are large enough to fill them
  int wm = knob(5);
  if (wm != 2 && wm != 4) wm = (T >= 1024) ? 4 : 2;
  const int bm = 64 * wm;
  dim3 grid((unsigned)((sh.N + kBN - 1) / kBN), (unsigned)(T / bm + MBQ_N_PRECISIONS));
  if (wm == 4)
    hipLaunchKernelGGL(prefill_kernel<4>, grid, dim3(512), 0, stream, X, T, sh.K, codes, sh.slice_words, meta,
                       sh.N, sh.KB, perm, offsets, Sx, Y);
  else
    hipLaunchKernelGGL(prefill_kernel<2>, grid, dim3(256), 0, stream, X, T, sh.K, codes, sh.slice_words, meta,
                       sh.N, sh.KB, perm, offsets, Sx, Y);
  return hip_status(hipGetLastError(), "prefill_kernel launch");
}

}  // namespace mbq
