// Decode-side routed linear for one token tile (T <= 16): the bandwidth-bound path.
//
// Paper Sec. 4.2 Eq. 6 evaluated slice by slice, Y_i = sum_{e <= p_i} W_e^T X_i, with the
// shared-scale structure of App. B (s_e = s0/4^e, z_e = 2 for e >= 1); only slices
// 0..max_i p_i are fetched (Sec. 4.3, on-demand slice access).
//
// Work split: a workgroup of WAVES wavefronts owns 16-row code tiles nt = blockIdx.x,
// blockIdx.x + gridDim.x, ...; wavefront w owns the 256-column blocks kb = w, w + WAVES, ...
// When the row fits (KB <= WAVES) the wavefront's activation fragments and their group
// sums stay in registers for the whole kernel and only packed weights stream from HBM,
// the next tile's loads being issued before the current tile is consumed.
//
// Per tile and slice a lane issues ONE 128-bit load (64 two-bit codes).  A dword becomes
// MFMA B operands with a rotate and an and-or per pair of codes: the 2-bit field is OR-ed
// into the mantissa of a bf16 power of two chosen per slice and field position so that the
// operand equals  beta + c / 4^e  exactly (e.g. 32 + c/4).  Tokens are the 16 rows of the
// v_mfma_f32_16x16x32_bf16 A operand, read straight from X in original token order.  All
// slices of a group chain into one accumulator; the accumulator after slice p is kept, so a
// row of precision p simply selects snapshot p.  The known offsets (beta times the group
// sums of x, delivered in accumulator layout by MFMAs against an all-ones operand), the zero
// points and the group scale are applied once per group of 128 columns in fp32.
#include "mbq_common.h"

namespace mbq {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace d16 {

__device__ inline floatx4 mfma(const uint4& a, const uint4& b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                 c, 0, 0, 0);
}

template <int R>
__device__ inline uint32_t rotr(uint32_t w) {
  if constexpr (R == 0) return w;
  return __builtin_amdgcn_alignbit(w, w, R);
}

// bf16 pairs of 2^5, 2^3, 2^1, 2^-1
constexpr uint32_t kPow5 = 0x42004200u, kPow3 = 0x41004100u, kPow1 = 0x40004000u, kPowM1 = 0x3F003F00u;

// B operands (a-step, b-step) of the two k-steps held by one dword of slice E.
// The unrotated field of (step, slot s = 2j + h) sits at bit 16h + 4j + 2 step; slice E is
// stored rotated left by 2 - 2E.  Slice 0 is consumed one field position up (no rotation
// for j = 0); its bias exponents are lowered accordingly.  Operand values:
//   slice 0: 32 + c, 8 + c     slice 1: 32 + c/4, 8 + c/4
//   slice 2: 8 + c/16, 2 + c/16   slice 3: 2 + c/64, 0.5 + c/64
template <int E>
__device__ inline void unpack_dword(uint32_t w, uint4& Ba, uint4& Bb) {
  constexpr int rho = (2 - 2 * E) & 31;
  constexpr int a0 = (E == 0) ? 2 : 0;
  constexpr uint32_t ma = 0x00030003u << a0;
  constexpr uint32_t mb = 0x000C000Cu << a0;
  constexpr uint32_t ba = (E <= 1) ? kPow5 : (E == 2 ? kPow3 : kPow1);
  constexpr uint32_t bb = (E <= 1) ? kPow3 : (E == 2 ? kPow1 : kPowM1);
  const uint32_t t0 = rotr<(0 + rho - a0) & 31>(w);
  const uint32_t t1 = rotr<(4 + rho - a0) & 31>(w);
  const uint32_t t2 = rotr<(8 + rho - a0) & 31>(w);
  const uint32_t t3 = rotr<(12 + rho - a0) & 31>(w);
  Ba.x = (t0 & ma) | ba; Bb.x = (t0 & mb) | bb;
  Ba.y = (t1 & ma) | ba; Bb.y = (t1 & mb) | bb;
  Ba.z = (t2 & ma) | ba; Bb.z = (t2 & mb) | bb;
  Ba.w = (t3 & ma) | ba; Bb.w = (t3 & mb) | bb;
}

// D += X_group * slice-E operands of the two dwords (w_lo, w_hi) of one group.
template <int E>
__device__ inline floatx4 slice_group(const uint4 A[4], uint32_t w_lo, uint32_t w_hi, floatx4 D) {
  uint4 Ba, Bb;
  unpack_dword<E>(w_lo, Ba, Bb);
  D = mfma(A[0], Ba, D);
  D = mfma(A[1], Bb, D);
  unpack_dword<E>(w_hi, Ba, Bb);
  D = mfma(A[2], Ba, D);
  D = mfma(A[3], Bb, D);
  return D;
}

struct Item {
  uint4 w[4];
  float2 mt[2];
};

}  // namespace d16

template <int WAVES, bool STATIONARY>
__global__ __launch_bounds__(WAVES * 64) void decode16_kernel(
    const uint16_t* __restrict__ X, int T, int64_t K, const uint4* __restrict__ codes, size_t slice_vec,
    const float2* __restrict__ meta, int64_t N, int NT, int KB, const int32_t* __restrict__ prec,
    float* __restrict__ Y, int dbg) {
  using namespace d16;
  if (dbg & 16) return;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int m = lane & 15;   // token row of A / weight row of B / output column
  const int kq = lane >> 4;  // k quarter of a k-step; output rows 4 kq .. 4 kq + 3

  // 16 wavefronts that also reload activations per block have no registers left for a second
  // set of weight fragments: they fetch the next block after finishing the current one.
  constexpr bool kPrefetch = STATIONARY || WAVES < 16;
  const int phases = STATIONARY ? 1 : (KB + WAVES - 1) / WAVES;
  const int my_tiles = (NT - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
  const int n_items = my_tiles * phases;

  // ---- loads that depend on nothing: precisions first, then activations, slice 0 ----
  const int pl = (dbg & 8) ? ((lane < T) ? 3 : -1) : (lane < T) ? prec[lane] : -1;
  const uint16_t* xrow = (m < T) ? (X + (int64_t)m * K) : nullptr;
  uint4 xa[8];
  auto load_x = [&](int kb) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int64_t k = (int64_t)kb * kTileK + 32 * j + 8 * kq;
      xa[j] = (xrow != nullptr && k < K && !(dbg & 4)) ? *reinterpret_cast<const uint4*>(xrow + k) : uint4{0u, 0u, 0u, 0u};
    }
  };
  auto tile_of = [&](int it) { return (int)blockIdx.x + (it / phases) * (int)gridDim.x; };
  auto block_of = [&](int it) { return (it % phases) * WAVES + wave; };
  auto load_slice0 = [&](int nt, int kb, Item& I) {
    const size_t tile = ((size_t)nt * KB + kb) * 64 + lane;
    I.w[0] = codes[tile];
    I.mt[0] = meta[((size_t)nt * (2 * KB) + 2 * kb) * kTileN + m];
    I.mt[1] = meta[((size_t)nt * (2 * KB) + 2 * kb + 1) * kTileN + m];
  };
  int pmax = 0;
  auto load_rest = [&](int nt, int kb, Item& I) {
    const size_t tile = ((size_t)nt * KB + kb) * 64 + lane;
    if (pmax >= 1) I.w[1] = codes[slice_vec + tile];
    if (pmax >= 2) I.w[2] = codes[2 * slice_vec + tile];
    if (pmax >= 3) I.w[3] = codes[3 * slice_vec + tile];
  };

  Item cur, nxt;
  if (n_items > 0 && block_of(0) < KB) {
    load_x(block_of(0));
    load_slice0(tile_of(0), block_of(0), cur);
  }

  // ---- routing facts (first dependent step): highest precision present, per-row constants ----
  pmax = (__ballot(pl == 3) != 0ull) ? 3 : (__ballot(pl == 2) != 0ull) ? 2 : (__ballot(pl == 1) != 0ull) ? 1 : 0;
  if (n_items > 0 && block_of(0) < KB) load_rest(tile_of(0), block_of(0), cur);

  int prow[4];
  float coefA[4], coefB[4], coefS[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int p = __shfl(pl, 4 * kq + i, 64);
    prow[i] = p;
    // offsets accumulated by snapshot p: sum of the operand biases of slices 0..p
    coefA[i] = (p >= 3) ? 74.f : (p == 2) ? 72.f : (p == 1) ? 64.f : 32.f;
    coefB[i] = (p >= 3) ? 18.5f : (p == 2) ? 18.f : (p == 1) ? 16.f : 8.f;
    // residual zero points: sum_{1 <= e <= p} 4^-e (2 - 0.5), and the base slice's -0.5
    const float q = (p >= 3) ? 0.328125f : (p == 2) ? 0.3125f : (p == 1) ? 0.25f : 0.f;
    coefS[i] = 1.5f * q - 0.5f;
  }

  const uint4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};
  floatx4 C1[2], SS[2];  // per group of the current k-block: offset term and sum of x, per output row
  auto group_sums = [&]() {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      floatx4 Sa = mfma(xa[4 * h + 0], ones, zero4);
      Sa = mfma(xa[4 * h + 2], ones, Sa);
      floatx4 Sb = mfma(xa[4 * h + 1], ones, zero4);
      Sb = mfma(xa[4 * h + 3], ones, Sb);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        SS[h][i] = Sa[i] + Sb[i];
        C1[h][i] = coefA[i] * Sa[i] + coefB[i] * Sb[i] + coefS[i] * SS[h][i];
      }
    }
  };
  if (STATIONARY && n_items > 0 && block_of(0) < KB) group_sums();

  __shared__ float red[2][WAVES][64][4];
  floatx4 acc = zero4;
  for (int it = 0; it < n_items; ++it) {
    const int nt = tile_of(it), kb = block_of(it);
    const bool active = kb < KB;
    const bool has_next = it + 1 < n_items;
    const bool next_active = has_next && block_of(it + 1) < KB;
    if (kPrefetch && next_active) {
      load_slice0(tile_of(it + 1), block_of(it + 1), nxt);
      load_rest(tile_of(it + 1), block_of(it + 1), nxt);
    }
    if (active && (dbg & 1)) {
      acc[0] += __uint_as_float((cur.w[0].x ^ cur.w[1].y ^ cur.w[2].z ^ cur.w[3].w) & 0x3FFFFFu) + cur.mt[0].x + cur.mt[1].y;
    } else if (active) {
      if (!STATIONARY) {
        if (it > 0) load_x(kb);
        group_sums();
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const uint4* A = &xa[4 * h];
        const uint32_t l0 = h ? cur.w[0].z : cur.w[0].x, h0 = h ? cur.w[0].w : cur.w[0].y;
        // all slices chain into one accumulator; a row keeps the value after its last slice
        floatx4 D = slice_group<0>(A, l0, h0, zero4);
        floatx4 v = D;
        if (pmax >= 1) {
          D = slice_group<1>(A, h ? cur.w[1].z : cur.w[1].x, h ? cur.w[1].w : cur.w[1].y, D);
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = (prow[i] >= 1) ? D[i] : v[i];
        }
        if (pmax >= 2) {
          D = slice_group<2>(A, h ? cur.w[2].z : cur.w[2].x, h ? cur.w[2].w : cur.w[2].y, D);
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = (prow[i] >= 2) ? D[i] : v[i];
        }
        if (pmax >= 3) {
          D = slice_group<3>(A, h ? cur.w[3].z : cur.w[3].x, h ? cur.w[3].w : cur.w[3].y, D);
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = (prow[i] >= 3) ? D[i] : v[i];
        }
        const float s0 = cur.mt[h].x, s0z0 = cur.mt[h].x * cur.mt[h].y;
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] += s0 * (v[i] - C1[h][i]) - s0z0 * SS[h][i];
      }
    }
    if ((it % phases) == phases - 1 && (!(dbg & 2) || it == n_items - 1)) {
      // all column blocks of tile nt are done: sum the wavefronts, store rows in token order
      const int buf = (it / phases) & 1;
#pragma unroll
      for (int i = 0; i < 4; ++i) red[buf][wave][lane][i] = acc[i];
      acc = zero4;
      __syncthreads();
      if (threadIdx.x < 256) {
        const int r = threadIdx.x >> 4, c = threadIdx.x & 15;
        const int64_t n = (int64_t)nt * kTileN + c;
        if (r < T && n < N) {
          float sum = 0.f;
#pragma unroll
          for (int wv = 0; wv < WAVES; ++wv) sum += red[buf][wv][16 * (r >> 2) + c][r & 3];
          Y[(int64_t)r * N + n] = sum;
        }
      }
    }
    if (next_active) {
      if (kPrefetch) {
        cur = nxt;
      } else {
        load_slice0(tile_of(it + 1), block_of(it + 1), cur);
        load_rest(tile_of(it + 1), block_of(it + 1), cur);
      }
    }
  }
}

template <int WAVES, bool STATIONARY>
static void launch_decode16(int grid, hipStream_t stream, const uint16_t* X, int T, const Shape& sh,
                            const uint4* codes, const float2* meta, const int32_t* prec, float* Y) {
  hipLaunchKernelGGL((decode16_kernel<WAVES, STATIONARY>), dim3(grid), dim3(WAVES * 64), 0, stream, X, T, sh.K,
                     codes, sh.slice_words / 4, meta, sh.N, sh.NT, sh.KB, prec, Y, knob(4));
}

static int compute_units() {
  static int cached = 0;
  if (cached == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cached = n;
    else
      cached = 256;
  }
  return cached;
}

mbq_status launch_linear_decode16(const uint16_t* X, int64_t T, const void* blob, const Shape& sh,
                                  const int32_t* prec, float* Y, hipStream_t stream) {
  const uint4* codes = reinterpret_cast<const uint4*>(blob);
  const float2* meta = reinterpret_cast<const float2*>(reinterpret_cast<const char*>(blob) + sh.meta_offset);
  int waves = knob(0);
  if (waves != 4 && waves != 8 && waves != 16) waves = (sh.KB <= 4) ? 4 : (sh.KB <= 8 ? 8 : 16);
  const bool stationary = sh.KB <= waves;
  int per_cu = knob(2);
  if (per_cu <= 0) per_cu = 16 / waves;  // 16 wavefronts per compute unit
  int grid = compute_units() * per_cu;
  if (grid > sh.NT) grid = sh.NT;
#define MBQ_D16(WV)                                                                        \
  if (waves == WV) {                                                                       \
    if (stationary) launch_decode16<WV, true>(grid, stream, X, (int)T, sh, codes, meta, prec, Y);  \
    else launch_decode16<WV, false>(grid, stream, X, (int)T, sh, codes, meta, prec, Y);    \
  }
  MBQ_D16(4) MBQ_D16(8) MBQ_D16(16)
#undef MBQ_D16
  return hip_status(hipGetLastError(), "decode16_kernel launch");
}

}  // namespace mbq
