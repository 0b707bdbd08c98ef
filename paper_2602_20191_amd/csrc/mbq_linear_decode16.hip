// Decode-side routed linear for one token tile (T <= 16): the bandwidth-bound path.
//
// Paper Sec. 4.2 Eq. 6 evaluated slice by slice, Y_i = sum_{e <= p_i} W_e^T X_i, with the
// shared-scale structure of App. B (s_e = s0/4^e, z_e = 2 for e >= 1); only slices
// 0..max_i p_i are fetched (Sec. 4.3, on-demand slice access).
//
// Work split: a workgroup of WAVES wavefronts owns the 16-row code tiles nt = blockIdx.x,
// blockIdx.x + gridDim.x, ...  The K axis is cut into chunks of WAVES 256-column blocks;
// inside a chunk wavefront w owns block chunk*WAVES + w, keeps its activation fragments in
// registers (and their group sums in LDS) and streams only packed weights from HBM while it
// walks over the workgroup's tiles, always fetching the next tile before consuming the
// current one.  Partial tiles of different chunks are summed in LDS.
//
// Per tile and slice a lane issues ONE 128-bit load (64 two-bit codes).  A dword becomes
// MFMA B operands with a rotate and an and-or per pair of codes: the 2-bit field is OR-ed
// into the mantissa of a bf16 power of two chosen per slice and field position so that the
// operand equals  beta + c / 4^e  exactly (e.g. 32 + c/4).  Tokens are the 16 rows of the
// v_mfma_f32_16x16x32_bf16 A operand, read straight from X in original token order.  All
// slices of a group chain into one accumulator; a row of precision p keeps the value the
// accumulator had after slice p.  The known offsets (beta times the group sums of x, which
// MFMAs against an all-ones operand deliver in accumulator layout), the zero points and the
// group scale are applied once per group of 128 columns in fp32.
#include <type_traits>

#include "mbq_common.h"

namespace mbq {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace d16 {

constexpr int kMaxTilesMulti = 32;  // tiles per workgroup whose partial sums fit the LDS budget
constexpr int kStageStride = 272;   // bytes between token rows of the activation staging area (256 + 16: no bank conflicts)
constexpr int kAreaBytes = 16 * kStageStride;  // >= 4 * 64 * 16 bytes of per-block constants

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

// Unpack constants kept in registers.  (t & mask) | bias is one v_and_or_b32 only when neither
// operand is a literal (a VOP3 instruction cannot carry one on gfx9), so the three field masks live
// in scalar registers and the four bf16-pair biases 2^5, 2^3, 2^1, 2^-1 in vector registers; both are
// made opaque to constant folding once, at kernel entry.
struct UnpackConsts {
  uint32_t mask[3];  // 0x00030003 << 0, 2, 4
  uint32_t bias[4];
};

__device__ inline UnpackConsts make_unpack_consts() {
  UnpackConsts c;
  c.mask[0] = 0x00030003u; c.mask[1] = 0x000C000Cu; c.mask[2] = 0x00300030u;
  c.bias[0] = kPow5; c.bias[1] = kPow3; c.bias[2] = kPow1; c.bias[3] = kPowM1;
#pragma unroll
  for (int i = 0; i < 3; ++i) asm volatile("" : "+s"(c.mask[i]));
#pragma unroll
  for (int i = 0; i < 4; ++i) asm volatile("" : "+v"(c.bias[i]));
  return c;
}

// B operands (a-step, b-step) of the two k-steps held by one dword of slice E.
// The unrotated field of (step, slot s = 2j + h) sits at bit 16h + 4j + 2 step; slice E is
// stored rotated left by 2 - 2E.  Slice 0 is consumed one field position up (no rotation
// for j = 0); its bias exponents are lowered accordingly.  Operand values:
//   slice 0: 32 + c, 8 + c          slice 1: 32 + c/4, 8 + c/4
//   slice 2: 8 + c/16, 2 + c/16     slice 3: 2 + c/64, 0.5 + c/64
template <int E>
__device__ inline void unpack_dword(uint32_t w, const UnpackConsts& uc, uint4& Ba, uint4& Bb) {
  constexpr int rho = (2 - 2 * E) & 31;
  constexpr int a0 = (E == 0) ? 2 : 0;
  const uint32_t ma = uc.mask[(E == 0) ? 1 : 0];
  const uint32_t mb = uc.mask[(E == 0) ? 2 : 1];
  const uint32_t ba = uc.bias[(E <= 1) ? 0 : (E == 2 ? 1 : 2)];
  const uint32_t bb = uc.bias[(E <= 1) ? 1 : (E == 2 ? 2 : 3)];
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
__device__ inline floatx4 slice_group(const uint4 A[4], const UnpackConsts& uc, uint32_t w_lo, uint32_t w_hi,
                                       floatx4 D) {
  uint4 Ba, Bb;
  unpack_dword<E>(w_lo, uc, Ba, Bb);
  D = mfma(A[0], Ba, D);
  D = mfma(A[1], Bb, D);
  unpack_dword<E>(w_hi, uc, Ba, Bb);
  D = mfma(A[2], Ba, D);
  D = mfma(A[3], Bb, D);
  return D;
}

struct Item {
  uint4 w[4];
  float2 mt[2];
};

}  // namespace d16

// MULTI: the K axis needs more than one chunk (KB > WAVES); partial tiles go through LDS.
template <int WAVES, bool MULTI>
__global__ __launch_bounds__(WAVES * 64) void decode16_kernel(
    const uint16_t* __restrict__ X, int T, int64_t K, const uint4* __restrict__ codes, size_t slice_vec,
    const float2* __restrict__ meta, int64_t N, int NT, int KB, const int32_t* __restrict__ prec,
    const int32_t* __restrict__ perm, float* __restrict__ Y) {
  using namespace d16;
  // blockIdx.y = token tile: rows 16 y .. 16 y + 15 of the token order (of the precision-sorted
  // order `perm` when there are several tiles, so that a tile reads only the slices it needs)
  const int row0 = 16 * (int)blockIdx.y;
  T = min(16, T - row0);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: keeps tile addresses scalar
  const int m = lane & 15;   // token row of A / weight row of B / output column
  const int kq = lane >> 4;  // k quarter of a k-step; output rows 4 kq .. 4 kq + 3
  const int chunks = MULTI ? (KB + WAVES - 1) / WAVES : 1;
  const int my_tiles = (NT - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;

  __shared__ float red[2][WAVES][64][4];                   // per-wavefront partial tiles, double buffered
  // Private to each wavefront: first the staging rows of its activation block (16 tokens x 128
  // columns, row stride kStageStride bytes), afterwards C1[2], SS[2] of that block.
  __shared__ __attribute__((aligned(16))) char area[WAVES][kAreaBytes];
  __shared__ float part[MULTI ? kMaxTilesMulti : 1][256];  // sums over chunks
  char* const stage = area[wave];
  floatx4* const cst = reinterpret_cast<floatx4*>(area[wave]);  // [4][64]

  // ---- loads that depend on nothing: precisions first, then activations, slice 0 ----
  const int my_token = (lane < T) ? (perm ? perm[row0 + lane] : row0 + lane) : -1;
  const int pl = (lane < T) ? prec[my_token] : -1;
  // Activations: a load instruction covers four token rows, a quarter wavefront reading 256
  // contiguous bytes of each (whole cache lines); the MFMA A layout (token = lane % 16) is then
  // produced by a round trip through the wavefront's LDS rows, one half block at a time (LDS
  // operations of one wavefront execute in order; every access to the area uses one vector type).
  uint4 xa[8];
  auto load_x = [&](int kb) {
    const int64_t k0 = (int64_t)kb * kTileK + 8 * m;  // K is a multiple of 128: a half block is all there or absent
    const uint16_t* col = X + k0;
    const int second = (k0 + 128 < K) ? 128 : 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int tok = __shfl(my_token, 4 * i + kq, 64);
      const uint16_t* src = col + (int64_t)max(tok, 0) * K;  // always a valid address
      xa[i] = *reinterpret_cast<const uint4*>(src);
      xa[4 + i] = *reinterpret_cast<const uint4*>(src + second);
    }
  };
  // Rows past the last token and an absent second half block become zeros on the way through.
  auto transpose_x = [&](int kb) {
    const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
    const bool second = (int64_t)kb * kTileK + 128 < K;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool there = (4 * i + kq < T) && (h == 0 || second);
        *reinterpret_cast<floatx4*>(stage + (4 * i + kq) * kStageStride + 16 * m) =
            there ? __builtin_bit_cast(floatx4, xa[4 * h + i]) : zero;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j)
        xa[4 * h + j] = __builtin_bit_cast(
            uint4, *reinterpret_cast<const floatx4*>(stage + m * kStageStride + 64 * j + 16 * kq));
    }
  };
  auto load_base = [&](int nt, int kb, Item& I) {
    const size_t tile = ((size_t)nt * KB + kb) * 64 + lane;
    I.w[0] = codes[tile];
    I.mt[0] = meta[((size_t)nt * (2 * KB) + 2 * kb) * kTileN + m];
    I.mt[1] = meta[((size_t)nt * (2 * KB) + 2 * kb + 1) * kTileN + m];
  };
  Item cur, nxt;
  if (!MULTI && my_tiles > 0 && wave < KB) {
    load_x(wave);
    load_base((int)blockIdx.x, wave, cur);
  }

  // ---- routing facts (the only dependent step): highest precision present, per-row constants ----
  const int pmax =
      (__ballot(pl == 3) != 0ull) ? 3 : (__ballot(pl == 2) != 0ull) ? 2 : (__ballot(pl == 1) != 0ull) ? 1 : 0;
  int prow[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) prow[i] = __shfl(pl, 4 * kq + i, 64);
  const int y_token = __shfl(my_token, (int)(threadIdx.x >> 4) & 15, 64);  // output row of the reducing thread

  const UnpackConsts uc = make_unpack_consts();
  const uint4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};

  // The body is instantiated per highest precision so that every load count is static: the
  // hardware wait counters can then let the next tile's loads stay in flight.
  auto body = [&](auto pm_tag) {
    constexpr int PM = decltype(pm_tag)::value;
    auto load_rest = [&](int nt, int kb, Item& I) {
      const size_t tile = ((size_t)nt * KB + kb) * 64 + lane;
      if constexpr (PM >= 1) I.w[1] = codes[slice_vec + tile];
      if constexpr (PM >= 2) I.w[2] = codes[2 * slice_vec + tile];
      if constexpr (PM >= 3) I.w[3] = codes[3 * slice_vec + tile];
    };
    int step_count = 0;
#pragma unroll 1
    for (int chunk = 0; chunk < chunks; ++chunk) {
      const int kb = chunk * WAVES + wave;
      const bool active = (kb < KB) && my_tiles > 0;
      if (active) {
        if (MULTI) {
          load_x(kb);
          load_base((int)blockIdx.x, kb, cur);
        }
        load_rest((int)blockIdx.x, kb, cur);
        transpose_x(kb);
        // group sums of this block's activations, in accumulator layout, and the offset term
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          floatx4 Sa = mfma(xa[4 * h + 0], ones, zero4);
          Sa = mfma(xa[4 * h + 2], ones, Sa);
          floatx4 Sb = mfma(xa[4 * h + 1], ones, zero4);
          Sb = mfma(xa[4 * h + 3], ones, Sb);
          floatx4 c1, ss;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int p = prow[i];
            // offsets accumulated up to slice p: sums of the operand biases of slices 0..p
            const float coefA = (p >= 3) ? 74.f : (p == 2) ? 72.f : (p == 1) ? 64.f : 32.f;
            const float coefB = (p >= 3) ? 18.5f : (p == 2) ? 18.f : (p == 1) ? 16.f : 8.f;
            // residual zero points: sum_{1 <= e <= p} 4^-e (2 - 0.5), and the base slice's -0.5
            const float q = (p >= 3) ? 0.328125f : (p == 2) ? 0.3125f : (p == 1) ? 0.25f : 0.f;
            ss[i] = Sa[i] + Sb[i];
            c1[i] = coefA * Sa[i] + coefB * Sb[i] + (1.5f * q - 0.5f) * ss[i];
          }
          cst[h * 64 + lane] = c1;
          cst[(2 + h) * 64 + lane] = ss;
        }
      }
      // one step: fetch tile ti+1 into `n`, consume tile ti from `c`, reduce and store
      auto step = [&](int ti, Item& c, Item& n) {
        const int nt = (int)blockIdx.x + ti * (int)gridDim.x;
        floatx4 acc = zero4;
        if (active) {
          const int tn = (int)blockIdx.x + min(ti + 1, my_tiles - 1) * (int)gridDim.x;
          load_base(tn, kb, n);
          load_rest(tn, kb, n);
          // the two groups of the block run as two independent accumulator chains
          floatx4 D[2], v[2];
          D[0] = slice_group<0>(&xa[0], uc, c.w[0].x, c.w[0].y, zero4);
          D[1] = slice_group<0>(&xa[4], uc, c.w[0].z, c.w[0].w, zero4);
          v[0] = D[0];
          v[1] = D[1];
          if constexpr (PM >= 1) {
            D[0] = slice_group<1>(&xa[0], uc, c.w[1].x, c.w[1].y, D[0]);
            D[1] = slice_group<1>(&xa[4], uc, c.w[1].z, c.w[1].w, D[1]);
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
              for (int i = 0; i < 4; ++i) v[h][i] = (prow[i] >= 1) ? D[h][i] : v[h][i];
          }
          if constexpr (PM >= 2) {
            D[0] = slice_group<2>(&xa[0], uc, c.w[2].x, c.w[2].y, D[0]);
            D[1] = slice_group<2>(&xa[4], uc, c.w[2].z, c.w[2].w, D[1]);
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
              for (int i = 0; i < 4; ++i) v[h][i] = (prow[i] >= 2) ? D[h][i] : v[h][i];
          }
          if constexpr (PM >= 3) {
            D[0] = slice_group<3>(&xa[0], uc, c.w[3].x, c.w[3].y, D[0]);
            D[1] = slice_group<3>(&xa[4], uc, c.w[3].z, c.w[3].w, D[1]);
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
              for (int i = 0; i < 4; ++i) v[h][i] = (prow[i] >= 3) ? D[h][i] : v[h][i];
          }
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const float s0 = c.mt[h].x, s0z0 = c.mt[h].x * c.mt[h].y;
            const floatx4 c1 = cst[h * 64 + lane];
            const floatx4 ss = cst[(2 + h) * 64 + lane];
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] += s0 * (v[h][i] - c1[i]) - s0z0 * ss[i];
          }
        }
        // sum the wavefronts' partial tiles; rows leave in original token order
        const int buf = step_count & 1;
        ++step_count;
#pragma unroll
        for (int i = 0; i < 4; ++i) red[buf][wave][lane][i] = acc[i];
        __syncthreads();
        if (threadIdx.x < 256) {
          const int r = threadIdx.x >> 4, cc = threadIdx.x & 15;
          const int64_t col = (int64_t)nt * kTileN + cc;
          float sum = 0.f;
#pragma unroll
          for (int wv = 0; wv < WAVES; ++wv) sum += red[buf][wv][16 * (r >> 2) + cc][r & 3];
          if (MULTI) {
            if (chunk > 0) sum += part[ti][threadIdx.x];
            if (chunk + 1 < chunks) part[ti][threadIdx.x] = sum;
          }
          if (chunk + 1 == chunks && r < T && col < N) Y[(int64_t)y_token * N + col] = sum;
        }
      };
#pragma unroll 1
      for (int ti = 0; ti < my_tiles; ti += 2) {
        step(ti, cur, nxt);
        if (ti + 1 < my_tiles) step(ti + 1, nxt, cur);
      }
    }
  };
  switch (pmax) {
    case 0: body(std::integral_constant<int, 0>{}); break;
    case 1: body(std::integral_constant<int, 1>{}); break;
    case 2: body(std::integral_constant<int, 2>{}); break;
    default: body(std::integral_constant<int, 3>{}); break;
  }
}

template <int WAVES, bool MULTI>
static void launch_decode16(int grid, hipStream_t stream, const uint16_t* X, int T, const Shape& sh,
                            const uint4* codes, const float2* meta, const int32_t* prec, const int32_t* perm,
                            float* Y) {
  hipLaunchKernelGGL((decode16_kernel<WAVES, MULTI>), dim3(grid, (T + 15) / 16), dim3(WAVES * 64), 0, stream, X, T,
                     sh.K, codes, sh.slice_words / 4, meta, sh.N, sh.NT, sh.KB, prec, T > 16 ? perm : nullptr, Y);
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
                                  const int32_t* prec, const int32_t* perm, float* Y, hipStream_t stream) {
  const uint4* codes = reinterpret_cast<const uint4*>(blob);
  const float2* meta = reinterpret_cast<const float2*>(reinterpret_cast<const char*>(blob) + sh.meta_offset);
  int waves = knob(0);
  // eight wavefronts leave 256 registers each: room for the staged activations and both weight buffers
  if (waves != 4 && waves != 8 && waves != 16) waves = (sh.KB <= 4) ? 4 : 8;
  const bool multi = sh.KB > waves;
  int per_cu = knob(2);
  if (per_cu <= 0) per_cu = (waves == 4) ? 2 : 1;  // resident workgroups per compute unit at these register counts
  const int token_tiles = (int)((T + 15) / 16);
  int grid = (compute_units() * per_cu + token_tiles - 1) / token_tiles;  // workgroups per token tile
  if (grid > sh.NT) grid = sh.NT;
  // with several K chunks the per-tile partial sums live in LDS: bound the tiles per workgroup
  if (multi && (sh.NT + grid - 1) / grid > d16::kMaxTilesMulti)
    grid = (sh.NT + d16::kMaxTilesMulti - 1) / d16::kMaxTilesMulti;
#define MBQ_D16(WV)                                                                          \
  if (waves == WV) {                                                                         \
    if (multi) launch_decode16<WV, true>(grid, stream, X, (int)T, sh, codes, meta, prec, perm, Y);  \
    else launch_decode16<WV, false>(grid, stream, X, (int)T, sh, codes, meta, prec, perm, Y);       \
  }
  MBQ_D16(4) MBQ_D16(8) MBQ_D16(16)
#undef MBQ_D16
  return hip_status(hipGetLastError(), "decode16_kernel launch");
}

}  // namespace mbq
