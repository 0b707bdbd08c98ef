// Decode-side routed linear for one token tile (T <= 16): the bandwidth-bound path.
//
// Paper Sec. 4.2 Eq. 6 evaluated slice by slice, Y_i = sum_{e <= p_i} W_e^T X_i, with the
// shared-scale structure of App. B (s_e = s0/4^e, z_e = 2 for e >= 1); only slices
// 0..max_i p_i are fetched (Sec. 4.3, on-demand slice access).
//
// Work split: a workgroup of WAVES wavefronts owns the 16-row code tiles nt = w, w + W, ... of its matrix
// (w = its index among the W workgroups of that matrix).  The K axis is cut into chunks of WAVES 256-column blocks;
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

constexpr int kMaxTilesMulti = 32;  // tiles per workgroup whose partial sums fit the LDS budget (per token tile: 32 / TT)
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

// the four B operands of one group (two dwords) of slice E, and the four MFMAs that consume them
template <int E>
__device__ inline void unpack_group(const UnpackConsts& uc, uint32_t w_lo, uint32_t w_hi, uint4 (&B)[4]) {
  unpack_dword<E>(w_lo, uc, B[0], B[1]);
  unpack_dword<E>(w_hi, uc, B[2], B[3]);
}
__device__ inline floatx4 mfma_group(const uint4 A[4], const uint4 (&B)[4], floatx4 D) {
  D = mfma(A[0], B[0], D);
  D = mfma(A[1], B[1], D);
  D = mfma(A[2], B[2], D);
  D = mfma(A[3], B[3], D);
  return D;
}

struct Item {
  uint4 w[4];
  float2 mt[2];
};

// One launch serves up to MBQ_MAX_GROUP matrices that read the same activations (each with its own
// routing): matrix j owns workgroups wg_begin .. wg_begin + wg_count - 1 of every token pass.
struct Proj {
  const uint4* codes;
  size_t slice_vec;
  const float2* meta;
  int64_t N;
  int NT;
  const int32_t* prec;
  const int32_t* perm;   // precision-sorted token order (read), or null: original order (one tile) / sorted here
  // sort_perm != null (T <= 128): the tokens have not been sorted yet.  Every wavefront derives the order from
  // the precisions itself (one load and a few ballots instead of two dependent loads), and the matrix's
  // first workgroup writes perm and offsets out for the caller.
  int32_t* sort_perm;
  int32_t* sort_offsets;
  const int32_t* gate_offsets;  // non-null: run only if mix_prefers_stationary says so (the prefill launch follows)
  float* Y;
  int wg_begin, wg_count;
  // 2: the K chunks are dealt to two workgroups per tile set (even / odd workgroup of the matrix take the first /
  // second half of the chunks) that ADD their results into Y, which the caller has zeroed; 1: one workgroup, stores
  int ksplit;
};
struct Group {
  Proj p[MBQ_MAX_GROUP];
  int n;
};

}  // namespace d16

// MULTI: the K axis needs more than one chunk (KB > WAVES); partial tiles go through LDS.
// TT: token tiles of 16 per workgroup (1 or 2): the weights of a block are unpacked once and meet the
// activation fragments of every tile, so 17..64 tokens take one pass over the weights per 32 tokens.
template <int WAVES, bool MULTI, int TT>
__global__ __launch_bounds__(WAVES * 64) void decode16_kernel(const uint16_t* __restrict__ X, int T, int64_t K,
                                                              int KB, const d16::Group g) {
  using namespace d16;
  // which matrix this workgroup works on (uniform), and its place among that matrix's workgroups
  // (selects between the argument block's entries: indexing it with a run-time value would move it to scratch)
  Proj P = g.p[0];
#pragma unroll
  for (int j = 1; j < MBQ_MAX_GROUP; ++j)
    if (j < g.n && (int)blockIdx.x >= g.p[j].wg_begin) P = g.p[j];
  const uint4* __restrict__ codes = P.codes;
  const size_t slice_vec = P.slice_vec;
  const float2* __restrict__ meta = P.meta;
  const int64_t N = P.N;
  const int NT = P.NT;
  const int32_t* __restrict__ prec = P.prec;
  const int32_t* __restrict__ perm = P.perm;
  float* __restrict__ Y = P.Y;
  if (P.gate_offsets != nullptr && !mix_prefers_stationary(P.gate_offsets, T)) return;
  const int halves = MULTI ? P.ksplit : 1;
  const int wg = ((int)blockIdx.x - P.wg_begin) / halves, wgs = P.wg_count / halves;
  const int half = ((int)blockIdx.x - P.wg_begin) % halves;
  // blockIdx.y = token tile: rows 16 y .. 16 y + 15 of the token order (of the precision-sorted
  // order `perm` when there are several tiles, so that a tile reads only the slices it needs)
  // the tokens are dealt evenly to the passes (65 tokens: 22 + 22 + 21, not 32 + 32 + 1: a pass costs its slices
  // whatever its token count)
  const int per_pass = (T + (int)gridDim.y - 1) / (int)gridDim.y;  // <= 16 TT
  const int row0 = per_pass * (int)blockIdx.y;
  const int T_all = T;
  T = min(per_pass, T - row0);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: keeps tile addresses scalar
  const int m = lane & 15;   // token row of A / weight row of B / output column
  const int kq = lane >> 4;  // k quarter of a k-step; output rows 4 kq .. 4 kq + 3
  const int chunks_all = MULTI ? (KB + WAVES - 1) / WAVES : 1;
  // this workgroup's chunks: all of them, or the first / second half
  const int chunk_begin = (halves == 2 && half == 1) ? (chunks_all + 1) / 2 : 0;
  const int chunks = (halves == 2 && half == 0) ? (chunks_all + 1) / 2 : chunks_all;
  const int my_tiles = (NT - wg + wgs - 1) / wgs;

  __shared__ float red[2][TT][WAVES][64][4];               // per-wavefront partial tiles, double buffered
  // Private to each wavefront: first the staging rows of its activation block (16 tokens x 128
  // columns, row stride kStageStride bytes; one token tile after the other), afterwards C1[2], SS[2]
  // of that block for every token tile.
  __shared__ __attribute__((aligned(16))) char area[WAVES][TT * kAreaBytes];
  __shared__ float part[MULTI ? kMaxTilesMulti / TT : 1][TT][256];  // sums over chunks
  char* const stage = area[wave];
  auto cst_of = [&](int tt) { return reinterpret_cast<floatx4*>(area[wave] + tt * kAreaBytes); };  // [4][64]

  // ---- loads that depend on nothing: precisions first, then activations, slice 0 ----
  int my_token[TT], pl[TT];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) {
    const int r = 16 * tt + lane;  // lanes 0..15 of each tile hold its tokens
    my_token[tt] = (lane < 16 && r < T) ? (perm ? perm[row0 + r] : row0 + r) : -1;
    pl[tt] = (my_token[tt] >= 0 && P.sort_perm == nullptr) ? prec[my_token[tt]] : -1;
  }
  if (P.sort_perm != nullptr) {
    // stable counting sort of all T_all <= 128 tokens by precision (Sec. 4.3, token permutation): a lane holds
    // tokens lane and lane + 64
    const int p_mine = lane < T_all ? min(max(prec[lane], 0), MBQ_N_PRECISIONS - 1) : -1;
    const int p_two = lane + 64 < T_all ? min(max(prec[lane + 64], 0), MBQ_N_PRECISIONS - 1) : -1;
    const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    int start = 0, my_pos = 0, my_pos_two = 0, off_mine = 0;
#pragma unroll
    for (int q = 0; q < MBQ_N_PRECISIONS; ++q) {
      const uint64_t b = __ballot(p_mine == q), b2 = __ballot(p_two == q);
      if (p_mine == q) my_pos = start + __popcll(b & below);
      if (p_two == q) my_pos_two = start + __popcll(b) + __popcll(b2 & below);
      if (lane == q) off_mine = start;
      start += __popcll(b) + __popcll(b2);
    }
    if (lane == MBQ_N_PRECISIONS) off_mine = start;
    // position -> (token, precision) through the wavefront's own LDS rows (in order within a wavefront)
    int* const order = reinterpret_cast<int*>(stage);
    if (p_mine >= 0) order[my_pos] = lane | (p_mine << 8);
    if (p_two >= 0) order[my_pos_two] = (lane + 64) | (p_two << 8);
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
      const int r = 16 * tt + lane;
      const int e = (lane < 16 && r < T) ? order[row0 + r] : -1;
      my_token[tt] = e < 0 ? -1 : (e & 0xFF);
      pl[tt] = e < 0 ? -1 : (e >> 8);
    }
    asm volatile("" ::: "memory");  // the rows are reused below through another type: keep these reads in front
    if ((int)blockIdx.x == P.wg_begin && blockIdx.y == 0 && wave == 0) {
      if (p_mine >= 0) P.sort_perm[my_pos] = lane;
      if (p_two >= 0) P.sort_perm[my_pos_two] = lane + 64;
      if (lane <= MBQ_N_PRECISIONS) P.sort_offsets[lane] = off_mine;
    }
  }
  // Activations: a load instruction covers four token rows, a quarter wavefront reading 256
  // contiguous bytes of each (whole cache lines); the MFMA A layout (token = lane % 16) is then
  // produced by a round trip through the wavefront's LDS rows, one half block at a time (LDS
  // operations of one wavefront execute in order; every access to the area uses one vector type).
  uint4 xa[TT][8];
  auto load_x = [&](int kb) {
    const int64_t k0 = (int64_t)kb * kTileK + 8 * m;  // K is a multiple of 128: a half block is all there or absent
    const uint16_t* col = X + k0;
    const int second = (k0 + 128 < K) ? 128 : 0;
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int tok = __shfl(my_token[tt], 4 * i + kq, 64);
        const uint16_t* src = col + (int64_t)max(tok, 0) * K;  // always a valid address
        xa[tt][i] = *reinterpret_cast<const uint4*>(src);
        xa[tt][4 + i] = *reinterpret_cast<const uint4*>(src + second);
      }
  };
  // Rows past the last token and an absent second half block become zeros on the way through.
  auto transpose_x = [&](int kb) {
    const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
    const bool second = (int64_t)kb * kTileK + 128 < K;
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const bool there = (16 * tt + 4 * i + kq < T) && (h == 0 || second);
          *reinterpret_cast<floatx4*>(stage + (4 * i + kq) * kStageStride + 16 * m) =
              there ? __builtin_bit_cast(floatx4, xa[tt][4 * h + i]) : zero;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
          xa[tt][4 * h + j] = __builtin_bit_cast(
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
    load_base(wg, wave, cur);
  }

  // ---- routing facts (the only dependent step): highest precision present, per-row constants ----
  int plmax = pl[0];
#pragma unroll
  for (int tt = 1; tt < TT; ++tt) plmax = max(plmax, pl[tt]);
  const int pmax = (__ballot(plmax == 3) != 0ull) ? 3 : (__ballot(plmax == 2) != 0ull) ? 2
                   : (__ballot(plmax == 1) != 0ull) ? 1 : 0;
  int prow[TT][4], y_token[TT];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) prow[tt][i] = __shfl(pl[tt], 4 * kq + i, 64);
    y_token[tt] = __shfl(my_token[tt], (int)(threadIdx.x >> 4) & 15, 64);  // output row of the reducing thread
  }

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
    for (int chunk = chunk_begin; chunk < chunks; ++chunk) {
      const int kb = chunk * WAVES + wave;
      const bool active = (kb < KB) && my_tiles > 0;
      if (active) {
        if (MULTI) {
          load_x(kb);
          load_base(wg, kb, cur);
        }
        load_rest(wg, kb, cur);
        transpose_x(kb);
        // group sums of this block's activations, in accumulator layout, and the offset term
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            floatx4 Sa = mfma(xa[tt][4 * h + 0], ones, zero4);
            Sa = mfma(xa[tt][4 * h + 2], ones, Sa);
            floatx4 Sb = mfma(xa[tt][4 * h + 1], ones, zero4);
            Sb = mfma(xa[tt][4 * h + 3], ones, Sb);
            floatx4 c1, ss;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const int p = prow[tt][i];
              // offsets accumulated up to slice p: sums of the operand biases of slices 0..p
              const float coefA = (p >= 3) ? 74.f : (p == 2) ? 72.f : (p == 1) ? 64.f : 32.f;
              const float coefB = (p >= 3) ? 18.5f : (p == 2) ? 18.f : (p == 1) ? 16.f : 8.f;
              // residual zero points: sum_{1 <= e <= p} 4^-e (2 - 0.5), and the base slice's -0.5
              const float q = (p >= 3) ? 0.328125f : (p == 2) ? 0.3125f : (p == 1) ? 0.25f : 0.f;
              ss[i] = Sa[i] + Sb[i];
              c1[i] = coefA * Sa[i] + coefB * Sb[i] + (1.5f * q - 0.5f) * ss[i];
            }
            cst_of(tt)[h * 64 + lane] = c1;
            cst_of(tt)[(2 + h) * 64 + lane] = ss;
          }
      }
      // one step: fetch tile ti+1 into `n`, consume tile ti from `c`, reduce and store
      auto step = [&](int ti, Item& c, Item& n) {
        const int nt = wg + ti * wgs;
        floatx4 acc[TT];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) acc[tt] = zero4;
        if (active) {
          const int tn = wg + min(ti + 1, my_tiles - 1) * wgs;
          load_base(tn, kb, n);
          load_rest(tn, kb, n);
          // the two groups of the block run as two independent accumulator chains per token tile; the
          // operands built from a packed dword serve every token tile
          floatx4 D[TT][2], v[TT][2];
          auto slice = [&](auto e_tag) {
            constexpr int E = decltype(e_tag)::value;
            uint4 B0[4], B1[4];
            unpack_group<E>(uc, c.w[E].x, c.w[E].y, B0);
            unpack_group<E>(uc, c.w[E].z, c.w[E].w, B1);
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
              D[tt][0] = mfma_group(&xa[tt][0], B0, E == 0 ? zero4 : D[tt][0]);
              D[tt][1] = mfma_group(&xa[tt][4], B1, E == 0 ? zero4 : D[tt][1]);
#pragma unroll
              for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int i = 0; i < 4; ++i) v[tt][h][i] = (E == 0 || prow[tt][i] >= E) ? D[tt][h][i] : v[tt][h][i];
            }
          };
          slice(std::integral_constant<int, 0>{});
          if constexpr (PM >= 1) slice(std::integral_constant<int, 1>{});
          if constexpr (PM >= 2) slice(std::integral_constant<int, 2>{});
          if constexpr (PM >= 3) slice(std::integral_constant<int, 3>{});
#pragma unroll
          for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              const float s0 = c.mt[h].x, s0z0 = c.mt[h].x * c.mt[h].y;
              const floatx4 c1 = cst_of(tt)[h * 64 + lane];
              const floatx4 ss = cst_of(tt)[(2 + h) * 64 + lane];
#pragma unroll
              for (int i = 0; i < 4; ++i) acc[tt][i] += s0 * (v[tt][h][i] - c1[i]) - s0z0 * ss[i];
            }
        }
        // sum the wavefronts' partial tiles; rows leave in original token order
        const int buf = step_count & 1;
        ++step_count;
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
          for (int i = 0; i < 4; ++i) red[buf][tt][wave][lane][i] = acc[tt][i];
        __syncthreads();
        if (threadIdx.x < 256) {
          const int r = threadIdx.x >> 4, cc = threadIdx.x & 15;
          const int64_t col = (int64_t)nt * kTileN + cc;
#pragma unroll
          for (int tt = 0; tt < TT; ++tt) {
            float sum = 0.f;
#pragma unroll
            for (int wv = 0; wv < WAVES; ++wv) sum += red[buf][tt][wv][16 * (r >> 2) + cc][r & 3];
            if (MULTI) {
              if (chunk > chunk_begin) sum += part[ti][tt][threadIdx.x];
              if (chunk + 1 < chunks) part[ti][tt][threadIdx.x] = sum;
            }
            if (chunk + 1 == chunks && 16 * tt + r < T && col < N) {
              float* const y = &Y[(int64_t)y_token[tt] * N + col];
              if (halves == 2) unsafeAtomicAdd(y, sum);  // two addends into a zeroed output: order-independent
              else *y = sum;
            }
          }
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

template <int WAVES, bool MULTI, int TT>
static void launch_decode16(int grid, hipStream_t stream, const uint16_t* X, int T, int64_t K, int KB,
                            const d16::Group& g) {
  hipLaunchKernelGGL((decode16_kernel<WAVES, MULTI, TT>), dim3(grid, (T + 16 * TT - 1) / (16 * TT)), dim3(WAVES * 64), 0,
                     stream, X, T, K, KB, g);
}

namespace d16 {
// Launch shape of a call (common K): kernel variant, workgroups per token pass and matrix, K split per matrix.
struct Plan {
  int waves, tt, token_passes;
  bool multi;
  int share[MBQ_MAX_GROUP];   // workgroups per pass (tile sets)
  int ksplit[MBQ_MAX_GROUP];  // workgroups per tile set along K (1 or 2)
};

static Plan make_plan(int64_t T, int n, const Shape* shapes) {
  const Shape& sh = shapes[0];  // K, and with it the kernel variant, is common to the matrices of a call
  Plan pl;
  pl.waves = knob(0);
  // eight wavefronts leave 256 registers each: room for the staged activations and both weight buffers
  if (pl.waves != 4 && pl.waves != 8 && pl.waves != 16) pl.waves = (sh.KB <= 4) ? 4 : 8;
  pl.multi = sh.KB > pl.waves;
  int per_cu = knob(2);
  if (per_cu <= 0) per_cu = (pl.waves == 4) ? 2 : 1;  // resident workgroups per compute unit at these register counts
  // two token tiles per workgroup above 32 tokens (eight wavefronts: the second tile's fragments need the
  // registers): two passes over the weights instead of three or four; measured on cold weights, 14336 x 4096 at 48
  // tokens 39 us against 57 us, at 64 tokens 39 against 44; up to 32 tokens two one-tile passes side by side are as fast
  pl.tt = (T > 32 && pl.waves == 8 && knob(7) != 3) ? 2 : 1;
  pl.token_passes = (int)((T + 16 * pl.tt - 1) / (16 * pl.tt));
  const int budget = (device_compute_units() * per_cu + pl.token_passes - 1) / pl.token_passes;  // workgroups per pass
  // with several K chunks the per-tile partial sums live in LDS: bound the tiles per workgroup
  const int max_tiles = kMaxTilesMulti / pl.tt;
  int64_t all_tiles = 0;
  for (int i = 0; i < n; ++i) all_tiles += shapes[i].NT;
  for (int i = 0; i < MBQ_MAX_GROUP; ++i) {
    pl.share[i] = 0;
    pl.ksplit[i] = 1;
    if (i >= n) continue;
    const Shape& s = shapes[i];
    // the pass's workgroups are dealt to the matrices in proportion to their row tiles
    int share = (int)(((int64_t)budget * s.NT + all_tiles - 1) / all_tiles);
    if (share < 1) share = 1;
    if (share > s.NT) share = s.NT;
    const int min_share = pl.multi ? (s.NT + max_tiles - 1) / max_tiles : 1;
    if (share < min_share) share = min_share;
    // A workgroup pays a prologue per K chunk (the chunk's activations through LDS, group sums: about 4 us);
    // with few tiles per workgroup that dominates (4096 x 14336 at 64 tokens: seven chunks of two tiles each).
    // Two workgroups along K with twice the tiles each halve the prologues per tile; they add into an output
    // that the caller zeroes first, so only small outputs take the split.
    // The choice looks at the matrix alone (not at its share of a grouped launch), so that a matrix gives the
    // same bits in a grouped and in a single call.
    if (pl.multi && s.NT <= 6 * budget && (int64_t)T * s.N * 4 <= (2 << 20)) {
      pl.ksplit[i] = 2;
      share = share / 2 > min_share ? share / 2 : min_share;
    }
    pl.share[i] = share;
  }
  return pl;
}
}  // namespace d16

// outputs that the launch below ADDS into: the caller clears them first (zero_outputs, or the router launch)
void decode16_zero_list(int64_t T, int n, const Shape* shapes, float* const* Y, ZeroList* zl) {
  const d16::Plan pl = d16::make_plan(T, n, shapes);
  for (int i = 0; i < MBQ_MAX_GROUP; ++i) {
    const bool add = i < n && pl.ksplit[i] == 2;
    zl->p[i] = add ? Y[i] : nullptr;
    zl->n[i] = add ? (long long)T * shapes[i].N : 0;
  }
}

__global__ __launch_bounds__(256) void zero_outputs_kernel(const ZeroList zl) {
  zero_share(zl, (int)blockIdx.x, (int)gridDim.x, (int)threadIdx.x, 256);
}

mbq_status launch_zero_outputs(const ZeroList& zl, hipStream_t stream) {
  bool any = false;
  for (int i = 0; i < MBQ_MAX_GROUP; ++i) any = any || zl.p[i] != nullptr;
  if (!any) return MBQ_OK;
  hipLaunchKernelGGL(zero_outputs_kernel, dim3(128), dim3(256), 0, stream, zl);
  return hip_status(hipGetLastError(), "zero_outputs_kernel launch");
}

mbq_status launch_linear_decode16_group(const uint16_t* X, int64_t T, int n, const void* const* blobs,
                                        const Shape* shapes, const int32_t* const* prec, const int32_t* const* perm,
                                        float* const* Y, hipStream_t stream, int32_t* const* sort_perm,
                                        int32_t* const* sort_offsets, const int32_t* const* gate_offsets) {
  const Shape& sh = shapes[0];
  const d16::Plan pl = d16::make_plan(T, n, shapes);
  const int waves = pl.waves, tt = pl.tt;
  const bool multi = pl.multi;
  d16::Group g;
  int grid = 0;
  for (int i = 0; i < MBQ_MAX_GROUP; ++i) {
    const int j = i < n ? i : 0;
    const Shape& s = shapes[j];
    d16::Proj& p = g.p[i];
    p.codes = reinterpret_cast<const uint4*>(blobs[j]);
    p.slice_vec = s.slice_words / 4;
    p.meta = reinterpret_cast<const float2*>(reinterpret_cast<const char*>(blobs[j]) + s.meta_offset);
    p.N = s.N;
    p.NT = s.NT;
    p.prec = prec[j];
    p.perm = (T > 16 && !sort_perm) ? perm[j] : nullptr;
    p.sort_perm = sort_perm ? sort_perm[j] : nullptr;
    p.sort_offsets = sort_perm ? sort_offsets[j] : nullptr;
    p.gate_offsets = gate_offsets ? gate_offsets[j] : nullptr;
    p.Y = Y[j];
    p.ksplit = i < n ? pl.ksplit[i] : 1;
    p.wg_begin = grid;
    p.wg_count = i < n ? pl.share[i] * pl.ksplit[i] : 0;
    if (i < n) grid += pl.share[i] * pl.ksplit[i];
  }
  g.n = n;
#define MBQ_D16(WV, TTV)                                                                     \
  if (waves == WV && tt == TTV) {                                                            \
    if (multi) launch_decode16<WV, true, TTV>(grid, stream, X, (int)T, sh.K, sh.KB, g);      \
    else launch_decode16<WV, false, TTV>(grid, stream, X, (int)T, sh.K, sh.KB, g);           \
  }
  MBQ_D16(4, 1) MBQ_D16(8, 1) MBQ_D16(16, 1) MBQ_D16(8, 2)
#undef MBQ_D16
  return hip_status(hipGetLastError(), "decode16_kernel launch");
}

mbq_status launch_linear_decode16(const uint16_t* X, int64_t T, const void* blob, const Shape& sh,
                                  const int32_t* prec, const int32_t* perm, float* Y, hipStream_t stream) {
  return launch_linear_decode16_group(X, T, 1, &blob, &sh, &prec, &perm, &Y, stream, nullptr, nullptr);
}

}  // namespace mbq
