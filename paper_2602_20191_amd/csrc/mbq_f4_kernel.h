// What the one-token-tile (T <= 16) FP4-operand decode kernels share: the description of a launch's matrices,
// the operand construction from packed code dwords, the scaled MFMA of one slice and group, the token sort.
// (Arithmetic and layout are explained at the top of mbq_linear_decode_f4.hip.)
#pragma once

#include "mbq_common.h"
#include "mbq_f4_prep.h"

namespace mbq {

typedef int intx8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace f4 {


struct Proj {
  const uint4* codes;
  const float2* meta;
  const int32_t* prec;
  int32_t* perm;     // with offsets: where the launch leaves the tokens sorted by precision (null: nowhere)
  int32_t* offsets;
  float* Y;
  size_t slice_vec;  // uint4 per slice
  int64_t N;
  int tile_begin;    // index of this matrix's first tile in the joint list
  int pad;
};
struct Group {
  Proj p[MBQ_MAX_GROUP];
  int n;
  int tiles;
  unsigned long long* stamps;  // timeline build of the kernel only: where the stamps go
  int bit_view;                // the precision arrays hold bits - 1 instead of digit precisions (see RouteView)
};

template <int R>
__device__ inline uint32_t rotr(uint32_t w) {
  if constexpr (R == 0) return w;
  return __builtin_amdgcn_alignbit(w, w, R);
}

// FP4 operand dwords of one packed dword of slice E: eight codes of k-step 0, eight of k-step 1.
// The unrotated field of (step, slot s = 2j + h) sits at bit 16h + 4j + 2 step and slice E is
// stored rotated left by 2 - 2E; nibble 4h + j of the result holds slot 2j + h.
template <int E>
__device__ inline void nibbles(uint32_t w, uint32_t mask, int& step0, int& step1) {
  constexpr int r0 = (2 - 2 * E) & 31, r1 = (4 - 2 * E) & 31;
  step0 = (int)(rotr<r0>(w) & mask);
  step1 = (int)(rotr<r1>(w) & mask);
}

template <int E>
__device__ inline floatx4 slice_group(const intx8* A, uint32_t w_lo, uint32_t w_hi, uint32_t mask, int sa, int sa2, int sb,
                                       floatx4 D) {
  intx8 B = {0, 0, 0, 0, 0, 0, 0, 0};
  int b0, b1, b2, b3;
  nibbles<E>(w_lo, mask, b0, b1);
  nibbles<E>(w_hi, mask, b2, b3);
  B[0] = b0; B[1] = b1; B[2] = b2; B[3] = b3;
#pragma unroll
  for (int piece = 0; piece < kPieces; ++piece)
    D = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(A[piece], B, D, 0 /* A: FP8 E4M3 */, 4 /* B: FP4 */, E,
                                                         piece == 0 ? sa : sa2, E, sb);
  return D;
}

// Stable counting sort of the T <= 64 tokens of one matrix by precision (Sec. 4.3, token permutation),
// by one wavefront: p = precision of token `lane`, -1 past the last token.
__device__ inline void bucket_by_wave(int p, int lane, int32_t* __restrict__ perm, int32_t* __restrict__ offsets) {
  const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  int start = 0, my_pos = 0;
#pragma unroll
  for (int q = 0; q < MBQ_N_PRECISIONS; ++q) {
    const uint64_t b = __ballot(p == q);
    if (p == q) my_pos = start + __popcll(b & below);
    if (lane == q) offsets[q] = start;
    start += __popcll(b);
  }
  if (lane == MBQ_N_PRECISIONS) offsets[MBQ_N_PRECISIONS] = start;
  if (p >= 0) perm[my_pos] = lane;
}

// A value that is the same in every lane, moved to scalar registers (the compiler cannot always see that it is).
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ size_t uniform(size_t v) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
  return ((size_t)hi << 32) | lo;
}
template <typename P>
__device__ __forceinline__ P* uniform(P* p) { return reinterpret_cast<P*>(uniform((size_t)(uintptr_t)p)); }
// workgroup barrier that orders LDS traffic only (loads from global memory stay in flight across it)
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

struct Item {  // one 16 x 256 block: four slices and the {s0, z0} of its two groups
  uint4 w[4];
  float2 mt[2];
};

}  // namespace f4

// launch geometry shared by the kernels' launchers
int f4_compute_units();
// T <= 16 and at most 32 column blocks (K <= 8192), or up to 64 when the call has few enough row tiles (`tiles` = row
// tiles of all matrices of the call): a loader wavefront and eight arithmetic wavefronts per workgroup
bool decode_f4_ws_supports(int KB, int tiles);
int decode_f4_ws_parts(int KB);  // 2: the launch adds into outputs that must be zero when it starts
int decode_f4_ws_stamp_wavefronts();
mbq_status launch_linear_decode_f4_ws(int64_t T, const f4::Group& g, int KB, const void* ws, hipStream_t stream);

}  // namespace mbq
