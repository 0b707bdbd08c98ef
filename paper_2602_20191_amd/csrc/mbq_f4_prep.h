// Preparation of the activations for the FP4-operand decode kernel: bf16 -> two FP8 (E4M3)
// pieces in MFMA A-operand order, group sums and per-block scale exponents.  Shared by the
// stand-alone preparation kernel and by the router launch that carries it along.
#pragma once

#include "mbq_common.h"

namespace mbq {
namespace f4 {

constexpr int kPieces = 2;
// The second piece holds the remainder of the first multiplied by 2^kPieceShift (its MFMAs get a block
// scale that much smaller): a bf16 value v = 2^a (1.f) with a >= -6 in the scaled block is then
// exactly piece0 + piece1 / 16 (four significant bits each), i.e. the split is exact over 13 binades
// below the block's largest element and off by at most 2^-21 of that element further down.
constexpr int kPieceShift = 4;
// Prepared activations of one 256-column block: [2 groups][2 pieces][2 halves][64 lanes] x 16 bytes
// (a lane's 32 operand bytes are split so that each 16-byte load of a wavefront is contiguous), then
// per group the 16 token sums (fp32), then the 16 scale exponents (int32).
constexpr size_t kPrepVecPerBlock = 2 * kPieces * 64 * 2;  // uint4 units
constexpr size_t kPrepBytesPerBlock = kPrepVecPerBlock * 16 + 2 * 16 * 4 + 16 * 4;

// One wavefront per 256-column block: lane (m, qa) = (token, k sub-block of the MFMA A operand).
// A lane's 32 bytes of one (group, piece) are the A operand registers of one MFMA: bytes
// 16 c + 8 step + 4 h + j hold column 128 g + 64 (qa & 1) + 32 step + 8 (2 c + (qa >> 1)) + 2 j + h
// of the block, which is where the FP4 operand built from lane group 2 c + (qa >> 1) of the packed
// tile puts the matching weight.
// `token` is the row of X that is row m = lane % 16 of the tile (-1: no token, zeros); `base` is where
// the prepared block goes.
__device__ inline void prep_block_rows(const uint16_t* __restrict__ X, int token, int64_t K, char* __restrict__ base,
                                       int kb, int lane) {
  const int m = lane & 15, qa = lane >> 4;
  uint4* out = reinterpret_cast<uint4*>(base);
  float* sums = reinterpret_cast<float*>(base + kPrepVecPerBlock * 16);
  int* scl = reinterpret_cast<int*>(base + kPrepVecPerBlock * 16 + 2 * 16 * 4);

  uint4 raw[2][2][2];  // [group][c][step]
#pragma unroll
  for (int g = 0; g < 2; ++g)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int step = 0; step < 2; ++step) {
        const int64_t col = (int64_t)kb * kTileK + 128 * g + 64 * (qa & 1) + 32 * step + 8 * (2 * c + (qa >> 1));
        raw[g][c][step] = (token >= 0 && col < K) ? *reinterpret_cast<const uint4*>(X + (int64_t)token * K + col)
                                                  : uint4{0u, 0u, 0u, 0u};
      }
  // largest exponent of the token's block
  uint32_t mx = 0u;
#pragma unroll
  for (int g = 0; g < 2; ++g)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int step = 0; step < 2; ++step) {
        const uint32_t u[4] = {raw[g][c][step].x, raw[g][c][step].y, raw[g][c][step].z, raw[g][c][step].w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          mx = max(mx, u[t] & 0x7F800000u);
          mx = max(mx, (u[t] << 16) & 0x7F800000u);
        }
      }
  mx = max(mx, (uint32_t)__shfl_xor((int)mx, 16, 64));
  mx = max(mx, (uint32_t)__shfl_xor((int)mx, 32, 64));
  // scale the largest element into [2^7, 2^8): below the FP8 (E4M3) maximum 448
  int scale_byte = (int)(mx >> 23) - 7;  // = 127 + k, x = 2^k * scaled
  scale_byte = min(max(scale_byte, 1 + kPieceShift), 254);
  const int down = 127 - scale_byte;      // exponent of the factor applied to x
  if (qa == 0) scl[m] = scale_byte;

#pragma unroll
  for (int g = 0; g < 2; ++g) {
    float sum = 0.f;
    int piece_regs[kPieces][8];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int step = 0; step < 2; ++step) {
        const uint32_t u[4] = {raw[g][c][step].x, raw[g][c][step].y, raw[g][c][step].z, raw[g][c][step].w};
        float v[2][4];  // [h][j]: column 2 j + h of the run
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          v[0][j] = __uint_as_float(u[j] << 16);
          v[1][j] = __uint_as_float(u[j] & 0xFFFF0000u);
          sum += v[0][j] + v[1][j];
          v[0][j] = __builtin_ldexpf(v[0][j], down);
          v[1][j] = __builtin_ldexpf(v[1][j], down);
        }
#pragma unroll
        for (int piece = 0; piece < kPieces; ++piece)
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            int packed = __builtin_amdgcn_cvt_pk_fp8_f32(v[h][0], v[h][1], 0, false);
            packed = __builtin_amdgcn_cvt_pk_fp8_f32(v[h][2], v[h][3], packed, true);
            piece_regs[piece][4 * c + 2 * step + h] = packed;
            v[h][0] = (v[h][0] - __builtin_amdgcn_cvt_f32_fp8(packed, 0)) * (float)(1 << kPieceShift);
            v[h][1] = (v[h][1] - __builtin_amdgcn_cvt_f32_fp8(packed, 1)) * (float)(1 << kPieceShift);
            v[h][2] = (v[h][2] - __builtin_amdgcn_cvt_f32_fp8(packed, 2)) * (float)(1 << kPieceShift);
            v[h][3] = (v[h][3] - __builtin_amdgcn_cvt_f32_fp8(packed, 3)) * (float)(1 << kPieceShift);
          }
      }
    sum += __shfl_xor(sum, 16, 64);
    sum += __shfl_xor(sum, 32, 64);
    if (qa == 0) sums[16 * g + m] = sum;
#pragma unroll
    for (int piece = 0; piece < kPieces; ++piece) {
      uint4* dst = out + (size_t)(g * kPieces + piece) * 128 + lane;
      const int* r = piece_regs[piece];
      dst[0] = uint4{(uint32_t)r[0], (uint32_t)r[1], (uint32_t)r[2], (uint32_t)r[3]};
      dst[64] = uint4{(uint32_t)r[4], (uint32_t)r[5], (uint32_t)r[6], (uint32_t)r[7]};
    }
  }
}

// One token tile in original order: row m is token m.
__device__ inline void prep_block(const uint16_t* __restrict__ X, int T, int64_t K, char* __restrict__ prep,
                                  int kb, int lane) {
  const int m = lane & 15;
  prep_block_rows(X, m < T ? m : -1, K, prep + (size_t)kb * kPrepBytesPerBlock, kb, lane);
}

}  // namespace f4
}  // namespace mbq
