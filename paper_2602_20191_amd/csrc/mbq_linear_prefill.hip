// Prefill-side routed linear: a bf16 MFMA tiled GEMM per precision bucket.
//
// Paper Sec. 4.2 Eq. 6 in the merged-code form of App. B (truncating the merged
// integer code is the coarser quantiser): for a token of precision p,
//   Y[i][n] = sum_g (s0/64) * ( sum_{k in g} x_ik V_nk + (0.5 * 4^(3-p) - 64 z0) * Sx[i][g] )
// with V = I_p * 4^(3-p) the 8-bit code whose unused low digits are zero and Sx the group
// sums of x.  Tokens arrive sorted by precision (Sec. 4.3, token permutation), so a tile of
// sorted rows has one precision and reads only slices 0..p.
//
// How the group scale reaches the matrix cores without a second accumulator set:
//   s0 = m * 2^t with m in [1/2, 2) chosen so that the bf16 exponent below is even.  The MFMA
//   B operand is the exact bf16 number (OFF + V) * 2^t (OFF = 256 for p <= 2, where V/2 sits in
//   the seven mantissa bits under a per-row exponent byte; OFF = 0 for p = 3), so a group's
//   products are already in units of 2^t and only the mantissa factor m is left.  The running
//   accumulator R is kept in units of the CURRENT group's m:  R <- R * (m_prev / m_cur) at a
//   group boundary (one multiply per element, ratio in (1/4, 4)), then the group's MFMAs
//   accumulate straight into R.  After the last group R * m_last / 64 is the sum in true units.
//   The zero-point / offset term  -sum_g s0 (OFF/64 - half/64 + z0) Sx[i][g]  is a rank-G update
//   done at the end with fp32 MFMAs (32x32x2), so it costs no vector work in the K loop.
//
// Workgroup: 512 threads = 2 (tokens) x 4 (outputs) wavefronts, tile 256 sorted tokens x 256
// outputs, wavefront tile 128 x 64 as 4 x 2 MFMAs of 32x32x16, K step 32 (a quarter group) with
// one workgroup barrier per step; the schedule is described at prefill_tile.  A small pre-kernel
// gathers the activations into sorted order (so the main kernel streams contiguous rows straight
// into LDS) and writes the group sums transposed ([group][sorted row]).
#include <type_traits>

#include "mbq_common.h"

namespace mbq {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBM = 256, kBN = 256, kBK = 32;
constexpr int kBRowBytes = 2 * kBK + 16;           // LDS row pitch of the weight tile (80 bytes): conflict-free
constexpr int kBSlotBytes = kBN * kBRowBytes;      // 20 KiB per weight slot, ring of three
constexpr int kBRingBytes = 3 * kBSlotBytes;
constexpr int kARowBytes = 2 * kBK;                // activation rows are unpadded (64 bytes), chunks swizzled
constexpr int kASlotBytes = kBM * kARowBytes;      // 16 KiB per activation slot, ring of five
constexpr int kSmemBytes = kBRingBytes + 5 * kASlotBytes;
constexpr int kPadRows = 256;       // spare sorted rows after the last token (tile loads stay in bounds)

__device__ inline floatx16 mfma_bf16(const u32x4& a, const u32x4& b, floatx16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                 c, 0, 0, 0);
}

__device__ inline uint32_t rotr32(uint32_t w, int r) {  // r in 0..31, compile-time after inlining
  return (r & 31) == 0 ? w : __builtin_amdgcn_alignbit(w, w, r & 31);
}
__host__ __device__ constexpr uint32_t rotl_c(uint32_t m, int r) {
  return ((r & 31) == 0) ? m : ((m << (r & 31)) | (m >> (32 - (r & 31))));
}

// ---- pre-kernel: Xs[r][:] = X[perm[r]][:], SxT[g][r] = sum_{k in g} X[perm[r]][k];
// with a K split also Y[r][:] = 0 (the tile kernel then adds its partial sums) ----------
__global__ __launch_bounds__(256) void prefill_prep_kernel(const uint16_t* __restrict__ X, int64_t T, int64_t K,
                                                           const int32_t* __restrict__ perm,
                                                           uint16_t* __restrict__ Xs, float* __restrict__ SxT,
                                                           int64_t ldT, float* __restrict__ Yzero, int64_t N,
                                                           const int32_t* __restrict__ gate_offsets) {
  // gate_offsets != null: the register-stationary kernel was launched first and has done the work if the mix suits it
  if (gate_offsets != nullptr && mix_prefers_stationary(gate_offsets, (int)T)) return;
  const int64_t r = blockIdx.x;
  if (Yzero)
    for (int64_t n = threadIdx.x; n < N; n += 256) Yzero[r * N + n] = 0.f;
  const uint4* src = reinterpret_cast<const uint4*>(X + (int64_t)perm[r] * K);
  uint4* dst = reinterpret_cast<uint4*>(Xs + r * K);
  const int chunks = (int)(K >> 3);  // a multiple of 16: groups of 16 lanes are whole
  for (int c = threadIdx.x; c < chunks; c += 256) {
    const uint4 v = src[c];
    dst[c] = v;
    const uint32_t u[4] = {v.x, v.y, v.z, v.w};
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) s += __uint_as_float(u[j] << 16) + __uint_as_float(u[j] & 0xFFFF0000u);
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
    if ((threadIdx.x & 15) == 0) SxT[(int64_t)(c >> 4) * ldT + r] = s;
  }
}

// mantissa factor m of a group scale (see the header): exponent field forced to 126 or 127
__device__ inline float scale_mantissa(float s0) {
  return __uint_as_float((__float_as_uint(s0) & 0x00FFFFFFu) ^ 0x3F800000u);
}
// biased bf16 exponent E (even) of (256 + V) * 2^t
__device__ inline uint32_t scale_exponent(float s0) { return ((__float_as_uint(s0) >> 23) + 9u) & ~1u; }

// LDS synchronisation that leaves global loads in flight (a full fence would wait for them).
__device__ __forceinline__ void lds_writes_done() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }
template <int N>
__device__ __forceinline__ void vmem_outstanding_at_most() {  // s_waitcnt vmcnt(N), N <= 63
  static_assert(N >= 0 && N <= 63, "vmcnt range");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// the same wait, needed only where registers are loaded behind the compiler's back
template <int N>
__device__ __forceinline__ void untracked_loads_outstanding_at_most() {
  vmem_outstanding_at_most<N>();
}
// 16 bytes per lane from global memory straight into LDS at lds_base + 16 * lane (wave-uniform base).
__device__ __forceinline__ void global_to_lds_16(const void* gptr, char* lds_base) {
  __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)gptr,
                                   (void __attribute__((address_space(3)))*)lds_base, 16, 0, 0);
}

// Loads whose completion the kernel tracks itself: the compiler sees an ordinary register result, so
// it inserts no vmcnt wait of its own (its waits are all-or-nothing across the loop back edge and
// would drain the activation loads that are meant to stay in flight for three steps).  Every use of
// such a register comes after vmem_outstanding_at_most<N>() followed by settled(...) on it.
__device__ __forceinline__ uint32_t load_dword_untracked(const uint32_t* p) {
  uint32_t r;
  asm volatile("global_load_dword %0, %1, off" : "=v"(r) : "v"(p) : "memory");
  return r;
}
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x2_t load_dwordx2_untracked(const uint32_t* p) {
  u32x2_t r;
  asm volatile("global_load_dwordx2 %0, %1, off" : "=v"(r) : "v"(p) : "memory");
  return r;
}
__device__ __forceinline__ void settled(u32x2_t& a) {
  asm volatile("" : "+v"(a));
}
__device__ __forceinline__ void settled(uint32_t& a) {
  asm volatile("" : "+v"(a));
}
// LDS fragment reads are ordinary loads; touching a fragment makes the compiler place its lgkmcnt wait here
__device__ __forceinline__ void touch(u32x4& a) { asm volatile("" : "+v"(a)); }
// One tile.  P = precision index of the tile's tokens, FULL = all 256 rows are tokens.
//
// Schedule: the K loop advances in steps of 32 columns, one workgroup barrier per step.  A step has
// a memory part X (unpack the weights of step h+2 into LDS, issue global loads several steps ahead,
// rescale the accumulator at a group boundary) and a compute part Y (16 MFMAs on step h).
// Wavefronts 0..3 (ORDER 0) run X then Y, wavefronts 4..7 (ORDER 1) run Y then X; wavefronts w and
// w+4 share a SIMD, so while one of them feeds the matrix core the other does its vector and memory
// work, and the hand-over inside a step needs no barrier.  Everything a step reads was complete at
// the barrier that opened it: weights are written two steps ahead into a ring of three slots
// (B, 256 x 32 bf16, 80-byte rows), so the writes of step h+2 never meet readers of step h-1.
// The activations (A) are loaded by the memory pipeline directly into LDS (no registers, no vector
// work), four steps ahead (two to three steps of flight), into a ring of five unpadded 16 KiB slots whose 16-byte chunks are
// XOR-swizzled by the row so that fragment reads are bank-conflict free; each wavefront loads 32
// rows that its own half of the workgroup consumes, waits for them itself (vmcnt) and publishes
// them with the barrier at the end of the step.  The first half's operand fragments of a step are
// read while the memory part runs (ORDER 1: those of the next step, before the barrier).
template <int P, bool FULL, int ORDER>
__device__ __forceinline__ void prefill_tile(const uint16_t* __restrict__ Xs, int64_t K,
                                             const uint32_t* __restrict__ codes, size_t slice_words,
                                             const float2* __restrict__ meta, int64_t N, int NT, int KB,
                                             const int32_t* __restrict__ perm, const float* __restrict__ SxT,
                                             int64_t ldT, float* __restrict__ Y, int row0, int rows, int ntile_n,
                                             char* smem, int g0, int Gs, bool accumulate) {
  constexpr float kOff = (P == 3) ? 0.f : 256.f;
  constexpr float kHalf = 0.5f * (float)(1 << (2 * (3 - P)));
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;
  const int G = Gs;                                        // this workgroup's groups: g0 .. g0 + Gs - 1
  const int H = 4 * G;                                     // steps of 32 columns
  const int units = FULL ? 8 : (rows + 31) >> 5;           // 32-row units that hold tokens
  const int na = FULL ? 4 : (units - wm + 1) >> 1;         // this wavefront's units: 2a + wm, a < na

  // ---- A: this wavefront loads unit 2 wn + wm (32 rows) of every step: two 1 KiB instructions ----
  // lane -> row 16 j + (lane >> 2) of the unit, LDS chunk position lane & 3, which holds the global
  // chunk (lane & 3) ^ ((row >> 2) & 3)
  const int a_unit = 2 * wn + wm;
  const int a_row = lane >> 2;                                      // + 16 j
  const int a_chunk = (lane & 3) ^ ((a_row >> 2) & 3);              // same for j = 0, 1 (16 j adds 4 to row >> 2)
  const uint16_t* a_src = Xs + (int64_t)(row0 + 32 * a_unit + a_row) * K + (int64_t)g0 * kGroup + 8 * a_chunk;
  const int64_t a_src_j = 16 * K;                                   // 16 rows further
  char* const a_ring = smem + kBRingBytes;
  const uint32_t a_dst = (uint32_t)(32 * a_unit * kARowBytes);      // + slot, + 1 KiB j
  auto load_a = [&](int h, uint32_t slot) {                         // h is clamped: loads are always issued
    const int hc = h < H ? h : H - 1;
#pragma unroll
    for (int j = 0; j < 2; ++j)
      global_to_lds_16(a_src + a_src_j * j + (int64_t)hc * kBK, a_ring + slot + a_dst + 1024 * j);
  };
  // ---- B staging: items j = 0, 1: code tile (wave + 8 j) of the 16 tiles of this workgroup ----
  const int ntile0 = ntile_n * (kBN / kTileN);
  // packed weights of one group (four steps) per item and slice: two dwords, each holding two steps.
  // b_cur is the group being unpacked; b_nxt receives the following group (one 8-byte load per item
  // and slice, issued in the first step of a group, first used two steps later) and is moved into
  // b_cur once it has landed, so no register with a load in flight lives across the loop's back edge.
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  u32x2 b_cur_reg[2][P + 1], b_nxt_reg[2][P + 1];
  uint32_t b_s0[2], b_s0_next[2];  // group scale (fp32 bits) of the item's row
  size_t b_word[2];
  size_t b_meta[2];
  const uint32_t b_lds = (uint32_t)((16 * wave + (lane & 15)) * kBRowBytes + (lane >> 4) * 16);
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    // row tiles past the matrix (N not a multiple of 256) read tile 0: their columns are never stored
    const int nt = (ntile0 + wave + 8 * j < NT) ? ntile0 + wave + 8 * j : 0;
    b_word[j] = ((size_t)nt * KB * 64 + lane) * 4;
    b_meta[j] = (size_t)nt * (2 * KB) * kTileN + (lane & 15);
  }
  auto load_b = [&](int g, u32x2 (&dst)[2][P + 1]) {  // the two dwords of group g (clamped: always issued)
    const int gc = g < G ? g : G - 1;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int ga = g0 + gc;
      const size_t v = b_word[j] + (size_t)(ga >> 1) * kTileWords + 2 * (ga & 1);
#pragma unroll
      for (int e = 0; e <= P; ++e) dst[j][e] = load_dwordx2_untracked(codes + e * slice_words + v);
    }
  };
  auto load_b_scale = [&](int g, uint32_t (&dst)[2]) {
    const int gc = g < G ? g : G - 1;
#pragma unroll
    for (int j = 0; j < 2; ++j)
      dst[j] = load_dword_untracked(reinterpret_cast<const uint32_t*>(meta + b_meta[j] + (size_t)(g0 + gc) * kTileN));
  };
  // registers -> B ring slot, unpacked to exact bf16, in pieces that the full-tile loop spreads between
  // its MFMAs.  b_x[j] is the per-row operand constant of the group being staged: the replicated
  // high exponent byte (P <= 2) or the bits of 2^t (P = 3).
  uint32_t b_x[2];
  auto set_b_const = [&](const uint32_t (&s0)[2]) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const uint32_t E = scale_exponent(__uint_as_float(s0[j]));
      b_x[j] = (P == 3) ? ((E - 8u) << 23) : ((E >> 1) * 0x01010101u);
    }
  };
  // merged fields of the four weights with bit residue 2 r (r = step or step + 2), byte aligned:
  // byte b = V of slot 2 (b & 1) + (b >> 1) ...; P <= 2: one bit further, V / 2
  auto merge_bits = [&](int pair, int j, int r) -> uint32_t {  // pair = which dword of the group
    uint32_t bits = b_cur_reg[j][0][pair] & rotl_c(0xC0C0C0C0u, 2 * r - 4);
    if constexpr (P >= 1) bits |= b_cur_reg[j][1][pair] & rotl_c(0x30303030u, 2 * r - 4);
    if constexpr (P >= 2) bits |= b_cur_reg[j][2][pair] & rotl_c(0x0C0C0C0Cu, 2 * r - 4);
    if constexpr (P >= 3) bits |= b_cur_reg[j][3][pair] & rotl_c(0x03030303u, 2 * r - 4);
    return rotr32(bits, (2 * r - 4 + (P == 3 ? 0 : 1)) & 31);
  };
  // two bf16 pairs of one merged word: bytes (0, 2) and (1, 3)
  auto expand_pair = [&](uint32_t w, int j, int b0) -> uint32_t {
    if constexpr (P == 3) {
      const float sc = __uint_as_float(b_x[j]);
      const float f0 = (float)((w >> (8 * b0)) & 0xFFu) * sc;
      const float f1 = (float)((w >> (8 * (b0 + 2))) & 0xFFu) * sc;
      return __builtin_amdgcn_perm(__float_as_uint(f1), __float_as_uint(f0), 0x07060302u);
    } else {
      return __builtin_amdgcn_perm(b_x[j], w, b0 ? 0x04030401u : 0x04020400u);
    }
  };
  auto write_b = [&](uint32_t slot, int j, const u32x4& v) {
    *reinterpret_cast<u32x4*>(smem + slot + b_lds + j * 128 * kBRowBytes) = v;
  };
  // step = which half of the staged dword (steps alternate 0, 1)
  auto store_b = [&](uint32_t slot, int pair, int step) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const uint32_t lo = merge_bits(pair, j, step), hi = merge_bits(pair, j, step + 2);
      u32x4 v;
      v.x = expand_pair(lo, j, 0);
      v.y = expand_pair(hi, j, 0);
      v.z = expand_pair(lo, j, 1);
      v.w = expand_pair(hi, j, 1);
      write_b(slot, j, v);
    }
  };

  // ---- consumer side: this lane's two output columns and their group scales ----
  int64_t ncol[2];
  size_t c_meta[2];
  bool c_ok[2];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    ncol[b] = (int64_t)ntile_n * kBN + 64 * wn + 32 * b + (lane & 31);
    c_ok[b] = ncol[b] < (int64_t)NT * kTileN;
    const int64_t n = c_ok[b] ? ncol[b] : 0;  // columns past the matrix use column 0's scales; never stored
    c_meta[b] = (size_t)(n >> 4) * (2 * KB) * kTileN + (size_t)(n & 15);
  }
  float m_cur[2];
  uint32_t m_next[2];  // raw scale bits of the next group; mantissa taken at use
  auto load_m = [&](int g, uint32_t (&dst)[2]) {
    const int gc = g < G ? g : G - 1;
#pragma unroll
    for (int b = 0; b < 2; ++b)
      dst[b] = load_dword_untracked(reinterpret_cast<const uint32_t*>(meta + c_meta[b] + (size_t)(g0 + gc) * kTileN));
  };
  // fragment addresses: A row 32 (2a + wm) + (lane & 31), chunk 2 kk + (lane >> 5), swizzled
  const int f_row = lane & 31;
  const uint32_t fa_lds0 = (uint32_t)((32 * wm + f_row) * kARowBytes + (((lane >> 5)) ^ ((f_row >> 2) & 3)) * 16);
  const uint32_t fa_lds1 = (uint32_t)((32 * wm + f_row) * kARowBytes + ((2 + (lane >> 5)) ^ ((f_row >> 2) & 3)) * 16);
  const uint32_t fb_lds = (uint32_t)((64 * wn + f_row) * kBRowBytes + (lane >> 5) * 16);

  floatx16 acc[4][2];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  u32x4 af0[4], bf0[2];
  // kk = which 16 columns of the step: 4 (or na) + 2 reads of 16 bytes per lane
  auto read_frags = [&](uint32_t a_slot, uint32_t b_slot, auto kk_tag, u32x4 (&af)[4], u32x4 (&bf)[2]) {
    constexpr int kk = decltype(kk_tag)::value;
#pragma unroll
    for (int a = 0; a < 4; ++a)
      if (FULL || a < na)
        af[a] = *reinterpret_cast<const u32x4*>(a_ring + a_slot + (kk ? fa_lds1 : fa_lds0) + a * 64 * kARowBytes);
#pragma unroll
    for (int b = 0; b < 2; ++b)
      bf[b] = *reinterpret_cast<const u32x4*>(smem + b_slot + fb_lds + b * 32 * kBRowBytes + kk * 32);
  };
  auto mfma_frags = [&](const u32x4 (&af)[4], const u32x4 (&bf)[2]) {
#pragma unroll
    for (int a = 0; a < 4; ++a)
      if (FULL || a < na) {
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = mfma_bf16(af[a], bf[b], acc[a][b]);
      }
  };

  // ---- prologue: A steps 0..3 on their way, group 0's packed weights in registers, steps 0 and 1 unpacked ----
  load_a(0, 0u);
  load_a(1, kASlotBytes);
  load_a(2, 2 * kASlotBytes);
  load_a(3, 3 * kASlotBytes);
  load_b(0, b_cur_reg);
  load_b_scale(0, b_s0);
  load_m(0, m_next);
  vmem_outstanding_at_most<0>();
#pragma unroll
  for (int j = 0; j < 2; ++j) {
#pragma unroll
    for (int e = 0; e <= P; ++e) settled(b_cur_reg[j][e]), b_nxt_reg[j][e] = b_cur_reg[j][e];
    settled(b_s0[j]);
    settled(m_next[j]);
    m_cur[j] = scale_mantissa(__uint_as_float(m_next[j]));
    b_s0_next[j] = b_s0[j];
  }
  set_b_const(b_s0);
  store_b(0u, 0, 0);
  store_b(kBSlotBytes, 0, 1);
  lds_writes_done();
  wg_barrier();
  // the fragments are needed from here on (full tiles: the compiler waits for their reads at this point)
  auto settle_frags = [&](u32x4 (&af)[4], u32x4 (&bf)[2]) {
    if constexpr (FULL) {
#pragma unroll
      for (int a = 0; a < 4; ++a) touch(af[a]);
      touch(bf[0]);
      touch(bf[1]);
    }
  };
  if (FULL || ORDER == 1) {
    read_frags(0u, 0u, std::integral_constant<int, 0>{}, af0, bf0);
    settle_frags(af0, bf0);
  }
  // ring positions: B slot of step h and of step h + 2; A slot of step h and of step h + 4 (= h - 1)
  uint32_t b_cur = 0u, b_new = 2 * kBSlotBytes;
  uint32_t a_cur = 0u, a_new = 4 * kASlotBytes;
  auto b_after = [](uint32_t x) { return x == 2 * kBSlotBytes ? 0u : x + kBSlotBytes; };
  auto a_after = [](uint32_t x) { return x == 4 * kASlotBytes ? 0u : x + kASlotBytes; };
  // VMEM instructions a wavefront issues in step 4q + i (the two A loads first)
  constexpr int kAll[4] = {2 + 2 * (P + 1) + 4, 2, 2, 2};
  if constexpr (FULL) {
    // ---- full tiles: every wavefront runs the same hand-ordered step; the vector, LDS and memory
    // work of a step is spread between its 16 MFMAs (one scheduling fence per MFMA), so the matrix
    // core issues back to back while the unpack runs in its shadow.  On entry to a step af0/bf0 hold
    // the first half's fragments; the second half's are read under the first eight MFMAs and the
    // next step's first half under the last eight.
#define MBQ_FENCE() __builtin_amdgcn_sched_barrier(0)
    for (int q = 0; q < G; ++q) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int h = 4 * q + i;
        const int set = i < 2 ? 1 : 0, half = i & 1;   // which dword of b_cur and which half of it: step h + 2
        MBQ_FENCE();
        load_a(h + 4, a_new);
        MBQ_FENCE();  // the A loads stay first in the step (vmcnt bookkeeping)
        float ratio[2] = {1.f, 1.f};
        if (i == 0) {
#pragma unroll
          for (int b = 0; b < 2; ++b) {
            const float r = m_cur[b] * __builtin_amdgcn_rcpf(scale_mantissa(__uint_as_float(m_next[b])));
            ratio[b] = (q > 0) ? r : 1.f;
            m_cur[b] = m_cur[b] / ratio[b];
          }
          load_b(q + 1, b_nxt_reg);
          load_b_scale(q + 1, b_s0_next);
          load_m(q + 1, m_next);
        }
        if (i == 2) {
          untracked_loads_outstanding_at_most<kAll[1] + 2>();
#pragma unroll
          for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int e = 0; e <= P; ++e) settled(b_nxt_reg[j][e]), b_cur_reg[j][e] = b_nxt_reg[j][e];
            settled(b_s0_next[j]);
            settled(m_next[j]);
            b_s0[j] = b_s0_next[j];
          }
          set_b_const(b_s0);
        }
        MBQ_FENCE();
        u32x4 af1[4], bf1[2];
        read_frags(a_cur, b_cur, std::integral_constant<int, 1>{}, af1, bf1);
        MBQ_FENCE();
        uint32_t lo[2], hi[2];
        u32x4 v[2];
        // ---- first half: MFMA (a, b), then a piece of the unpack of item j = a / 2 ----
#pragma unroll
        for (int a = 0; a < 4; ++a) {
#pragma unroll
          for (int b = 0; b < 2; ++b) {
            if (i == 0) {
#pragma unroll
              for (int e = 0; e < 16; ++e) acc[a][b][e] *= ratio[b];
            }
            acc[a][b] = mfma_bf16(af0[a], bf0[b], acc[a][b]);
            const int j = a >> 1, piece = 2 * (a & 1) + b;
            if (piece == 0) lo[j] = merge_bits(set, j, half);
            if (piece == 1) hi[j] = merge_bits(set, j, half + 2);
            if (piece == 2) {
              v[j].x = expand_pair(lo[j], j, 0);
              v[j].y = expand_pair(hi[j], j, 0);
              v[j].z = expand_pair(lo[j], j, 1);
              v[j].w = expand_pair(hi[j], j, 1);
            }
            if (piece == 3) write_b(b_new, j, v[j]);
            MBQ_FENCE();
          }
        }
        // the second half's fragments: only the two weight writes were issued after their reads
        settle_frags(af1, bf1);
        MBQ_FENCE();
        read_frags(a_after(a_cur), b_after(b_cur), std::integral_constant<int, 0>{}, af0, bf0);  // step h + 1
        MBQ_FENCE();
#pragma unroll
        for (int a = 0; a < 4; ++a) {
#pragma unroll
          for (int b = 0; b < 2; ++b) {
            acc[a][b] = mfma_bf16(af1[a], bf1[b], acc[a][b]);
            MBQ_FENCE();
          }
        }
        lds_writes_done();  // the weight writes and the fragment reads of the next step
        settle_frags(af0, bf0);
        // the A loads of step h + 2 (issued two steps ago, first in their step) must have landed before
        // the barrier publishes them
        if (i == 0) vmem_outstanding_at_most<(kAll[2] - 2) + kAll[3] + kAll[0]>();
        if (i == 1) vmem_outstanding_at_most<(kAll[3] - 2) + kAll[0] + kAll[1]>();
        if (i == 2) vmem_outstanding_at_most<(kAll[0] - 2) + kAll[1] + kAll[2]>();
        if (i == 3) vmem_outstanding_at_most<(kAll[1] - 2) + kAll[2] + kAll[3]>();
        wg_barrier();
        MBQ_FENCE();
        b_cur = b_after(b_cur);
        b_new = b_after(b_new);
        a_cur = a_after(a_cur);
        a_new = a_after(a_new);
      }
    }
#undef MBQ_FENCE
  } else
  for (int q = 0; q < G; ++q) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int h = 4 * q + i;
      // ---- memory part X of step h: weights of step h + 2 into LDS, loads, accumulator rescale ----
      auto memory_part = [&]() {
        load_a(h + 4, a_new);
        __builtin_amdgcn_sched_barrier(0);  // the A loads stay first in the step (vmcnt bookkeeping)
        if (i == 2) {
          // first use of the next group's packed weights and scales (issued two steps ago): only step
          // 4q+1's and this step's A loads may stay in flight
          vmem_outstanding_at_most<kAll[1] + 2>();
#pragma unroll
          for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int e = 0; e <= P; ++e) settled(b_nxt_reg[j][e]), b_cur_reg[j][e] = b_nxt_reg[j][e];
            settled(b_s0_next[j]);
            settled(m_next[j]);
            b_s0[j] = b_s0_next[j];
          }
          set_b_const(b_s0);
        }
        // step h + 2 = 4q + i + 2: second dword of group q for i = 0, 1; first dword of group q + 1
        // (just moved into b_cur_reg) for i = 2, 3; half i & 1
        store_b(b_new, i < 2 ? 1 : 0, i & 1);
        // the accumulator moves to the next group's scale mantissa between the last MFMA of a group
        // and the first of the next: X comes before Y of the same step for ORDER 0, after it for ORDER 1
        const bool boundary = (ORDER == 0) ? (i == 0) : (i == 3);
        const bool rescale = boundary && ((ORDER == 0) ? (q > 0) : (q + 1 < G));
        float ratio[2] = {1.f, 1.f};
        if (boundary) {
#pragma unroll
          for (int b = 0; b < 2; ++b) {
            const float r = m_cur[b] * __builtin_amdgcn_rcpf(scale_mantissa(__uint_as_float(m_next[b])));
            ratio[b] = rescale ? r : 1.f;      // a select, not a branch: fragment reads may be in flight here
            m_cur[b] = m_cur[b] / ratio[b];    // the factor actually in force (keeps the chain consistent)
          }
        }
        if (i == 0) {
          load_b(q + 1, b_nxt_reg);
          load_b_scale(q + 1, b_s0_next);
          load_m(q + 1, m_next);
        }
        if (boundary) {
#pragma unroll
          for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int a = 0; a < 4; ++a)
              if (FULL || a < na) {
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[a][b][e] *= ratio[b];
              }
        }
        lds_writes_done();  // also the end of any fragment read issued before this part
      };
      // ---- compute part Y of step h: 16 MFMAs; af0/bf0 hold the first half's fragments ----
      auto compute_part = [&]() {
        u32x4 af1[4], bf1[2];
        read_frags(a_cur, b_cur, std::integral_constant<int, 1>{}, af1, bf1);
        __builtin_amdgcn_sched_barrier(0);
        mfma_frags(af0, bf0);
        __builtin_amdgcn_sched_barrier(0);  // the first eight MFMAs are issued before the wait
        settle_frags(af1, bf1);
        mfma_frags(af1, bf1);
      };
      __builtin_amdgcn_sched_barrier(0);
      if (ORDER == 0) {
        read_frags(a_cur, b_cur, std::integral_constant<int, 0>{}, af0, bf0);
        memory_part();
        settle_frags(af0, bf0);
        __builtin_amdgcn_sched_barrier(0);
        compute_part();
      } else {
        compute_part();
        __builtin_amdgcn_sched_barrier(0);
        read_frags(a_after(a_cur), b_after(b_cur), std::integral_constant<int, 0>{}, af0, bf0);  // step h + 1
        memory_part();
        settle_frags(af0, bf0);
      }
      __builtin_amdgcn_sched_barrier(0);
      // the A loads of step h + 2 (issued two steps ago, first in their step) must have landed before
      // the barrier publishes them
      if (i == 0) vmem_outstanding_at_most<(kAll[2] - 2) + kAll[3] + kAll[0]>();
      if (i == 1) vmem_outstanding_at_most<(kAll[3] - 2) + kAll[0] + kAll[1]>();
      if (i == 2) vmem_outstanding_at_most<(kAll[0] - 2) + kAll[1] + kAll[2]>();
      if (i == 3) vmem_outstanding_at_most<(kAll[1] - 2) + kAll[2] + kAll[3]>();
      wg_barrier();
      __builtin_amdgcn_sched_barrier(0);
      b_cur = b_after(b_cur);
      b_new = b_after(b_new);
      a_cur = a_after(a_cur);
      a_new = a_after(a_new);
    }
  }
  vmem_outstanding_at_most<0>();  // clamped loads past the last step: nothing may still write LDS at exit

  // ---- true units, then the zero-point / offset term as a rank-G fp32 MFMA update ----
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const float f = m_cur[b] * (1.f / 64.f);
#pragma unroll
    for (int a = 0; a < 4; ++a)
      if (FULL || a < na) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[a][b][i] *= f;
      }
  }
  {
    constexpr float kC = (kHalf - kOff) * (1.f / 64.f);
    const float* sx_ptr = SxT + row0 + 32 * wm + (lane & 31);
    // operands of one MFMA step (groups g2 and g2 + 1, one per half wavefront); loaded two steps
    // ahead of their use through two register sets
    struct TailOps {
      float2 mt[2];
      float av[4];
    };
    auto fetch = [&](int g2, TailOps& o) {
      const int g = g2 + (lane >> 5);
      const bool valid = g < G;
      const int gc = valid ? g : G - 1;
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const float2 mt = meta[c_meta[b] + (size_t)(g0 + gc) * kTileN];
        o.mt[b] = (valid && c_ok[b]) ? mt : float2{0.f, 0.f};
      }
#pragma unroll
      for (int a = 0; a < 4; ++a)
        if (FULL || a < na) {
          const float v = sx_ptr[(int64_t)(g0 + gc) * ldT + 64 * a];
          o.av[a] = valid ? v : 0.f;
        }
    };
    auto apply = [&](const TailOps& o) {
      float bv[2];
#pragma unroll
      for (int b = 0; b < 2; ++b) bv[b] = o.mt[b].x * (kC - o.mt[b].y);
#pragma unroll
      for (int a = 0; a < 4; ++a)
        if (FULL || a < na) {
#pragma unroll
          for (int b = 0; b < 2; ++b)
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(o.av[a], bv[b], acc[a][b], 0, 0, 0);
        }
    };
    TailOps t0, t1;
    fetch(0, t0);
    if (2 < G) fetch(2, t1);
    for (int g2 = 0; g2 < G; g2 += 4) {
      apply(t0);
      if (g2 + 4 < G) fetch(g2 + 4, t0);
      if (g2 + 2 < G) {
        apply(t1);
        if (g2 + 6 < G) fetch(g2 + 6, t1);
      }
    }
  }

  // ---- write the tile in original token order ----
  // The accumulator layout gives a store instruction 32 consecutive columns of two rows (2 x 128 bytes); 128 such
  // instructions per wavefront cost more address-unit time than their bytes.  When rows can take 16-byte stores the
  // tile goes through LDS once (the rings are free now; 64 x 64 floats per wavefront and half) and leaves as
  // 16 bytes per lane, four rows of 256 bytes per instruction: a quarter of the instructions.
  if (!accumulate && (N & 3) == 0 && (reinterpret_cast<uintptr_t>(Y) & 15) == 0) {
    static_assert(kSmemBytes >= 8 * 64 * 64 * 4, "staging area of the epilogue");
    wg_barrier();  // every wavefront has left the rings
    float* stg = reinterpret_cast<float*>(smem) + wave * (64 * 64);
    const int64_t col4 = (int64_t)ntile_n * kBN + 64 * wn + 4 * (lane & 15);
#pragma unroll
    for (int half = 0; half < 2; ++half) {
#pragma unroll
      for (int aa = 0; aa < 2; ++aa) {
        const int a = 2 * half + aa;
        if (FULL || a < na) {
#pragma unroll
          for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i)
              stg[(32 * aa + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3)) * 64 + 32 * b + (lane & 31)] = acc[a][b][i];
        }
      }
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int rowl = 4 * q + (lane >> 4);  // row of the staged 64
        const int a = 2 * half + (rowl >> 5);
        const int r = 32 * (2 * a + wm) + (rowl & 31);
        if ((FULL || (a < na && r < rows)) && col4 < N) {
          const floatx4 v = *reinterpret_cast<const floatx4*>(stg + rowl * 64 + 4 * (lane & 15));
          const int64_t tok = perm[row0 + r];
          *reinterpret_cast<floatx4*>(Y + tok * N + col4) = v;
        }
      }
    }
    return;
  }
#pragma unroll
  for (int a = 0; a < 4; ++a)
    if (FULL || a < na) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int r = 32 * (2 * a + wm) + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
        if (FULL || r < rows) {
          const int64_t tok = perm[row0 + r];
#pragma unroll
          for (int b = 0; b < 2; ++b)
            if (ncol[b] < N) {
              if (accumulate)
                unsafeAtomicAdd(&Y[tok * N + ncol[b]], acc[a][b][i]);  // K split: Y was zeroed by the pre-kernel
              else
                Y[tok * N + ncol[b]] = acc[a][b][i];
            }
        }
      }
    }
}

__global__ __launch_bounds__(512, 1) void prefill_kernel(const uint16_t* __restrict__ Xs, int64_t K,
                                                         const uint32_t* __restrict__ codes, size_t slice_words,
                                                         const float2* __restrict__ meta, int64_t N, int NT, int KB,
                                                         const int32_t* __restrict__ perm,
                                                         const int32_t* __restrict__ offsets,
                                                         const float* __restrict__ SxT, int64_t ldT,
                                                         float* __restrict__ Y, int n_tiles_n, int splits,
                                                         int mix_gate) {
  __shared__ __attribute__((aligned(1024))) char smem[kSmemBytes];
  if (mix_gate && mix_prefers_stationary(offsets, offsets[MBQ_N_PRECISIONS])) return;  // see prefill_prep_kernel
  // ---- which tile: full tiles of every bucket first, then the ragged last tile of each bucket ----
  // (tile row, tile column, K split): workgroups of one tile row are neighbours (they share activations)
  const int per_mt = n_tiles_n * splits;
  const int mt = blockIdx.x / per_mt, ntile_n = (blockIdx.x % per_mt) / splits, split = blockIdx.x % splits;
  const int Gtot = (int)(K / kGroup);
  const int g0 = (int)((int64_t)split * Gtot / splits);
  const int Gs = (int)((int64_t)(split + 1) * Gtot / splits) - g0;
  int off[MBQ_N_PRECISIONS + 1];
#pragma unroll
  for (int q = 0; q <= MBQ_N_PRECISIONS; ++q) off[q] = offsets[q];
  int p = -1, row0 = 0, rows = 0, idx = mt;
#pragma unroll
  for (int q = 0; q < MBQ_N_PRECISIONS; ++q) {
    const int full = (off[q + 1] - off[q]) / kBM;
    if (p < 0) {
      if (idx < full) {
        p = q;
        row0 = off[q] + idx * kBM;
        rows = kBM;
      } else {
        idx -= full;
      }
    }
  }
#pragma unroll
  for (int q = 0; q < MBQ_N_PRECISIONS; ++q) {
    const int cnt = off[q + 1] - off[q];
    const int rem = cnt % kBM;
    if (p < 0 && rem > 0) {
      if (idx == 0) {
        p = q;
        row0 = off[q] + cnt - rem;
        rows = rem;
      } else {
        --idx;
      }
    }
  }
  if (p < 0) return;
  // wavefronts 0..3 run each step memory part first, wavefronts 4..7 compute part first (wave-uniform branch)
  const bool first_half = __builtin_amdgcn_readfirstlane(threadIdx.x >> 8) == 0;
#define MBQ_TILE(PP, FF)                                                                                       \
  do {                                                                                                         \
    if (FF || first_half)                                                                                      \
      prefill_tile<PP, FF, 0>(Xs, K, codes, slice_words, meta, N, NT, KB, perm, SxT, ldT, Y, row0, rows,        \
                              ntile_n, smem, g0, Gs, splits > 1);                                              \
    else                                                                                                       \
      prefill_tile<PP, FF, 1>(Xs, K, codes, slice_words, meta, N, NT, KB, perm, SxT, ldT, Y, row0, rows,        \
                              ntile_n, smem, g0, Gs, splits > 1);                                              \
  } while (0)
  if (rows == kBM) {
    switch (p) {
      case 0: MBQ_TILE(0, true); break;
      case 1: MBQ_TILE(1, true); break;
      case 2: MBQ_TILE(2, true); break;
      default: MBQ_TILE(3, true); break;
    }
  } else {
    switch (p) {
      case 0: MBQ_TILE(0, false); break;
      case 1: MBQ_TILE(1, false); break;
      case 2: MBQ_TILE(2, false); break;
      default: MBQ_TILE(3, false); break;
    }
  }
#undef MBQ_TILE
}

static inline int64_t prefill_ld(int64_t T) { return (T + 32 + 63) / 64 * 64; }

size_t prefill_workspace_bytes(int64_t T, const Shape& sh) {
  const size_t xs = (size_t)(T + kPadRows) * sh.K * sizeof(uint16_t);
  const size_t sx = (size_t)sh.G * prefill_ld(T) * sizeof(float);
  return xs + sx + 256;
}

mbq_status launch_linear_prefill(const uint16_t* X, int64_t T, const void* blob, const Shape& sh,
                                 const int32_t* perm, const int32_t* offsets, float* Y, void* ws,
                                 hipStream_t stream, bool mix_gate) {
  const uint32_t* codes = reinterpret_cast<const uint32_t*>(blob);
  const float2* meta = reinterpret_cast<const float2*>(reinterpret_cast<const char*>(blob) + sh.meta_offset);
  uint16_t* Xs = reinterpret_cast<uint16_t*>(ws);
  const size_t xs_bytes = ((size_t)(T + kPadRows) * sh.K * sizeof(uint16_t) + 255) / 256 * 256;
  float* SxT = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + xs_bytes);
  const int64_t ldT = prefill_ld(T);
  const int n_tiles_n = (int)((sh.N + kBN - 1) / kBN);
  const int64_t m_tiles_max = T / kBM + MBQ_N_PRECISIONS;
  // K split: a launch with few tiles leaves compute units idle in its last round (a tile of K = 4096 holds its
  // compute unit for about 110 us however few tiles there are), so tiles are cut along K into S workgroups that add
  // their partial sums into a zeroed Y.  S (1..6) minimises the estimated makespan ceil(tiles S / compute units) / S,
  // each further part priced at 5 % of a tile of K = 11008 (its prologue, its atomic adds: a fixed cost, so the
  // price grows as K shrinks; measured on 4096 x 11008, 8192 x 28672, and on 4096 x 4096 .. 8192 x 4096 at 192..512
  // tokens).  Tile rows: the full ones plus one ragged row per bucket, at least four.  knob 5 forces the split (1..8).
  constexpr int kComputeUnits = 256;
  int splits = 1;
  if (knob(5) >= 1 && knob(5) <= 8) {
    splits = knob(5);
  } else {
    const int64_t est_rows = (T / kBM + 2 > 4) ? T / kBM + 2 : 4;
    const int64_t est_tiles = est_rows * n_tiles_n;
    const double per_part = 0.05 * 11008.0 / (double)sh.K;
    double best = 0.0;
    for (int s = 1; s <= 6; ++s) {
      const int64_t rounds = (est_tiles * s + kComputeUnits - 1) / kComputeUnits;
      const double cost = (double)rounds / s * (1.0 + per_part * (s - 1));
      if (s == 1 || cost < best) {
        best = cost;
        splits = s;
      }
    }
  }
  while (splits > 1 && sh.G / splits < 4) --splits;
  hipLaunchKernelGGL(prefill_prep_kernel, dim3((unsigned)T), dim3(256), 0, stream, X, T, sh.K, perm, Xs, SxT, ldT,
                     splits > 1 ? Y : nullptr, sh.N, mix_gate ? offsets : nullptr);
  mbq_status st = hip_status(hipGetLastError(), "prefill_prep_kernel launch");
  if (st != MBQ_OK) return st;
  hipLaunchKernelGGL(prefill_kernel, dim3((unsigned)(m_tiles_max * n_tiles_n * splits)), dim3(512), 0, stream, Xs,
                     sh.K, codes, sh.slice_words, meta, sh.N, sh.NT, sh.KB, perm, offsets, SxT, ldT, Y, n_tiles_n,
                     splits, mix_gate ? 1 : 0);
  return hip_status(hipGetLastError(), "prefill_kernel launch");
}

}  // namespace mbq
