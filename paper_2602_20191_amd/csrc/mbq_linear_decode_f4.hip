// Decode-side routed linear for one token tile (T <= 16) and up to MBQ_MAX_GROUP
// weight matrices that read the SAME activations: the 2-bit codes go to the matrix cores as FP4.
//
// Paper Sec. 4.2 Eq. 6 evaluated slice by slice, Y_i = sum_{e <= p_i} W_e^T X_i, with the
// shared-scale structure of App. B (s_e = s0/4^e, z_e = 2 for e >= 1); a tile fetches only
// slices 0..max_i p_i of its own matrix (Sec. 4.3, on-demand slice access), and the matrices of
// one call share one launch and one pass over the activations (Sec. 4.3, fused launch for the
// projections of a layer).
//
// Arithmetic.  A 2-bit code c zero-extended to four bits IS the FP4 (E2M1) number c/2, so a
// packed dword turns into MFMA operands with a rotate and a mask per eight codes.  The bf16
// activations are split once, by a small preparation kernel, into two FP8 (E4M3) pieces
// x = x1 + x2 / 16 (x1 the round-to-nearest of x, x2 that of 16 (x - x1); four significant bits
// each), after a power-of-two scale per (token, 256-column block) that puts the block's largest
// element just below 2^8: the split is exact for every element within 13 binades of that largest
// element and off by at most 2^-21 of it below.  Every product piece x code is exact and
// v_mfma_scale_f32_16x16x128_f8f6f4 accumulates in fp32.  Its per-lane block scales do the rest of
// the bookkeeping at no cost:
//   - the B scale of slice e is 2^(1-2e): the operand c/2 counts as c / 4^e;
//   - the A scale byte of token i and slice e undoes the block scale (times 2^-4 for the second
//     piece) when e <= p_i and is 2^-127 otherwise, so one accumulator chain over the slices yields
//     sum_{e<=p_i} for every token at once (the leak of a masked slice is below 2^-100 of the output).
// With D that chain and Sx the group sum of x,
//   y += s0 * (D + (0.5 - 1.5 q_p - z0) Sx),   q_p = sum_{1 <= e <= p} 4^-e.
//
// Work split: the 16-row code tiles of all matrices form one list; a workgroup of 8 wavefronts
// owns tiles blockIdx.x, blockIdx.x + gridDim.x, ...  A wavefront owns two 256-column blocks of
// every tile (K <= 4096) and keeps their activation pieces in registers for the whole kernel, so
// only packed weights stream; they travel through a per-wavefront ring in LDS that the memory
// system fills directly (see decode_f4_ring_kernel).  The load count per block is fixed (a slice
// that the tile does not need is replaced by a load of one fixed KiB that stays in the vector
// cache), so the wavefront can count its own outstanding loads.
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
  unsigned long long* stamps;  // timeline build of the kernel only (see decode_f4_ring_kernel): where the stamps go
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

struct Item {  // one 16 x 256 block: four slices and the {s0, z0} of its two groups
  uint4 w[4];
  float2 mt[2];
};

}  // namespace f4

// ---- the same kernel with the packed weights in flight in LDS instead of registers -------------
// A load that is in flight to a register pins that register, and the register file (activation
// pieces + one tile being consumed + one arriving) allows one tile ahead: 64 KiB per compute unit,
// too little to cover the memory latency at 8 TB/s.  Here each wavefront owns a ring of kRingDepth
// slots in LDS and asks the memory system to write the 16 x 256 blocks ("items": four slices of
// 1 KiB + the 256 bytes of {s0, z0}) straight into them (global_load_lds), kRingDepth items ahead;
// an item is copied to registers just before it is consumed, and its slot is handed to the item
// kRingDepth further on.  Slots are private to a wavefront, so no barrier guards them; the wavefront
// counts its own outstanding loads (they complete in issue order; a younger store or load in the
// count only makes a wait stricter).
namespace f4 {
constexpr int kRingDepth = 4;
constexpr int kLoadsPerItem = 5;                // 4 slices (16 bytes per lane) + 1 meta (4 bytes per lane)
constexpr int kSlotBytes = 4 * 1024 + 256;

__device__ __forceinline__ void to_lds_16(const void* gptr, char* lds_base) {
  __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)gptr,
                                   (void __attribute__((address_space(3)))*)lds_base, 16, 0, 2);
}
__device__ __forceinline__ void to_lds_4(const void* gptr, char* lds_base) {
  __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)gptr,
                                   (void __attribute__((address_space(3)))*)lds_base, 4, 0, 2);
}
// wait until at most `items_behind` later items are still on their way
__device__ __forceinline__ void ring_wait(int items_behind) {
  if (items_behind >= 3) asm volatile("s_waitcnt vmcnt(15)" ::: "memory");
  else if (items_behind == 2) asm volatile("s_waitcnt vmcnt(10)" ::: "memory");
  else if (items_behind == 1) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}
// One item from its slot to registers.  Written as one asm block (reads + their wait) for two
// reasons: the compiler orders every LDS read it knows about after ALL outstanding loads into LDS,
// which would drain the ring; and no register is visible to it while its read is in flight.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void read_slot(uint32_t lane_addr, uint32_t row_addr, u32x4 (&w)[4], f32x2 (&mt)[2]) {
  asm volatile(
      "ds_read_b128 %0, %6\n\t"
      "ds_read_b128 %1, %6 offset:1024\n\t"
      "ds_read_b128 %2, %6 offset:2048\n\t"
      "ds_read_b128 %3, %6 offset:3072\n\t"
      "ds_read_b64 %4, %7 offset:4096\n\t"
      "ds_read_b64 %5, %7 offset:4224\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(w[0]), "=&v"(w[1]), "=&v"(w[2]), "=&v"(w[3]), "=&v"(mt[0]), "=&v"(mt[1])
      : "v"(lane_addr), "v"(row_addr)
      : "memory");
}
// the eight wavefronts' partial sums of one output (1 KiB apart), same reasons
__device__ __forceinline__ float read_partials_sum(uint32_t addr) {
  float v[8];
  asm volatile(
      "ds_read_b32 %0, %8\n\t"
      "ds_read_b32 %1, %8 offset:1024\n\t"
      "ds_read_b32 %2, %8 offset:2048\n\t"
      "ds_read_b32 %3, %8 offset:3072\n\t"
      "ds_read_b32 %4, %8 offset:4096\n\t"
      "ds_read_b32 %5, %8 offset:5120\n\t"
      "ds_read_b32 %6, %8 offset:6144\n\t"
      "ds_read_b32 %7, %8 offset:7168\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7])
      : "v"(addr)
      : "memory");
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) sum += v[i];
  return sum;
}
// workgroup barrier that orders LDS traffic only (the loads into the ring stay in flight across it)
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
// wait until at most `kLater` younger loads are outstanding; the four registers, written by loads
// that the compiler does not know about, may be looked at only after this
template <int kLater>
__device__ __forceinline__ void loads_arrived(int& a, int& b, int& c, int& d) {
  asm volatile("s_waitcnt vmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(kLater) : "memory");
}
static_assert(kPieces == 2, "slice_group picks the scale of a piece by piece == 0");
static_assert(kRingDepth == 4 && kLoadsPerItem == 5, "ring_wait's constants are (kRingDepth - 1 .. 0) * kLoadsPerItem");
}  // namespace f4

// kStamp: the timeline build.  Lane 0 of every wavefront notes the 100 MHz wall clock at the phase boundaries in LDS
// and the workgroup copies the notes to g.stamps when it is done: slot 0 entry, 1 precisions here, 2 first item
// requested, 3 activations and first item here, 4 + 2 i tile i's MFMAs done, 5 + 2 i tile i's outputs stored,
// kStampSlots - 2 end, kStampSlots - 1 the hardware id word (which XCD / compute unit ran the workgroup).
namespace f4 {
constexpr int kStampSlots = 32;
}
template <int CPW, int S, bool kStamp = false>
__global__ __launch_bounds__(512) void decode_f4_ring_kernel(const char* __restrict__ prep, int T, int KB,
                                                             const f4::Group g) {
  using namespace f4;
  constexpr int kWaves = 8;
  __shared__ unsigned long long s_stamp[kStamp ? kWaves * kStampSlots : 1];
  const uint32_t stamp_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)&s_stamp[0] +
                              (uint32_t)(__builtin_amdgcn_readfirstlane(threadIdx.x >> 6) * kStampSlots * 8);
  auto stamp = [&](int slot) {
    if constexpr (kStamp) {
      if (slot < kStampSlots - 2 && (threadIdx.x & 63) == 0) {
        const unsigned long long now = __builtin_amdgcn_s_memrealtime();
        asm volatile("ds_write_b64 %0, %1" ::"v"(stamp_addr + (uint32_t)slot * 8u), "v"(now) : "memory");
      }
    }
  };
  if constexpr (kStamp) {
    for (int i = threadIdx.x; i < kWaves * kStampSlots; i += 512) s_stamp[i] = 0ull;
    __syncthreads();
  }
  stamp(0);
  constexpr int kXaLoads = 2 * kPieces * 2 + 2 + 1;  // loads of one block's prepared activations
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m = lane & 15;
  const int kq = lane >> 4;
  // S = 2: the K axis is cut in two parts of 8 CPW blocks; workgroups 2 r and 2 r + 1 take the two parts
  // of the same tiles and add their results into a Y that the preparation launch has zeroed (two
  // addends: the sum does not depend on who comes first).  Each compute unit then fetches half of the
  // prepared activations, which it would otherwise pull through the same port as the weights.
  static_assert(S == 1 || S == 2, "one or two parts");
  const int part = (int)blockIdx.x % S;
  const int bid = (int)blockIdx.x / S;        // position in the tile list
  const int stride = (int)gridDim.x / S;      // the launcher makes gridDim.x a multiple of S
  const int my_tiles = (g.tiles - bid + stride - 1) / stride;
  if (my_tiles <= 0) return;
  const int total = my_tiles * CPW;  // items of this wavefront: (tile index q / CPW, chunk q % CPW)
  // This wavefront's 256-column blocks are blk0 and blk0 + 8.  The assignment rotates with the
  // workgroup so that the compute units of one XCD, which all start by fetching the prepared
  // activations of their blocks, do not all ask the L2 for the same lines at the same moment.
  const int rot = (wave + bid) & (kWaves - 1);
  const int blk0 = part * (kWaves * CPW) + rot;

  __shared__ __attribute__((aligned(1024))) char ring[kWaves * kRingDepth * kSlotBytes];
  __shared__ float red[2][kWaves][64][4];
  char* const my_ring = ring + wave * (kRingDepth * kSlotBytes);
  const uint32_t red_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)&red[0][0][0][0];
  const uint32_t my_ring_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)my_ring;

  const uint4* dummy = reinterpret_cast<const uint4*>(prep);  // 1 KiB that stays in the vector cache
  // The per-matrix facts live in scalar registers for the whole kernel (pinned: left to itself the
  // compiler re-reads them from the argument block in every tile, a chain of scalar-load round trips
  // that costs more than the tile's MFMAs).
  const uint4* m_codes[MBQ_MAX_GROUP];
  const float2* m_meta[MBQ_MAX_GROUP];
  float* m_Y[MBQ_MAX_GROUP];
  size_t m_slice_vec[MBQ_MAX_GROUP];
  int m_N[MBQ_MAX_GROUP], m_begin[MBQ_MAX_GROUP];
#pragma unroll
  for (int i = 0; i < MBQ_MAX_GROUP; ++i) {
    m_codes[i] = g.p[i].codes;
    m_meta[i] = g.p[i].meta;
    m_Y[i] = g.p[i].Y;
    m_slice_vec[i] = g.p[i].slice_vec;
    m_N[i] = (int)g.p[i].N;
    m_begin[i] = i < g.n ? g.p[i].tile_begin : 0x7fffffff;  // unused slots are never reached
    asm volatile("" : "+s"(m_codes[i]), "+s"(m_meta[i]), "+s"(m_Y[i]), "+s"(m_slice_vec[i]), "+s"(m_N[i]), "+s"(m_begin[i]));
  }
  auto proj_of = [&](int t) {
    int j = 0;
#pragma unroll
    for (int i = 1; i < MBQ_MAX_GROUP; ++i)
      if (t >= m_begin[i]) j = i;
    return j;
  };
#define MBQ_PICK(arr, j) ((j) == 0 ? arr[0] : (j) == 1 ? arr[1] : (j) == 2 ? arr[2] : arr[3])
  // request item q (q < total) with slices 0..pm
  auto request = [&](int q, int pm) {
    const int t = bid + (q / CPW) * stride;
    int kb = blk0 + kWaves * (q % CPW);
    if (kb >= KB) kb = 0;  // a block past the end: its activations are zeros, any weights will do
    const int j = proj_of(t);
    const uint4* codes = MBQ_PICK(m_codes, j);
    const size_t slice_vec = MBQ_PICK(m_slice_vec, j);
    const int nt = t - MBQ_PICK(m_begin, j);
    char* slot = my_ring + (q % kRingDepth) * kSlotBytes;
    const size_t tile = ((size_t)nt * KB + kb) * 64 + lane;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint4* src = (e <= pm) ? codes + ((size_t)e * slice_vec + tile) : dummy + lane;
      to_lds_16(src, slot + e * 1024);
    }
    to_lds_4(reinterpret_cast<const char*>(MBQ_PICK(m_meta, j) + ((size_t)nt * (2 * KB) + 2 * kb) * kTileN) + 4 * lane,
             slot + 4096);
  };

  // Every load of the prologue is hidden from the compiler (it orders each wait of its own after ALL
  // loads into LDS, which would serialise the prologue); the registers they write are looked at only
  // after the hand-counted waits below, and only straight-line code lies between a load and its wait.
  //   precisions of every matrix: no branch on g.n (an unused slot of g repeats matrix 0 and its result
  //   is never looked at); lanes past T are set to -1 in find_pmax
  int pl[MBQ_MAX_GROUP];
  auto load_precisions = [&]() {
#pragma unroll
    for (int j = 0; j < MBQ_MAX_GROUP; ++j)
      asm volatile("global_load_dword %0, %1, off" : "=v"(pl[j]) : "v"(g.p[j].prec + (lane < T ? lane : 0)) : "memory");
  };
  //   prepared activations of this wavefront's blocks (kept in registers throughout); a block past the
  //   end reads block 0 and is zeroed after the wait
  u32x4 xa_raw[CPW][2][kPieces][2];
  floatx4 sx[CPW][2];
  int tok_scale[CPW];
  auto load_activations = [&](int c) {
    const int kb = blk0 + kWaves * c;
    const char* base = prep + (size_t)(kb < KB ? kb : 0) * kPrepBytesPerBlock;
    const char* lane_vec = base + (size_t)lane * 16;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int piece = 0; piece < kPieces; ++piece) {
        const char* src = lane_vec + (size_t)(h * kPieces + piece) * 2048;
        asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(xa_raw[c][h][piece][0]) : "v"(src) : "memory");
        asm volatile("global_load_dwordx4 %0, %1, off offset:1024" : "=v"(xa_raw[c][h][piece][1]) : "v"(src) : "memory");
      }
      asm volatile("global_load_dwordx4 %0, %1, off"
                   : "=v"(sx[c][h]) : "v"(base + kPrepVecPerBlock * 16 + (16 * h + 4 * kq) * 4) : "memory");
    }
    asm volatile("global_load_dword %0, %1, off"
                 : "=v"(tok_scale[c]) : "v"(base + kPrepVecPerBlock * 16 + 2 * 16 * 4 + 4 * m) : "memory");
  };

  // Routing facts: highest precision present per matrix.
  int pmax[MBQ_MAX_GROUP];
  auto find_pmax = [&]() {
#pragma unroll
    for (int j = 0; j < MBQ_MAX_GROUP; ++j) pl[j] = lane < T ? pl[j] : -1;
#pragma unroll
    for (int j = 0; j < MBQ_MAX_GROUP; ++j)
      pmax[j] = (__ballot(pl[j] == 3) != 0ull) ? 3 : (__ballot(pl[j] == 2) != 0ull) ? 2 : (__ballot(pl[j] == 1) != 0ull) ? 1 : 0;
  };
  auto pmax_of = [&](int j) { return j == 0 ? pmax[0] : j == 1 ? pmax[1] : j == 2 ? pmax[2] : pmax[3]; };
  auto request_routed = [&](int q) { request(q, pmax_of(proj_of(bid + (q / CPW) * stride))); };

  // Order of the prologue: precisions, then the activations, then (once the precisions are here) the
  // first tile.  Only the first tile is requested before the loop: the memory pipeline of the compute
  // unit serves requests in order, and what the first MFMAs need should not queue behind prefetches.
  // The loop then fills the ring.
  load_precisions();
#pragma unroll
  for (int c = 0; c < CPW; ++c) load_activations(c);
  loads_arrived<CPW * kXaLoads>(pl[0], pl[1], pl[2], pl[3]);
  stamp(1);
  find_pmax();
  for (int q = 0; q < CPW; ++q) request_routed(q);
  int next_request = CPW;
  stamp(2);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the activations (and the first tile) have arrived
  stamp(3);
  intx8 xa[CPW][2][kPieces];
#pragma unroll
  for (int c = 0; c < CPW; ++c) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int piece = 0; piece < kPieces; ++piece) {
        asm volatile("" : "+v"(xa_raw[c][h][piece][0]), "+v"(xa_raw[c][h][piece][1]));
        const u32x4 lo = xa_raw[c][h][piece][0], hi = xa_raw[c][h][piece][1];
        xa[c][h][piece] = intx8{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
      }
      asm volatile("" : "+v"(sx[c][h]));
    }
    asm volatile("" : "+v"(tok_scale[c]));
    if (blk0 + kWaves * c >= KB) {
      tok_scale[c] = 0;
      sx[c][0] = floatx4{0.f, 0.f, 0.f, 0.f};
      sx[c][1] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
  }

  // per matrix: the A scale gate of this lane's token (row m of the A operand: slice e counts iff
  // e <= its precision) and 0.5 - 1.5 q_p of the output rows 4 kq + i
  uint32_t m_gate[MBQ_MAX_GROUP];
  floatx4 m_kp[MBQ_MAX_GROUP];
#pragma unroll
  for (int jj = 0; jj < MBQ_MAX_GROUP; ++jj) {
    const int pa = __shfl(pl[jj], m, 64);
    m_gate[jj] = (pa >= 3) ? 0xFFFFFFFFu : (pa == 2) ? 0x00FFFFFFu : (pa == 1) ? 0x0000FFFFu : (pa == 0) ? 0x000000FFu : 0u;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int p = __shfl(pl[jj], 4 * kq + i, 64);
      m_kp[jj][i] = (p >= 3) ? 0.0078125f : (p == 2) ? 0.03125f : (p == 1) ? 0.125f : 0.5f;
    }
  }

  if (blockIdx.x == 0 && wave == 0) {  // one wavefront of the launch sorts the tokens, where the caller wants them sorted
#pragma unroll
    for (int j = 0; j < MBQ_MAX_GROUP; ++j)
      if (j < g.n && g.p[j].perm != nullptr) bucket_by_wave(pl[j], lane, g.p[j].perm, g.p[j].offsets);
  }

  uint32_t nib_mask = 0x33333333u;
  asm volatile("" : "+s"(nib_mask));  // keep the mask in a register: one v_and_b32 per operand dword
  const int sb = 0x7A7C7E80;          // B scale bytes 2^(1-2e), e = 0..3
  const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};

#pragma unroll 1
  for (int ti = 0; ti < my_tiles; ++ti) {
    const int t = bid + ti * stride;
    const int j = proj_of(t);
    const int pm = pmax_of(j);
    const uint32_t gate = MBQ_PICK(m_gate, j);
    float kp[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) kp[i] = MBQ_PICK(m_kp, j)[i];
    floatx4 acc = zero4;
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
      const int q = ti * CPW + c;
      const uint32_t slot = my_ring_addr + (uint32_t)((q % kRingDepth) * kSlotBytes);
      ring_wait(min(next_request, total) - 1 - q);  // items q + 1 .. next_request - 1 may still be on their way
      u32x4 wv[4];
      f32x2 mv[2];
      read_slot(slot + lane * 16, slot + m * 8, wv, mv);
      // The slot has been read: items up to q + kRingDepth fit in the ring.  At most two requests per
      // item: the ring fills over the first steps instead of holding the first MFMAs back behind a burst
      // of loads (a wavefront issues in order).
#pragma unroll
      for (int r = 0; r < 2; ++r)
        if (next_request <= q + kRingDepth && next_request < total) request_routed(next_request++);
      Item I;
#pragma unroll
      for (int e = 0; e < 4; ++e) I.w[e] = uint4{wv[e].x, wv[e].y, wv[e].z, wv[e].w};
      I.mt[0] = float2{mv[0].x, mv[0].y};
      I.mt[1] = float2{mv[1].x, mv[1].y};

      const int sa = (int)(((uint32_t)tok_scale[c] * 0x01010101u) & gate);
      const int sa2 = (int)(((uint32_t)max(tok_scale[c] - kPieceShift, 0) * 0x01010101u) & gate);  // second piece is stored 2^kPieceShift times larger
      floatx4 D0, D1;
      if (pm >= 3) {
        // all four slices (the usual case at 16 tokens) as one straight run of code: the operands of a slice
        // are then built while the MFMAs of the slice before occupy the matrix core
        D0 = slice_group<0>(xa[c][0], I.w[0].x, I.w[0].y, nib_mask, sa, sa2, sb, zero4);
        D1 = slice_group<0>(xa[c][1], I.w[0].z, I.w[0].w, nib_mask, sa, sa2, sb, zero4);
        D0 = slice_group<1>(xa[c][0], I.w[1].x, I.w[1].y, nib_mask, sa, sa2, sb, D0);
        D1 = slice_group<1>(xa[c][1], I.w[1].z, I.w[1].w, nib_mask, sa, sa2, sb, D1);
        D0 = slice_group<2>(xa[c][0], I.w[2].x, I.w[2].y, nib_mask, sa, sa2, sb, D0);
        D1 = slice_group<2>(xa[c][1], I.w[2].z, I.w[2].w, nib_mask, sa, sa2, sb, D1);
        D0 = slice_group<3>(xa[c][0], I.w[3].x, I.w[3].y, nib_mask, sa, sa2, sb, D0);
        D1 = slice_group<3>(xa[c][1], I.w[3].z, I.w[3].w, nib_mask, sa, sa2, sb, D1);
#pragma unroll
        for (int k = 0; k < 16; ++k) {  // scheduling hint: one MFMA, then three vector instructions, sixteen times
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
        }
      } else {
        D0 = slice_group<0>(xa[c][0], I.w[0].x, I.w[0].y, nib_mask, sa, sa2, sb, zero4);
        D1 = slice_group<0>(xa[c][1], I.w[0].z, I.w[0].w, nib_mask, sa, sa2, sb, zero4);
        if (pm >= 1) {
          D0 = slice_group<1>(xa[c][0], I.w[1].x, I.w[1].y, nib_mask, sa, sa2, sb, D0);
          D1 = slice_group<1>(xa[c][1], I.w[1].z, I.w[1].w, nib_mask, sa, sa2, sb, D1);
        }
        if (pm >= 2) {
          D0 = slice_group<2>(xa[c][0], I.w[2].x, I.w[2].y, nib_mask, sa, sa2, sb, D0);
          D1 = slice_group<2>(xa[c][1], I.w[2].z, I.w[2].w, nib_mask, sa, sa2, sb, D1);
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[i] += I.mt[0].x * (D0[i] + (kp[i] - I.mt[0].y) * sx[c][0][i]);
        acc[i] += I.mt[1].x * (D1[i] + (kp[i] - I.mt[1].y) * sx[c][1][i]);
      }
    }
    // sum the wavefronts' partial tiles; rows leave in token order
    const int buf = ti & 1;
    if constexpr (kStamp) {
      asm volatile("" ::"v"(acc[0]), "v"(acc[1]), "v"(acc[2]), "v"(acc[3]));
      stamp(4 + 2 * ti);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) red[buf][rot][lane][i] = acc[i];  // filed by block, so the sum below does not depend on the rotation
    lds_barrier();
    if (threadIdx.x < 256) {
      float* Yj = MBQ_PICK(m_Y, j);
      const int Nj = MBQ_PICK(m_N, j);
      const int r = threadIdx.x >> 4, cc = threadIdx.x & 15;
      const int col = (t - MBQ_PICK(m_begin, j)) * kTileN + cc;
      const float sum = read_partials_sum(red_addr + (uint32_t)(buf * (kWaves * 1024) + (16 * (r >> 2) + cc) * 16 + (r & 3) * 4));
      if (r < T && col < Nj) {
        if constexpr (S == 1) Yj[(int64_t)r * Nj + col] = sum;
        else unsafeAtomicAdd(&Yj[(int64_t)r * Nj + col], sum);
      }
    }
    stamp(5 + 2 * ti);
  }
  if constexpr (kStamp) {
    if (lane == 0) {
      s_stamp[wave * kStampSlots + kStampSlots - 2] = __builtin_amdgcn_s_memrealtime();
      s_stamp[wave * kStampSlots + kStampSlots - 1] =
          ((unsigned long long)__builtin_amdgcn_s_getreg(20 | (0 << 6) | (31 << 11)) << 32) |  // XCC_ID
          (unsigned long long)__builtin_amdgcn_s_getreg(4 | (0 << 6) | (31 << 11));             // HW_ID
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kWaves * kStampSlots; i += 512)
      g.stamps[(size_t)blockIdx.x * (kWaves * kStampSlots) + i] = s_stamp[i];
  }
}
#undef MBQ_PICK


// K > 4096: the activation pieces no longer fit in registers next to two weight buffers, so
// they are streamed like the weights (they stay in L2: 12 KiB per block against 4.3 KiB of packed
// weights from HBM).  Wavefront w walks over blocks w, w + 8, ... of a tile and over the
// workgroup's tiles as ONE sequence of (tile, block) items, always fetching the next item before
// consuming the current one; its partial tile stays in registers until the tile's last block, then
// the eight partial tiles are summed through LDS.
namespace f4 {
struct StreamItem {
  intx8 xa[2][kPieces];
  floatx4 sx[2];
  int scale;
  Item w;
};
}  // namespace f4

__global__ __launch_bounds__(512) void decode_f4_stream_kernel(const char* __restrict__ prep, int T, int KB,
                                                               const f4::Group g) {
  using namespace f4;
  constexpr int kWaves = 8;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m = lane & 15, kq = lane >> 4;
  const int my_tiles = (g.tiles - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
  if (my_tiles <= 0) return;
  const int nblk = (KB - wave + kWaves - 1) / kWaves;  // >= 2 here (KB > 16)

  __shared__ float red[2][kWaves][64][4];

  int pl[MBQ_MAX_GROUP];
#pragma unroll
  for (int j = 0; j < MBQ_MAX_GROUP; ++j) pl[j] = (j < g.n && lane < T) ? g.p[j].prec[lane] : -1;

  const uint4* dummy = reinterpret_cast<const uint4*>(prep);
  auto proj_of = [&](int t) {
    int j = 0;
#pragma unroll
    for (int i = 1; i < MBQ_MAX_GROUP; ++i)
      if (i < g.n && t >= g.p[i].tile_begin) j = i;
    return j;
  };
  // everything of item (tile t, block kb) except slices 1..3
  auto load_first = [&](int t, int kb, StreamItem& I) {
    const char* base = prep + (size_t)kb * kPrepBytesPerBlock;
    const uint4* src = reinterpret_cast<const uint4*>(base);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int piece = 0; piece < kPieces; ++piece) {
        const uint4 lo = src[(size_t)(h * kPieces + piece) * 128 + lane];
        const uint4 hi = src[(size_t)(h * kPieces + piece) * 128 + 64 + lane];
        I.xa[h][piece] = intx8{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
      }
      I.sx[h] = *reinterpret_cast<const floatx4*>(base + kPrepVecPerBlock * 16 + (16 * h + 4 * kq) * 4);
    }
    I.scale = reinterpret_cast<const int*>(base + kPrepVecPerBlock * 16 + 2 * 16 * 4)[m];
    const Proj& P = g.p[proj_of(t)];
    const int nt = t - P.tile_begin;
    I.w.w[0] = load_once(P.codes + ((size_t)nt * KB + kb) * 64 + lane);
    I.w.mt[0] = P.meta[((size_t)nt * (2 * KB) + 2 * kb) * kTileN + m];
    I.w.mt[1] = P.meta[((size_t)nt * (2 * KB) + 2 * kb + 1) * kTileN + m];
  };
  auto load_rest = [&](int t, int kb, int pm, StreamItem& I) {
    const Proj& P = g.p[proj_of(t)];
    const int nt = t - P.tile_begin;
    const size_t tile = ((size_t)nt * KB + kb) * 64 + lane;
#pragma unroll
    for (int e = 1; e < 4; ++e) {
      const uint4* src = (e <= pm) ? P.codes + ((size_t)e * P.slice_vec + tile) : dummy + lane;
      I.w.w[e] = load_once(src);
    }
  };
  StreamItem A, B;
  load_first((int)blockIdx.x, wave, A);

  int pmax[MBQ_MAX_GROUP];
#pragma unroll
  for (int j = 0; j < MBQ_MAX_GROUP; ++j)
    pmax[j] = (__ballot(pl[j] == 3) != 0ull) ? 3 : (__ballot(pl[j] == 2) != 0ull) ? 2 : (__ballot(pl[j] == 1) != 0ull) ? 1 : 0;
  auto pmax_of = [&](int j) { return j == 0 ? pmax[0] : j == 1 ? pmax[1] : j == 2 ? pmax[2] : pmax[3]; };
  load_rest((int)blockIdx.x, wave, pmax_of(proj_of((int)blockIdx.x)), A);
  if (blockIdx.x == 0 && wave == 0) {
#pragma unroll
    for (int j = 0; j < MBQ_MAX_GROUP; ++j)
      if (j < g.n && g.p[j].perm != nullptr) bucket_by_wave(pl[j], lane, g.p[j].perm, g.p[j].offsets);
  }

  uint32_t nib_mask = 0x33333333u;
  asm volatile("" : "+s"(nib_mask));
  const int sb = 0x7A7C7E80;
  const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};
  floatx4 acc = zero4;

  // item (ti, b): tile index in this workgroup's list, block index in this wavefront's list
  auto item = [&](int ti, int b, StreamItem& cu, StreamItem& nx) {
    // next item: same tile, next block; or first block of the next tile; the last item refetches itself
    int tin = ti, bn = b + 1;
    if (bn == nblk) {
      bn = 0;
      tin = ti + 1;
    }
    if (tin == my_tiles) {
      tin = ti;
      bn = b;
    }
    const int tn = (int)blockIdx.x + tin * (int)gridDim.x;
    load_first(tn, wave + kWaves * bn, nx);
    load_rest(tn, wave + kWaves * bn, pmax_of(proj_of(tn)), nx);

    const int t = (int)blockIdx.x + ti * (int)gridDim.x;
    const int j = proj_of(t);
    const int pm = pmax_of(j);
    const int plv = j == 0 ? pl[0] : j == 1 ? pl[1] : j == 2 ? pl[2] : pl[3];
    const int pa = __shfl(plv, m, 64);
    const uint32_t gate = (pa >= 3) ? 0xFFFFFFFFu : (pa == 2) ? 0x00FFFFFFu : (pa == 1) ? 0x0000FFFFu
                          : (pa == 0) ? 0x000000FFu : 0u;
    float kp[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int p = __shfl(plv, 4 * kq + i, 64);
      kp[i] = (p >= 3) ? 0.0078125f : (p == 2) ? 0.03125f : (p == 1) ? 0.125f : 0.5f;
    }
    const Item& I = cu.w;
    const int sa = (int)(((uint32_t)cu.scale * 0x01010101u) & gate);
    const int sa2 = (int)(((uint32_t)max(cu.scale - kPieceShift, 0) * 0x01010101u) & gate);
    floatx4 D0 = slice_group<0>(cu.xa[0], I.w[0].x, I.w[0].y, nib_mask, sa, sa2, sb, zero4);
    floatx4 D1 = slice_group<0>(cu.xa[1], I.w[0].z, I.w[0].w, nib_mask, sa, sa2, sb, zero4);
    if (pm >= 1) {
      D0 = slice_group<1>(cu.xa[0], I.w[1].x, I.w[1].y, nib_mask, sa, sa2, sb, D0);
      D1 = slice_group<1>(cu.xa[1], I.w[1].z, I.w[1].w, nib_mask, sa, sa2, sb, D1);
    }
    if (pm >= 2) {
      D0 = slice_group<2>(cu.xa[0], I.w[2].x, I.w[2].y, nib_mask, sa, sa2, sb, D0);
      D1 = slice_group<2>(cu.xa[1], I.w[2].z, I.w[2].w, nib_mask, sa, sa2, sb, D1);
    }
    if (pm >= 3) {
      D0 = slice_group<3>(cu.xa[0], I.w[3].x, I.w[3].y, nib_mask, sa, sa2, sb, D0);
      D1 = slice_group<3>(cu.xa[1], I.w[3].z, I.w[3].w, nib_mask, sa, sa2, sb, D1);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc[i] += I.mt[0].x * (D0[i] + (kp[i] - I.mt[0].y) * cu.sx[0][i]);
      acc[i] += I.mt[1].x * (D1[i] + (kp[i] - I.mt[1].y) * cu.sx[1][i]);
    }
    if (b == nblk - 1) {  // the tile is complete in this wavefront
      const int buf = ti & 1;
#pragma unroll
      for (int i = 0; i < 4; ++i) red[buf][wave][lane][i] = acc[i];
      acc = zero4;
      __syncthreads();
      if (threadIdx.x < 256) {
        const Proj& P = g.p[j];
        const int r = threadIdx.x >> 4, cc = threadIdx.x & 15;
        const int64_t col = (int64_t)(t - P.tile_begin) * kTileN + cc;
        float sum = 0.f;
#pragma unroll
        for (int wv = 0; wv < kWaves; ++wv) sum += red[buf][wv][16 * (r >> 2) + cc][r & 3];
        if (r < T && col < P.N) P.Y[(int64_t)r * P.N + col] = sum;
      }
    }
  };
  const int total = my_tiles * nblk;
  int ti = 0, b = 0;
#pragma unroll 1
  for (int q = 0; q < total; q += 2) {
    item(ti, b, A, B);
    if (++b == nblk) { b = 0; ++ti; }
    if (q + 1 < total) {
      item(ti, b, B, A);
      if (++b == nblk) { b = 0; ++ti; }
    }
  }
}

static int f4_compute_units() {
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

bool decode_f4_supports(int64_t T, const Shape& sh) { return T >= 1 && T <= 16; }
int decode_f4_timeline_workgroups() { return f4_compute_units(); }
int decode_f4_timeline_slots() { return 8 * f4::kStampSlots; }
// Blocks per part, in units of 8: up to two blocks per wavefront (K <= 8192 in two parts); beyond
// that the streaming kernel, which keeps nothing resident, is the faster one.
static int f4_max_parts_blocks() { return 2; }
// Parts of the K axis the linear kernel works in (2: Y must be zero when it starts; see
// decode_f4_zero_list).  Up to 8 blocks one workgroup holds everything in a single block per wavefront.
int decode_f4_k_parts(const Shape& sh) {
  if (sh.KB <= 8 || sh.KB > 16 * f4_max_parts_blocks()) return 1;
  return (knob(7) == 1 && sh.KB <= 8 * f4_max_parts_blocks()) ? 1 : 2;  // knob 7 = 1: one part where it fits (comparison runs)
}
void decode_f4_zero_list(int64_t T, int n, const Shape* shapes, float* const* Y, ZeroList* zl) {
  for (int i = 0; i < MBQ_MAX_GROUP; ++i) {
    zl->p[i] = nullptr;
    zl->n[i] = 0;
  }
  if (decode_f4_k_parts(shapes[0]) != 2) return;
  for (int i = 0; i < n; ++i) {
    zl->p[i] = Y[i];
    zl->n[i] = (long long)T * shapes[i].N;
  }
}
size_t decode_f4_workspace_bytes(int64_t T, const Shape& sh) {
  return decode_f4_supports(T, sh) ? (size_t)sh.KB * f4::kPrepBytesPerBlock : 0;
}

__global__ __launch_bounds__(256) void decode_f4_prep_kernel(const uint16_t* __restrict__ X, int T, int64_t K,
                                                             char* __restrict__ prep, const ZeroList zl) {
  if (threadIdx.x < 64) f4::prep_block(X, T, K, prep, (int)blockIdx.x, (int)threadIdx.x);
  else zero_share(zl, (int)blockIdx.x, (int)gridDim.x, (int)threadIdx.x - 64, 192);
}

mbq_status launch_decode_f4_prep(const uint16_t* X, int64_t T, int64_t K, int KB, void* ws, const ZeroList& zl,
                                 hipStream_t stream) {
  hipLaunchKernelGGL(decode_f4_prep_kernel, dim3(KB), dim3(256), 0, stream, X, (int)T, K, reinterpret_cast<char*>(ws),
                     zl);
  return hip_status(hipGetLastError(), "decode_f4_prep_kernel launch");
}

// All matrices share K (the caller has checked); T <= 16; ws holds the prepared activations.
mbq_status launch_linear_decode_f4(int64_t T, int n, const void* const* blobs, const Shape* shapes,
                                   const int32_t* const* prec, float* const* Y, const void* ws, hipStream_t stream,
                                   int32_t* const* perm, int32_t* const* offsets, unsigned long long* stamps) {
  f4::Group g;
  int tiles = 0;
  for (int i = 0; i < MBQ_MAX_GROUP; ++i) {
    const int j = i < n ? i : 0;
    const Shape& sh = shapes[j];
    g.p[i].codes = reinterpret_cast<const uint4*>(blobs[j]);
    g.p[i].meta = reinterpret_cast<const float2*>(reinterpret_cast<const char*>(blobs[j]) + sh.meta_offset);
    g.p[i].prec = prec[j];
    g.p[i].perm = (perm && offsets && i < n) ? perm[i] : nullptr;
    g.p[i].offsets = (perm && offsets && i < n) ? offsets[i] : nullptr;
    g.p[i].Y = Y[j];
    g.p[i].slice_vec = sh.slice_words / 4;
    g.p[i].N = sh.N;
    g.p[i].tile_begin = tiles;
    g.p[i].pad = 0;
    if (i < n) tiles += sh.NT;
  }
  g.n = n;
  g.tiles = tiles;
  g.stamps = stamps;
  const Shape& s0 = shapes[0];
  int grid = f4_compute_units();
  const char* prep = reinterpret_cast<const char*>(ws);
  if (s0.KB > 16 * f4_max_parts_blocks()) {
    if (stamps) {
      set_error("the timeline build exists for the ring kernel only (K <= 8192)");
      return MBQ_ERR_BAD_SHAPE;
    }
    if (grid > tiles) grid = tiles;
    hipLaunchKernelGGL(decode_f4_stream_kernel, dim3(grid), dim3(512), 0, stream, prep, (int)T, s0.KB, g);
  } else {
    const int S = decode_f4_k_parts(shapes[0]);
    grid = grid / S * S;
    if (grid > tiles * S) grid = tiles * S;
    const int cpw = (s0.KB + 8 * S - 1) / (8 * S);
#define MBQ_RING(C, P, ST) hipLaunchKernelGGL((decode_f4_ring_kernel<C, P, ST>), dim3(grid), dim3(512), 0, stream, prep, (int)T, s0.KB, g)
    if (stamps) {
      if (S == 1 && cpw == 1) MBQ_RING(1, 1, true);
      else if (S == 1) MBQ_RING(2, 1, true);
      else if (cpw == 1) MBQ_RING(1, 2, true);
      else MBQ_RING(2, 2, true);
    } else {
      if (S == 1 && cpw == 1) MBQ_RING(1, 1, false);
      else if (S == 1) MBQ_RING(2, 1, false);
      else if (cpw == 1) MBQ_RING(1, 2, false);
      else MBQ_RING(2, 2, false);
    }
#undef MBQ_RING
  }
  return hip_status(hipGetLastError(), "decode_f4_kernel launch");
}

}  // namespace mbq
