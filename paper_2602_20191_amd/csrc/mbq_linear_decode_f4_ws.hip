// One-token-tile (T <= 16) FP4-operand decode kernel with a LOADER wavefront: K <= 4096 in one part, K <= 8192 in
// two parts (the second adds into outputs cleared beforehand; two addends, so the result does not depend on order).
//
// Why a loader.  A compute unit takes further vector-memory loads only while a few dozen KiB are outstanding
// (measured: 8 wavefronts x 5 loads of 1 KiB are accepted in ~500 clocks, the next 40 only as the first return).
// A wavefront that asks for its next block therefore parks at the load instruction whenever the memory pipe is
// full, which it should always be, with its MFMAs queued behind the load: loading and arithmetic of one wavefront
// take turns instead of overlapping, and a deeper prefetch only parks it longer.  Here one extra wavefront does
// nothing but issue loads (it may stand at the load instruction all the time: that means the pipe is full), the
// memory system writes the blocks straight into a ring in LDS (global_load_lds), and eight wavefronts do the
// arithmetic without ever issuing a weight load.
//
//   loader (wavefront 8): walks the workgroup's tiles block by block; item q = 4 slices of 1 KiB + 256 bytes of
//     {s0, z0} -> ring slot q % kWsRing, at most kWsDepth items in flight (loads complete in issue order, so
//     `s_waitcnt vmcnt(5 kWsDepth)` after issuing item q says that item q - kWsDepth has landed), then
//     ready[slot] = lap + 1.  Before re-using a slot it waits for done[slot] = lap of the previous occupant.
//   arithmetic (wavefront w < 8): owns blocks w, w + 8 of the part (activations in registers); waits for
//     ready[slot], copies the item to registers, sets done[slot], runs the 16 scaled MFMAs.  After its blocks of a
//     tile it files its partial 16 x 16 tile in LDS and counts itself in; the wavefront that arrives last sums the
//     eight partial tiles in a fixed order and stores the outputs.  No workgroup barrier in the loop (the loader
//     could not take part in one).
// Every wait on a flag is a bounded spin (kWsPollCap probes); if one ever runs out the launch finishes with wrong
// numbers instead of hanging.
//
// Arithmetic, operand layout and the A/B block scales: see mbq_linear_decode_f4.hip.  Paper: Sec. 4.2 Eq. 6 slice by
// slice; Sec. 4.3 (on-demand slice access: a tile fetches slices 0..max precision of its matrix; fused launch for the
// projections of a layer).
#include <type_traits>

#include "mbq_f4_kernel.h"

namespace mbq {

namespace f4 {
constexpr int kWsRing = 32;        // ring slots (items of 4352 bytes), four groups of eight
constexpr int kWsDepth = 12;       // items in flight at most: 60 loads, the wavefront's counter holds 63
constexpr int kWsRed = 2;          // partial-tile buffers: a wavefront may run this many tiles ahead of the slowest
constexpr int kWsChunkTiles = 8;   // kChunks > 1: tiles per workgroup at most (their sums wait in LDS between chunks)
constexpr int kWsPollCap = 1 << 17;  // x ~0.1 us: three orders of magnitude above any real wait
constexpr int kWsSlotBytes = 4 * 1024 + 256;
constexpr int kWsStampSlots = 32;  // timeline build, slots as documented in mbq_bench.h (wavefront 8 = loader: slot 1
                                   // precisions here, 2 first item issued, 4 + i item i published (i < 26))

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t lds_load_u32(uint32_t addr) {
  uint32_t v;
  asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
  return v;
}
__device__ __forceinline__ void lds_store_u32(uint32_t addr, uint32_t v) {
  asm volatile("ds_write_b32 %0, %1" ::"v"(addr), "v"(v) : "memory");
}
// spins until the word at addr equals `want` (same in all lanes); bounded
__device__ __forceinline__ void wait_flag(uint32_t addr, uint32_t want) {
  for (int spin = 0; spin < kWsPollCap; ++spin) {
    if (__builtin_amdgcn_readfirstlane((int)lds_load_u32(addr)) == (int)want) return;
    __builtin_amdgcn_s_sleep(1);
  }
}
// spins until the word at addr, a count that only grows, has reached `want`; bounded
__device__ __forceinline__ void wait_count(uint32_t addr, uint32_t want) {
  for (int spin = 0; spin < kWsPollCap; ++spin) {
    if ((uint32_t)__builtin_amdgcn_readfirstlane((int)lds_load_u32(addr)) >= want) return;
    __builtin_amdgcn_s_sleep(1);
  }
}
// the same for eight consecutive words (addr 16-byte aligned)
__device__ __forceinline__ void wait_flags8(uint32_t addr, uint32_t want) {
  for (int spin = 0; spin < kWsPollCap; ++spin) {
    u32x4 lo, hi;
    asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:16\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(lo), "=&v"(hi)
                 : "v"(addr)
                 : "memory");
    const uint32_t differ = (lo.x ^ want) | (lo.y ^ want) | (lo.z ^ want) | (lo.w ^ want) | (hi.x ^ want) |
                            (hi.y ^ want) | (hi.z ^ want) | (hi.w ^ want);
    if (__builtin_amdgcn_readfirstlane((int)differ) == 0) return;
    __builtin_amdgcn_s_sleep(1);
  }
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// at most 5 n loads outstanding, n = 0 .. 12
__device__ __forceinline__ void wait_items_behind(int n) {
  switch (n) {
    case 0: wait_vmcnt<0>(); break;
    case 1: wait_vmcnt<5>(); break;
    case 2: wait_vmcnt<10>(); break;
    case 3: wait_vmcnt<15>(); break;
    case 4: wait_vmcnt<20>(); break;
    case 5: wait_vmcnt<25>(); break;
    case 6: wait_vmcnt<30>(); break;
    case 7: wait_vmcnt<35>(); break;
    case 8: wait_vmcnt<40>(); break;
    case 9: wait_vmcnt<45>(); break;
    case 10: wait_vmcnt<50>(); break;
    case 11: wait_vmcnt<55>(); break;
    default: wait_vmcnt<60>(); break;
  }
}
__device__ __forceinline__ void dma_16(const void* gptr, char* lds_base) {
  __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)gptr,
                                   (void __attribute__((address_space(3)))*)lds_base, 16, 0, 2);
}
__device__ __forceinline__ void dma_4(const void* gptr, char* lds_base) {
  __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)gptr,
                                   (void __attribute__((address_space(3)))*)lds_base, 4, 0, 2);
}
static_assert(kWsDepth <= 12 && kWsDepth < kWsRing, "60 loads in flight at most; the ring must hold what is in flight");
static_assert(kWsRing % 8 == 0, "the loader checks the slots in groups of eight");
}  // namespace f4

// kBits: the precision arrays hold bits - 1 (1 to 8 bits, see RouteView) instead of digit precisions: a token may stop
// at the high bit of its last digit, so the two bits of every 2-bit code go to the matrix cores as two operands (the
// high bit as the FP4 number (c & 2) / 2, the low bit as (c & 1) / 2), each gated by its own A scale byte: twice the
// MFMAs, same loads.
// kChunks > 1 (8192 < K <= 16384): a part of the K axis is more than the registers hold, so a workgroup works through
// it in kChunks chunks of at most 16 blocks - all its tiles for the first chunk, then the activations of the second
// chunk, all its tiles again - and keeps the tiles' sums of the earlier chunks in LDS (at most kWsChunkTiles tiles per
// workgroup; the ring gives up a quarter of its slots for them).  The parts still meet by adding two addends.
template <int CPW, int S, bool kStamp, bool kBits = false, int kChunks = 1>
__global__ __launch_bounds__(576) void decode_f4_ws_kernel(const char* __restrict__ prep, int T, int KB,
                                                           const f4::Group g) {
  using namespace f4;
  constexpr int kWaves = 8;  // arithmetic wavefronts; wavefront 8 loads
  static_assert(S == 1 || S == 2, "one or two parts");
  static_assert(CPW == 1 || CPW == 2, "one or two blocks per wavefront");
  static_assert(kChunks == 1 || (CPW == 2 && S == 2 && !kStamp), "the chunked variant: two parts, two blocks per wavefront");
  constexpr int kRing = kChunks > 1 ? kWsRing - 8 : kWsRing;
  __shared__ __attribute__((aligned(16))) float s_held[kChunks > 1 ? kWsChunkTiles : 1][64][4];  // sums of earlier chunks
  __shared__ __attribute__((aligned(1024))) char ring[kRing * kWsSlotBytes];
  __shared__ __attribute__((aligned(16))) float red[kWsRed][kWaves][64][4];
  __shared__ __attribute__((aligned(16))) uint32_t s_done[kRing], s_cnt[kWsRed], s_fin[kWsRed];
  __shared__ uint32_t s_count;  // items that have landed in the ring (they land in issue order)
  __shared__ unsigned long long s_stamp[kStamp ? (kWaves + 1) * kWsStampSlots : 1];
  constexpr int kThreads = 64 * (kWaves + 1);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m = lane & 15, kq = lane >> 4;
  auto lds_addr = [](const void* p) { return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p; };
  const uint32_t ring_addr = lds_addr(ring), red_addr = lds_addr(red),
                 done_addr = lds_addr(s_done), cnt_addr = lds_addr(s_cnt), fin_addr = lds_addr(s_fin),
                 count_addr = lds_addr(&s_count);
  const uint32_t stamp_addr = lds_addr(s_stamp) + (uint32_t)(wave * kWsStampSlots * 8);
  auto stamp = [&](int slot) {
    if constexpr (kStamp) {
      if (slot < kWsStampSlots - 2 && lane == 0) {
        const unsigned long long now = __builtin_amdgcn_s_memrealtime();
        asm volatile("ds_write_b64 %0, %1" ::"v"(stamp_addr + (uint32_t)slot * 8u), "v"(now) : "memory");
      }
    }
  };
  for (int i = threadIdx.x; i < kRing; i += kThreads) s_done[i] = 0u;
  if (threadIdx.x < kWsRed) {
    s_cnt[threadIdx.x] = 0u;
    s_fin[threadIdx.x] = 0u;
  }
  if (threadIdx.x == 0) s_count = 0u;
  if constexpr (kStamp)
    for (int i = threadIdx.x; i < (kWaves + 1) * kWsStampSlots; i += kThreads) s_stamp[i] = 0ull;
  __syncthreads();  // the only workgroup barrier: nothing is in flight yet
  stamp(0);

  const int part = (int)blockIdx.x % S;
  const int bid = (int)blockIdx.x / S;     // position in the tile list
  const int stride = (int)gridDim.x / S;   // the launcher makes gridDim.x a multiple of S
  const int my_tiles = (g.tiles - bid + stride - 1) / stride;
  const int nbp = (KB + S - 1) / S;        // blocks per part
  const int kb_first = part * nbp;
  const int nb = min(KB - kb_first, nbp);  // blocks of this part (the launcher makes sure it is positive)
  const bool has_work = my_tiles > 0 && nb > 0;
  const int nbc = (nb + kChunks - 1) / kChunks;  // blocks per chunk (<= 8 CPW); chunk c: blocks c nbc .. of the part

  int pl[MBQ_MAX_GROUP];  // precisions of every matrix (arithmetic wavefronts; the loader is told the highest ones)

  // The per-matrix facts are fetched from the argument block once, all at the same time, and kept in scalar registers:
  // looking a matrix up later (when the tile list crosses into it) then costs selects, not a chain of dependent loads.
  const char* m_codes[MBQ_MAX_GROUP];
  const char* m_meta[MBQ_MAX_GROUP];
  float* m_Y[MBQ_MAX_GROUP];
  size_t m_slice_bytes[MBQ_MAX_GROUP];
  int m_N[MBQ_MAX_GROUP], m_begin[MBQ_MAX_GROUP];
#pragma unroll
  for (int i = 0; i < MBQ_MAX_GROUP; ++i) {
    m_codes[i] = reinterpret_cast<const char*>(g.p[i].codes);
    m_meta[i] = reinterpret_cast<const char*>(g.p[i].meta);
    m_Y[i] = g.p[i].Y;
    m_slice_bytes[i] = g.p[i].slice_vec * 16u;
    m_N[i] = (int)g.p[i].N;
    m_begin[i] = i < g.n ? g.p[i].tile_begin : 0x7fffffff;  // matrices past g.n start where no tile reaches
    asm volatile("" : "+s"(m_codes[i]), "+s"(m_meta[i]), "+s"(m_Y[i]), "+s"(m_slice_bytes[i]), "+s"(m_N[i]), "+s"(m_begin[i]));
  }
#define MBQ_PICK(arr, j) ((j) == 0 ? arr[0] : (j) == 1 ? arr[1] : (j) == 2 ? arr[2] : arr[3])
  auto proj_of = [&](int t) {
    int j = 0;
#pragma unroll
    for (int i = 1; i < MBQ_MAX_GROUP; ++i)
      if (t >= m_begin[i]) j = i;
    return j;
  };
  auto next_begin_of = [&](int j) {  // first tile of the matrix after matrix j
    int b = 0x7fffffff;
#pragma unroll
    for (int i = MBQ_MAX_GROUP - 1; i >= 1; --i)
      if (i > j) b = m_begin[i];
    return b;
  };
  int pmax[MBQ_MAX_GROUP];
  auto digits_of = [](int stored) { return kBits ? (stored >> 1) : stored; };  // (-1 stays -1)
  auto find_pmax = [&]() {
#pragma unroll
    for (int j = 0; j < MBQ_MAX_GROUP; ++j) pl[j] = lane < T ? pl[j] : -1;
#pragma unroll
    for (int j = 0; j < MBQ_MAX_GROUP; ++j) {
      const int d = digits_of(pl[j]);
      pmax[j] = (__ballot(d == 3) != 0ull) ? 3 : (__ballot(d == 2) != 0ull) ? 2 : (__ballot(d == 1) != 0ull) ? 1 : 0;
    }
  };
  auto pmax_of = [&](int j) { return j == 0 ? pmax[0] : j == 1 ? pmax[1] : j == 2 ? pmax[2] : pmax[3]; };

  if (wave == kWaves) {
    // ================================================= loader =================================================
    __builtin_amdgcn_s_setprio(3);  // its few instructions go ahead of the arithmetic of the wavefronts it shares a SIMD with
#pragma unroll
    for (int j = 0; j < MBQ_MAX_GROUP; ++j) pl[j] = g.p[j].prec[lane < T ? lane : 0];  // (an unused slot of g repeats matrix 0)
    find_pmax();
    stamp(1);
    if (has_work) {
      const int total = my_tiles * nb;
      const uint32_t held_addr = lds_addr(s_held);
      (void)held_addr;
      const size_t code_step = (size_t)stride * (size_t)KB * 1024u;  // from one of this workgroup's tiles to the next
      const size_t meta_step = (size_t)stride * (size_t)KB * 256u;
      // wave-uniform pointers to block kb_first of the current row of tiles; a slice the matrix does not need at this
      // call's precisions stands on `prep` (a KiB that stays cached) and does not move: every item is five loads
      const char* p[4];
      size_t step[4];
      const char* pmeta;
      int t = bid, next_begin = 0;
      int chunk_first = kb_first;  // first block of the chunk being loaded
      auto enter = [&]() {
        const int j = proj_of(t);
        const int nt = t - MBQ_PICK(m_begin, j);
        const int pm = pmax_of(j);
        const char* row = MBQ_PICK(m_codes, j) + ((size_t)nt * (size_t)KB + (size_t)chunk_first) * 1024u;
        const size_t slice_bytes = MBQ_PICK(m_slice_bytes, j);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          p[e] = uniform((e <= pm) ? row + (size_t)e * slice_bytes : prep);
          step[e] = uniform((e <= pm) ? code_step : (size_t)0);
        }
        pmeta = uniform(MBQ_PICK(m_meta, j) + ((size_t)nt * (size_t)KB + (size_t)chunk_first) * 256u);
        next_begin = uniform(next_begin_of(j));
      };
      auto next_tile = [&]() {
#pragma unroll
        for (int e = 0; e < 4; ++e) p[e] += step[e];
        pmeta += meta_step;
        t += stride;
        if (t >= next_begin && t < g.tiles) enter();
      };
      enter();
      int slot = 0, lap = 0;     // ring position of the next item: q = lap kRing + slot
      uint32_t landed = 0u;      // items published so far (they land, and are published, in order)
      const uint32_t lane16 = (uint32_t)lane * 16u, lane4 = (uint32_t)lane * 4u;
      // five loads of the item that is block b of the cursor's tile, into ring slot sl
      auto issue = [&](int b, int sl) {
        char* dst = ring + sl * kWsSlotBytes;
        const uint32_t co = (uint32_t)b * 1024u + lane16, mo = (uint32_t)b * 256u + lane4;
#pragma unroll
        for (int e = 0; e < 4; ++e) dma_16(p[e] + co, dst + e * 1024);
        dma_4(pmeta + mo, dst + 4096);
      };
      // after item q has been issued: item q - kDepth has landed (loads complete in issue order); say so
      constexpr int kDepth = kWsDepth;
      auto publish_behind = [&](int q) {
        if (q >= kDepth) {
          wait_vmcnt<5 * kDepth>();
          lds_store_u32(count_addr, ++landed);
          if constexpr (kStamp)
            if (q - kDepth < kWsStampSlots - 6) stamp(4 + q - kDepth);
        }
      };
      stamp(2);
      const int issued = total;
      if constexpr (kChunks > 1) {
        int q = 0;
#pragma unroll 1
        for (int c = 0; c < kChunks; ++c) {
          const int nb_c = min(nbc, nb - c * nbc);
          chunk_first = kb_first + c * nbc;
          t = bid;
          enter();
          int b = 0;
#pragma unroll 1
          for (int n = my_tiles * nb_c; n > 0; --n, ++q) {
            asm volatile("" : "+s"(p[0]), "+s"(p[1]), "+s"(p[2]), "+s"(p[3]), "+s"(pmeta), "+s"(b), "+s"(slot), "+s"(lap),
                         "+s"(t), "+s"(next_begin), "+s"(q));
            if (lap > 0 && (slot & 7) == 0) wait_flags8(done_addr + (uint32_t)slot * 4u, (uint32_t)lap);
            issue(b, slot);
            publish_behind(q);
            if (++slot == kRing) {
              slot = 0;
              ++lap;
            }
            if (++b == nb_c) {
              b = 0;
              next_tile();
            }
          }
        }
      } else if ((nb & 7) == 0) {
        // The usual shapes (8 or 16 blocks per part): eight items at a time, no bookkeeping between them.  The loader is
        // a single wavefront and every instruction it spends per item comes off the stream's rate.
        const int groups = nb >> 3;
        int q = 0;
#pragma unroll 1
        for (int ti = 0; ti < my_tiles; ++ti) {
#pragma unroll 1
          for (int gi = 0; gi < groups; ++gi) {
            asm volatile("" : "+s"(p[0]), "+s"(p[1]), "+s"(p[2]), "+s"(p[3]), "+s"(pmeta), "+s"(slot), "+s"(lap), "+s"(t),
                         "+s"(next_begin), "+s"(q));
            // before eight slots are filled again: their previous occupants have been read
            if (lap > 0) wait_flags8(done_addr + (uint32_t)slot * 4u, (uint32_t)lap);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              issue(gi * 8 + i, slot + i);
              publish_behind(q + i);
            }
            q += 8;
            slot += 8;
            if (slot == kRing) {
              slot = 0;
              ++lap;
            }
          }
          next_tile();
        }
      } else {
        int b = 0;  // block of the tile the next item is
#pragma unroll 1
        for (int q = 0; q < total; ++q) {
          asm volatile("" : "+s"(p[0]), "+s"(p[1]), "+s"(p[2]), "+s"(p[3]), "+s"(pmeta), "+s"(b), "+s"(slot), "+s"(lap),
                       "+s"(t), "+s"(next_begin));
          if (lap > 0 && (slot & 7) == 0) wait_flags8(done_addr + (uint32_t)slot * 4u, (uint32_t)lap);
          issue(b, slot);
          publish_behind(q);
          if (++slot == kRing) {
            slot = 0;
            ++lap;
          }
          if (++b == nb) {
            b = 0;
            next_tile();
          }
        }
      }
      // what is still in flight
      const int left = min(issued, kDepth);
#pragma unroll 1
      for (int i = 0; i < left; ++i) {
        wait_items_behind(left - 1 - i);
        lds_store_u32(count_addr, ++landed);
        if constexpr (kStamp)
          if (issued - left + i < kWsStampSlots - 6) stamp(4 + issued - left + i);
      }
    }
  } else {
    // =============================================== arithmetic ===============================================
    // prepared activations of this wavefront's blocks (registers, for the whole kernel); a block the part does not
    // have is never asked for
#pragma unroll
    for (int j = 0; j < MBQ_MAX_GROUP; ++j) pl[j] = g.p[j].prec[lane < T ? lane : 0];  // (an unused slot of g repeats matrix 0)
    intx8 xa[CPW][2][kPieces];
    floatx4 sx[CPW][2];
    int tok_scale[CPW];
    // (chunked variant: blocks first .. first + count - 1 of the K axis; called once per chunk)
    auto load_activations = [&](int first, int count) {
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
      const int b = wave + kWaves * c;
      const char* base = prep + (size_t)(b < count ? first + b : 0) * kPrepBytesPerBlock;
      const uint4* src = reinterpret_cast<const uint4*>(base);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int piece = 0; piece < kPieces; ++piece) {
          const uint4 lo = src[(size_t)(h * kPieces + piece) * 128 + lane];
          const uint4 hi = src[(size_t)(h * kPieces + piece) * 128 + 64 + lane];
          xa[c][h][piece] = intx8{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
        }
        sx[c][h] = *reinterpret_cast<const floatx4*>(base + kPrepVecPerBlock * 16 + (16 * h + 4 * kq) * 4);
      }
      tok_scale[c] = reinterpret_cast<const int*>(base + kPrepVecPerBlock * 16 + 2 * 16 * 4)[m];
    }
    };
    load_activations(kb_first, kChunks > 1 ? min(nbc, nb) : nb);
    find_pmax();
    stamp(1);
    if (blockIdx.x == 0 && wave == 0) {  // one wavefront of the launch sorts the tokens, where the caller wants them sorted
#pragma unroll
      for (int j = 0; j < MBQ_MAX_GROUP; ++j)
        if (j < g.n && g.p[j].perm != nullptr) bucket_by_wave(digits_of(pl[j]), lane, g.p[j].perm, g.p[j].offsets);
    }
    if (has_work) {
      uint32_t nib_mask = 0x33333333u;
      asm volatile("" : "+s"(nib_mask));  // keep the mask in a register: one v_and_b32 per operand dword
      const int sb = 0x7A7C7E80;          // B scale bytes 2^(1-2e), e = 0..3
      const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};
      // the matrix of the current tile, looked up when the tile list crosses into it
      int cs_t = bid, cs_next_begin = 0, cs_pm = 0, cs_N = 0, cs_col0 = 0;
      float* cs_Y = nullptr;
      uint32_t cs_gate = 0u;  // A scale gate of this lane's token (row m of the A operand): slice e counts iff e <= its precision
      uint32_t cs_gate_lo = 0u;  // kBits: cs_gate gates the high bits of the codes, this one the low bits
      floatx4 cs_kp = zero4;  // 0.5 - 1.5 q_p of the output rows 4 kq + i
      auto cs_enter = [&]() {
        const int j = proj_of(cs_t);
        cs_pm = uniform(pmax_of(j));
        cs_N = uniform(MBQ_PICK(m_N, j));
        cs_Y = uniform(MBQ_PICK(m_Y, j));
        cs_col0 = uniform((cs_t - MBQ_PICK(m_begin, j)) * kTileN);
        cs_next_begin = uniform(next_begin_of(j));
        const int plj = j == 0 ? pl[0] : j == 1 ? pl[1] : j == 2 ? pl[2] : pl[3];
        const int pa = __shfl(plj, m, 64);
        auto gate_of = [](int d) {  // slices 0..d
          return (d >= 3) ? 0xFFFFFFFFu : (d == 2) ? 0x00FFFFFFu : (d == 1) ? 0x0000FFFFu : (d == 0) ? 0x000000FFu : 0u;
        };
        if constexpr (kBits) {
          // pa + 1 bits: the high bit of digit e counts from 2 e + 1 bits on, its low bit from 2 e + 2
          cs_gate = gate_of(pa >= 0 ? pa >> 1 : -1);
          cs_gate_lo = gate_of(pa >= 0 ? ((pa + 1) >> 1) - 1 : -1);
        } else {
          cs_gate = gate_of(pa);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int p = __shfl(plj, 4 * kq + i, 64);
          // the constant of the reconstruction: 2^(1 - bits)
          if constexpr (kBits) cs_kp[i] = __builtin_ldexpf(1.f, -max(p, 0));
          else cs_kp[i] = (p >= 3) ? 0.0078125f : (p == 2) ? 0.03125f : (p == 1) ? 0.125f : 0.5f;
        }
      };
      cs_enter();
      int rb = 0, rlap = 0;  // partial-tile buffer of the current tile: (chunk my_tiles + ti) = rlap kWsRed + rb
      int q_base = 0;        // items of the chunks before this one
      const uint32_t held_addr = lds_addr(s_held);
#pragma unroll 1
      for (int chunk = 0; chunk < kChunks; ++chunk) {
      const int nb_c = kChunks > 1 ? min(nbc, nb - chunk * nbc) : nb;  // blocks of this chunk
      if (kChunks > 1 && chunk > 0) {
        load_activations(kb_first + chunk * nbc, nb_c);
        cs_t = bid;
        cs_enter();
      }
#pragma unroll 1
      for (int ti = 0; ti < my_tiles; ++ti) {
        asm volatile("" : "+s"(cs_t), "+s"(cs_next_begin), "+s"(cs_pm), "+s"(cs_N), "+s"(cs_col0), "+s"(cs_Y), "+s"(rb),
                     "+s"(rlap));
        const int pm = cs_pm;
        floatx4 acc = zero4;
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
          const int b = wave + kWaves * c;
          if (b < nb_c) {
            const int q = q_base + ti * nb_c + b;  // position in the ring's sequence of items
            wait_count(count_addr, (uint32_t)q + 1u);
            const int qlap = q / kRing, qslot = q - qlap * kRing;
            const uint32_t slot = ring_addr + (uint32_t)(qslot * kWsSlotBytes);
            u32x4 wv[4];
            f32x2 mv[2];
            asm volatile(
                "ds_read_b128 %0, %6\n\t"
                "ds_read_b128 %1, %6 offset:1024\n\t"
                "ds_read_b128 %2, %6 offset:2048\n\t"
                "ds_read_b128 %3, %6 offset:3072\n\t"
                "ds_read_b64 %4, %7 offset:4096\n\t"
                "ds_read_b64 %5, %7 offset:4224\n\t"
                "s_waitcnt lgkmcnt(0)"
                : "=&v"(wv[0]), "=&v"(wv[1]), "=&v"(wv[2]), "=&v"(wv[3]), "=&v"(mv[0]), "=&v"(mv[1])
                : "v"(slot + (uint32_t)lane * 16u), "v"(slot + (uint32_t)m * 8u)
                : "memory");
            lds_store_u32(done_addr + (uint32_t)qslot * 4u, (uint32_t)(qlap + 1));  // the slot may be filled again
            Item I;
#pragma unroll
            for (int e = 0; e < 4; ++e) I.w[e] = uint4{wv[e].x, wv[e].y, wv[e].z, wv[e].w};
            I.mt[0] = float2{mv[0].x, mv[0].y};
            I.mt[1] = float2{mv[1].x, mv[1].y};
            const int sa = (int)(((uint32_t)tok_scale[c] * 0x01010101u) & cs_gate);
            const int sa2 = (int)(((uint32_t)max(tok_scale[c] - kPieceShift, 0) * 0x01010101u) & cs_gate);  // second piece is stored 2^kPieceShift times larger
            floatx4 D0, D1;
            if constexpr (kBits) {
              const int sl = (int)(((uint32_t)tok_scale[c] * 0x01010101u) & cs_gate_lo);
              const int sl2 = (int)(((uint32_t)max(tok_scale[c] - kPieceShift, 0) * 0x01010101u) & cs_gate_lo);
              uint32_t mask_hi = 0x22222222u, mask_lo = 0x11111111u;
              asm volatile("" : "+s"(mask_hi), "+s"(mask_lo));
              D0 = zero4;
              D1 = zero4;
              auto planes = [&](auto e_tag) {
                constexpr int E = decltype(e_tag)::value;
                if (E > pm) return;
                D0 = slice_group<E>(xa[c][0], I.w[E].x, I.w[E].y, mask_hi, sa, sa2, sb, D0);
                D1 = slice_group<E>(xa[c][1], I.w[E].z, I.w[E].w, mask_hi, sa, sa2, sb, D1);
                D0 = slice_group<E>(xa[c][0], I.w[E].x, I.w[E].y, mask_lo, sl, sl2, sb, D0);
                D1 = slice_group<E>(xa[c][1], I.w[E].z, I.w[E].w, mask_lo, sl, sl2, sb, D1);
              };
              planes(std::integral_constant<int, 0>{});
              planes(std::integral_constant<int, 1>{});
              planes(std::integral_constant<int, 2>{});
              planes(std::integral_constant<int, 3>{});
            } else if (pm >= 3) {
              // all four slices (the usual case at 16 tokens) as one straight run of code: the operands of a slice are
              // built while the MFMAs of the slice before occupy the matrix core
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
              acc[i] += I.mt[0].x * (D0[i] + (cs_kp[i] - I.mt[0].y) * sx[c][0][i]);
              acc[i] += I.mt[1].x * (D1[i] + (cs_kp[i] - I.mt[1].y) * sx[c][1][i]);
            }
          }
        }
        if constexpr (kStamp) {
          asm volatile("" ::"v"(acc[0]), "v"(acc[1]), "v"(acc[2]), "v"(acc[3]));
          if (ti < 13) stamp(4 + 2 * ti);
        }
        // File the partial tile and count in; the wavefront that is last sums the eight in wavefront order and stores.
        if (rlap > 0) wait_flag(fin_addr + (uint32_t)rb * 4u, (uint32_t)rlap);  // the buffer's previous tile has been summed
        const uint32_t mine = red_addr + (uint32_t)(((rb * kWaves + wave) * 64 + lane) * 16);
        asm volatile("ds_write_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" ::"v"(mine), "v"(acc) : "memory");
        uint32_t arrived = 0u;
        if (lane == 0)
          asm volatile("ds_add_rtn_u32 %0, %1, %2\n\ts_waitcnt lgkmcnt(0)"
                       : "=&v"(arrived)
                       : "v"(cnt_addr + (uint32_t)rb * 4u), "v"(1u)
                       : "memory");
        const uint32_t after_me = (uint32_t)__builtin_amdgcn_readfirstlane((int)arrived) + 1u;
        if (after_me == (uint32_t)(rlap + 1) * (uint32_t)kWaves) {
          floatx4 sum = zero4;
          const uint32_t base = red_addr + (uint32_t)((rb * kWaves * 64 + lane) * 16);
          floatx4 part[kWaves];
          asm volatile(
              "ds_read_b128 %0, %8\n\t"
              "ds_read_b128 %1, %8 offset:1024\n\t"
              "ds_read_b128 %2, %8 offset:2048\n\t"
              "ds_read_b128 %3, %8 offset:3072\n\t"
              "ds_read_b128 %4, %8 offset:4096\n\t"
              "ds_read_b128 %5, %8 offset:5120\n\t"
              "ds_read_b128 %6, %8 offset:6144\n\t"
              "ds_read_b128 %7, %8 offset:7168\n\t"
              "s_waitcnt lgkmcnt(0)"
              : "=&v"(part[0]), "=&v"(part[1]), "=&v"(part[2]), "=&v"(part[3]), "=&v"(part[4]), "=&v"(part[5]),
                "=&v"(part[6]), "=&v"(part[7])
              : "v"(base)
              : "memory");
          lds_store_u32(fin_addr + (uint32_t)rb * 4u, (uint32_t)(rlap + 1));
#pragma unroll
          for (int w = 0; w < kWaves; ++w) sum += part[w];
          bool last_chunk = true;
          if constexpr (kChunks > 1) {
            // sums of the earlier chunks of this tile wait in LDS (written by whichever wavefront summed then: it filed
            // its later partial tiles after that write, and all eight have been counted in here)
            const uint32_t held = held_addr + (uint32_t)((ti * 64 + lane) * 16);
            if (chunk > 0) {
              floatx4 before;
              asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(before) : "v"(held) : "memory");
              sum = before + sum;
            }
            last_chunk = chunk == kChunks - 1;
            if (!last_chunk) asm volatile("ds_write_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" ::"v"(held), "v"(sum) : "memory");
          }
          const int col = cs_col0 + m;
          if (last_chunk && col < cs_N) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const int r = 4 * kq + i;
              if (r < T) {
                // (explicitly global: through a generic pointer these would be FLAT instructions)
                float* dst = &cs_Y[(int64_t)r * cs_N + col];
                if constexpr (S == 1) asm volatile("global_store_dword %0, %1, off" ::"v"(dst), "v"(sum[i]) : "memory");
                else asm volatile("global_atomic_add_f32 %0, %1, off" ::"v"(dst), "v"(sum[i]) : "memory");
              }
            }
          }
        }
        if (ti < 13) stamp(5 + 2 * ti);
        if (++rb == kWsRed) {
          rb = 0;
          ++rlap;
        }
        cs_t += stride;
        cs_col0 += stride * kTileN;
        if (cs_t >= cs_next_begin && cs_t < g.tiles) cs_enter();
      }
      q_base += my_tiles * nb_c;
      }
    }
  }
  if constexpr (kStamp) {
    if (lane == 0) {
      const unsigned long long now = __builtin_amdgcn_s_memrealtime();
      const unsigned long long hw =
          ((unsigned long long)__builtin_amdgcn_s_getreg(20 | (0 << 6) | (31 << 11)) << 32) |  // XCC_ID
          (unsigned long long)__builtin_amdgcn_s_getreg(4 | (0 << 6) | (31 << 11));             // HW_ID
      asm volatile("ds_write_b64 %0, %1\n\tds_write_b64 %2, %3" ::"v"(stamp_addr + (uint32_t)(kWsStampSlots - 2) * 8u),
                   "v"(now), "v"(stamp_addr + (uint32_t)(kWsStampSlots - 1) * 8u), "v"(hw)
                   : "memory");
    }
    wait_vmcnt<0>();
    __syncthreads();
    for (int i = threadIdx.x; i < (kWaves + 1) * kWsStampSlots; i += kThreads)
      g.stamps[(size_t)blockIdx.x * ((kWaves + 1) * kWsStampSlots) + i] = s_stamp[i];
  }
}

#undef MBQ_PICK

// one to 32 column blocks: activations of a part in registers; up to 64: two chunks per part, if the workgroups'
// tile lists are short enough for the sums to wait in LDS
bool decode_f4_ws_supports(int KB, int tiles) {
  if (KB >= 1 && KB <= 32) return true;
  const int per_part = f4_compute_units() / 2;
  return KB <= 64 && per_part >= 1 && (tiles + per_part - 1) / per_part <= f4::kWsChunkTiles && knob(7) != 1;
}
int decode_f4_ws_parts(int KB) { return KB <= 16 ? 1 : 2; }
int decode_f4_ws_stamp_wavefronts() { return 9; }

// T <= 16, KB <= 32; ws holds the prepared activations; with two parts the outputs must be zero when the launch starts;
// g.stamps != nullptr selects the timeline build
mbq_status launch_linear_decode_f4_ws(int64_t T, const f4::Group& g, int KB, const void* ws, hipStream_t stream) {
  const int S = decode_f4_ws_parts(KB);
  int grid = f4_compute_units() / S * S;
  if (grid > g.tiles * S) grid = g.tiles * S;
  const int cpw = ((KB + S - 1) / S + 7) / 8;
  const char* prep = reinterpret_cast<const char*>(ws);
  if (KB > 32) {  // two chunks per part
    if (g.stamps) {
      set_error("the timeline build exists for K <= 8192 only");
      return MBQ_ERR_BAD_SHAPE;
    }
    if (g.bit_view)
      hipLaunchKernelGGL((decode_f4_ws_kernel<2, 2, false, true, 2>), dim3(grid), dim3(576), 0, stream, prep, (int)T, KB, g);
    else
      hipLaunchKernelGGL((decode_f4_ws_kernel<2, 2, false, false, 2>), dim3(grid), dim3(576), 0, stream, prep, (int)T, KB, g);
    return hip_status(hipGetLastError(), "decode_f4_ws_kernel launch");
  }
#define MBQ_WS(C, P, ST) \
  hipLaunchKernelGGL((decode_f4_ws_kernel<C, P, ST>), dim3(grid), dim3(576), 0, stream, prep, (int)T, KB, g)
  if (g.bit_view) {  // (no timeline build of this variant)
    if (g.stamps) {
      set_error("the timeline build exists for digit precisions only");
      return MBQ_ERR_BAD_SHAPE;
    }
    if (S == 1 && cpw == 1)
      hipLaunchKernelGGL((decode_f4_ws_kernel<1, 1, false, true>), dim3(grid), dim3(576), 0, stream, prep, (int)T, KB, g);
    else if (S == 1)
      hipLaunchKernelGGL((decode_f4_ws_kernel<2, 1, false, true>), dim3(grid), dim3(576), 0, stream, prep, (int)T, KB, g);
    else
      hipLaunchKernelGGL((decode_f4_ws_kernel<2, 2, false, true>), dim3(grid), dim3(576), 0, stream, prep, (int)T, KB, g);
  } else if (g.stamps) {
    if (S == 1 && cpw == 1) MBQ_WS(1, 1, true);
    else if (S == 1) MBQ_WS(2, 1, true);
    else MBQ_WS(2, 2, true);
  } else {
    if (S == 1 && cpw == 1) MBQ_WS(1, 1, false);
    else if (S == 1) MBQ_WS(2, 1, false);
    else MBQ_WS(2, 2, false);
  }
#undef MBQ_WS
  return hip_status(hipGetLastError(), "decode_f4_ws_kernel launch");
}

}  // namespace mbq
