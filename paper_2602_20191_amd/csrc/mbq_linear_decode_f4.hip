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
// Kernels: up to 32 column blocks (K <= 8192) the kernel of mbq_linear_decode_f4_ws.hip (a loader wavefront streams
// the packed weights into an LDS ring, eight wavefronts with the activations in registers do the arithmetic);
// beyond, decode_f4_stream_kernel below, which streams the activations along with the weights.  This file also
// holds the activation preparation launch and the launcher that picks the kernel.
#include <type_traits>

#include "mbq_f4_kernel.h"

namespace mbq {

// K > 8192: the activation pieces of a wavefront's blocks no longer fit in registers, so
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

// kBits: the precision arrays hold bits - 1 (see RouteView); as in the loader-wavefront kernel the two bits of a code
// then go to the matrix cores as two operands with their own gates.
template <bool kBits>
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
  auto digits_of = [](int stored) { return kBits ? (stored >> 1) : stored; };  // (-1 stays -1)
#pragma unroll
  for (int j = 0; j < MBQ_MAX_GROUP; ++j) {
    const int d = digits_of(pl[j]);
    pmax[j] = (__ballot(d == 3) != 0ull) ? 3 : (__ballot(d == 2) != 0ull) ? 2 : (__ballot(d == 1) != 0ull) ? 1 : 0;
  }
  auto pmax_of = [&](int j) { return j == 0 ? pmax[0] : j == 1 ? pmax[1] : j == 2 ? pmax[2] : pmax[3]; };
  load_rest((int)blockIdx.x, wave, pmax_of(proj_of((int)blockIdx.x)), A);
  if (blockIdx.x == 0 && wave == 0) {
#pragma unroll
    for (int j = 0; j < MBQ_MAX_GROUP; ++j)
      if (j < g.n && g.p[j].perm != nullptr) bucket_by_wave(digits_of(pl[j]), lane, g.p[j].perm, g.p[j].offsets);
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
    auto gate_of = [](int d) {  // slices 0..d
      return (d >= 3) ? 0xFFFFFFFFu : (d == 2) ? 0x00FFFFFFu : (d == 1) ? 0x0000FFFFu : (d == 0) ? 0x000000FFu : 0u;
    };
    // kBits: pa + 1 bits; the high bit of digit e counts from 2 e + 1 bits on, its low bit from 2 e + 2
    const uint32_t gate = kBits ? gate_of(pa >= 0 ? pa >> 1 : -1) : gate_of(pa);
    const uint32_t gate_lo = kBits ? gate_of(pa >= 0 ? ((pa + 1) >> 1) - 1 : -1) : 0u;
    float kp[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int p = __shfl(plv, 4 * kq + i, 64);
      if constexpr (kBits) kp[i] = __builtin_ldexpf(1.f, -max(p, 0));  // 2^(1 - bits)
      else kp[i] = (p >= 3) ? 0.0078125f : (p == 2) ? 0.03125f : (p == 1) ? 0.125f : 0.5f;
    }
    const Item& I = cu.w;
    const int sa = (int)(((uint32_t)cu.scale * 0x01010101u) & gate);
    const int sa2 = (int)(((uint32_t)max(cu.scale - kPieceShift, 0) * 0x01010101u) & gate);
    floatx4 D0 = zero4, D1 = zero4;
    if constexpr (kBits) {
      const int sl = (int)(((uint32_t)cu.scale * 0x01010101u) & gate_lo);
      const int sl2 = (int)(((uint32_t)max(cu.scale - kPieceShift, 0) * 0x01010101u) & gate_lo);
      const uint32_t mask_hi = nib_mask & 0xAAAAAAAAu, mask_lo = nib_mask & 0x55555555u;
      auto planes = [&](auto e_tag) {
        constexpr int E = decltype(e_tag)::value;
        if (E > pm) return;
        D0 = slice_group<E>(cu.xa[0], I.w[E].x, I.w[E].y, mask_hi, sa, sa2, sb, D0);
        D1 = slice_group<E>(cu.xa[1], I.w[E].z, I.w[E].w, mask_hi, sa, sa2, sb, D1);
        D0 = slice_group<E>(cu.xa[0], I.w[E].x, I.w[E].y, mask_lo, sl, sl2, sb, D0);
        D1 = slice_group<E>(cu.xa[1], I.w[E].z, I.w[E].w, mask_lo, sl, sl2, sb, D1);
      };
      planes(std::integral_constant<int, 0>{});
      planes(std::integral_constant<int, 1>{});
      planes(std::integral_constant<int, 2>{});
      planes(std::integral_constant<int, 3>{});
    } else {
      D0 = slice_group<0>(cu.xa[0], I.w[0].x, I.w[0].y, nib_mask, sa, sa2, sb, zero4);
      D1 = slice_group<0>(cu.xa[1], I.w[0].z, I.w[0].w, nib_mask, sa, sa2, sb, zero4);
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

int f4_compute_units() { return device_compute_units(); }

bool decode_f4_supports(int64_t T, const Shape& sh) { return T >= 1 && T <= 16; }
bool decode_f4_takes_bit_view(int64_t T, const Shape& sh) { return decode_f4_supports(T, sh); }
int decode_f4_timeline_workgroups() { return f4_compute_units(); }
int decode_f4_timeline_slots() { return decode_f4_ws_stamp_wavefronts() * 32; }
// Parts of the K axis the linear kernel works in (2: it adds into Y, which must be zero when it starts; see
// decode_f4_zero_list).
static int call_tiles(int n, const Shape* shapes) {
  int tiles = 0;
  for (int i = 0; i < n; ++i) tiles += shapes[i].NT;
  return tiles;
}
int decode_f4_k_parts(int n, const Shape* shapes) {
  return decode_f4_ws_supports(shapes[0].KB, call_tiles(n, shapes)) ? decode_f4_ws_parts(shapes[0].KB) : 1;
}
void decode_f4_zero_list(int64_t T, int n, const Shape* shapes, float* const* Y, ZeroList* zl) {
  for (int i = 0; i < MBQ_MAX_GROUP; ++i) {
    zl->p[i] = nullptr;
    zl->n[i] = 0;
  }
  if (decode_f4_k_parts(n, shapes) != 2) return;
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
                                   int32_t* const* perm, int32_t* const* offsets, unsigned long long* stamps,
                                   bool bit_view) {
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
  g.bit_view = bit_view ? 1 : 0;
  const Shape& s0 = shapes[0];
  if (decode_f4_ws_supports(s0.KB, tiles)) return launch_linear_decode_f4_ws(T, g, s0.KB, ws, stream);
  if (stamps) {
    set_error("the timeline build exists for K <= 8192 only");
    return MBQ_ERR_BAD_SHAPE;
  }
  int grid = f4_compute_units();
  if (grid > tiles) grid = tiles;
  if (bit_view)
    hipLaunchKernelGGL(decode_f4_stream_kernel<true>, dim3(grid), dim3(512), 0, stream,
                       reinterpret_cast<const char*>(ws), (int)T, s0.KB, g);
  else
    hipLaunchKernelGGL(decode_f4_stream_kernel<false>, dim3(grid), dim3(512), 0, stream,
                       reinterpret_cast<const char*>(ws), (int)T, s0.KB, g);
  return hip_status(hipGetLastError(), "decode_f4_kernel launch");
}

}  // namespace mbq
