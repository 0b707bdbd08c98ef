// Decode-side routed linear for one token tile (T <= 16) and up to MBQ_MAX_GROUP weight
// matrices that read the SAME activations (q/k/v or gate/up of a decoder block), K <= 4096.
//
// Paper Sec. 4.2 Eq. 6 evaluated slice by slice, Y_i = sum_{e <= p_i} W_e^T X_i, with the
// shared-scale structure of App. B (s_e = s0/4^e, z_e = 2 for e >= 1); a tile fetches only
// slices 0..max_i p_i of its own matrix (Sec. 4.3, on-demand slice access), and the matrices of
// one call share one launch and one pass over the activations (Sec. 4.3, fused launch for the
// projections of a layer).
//
// Work split: the 16-row code tiles of all matrices form one list; a workgroup of 8 wavefronts
// owns tiles blockIdx.x, blockIdx.x + gridDim.x, ...  Wavefront w owns the 256-column blocks
// w and w + 8 (CPW = 2) of every tile, keeps their activation fragments in registers for the
// whole kernel and streams only packed weights, always fetching the next tile before consuming
// the current one.  The load count per tile is fixed (a slice that the tile does not need is
// replaced by a second load of slice pmax, which hits in the vector cache), so that the
// hardware wait counters let the next tile's loads stay in flight.
//
// Arithmetic as in the single-matrix kernel: a 2-bit field is OR-ed into the mantissa of a
// bf16 power of two chosen per slice and field position (operand = beta + c / 4^e exactly),
// tokens are the 16 rows of the v_mfma_f32_16x16x32_bf16 A operand, all slices of a group
// chain into one accumulator and a row of precision p keeps the value the accumulator had
// after slice p.  With Sa, Sb the sums of x over the columns that meet the two bias patterns,
//   y += s0 * (v - a_p Sa - b_p Sb) - s0 z0 (Sa + Sb),
// a_p, b_p = accumulated biases of slices 0..p plus the zero-point constant 1.5 q_p - 0.5,
// q_p = sum_{1 <= e <= p} 4^-e.
#include "mbq_common.h"

namespace mbq {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace dg {

constexpr int kWaves = 8;
constexpr int kStageStride = 272;  // bytes between token rows of the staging area (256 + 16: no bank conflicts)

struct Proj {
  const uint4* codes;
  const float2* meta;
  const int32_t* prec;
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
};

__device__ inline floatx4 mfma(const uint4& a, const uint4& b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                 c, 0, 0, 0);
}

template <int R>
__device__ inline uint32_t rotr(uint32_t w) {
  if constexpr (R == 0) return w;
  return __builtin_amdgcn_alignbit(w, w, R);
}

// (t & mask) | bias is one v_and_or_b32 only when neither operand is a literal, so the field
// masks and the bf16-pair biases 2^5, 2^3, 2^1, 2^-1 are kept in registers, made opaque to
// constant folding once at kernel entry.
struct UnpackConsts {
  uint32_t mask[3];  // 0x00030003 << 0, 2, 4
  uint32_t bias[4];
};

__device__ inline UnpackConsts make_unpack_consts() {
  UnpackConsts c;
  c.mask[0] = 0x00030003u; c.mask[1] = 0x000C000Cu; c.mask[2] = 0x00300030u;
  c.bias[0] = 0x42004200u; c.bias[1] = 0x41004100u; c.bias[2] = 0x40004000u; c.bias[3] = 0x3F003F00u;
#pragma unroll
  for (int i = 0; i < 3; ++i) asm volatile("" : "+s"(c.mask[i]));
#pragma unroll
  for (int i = 0; i < 4; ++i) asm volatile("" : "+v"(c.bias[i]));
  return c;
}

// B operands (a-step, b-step) of the two k-steps held by one dword of slice E.  The unrotated
// field of (step, slot s = 2j + h) sits at bit 16h + 4j + 2 step; slice E is stored rotated left
// by 2 - 2E.  Slice 0 is consumed one field position up.  Operand values:
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
__device__ inline floatx4 slice_group(const uint4* A, const UnpackConsts& uc, uint32_t w_lo, uint32_t w_hi,
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

struct Item {  // one 16 x 256 block: four slices and the {s0, z0} of its two groups
  uint4 w[4];
  float2 mt[2];
};

}  // namespace dg

template <int CPW>
__global__ __launch_bounds__(dg::kWaves * 64) void decode_group_kernel(const uint16_t* __restrict__ X, int T,
                                                                        int64_t K, int KB, const dg::Group g) {
  using namespace dg;
  constexpr int kAreaBytes = (CPW * 4096 > 16 * kStageStride) ? CPW * 4096 : 16 * kStageStride;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m = lane & 15;   // token row of A / weight row of B / output column
  const int kq = lane >> 4;  // k quarter of a k-step; output rows 4 kq .. 4 kq + 3
  const int my_tiles = (g.tiles - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
  if (my_tiles <= 0) return;

  __shared__ float red[2][kWaves][64][4];  // per-wavefront partial tiles, double buffered
  // Private to each wavefront: first the staging rows of an activation half block, afterwards
  // the column sums Sa, Sb of its blocks' groups: [CPW][2 groups][2][64 lanes] floatx4.
  __shared__ __attribute__((aligned(16))) char area[kWaves][kAreaBytes];
  char* const stage = area[wave];
  floatx4* const sums = reinterpret_cast<floatx4*>(area[wave]);

  // ---- precisions of every matrix (the first loads issued: what depends on them waits least) ----
  int pl[MBQ_MAX_GROUP];
#pragma unroll
  for (int j = 0; j < MBQ_MAX_GROUP; ++j) pl[j] = (j < g.n && lane < T) ? g.p[j].prec[lane] : -1;

  // ---- activations: whole cache lines per quarter wavefront, raw for now ----
  // block c of this wavefront is wave + 8 c; a block past the end contributes zeros and its
  // weight loads are pointed at block 0 of the tile.
  uint4 xa[CPW][8];
  int kb_of[CPW];
#pragma unroll
  for (int c = 0; c < CPW; ++c) {
    const int kb = wave + kWaves * c;
    const bool there = kb < KB;
    kb_of[c] = there ? kb : 0;
    const int64_t k0 = (int64_t)kb_of[c] * kTileK + 8 * m;
    const int second = (k0 + 128 < K) ? 128 : 0;  // K is a multiple of 128
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = min(4 * i + kq, T - 1);  // always a valid address
      const uint16_t* src = X + (int64_t)row * K + k0;
      xa[c][i] = *reinterpret_cast<const uint4*>(src);
      xa[c][4 + i] = *reinterpret_cast<const uint4*>(src + second);
    }
  }

  auto proj_of = [&](int t) {
    int j = 0;
#pragma unroll
    for (int i = 1; i < MBQ_MAX_GROUP; ++i)
      if (i < g.n && t >= g.p[i].tile_begin) j = i;
    return j;
  };
  auto load_base = [&](int t, Item (&I)[CPW]) {
    const Proj& P = g.p[proj_of(t)];
    const int nt = t - P.tile_begin;
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
      I[c].w[0] = P.codes[((size_t)nt * KB + kb_of[c]) * 64 + lane];
      I[c].mt[0] = P.meta[((size_t)nt * (2 * KB) + 2 * kb_of[c]) * kTileN + m];
      I[c].mt[1] = P.meta[((size_t)nt * (2 * KB) + 2 * kb_of[c] + 1) * kTileN + m];
    }
  };
  auto load_rest = [&](int t, int pm, Item (&I)[CPW]) {
    const Proj& P = g.p[proj_of(t)];
    const int nt = t - P.tile_begin;
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
      const size_t tile = ((size_t)nt * KB + kb_of[c]) * 64 + lane;
#pragma unroll
      for (int e = 1; e < 4; ++e) I[c].w[e] = P.codes[(size_t)min(e, pm) * P.slice_vec + tile];
    }
  };
  Item cur[CPW], nxt[CPW];
  load_base((int)blockIdx.x, cur);

  // ---- routing facts: highest precision present per matrix ----
  int pmax[MBQ_MAX_GROUP];
#pragma unroll
  for (int j = 0; j < MBQ_MAX_GROUP; ++j)
    pmax[j] = (__ballot(pl[j] == 3) != 0ull) ? 3 : (__ballot(pl[j] == 2) != 0ull) ? 2 : (__ballot(pl[j] == 1) != 0ull) ? 1 : 0;
  auto pmax_of = [&](int j) { return j == 0 ? pmax[0] : j == 1 ? pmax[1] : j == 2 ? pmax[2] : pmax[3]; };
  load_rest((int)blockIdx.x, pmax_of(proj_of((int)blockIdx.x)), cur);

  const UnpackConsts uc = make_unpack_consts();
  const uint4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};

  // ---- activations into the MFMA A layout (token = lane % 16) through the staging rows, then
  //      the column sums of every group in accumulator layout ----
#pragma unroll
  for (int c = 0; c < CPW; ++c) {
    const int kb = wave + kWaves * c;
    const bool there = kb < KB;
    const bool second = (int64_t)kb * kTileK + 128 < K;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool live = there && (4 * i + kq < T) && (h == 0 || second);
        *reinterpret_cast<floatx4*>(stage + (4 * i + kq) * kStageStride + 16 * m) =
            live ? __builtin_bit_cast(floatx4, xa[c][4 * h + i]) : zero4;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j)
        xa[c][4 * h + j] = __builtin_bit_cast(
            uint4, *reinterpret_cast<const floatx4*>(stage + m * kStageStride + 64 * j + 16 * kq));
    }
  }
#pragma unroll
  for (int c = 0; c < CPW; ++c)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      floatx4 Sa = mfma(xa[c][4 * h + 0], ones, zero4);
      Sa = mfma(xa[c][4 * h + 2], ones, Sa);
      floatx4 Sb = mfma(xa[c][4 * h + 1], ones, zero4);
      Sb = mfma(xa[c][4 * h + 3], ones, Sb);
      sums[((c * 2 + h) * 2 + 0) * 64 + lane] = Sa;
      sums[((c * 2 + h) * 2 + 1) * 64 + lane] = Sb;
    }

  // one step: fetch tile ti+1 into `n`, consume tile ti from `c`, reduce and store
  auto step = [&](int ti, Item (&cu)[CPW], Item (&nx)[CPW]) {
    const int t = (int)blockIdx.x + ti * (int)gridDim.x;
    const int tn = (int)blockIdx.x + min(ti + 1, my_tiles - 1) * (int)gridDim.x;
    load_base(tn, nx);
    load_rest(tn, pmax_of(proj_of(tn)), nx);

    const int j = proj_of(t);
    const int pm = pmax_of(j);
    const int plv = j == 0 ? pl[0] : j == 1 ? pl[1] : j == 2 ? pl[2] : pl[3];
    int prow[4];
    float ca[4], cb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int p = __shfl(plv, 4 * kq + i, 64);
      prow[i] = p;
      ca[i] = (p >= 3) ? 73.9921875f : (p == 2) ? 71.96875f : (p == 1) ? 63.875f : 31.5f;
      cb[i] = (p >= 3) ? 18.4921875f : (p == 2) ? 17.96875f : (p == 1) ? 15.875f : 7.5f;
    }
    floatx4 acc = zero4;
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
      const Item& I = cu[c];
      // the two groups of the block run as two independent accumulator chains
      floatx4 D[2], v[2];
      D[0] = slice_group<0>(&xa[c][0], uc, I.w[0].x, I.w[0].y, zero4);
      D[1] = slice_group<0>(&xa[c][4], uc, I.w[0].z, I.w[0].w, zero4);
      v[0] = D[0];
      v[1] = D[1];
      if (pm >= 1) {
        D[0] = slice_group<1>(&xa[c][0], uc, I.w[1].x, I.w[1].y, D[0]);
        D[1] = slice_group<1>(&xa[c][4], uc, I.w[1].z, I.w[1].w, D[1]);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int i = 0; i < 4; ++i) v[h][i] = (prow[i] >= 1) ? D[h][i] : v[h][i];
      }
      if (pm >= 2) {
        D[0] = slice_group<2>(&xa[c][0], uc, I.w[2].x, I.w[2].y, D[0]);
        D[1] = slice_group<2>(&xa[c][4], uc, I.w[2].z, I.w[2].w, D[1]);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int i = 0; i < 4; ++i) v[h][i] = (prow[i] >= 2) ? D[h][i] : v[h][i];
      }
      if (pm >= 3) {
        D[0] = slice_group<3>(&xa[c][0], uc, I.w[3].x, I.w[3].y, D[0]);
        D[1] = slice_group<3>(&xa[c][4], uc, I.w[3].z, I.w[3].w, D[1]);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int i = 0; i < 4; ++i) v[h][i] = (prow[i] >= 3) ? D[h][i] : v[h][i];
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const float s0 = I.mt[h].x, s0z0 = I.mt[h].x * I.mt[h].y;
        const floatx4 Sa = sums[((c * 2 + h) * 2 + 0) * 64 + lane];
        const floatx4 Sb = sums[((c * 2 + h) * 2 + 1) * 64 + lane];
#pragma unroll
        for (int i = 0; i < 4; ++i)
          acc[i] += s0 * (v[h][i] - ca[i] * Sa[i] - cb[i] * Sb[i]) - s0z0 * (Sa[i] + Sb[i]);
      }
    }
    // sum the wavefronts' partial tiles; rows leave in token order
    const int buf = ti & 1;
#pragma unroll
    for (int i = 0; i < 4; ++i) red[buf][wave][lane][i] = acc[i];
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
  };
#pragma unroll 1
  for (int ti = 0; ti < my_tiles; ti += 2) {
    step(ti, cur, nxt);
    if (ti + 1 < my_tiles) step(ti + 1, nxt, cur);
  }
}

static int group_compute_units() {
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

bool decode_group_supports(int64_t T, const Shape& sh) { return T >= 1 && T <= 16 && sh.KB <= 2 * dg::kWaves; }

// All matrices share K (the caller has checked); T <= 16, KB <= 16.
mbq_status launch_linear_decode_group(const uint16_t* X, int64_t T, int n, const void* const* blobs,
                                      const Shape* shapes, const int32_t* const* prec, float* const* Y,
                                      hipStream_t stream) {
  dg::Group g;
  int tiles = 0;
  for (int i = 0; i < MBQ_MAX_GROUP; ++i) {
    const int j = i < n ? i : 0;
    const Shape& sh = shapes[j];
    g.p[i].codes = reinterpret_cast<const uint4*>(blobs[j]);
    g.p[i].meta = reinterpret_cast<const float2*>(reinterpret_cast<const char*>(blobs[j]) + sh.meta_offset);
    g.p[i].prec = prec[j];
    g.p[i].Y = Y[j];
    g.p[i].slice_vec = sh.slice_words / 4;
    g.p[i].N = sh.N;
    g.p[i].tile_begin = tiles;
    g.p[i].pad = 0;
    if (i < n) tiles += sh.NT;
  }
  g.n = n;
  g.tiles = tiles;
  const Shape& s0 = shapes[0];
  int per_cu = knob(2) > 0 ? knob(2) : 1;
  int grid = group_compute_units() * per_cu;
  if (grid > tiles) grid = tiles;
  if (s0.KB <= dg::kWaves)
    hipLaunchKernelGGL(decode_group_kernel<1>, dim3(grid), dim3(dg::kWaves * 64), 0, stream, X, (int)T, s0.K, s0.KB,
                       g);
  else
    hipLaunchKernelGGL(decode_group_kernel<2>, dim3(grid), dim3(dg::kWaves * 64), 0, stream, X, (int)T, s0.K, s0.KB,
                       g);
  return hip_status(hipGetLastError(), "decode_group_kernel launch");
}

}  // namespace mbq
