// Internal definitions shared by the translation units of libmbq.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mbq.h"

namespace mbq {

constexpr int kGroup = 128;    // input features per quantisation group (paper App. C.1)
constexpr int kSlices = 4;     // E, number of 2-bit slices (paper Sec. 4.1 default)
constexpr int kTileN = 16;     // rows of one code tile
constexpr int kTileK = 256;    // columns of one code tile
constexpr int kTileWords = 256;  // uint32 words of one code tile of one slice (64 lanes x 4)
constexpr int kMaxDecodeTokens = 64;
constexpr int kMaxKSplit = 8;

// Geometry of the packed blob of an N x K matrix.
struct Shape {
  int64_t N, K;
  int NT;               // row tiles, ceil(N / 16)
  int KB;               // column tiles, ceil(K / 256)
  int G;                // real groups per row, K / group
  size_t slice_words;   // uint32 words of one slice = NT * KB * 256
  size_t meta_offset;   // byte offset of the {s0, z0} section
  size_t bytes;         // total blob bytes
  int group;            // columns per quantisation group: 128, or 64 / 32 (configurations; slow kernels only)
  int gshift;           // log2(group)
};

// false (and error set) if invalid
bool make_shape(int64_t N, int64_t K, Shape* out, int group = kGroup);
void set_error(const char* fmt, ...);
mbq_status hip_status(hipError_t e, const char* what);
int knob(int index);  // the calling thread's snapshot of the hooks, taken by the outermost ApiScope
// Every entry point that dispatches opens one; the outermost on a thread snapshots the test/experiment hooks, so
// all decisions of one call (also of the calls it makes in turn) see the same values.
// Compute units of the CURRENT device (asked once per device; 256 if the query fails).  Launch shapes are sized
// by it, so a process that drives several devices gets each device's own figure.
int device_compute_units();

struct ApiScope {
  ApiScope();
  ~ApiScope();
};

// ---- blob addressing (device + host) -------------------------------------------
// Word index, inside one slice, of the dword holding weight (n, k).
__host__ __device__ inline size_t code_word(int NT, int KB, int64_t n, int64_t k) {
  const int r = (int)(k & 255);
  const int d = r >> 6;
  const int kq = (r & 31) >> 3;
  const int lane = 16 * kq + (int)(n & 15);
  return ((size_t)(n >> 4) * KB + (size_t)(k >> 8)) * kTileWords + (size_t)lane * 4 + d;
}
// Bit position of the 2-bit field of weight column k in slice e's (rotated) dword.
__host__ __device__ inline int code_bit(int e, int64_t k) {
  const int r = (int)(k & 255);
  const int step = (r & 63) >> 5;
  const int s = r & 7;
  return (16 * (s & 1) + 4 * (s >> 1) + 2 * step + 2 - 2 * e) & 31;
}
// Index of the float2 {s0, z0} of (row n, group g) inside the meta section; per_tile = groups per 256 columns.
__host__ __device__ inline size_t meta_index(int KB, int64_t n, int g, int per_tile = 2) {
  return ((size_t)(n >> 4) * (per_tile * KB) + g) * kTileN + (size_t)(n & 15);
}

// Output arrays that the activation-preparation launch clears for a linear kernel that adds into
// them (all null: nothing to clear).
struct ZeroList {
  float* p[MBQ_MAX_GROUP];
  long long n[MBQ_MAX_GROUP];  // floats
};

// How a router's outputs map onto the blob's eight-bit code (Sec. 4.1 with other slice widths, App. C.1): the router
// has P outputs (one per slice of the configuration) and output q stands for the first bits[q] bits of the code.
// digits[q] = base-4 digits that precision touches, minus one (what the tokens are sorted and bucketed by, and what the
// weight loaders go by).  A precision array holds value[q]: digits[q] when every bits[q] is even (the linear kernels'
// native precision), bits[q] - 1 otherwise (a token may then stop at the high bit of its last digit; only the kernels
// that say so understand that); shift = 0 / 1 turns a stored value back into digits.
// Default: four outputs of 2, 4, 6, 8 bits.
struct RouteView {
  int P;
  int bits[MBQ_N_PRECISIONS];
  int digits[MBQ_N_PRECISIONS];
  int value[MBQ_N_PRECISIONS];
  int shift;
  int group;  // columns per quantisation group (the routers do not care; the blob's metadata section does)
};
constexpr RouteView kDefaultView = {MBQ_N_PRECISIONS, {2, 4, 6, 8}, {0, 1, 2, 3}, {0, 1, 2, 3}, 0, kGroup};

// ---- kernels' host launchers (each enqueues on `stream`, returns a status) ------
mbq_status launch_encode(const float* W, const Shape& sh, void* blob, const float* ext_scale, const float* ext_zero,
                         hipStream_t stream);
// groups of 64 or 32 columns (sh.group): same code section, a metadata section of 256 / group pairs per tile row
mbq_status launch_encode_small_group(const float* W, const Shape& sh, void* blob, hipStream_t stream);
mbq_status launch_unpack(const void* blob, const Shape& sh, uint8_t* codes, float* scale, float* zero,
                         hipStream_t stream);
mbq_status launch_dequant(const void* blob, const Shape& sh, int p, float* What, hipStream_t stream);
mbq_status launch_dequant_bits(const void* blob, const Shape& sh, int bits, float* What, hipStream_t stream);
mbq_status launch_unpack_view(const void* blob, const Shape& sh, const RouteView& view, uint8_t* codes, float* scale,
                              float* zero, hipStream_t stream);
mbq_status launch_route(const uint16_t* X, int64_t T, int64_t K, const float* Wr, const float* br,
                        int32_t* prec, int32_t* perm, int32_t* offsets, double* logits, void* ws,
                        hipStream_t stream, const RouteView& view = kDefaultView);
mbq_status launch_route_group(const uint16_t* X, int64_t T, int64_t K, int n, const float* const* Wr,
                              const float* const* br, int32_t* const* prec, int32_t* const* perm,
                              int32_t* const* offsets, double* const* logits, void* ws, hipStream_t stream,
                              void* prep, int prep_blocks, const ZeroList* zl, bool defer_bucket,
                              const RouteView& view = kDefaultView, const uint16_t* Xprep = nullptr);
bool route_can_carry_prep(int64_t T);
bool route_defers_sort(int64_t T);
mbq_status launch_route_mlp(const uint16_t* X, int64_t T, int64_t K, const float* W1, const float* b1, int H,
                            const float* W2, const float* b2, double delta, int32_t* prec, int32_t* perm,
                            int32_t* offsets, double* scores, void* ws, hipStream_t stream);
int route_mlp_max_hidden();
size_t route_mlp_workspace_bytes(int64_t T, int H);
mbq_status launch_threshold_quantile(const double* scores, int64_t T, long long k, double* delta_out,
                                     hipStream_t stream);
mbq_status launch_linear_simple(const uint16_t* X, int64_t T, const void* blob, const Shape& sh,
                                const int32_t* prec, float* Y, hipStream_t stream, bool bit_view = false);
mbq_status launch_linear_decode(const uint16_t* X, int64_t T, const void* blob, const Shape& sh,
                                const int32_t* perm, const int32_t* offsets, float* Y, void* ws,
                                hipStream_t stream);
mbq_status launch_linear_prefill(const uint16_t* X, int64_t T, const void* blob, const Shape& sh,
                                 const int32_t* perm, const int32_t* offsets, float* Y, void* ws,
                                 hipStream_t stream, bool mix_gate = false);
mbq_status launch_linear_decode16(const uint16_t* X, int64_t T, const void* blob, const Shape& sh,
                                  const int32_t* prec, const int32_t* perm, float* Y, hipStream_t stream);
// the same for up to MBQ_MAX_GROUP matrices over one X (one K), each with its own routing, in one launch
// Outputs that launch_linear_decode16(_group) ADDS into for this call (K split of small outputs): the caller clears
// them first, with launch_zero_outputs or through the router launch.
void decode16_zero_list(int64_t T, int n, const Shape* shapes, float* const* Y, ZeroList* zl);
mbq_status launch_zero_outputs(const ZeroList& zl, hipStream_t stream);
// sort_perm / sort_offsets (arrays of n, or null): the tokens are not sorted yet (perm is ignored); the launch sorts
// them by the precisions itself and writes the order and the bucket offsets there (T <= 128)
mbq_status launch_linear_decode16_group(const uint16_t* X, int64_t T, int n, const void* const* blobs,
                                        const Shape* shapes, const int32_t* const* prec, const int32_t* const* perm,
                                        float* const* Y, hipStream_t stream, int32_t* const* sort_perm,
                                        int32_t* const* sort_offsets, const int32_t* const* gate_offsets = nullptr);
bool decode_f4_supports(int64_t T, const Shape& sh);
int decode_f4_k_parts(int n, const Shape* shapes);
void decode_f4_zero_list(int64_t T, int n, const Shape* shapes, float* const* Y, ZeroList* zl);
// share `part` of `parts` of the clearing, done by `nthreads` threads of which this is `tid`
// Between 129 and 256 tokens the better of the register-stationary kernel and the prefill kernel depends on the
// precision mix, which only the device knows; both are launched and each asks this question about the bucket
// offsets first, the one that is not wanted returns at once.  The stationary kernel walks the sorted tokens in
// passes of at most 32 and reads slices 0..p of the pass's last token: it is taken when that is two slices per pass
// or fewer on average (measured on the 70B-shaped linears at 256 tokens: {70,20,8,2}% mix 0.38 ms against 0.46 for
// the prefill kernel, uniform mix 0.44 against 0.41).
__device__ inline bool mix_prefers_stationary(const int32_t* __restrict__ offsets, int T) {
  const int o1 = offsets[1], o2 = offsets[2], o3 = offsets[3];
  const int passes = (T + 31) / 32, per_pass = (T + passes - 1) / passes;
  int slices = 0;
  for (int y = 0; y < passes; ++y) {
    const int last = min(T, per_pass * (y + 1)) - 1;
    slices += 1 + (last >= o1) + (last >= o2) + (last >= o3);
  }
  return slices <= 2 * passes;
}
// A 16-byte load of data that a launch reads once (packed weights in the decode kernels), with the
// non-temporal hint: the stream then does not push the activations, router parameters and outputs that
// the neighbouring launches share out of the caches.
__device__ __forceinline__ uint4 load_once(const uint4* p) {
  typedef uint32_t u32x4_nt __attribute__((ext_vector_type(4)));
  const u32x4_nt v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt*>(p));
  return uint4{v.x, v.y, v.z, v.w};
}
__device__ inline void zero_share(const ZeroList& zl, int part, int parts, int tid, int nthreads) {
#pragma unroll
  for (int j = 0; j < MBQ_MAX_GROUP; ++j) {
    float* p = zl.p[j];
    if (p == nullptr) continue;
    const long long n = zl.n[j];
    for (long long i = (long long)part * nthreads + tid; i < n; i += (long long)parts * nthreads) p[i] = 0.f;
  }
}
size_t decode_f4_workspace_bytes(int64_t T, const Shape& sh);
mbq_status launch_decode_f4_prep(const uint16_t* X, int64_t T, int64_t K, int KB, void* ws, const ZeroList& zl,
                                 hipStream_t stream);
// perm/offsets (arrays of n, or null): the launch also sorts the tokens of every matrix by precision
mbq_status launch_linear_decode_f4(int64_t T, int n, const void* const* blobs, const Shape* shapes,
                                   const int32_t* const* prec, float* const* Y, const void* ws, hipStream_t stream,
                                   int32_t* const* perm, int32_t* const* offsets, unsigned long long* stamps = nullptr,
                                   bool bit_view = false);
// bit_view (the precision arrays hold bits - 1, see RouteView) is understood by the one-token-tile kernels only
bool decode_f4_takes_bit_view(int64_t T, const Shape& sh);
// timeline build of the ring kernel: workgroups it launches at most, and 8-byte slots each of them writes
int decode_f4_timeline_workgroups();
int decode_f4_timeline_slots();
// activation-quantised variant (App. E.4): per-token quantiser and the row scaling that finishes the main path
mbq_status launch_act_quant(const uint16_t* X, int64_t T, int64_t K, int abits, const float* let_shift,
                            const float* let_scale, uint16_t* Xint, float* row_scale, uint16_t* Xr,
                            hipStream_t stream);
mbq_status launch_scale_rows(float* Y, int64_t T, int64_t N, const float* row_scale, const float* bias,
                             hipStream_t stream);
// the same for the outputs of up to MBQ_MAX_GROUP projections in one launch (bias: array of n, entries may be null)
mbq_status launch_scale_rows_group(int n, float* const* Y, int64_t T, const int64_t* N, const float* row_scale,
                                   const float* const* bias, hipStream_t stream);
size_t decode_workspace_bytes(int64_t T, const Shape& sh);
size_t prefill_workspace_bytes(int64_t T, const Shape& sh);

}  // namespace mbq
