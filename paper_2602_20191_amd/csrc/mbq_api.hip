// C-ABI entry points of libmbq.so: argument checks, shape arithmetic, dispatch.
#include <stdarg.h>
#include <stdio.h>

#include <atomic>

#include "mbq_bench.h"
#include "mbq_common.h"

namespace mbq {

static thread_local char g_error[512] = "";
// Test and experiment hooks (mbq_set_knob).  A call takes one snapshot of them when it enters the library and
// dispatches on that snapshot only, so a change made by another thread never splits one call's decisions.
constexpr int kKnobs = 8;
static std::atomic<int> g_knobs[kKnobs];
static thread_local int t_knobs[kKnobs] = {0, 0, 0, 0, 0, 0, 0, 0};
static thread_local int t_depth = 0;
ApiScope::ApiScope() {
  if (t_depth++ == 0)
    for (int i = 0; i < kKnobs; ++i) t_knobs[i] = g_knobs[i].load(std::memory_order_relaxed);
}
ApiScope::~ApiScope() { --t_depth; }

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
}

mbq_status hip_status(hipError_t e, const char* what) {
  if (e == hipSuccess) return MBQ_OK;
  set_error("%s: %s", what, hipGetErrorString(e));
  return MBQ_ERR_HIP;
}

int knob(int index) { return (index >= 0 && index < kKnobs) ? t_knobs[index] : 0; }

bool make_shape(int64_t N, int64_t K, Shape* out, int group) {
  if (N <= 0 || K <= 0) {
    set_error("N and K must be positive (N=%lld, K=%lld)", (long long)N, (long long)K);
    return false;
  }
  if (K % kGroup != 0) {
    set_error("K=%lld is not a multiple of the group size %d", (long long)K, kGroup);
    return false;
  }
  if (N > (int64_t)1 << 24 || K > (int64_t)1 << 24 || N * K > (int64_t)1 << 36) {
    set_error("shape %lld x %lld is too large", (long long)N, (long long)K);
    return false;
  }
  Shape s;
  s.N = N;
  s.K = K;
  s.NT = (int)((N + kTileN - 1) / kTileN);
  s.KB = (int)((K + kTileK - 1) / kTileK);
  s.group = group;
  s.gshift = group == 128 ? 7 : (group == 64 ? 6 : 5);
  s.G = (int)(K / group);
  s.slice_words = (size_t)s.NT * s.KB * kTileWords;
  s.meta_offset = (size_t)kSlices * s.slice_words * 4;
  s.bytes = s.meta_offset + (size_t)s.NT * ((kTileK / group) * s.KB) * kTileN * 8;
  *out = s;
  return true;
}

int device_compute_units() {
  constexpr int kDevices = 64;
  static std::atomic<int> cached[kDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kDevices) return 256;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

static bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

// The slice configuration a call runs under (the *_cfg entry points set it for the duration of the call they forward
// to; everything else sees the default: four slices of two bits).
static thread_local const RouteView* t_view = &kDefaultView;
struct ViewScope {
  const RouteView* saved;
  explicit ViewScope(const RouteView* v) : saved(t_view) { t_view = v; }
  ~ViewScope() { t_view = saved; }
};
// The activations the linear kernels of a routed stage multiply when they are not the router's input (the
// activation-quantised stage call sets it for the duration of the call it forwards to; null: the router's input).
static thread_local const uint16_t* t_linear_X = nullptr;
struct LinearInputScope {
  explicit LinearInputScope(const uint16_t* x) { t_linear_X = x; }
  ~LinearInputScope() { t_linear_X = nullptr; }
};
// cfg -> view; the configurations this library runs are those that cut the blob's eight-bit code
static bool make_view(const mbq_config* cfg, RouteView* v, const char* who) {
  if (!cfg) {
    set_error("%s: null configuration", who);
    return false;
  }
  if (cfg->n_slices < 1 || cfg->n_slices > MBQ_MAX_SLICES) {
    set_error("%s: %d slices, supported 1..%d", who, cfg->n_slices, MBQ_MAX_SLICES);
    return false;
  }
  if (cfg->group != kGroup && cfg->group != 64 && cfg->group != 32) {
    set_error("%s: group size %d, supported: %d, 64, 32", who, cfg->group, kGroup);
    return false;
  }
  int bits = 0;
  bool odd = false;
  *v = kDefaultView;
  v->P = cfg->n_slices;
  for (int e = 0; e < cfg->n_slices; ++e) {
    const int b = cfg->slice_bits[e];
    if (b < 1 || bits + b > 2 * kSlices) {
      set_error("%s: slice %d has %d bits; supported: widths of at least 1 bit that add up to at most %d bits", who, e, b,
                2 * kSlices);
      return false;
    }
    bits += b;
    v->bits[e] = bits;
    v->digits[e] = (bits + 1) / 2 - 1;
    odd = odd || (bits & 1) != 0;
  }
  for (int e = cfg->n_slices; e < MBQ_N_PRECISIONS; ++e) {
    v->bits[e] = v->bits[cfg->n_slices - 1];
    v->digits[e] = v->digits[cfg->n_slices - 1];
  }
  v->shift = odd ? 1 : 0;
  v->group = cfg->group;
  for (int e = 0; e < MBQ_N_PRECISIONS; ++e) v->value[e] = odd ? v->bits[e] - 1 : v->digits[e];
  return true;
}

// Precision arrays that count bits (see RouteView) above one token tile: the one-token-tile decode kernels, which
// understand them, run once per 16 tokens - a pass over the weights each, far from the kernels of the digit
// configurations at these token counts, and three to four orders of magnitude from the one-thread-per-output kernel
// that would run otherwise.  The chunks follow each other on the stream and share the prepared-activation area.
static mbq_status bit_view_in_chunks(const uint16_t* X, int64_t T, int n, const void* const* blobs, const Shape* sh,
                                     const int32_t* const* prec, float* const* Y, void* ws, hipStream_t s) {
  for (int64_t t0 = 0; t0 < T; t0 += 16) {
    const int64_t tc = T - t0 < 16 ? T - t0 : 16;
    const int32_t* pc[MBQ_MAX_GROUP];
    float* yc[MBQ_MAX_GROUP];
    for (int i = 0; i < n; ++i) {
      pc[i] = prec[i] + t0;
      yc[i] = Y[i] + t0 * sh[i].N;
    }
    ZeroList zl;
    decode_f4_zero_list(tc, n, sh, yc, &zl);
    mbq_status st = launch_decode_f4_prep(X + t0 * sh[0].K, tc, sh[0].K, sh[0].KB, ws, zl, s);
    if (st != MBQ_OK) return st;
    st = launch_linear_decode_f4(tc, n, blobs, sh, pc, yc, ws, s, nullptr, nullptr, nullptr, true);
    if (st != MBQ_OK) return st;
  }
  return MBQ_OK;
}

// 17..64 tokens (and one token tile when the FP4-operand kernels are switched off): the register-stationary
// kernel, except for matrices with few row tiles (see dispatch_linear)
static bool takes_stationary_kernel(int64_t T, const Shape& sh) {
  // (re-measured with the K split of the stationary kernel: up to 32 column blocks it is as fast or faster - 1536 x
  // 5120 at 17..32 tokens 13 us against 16; beyond, few row tiles favour the other kernel - 1024 x 14336 16 us against 21)
  return knob(3) != 1 && (knob(3) == 2 || sh.KB <= 32 || sh.NT >= 128 || (T > 32 && sh.NT >= 32));
}

// Above the decode limit the register-stationary kernel still beats the prefill kernel for a while: it walks the
// weights once per 32 sorted tokens, the prefill kernel unpacks them once per bucket into 256-row tiles that are
// mostly empty at these token counts.  Measured, stationary / prefill in us per call:
//   4096 x 4096: 31 / 36 at 65 tokens, 25 / 39 at 128, 49 / 43 at 192;  14336 x 4096: 80 / 98, 68 / 102, 116 / 111;
//   4096 x 14336: 97 / 96, 82 / 106, 147 / 106;  28672 x 8192: 212 / 351, 237 / 370, 365 / 391;
//   1024 x 4096: 12 / 29, 12 / 33, 16 / 34, and 25 / 52 at 512 tokens.
// AUTO takes it up to 128 tokens, and up to 512 for matrices of at most 2048 code blocks of 16 x 256.
constexpr int kMaxStationaryTokens = 128, kMaxStationaryTokensSmall = 512;
constexpr int64_t kSmallMatrixBlocks = 2048;
// From there to 256 tokens the better kernel depends on the precision mix (see mix_prefers_stationary): both are
// launched and the device decides.
constexpr int kMaxByMixTokens = 256;
constexpr int kAlgoStationary = 100;  // internal: what AUTO resolves to in those ranges
constexpr int kAlgoByMix = 101;
static int resolve_auto(int64_t T, const Shape& sh) {
  if (T <= kMaxDecodeTokens) return MBQ_ALGO_DECODE;
  const int limit = (int64_t)sh.NT * sh.KB <= kSmallMatrixBlocks ? kMaxStationaryTokensSmall : kMaxStationaryTokens;
  const bool can = knob(3) == 0 && takes_stationary_kernel(T, sh);
  if (T <= limit && can) return kAlgoStationary;
  // (up to 32 column blocks: with more, the stationary kernel's per-chunk prologues cost it the advantage - 8192 x
  // 28672 at 256 tokens on the skewed mix 0.49 ms against 0.48)
  if (T <= kMaxByMixTokens && can && sh.KB <= 32) return kAlgoByMix;
  return MBQ_ALGO_PREFILL;
}

// algo is DECODE (T <= 64), PREFILL, SIMPLE, kAlgoStationary or kAlgoByMix here
mbq_status dispatch_linear(const uint16_t* X, int64_t T, const void* blob, const Shape& sh, const int32_t* prec,
                           const int32_t* perm, const int32_t* offsets, float* Y, void* ws, int algo,
                           hipStream_t s) {
  switch (algo) {
    case MBQ_ALGO_SIMPLE:
      return launch_linear_simple(X, T, blob, sh, prec, Y, s);
    case kAlgoByMix: {
      ZeroList zl;
      decode16_zero_list(T, 1, &sh, &Y, &zl);
      mbq_status st = launch_zero_outputs(zl, s);
      if (st != MBQ_OK) return st;
      st = launch_linear_decode16_group(X, T, 1, &blob, &sh, &prec, &perm, &Y, s, nullptr, nullptr, &offsets);
      if (st != MBQ_OK) return st;
      return launch_linear_prefill(X, T, blob, sh, perm, offsets, Y, ws, s, true);
    }
    case kAlgoStationary: {
      ZeroList zl;
      decode16_zero_list(T, 1, &sh, &Y, &zl);
      mbq_status st = launch_zero_outputs(zl, s);
      if (st != MBQ_OK) return st;
      return launch_linear_decode16(X, T, blob, sh, prec, perm, Y, s);
    }
    case MBQ_ALGO_DECODE:
      // One token tile (T <= 16): the FP4-operand kernels (activation preparation, then the
      // linear kernel).  17..64 tokens run the bf16-operand kernels, one pass per 16
      // precision-sorted tokens: the register-stationary chunked kernel, except for matrices with few
      // row tiles, where keeping every column block in flight (K split + reduction) fills the chip
      // better (measured on weights that are not in the last-level cache).
      if (knob(3) == 0 && decode_f4_supports(T, sh)) {
        ZeroList zl;
        decode_f4_zero_list(T, 1, &sh, &Y, &zl);
        mbq_status st = launch_decode_f4_prep(X, T, sh.K, sh.KB, ws, zl, s);
        if (st != MBQ_OK) return st;
        return launch_linear_decode_f4(T, 1, &blob, &sh, &prec, &Y, ws, s, nullptr, nullptr);
      }
      if (takes_stationary_kernel(T, sh)) {
        ZeroList zl;
        decode16_zero_list(T, 1, &sh, &Y, &zl);
        mbq_status st = launch_zero_outputs(zl, s);  // nothing to do unless the launch splits K
        if (st != MBQ_OK) return st;
        return launch_linear_decode16(X, T, blob, sh, prec, perm, Y, s);
      }
      return launch_linear_decode(X, T, blob, sh, perm, offsets, Y, ws, s);
    default:
      return launch_linear_prefill(X, T, blob, sh, perm, offsets, Y, ws, s);
  }
}

// ---- scratch memory of mbq_linear_static ---------------------------------------------------------------------------
// Device memory that belongs to the library image: every GPU the library runs on holds its own copy at its own address
// until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress, never an address.
static __device__ __align__(256) unsigned char scratch[MBQ_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

// the address of `scratch` on the current device (looked up once per device, with that device current)
static mbq_status scratch_on_current_device(void** out) {
  int dev = -1;
  mbq_status st = hip_status(hipGetDevice(&dev), "hipGetDevice");
  if (st != MBQ_OK) return st;
  if (dev < 0 || dev >= kMaxDevices) {
    set_error("mbq_linear_static: device index %d outside 0..%d", dev, kMaxDevices - 1);
    return MBQ_ERR_INVALID_ARG;
  }
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr == nullptr) {
    st = hip_status(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
    if (st != MBQ_OK) return st;
    if (ptr == nullptr) {
      set_error("mbq_linear_static: hipGetSymbolAddress returned a null address");
      return MBQ_ERR_HIP;
    }
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // (a second thread may look it up too: same value)
  }
  *out = ptr;
  return MBQ_OK;
}

}  // namespace mbq

using namespace mbq;

extern "C" {

size_t mbq_static_scratch_bytes(void) { return MBQ_STATIC_SCRATCH_BYTES; }

mbq_status mbq_linear_static(const uint16_t* X, int64_t T, const void* blob, int64_t N, int64_t K,
                             const int32_t* prec, const int32_t* perm, const int32_t* offsets, float* Y, int algo,
                             void* stream) {
  ApiScope scope;
  Shape sh;
  if (!make_shape(N, K, &sh)) return MBQ_ERR_BAD_SHAPE;
  if (T < 0 || T > (int64_t)1 << 24) {
    set_error("mbq_linear_static: bad token count %lld", (long long)T);
    return MBQ_ERR_BAD_SHAPE;
  }
  const size_t need = mbq_linear_workspace_bytes(T, N, K);
  if (need > (size_t)MBQ_STATIC_SCRATCH_BYTES) {
    set_error("mbq_linear_static: T=%lld, N=%lld, K=%lld needs %zu bytes of scratch memory, the built-in buffer holds "
              "%zu: use mbq_linear with a workspace of your own", (long long)T, (long long)N, (long long)K, need,
              (size_t)MBQ_STATIC_SCRATCH_BYTES);
    return MBQ_ERR_WORKSPACE;
  }
  if (T == 0) return mbq_linear(X, T, blob, N, K, prec, perm, offsets, Y, nullptr, 0, algo, stream);
  void* ws = nullptr;
  mbq_status st = scratch_on_current_device(&ws);
  if (st != MBQ_OK) return st;
  return mbq_linear(X, T, blob, N, K, prec, perm, offsets, Y, ws, (size_t)MBQ_STATIC_SCRATCH_BYTES, algo, stream);
}

const char* mbq_version(void) { return "mbq 0.1 (gfx950)"; }

const char* mbq_last_error(void) { return g_error; }

size_t mbq_blob_bytes(int64_t N, int64_t K) {
  Shape sh;
  return make_shape(N, K, &sh) ? sh.bytes : 0;
}

size_t mbq_route_workspace_bytes(int64_t T, int64_t K) {
  (void)T;
  (void)K;
  return 256;
}

size_t mbq_linear_workspace_bytes(int64_t T, int64_t N, int64_t K) {
  ApiScope scope;
  Shape sh;
  if (T < 0 || !make_shape(N, K, &sh)) return 0;
  size_t a = decode_workspace_bytes(T, sh);
  size_t b = prefill_workspace_bytes(T, sh);
  size_t c = decode_f4_workspace_bytes(T, sh);
  if (b > a) a = b;
  if (c > a) a = c;
  return a + 256;
}

mbq_status mbq_set_knob(int k, int value) {
  if (k < 0 || k >= kKnobs || k == 6) {
    set_error("unknown knob %d", k);
    return MBQ_ERR_INVALID_ARG;
  }
  g_knobs[k].store(value, std::memory_order_relaxed);
  return MBQ_OK;
}

mbq_status mbq_encode(const float* W, int64_t N, int64_t K, void* blob, void* stream) {
  Shape sh;
  if (!make_shape(N, K, &sh)) return MBQ_ERR_BAD_SHAPE;
  if (!W || !blob || !aligned(blob, 256) || !aligned(W, 16)) {
    set_error("mbq_encode: W must be 16-byte and blob 256-byte aligned and non-null");
    return MBQ_ERR_INVALID_ARG;
  }
  return launch_encode(W, sh, blob, nullptr, nullptr, (hipStream_t)stream);
}

mbq_status mbq_encode_with_params(const float* W, int64_t N, int64_t K, const float* scale, const float* zero,
                                  void* blob, void* stream) {
  Shape sh;
  if (!make_shape(N, K, &sh)) return MBQ_ERR_BAD_SHAPE;
  if (!W || !blob || !scale || !zero || !aligned(blob, 256) || !aligned(W, 16)) {
    set_error("mbq_encode_with_params: W must be 16-byte and blob 256-byte aligned; W, scale, zero, blob non-null");
    return MBQ_ERR_INVALID_ARG;
  }
  return launch_encode(W, sh, blob, scale, zero, (hipStream_t)stream);
}

mbq_status mbq_unpack(const void* blob, int64_t N, int64_t K, uint8_t* codes, float* scale, float* zero,
                      void* stream) {
  Shape sh;
  if (!make_shape(N, K, &sh)) return MBQ_ERR_BAD_SHAPE;
  if (!blob || !aligned(blob, 256)) {
    set_error("mbq_unpack: blob must be non-null and 256-byte aligned");
    return MBQ_ERR_INVALID_ARG;
  }
  return launch_unpack(blob, sh, codes, scale, zero, (hipStream_t)stream);
}

mbq_status mbq_dequant(const void* blob, int64_t N, int64_t K, int p, float* What, void* stream) {
  Shape sh;
  if (!make_shape(N, K, &sh)) return MBQ_ERR_BAD_SHAPE;
  if (!blob || !What || !aligned(blob, 256) || p < 0 || p >= MBQ_N_PRECISIONS) {
    set_error("mbq_dequant: null/misaligned pointer or precision index %d outside 0..3", p);
    return MBQ_ERR_INVALID_ARG;
  }
  return launch_dequant(blob, sh, p, What, (hipStream_t)stream);
}

mbq_status mbq_route(const uint16_t* X, int64_t T, int64_t K, const float* Wr, const float* br, int P,
                     int32_t* prec, int32_t* perm, int32_t* offsets, double* logits, void* ws,
                     size_t ws_bytes, void* stream) {
  ApiScope scope;
  if (P != t_view->P) {
    set_error("mbq_route: P=%d, the slice configuration has %d precisions", P, t_view->P);
    return MBQ_ERR_BAD_SHAPE;
  }
  if (T < 0 || K <= 0 || K % kGroup != 0 || T > (int64_t)1 << 24 || K > (int64_t)1 << 24) {
    set_error("mbq_route: bad sizes T=%lld K=%lld", (long long)T, (long long)K);
    return MBQ_ERR_BAD_SHAPE;
  }
  if (!offsets || (T > 0 && (!X || !Wr || !br || !prec || !perm)) || !aligned(X, 16) || !aligned(Wr, 16)) {
    set_error("mbq_route: null or misaligned pointer (X and Wr need 16-byte alignment)");
    return MBQ_ERR_INVALID_ARG;
  }
  if (ws_bytes < mbq_route_workspace_bytes(T, K) || !ws || !aligned(ws, 256)) {
    set_error("mbq_route: workspace too small or misaligned (%zu < %zu)", ws_bytes, mbq_route_workspace_bytes(T, K));
    return MBQ_ERR_WORKSPACE;
  }
  return launch_route(X, T, K, Wr, br, prec, perm, offsets, logits, ws, (hipStream_t)stream, *t_view);
}

mbq_status mbq_route_group(const uint16_t* X, int64_t T, int64_t K, int n_proj, const float* const* Wr_host,
                           const float* const* br_host, int P, int32_t* const* prec_host,
                           int32_t* const* perm_host, int32_t* const* offsets_host, void* ws, size_t ws_bytes,
                           void* stream) {
  ApiScope scope;
  if (P != t_view->P) {
    set_error("mbq_route_group: P=%d, the slice configuration has %d precisions", P, t_view->P);
    return MBQ_ERR_BAD_SHAPE;
  }
  if (n_proj < 1 || n_proj > MBQ_MAX_GROUP) {
    set_error("mbq_route_group: n_proj=%d outside 1..%d", n_proj, MBQ_MAX_GROUP);
    return MBQ_ERR_INVALID_ARG;
  }
  if (T < 0 || K <= 0 || K % kGroup != 0 || T > (int64_t)1 << 24 || K > (int64_t)1 << 24) {
    set_error("mbq_route_group: bad sizes T=%lld K=%lld", (long long)T, (long long)K);
    return MBQ_ERR_BAD_SHAPE;
  }
  if (!Wr_host || !br_host || !prec_host || !perm_host || !offsets_host || (T > 0 && (!X || !aligned(X, 16)))) {
    set_error("mbq_route_group: null pointer array or null/misaligned X");
    return MBQ_ERR_INVALID_ARG;
  }
  for (int i = 0; i < n_proj; ++i)
    if (!offsets_host[i] ||
        (T > 0 && (!Wr_host[i] || !br_host[i] || !prec_host[i] || !perm_host[i] || !aligned(Wr_host[i], 16)))) {
      set_error("mbq_route_group: null or misaligned pointer for projection %d", i);
      return MBQ_ERR_INVALID_ARG;
    }
  if (ws_bytes < mbq_route_workspace_bytes(T, K) || !ws || !aligned(ws, 256)) {
    set_error("mbq_route_group: workspace too small or misaligned (%zu < %zu)", ws_bytes,
              mbq_route_workspace_bytes(T, K));
    return MBQ_ERR_WORKSPACE;
  }
  return launch_route_group(X, T, K, n_proj, Wr_host, br_host, prec_host, perm_host, offsets_host, nullptr, ws,
                            (hipStream_t)stream, nullptr, 0, nullptr, false, *t_view);
}

size_t mbq_route_mlp_workspace_bytes(int64_t T, int64_t K, int H) {
  (void)K;
  if (T < 0 || H < 1 || H > route_mlp_max_hidden()) return 0;
  return route_mlp_workspace_bytes(T, H);
}

mbq_status mbq_route_mlp(const uint16_t* X, int64_t T, int64_t K, const float* W1, const float* b1, int H,
                         const float* W2, const float* b2, int E, double delta, int32_t* prec, int32_t* perm,
                         int32_t* offsets, double* scores, void* ws, size_t ws_bytes, void* stream) {
  if (E != MBQ_N_PRECISIONS || H < 1 || H > route_mlp_max_hidden()) {
    set_error("mbq_route_mlp: E=%d (must be %d) or hidden width %d outside 1..%d", E, MBQ_N_PRECISIONS, H,
              route_mlp_max_hidden());
    return MBQ_ERR_BAD_SHAPE;
  }
  if (T < 0 || K <= 0 || K % kGroup != 0 || T > (int64_t)1 << 24 || K > (int64_t)1 << 24) {
    set_error("mbq_route_mlp: bad sizes T=%lld K=%lld", (long long)T, (long long)K);
    return MBQ_ERR_BAD_SHAPE;
  }
  if (!offsets || (T > 0 && (!X || !W1 || !b1 || !W2 || !b2 || !prec || !perm)) || !aligned(X, 16) ||
      !aligned(W1, 16) || delta != delta) {
    set_error("mbq_route_mlp: null or misaligned pointer (X and W1 need 16-byte alignment) or delta is NaN");
    return MBQ_ERR_INVALID_ARG;
  }
  if (ws_bytes < mbq_route_mlp_workspace_bytes(T, K, H) || !ws || !aligned(ws, 256)) {
    set_error("mbq_route_mlp: workspace too small or misaligned (%zu < %zu)", ws_bytes,
              mbq_route_mlp_workspace_bytes(T, K, H));
    return MBQ_ERR_WORKSPACE;
  }
  return launch_route_mlp(X, T, K, W1, b1, H, W2, b2, delta, prec, perm, offsets, scores, ws, (hipStream_t)stream);
}

mbq_status mbq_threshold_quantile(const double* scores, int64_t T, int E, double rho, double* delta_out,
                                  void* stream) {
  if (E != MBQ_N_PRECISIONS || T < 1 || T > (int64_t)1 << 28) {
    set_error("mbq_threshold_quantile: E=%d (must be %d) or T=%lld outside 1..2^28", E, MBQ_N_PRECISIONS,
              (long long)T);
    return MBQ_ERR_BAD_SHAPE;
  }
  if (!scores || !delta_out || !(rho >= 0.0 && rho <= 1.0)) {
    set_error("mbq_threshold_quantile: null pointer or rho outside [0, 1]");
    return MBQ_ERR_INVALID_ARG;
  }
  const int64_t M = T * (E - 1);
  long long k = (long long)__builtin_floor(rho * (double)M + 0.5);
  if (k < 0) k = 0;
  if (k > M) k = M;
  return launch_threshold_quantile(scores, T, k, delta_out, (hipStream_t)stream);
}

mbq_status mbq_routed_linear_group(const uint16_t* X, int64_t T, int64_t K, int n_proj,
                                   const float* const* Wr_host, const float* const* br_host, int P,
                                   const void* const* blob_host, const int64_t* N_host, int32_t* const* prec_host,
                                   int32_t* const* perm_host, int32_t* const* offsets_host, float* const* Y_host,
                                   void* ws_route, size_t ws_route_bytes, void* ws_linear, size_t ws_linear_bytes,
                                   int algo, void* stream) {
  ApiScope scope;
  const uint16_t* XL = t_linear_X ? t_linear_X : X;  // what the linear kernels multiply
  if (t_view->shift != 0 || t_view->group != kGroup) {
    // A configuration with an odd cumulative width: the precision arrays count bits.  The loader-wavefront decode
    // kernels understand that (one token tile); every other shape goes through the slow
    // one-thread-per-output kernel, and so does every shape of a configuration with groups of 64 or 32 columns.
    // (T = 0: the routing call writes the empty offsets.)
    const bool bit_view = t_view->shift != 0;
    if (T == 0)  // the routing call checks its arguments and writes the empty offsets; there is nothing to multiply
      return mbq_route_group(X, T, K, n_proj, Wr_host, br_host, P, prec_host, perm_host, offsets_host, ws_route,
                             ws_route_bytes, stream);
    if (P != t_view->P || n_proj < 1 || n_proj > MBQ_MAX_GROUP || T < 0 || T > (int64_t)1 << 24 || K <= 0 ||
        K % kGroup != 0 || K > (int64_t)1 << 24) {
      set_error("mbq_routed_linear_group_cfg: bad sizes (P=%d, n_proj=%d, T=%lld, K=%lld)", P, n_proj, (long long)T,
                (long long)K);
      return MBQ_ERR_BAD_SHAPE;
    }
    if (algo < MBQ_ALGO_AUTO || algo > MBQ_ALGO_PREFILL || !N_host || !blob_host || !Y_host || !Wr_host || !br_host ||
        !prec_host || !perm_host || !offsets_host) {
      set_error("mbq_routed_linear_group_cfg: bad algo or null pointer array");
      return MBQ_ERR_INVALID_ARG;
    }
    for (int i = 0; i < n_proj; ++i)
      if (!Wr_host[i] || !aligned(Wr_host[i], 16) || !br_host[i] || !prec_host[i] || !perm_host[i] || !offsets_host[i]) {
        set_error("mbq_routed_linear_group_cfg: null or misaligned router pointer for projection %d", i);
        return MBQ_ERR_INVALID_ARG;
      }
    if (!ws_route || !aligned(ws_route, 256) || ws_route_bytes < mbq_route_workspace_bytes(T, K)) {
      set_error("mbq_routed_linear_group_cfg: route workspace too small or misaligned");
      return MBQ_ERR_WORKSPACE;
    }
    Shape sh[MBQ_MAX_GROUP];
    for (int i = 0; i < n_proj; ++i) {
      if (!make_shape(N_host[i], K, &sh[i], t_view->group)) return MBQ_ERR_BAD_SHAPE;
      if (!blob_host[i] || !aligned(blob_host[i], 256) || !Y_host[i] || !X || !aligned(X, 16)) {
        set_error("mbq_routed_linear_group_cfg: null or misaligned pointer for projection %d", i);
        return MBQ_ERR_INVALID_ARG;
      }
      if (!ws_linear || !aligned(ws_linear, 256) || ws_linear_bytes < mbq_linear_workspace_bytes(T, N_host[i], K)) {
        set_error("mbq_routed_linear_group_cfg: linear workspace too small or misaligned");
        return MBQ_ERR_WORKSPACE;
      }
    }
    if (bit_view && t_view->group == kGroup && algo != MBQ_ALGO_SIMPLE && algo != MBQ_ALGO_PREFILL && knob(3) == 0 &&
        decode_f4_takes_bit_view(T, sh[0]) && route_can_carry_prep(T)) {
      ZeroList zl;
      decode_f4_zero_list(T, n_proj, sh, Y_host, &zl);
      mbq_status st = launch_route_group(X, T, K, n_proj, Wr_host, br_host, prec_host, perm_host, offsets_host,
                                         nullptr, ws_route, (hipStream_t)stream, ws_linear, sh[0].KB, &zl, true,
                                         *t_view, XL);
      if (st != MBQ_OK) return st;
      return launch_linear_decode_f4(T, n_proj, blob_host, sh, prec_host, Y_host, ws_linear, (hipStream_t)stream,
                                     perm_host, offsets_host, nullptr, true);
    }
    mbq_status st = launch_route_group(X, T, K, n_proj, Wr_host, br_host, prec_host, perm_host, offsets_host, nullptr,
                                       ws_route, (hipStream_t)stream, nullptr, 0, nullptr, false, *t_view);
    if (st == MBQ_OK && bit_view && t_view->group == kGroup && (algo == MBQ_ALGO_AUTO || algo == MBQ_ALGO_DECODE) &&
        knob(3) == 0 && decode_f4_takes_bit_view(16, sh[0]))
      return bit_view_in_chunks(XL, T, n_proj, blob_host, sh, prec_host, Y_host, ws_linear, (hipStream_t)stream);
    for (int i = 0; st == MBQ_OK && i < n_proj; ++i)
      st = launch_linear_simple(XL, T, blob_host[i], sh[i], prec_host[i], Y_host[i], (hipStream_t)stream, bit_view);
    return st;
  }
  // the fused form: the router launch also prepares the activations of the decode kernel
  if (algo == MBQ_ALGO_AUTO || algo == MBQ_ALGO_DECODE) {
    Shape sh[MBQ_MAX_GROUP];
    bool ok = n_proj >= 1 && n_proj <= MBQ_MAX_GROUP && N_host && blob_host && Y_host && P == t_view->P &&
              T >= 1 && K > 0 && K % kGroup == 0 && X && aligned(X, 16) && Wr_host && br_host && prec_host &&
              perm_host && offsets_host && ws_route && aligned(ws_route, 256) &&
              ws_route_bytes >= mbq_route_workspace_bytes(T, K) && ws_linear && aligned(ws_linear, 256);
    for (int i = 0; ok && i < n_proj; ++i) {
      ok = N_host[i] > 0 && make_shape(N_host[i], K, &sh[i]) && blob_host[i] && aligned(blob_host[i], 256) &&
           Y_host[i] && Wr_host[i] && aligned(Wr_host[i], 16) && br_host[i] && prec_host[i] && perm_host[i] &&
           offsets_host[i] && ws_linear_bytes >= mbq_linear_workspace_bytes(T, N_host[i], K);
    }
    if (ok && knob(3) == 0 && decode_f4_supports(T, sh[0]) && route_can_carry_prep(T)) {
      ZeroList zl;
      decode_f4_zero_list(T, n_proj, sh, Y_host, &zl);
      mbq_status st = launch_route_group(X, T, K, n_proj, Wr_host, br_host, prec_host, perm_host, offsets_host,
                                         nullptr, ws_route, (hipStream_t)stream, ws_linear, sh[0].KB, &zl, true,
                                         *t_view, XL);
      if (st != MBQ_OK) return st;
      return launch_linear_decode_f4(T, n_proj, blob_host, sh, prec_host, Y_host, ws_linear, (hipStream_t)stream,
                                     perm_host, offsets_host);
    }
    // up to 128 tokens with every matrix on the register-stationary kernel: the router launch only writes the
    // precisions (no meeting of its workgroups), the linear launch sorts the tokens itself
    const int64_t defer_limit = (algo == MBQ_ALGO_AUTO) ? kMaxStationaryTokens : kMaxDecodeTokens;
    if (ok && T <= defer_limit && route_defers_sort(T)) {
      bool all = true;
      for (int i = 0; i < n_proj; ++i)
        all = all && (T <= kMaxDecodeTokens ? takes_stationary_kernel(T, sh[i])
                                            : resolve_auto(T, sh[i]) == kAlgoStationary);
      if (all) {
        ZeroList zl;  // outputs the linear launch adds into: cleared by a plane of the router launch
        decode16_zero_list(T, n_proj, sh, Y_host, &zl);
        mbq_status st = launch_route_group(X, T, K, n_proj, Wr_host, br_host, prec_host, perm_host, offsets_host,
                                           nullptr, ws_route, (hipStream_t)stream, nullptr, 0, &zl, true, *t_view);
        if (st != MBQ_OK) return st;
        return launch_linear_decode16_group(XL, T, n_proj, blob_host, sh, prec_host, perm_host, Y_host,
                                            (hipStream_t)stream, perm_host, offsets_host);
      }
    }
  }
  // otherwise exactly the two calls (they check the arguments)
  mbq_status st = mbq_route_group(X, T, K, n_proj, Wr_host, br_host, P, prec_host, perm_host, offsets_host,
                                  ws_route, ws_route_bytes, stream);
  if (st != MBQ_OK) return st;
  return mbq_linear_group(XL, T, K, n_proj, blob_host, N_host, prec_host, perm_host, offsets_host, Y_host, ws_linear,
                          ws_linear_bytes, algo, stream);
}

mbq_status mbq_linear(const uint16_t* X, int64_t T, const void* blob, int64_t N, int64_t K,
                      const int32_t* prec, const int32_t* perm, const int32_t* offsets, float* Y, void* ws,
                      size_t ws_bytes, int algo, void* stream) {
  ApiScope scope;
  Shape sh;
  if (!make_shape(N, K, &sh)) return MBQ_ERR_BAD_SHAPE;
  if (T < 0 || T > (int64_t)1 << 24) {
    set_error("mbq_linear: bad token count %lld", (long long)T);
    return MBQ_ERR_BAD_SHAPE;
  }
  if (algo < MBQ_ALGO_AUTO || algo > MBQ_ALGO_PREFILL) {
    set_error("mbq_linear: unknown algo %d", algo);
    return MBQ_ERR_INVALID_ARG;
  }
  if (T == 0) return MBQ_OK;
  if (!X || !blob || !prec || !perm || !offsets || !Y || !aligned(blob, 256) || !aligned(X, 16)) {
    set_error("mbq_linear: null or misaligned pointer (X 16-byte, blob 256-byte alignment)");
    return MBQ_ERR_INVALID_ARG;
  }
  if (!ws || !aligned(ws, 256) || ws_bytes < mbq_linear_workspace_bytes(T, N, K)) {
    set_error("mbq_linear: workspace too small or misaligned (%zu < %zu)", ws_bytes,
              mbq_linear_workspace_bytes(T, N, K));
    return MBQ_ERR_WORKSPACE;
  }
  if (algo == MBQ_ALGO_AUTO) algo = resolve_auto(T, sh);
  if (algo == MBQ_ALGO_DECODE && T > kMaxDecodeTokens) {
    set_error("mbq_linear: the decode kernel handles at most %d tokens (T=%lld)", kMaxDecodeTokens,
              (long long)T);
    return MBQ_ERR_BAD_SHAPE;
  }
  return dispatch_linear(X, T, blob, sh, prec, perm, offsets, Y, ws, algo, (hipStream_t)stream);
}

mbq_status mbq_linear_group(const uint16_t* X, int64_t T, int64_t K, int n_proj, const void* const* blob_host,
                            const int64_t* N_host, const int32_t* const* prec_host,
                            const int32_t* const* perm_host, const int32_t* const* offsets_host,
                            float* const* Y_host, void* ws, size_t ws_bytes, int algo, void* stream) {
  ApiScope scope;
  if (n_proj < 1 || n_proj > MBQ_MAX_GROUP) {
    set_error("mbq_linear_group: n_proj=%d outside 1..%d", n_proj, MBQ_MAX_GROUP);
    return MBQ_ERR_INVALID_ARG;
  }
  if (!blob_host || !N_host || !prec_host || !perm_host || !offsets_host || !Y_host) {
    set_error("mbq_linear_group: null pointer array");
    return MBQ_ERR_INVALID_ARG;
  }
  if (T < 0 || T > (int64_t)1 << 24) {
    set_error("mbq_linear_group: bad token count %lld", (long long)T);
    return MBQ_ERR_BAD_SHAPE;
  }
  if (algo < MBQ_ALGO_AUTO || algo > MBQ_ALGO_PREFILL) {
    set_error("mbq_linear_group: unknown algo %d", algo);
    return MBQ_ERR_INVALID_ARG;
  }
  Shape sh[MBQ_MAX_GROUP];
  size_t need = 0;
  for (int i = 0; i < n_proj; ++i) {
    if (!make_shape(N_host[i], K, &sh[i])) return MBQ_ERR_BAD_SHAPE;
    const size_t b = mbq_linear_workspace_bytes(T, N_host[i], K);
    if (b > need) need = b;
  }
  if (T == 0) return MBQ_OK;
  if (!X || !aligned(X, 16)) {
    set_error("mbq_linear_group: null or misaligned X");
    return MBQ_ERR_INVALID_ARG;
  }
  for (int i = 0; i < n_proj; ++i)
    if (!blob_host[i] || !prec_host[i] || !perm_host[i] || !offsets_host[i] || !Y_host[i] ||
        !aligned(blob_host[i], 256)) {
      set_error("mbq_linear_group: null or misaligned pointer for projection %d", i);
      return MBQ_ERR_INVALID_ARG;
    }
  if (!ws || !aligned(ws, 256) || ws_bytes < need) {
    set_error("mbq_linear_group: workspace too small or misaligned (%zu < %zu)", ws_bytes, need);
    return MBQ_ERR_WORKSPACE;
  }
  int algo_of[MBQ_MAX_GROUP];  // per matrix: AUTO may pick different kernels above the decode limit
  bool all_stationary = true;
  for (int i = 0; i < n_proj; ++i) {
    algo_of[i] = algo == MBQ_ALGO_AUTO ? resolve_auto(T, sh[i]) : algo;
    all_stationary = all_stationary && algo_of[i] == kAlgoStationary;
  }
  if (algo == MBQ_ALGO_AUTO) algo = all_stationary ? kAlgoStationary : (T <= kMaxDecodeTokens ? MBQ_ALGO_DECODE : MBQ_ALGO_PREFILL);
  if (algo == MBQ_ALGO_DECODE && T > kMaxDecodeTokens) {
    set_error("mbq_linear_group: the decode kernel handles at most %d tokens (T=%lld)", kMaxDecodeTokens,
              (long long)T);
    return MBQ_ERR_BAD_SHAPE;
  }
  hipStream_t s = (hipStream_t)stream;
  if (algo == MBQ_ALGO_DECODE && knob(3) == 0 && decode_f4_supports(T, sh[0])) {
    ZeroList zl;
    decode_f4_zero_list(T, n_proj, sh, Y_host, &zl);
    mbq_status st = launch_decode_f4_prep(X, T, K, sh[0].KB, ws, zl, s);
    if (st != MBQ_OK) return st;
    return launch_linear_decode_f4(T, n_proj, blob_host, sh, prec_host, Y_host, ws, s, nullptr, nullptr);
  }
  if ((algo == MBQ_ALGO_DECODE || algo == kAlgoStationary) && n_proj > 1) {
    // the matrices share one launch of the register-stationary kernel when each of them would take it
    bool all = true;
    for (int i = 0; i < n_proj; ++i) all = all && takes_stationary_kernel(T, sh[i]);
    if (all) {
      ZeroList zl;
      decode16_zero_list(T, n_proj, sh, Y_host, &zl);
      mbq_status st = launch_zero_outputs(zl, s);
      if (st != MBQ_OK) return st;
      return launch_linear_decode16_group(X, T, n_proj, blob_host, sh, prec_host, perm_host, Y_host, s, nullptr,
                                          nullptr);
    }
  }
  for (int i = 0; i < n_proj; ++i) {
    mbq_status st =
        dispatch_linear(X, T, blob_host[i], sh[i], prec_host[i], perm_host[i], offsets_host[i], Y_host[i], ws, algo_of[i], s);
    if (st != MBQ_OK) return st;
  }
  return MBQ_OK;
}

// ---- other slice configurations (Sec. 4.1 general E and b_e; App. C.1 slice_bits_list) ---------------------------
// The blob holds the eight-bit code of every weight as four base-4 digits whatever the configuration: a
// configuration whose slices end on digit boundaries cuts the same code at other places (a 4-bit slice with the
// centred zero point 8 and scale s/16 IS two 2-bit slices with zero point 2 and scales s/4, s/16), and its first-slice
// parameters are the stored ones moved by a power of two.  So only the router (how many outputs, which digit count
// each stands for) and the checking helpers know about it.

mbq_status mbq_config_check(const mbq_config* cfg) {
  RouteView v;
  return make_view(cfg, &v, "mbq_config_check") ? MBQ_OK : MBQ_ERR_BAD_SHAPE;
}

int mbq_config_bits(const mbq_config* cfg, int p) {
  RouteView v;
  if (!make_view(cfg, &v, "mbq_config_bits") || p < 0 || p >= v.P) return -1;
  return v.bits[p];
}

int mbq_config_precision_value(const mbq_config* cfg, int p) {
  RouteView v;
  if (!make_view(cfg, &v, "mbq_config_precision_value") || p < 0 || p >= v.P) return -1;
  return v.value[p];
}

int mbq_config_counts_bits(const mbq_config* cfg) {
  RouteView v;
  if (!make_view(cfg, &v, "mbq_config_counts_bits")) return -1;
  return v.shift;
}

size_t mbq_blob_bytes_cfg(const mbq_config* cfg, int64_t N, int64_t K) {
  RouteView v;
  Shape sh;
  return make_view(cfg, &v, "mbq_blob_bytes_cfg") && make_shape(N, K, &sh, v.group) ? sh.bytes : 0;
}

mbq_status mbq_encode_cfg(const float* W, int64_t N, int64_t K, const mbq_config* cfg, void* blob, void* stream) {
  RouteView v;
  if (!make_view(cfg, &v, "mbq_encode_cfg")) return MBQ_ERR_BAD_SHAPE;
  if (v.group == kGroup) return mbq_encode(W, N, K, blob, stream);
  Shape sh;
  if (!make_shape(N, K, &sh, v.group)) return MBQ_ERR_BAD_SHAPE;
  if (!W || !blob || !aligned(blob, 256) || !aligned(W, 16)) {
    set_error("mbq_encode_cfg: W must be 16-byte and blob 256-byte aligned and non-null");
    return MBQ_ERR_INVALID_ARG;
  }
  return launch_encode_small_group(W, sh, blob, (hipStream_t)stream);
}

mbq_status mbq_unpack_cfg(const void* blob, int64_t N, int64_t K, const mbq_config* cfg, uint8_t* codes,
                          float* scale, float* zero, void* stream) {
  RouteView v;
  if (!make_view(cfg, &v, "mbq_unpack_cfg")) return MBQ_ERR_BAD_SHAPE;
  Shape sh;
  if (!make_shape(N, K, &sh, v.group)) return MBQ_ERR_BAD_SHAPE;
  if (!blob || !aligned(blob, 256)) {
    set_error("mbq_unpack_cfg: blob must be non-null and 256-byte aligned");
    return MBQ_ERR_INVALID_ARG;
  }
  return launch_unpack_view(blob, sh, v, codes, scale, zero, (hipStream_t)stream);
}

mbq_status mbq_dequant_cfg(const void* blob, int64_t N, int64_t K, const mbq_config* cfg, int p, float* What,
                           void* stream) {
  RouteView v;
  if (!make_view(cfg, &v, "mbq_dequant_cfg")) return MBQ_ERR_BAD_SHAPE;
  if (p < 0 || p >= v.P) {
    set_error("mbq_dequant_cfg: precision index %d outside 0..%d", p, v.P - 1);
    return MBQ_ERR_INVALID_ARG;
  }
  Shape sh;
  if (!make_shape(N, K, &sh, v.group)) return MBQ_ERR_BAD_SHAPE;
  if (!blob || !What || !aligned(blob, 256)) {
    set_error("mbq_dequant_cfg: null or misaligned pointer");
    return MBQ_ERR_INVALID_ARG;
  }
  return launch_dequant_bits(blob, sh, v.bits[p], What, (hipStream_t)stream);
}

mbq_status mbq_linear_cfg(const uint16_t* X, int64_t T, const void* blob, int64_t N, int64_t K,
                          const mbq_config* cfg, const int32_t* prec, const int32_t* perm, const int32_t* offsets,
                          float* Y, void* ws, size_t ws_bytes, int algo, void* stream) {
  RouteView v;
  if (!make_view(cfg, &v, "mbq_linear_cfg")) return MBQ_ERR_BAD_SHAPE;
  if (v.shift == 0 && v.group == kGroup)
    return mbq_linear(X, T, blob, N, K, prec, perm, offsets, Y, ws, ws_bytes, algo, stream);
  ApiScope scope;
  Shape sh;
  if (!make_shape(N, K, &sh, v.group)) return MBQ_ERR_BAD_SHAPE;
  if (T < 0 || T > (int64_t)1 << 24) {
    set_error("mbq_linear_cfg: bad token count %lld", (long long)T);
    return MBQ_ERR_BAD_SHAPE;
  }
  if (algo < MBQ_ALGO_AUTO || algo > MBQ_ALGO_PREFILL) {
    set_error("mbq_linear_cfg: unknown algo %d", algo);
    return MBQ_ERR_INVALID_ARG;
  }
  if (T == 0) return MBQ_OK;
  if (!X || !blob || !prec || !Y || !aligned(blob, 256) || !aligned(X, 16)) {
    set_error("mbq_linear_cfg: null or misaligned pointer (X 16-byte, blob 256-byte alignment)");
    return MBQ_ERR_INVALID_ARG;
  }
  if (!ws || !aligned(ws, 256) || ws_bytes < mbq_linear_workspace_bytes(T, N, K)) {
    set_error("mbq_linear_cfg: workspace too small or misaligned (%zu < %zu)", ws_bytes,
              mbq_linear_workspace_bytes(T, N, K));
    return MBQ_ERR_WORKSPACE;
  }
  hipStream_t s = (hipStream_t)stream;
  if (v.group == kGroup && algo != MBQ_ALGO_SIMPLE && algo != MBQ_ALGO_PREFILL && knob(3) == 0 &&
      decode_f4_takes_bit_view(T, sh)) {
    ZeroList zl;
    decode_f4_zero_list(T, 1, &sh, &Y, &zl);
    mbq_status st = launch_decode_f4_prep(X, T, sh.K, sh.KB, ws, zl, s);
    if (st != MBQ_OK) return st;
    return launch_linear_decode_f4(T, 1, &blob, &sh, &prec, &Y, ws, s, nullptr, nullptr, nullptr, true);
  }
  if (v.shift != 0 && v.group == kGroup && (algo == MBQ_ALGO_AUTO || algo == MBQ_ALGO_DECODE) && knob(3) == 0 &&
      decode_f4_takes_bit_view(16, sh))
    return bit_view_in_chunks(X, T, 1, &blob, &sh, &prec, &Y, ws, s);
  return launch_linear_simple(X, T, blob, sh, prec, Y, s, v.shift != 0);
}

mbq_status mbq_route_cfg(const uint16_t* X, int64_t T, int64_t K, const float* Wr, const float* br,
                         const mbq_config* cfg, int32_t* prec, int32_t* perm, int32_t* offsets, double* logits,
                         void* ws, size_t ws_bytes, void* stream) {
  RouteView v;
  if (!make_view(cfg, &v, "mbq_route_cfg")) return MBQ_ERR_BAD_SHAPE;
  ViewScope scope(&v);
  return mbq_route(X, T, K, Wr, br, v.P, prec, perm, offsets, logits, ws, ws_bytes, stream);
}

mbq_status mbq_route_group_cfg(const uint16_t* X, int64_t T, int64_t K, int n_proj, const float* const* Wr_host,
                               const float* const* br_host, const mbq_config* cfg, int32_t* const* prec_host,
                               int32_t* const* perm_host, int32_t* const* offsets_host, void* ws, size_t ws_bytes,
                               void* stream) {
  RouteView v;
  if (!make_view(cfg, &v, "mbq_route_group_cfg")) return MBQ_ERR_BAD_SHAPE;
  ViewScope scope(&v);
  return mbq_route_group(X, T, K, n_proj, Wr_host, br_host, v.P, prec_host, perm_host, offsets_host, ws, ws_bytes,
                         stream);
}

mbq_status mbq_routed_linear_group_cfg(const uint16_t* X, int64_t T, int64_t K, int n_proj,
                                       const float* const* Wr_host, const float* const* br_host,
                                       const mbq_config* cfg, const void* const* blob_host, const int64_t* N_host,
                                       int32_t* const* prec_host, int32_t* const* perm_host,
                                       int32_t* const* offsets_host, float* const* Y_host, void* ws_route,
                                       size_t ws_route_bytes, void* ws_linear, size_t ws_linear_bytes, int algo,
                                       void* stream) {
  RouteView v;
  if (!make_view(cfg, &v, "mbq_routed_linear_group_cfg")) return MBQ_ERR_BAD_SHAPE;
  ViewScope scope(&v);
  return mbq_routed_linear_group(X, T, K, n_proj, Wr_host, br_host, v.P, blob_host, N_host, prec_host, perm_host,
                                 offsets_host, Y_host, ws_route, ws_route_bytes, ws_linear, ws_linear_bytes, algo,
                                 stream);
}

mbq_status mbq_act_quant(const uint16_t* X, int64_t T, int64_t K, int abits, const float* let_shift,
                         const float* let_scale, uint16_t* Xint, float* row_scale, uint16_t* Xr, void* stream) {
  if (T < 0 || K <= 0 || K % kGroup != 0 || T > (int64_t)1 << 24 || K > (int64_t)1 << 24) {
    set_error("mbq_act_quant: bad sizes (T=%lld, K=%lld; K must be a multiple of %d)", (long long)T, (long long)K,
              kGroup);
    return MBQ_ERR_BAD_SHAPE;
  }
  if (abits < 2 || abits > 8) {
    set_error("mbq_act_quant: abits = %d, supported 2..8", abits);
    return MBQ_ERR_INVALID_ARG;
  }
  if ((let_shift == nullptr) != (let_scale == nullptr)) {
    set_error("mbq_act_quant: pass both the shift and the scale of the transform, or neither");
    return MBQ_ERR_INVALID_ARG;
  }
  if (T == 0) return MBQ_OK;
  if (!X || !Xint || !row_scale || !aligned(X, 16) || !aligned(Xint, 16) || !aligned(Xr, 16) ||
      !aligned(let_shift, 16) || !aligned(let_scale, 16)) {
    set_error("mbq_act_quant: null or misaligned pointer (16-byte alignment for X, Xint, Xr, shift and scale)");
    return MBQ_ERR_INVALID_ARG;
  }
  return launch_act_quant(X, T, K, abits, let_shift, let_scale, Xint, row_scale, Xr, (hipStream_t)stream);
}

mbq_status mbq_routed_linear_group_act(const uint16_t* X, int64_t T, int64_t K, int abits, const float* let_shift,
                                       const float* let_scale, int n_proj, const float* const* Wr_host,
                                       const float* const* br_host, int P, const void* const* blob_host,
                                       const int64_t* N_host, const float* const* bias_host,
                                       int32_t* const* prec_host, int32_t* const* perm_host,
                                       int32_t* const* offsets_host, float* const* Y_host, uint16_t* Xint,
                                       float* row_scale, uint16_t* Xr, void* ws_route, size_t ws_route_bytes,
                                       void* ws_linear, size_t ws_linear_bytes, int algo, void* stream) {
  ApiScope scope;
  if (n_proj < 1 || n_proj > MBQ_MAX_GROUP || !N_host || !Y_host) {
    set_error("mbq_routed_linear_group_act: n_proj = %d (1..%d) or a null N / Y array", n_proj, MBQ_MAX_GROUP);
    return MBQ_ERR_INVALID_ARG;
  }
  if (T > 0 && !Xr) {
    set_error("mbq_routed_linear_group_act: the buffer for the router's input is null");
    return MBQ_ERR_INVALID_ARG;
  }
  for (int i = 0; i < n_proj; ++i)
    if (N_host[i] <= 0 || N_host[i] > (int64_t)1 << 24 || (T > 0 && !Y_host[i])) {
      set_error("mbq_routed_linear_group_act: bad N or null Y for projection %d", i);
      return MBQ_ERR_INVALID_ARG;
    }
  mbq_status st = mbq_act_quant(X, T, K, abits, let_shift, let_scale, Xint, row_scale, Xr, stream);
  if (st != MBQ_OK) return st;
  {
    LinearInputScope linear_input(Xint);
    st = mbq_routed_linear_group(Xr, T, K, n_proj, Wr_host, br_host, P, blob_host, N_host, prec_host, perm_host,
                                 offsets_host, Y_host, ws_route, ws_route_bytes, ws_linear, ws_linear_bytes, algo,
                                 stream);
  }
  if (st != MBQ_OK || T == 0) return st;
  return launch_scale_rows_group(n_proj, Y_host, T, N_host, row_scale, bias_host, (hipStream_t)stream);
}

mbq_status mbq_scale_rows(float* Y, int64_t T, int64_t N, const float* row_scale, const float* bias, void* stream) {
  if (T < 0 || N <= 0 || T > (int64_t)1 << 24 || N > (int64_t)1 << 24) {
    set_error("mbq_scale_rows: bad sizes (T=%lld, N=%lld)", (long long)T, (long long)N);
    return MBQ_ERR_BAD_SHAPE;
  }
  if (T == 0) return MBQ_OK;
  if (!Y || !row_scale) {
    set_error("mbq_scale_rows: null pointer");
    return MBQ_ERR_INVALID_ARG;
  }
  return launch_scale_rows(Y, T, N, row_scale, bias, (hipStream_t)stream);
}

}  // extern "C"
