/*
 * mbq - token-routed any-precision linear layer (MoBiQuant inference hot path)
 * for AMD MI355X (gfx950).  C ABI of libmbq.so.
 *
 * The layer:  a weight matrix W (N output features x K input features) is stored
 * once as four 2-bit slices produced by recursive residual quantisation (paper
 * Sec. 4.1, Eq. 2; quantiser and scale refinement of App. B).  At run time a
 * per-token router picks a precision index p in {0,1,2,3} (2, 4, 6 or 8 bits) and
 * the token's output row is its activation row times the weight rebuilt from
 * slices 0..p only (Sec. 4.1 Eq. 3, Sec. 4.2 Eq. 6).
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its name ends in _host.
 *   - The caller owns every buffer.  The library allocates nothing, keeps no state
 *     between calls and never synchronises: all work is enqueued on `stream` (a
 *     hipStream_t passed as void*; NULL is the default stream).  Outputs are valid
 *     once the stream reaches that point.  What a call launches depends on its
 *     arguments alone (the test hooks of mbq_bench.h aside, which default to off);
 *     calls may be made from several threads at once as long as they do not share a
 *     workspace.
 *   - Every entry point returns an mbq_status.  On failure nothing has been
 *     enqueued and mbq_last_error() describes the cause (thread-local string).
 *   - bf16 values are passed as uint16_t bit patterns.
 *   - The calls without _cfg in their names run the paper's default configuration: group
 *     size 128 along K, four slices of two bits (App. C.1).  Other slice widths and groups of
 *     64 or 32: the *_cfg calls at the end of this file.  K must be a multiple of 128.
 *
 * Packed weight blob (written by mbq_encode, read by every other call)
 *   Let NT = ceil(N/16), KB = ceil(K/256); rows and columns beyond N, K are padded
 *   with code 0 and scale 0.  The blob is, in this order,
 *     codes : uint32 [4 slices][NT][KB][64 lanes][4 dwords]      (1 KiB per tile)
 *     meta  : float  [NT][2*KB groups][16 rows][2]  = {s0, z0}    (128 B per tile-group)
 *   A code tile holds 16 rows x 256 columns of one slice.  For weight (n, k):
 *     r = k mod 256, d = r / 64, step = (r mod 64) / 32, kq = (r mod 32) / 8, s = r mod 8,
 *     lane = 16*kq + (n mod 16), dword d of that lane,
 *     bit  = (16*(s&1) + 4*(s>>1) + 2*step + (2 - 2*slice)) mod 32   (2-bit field).
 *   (Slice e is stored rotated left by 2-2e bits so that the four slices of one
 *   weight line up as one byte after a common rotation; the decode kernel reads a
 *   tile with one 128-bit load per lane and feeds it to 16x16x32 MFMAs without
 *   transposition.)  s0 is the base-slice scale, z0 its continuous zero point;
 *   slice e uses s0 / 4^e and, for e >= 1, zero point 2.
 */
#ifndef MBQ_H_
#define MBQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum mbq_status {
  MBQ_OK = 0,
  MBQ_ERR_INVALID_ARG = 1, /* null pointer, negative size, bad enum value          */
  MBQ_ERR_BAD_SHAPE = 2,   /* K not a multiple of 128, size overflow, P != 4       */
  MBQ_ERR_WORKSPACE = 3,   /* workspace smaller than mbq_*_workspace_bytes()       */
  MBQ_ERR_HIP = 4          /* a HIP call or kernel launch failed                   */
} mbq_status;

/* Which kernel family mbq_linear uses.  AUTO picks by token count and matrix size: the decode kernels up to 64
 * tokens, one of them (one pass over the weights per 32 precision-sorted tokens) on to 128 tokens, 512 for small
 * matrices, where it still beats the tiled GEMM; from there to 256 tokens (K <= 8192) both are enqueued and the one
 * that suits the precision mix, which only the device knows, does the work; then PREFILL. */
typedef enum mbq_algo {
  MBQ_ALGO_AUTO = 0,
  MBQ_ALGO_SIMPLE = 1, /* one thread per output, fp64 accumulate: slow checker path   */
  MBQ_ALGO_DECODE = 2, /* the decode kernels; as a request: T <= 64 only             */
  MBQ_ALGO_PREFILL = 3 /* merged-code bf16 MFMA tiled GEMM, any T                     */
} mbq_algo;

#define MBQ_N_PRECISIONS 4
#define MBQ_GROUP 128
#define MBQ_MAX_GROUP 4 /* most projections one mbq_*_group call takes */

const char* mbq_version(void);
const char* mbq_last_error(void);

/* Bytes of the packed weight blob for an N x K matrix (0 if the shape is invalid). */
size_t mbq_blob_bytes(int64_t N, int64_t K);

/* Workspace sizes (bytes) for mbq_route / mbq_linear at the given sizes. */
size_t mbq_route_workspace_bytes(int64_t T, int64_t K);
size_t mbq_linear_workspace_bytes(int64_t T, int64_t N, int64_t K);

/*
 * mbq_encode - recursive residual quantisation of W into the packed blob.
 * Sec. 4.1 Eq. 2 with the floor-aligned quantiser, scale refinement s_{e+1} = s_e/4
 * and centred residual zero point of App. B.  Per (row, group of 128): s0 =
 * (max-min)/4 and z0 = -min/s0 in fp32 (range floored at 2^-16 of the group's
 * magnitude and at 2^-100); codes from the fp64 recursion
 *   c_e = clamp(floor(R/s_e + z_e), 0, 3),  R <- R - s_e (c_e - z_e + 0.5).
 *   W    : fp32 [N][K] row-major (read)
 *   blob : mbq_blob_bytes(N, K) bytes, 256-byte aligned (written, fully)
 */
mbq_status mbq_encode(const float* W, int64_t N, int64_t K, void* blob, void* stream);

/*
 * mbq_encode_with_params - the same recursion with the base-slice scale and zero point given by the
 * caller instead of fitted: the paper calibrates (s0, z0) with a learned clipping range (Sec. 4.1,
 * App. B "first slice (s0, z0) is calibrated"), which is outside this library.  A weight outside the
 * range the parameters span saturates: the clamp of App. B's quantiser gives it code 0 (or 3) in
 * every slice.
 *   scale, zero : fp32 [N][K/128] row-major (read); every scale must be finite and > 0, every zero
 *                 point finite (not checked: other values give meaningless codes, never a fault)
 *   W, blob     : as in mbq_encode; the blob stores scale and zero as given
 */
mbq_status mbq_encode_with_params(const float* W, int64_t N, int64_t K, const float* scale, const float* zero,
                                  void* blob, void* stream);

/*
 * mbq_unpack - blob -> canonical arrays, for inspection and tests.
 *   codes : uint8 [4][N][K], one code (0..3) per byte          (may be NULL)
 *   scale : fp32 [N][K/128]  base-slice scale s0               (may be NULL)
 *   zero  : fp32 [N][K/128]  base-slice zero point z0          (may be NULL)
 */
mbq_status mbq_unpack(const void* blob, int64_t N, int64_t K, uint8_t* codes, float* scale,
                      float* zero, void* stream);

/*
 * mbq_dequant - weight at precision index p (Sec. 4.1 Eq. 3):
 *   What[n][k] = (s0/4^p) * (I_p - 4^p z0 + 0.5),  I_p = sum_{e<=p} c_e 4^{p-e},
 * evaluated in fp64 and rounded once to fp32.  What : fp32 [N][K].
 */
mbq_status mbq_dequant(const void* blob, int64_t N, int64_t K, int p, float* What, void* stream);

/*
 * mbq_route - router scores, precision choice and token permutation
 * (Sec. 4.2 Eq. 4 read as one linear map to P = 4 logits; Sec. 4.3 challenge 3).
 *   logits[i][q] = sum_k X[i][k] * Wr[q][k] + br[q]   accumulated in fp64
 *   prec[i]      = argmax_q logits[i][q], first maximum on ties
 *   perm/offsets = stable grouping of token ids by ascending prec:
 *                  tokens of precision q are perm[offsets[q] .. offsets[q+1]-1]
 *   X      : bf16 [T][K]           Wr : fp32 [P][K]        br : fp32 [P]
 *   prec   : int32 [T] (out)       perm : int32 [T] (out)  offsets : int32 [P+1] (out)
 *   logits : fp64 [T][P] (out, may be NULL)
 *   ws     : at least mbq_route_workspace_bytes(T, K) bytes, 256-byte aligned.  It holds the
 *            counters by which the workgroups of the launch find out who is last; the call
 *            clears them itself (a small launch ahead of the router's), so the contents before
 *            the call do not matter.  Calls sharing one workspace must not overlap in time.
 * T = 0 is legal (offsets are zero-filled).
 */
mbq_status mbq_route(const uint16_t* X, int64_t T, int64_t K, const float* Wr, const float* br,
                     int P, int32_t* prec, int32_t* perm, int32_t* offsets, double* logits,
                     void* ws, size_t ws_bytes, void* stream);

/*
 * mbq_route_group - mbq_route for n_proj routers that read the SAME activations (the
 * projections of a decoder block that share their input: q/k/v, gate/up), in one launch
 * up to 128 tokens (Sec. 4.3, fused router launch for all projections of a layer).
 * Results are those of n_proj separate mbq_route calls, bit for bit.
 *   Wr_host, br_host, prec_host, perm_host, offsets_host : HOST arrays of n_proj DEVICE
 *   pointers, each pointing to what the argument of the same name is in mbq_route; they are
 *   read before the call returns.  1 <= n_proj <= MBQ_MAX_GROUP.  ws as in mbq_route.
 */
mbq_status mbq_route_group(const uint16_t* X, int64_t T, int64_t K, int n_proj,
                           const float* const* Wr_host, const float* const* br_host, int P,
                           int32_t* const* prec_host, int32_t* const* perm_host,
                           int32_t* const* offsets_host, void* ws, size_t ws_bytes, void* stream);

/*
 * mbq_route_mlp - the paper's own router (Sec. 4.2 Eq. 4: a 2-layer MLP gives one score per slice) with
 * the run-time threshold of Sec. 4.2 (efficient runtime precision switching, G = 1[(S - delta) > 0]):
 *   S[i][e] = sum_j relu(sum_k X[i][k] W1[j][k] + b1[j]) * W2[e][j] + b2[e]      accumulated in fp64
 *   slice e >= 1 of token i is active iff (S[i][e] - delta) > 0;  slice 0 is always active (the
 *   shared-expert slice), its score is computed but never used
 *   prec[i] = number of leading active residual slices e = 1, 2, 3 (a precision names a prefix of
 *             slices, so an active slice behind an inactive one is ignored)
 *   perm/offsets = as in mbq_route.
 * The paper gives neither the hidden width nor the activation of the MLP; ReLU is the reading taken.
 * delta is the layer's threshold plus any global shift: raising it lowers precisions, the packed blob is
 * untouched.
 *   X : bf16 [T][K]   W1 : fp32 [H][K]   b1 : fp32 [H]   W2 : fp32 [E][H]   b2 : fp32 [E]
 *   1 <= H <= 512, E = 4;  prec, perm, offsets as in mbq_route;  scores : fp64 [T][E] (out, may be NULL)
 *   ws : at least mbq_route_mlp_workspace_bytes(T, K, H) bytes, 256-byte aligned; its first 256 bytes
 *        hold a ticket counter (cleared by the call itself), the rest the hidden layer.
 * T = 0 is legal.
 */
size_t mbq_route_mlp_workspace_bytes(int64_t T, int64_t K, int H);
mbq_status mbq_route_mlp(const uint16_t* X, int64_t T, int64_t K, const float* W1, const float* b1, int H,
                         const float* W2, const float* b2, int E, double delta, int32_t* prec,
                         int32_t* perm, int32_t* offsets, double* scores, void* ws, size_t ws_bytes,
                         void* stream);

/*
 * mbq_threshold_quantile - layer-wise threshold calibration (App. C.2): from the scores of a
 * calibration batch, the threshold that leaves a fraction rho of the T (E - 1) residual-slice scores
 * active.  With k = floor(rho T (E-1) + 1/2) clipped to 0 .. T (E-1), *delta_out is the (k+1)-th
 * largest residual score, so exactly the k largest satisfy score - delta > 0 (ties aside); -inf if
 * k = T (E-1).  For the default slices a target of b average bits is rho = (b - 2) / 6.  An offline
 * step (one workgroup).
 *   scores : fp64 [T][E] as written by mbq_route_mlp, T >= 1, E = 4;  0 <= rho <= 1
 *   delta_out : one double (device, out)
 */
mbq_status mbq_threshold_quantile(const double* scores, int64_t T, int E, double rho, double* delta_out,
                                  void* stream);

/*
 * mbq_linear - routed output (Sec. 4.2 Eq. 6 with the prefix mask of slices 0..p_i):
 *   Y[i][n] = sum_k X[i][k] * What^(prec[i])[n][k],  fp32 accumulate, fp32 output,
 * reading for each token only the slices its precision needs.
 *   X    : bf16 [T][K]            blob : packed weights of an N x K matrix
 *   prec, perm, offsets : as written by mbq_route (must be mutually consistent)
 *   Y    : fp32 [T][N] in ORIGINAL token order (written for every token)
 *   ws   : at least mbq_linear_workspace_bytes(T, N, K) bytes, 256-byte aligned
 *   algo : an mbq_algo value
 * T = 0 is legal (no-op).
 * Arithmetic.  Products of an activation and a code are exact everywhere and sums are fp32.  Up to 16 tokens the
 * bf16 activations reach the matrix cores as two FP8 (E4M3) pieces per element under a power-of-two scale per
 * (token, block of 256 columns): exact for every element within 13 binades of the block's largest, and off by at
 * most 2^-21 of that largest element below (the piece that would carry it underflows) - a data-dependent error far
 * inside the 1e-3 bar, none at all for blocks without such a spread.  The scale is an 8-bit exponent: a block whose
 * largest element is under 2^-115 (bf16 subnormals and their neighbours) is scaled by 2^122 at most, and its elements
 * are then rounded to multiples of 2^-135, an eighth of bf16's subnormal spacing.
 * Reproducibility.  The decode kernels (up to 64 tokens, and on with AUTO while it keeps them) give the same bits on
 * every call and in grouped and single calls.  The tiled GEMM does too unless a launch with few tiles splits K into
 * more than two parts: those partial sums are added with float atomics in whatever order they arrive, and results
 * then agree to rounding, not bit for bit.
 */
mbq_status mbq_linear(const uint16_t* X, int64_t T, const void* blob, int64_t N, int64_t K,
                      const int32_t* prec, const int32_t* perm, const int32_t* offsets, float* Y,
                      void* ws, size_t ws_bytes, int algo, void* stream);

/*
 * mbq_linear_static - mbq_linear without a workspace argument, for callers that cannot allocate device memory
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the workspace is a buffer of
 * MBQ_STATIC_SCRATCH_BYTES that is part of the library image on every GPU (it costs that much device memory per
 * GPU the library runs on, until the process ends).  The call allocates nothing and frees nothing.
 *   - Same arguments, results and errors as mbq_linear otherwise; the kernels are the same.
 *   - Shapes whose mbq_linear_workspace_bytes(T, N, K) exceeds the buffer are refused with MBQ_ERR_WORKSPACE
 *     (nothing is enqueued); mbq_static_scratch_bytes() returns the size.
 *   - All calls on one GPU share the one buffer (its contents are whatever the last call left; nothing in it has to
 *     start at zero): two calls on the same GPU whose execution overlaps (different streams, different threads)
 *     race.  Calls on one stream are ordered and safe.
 */
#define MBQ_STATIC_SCRATCH_BYTES (8u << 20)
size_t mbq_static_scratch_bytes(void);
mbq_status mbq_linear_static(const uint16_t* X, int64_t T, const void* blob, int64_t N, int64_t K,
                             const int32_t* prec, const int32_t* perm, const int32_t* offsets, float* Y,
                             int algo, void* stream);

/*
 * mbq_linear_group - mbq_linear for n_proj weight matrices with the same K that read the SAME
 * activations (q/k/v, gate/up of a decoder block), each with its own routing; one launch for all
 * of them while every matrix takes a decode kernel (up to 64 tokens, 128 with AUTO on matrices
 * that keep the register-stationary kernel; Sec. 4.3, fused launch for the projections of a
 * layer), otherwise one launch sequence per matrix.  Results are those of n_proj separate
 * mbq_linear calls (bit for bit where mbq_linear is reproducible, see there).
 *   blob_host, prec_host, perm_host, offsets_host, Y_host : HOST arrays of n_proj DEVICE
 *   pointers (meaning as in mbq_linear); N_host : HOST array of the n_proj row counts.  The
 *   arrays are read before the call returns.  1 <= n_proj <= MBQ_MAX_GROUP.
 *   ws : at least max_i mbq_linear_workspace_bytes(T, N_host[i], K) bytes, 256-byte aligned
 */
mbq_status mbq_linear_group(const uint16_t* X, int64_t T, int64_t K, int n_proj,
                            const void* const* blob_host, const int64_t* N_host,
                            const int32_t* const* prec_host, const int32_t* const* perm_host,
                            const int32_t* const* offsets_host, float* const* Y_host, void* ws,
                            size_t ws_bytes, int algo, void* stream);

/*
 * mbq_routed_linear_group - mbq_route_group followed by mbq_linear_group on the same
 * projections: one decoder-block stage (route the tokens for q/k/v, or gate/up, or one
 * projection alone, then compute their outputs).  Same results and the same outputs (prec,
 * perm, offsets, Y) as the two calls.  Up to 16 tokens the router launch also carries the decode
 * kernel's activation preparation, and up to 128 tokens (while every matrix takes a decode
 * kernel) the token sort moves into the linear launch, so the stage is two launches.
 *   ws_route  : as ws in mbq_route
 *   ws_linear : as ws in mbq_linear_group
 * const int32_t* and int32_t* arrays: prec_host etc. are written by the routing step and read
 * by the linear step.
 */
mbq_status mbq_routed_linear_group(const uint16_t* X, int64_t T, int64_t K, int n_proj,
                                   const float* const* Wr_host, const float* const* br_host, int P,
                                   const void* const* blob_host, const int64_t* N_host,
                                   int32_t* const* prec_host, int32_t* const* perm_host,
                                   int32_t* const* offsets_host, float* const* Y_host, void* ws_route,
                                   size_t ws_route_bytes, void* ws_linear, size_t ws_linear_bytes,
                                   int algo, void* stream);

/* ------------------------------------------------------------------------------------------------
 * Other slice configurations (Sec. 4.1: E slices of b_e bits; App. C.1: slice_bits_list, group size)
 * ------------------------------------------------------------------------------------------------
 * The method is stated for any number of slices E and any widths b_e: slice 0 is a b_0-bit quantiser with
 * s_0 = (max - min) / 2^b_0 and z_0 = -min / s_0, slice e >= 1 has s_e = s_(e-1) / 2^b_e and z_e = 2^(b_e - 1)
 * (App. B), precision p uses slices 0..p, B_p = b_0 + ... + b_p bits.
 *
 * What this library runs: 1 <= E <= MBQ_MAX_SLICES, b_e >= 1, B_(E-1) <= 8, group 128, 64 or 32 - e.g. {2,2,2,2}
 * (the default), {4,2,2}, {4,4}, {6,2}, {8}, {2,2,2}, {3,1,2,2}, {3,2,1}, {4,1,1,2}.  For all of these at group 128 the
 * packed blob is THE SAME as the default one: a slice of b bits with the centred zero point 2^(b-1) splits into narrower slices with their
 * centred zero points without changing a bit (the codes are runs of bits of one eight-bit code, the scales powers of
 * two of s_0), so a configuration only says where that code may be cut, and its (s_0, z_0) are the stored ones times
 * 2^(2 - b_0) and 2^(b_0 - 2).  mbq_encode_cfg therefore writes the blob of mbq_encode.
 * What does know the configuration is the router: it has E outputs, and output q stands for the first B_q bits.
 *   - Every B_q even ("digit configurations"): the prec arrays written by the *_cfg router calls hold B_q / 2 - 1,
 *     the number of 2-bit digits minus one, which is what every mbq_linear* call reads (for the default configuration
 *     that is q itself): all linear kernels run unchanged and at full speed.
 *   - Some B_q odd ("bit configurations"): the prec arrays hold B_q - 1, and only mbq_linear_cfg and
 *     mbq_routed_linear_group_cfg understand them.  The one-token-tile decode kernels run them (they hand
 *     the two bits of every 2-bit code to the matrix cores separately, gated per token: twice the MFMAs, the same
 *     memory traffic): one launch up to 16 tokens, and beyond, with algo AUTO or DECODE, one launch per 16 tokens -
 *     a pass over the weights each, so a long prompt under a bit configuration costs a multiple of what it costs
 *     under a digit configuration.  MBQ_ALGO_SIMPLE and MBQ_ALGO_PREFILL take the one-thread-per-output kernel,
 *     which is correct and very slow.
 * mbq_config_precision_value(cfg, q) is what a prec array holds for the configuration's precision q, and
 * mbq_config_counts_bits(cfg) says which of the two cases it is.  perm and offsets (always MBQ_N_PRECISIONS + 1
 * entries) sort and bucket the tokens by the number of 2-bit digits they touch, ceil(B_q / 2) - 1, in both cases.
 * Groups of 64 or 32 columns (K still a multiple of 128): the code section of the blob is laid out as for 128, the
 * {s0, z0} section holds 256 / group pairs per row and 256-column tile instead of two (pair of group g of row n at
 * index ((n / 16) * (256 / group) * KB + g) * 16 + n % 16), so the blob is larger: size it with mbq_blob_bytes_cfg,
 * write it with mbq_encode_cfg and hand it ONLY to the *_cfg calls with the same configuration (nothing in the blob
 * records its group size).  mbq_linear_cfg and mbq_routed_linear_group_cfg run these blobs through the
 * one-thread-per-output kernel of MBQ_ALGO_SIMPLE at every token count: correct and slow; none of the fast kernels
 * reads the larger metadata section.  scale / zero of mbq_unpack_cfg are then fp32 [N][K/group].
 * Other group sizes: not built; the calls below refuse them with MBQ_ERR_BAD_SHAPE.  Scale and zero point are
 * stored as fp32 whatever the configuration; a pipeline that keeps them in 16 bits hands its rounded values to
 * mbq_encode_with_params and gets the codes that belong to them.
 */
#define MBQ_MAX_SLICES 4
typedef struct mbq_config {
  int n_slices;                   /* E */
  int slice_bits[MBQ_MAX_SLICES]; /* b_e, e < n_slices */
  int group;                      /* columns per quantisation group */
} mbq_config;

/* MBQ_OK if the library runs this configuration, else MBQ_ERR_BAD_SHAPE (mbq_last_error says why). */
mbq_status mbq_config_check(const mbq_config* cfg);
/* B_p, the bits of precision p; -1 for a bad configuration or index. */
int mbq_config_bits(const mbq_config* cfg, int p);
/* What the prec arrays hold for the configuration's precision p; -1 for a bad configuration or index. */
int mbq_config_precision_value(const mbq_config* cfg, int p);
/* 1 if the configuration's prec arrays count bits (some B_p is odd), 0 if digits, -1 for a bad configuration. */
int mbq_config_counts_bits(const mbq_config* cfg);

/* Blob bytes under the configuration (= mbq_blob_bytes at group 128); 0 for a bad configuration or shape. */
size_t mbq_blob_bytes_cfg(const mbq_config* cfg, int64_t N, int64_t K);
/* mbq_encode for a configuration (Sec. 4.1 Eq. 2): checks it, then writes the blob described above. */
mbq_status mbq_encode_cfg(const float* W, int64_t N, int64_t K, const mbq_config* cfg, void* blob, void* stream);
/*
 * mbq_unpack in the configuration's own terms, for checking against an independent implementation of the
 * general recursion: codes uint8 [E][N][K] (slice e's b_e-bit codes), scale / zero fp32 [N][K/group] = (s_0, z_0) of
 * the configuration's first slice.  Any of the three outputs may be null.
 */
mbq_status mbq_unpack_cfg(const void* blob, int64_t N, int64_t K, const mbq_config* cfg, uint8_t* codes,
                          float* scale, float* zero, void* stream);
/* W^(p) of the configuration (Eq. 3), fp32 [N][K]; p < E. */
mbq_status mbq_dequant_cfg(const void* blob, int64_t N, int64_t K, const mbq_config* cfg, int p, float* What,
                           void* stream);
/*
 * mbq_route, mbq_route_group, mbq_routed_linear_group for a configuration: Wr is fp32 [E][K] and br fp32 [E] per
 * router, logits (mbq_route_cfg) fp64 [T][E]; argmax over the E outputs, first maximum wins; prec as described
 * above.  Everything else as in the calls without _cfg.
 */
/*
 * mbq_linear on precision arrays written under a configuration (see above): a digit configuration is mbq_linear
 * itself; a bit configuration takes the one-token-tile decode kernels (algo AUTO or DECODE; 16 tokens per launch)
 * or the slow checker kernel.  perm and offsets may be null for a bit configuration (neither kernel reads them).
 */
mbq_status mbq_linear_cfg(const uint16_t* X, int64_t T, const void* blob, int64_t N, int64_t K,
                          const mbq_config* cfg, const int32_t* prec, const int32_t* perm, const int32_t* offsets,
                          float* Y, void* ws, size_t ws_bytes, int algo, void* stream);
mbq_status mbq_route_cfg(const uint16_t* X, int64_t T, int64_t K, const float* Wr, const float* br,
                         const mbq_config* cfg, int32_t* prec, int32_t* perm, int32_t* offsets, double* logits,
                         void* ws, size_t ws_bytes, void* stream);
mbq_status mbq_route_group_cfg(const uint16_t* X, int64_t T, int64_t K, int n_proj, const float* const* Wr_host,
                               const float* const* br_host, const mbq_config* cfg, int32_t* const* prec_host,
                               int32_t* const* perm_host, int32_t* const* offsets_host, void* ws, size_t ws_bytes,
                               void* stream);
mbq_status mbq_routed_linear_group_cfg(const uint16_t* X, int64_t T, int64_t K, int n_proj,
                                       const float* const* Wr_host, const float* const* br_host,
                                       const mbq_config* cfg, const void* const* blob_host, const int64_t* N_host,
                                       int32_t* const* prec_host, int32_t* const* perm_host,
                                       int32_t* const* offsets_host, float* const* Y_host, void* ws_route,
                                       size_t ws_route_bytes, void* ws_linear, size_t ws_linear_bytes, int algo,
                                       void* stream);

/*
 * Activation-quantised variant (App. E.4; `abits` of App. C.1: the paper's W3A4 / W4A4 / W5A4 runs use abits = 4)
 * -------------------------------------------------------------------------------------------------------------
 * App. E.4 keeps the sliced weights and the routers and changes what they are fed.  With a per-input-channel shift
 * delta and scale s (the equivalent transform of the pipeline the paper builds on),
 *     X~ = (X - delta) / s,   W~ = s (.) W,   B~ = B + delta W      so that  X~ W~ + B~ = X W + B,
 * the main path multiplies the QUANTISED X~ with the slices of W~ (encode W~ with mbq_encode; folding s and delta into
 * the weights and the bias is the caller's offline step), and the router reads the same quantised activations taken
 * back to the original space, X_r = X~ (.) s + delta, so that it keeps working in the space it was trained in.
 * The quantiser is not spelled out by the paper; this library takes the usual dynamic per-token asymmetric one with
 * an integer zero point, every step ONE fp32 operation in this order: for a token's row t = X~[i][:],
 *     lo = min(min t, 0), hi = max(max t, 0), scale = max(hi - lo, 2^-100) / (2^abits - 1),
 *     zp = clamp(rint(-lo / scale), 0, 2^abits - 1),  q = clamp(rint(t / scale) + zp, 0, 2^abits - 1)
 * (rint: to nearest, ties to even; inputs must be finite).
 *
 * mbq_act_quant writes, for T tokens,
 *   Xint      : bf16 [T][K], the integers q - zp (|q - zp| <= 2^abits - 1: exact in bf16).  This is the X of the
 *               linear calls: they multiply it exactly (also the decode kernels, whose two-piece split holds eight
 *               bits), and Y[i][:] = row_scale[i] * (Xint[i][:] W~^(p_i)^T) + B~ is the layer's output;
 *   row_scale : fp32 [T], the token's scale;
 *   Xr        : bf16 [T][K] (may be NULL), the router's input ((q - zp) * scale) * s + delta, each step one fp32
 *               operation, then rounded to nearest even - pass it as X to the mbq_route* calls.
 *   X         : bf16 [T][K] (read) - the activations in the ORIGINAL space when let_shift / let_scale (fp32 [K]
 *               each, both or neither) are given: the call applies (x - delta) / s itself; with both NULL, X is
 *               taken as X~ and Xr is the dequantised X~.
 * 2 <= abits <= 8; K a multiple of 128; X, Xint, Xr, let_shift, let_scale 16-byte aligned.
 * mbq_scale_rows finishes the main path in place: Y[i][n] = Y[i][n] * row_scale[i] (+ bias[n] if bias is not NULL;
 * fp32 [N]), one multiplication and one addition.
 * Both are plain streaming launches (one workgroup per token / one thread per output); a stage of the variant is
 * mbq_act_quant, mbq_route_group on Xr, mbq_linear_group on Xint, mbq_scale_rows per projection.
 */
mbq_status mbq_act_quant(const uint16_t* X, int64_t T, int64_t K, int abits, const float* let_shift,
                         const float* let_scale, uint16_t* Xint, float* row_scale, uint16_t* Xr, void* stream);
mbq_status mbq_scale_rows(float* Y, int64_t T, int64_t N, const float* row_scale, const float* bias, void* stream);
/*
 * One stage of the variant in one call: mbq_act_quant on X, mbq_routed_linear_group with the routers reading Xr and
 * the linear kernels Xint (up to 16 tokens the router launch prepares Xint for the decode kernel as it prepares X in
 * the weight-only stage), then the row scaling and bias of all projections in one launch - four launches where the
 * weight-only stage has two.  Same results as the separate calls, bit for bit.
 *   bias_host : host array of n_proj device pointers, fp32 [N_i] each; the array or any entry may be NULL
 *   Xint, row_scale, Xr : as in mbq_act_quant, all three required (T > 0); they are outputs the caller may read
 *   everything else as in mbq_act_quant and mbq_routed_linear_group; on failure some launches may already have been
 *   enqueued (the calls it is made of check their own arguments in turn).
 */
mbq_status mbq_routed_linear_group_act(const uint16_t* X, int64_t T, int64_t K, int abits, const float* let_shift,
                                       const float* let_scale, int n_proj, const float* const* Wr_host,
                                       const float* const* br_host, int P, const void* const* blob_host,
                                       const int64_t* N_host, const float* const* bias_host,
                                       int32_t* const* prec_host, int32_t* const* perm_host,
                                       int32_t* const* offsets_host, float* const* Y_host, uint16_t* Xint,
                                       float* row_scale, uint16_t* Xr, void* ws_route, size_t ws_route_bytes,
                                       void* ws_linear, size_t ws_linear_bytes, int algo, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MBQ_H_ */
