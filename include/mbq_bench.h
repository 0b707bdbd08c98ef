/*
 * mbq_bench - measurement and diagnostic entry points of libmbq.so.
 *
 * Nothing here is part of the layer (include/mbq.h is): these calls exist so that the
 * benchmark can print what the machine itself reaches next to the published peaks (a plain
 * streaming copy, a read-only stream, an MFMA loop fed from LDS), time the decode linear
 * kernel without the launch that prepares its activations, and record where the time of
 * that kernel goes.  Conventions as in mbq.h: device pointers unless the name ends in
 * _host, work is enqueued on `stream`, every call returns an mbq_status.
 */
#ifndef MBQ_BENCH_H_
#define MBQ_BENCH_H_

#include "mbq.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * mbq_bench_copy - dst[0..bytes) = src[0..bytes), 16 bytes per lane, grid-stride, one workgroup of
 * 512 threads per compute unit times `waves_of_workgroups` (>= 1).  Moves 2 x bytes through HBM when
 * the buffers do not fit the last-level cache.  bytes must be a multiple of 16; src, dst 16-byte aligned.
 */
mbq_status mbq_bench_copy(const void* src, void* dst, size_t bytes, int waves_of_workgroups, void* stream);

/*
 * mbq_bench_read - reads src[0..bytes) once (same launch shape, loads carry the non-temporal hint
 * like the decode kernels' weight loads) and folds it into 4 bytes at `sink` (written only if the
 * fold hits one particular value, so that the loads cannot be dropped).
 */
mbq_status mbq_bench_read(const void* src, size_t bytes, int waves_of_workgroups, void* sink, void* stream);

/*
 * mbq_bench_mfma_loop - the matrix-core rate this chip sustains on the prefill kernel's
 * instruction (v_mfma_f32_32x32x16_bf16) with operands read from LDS: one workgroup of 8 wavefronts
 * per compute unit, every wavefront runs `steps` steps of 16 MFMAs on a 128 x 64 accumulator tile
 * (4 x 2 MFMA tiles, fragments re-read from LDS each step); with_barrier != 0 adds one workgroup
 * barrier per step.  *flops_host receives the flops of the launch (2 x 32 x 32 x 16 per MFMA).
 *   sink : 4 bytes (device), written only if the result hits one particular value
 */
mbq_status mbq_bench_mfma_loop(int steps, int with_barrier, void* sink, double* flops_host, void* stream);

/*
 * mbq_bench_linear_group_prepared - the linear kernel of mbq_linear_group alone, for T <= 16:
 * the launch that prepares the activations (and clears outputs the kernel adds into) is skipped,
 * so `ws` must hold what an earlier mbq_linear_group / mbq_routed_linear_group call on the same X
 * and T left there, and Y what that call left there.  The outputs are NOT meaningful (a kernel that
 * adds into Y adds a second time); only the duration of the launch is.  Arguments as in
 * mbq_linear_group.
 */
mbq_status mbq_bench_linear_group_prepared(int64_t T, int64_t K, int n_proj, const void* const* blob_host,
                                           const int64_t* N_host, const int32_t* const* prec_host,
                                           float* const* Y_host, const void* ws, size_t ws_bytes, void* stream);

/*
 * mbq_bench_decode_timeline - the same launch (T <= 16, K <= 8192) from a build of the kernel
 * that notes the 100 MHz wall clock at its phase boundaries.  stamps receives, per workgroup b
 * (b < mbq_bench_decode_timeline_workgroups()) and wavefront w (w < 9: eight arithmetic wavefronts,
 * then the loader), 32 words at stamps[(9 b + w) 32 ...]:
 *   arithmetic wavefronts: 0 kernel entry, 1 precisions and activations arrived, 4 + 2 i MFMAs of the
 *   workgroup's i-th tile done, 5 + 2 i its partial tile filed (and, by the wavefront that came last,
 *   the outputs stored) (i < 13), 30 end, 31 hardware id (XCC_ID << 32 | HW_ID);
 *   loader: 0 entry, 1 precisions arrived, 2 first weight block issued, 4 + i block i published to
 *   the arithmetic wavefronts (i < 26), 30 end, 31 hardware id.  Unused words are zero; the caller
 *   clears the buffer (workgroups that the launch does not need write nothing).
 * stamps_bytes >= mbq_bench_decode_timeline_bytes().
 */
size_t mbq_bench_decode_timeline_bytes(void);
int mbq_bench_decode_timeline_workgroups(void);
mbq_status mbq_bench_decode_timeline(int64_t T, int64_t K, int n_proj, const void* const* blob_host,
                                     const int64_t* N_host, const int32_t* const* prec_host,
                                     float* const* Y_host, const void* ws, size_t ws_bytes,
                                     unsigned long long* stamps, size_t stamps_bytes, void* stream);

/*
 * mbq_set_knob - test and experiment hooks (process-wide, 0 = default = off).  A call into the library reads
 * them once, on entry, so a change never takes effect in the middle of a call.
 *   knob 0: waves per workgroup of the 17..64-token decode kernels (4, 8 or 16)
 *   knob 1: K split (workgroups along K) of the multi-tile decode kernel, 0 = automatic
 *   knob 2: workgroups per compute unit of the register-stationary decode kernel, 0 = automatic
 *   knob 3: decode kernel choice: 0 automatic, 1 multi-tile kernel, 2 register-stationary kernel (both switch the
 *           FP4-operand kernels of T <= 16 off)
 *   knob 4: 1 = route small batches with the general router kernel too
 *   knob 5: K split of the prefill kernel (1..8 workgroups per tile, partial sums added into Y), 0 = automatic
 *   knob 7: 3 = the 17..64-token register-stationary kernel takes one token tile per workgroup
 */
mbq_status mbq_set_knob(int knob, int value);

#ifdef __cplusplus
}
#endif
#endif /* MBQ_BENCH_H_ */
