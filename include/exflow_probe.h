/* exflow_probe.h — measurement probes of libexflow_moe.so.
 *
 * Not part of the method's boundary (exflow_moe.h): these calls have no counterpart in the paper.
 * The benchmark uses them to report the rates this GPU sustains next to the data-sheet peaks and
 * to calibrate the profiler's HBM byte counters.  Same conventions as exflow_moe.h: device
 * pointers, caller-owned buffers, host-side validation before any launch, asynchronous on `stream`.
 */
#ifndef EXFLOW_PROBE_H
#define EXFLOW_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---------------------------------------------------------------------------------------
 *   exf_probe_copy: dst[0..bytes) = src[0..bytes), a plain streaming copy; bytes % 16 == 0,
 *                   both device pointers 16-byte aligned.
 *   exf_probe_mfma: `workgroups` x 256 threads, every wavefront issues 4*iters independent
 *                   32x32x16 bf16 MFMAs (4*iters*32768 flop per wavefront); out receives
 *                   workgroups*256 floats (device) so that the loop cannot be removed.
 *   exf_probe_gemm_loop: the bare K loop of a 256x256x64-tiled bf16 GEMM (direct-to-LDS operand
 *                   loads, LDS operand fetches, MFMAs, one barrier per K tile; no epilogue) over
 *                   caller-supplied operands: `operands` holds exf_probe_gemm_loop_bytes() bytes
 *                   (8 x [1024,1024] activations followed by 8 x [4096,1024] weights, bf16);
 *                   256 workgroups walk all 512 output tiles `passes` times, i.e.
 *                   passes * 512 * 2*256*256*1024 flop; out receives 256*256 floats.  The rate it
 *                   reaches depends on the operand values (all zeros against random numbers).
 *   exf_probe_ffn_timeline: moe_expert_ffn_fused (bf16, erf GELU, no biases; same arguments and
 *                   validation) that also records where the time of every workgroup of its two
 *                   grouped-GEMM launches goes.  timeline (device) holds 2 * capacity records of
 *                   eight uint64: records [0, capacity) belong to the first contraction, [capacity,
 *                   2 capacity) to the second; record b is written by workgroup b (workgroups b >=
 *                   capacity write nothing): [0] start, [1] tile located, [2] first K tile landed,
 *                   [3] K loop done, [4] end or 0 if the workgroup had no tile - all in ticks of the
 *                   constant 100 MHz device clock -, [5] hardware id, [6] tile kind (0 full, 1 remainder,
 *                   2 tall) | expert << 8 | column tile << 16 | rows << 32 | K tiles << 48, [7] the experts'
 *                   row ranges have arrived (same clock; between [0] and [1]).
 * ------------------------------------------------------------------------------------- */
int exf_probe_copy(void* dst, const void* src, size_t bytes, void* stream);
int exf_probe_mfma(int workgroups, int iters, float* out, void* stream);
size_t exf_probe_gemm_loop_bytes(void);
int exf_probe_gemm_loop(const void* operands, size_t bytes, int passes, float* out, void* stream);
int exf_probe_ffn_timeline(const void* x, const int32_t* src_of_sorted, const int32_t* sorted_of_src,
                           const float* topk_w, const int32_t* expert_offsets, const void* w1,
                           const void* w2, int64_t T, int k, int d, int f, int E_local, void* out,
                           void* workspace, size_t workspace_bytes, uint64_t* timeline, int capacity,
                           void* stream);

#ifdef __cplusplus
}
#endif
#endif /* EXFLOW_PROBE_H */
