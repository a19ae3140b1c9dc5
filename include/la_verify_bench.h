/*
 * la_verify_bench.h -- benchmark aids of the verification library: per-kernel
 * event timing, two calibration kernels and a self-test hook.  None of them is
 * part of the verification path.  They exist only in libla_verify_bench.so,
 * which is libla_verify.so's objects linked together with these aids (same
 * kernels, same entry points); the product library does not contain them and
 * keeps no state.
 */
#ifndef LA_VERIFY_BENCH_H
#define LA_VERIFY_BENCH_H

#include "la_verify.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ------------------------------------------------------------------------- *
 *  Calibration (benchmark aid, not part of the verification path): what the
 *  chip at hand reaches on a pure bf16 MFMA loop and on a pure streaming read,
 *  to quote a roofline fraction against the achievable rate beside the
 *  published peak.  Both only enqueue a kernel; time them with la_profile_*
 *  (slots "calib_mfma", "calib_read") or with events of your own.
 *
 *  la_calibrate_mfma: `workgroups` x 8 wavefronts, each `iters` rounds of four
 *  independent v_mfma_f32_32x32x16_bf16; *flops (host) receives the launch's
 *  flop count.  sink: dev, workgroups * 512 floats, written.
 *  la_calibrate_mfma_data: the same loop (same arguments, `iters` even, same
 *  profiling slot) on eight operand pairs per lane of pseudo-random bf16 values
 *  used in rotation: the matrix pipeline's inputs toggle as on real data, which
 *  is what a power-managed clock responds to.
 *  la_calibrate_read: reads `bytes` (a multiple of 16 is read) from src (dev,
 *  16-byte aligned) once; sink: dev, one word (written practically never).
 * ------------------------------------------------------------------------- */
LA_API la_status la_calibrate_mfma(int32_t workgroups, int32_t iters, float *sink, double *flops, void *hip_stream);
LA_API la_status la_calibrate_mfma_data(int32_t workgroups, int32_t iters, float *sink, double *flops,
                                        void *hip_stream);
LA_API la_status la_calibrate_read(const void *src, size_t bytes, uint32_t *sink, void *hip_stream);

/* Instruction-mix probe: `workgroups` workgroups of `waves` (4 or 8: one or two
 * per SIMD) wavefronts, each running `iters` rounds of a body of 16 slots of
 * mix `mix`:
 *   0 v_add_f32   1 v_exp_f32   2 v_cvt_pk_bf16_f32
 *   3 v_mfma_f32_32x32x16_bf16 (four accumulators in turn, one operand pair)
 *   4 the same with eight different operand register pairs
 *   5 MFMA + 4 v_add_f32        6 MFMA + 8 v_add_f32
 *   7 MFMA + v_exp_f32 + (every other slot) v_cvt_pk_bf16_f32 + 2 v_add_f32,
 *     the softmax share of one MFMA in the attention kernels.
 * mix_second >= 0 (only with waves == 8, and only 3 with 0 or 1): the second
 * wavefront of every SIMD runs that mix instead.  Time the launch with events
 * of your own: duration x clock / (iters x 16) is cycles per slot.  sink: dev,
 * workgroups * 512 floats, written.  Only enqueues a kernel.
 * LA_ERR_UNSUPPORTED for a pair of mixes that is not built. */
LA_API la_status la_calibrate_issue(int32_t mix, int32_t mix_second, int32_t waves, int32_t workgroups,
                                    int32_t iters, float *sink, void *hip_stream);

/* ------------------------------------------------------------------------- *
 *  Self-test hook (not part of the verification path): out[i] = exp(y[i]) as
 *  the fp64 resampling path of la_spec_accept evaluates it (its own routine:
 *  two-term argument reduction, degree-13 polynomial, ldexp; meant for
 *  y <= 0, arguments below -750 give 0), so that its accuracy can be checked
 *  against a reference exponential.  y, out: dev, n doubles each, n >= 1.
 *  Only enqueues a kernel.
 * ------------------------------------------------------------------------- */
LA_API la_status la_selftest_exp64(const double *y, double *out, size_t n, void *hip_stream);

/* ------------------------------------------------------------------------- *
 *  Self-test hook for the streaming kernel shapes of an fp8 cache.  Their
 *  unmasked tiles never move the base their probabilities are formed against
 *  (Section 3.2's verification pass needs no such thing; it is this
 *  implementation's way to keep the accumulators of O in place); a workgroup
 *  that meets a score 60 log2 units above its base gives up and reduces its
 *  chunk a second time in a general form.  With on != 0 every workgroup of
 *  those shapes takes that second attempt in the la_verify_attention calls
 *  that follow, whatever its scores, so that a test can compare the two.
 *  Process-wide, host side only; 0 restores the normal behaviour.
 * ------------------------------------------------------------------------- */
LA_API la_status la_selftest_second_attempt(int on);

/* ------------------------------------------------------------------------- *
 *  Index checks (debug aid).  The compute calls trust the indices the caller
 *  hands them -- cache block ids and drafted token ids are not range-checked
 *  on the device -- and a checked build of an application can run these two
 *  scans in front of them.  Each only enqueues small kernels on hip_stream and
 *  writes three int32 to `report` (dev): the number of offending entries, and
 *  the two coordinates of one of them (any one; -1, -1 when there is none).
 *  Read `report` after the stream has been synchronised.
 *
 *  la_check_block_tables: the entries of block_tables (dev
 *  [num_requests, max_blocks_per_request]) that a call with these prefix
 *  lengths plus `extra_tokens` appended tokens per request would touch, i.e.
 *  logical blocks 0 .. ceil((P_b + extra_tokens) / block_size) - 1 of request
 *  b; an entry offends when it is outside [0, num_cache_blocks).  Coordinates:
 *  request, logical block.  block_tables == NULL (contiguous cache): the
 *  identity ids b*max_blocks + j are checked against num_cache_blocks instead.
 *  LA_ERR_INVALID_ARG for a bad descriptor, a prefix (plus extra tokens) longer
 *  than max_blocks_per_request blocks, extra_tokens < 0, num_cache_blocks < 0.
 *
 *  la_check_draft_tokens: draft_tokens (dev [num_branches, num_draft]); an
 *  entry offends when it is outside [0, vocab).  Coordinates: branch, position.
 * ------------------------------------------------------------------------- */
LA_API la_status la_check_block_tables(const la_attn_desc *desc, const int32_t *block_tables,
                                       const int32_t *prefix_lens_host, int32_t extra_tokens,
                                       int64_t num_cache_blocks, int32_t *report, void *hip_stream);
LA_API la_status la_check_draft_tokens(const la_accept_desc *desc, const int32_t *draft_tokens, int32_t *report,
                                       void *hip_stream);

/* Per-kernel timing for benchmarks.  While enabled, every kernel the library
 * launches is bracketed by HIP events on the caller's stream (process-wide
 * state, not thread-safe; at most LA_PROFILE_MAX_RECORDS launches are kept,
 * later ones are dropped).  la_profile_collect synchronises on the recorded
 * events and accumulates them; la_profile_get then reports, per kernel slot,
 * its name, number of timed launches and their total duration.
 * la_profile_select narrows what is bracketed: bit k of slot_mask selects
 * kernel slot k (default: all), and of a selected slot's launches only every
 * stride-th one is timed (default 1); the event pairs cost a few microseconds
 * each on the stream, so a benchmark that wants its wall time undisturbed
 * times only the kernel it reports and a sample of its launches.  Returns
 * LA_ERR_INVALID_ARG for stride < 1. */
#define LA_PROFILE_MAX_RECORDS 8192
LA_API la_status la_profile_enable(int on);
LA_API la_status la_profile_select(uint32_t slot_mask, int32_t stride);
LA_API la_status la_profile_collect(void);
LA_API int32_t la_profile_num_kernels(void);
LA_API la_status la_profile_get(int32_t slot, const char **name, int64_t *launches, double *total_ms);
LA_API la_status la_profile_reset(void);

#ifdef __cplusplus
}
#endif
#endif /* LA_VERIFY_BENCH_H */
