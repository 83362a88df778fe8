/*
 * pact_measure.h - measurement and inspection entry points of libpact.  They are not part of
 * the method and no product call needs them: benchmarks and profiler runs use them to time the
 * library's kernels one by one, to calibrate hardware byte counters, and to look at how a batch
 * is dealt to the chip.  Status codes are those of pact.h.
 */
#ifndef PACT_MEASURE_H
#define PACT_MEASURE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Per-kernel timing.  While enabled, every kernel the library enqueues is bracketed by events
 * on its stream.  pact_profile_read synchronises those events and returns the number of records
 * since the last pact_profile_reset (or -1 if an event call failed); names[i] points to a static
 * string, ms[i] is the kernel's duration.  Host pointers.  Not thread-safe; leave disabled in
 * production (the brackets keep kernels from overlapping their launch with the previous one). */
int pact_profile_enable(int on);
int pact_profile_reset(void);
int pact_profile_read(const char** names, float* ms, int32_t max_records);

/* Plain device-to-device copy of `bytes` bytes (a multiple of 16; src and dst 16-byte aligned,
 * not overlapping) by one kernel named pact::calibration_copy_kernel: it reads and writes
 * exactly `bytes` bytes, which gives hardware byte counters (rocprofv3's FETCH_SIZE and
 * WRITE_SIZE) a dispatch of known traffic to be scaled by. */
int pact_calibration_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Host only, nothing is enqueued: how a matrix pass of a batched call deals the chip's 256
 * workgroup slots to the samples, given the number of output tiles each sample is expected to
 * have.  Slot i runs on XCD i mod 8.
 *   tiles     [batch] host      expected tiles per sample (>= 1)
 *   wg_map    [256] host out    (sample << 8) | (number of that workgroup within its sample), 0xFFFF = spare slot
 *   wg_count  [batch] host out  workgroups per sample: at least 1, at most its tiles, so that the
 *                               most loaded workgroup has as few tiles as 256 slots allow
 * Returns PACT_OK, PACT_ERR_NULL or PACT_ERR_SHAPE. */
int pact_plan_workgroups(const int32_t* tiles, int32_t batch, uint16_t* wg_map, uint16_t* wg_count);

#ifdef __cplusplus
}
#endif
#endif /* PACT_MEASURE_H */
