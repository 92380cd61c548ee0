/*
 * tli_bench.h -- benchmark, profiling and tuning utilities of the TLI library.  None of them is part of the
 * method; the method's calls are in tli.h.
 */
#ifndef TLI_BENCH_H
#define TLI_BENCH_H

#include <stddef.h>
#include <stdint.h>

#include "tli.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Optional per-kernel timing for benchmarks (not part of the method): while enabled, the hot calls
 * record a HIP event pair around each selected kernel on the caller's stream.  Not thread-safe.
 *   tli_profile_enable  : creates 2*max_calls events per selected kernel (bit k of kernel_mask selects
 *                         kernel k of tli_kernel_id) and records one launch in `every` (an event between two
 *                         kernels costs a few microseconds of idle GPU, so a timed loop samples);
 *                         recording stops silently once the events are used up.
 *   tli_profile_collect : waits for the recorded events of one kernel, returns the summed duration
 *                         in milliseconds and the number of launches, and resets that kernel's counter.
 *   tli_profile_disable : destroys the events.
 */
typedef enum {
    TLI_KERNEL_LSE = 0,        /* tli_verify: log-normalisers of the K target rows of every sequence      */
    TLI_KERNEL_ACCEPT = 1,     /* (no kernel of its own any more: the accept tests run inside ids 0 or 2)   */
    TLI_KERNEL_FINAL_SCAN = 2, /* tli_verify: chunk masses of the residual / bonus rows                   */
    TLI_KERNEL_FINAL_PICK = 3, /* tli_verify: draw of the extra token                                     */
    TLI_KERNEL_DRAFT_SCAN = 4, /* row samplers: scan of the rows (+ the draw, one workgroup/row); argmax scan  */
    TLI_KERNEL_DRAFT_PICK = 5, /* row samplers: the draw when rows are split over workgroups; argmax finish   */
    TLI_KERNEL_COUNT = 6
} tli_kernel_id;
int tli_profile_enable(uint32_t kernel_mask, int32_t max_calls, int32_t every);
int tli_profile_collect(int32_t kernel, double* total_ms, int32_t* launches);
void tli_profile_disable(void);

/*
 * Benchmark utility (not part of the method): a plain device-to-device copy of `bytes` (multiple of
 * 16, both pointers 16-byte aligned) by kernel k_calib_copy.  Hardware byte counters read for it are
 * compared with its known traffic (bytes read + bytes written) to calibrate those counters.
 */
int tli_calib_copy(const void* src_dev, void* dst_dev, size_t bytes, void* hip_stream);
/*
 * Benchmark utility (not part of the method): a read-only streaming pass over `bytes` of device memory with plain
 * 16-byte loads, the yardstick beside the vendor's peak that the streaming kernels are held against.  The buffer is
 * read as bytes / slab_bytes contiguous slabs, a workgroup of 256 threads per slab, in the access pattern of the
 * normaliser kernel (slab_bytes = one logit row's bytes gives that kernel's launch shape).
 *   src_dev      dev, 16-byte aligned; bytes a multiple of slab_bytes; slab_bytes a multiple of 4096
 *   nontemporal  0: ordinary loads, 1: loads that bypass cache allocation (what the kernels use)
 *   out_dev      dev [bytes / slab_bytes] uint32 scratch (a word per workgroup; practically never written)
 * Only enqueues a kernel on the stream.
 */
int tli_calib_read(const void* src_dev, size_t bytes, size_t slab_bytes, int32_t nontemporal, uint32_t* out_dev,
                   void* hip_stream);

/*
 * Benchmark utility (not part of the method): what the HIP runtime reports for the current device, so that a
 * bandwidth figure can be quoted against the machine's own numbers beside the vendor's.
 *   out [4] host : memory clock in kHz, memory bus width in bits, compute units, engine clock in kHz
 *                  (0 for an attribute the runtime does not report)
 * TLI_ERR_HIP if no device can be queried.
 */
int tli_device_info(int32_t* out);

/*
 * Tuning / test switch: which form the first steps of tli_verify take (standard SD appendix, verification loop).
 *   0 : by batch size (the default): a persistent workgroup per sequence, which streams the sequence's target rows
 *       and takes the accept tests as the rows complete, when the batch gives every compute unit about one sequence
 *       or several; else the split form;
 *   1 : always the split form (a workgroup per target row, then the kernel that takes the accept tests);
 *   2 : a workgroup per sequence wherever a row's chunk tables fit its LDS.
 * Both forms make the same decisions and return the same tokens and flags; normalisers agree to the rounding of the
 * last fp64 sum.  Process-wide, not thread-safe.  TLI_ERR_INVALID_ARG for any other value.
 */
int tli_tune_final_path(int32_t path);

#ifdef __cplusplus
}
#endif
#endif /* TLI_BENCH_H */
