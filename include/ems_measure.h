/*
 * ems_measure.h -- measurement aids of libems (same library, not part of the verification
 * step): HIP-event timing of the attention kernel, a read-only streaming probe, the switch
 * between the matrix-core and the vector-ALU formulation of the attention kernel, and the
 * memory figures the runtime reports.  Used by the benchmark and the tests; a serving path
 * needs none of them.
 *
 * Thread safety: the timing state and the formulation switch are PER CALLING THREAD (thread-
 * local): ems_profile_enable / ems_set_attention_variant affect only attention calls made
 * later by the same thread, so a measurement in one thread never changes what another
 * thread's ems_verify_attention runs or records.
 */
#ifndef EMS_MEASURE_H
#define EMS_MEASURE_H

#include "ems.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Kernel timing.  ems_profile_enable(n) creates n triples of HIP events (host objects); from
 * then on each of the next n attention calls made by this thread records one triple on its
 * stream: right before its main attention kernel, right after it, and after the partial-
 * merge kernel that ends the call.  ems_profile_read waits for the recorded triples, returns
 * the summed elapsed milliseconds of the main kernel and the number of triples, and rearms
 * them; ems_profile_read_calls also returns the summed time of the whole calls, merge
 * included (total_call_ms, may be NULL).
 * ems_profile_enable(0) destroys the events and switches timing off.
 * Errors: n outside [0, 65536], NULL total_ms / launches -> INVALID_ARG; event failure -> HIP.
 */
EMS_API ems_status ems_profile_enable(int max_records);
EMS_API ems_status ems_profile_read(double* total_ms, int* launches);
EMS_API ems_status ems_profile_read_calls(double* total_ms, double* total_call_ms, int* launches);

/*
 * Measurement aid: one launch of a plain read-only streaming kernel over `bytes` bytes of
 * device memory at `buf` (16-byte aligned, bytes >= 1024; a tail shorter than 1 KiB is not
 * read), asynchronous on hip_stream.  Its rate is the read ceiling of the device that the
 * attention kernel's bandwidth is compared with.  `sink`: 4 writable device bytes (written
 * only if the data folds to one particular pattern).  Touches nothing else.
 */
EMS_API ems_status ems_stream_read_probe(const void* buf, size_t bytes, void* sink, void* hip_stream);

/*
 * Measurement aid: which arithmetic units the attention kernel of ems_verify_attention and
 * ems_verify_attention_write_through uses for its two contractions (scores and weighted
 * sum of values).  EMS_ATTN_MFMA (the default) runs them on the matrix cores; EMS_ATTN_VALU
 * runs the same tiles, loads and merge on the vector ALU (packed dot products and FMAs),
 * so that the two can be timed against each other on one input.  Results of both meet
 * the same tolerance.  Per calling thread; takes effect with that thread's next call; the padded ablation
 * always uses the matrix cores.  Any other value: EMS_ERR_INVALID_ARG, setting unchanged.
 * While EMS_ATTN_VALU is selected, calls with D = 80, with a token tree, or with so many
 * samples that the per-row state no longer fits the 160 KiB of LDS next to the B+1 prefix
 * sums (D = 128: B > 3967) return EMS_ERR_UNSUPPORTED.
 */
typedef enum ems_attention_variant {
    EMS_ATTN_MFMA = 0,
    EMS_ATTN_VALU = 1
} ems_attention_variant;
EMS_API ems_status ems_set_attention_variant(int variant);
EMS_API int ems_get_attention_variant(void);

/*
 * What the HIP runtime reports for the current device's memory: clock in kHz, bus width in
 * bits (either may come back 0 where the runtime reports nothing).  Context for bandwidth
 * figures; the library itself does not use them.  Host pointers, both required.
 * Errors: NULL pointer -> INVALID_ARG; runtime failure -> HIP.
 */
EMS_API ems_status ems_device_memory_figures(int* memory_clock_khz, int* memory_bus_width_bits);

#ifdef __cplusplus
}
#endif
#endif /* EMS_MEASURE_H */
