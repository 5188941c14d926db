/*
 * libkda diagnostics: switches and queries for tests and measurement, not part of the product
 * interface of kda.h.  The switches are process-wide and read at the start of each call; they are
 * not synchronised with calls made from other threads at the same time.
 */
#ifndef KDA_DEBUG_H_
#define KDA_DEBUG_H_

#include "kda.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * 0 keeps the sequential stage of the matrix-core prefill to one workgroup per (sequence, head);
 * 1 (default) lets calls with few pairs and long sequences cut the chunk axis into ranges that
 * several workgroups walk at the same time.  The chunk recurrence of Section 3.1 is affine in the
 * state, S_out = T S_in + B, and decay makes T vanish: where the transition of the last 32 chunks of
 * a range is exactly zero in fp32, the state at the range's end is the offset of those chunks alone
 * and the next range starts after 32 steps (the short way).  A (sequence, head) for which some range
 * fails that test forms T and B of whole ranges and chains the range states through them (the
 * general way: two ranges' time instead of one).
 * Results agree within rounding, not bit for bit.  With 1 the library estimates whether, and into
 * how many ranges, a call is worth splitting; a value of 2..32 takes that many ranges whatever the
 * estimate says (still lowered to what the device and the sequence length allow; calls with fewer
 * than 24 chunks or more than 64 pairs are never split).
 * KDA_PREFILL_TIME_SPLIT=0 in the environment sets the default to 0.
 */
void kda_debug_set_time_split(int mode);

/*
 * Fault injection for the bounded waits of the matrix-core prefill, driven from the host so that
 * every kernel still runs to its end.  kda_debug_set_producers(0) makes the per-chunk workgroups of
 * later calls return at once: no slot is ever produced, so every wait of the sequential stage runs
 * out after kda_debug_set_wait_limit(ticks) ticks of the 100 MHz device wall clock (default
 * 200 000 000 = two seconds; 0 = give up at the first look).  Such a call still returns KDA_OK,
 * writes NaN to o and h_T (see kda_chunk_fwd) and leaves the status word that kda_chunk_fwd_check
 * reports.  kda_debug_set_producers(1) restores normal operation.
 */
void kda_debug_set_producers(int enabled);
void kda_debug_set_wait_limit(unsigned long long ticks);

/*
 * What kda_chunk_fwd (output_gate = 0) or kda_chunk_fwd_fused with an output gate (1) would do with
 * a workspace of `workspace_bytes` on the current device: out[0] chunk indices per time segment,
 * out[1] time segments, out[2] ranges of the time-split scan (1 = not split), out[3] chunks in the
 * first range of a segment, out[4] chunks in each of the others.  Launches nothing.
 */
kda_status kda_debug_chunk_fwd_plan(const kda_dims *dims, size_t workspace_bytes, int output_gate,
                                    int64_t out[5]);

/*
 * The raw status word that a bf16 prefill call left in `workspace` (same dims, workspace and size as
 * that call), after waiting for `hip_stream`.  Bits 1, 2, 4: the failures kda_chunk_fwd_check reports.
 * Bits 256 and 512 report, for a call whose scan was split into ranges, that some (sequence, head)
 * of any of its time segments took the short way (256) / the general way (512); no failure.
 */
kda_status kda_debug_chunk_fwd_status(const kda_dims *dims, const void *workspace, size_t workspace_bytes,
                                      void *hip_stream, unsigned *word);

/*
 * The device's own rates, for reading a roofline fraction against what this device delivers beside its
 * data-sheet peak.  Both launch one kernel on `hip_stream` and return at once; the caller times them.
 *
 * kda_debug_stream_probe: streams `bytes` (a multiple of 65 536, the size of one decode state) of the
 * device buffer `buffer` (16-byte aligned, overwritten) in tiles of 64 KiB, one workgroup of 256 threads per
 * tile, sixteen 16-byte accesses per thread: mode 0 reads only, 1 writes only, 2 reads, modifies and writes in
 * place, which is the traffic of kda_recurrent_step.
 *
 * kda_debug_mfma_probe: `workgroups` workgroups of four waves; every wave issues 16 * iters matrix products
 * 32x32x16 (f16 operands, fp32 accumulation, the instruction of the prefill kernels) on four independent
 * accumulators.  *flops (may be NULL) receives the floating-point operations of the launch; sink: one float of
 * device memory (never written in practice).
 */
kda_status kda_debug_stream_probe(int mode, float *buffer, size_t bytes, void *hip_stream);
/*
 * kda_debug_prefill_traffic_probe: the data movement of the two-stage matrix-core prefill and nothing else.  `buffer`
 * (device, 16-byte aligned, overwritten) holds bytes / 172 032 items of [64 KiB in][72 KiB slot][32 KiB out]; one
 * workgroup per item reads its input, writes its slot, reads the slot of the item half the buffer away (written by
 * another workgroup of the launch or an earlier one) and writes its output: 240 KiB through the memory system per
 * item, which is what kda_chunk_fwd moves per chunk and head with bf16 inputs and fp32 o.  *moved (may be NULL)
 * receives the bytes the launch moves.  The time of a launch is the floor of a prefill of that many chunks.
 */
kda_status kda_debug_prefill_traffic_probe(void *buffer, size_t bytes, size_t *moved, void *hip_stream);
kda_status kda_debug_mfma_probe(float *sink, int workgroups, int iters, double *flops, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* KDA_DEBUG_H_ */
