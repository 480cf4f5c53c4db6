/*
 * axconv_probe -- measurement helpers of libaxconv (gfx950).  Not part of the layer path:
 * unlike the entry points of axconv.h these create HIP events, may allocate temporary device
 * memory and wait for the stream.  They measure the denominators the layer's throughput is
 * compared with (LDS gather rates, instruction mix, copy bandwidth) and the duration of a
 * layer's main kernel.
 */
#ifndef AXCONV_PROBE_H
#define AXCONV_PROBE_H

#include "axconv.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * LDS gather micro-benchmark: one workgroup per compute unit keeps a table of
 * `table_bytes` in LDS and every lane repeatedly reads `width_bytes` (2, 4, 8 or 16)
 * from it.  pattern 0: lane l reads consecutive elements (no bank conflict);
 * pattern 1: every lane reads independent uniformly random aligned elements;
 * pattern 2: like 1, but half of the lanes (chosen at random) read element 0;
 * patterns 3..6 (16-byte reads only): sixteen tables interleaved entry by entry, element
 * index = 16 * v + slot with v uniformly random and the slot a function of the lane alone --
 * 3: lane % 16, 4: (lane / 4) % 16, 5: lane % 8 + 8 * ((lane / 32) % 2),
 * 6: lane % 4 + 4 * ((lane / 16) % 4) -- which shows which lanes the LDS serves together.
 * Outputs (host pointers): wave_reads = wave-level read instructions executed per workgroup,
 * cycles = mean shader-clock cycles per workgroup, seconds = elapsed time of the kernel,
 * workgroups = grid size.
 */
int ax_probe_lds_gather(int width_bytes, int pattern, int table_bytes, int threads, int iters,
                        double* wave_reads, double* cycles, double* seconds, int* workgroups,
                        void* hip_stream);

/*
 * Instruction-mix micro-benchmark.  mode 0: independent integer adds only (ops = lane adds);
 * modes 1..4: the inner loop of the table-tile kernels without table building or barriers,
 * for (threads, lane elements per thread, table groups) = (512,2,8), (1024,1,8), (512,4,4),
 * (1024,2,4) (ops = lookup-MACs).  pattern 1: uniform random codes, 2: half of the codes zero.
 * Outputs are host pointers.
 */
int ax_probe_mac(int mode, int pattern, int iters, int wgs_per_cu, double* ops, double* seconds,
                 void* hip_stream);

/* Plain device-to-device copy kernel of `bytes` (multiple of 16), for the HBM roofline and
 * for calibrating memory-traffic counters.  Asynchronous, allocates nothing. */
int ax_probe_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

/*
 * Duration of the main kernel of a prepared layer: enqueues the per-call operand preparation,
 * records an event, launches the main kernel `reps` (1..64) times back to back (the repeats
 * rewrite the same results and only dilute the events' own cost), records a second event,
 * enqueues the combination pass where the layer has one, waits for the stream and returns the
 * time between the events divided by reps in *ms.  Arguments as for ax_layer_run; the outputs
 * hold the layer's results afterwards.
 */
int ax_probe_layer_kernel_ms(const ax_layer_t* layer, const void* x, int32_t* acc_out,
                             float* y_out, void* workspace, size_t workspace_bytes, int reps,
                             float* ms, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* AXCONV_PROBE_H */
