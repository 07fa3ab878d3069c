/*
 * attn_probe.h -- C ABI of the measurement-aid library (libattn_probe.so) that the benchmark loads
 * beside the attention library.  Nothing here is part of the attention path of include/attn.h.
 *
 * The metric of the paper's section 4.1 is the TFLOPS of the fused forward pass, reported here as a
 * fraction of the nominal dense BF16 peak (256 CU x 4 SIMD x 1024 FLOP/clk x 2.4 GHz).  That peak
 * assumes the 2.4 GHz clock; under load the board lowers the clock with the power drawn, which
 * depends on the operand data and on the work done beside the MFMAs.  The probe measures that.
 */
#ifndef PAPER_2603_24517_ATTN_PROBE_H
#define PAPER_2603_24517_ATTN_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ATTN_PROBE_OK       =  0,
    ATTN_PROBE_E_ARG    = -1,   /* NULL or misaligned pointer, or a value outside the ranges below */
    ATTN_PROBE_E_LAUNCH = -2    /* the HIP runtime refused the launch or the query                 */
};

/* bits of `mode`: work that accompanies every MFMA */
#define ATTN_PROBE_VALU 1   /* the vector instructions the attention kernel spends on one score per lane:
                               multiply-add, exponential, addition, and a pack to BF16 every other MFMA     */
#define ATTN_PROBE_LDS  2   /* the A operand of every MFMA is read from LDS (16 bytes per lane)             */
#define ATTN_PROBE_DMA  4   /* four 1 KiB global -> LDS requests per wavefront and 32 MFMAs, from `tiles`   */

#define ATTN_PROBE_BLOCKS 256   /* workgroups per launch: one per compute unit of an MI355X */

/*
 * attn_probe_mfma -- enqueue one launch of ATTN_PROBE_BLOCKS workgroups of 4 * waves_per_simd
 * wavefronts; every wavefront issues iters * 32 v_mfma_f32_32x32x16_bf16 (32768 FLOP each) on four
 * accumulators, so one launch performs
 *     ATTN_PROBE_BLOCKS * 4 * waves_per_simd * iters * 32 * 32768 FLOP.
 *   operands        in   device, BF16 [12, 64, 8], 16-byte aligned (8 A and 4 B operand sets per lane)
 *   tiles           in   device, 16-byte aligned, read only with ATTN_PROBE_DMA (else may be NULL)
 *   tiles_bytes          size of `tiles`: a power of two from 1 MiB to 2 GiB
 *   sink            out  device, 1 float (written only in a case that does not occur in practice)
 *   clocks          out  device, 4 x 64-bit, 8-byte aligned: shader cycle counter before and after the
 *                        loop, then the constant 100 MHz counter before and after it; "before" as read
 *                        by the first wavefront of the first workgroup, "after" by its last wavefront
 *                        (clock in GHz = 0.1 * d cycles / d ticks)
 *   mode                 OR of the ATTN_PROBE_* bits above (0 = MFMAs alone)
 *   waves_per_simd       1, 2 or 4
 *   iters                1 .. 2^20
 *   stream               a hipStream_t, or NULL
 * Enqueues only, allocates nothing; the caller owns every buffer.  Returns ATTN_PROBE_OK or a
 * negative code after host-side checks.
 */
int attn_probe_mfma(const void *operands, const void *tiles, size_t tiles_bytes, float *sink,
                    unsigned long long *clocks, int mode, int waves_per_simd, int iters, void *stream);

/*
 * attn_probe_device_info -- what the current device reports.
 *   compute_units  out  host, number of compute units
 *   clock_khz      out  host, peak shader clock in kHz
 */
int attn_probe_device_info(int *compute_units, int *clock_khz);

/*
 * attn_clocks_read -- exported only by the build of the ATTENTION library with -DATTN_CLOCKS
 * (paper_2603_24517_amd/variants/libattn_clocks.so: the shipped kernels plus these stamps), not by
 * libattn_probe.so.  Waits for the device, then copies the stamps that the first wavefront of the
 * first workgroup of the last attn_fwd launch took:
 *   out[0], out[1]  shader cycle counter at its start and at its end
 *   out[2], out[3]  the constant 100 MHz counter at its start and at its end
 *   out[4..6]       256-row kernel only, second work item of that workgroup: cycle counter where its
 *                   key-block loop starts (first two score products and first softmax done) and where
 *                   it ends (last barrier passed), and the number of iterations in between
 *   out[7..9]       the same for its third work item (stale or zero if the workgroup had fewer items)
 *   out  out  host, 10 x 64-bit
 * Returns 0, or a negative ATTN_E_* code of include/attn.h.
 */
int attn_clocks_read(unsigned long long *out);

/*
 * attn_phases_read -- exported only by the build of the attention library with -DATTN_CLOCKS=2
 * (paper_2603_24517_amd/variants/libattn_phases.so, which exports attn_clocks_read too).  Waits for
 * the device, then copies what two wavefronts of the first workgroup of the last attn_fwd launch
 * (256-row kernel) added up over that workgroup's SECOND work item: shader cycles per phase of the
 * item as that wavefront went through it.  One wavefront's latencies, not the workgroup's
 * throughput: the other wavefront of its SIMD fills many of the gaps.
 *   out[0..11]   first wavefront:  0 set-up (lookup of the next item, state reset, Q request; for an
 *                item whose tiles were not requested ahead also those requests and their wait),
 *                1 the first two score products, 2 the first softmax, 3 the barrier and the tile
 *                requests before the loop, 4 iterations this wavefront ran on the fast path (no
 *                mask, in-loop requests), 5 their number, 6 the other iterations except the last,
 *                7 their number, 8 the last iteration (PV only), 9 the wait for outstanding loads,
 *                10 the epilogue, 11 the whole item
 *   out[12..23]  the same for the last wavefront
 *   out  out  host, 24 x 64-bit (zero or stale if that workgroup had fewer than two items)
 * A stamp per iteration lengthens the loop by about 1.5 %.
 * Returns 0, or a negative ATTN_E_* code of include/attn.h.
 */
int attn_phases_read(unsigned long long *out);

#ifdef __cplusplus
}
#endif
#endif
