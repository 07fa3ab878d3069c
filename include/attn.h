/*
 * attn.h -- C ABI of the MI355X (gfx950) fused attention forward library.
 *
 * The operation is the one the paper states in section 2.2 ("Attention
 * computation"): O = softmax(Q K^T * scale) V per head, computed tile by tile
 * over key blocks with a running row maximum and row sum, so that the
 * Sq x Skv score matrix is never stored.  Causal masking and grouped-query
 * heads follow the benchmark configurations of sections 4.1 and 4.3.
 *
 * All pointers are DEVICE pointers owned by the caller.  The library holds no
 * device memory, allocates nothing, never synchronises and never throws.
 */
#ifndef PAPER_2603_24517_ATTN_H
#define PAPER_2603_24517_ATTN_H

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ATTN_OK            =  0,
    ATTN_E_NULL        = -1,  /* a required pointer is NULL                                    */
    ATTN_E_SHAPE       = -2,  /* a dimension is <= 0, or Hq is not a multiple of Hkv           */
    ATTN_E_UNSUPPORTED = -3,  /* D != 128, or a tensor too large for the kernel's index math   */
    ATTN_E_ALIGN       = -4,  /* q, k, v or o not 16-byte aligned, or lse not 4-byte aligned   */
    ATTN_E_SCALE       = -5,  /* scale is NaN or infinite                                      */
    ATTN_E_LAUNCH      = -6   /* the HIP runtime refused the launch                            */
};

/*
 * attn_fwd -- fused attention forward (section 2.2; masks and head grouping
 * of sections 4.1 and 4.3).
 *
 * For every batch b, query head h and query row i, with g = h / (Hq / Hkv):
 *     s_j        = scale * sum_d Q[b,i,h,d] * K[b,j,g,d]
 *     valid(j)   = !causal  ||  j <= i + (Skv - Sq)        (bottom-right aligned)
 *     O[b,i,h,:] = sum_{valid j} softmax_j(s) * V[b,j,g,:]
 *     LSE[b,h,i] = ln sum_{valid j} exp(s_j)               (natural log)
 *     a row with no valid key gives O = 0 and LSE = -inf.
 * Products run on BF16 matrix cores with FP32 accumulation; the running
 * maximum, the running sum and LSE are FP32; softmax weights are rounded to
 * BF16 (nearest even) before they multiply V; O is rounded to BF16 once.
 *
 *   q    in   BF16 [B, Sq,  Hq,  D] contiguous
 *   k    in   BF16 [B, Skv, Hkv, D] contiguous
 *   v    in   BF16 [B, Skv, Hkv, D] contiguous
 *   o    out  BF16 [B, Sq,  Hq,  D] contiguous, fully overwritten
 *   lse  out  FP32 [B, Hq, Sq]      contiguous, fully overwritten
 *   B, Hq, Hkv, Sq, Skv  > 0, Hq % Hkv == 0;  D must be 128
 *   causal  0 = no mask, otherwise lower-triangular mask as above
 *   scale   any finite value (the caller passes 1/sqrt(D))
 *   stream  a hipStream_t, or NULL for the default stream
 *
 * Size limits (ATTN_E_UNSUPPORTED beyond them): Sq + Skv below 2^31 - 1024,
 * Hq and Hkv at most 32768, and fewer than 2^27 work items, one item being 256/p query rows of p query
 * heads that share a K/V head (p = 8, 4, 2 or 1, the largest that divides
 * Hq / Hkv).  The launch is one kernel: with one workgroup per compute unit of
 * the current device (all of its LDS), each working through a list of such
 * items -- or, when those items would occupy at most a quarter of the compute
 * units (few query rows, however long the key sequence), with one workgroup per
 * 32 query rows that share a K/V head (p heads x 32/p positions), whose
 * wavefronts share the item's keys and merge their partial results through LDS.  Either way nothing is allocated.
 * The first call on a device queries the device once and sets function
 * attributes, so make one ordinary call on a device before recording attn_fwd
 * into a HIP graph (later calls are one kernel launch and nothing else, and
 * replay correctly).
 *
 * Inputs and outputs must not overlap and must stay alive until the stream
 * reaches the end of the kernel.  The call only enqueues work.  Every
 * argument is checked on the host before the device is touched; the return
 * value is ATTN_OK or one of the negative codes above.
 */
int attn_fwd(const void *q, const void *k, const void *v, void *o, float *lse,
             int B, int Hq, int Hkv, int Sq, int Skv, int D,
             int causal, float scale, void *stream);

/* Static text for a return code of this library (never NULL). */
const char *attn_strerror(int code);

/* ABI version: major * 1000 + minor. */
int attn_version(void);

#ifdef __cplusplus
}
#endif
#endif
