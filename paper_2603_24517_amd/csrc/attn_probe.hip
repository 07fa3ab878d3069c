// Measurement aids for the benchmark (a library of their own; the attention library exports none of
// this): what the matrix pipe of an MI355X sustains, and at which shader clock, for given operand data
// and for the kinds of work that accompany the MFMAs in the attention kernel.  The metric of the
// paper's section 4.1 (TFLOPS of the fused forward pass) is read against these figures.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/attn_probe.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define LDS_AS __attribute__((address_space(3)))

constexpr int OPERAND_BYTES = 12 * 64 * 16;     // 8 A and 4 B operand sets of 64 lanes x 8 BF16
constexpr int DMA_BYTES_PER_WAVE = 1024;        // LDS that one wavefront's tile requests land in (never read)
constexpr int MAX_WAVES = 16;

// One wavefront: iters x 32 MFMAs (v_mfma_f32_32x32x16_bf16) on four accumulators, the A operand taken
// from registers or, with LDS, read from LDS three MFMAs ahead of its use (16 bytes per lane and MFMA,
// what the attention kernel reads per MFMA).  VALU adds, per MFMA, the vector instructions the
// attention kernel spends on one score per lane: a multiply-add, an exponential, an addition and, every
// other MFMA, a pack to BF16.  DMA adds four 1 KiB global -> LDS requests per 32 MFMAs.
template <bool VALU, bool LDS, bool DMA>
__global__ void probe_kernel(const bf16x8 *operands, const unsigned char *tiles, uint32_t tiles_mask,
                             float *sink, unsigned long long *clocks, int iters)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[OPERAND_BYTES + MAX_WAVES * DMA_BYTES_PER_WAVE];
    LDS_AS unsigned char *lds = (LDS_AS unsigned char *)smem;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    bf16x8 a[4], b[4];      // (the first four of the eight A sets: 128 registers per wavefront must do at 4 per SIMD)
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = operands[i * 64 + lane];
#pragma unroll
    for (int i = 0; i < 4; ++i) b[i] = operands[(8 + i) * 64 + lane];
    if (LDS) {
        for (int i = threadIdx.x; i < OPERAND_BYTES / 16; i += blockDim.x)
            *(LDS_AS u32x4 *)(lds + 16 * i) = ((const u32x4 *)operands)[i];
    }
    f32x16 c[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[n][r] = 0.0f;
    float y[8], x[4], e[2], sum = 0.0f, pk = 0.0f;    // y: lane-varying "scores" (operand values widened to FP32)
#pragma unroll
    for (int i = 0; i < 8; ++i) y[i] = (float)a[i & 3][(lane + i) & 7];
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = 0.0f;
    e[0] = e[1] = 0.0f;
    // every wavefront walks its own 1 KiB pieces of `tiles`
    uint32_t goff = ((uint32_t)(blockIdx.x * (blockDim.x >> 6) + wave) * 4096u) & tiles_mask;
    const uint32_t dma_lds = (uint32_t)(uintptr_t)lds + OPERAND_BYTES + wave * DMA_BYTES_PER_WAVE;
    __syncthreads();
    const unsigned long long r0 = wall_clock64();
    const unsigned long long t0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) {
        bf16x8 frag[32];
        if (LDS) {
#pragma unroll
            for (int s = 0; s < 3; ++s) frag[s] = *(const LDS_AS bf16x8 *)(lds + ((s & 7) * 64 + lane) * 16);
        }
#pragma unroll
        for (int s = 0; s < 32; ++s) {
            if (LDS && s + 3 < 32) frag[s + 3] = *(const LDS_AS bf16x8 *)(lds + (((s + 3) & 7) * 64 + lane) * 16);
            c[s & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(LDS ? frag[s] : a[(s >> 2) & 3], b[s & 3], c[s & 3], 0, 0, 0);
            if (VALU) {
                asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(x[s & 3]) : "v"(y[s & 7]), "v"(0.1275f), "v"(-0.25f));
                asm volatile("v_exp_f32 %0, %1" : "=v"(e[s & 1]) : "v"(x[s & 3]));
                asm volatile("v_add_f32 %0, %0, %1" : "+v"(sum) : "v"(e[s & 1]));
                if (s & 1) asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(pk) : "v"(e[0]), "v"(e[1]));
            }
            if (DMA && (s & 7) == 4) {
                const uint32_t vo = goff + 16u * lane;
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                             :
                             : "s"(dma_lds), "v"(vo), "s"(tiles)
                             : "memory");
                goff = (goff + 1024u) & tiles_mask;
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (DMA) __builtin_amdgcn_s_waitcnt(0x0F70 | 4);      // vmcnt(4): all but this iteration's requests have landed
    }
    if (DMA) __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0): nothing writes LDS after the kernel ends
    const unsigned long long t1 = __builtin_readcyclecounter();
    const unsigned long long r1 = wall_clock64();
    // the oldest wavefront of a SIMD is served first and ends first: start of the first wavefront, end of the last
    if (blockIdx.x == 0 && threadIdx.x == 0) { clocks[0] = t0; clocks[2] = r0; }
    if (blockIdx.x == 0 && threadIdx.x == blockDim.x - 64) { clocks[1] = t1; clocks[3] = r1; }
    float s = 0.0f;
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += c[n][r];
    s += sum + pk + x[0] + x[1] + x[2] + x[3];
    if (s == 123.456f) sink[0] = s;     // keeps the loop alive; practically never true
}

template <bool VALU, bool LDS, bool DMA>
void launch(int threads, hipStream_t st, const void *operands, const void *tiles, uint32_t mask, float *sink,
            unsigned long long *clocks, int iters)
{
    hipLaunchKernelGGL((probe_kernel<VALU, LDS, DMA>), dim3(ATTN_PROBE_BLOCKS), dim3(threads), 0, st,
                       (const bf16x8 *)operands, (const unsigned char *)tiles, mask, sink, clocks, iters);
}

}  // namespace

extern "C" {

int attn_probe_mfma(const void *operands, const void *tiles, size_t tiles_bytes, float *sink,
                    unsigned long long *clocks, int mode, int waves_per_simd, int iters, void *stream)
{
    if (!operands || !sink || !clocks) return ATTN_PROBE_E_ARG;
    if (((uintptr_t)operands & 15) || ((uintptr_t)clocks & 7)) return ATTN_PROBE_E_ARG;
    if (iters <= 0 || iters > (1 << 20)) return ATTN_PROBE_E_ARG;
    if (waves_per_simd != 1 && waves_per_simd != 2 && waves_per_simd != 4) return ATTN_PROBE_E_ARG;
    if (mode < 0 || mode > 7) return ATTN_PROBE_E_ARG;
    uint32_t mask = 0;
    if (mode & ATTN_PROBE_DMA) {
        // a power of two between 1 MiB and 2 GiB, so that offsets wrap with a mask and stay in bounds
        if (!tiles || ((uintptr_t)tiles & 15)) return ATTN_PROBE_E_ARG;
        if (tiles_bytes < (1u << 20) || tiles_bytes > (1u << 31) || (tiles_bytes & (tiles_bytes - 1))) return ATTN_PROBE_E_ARG;
        mask = (uint32_t)(tiles_bytes - 1) & ~1023u;
    }
    const int threads = 256 * waves_per_simd;
    hipStream_t st = (hipStream_t)stream;
    switch (mode) {
    case 0: launch<false, false, false>(threads, st, operands, tiles, mask, sink, clocks, iters); break;
    case 1: launch<true, false, false>(threads, st, operands, tiles, mask, sink, clocks, iters); break;
    case 2: launch<false, true, false>(threads, st, operands, tiles, mask, sink, clocks, iters); break;
    case 3: launch<true, true, false>(threads, st, operands, tiles, mask, sink, clocks, iters); break;
    case 4: launch<false, false, true>(threads, st, operands, tiles, mask, sink, clocks, iters); break;
    case 5: launch<true, false, true>(threads, st, operands, tiles, mask, sink, clocks, iters); break;
    case 6: launch<false, true, true>(threads, st, operands, tiles, mask, sink, clocks, iters); break;
    default: launch<true, true, true>(threads, st, operands, tiles, mask, sink, clocks, iters); break;
    }
    return hipGetLastError() == hipSuccess ? ATTN_PROBE_OK : ATTN_PROBE_E_LAUNCH;
}

int attn_probe_device_info(int *compute_units, int *clock_khz)
{
    if (!compute_units || !clock_khz) return ATTN_PROBE_E_ARG;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(compute_units, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipDeviceGetAttribute(clock_khz, hipDeviceAttributeClockRate, dev) != hipSuccess)
        return ATTN_PROBE_E_LAUNCH;
    return ATTN_PROBE_OK;
}

}  // extern "C"
