// Fused attention forward for MI355X (gfx950, CDNA4).
//
// Computes O = softmax(Q K^T * scale [+ causal mask]) V and the per-row
// log-sum-exp, tile by tile over key blocks with a running row maximum and
// running row sum (paper section 2.2), for multi-head and grouped-query
// attention (sections 4.1, 4.3).  BF16 operands on MFMA, FP32 accumulation.
//
// Data flow of one wavefront (64 lanes), which owns 32 query rows of one head:
//   * S^T = K Q^T with v_mfma_f32_32x32x16_bf16: A = 32 keys x 16 d read from
//     LDS, B = Q^T held in registers for the whole kernel.  The accumulator
//     layout puts ONE query (lane % 32) in each lane and 16 of the tile's 32
//     keys in its registers, so a row maximum / row sum is 15 in-lane
//     operations plus one exchange between lanes l and l^32.
//   * P is rounded to BF16 in registers and is directly the B operand of
//     O^T = V^T P^T: the contraction slots of each P^T operand are the keys
//     the lane already holds, and V^T is fetched from LDS with the matching
//     key order by the transposing read ds_read_b64_tr_b16.  No LDS round
//     trip and no shuffle for P.
//   * O^T keeps lane = query, so the rescale by alpha and the final 1/l are
//     lane-local multiplies.
// A workgroup is 8 wavefronts (256 query rows) sharing one K/V block stream
// through double-buffered LDS.  For grouped-query attention the 256 rows are
// PACK heads of one K/V group x 256/PACK positions, so that one K/V tile in
// LDS serves several query heads.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>

#include "../../include/attn.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int HD = 128;              // head dimension
constexpr int BN = 64;               // keys per K/V block
constexpr int NWAVES = 8;            // wavefronts per workgroup
constexpr int NTHREADS = NWAVES * 64;
constexpr int WG_ROWS = NWAVES * 32; // query rows per workgroup
constexpr int ROW_BYTES = HD * 2;    // one (token, head) row of BF16
constexpr int TILE_BYTES = BN * ROW_BYTES;
constexpr int LDS_BYTES = 4 * TILE_BYTES;   // K and V, two stages each
// The running maximum is only raised when a row's block maximum exceeds it by
// more than this many powers of two; until then probabilities are formed
// against the stale maximum (any reference point gives the same softmax) and
// stay below 2^RESCALE_SLACK.
constexpr float RESCALE_SLACK = 8.0f;

struct Params {
    const __bf16 *q, *k, *v;
    __bf16 *o;
    float *lse;
    int B, Hq, Hkv, Sq, Skv;
    int G;          // Hq / Hkv
    int pack;       // query heads of one K/V group served by one workgroup (1, 2, 4 or 8)
    int tile_pos;   // query positions per workgroup = 256 / pack
    int ntile;      // ceil(Sq / tile_pos)
    int chunks;     // G / pack
    int total;      // work items = B * Hkv * chunks * ntile
    int per_xcd;    // ceil(total / 8)
    float c;        // scale * log2(e)
};

// 16-byte units of a K row are XOR-swizzled with the row so that 16 lanes
// reading the same d-range of 16 consecutive rows hit 16 different units.
__device__ __forceinline__ int k_lds_off(int row, int unit) {
    return row * ROW_BYTES + ((unit ^ (row & 15)) << 4);
}
// V rows are read four at a time (transposing read, 64 bytes of each row per
// half-wave): rotate the 64-byte groups with the row.
__device__ __forceinline__ int v_lds_off(int row, int unit) {
    return row * ROW_BYTES + ((unit ^ ((row & 3) << 2)) << 4);
}

__device__ __forceinline__ float lane32_max(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float lane32_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    bf16x2 p = __builtin_convertvector((f32x2){a, b}, bf16x2);   // v_cvt_pk_bf16_f32, nearest even
    return __builtin_bit_cast(uint32_t, p);
}

template <bool CAUSAL>
__global__ __launch_bounds__(NTHREADS) void attn_fwd_kernel(const Params p)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    // ---- work item: workgroups are dealt round-robin to the 8 XCDs, so give
    // each XCD a contiguous range of items (neighbouring items share K/V in
    // that XCD's L2).
    const int bid = blockIdx.x;
    const int item = (bid & 7) * p.per_xcd + (bid >> 3);
    if (item >= p.total) return;
    int rem = item;
    const int tile_r = rem % p.ntile;  rem /= p.ntile;
    const int chunk = rem % p.chunks;  rem /= p.chunks;
    const int hkv = rem % p.Hkv;
    const int b = rem / p.Hkv;
    // heavy (late) query tiles first when causal
    const int tile = CAUSAL ? (p.ntile - 1 - tile_r) : tile_r;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l32 = lane & 31;
    const int hh = lane >> 5;

    const int head = hkv * p.G + chunk * p.pack + (wave % p.pack);
    const int q0 = tile * p.tile_pos + (wave / p.pack) * 32;   // first query row of this wave
    const int off = p.Skv - p.Sq;                               // causal: key j valid iff j <= i + off

    // ---- number of key blocks the workgroup walks
    int nblk = (p.Skv + BN - 1) / BN;
    if (CAUSAL) {
        int qlast = min(tile * p.tile_pos + p.tile_pos, p.Sq) - 1;
        int klast = qlast + off;
        nblk = klast < 0 ? 0 : min(nblk, klast / BN + 1);
    }

    // ---- Q fragments: lane holds query (q0 + l32), d = 16*s + 8*hh .. +7
    bf16x8 qf[8];
    {
        const int qrow = min(q0 + l32, p.Sq - 1);
        const __bf16 *qp = p.q + ((size_t)((size_t)b * p.Sq + qrow) * p.Hq + head) * HD + 8 * hh;
#pragma unroll
        for (int s = 0; s < 8; ++s) qf[s] = *(const bf16x8 *)(qp + 16 * s);
    }

    float m = -INFINITY;   // running maximum, in log2 units (scores times scale*log2 e)
    float l = 0.0f;        // this lane's share of the running sum (its 16 of every 32 keys)
    f32x16 acc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[dt][r] = 0.0f;

    // ---- cooperative K/V tile loads: thread -> rows (tid/16, tid/16 + 32), 16-byte unit tid%16
    const int ld_row = tid >> 4, ld_unit = tid & 15;
    const size_t kv_row_stride = (size_t)p.Hkv * HD;             // elements between consecutive keys
    const __bf16 *kbase = p.k + ((size_t)b * p.Skv * p.Hkv + hkv) * HD + ld_unit * 8;
    const __bf16 *vbase = p.v + ((size_t)b * p.Skv * p.Hkv + hkv) * HD + ld_unit * 8;
    u32x4 kreg[2], vreg[2];
    auto load_tile = [&](int j) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int row = min(j * BN + ld_row + 32 * i, p.Skv - 1);   // rows past the end are masked later
            kreg[i] = *(const u32x4 *)(kbase + row * kv_row_stride);
            vreg[i] = *(const u32x4 *)(vbase + row * kv_row_stride);
        }
    };
    auto store_tile = [&](int stage) {
        unsigned char *kb = smem + stage * 2 * TILE_BYTES;
        unsigned char *vb = kb + TILE_BYTES;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            *(u32x4 *)(kb + k_lds_off(ld_row + 32 * i, ld_unit)) = kreg[i];
            *(u32x4 *)(vb + v_lds_off(ld_row + 32 * i, ld_unit)) = vreg[i];
        }
    };

    if (nblk > 0) { load_tile(0); store_tile(0); }

    // per-lane constants of the transposing V read: lane (i = lane%16, g = (lane%32)/16, hh)
    // supplies the address of row 4*hh + i/4, d = 16*g + 4*(i%4) of a 16-key x 32-d block.
    const int tr_row = 4 * hh + ((lane & 15) >> 2);
    const int tr_d = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

    for (int j = 0; j < nblk; ++j) {
        __syncthreads();
        const bool more = (j + 1 < nblk);
        if (more) load_tile(j + 1);

        const unsigned char *kb = smem + (j & 1) * 2 * TILE_BYTES;
        const unsigned char *vb = kb + TILE_BYTES;
        const int j0 = j * BN;

        // which path does this wave take for this block?
        bool skip = false, masked = (j0 + BN > p.Skv);
        if (CAUSAL) {
            skip = (j0 > q0 + 31 + off);
            masked = masked || (j0 + BN - 1 > q0 + off);
        }

        if (!skip) {
            // ---- S^T = K Q^T : two 32-key tiles
            f32x16 s[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[t][r] = 0.0f;
#pragma unroll
                for (int st = 0; st < 8; ++st) {
                    bf16x8 a = *(const bf16x8 *)(kb + k_lds_off(32 * t + l32, 2 * st + hh));
                    s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[st], s[t], 0, 0, 0);
                }
            }

            // ---- online softmax
            uint32_t pb[2][8];   // P^T operands, BF16 pairs
            if (!masked) {
                float mx = s[0][0];
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[t][r]);
                mx = lane32_max(mx) * p.c;
                if (__builtin_amdgcn_ballot_w64(mx > m + RESCALE_SLACK) != 0) {
                    const float mn = fmaxf(m, mx);
                    const float alpha = __builtin_amdgcn_exp2f(m - mn);
                    m = mn;
                    l *= alpha;
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[dt][r] *= alpha;
                }
                float ls = 0.0f;
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int r = 0; r < 16; r += 2) {
                        float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][r], p.c, -m));
                        float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][r + 1], p.c, -m));
                        ls += e0 + e1;
                        pb[t][r >> 1] = pack_bf16(e0, e1);
                    }
                l += ls;
            } else {
                // diagonal or tail block: key index per register, limit per lane
                int lim = p.Skv - 1;
                if (CAUSAL) lim = min(lim, q0 + l32 + off);
                const int kbase_idx = j0 + 4 * hh;
                float mx = -INFINITY;
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = kbase_idx + 32 * t + 8 * (r >> 2) + (r & 3);
                        mx = fmaxf(mx, key <= lim ? s[t][r] : -INFINITY);
                    }
                mx = lane32_max(mx);
                mx = (mx == -INFINITY) ? -INFINITY : mx * p.c;
                if (__builtin_amdgcn_ballot_w64(mx > m + RESCALE_SLACK) != 0) {
                    const float mn = fmaxf(m, mx);
                    const float alpha = (mn == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m - mn);
                    m = mn;
                    l *= alpha;
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[dt][r] *= alpha;
                }
                const float mu = (m == -INFINITY) ? 0.0f : m;
                float ls = 0.0f;
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int r = 0; r < 16; r += 2) {
                        const int key = kbase_idx + 32 * t + 8 * (r >> 2) + (r & 3);
                        float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][r], p.c, -mu));
                        float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][r + 1], p.c, -mu));
                        e0 = (key <= lim) ? e0 : 0.0f;
                        e1 = (key + 1 <= lim) ? e1 : 0.0f;
                        ls += e0 + e1;
                        pb[t][r >> 1] = pack_bf16(e0, e1);
                    }
                l += ls;
            }

            // ---- O^T += V^T P^T : 4 groups of 16 keys x 4 tiles of 32 d
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    u32x4 pw = {pb[t][4 * u], pb[t][4 * u + 1], pb[t][4 * u + 2], pb[t][4 * u + 3]};
                    bf16x8 pv = __builtin_bit_cast(bf16x8, pw);
                    const int krow = 32 * t + 16 * u + tr_row;
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt) {
                        const int d = 32 * dt + tr_d;                // first of 4 d for this lane's address
                        const int unit = d >> 3, sub = (d & 7) * 2;
                        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (__attribute__((address_space(3))) s16x4 *)(vb + v_lds_off(krow, unit) + sub));
                        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (__attribute__((address_space(3))) s16x4 *)(vb + v_lds_off(krow + 8, unit) + sub));
                        s16x8 av = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                        acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, av), pv, acc[dt], 0, 0, 0);
                    }
                }
        }

        if (more) store_tile((j + 1) & 1);
    }

    // ---- epilogue: O = acc / l (BF16), LSE = ln2 * (m + log2 l)
    const float lt = lane32_sum(l);
    const float inv = lt > 0.0f ? 1.0f / lt : 0.0f;
    const int qrow = q0 + l32;
    if (qrow < p.Sq) {
        __bf16 *op = p.o + ((size_t)((size_t)b * p.Sq + qrow) * p.Hq + head) * HD + 4 * hh;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                u32x2 w = {pack_bf16(acc[dt][4 * rg] * inv, acc[dt][4 * rg + 1] * inv),
                           pack_bf16(acc[dt][4 * rg + 2] * inv, acc[dt][4 * rg + 3] * inv)};
                *(u32x2 *)(op + 32 * dt + 8 * rg) = w;
            }
        if (hh == 0) {
            const float lse = lt > 0.0f ? (m + __builtin_amdgcn_logf(lt)) * 0.6931471805599453f : -INFINITY;
            p.lse[((size_t)b * p.Hq + head) * p.Sq + qrow] = lse;
        }
    }
}

}  // namespace

extern "C" {

int attn_fwd(const void *q, const void *k, const void *v, void *o, float *lse,
             int B, int Hq, int Hkv, int Sq, int Skv, int D,
             int causal, float scale, void *stream)
{
    if (!q || !k || !v || !o || !lse) return ATTN_E_NULL;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Sq <= 0 || Skv <= 0 || D <= 0) return ATTN_E_SHAPE;
    if (Hq % Hkv != 0) return ATTN_E_SHAPE;
    if (D != HD) return ATTN_E_UNSUPPORTED;
    if (!(scale >= 0.0f) || isinf(scale)) return ATTN_E_SCALE;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15) return ATTN_E_ALIGN;
    if ((uintptr_t)lse & 3) return ATTN_E_ALIGN;

    Params p;
    p.q = (const __bf16 *)q; p.k = (const __bf16 *)k; p.v = (const __bf16 *)v;
    p.o = (__bf16 *)o; p.lse = lse;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.Sq = Sq; p.Skv = Skv;
    p.G = Hq / Hkv;
    p.pack = (p.G % 8 == 0) ? 8 : (p.G % 4 == 0) ? 4 : (p.G % 2 == 0) ? 2 : 1;
    p.tile_pos = WG_ROWS / p.pack;
    p.ntile = (Sq + p.tile_pos - 1) / p.tile_pos;
    p.chunks = p.G / p.pack;
    // Key/query indices and the work-item count are 32-bit in the kernel.
    if ((int64_t)Sq + Skv + WG_ROWS + BN >= INT32_MAX) return ATTN_E_UNSUPPORTED;
    const int64_t total = (int64_t)B * Hkv * p.chunks * p.ntile;
    if (total + 8 >= INT32_MAX) return ATTN_E_UNSUPPORTED;
    p.total = (int)total;
    p.per_xcd = (int)((total + 7) / 8);
    p.c = scale * 1.4426950408889634f;

    const dim3 grid((unsigned)(p.per_xcd * 8)), block(NTHREADS);
    hipStream_t st = (hipStream_t)stream;
    if (causal)
        hipLaunchKernelGGL(attn_fwd_kernel<true>, grid, block, LDS_BYTES, st, p);
    else
        hipLaunchKernelGGL(attn_fwd_kernel<false>, grid, block, LDS_BYTES, st, p);
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_E_LAUNCH;
}

const char *attn_strerror(int code)
{
    switch (code) {
    case ATTN_OK:            return "success";
    case ATTN_E_NULL:        return "null pointer argument";
    case ATTN_E_SHAPE:       return "bad shape: every dimension must be positive and Hq a multiple of Hkv";
    case ATTN_E_UNSUPPORTED: return "unsupported: head dimension must be 128 and sizes must fit 32-bit indices";
    case ATTN_E_ALIGN:       return "misaligned pointer: q, k, v, o need 16-byte and lse 4-byte alignment";
    case ATTN_E_SCALE:       return "scale must be finite and non-negative";
    case ATTN_E_LAUNCH:      return "kernel launch failed";
    default:                 return "unknown attn error code";
    }
}

int attn_version(void) { return 1000; }

}  // extern "C"
