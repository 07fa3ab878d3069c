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
//
// A workgroup is 8 wavefronts (256 query rows) sharing one K/V block stream:
// tiles go from global memory straight into double-buffered, XOR-swizzled LDS
// (global_load_lds_dwordx4).  For grouped-query attention the 256 rows are
// PACK heads of one K/V group x 256/PACK positions, so one K/V tile in LDS
// serves several query heads.
//
// The two wavefronts that share a SIMD run half an iteration apart: while one
// issues the 32 MFMAs of "S(j+1) = K(j+1) Q^T ; O += V(j)^T P(j)^T" the other
// runs the softmax VALU work of its own block, and a workgroup barrier ends
// each half.  This keeps the matrix pipe and the vector ALU busy at the same
// time (the paper's section 2.2 describes the same need, met on its hardware
// by specialised warps).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>

#include "../../include/attn.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define LDS_AS __attribute__((address_space(3)))
#define GLB_AS __attribute__((address_space(1)))

constexpr int HD = 128;              // head dimension
constexpr int BN = 64;               // keys per K/V block
constexpr int NWAVES = 8;            // wavefronts per workgroup
constexpr int NTHREADS = NWAVES * 64;
constexpr int WG_ROWS = NWAVES * 32; // query rows per workgroup
constexpr int ROW_BYTES = HD * 2;    // one (token, head) row of BF16
constexpr int TILE_BYTES = BN * ROW_BYTES;
constexpr int NSTAGE = 3;                   // K/V tiles in flight: requested two iterations ahead
constexpr int V_BASE = NSTAGE * TILE_BYTES; // K stages first, V stages after them
constexpr int LDS_BYTES = 2 * NSTAGE * TILE_BYTES;
// The running maximum is only raised when a row's block maximum exceeds it by
// more than this many powers of two; until then probabilities are formed
// against the stale maximum (any reference point gives the same softmax) and
// stay below 2^RESCALE_SLACK.
constexpr float RESCALE_SLACK = 8.0f;
// Largest partial row sum (16 probabilities of one lane) the fast softmax path accepts: probabilities
// stay below 2^14 relative to the reference maximum, far inside BF16 / FP32 range.
constexpr float P_SUM_LIMIT = 16384.0f;
#ifndef MAT_PREFETCH
#define MAT_PREFETCH 4
#endif
constexpr int WAIT_VMCNT0 = 0x0F70;  // s_waitcnt vmcnt(0), other counters untouched
constexpr int WAIT_VMCNT4 = 0x0F74;  // s_waitcnt vmcnt(4): all but the 4 most recent loads have landed

__device__ __forceinline__ void phase_barrier() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
}

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
// 16 bytes per lane from global memory straight into LDS: lane L's data lands at lds_base + 16*L.
// Issued as inline assembly so that the compiler's counter bookkeeping does not make every later
// LDS read wait for it; the caller waits with s_waitcnt vmcnt(0) before the barrier that publishes
// the tile.
__device__ __forceinline__ void lds_dma16(const unsigned char *base, uint32_t voffset, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base), "v"(voffset), "s"(base)
                 : "memory");
}
__device__ __forceinline__ float max3(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
// Order of the matrix half: LDS reads run PREFETCH MFMAs ahead of the MFMA that consumes them.
// (A PV MFMA takes two transposing 8-byte reads, a QK MFMA one 16-byte read.)
template <int SLOT>
__device__ __forceinline__ void schedule_matrix_slot() {
    constexpr int MFMA = 0x008, DS_READ = 0x100, NEXT = SLOT + MAT_PREFETCH;
    __builtin_amdgcn_sched_group_barrier(MFMA, 1, 0);
    // even slots (PV) take two transposing 8-byte reads, odd slots (QK) one 16-byte read
    if constexpr (NEXT < 32 && (NEXT & 1) == 0) __builtin_amdgcn_sched_group_barrier(DS_READ, 2, 0);
    if constexpr (NEXT < 32 && (NEXT & 1) == 1) __builtin_amdgcn_sched_group_barrier(DS_READ, 1, 0);
    if constexpr (SLOT + 1 < 32) schedule_matrix_slot<SLOT + 1>();
}
__device__ __forceinline__ void schedule_matrix_half() {
    constexpr int DS_READ = 0x100;
    __builtin_amdgcn_sched_group_barrier(DS_READ, (MAT_PREFETCH / 2) * 3 + (MAT_PREFETCH & 1) * 2, 0);
    schedule_matrix_slot<0>();
}
// Experiment switches (product build: one barrier per iteration, no priority change).
#ifdef ATTN_TWO_BARRIERS
#define MID_BARRIER() PHASE_BARRIER()
#else
#define MID_BARRIER() __builtin_amdgcn_sched_barrier(0)
#endif
#ifdef ATTN_MAT_PRIO
#define MAT_PRIO(x) __builtin_amdgcn_s_setprio((x) ? ATTN_MAT_PRIO : 0)
#else
#define MAT_PRIO(x) do { } while (0)
#endif

#ifdef ATTN_TRACE
// Debug build only: per-wavefront clock stamps around every phase barrier of one workgroup.
__device__ unsigned long long g_trace[NWAVES][1024];
__device__ __forceinline__ void trace_mark(int &n) {
    if (blockIdx.x == ATTN_TRACE && n < 1024) {
        const unsigned long long t = __builtin_readcyclecounter();
        if ((threadIdx.x & 63) == 0) g_trace[threadIdx.x >> 6][n] = t;
        ++n;
    }
}
#define TRACE_ALWAYS() do { __builtin_amdgcn_sched_barrier(0); trace_mark(trace_n); __builtin_amdgcn_sched_barrier(0); } while (0)
#ifdef ATTN_TRACE_LIGHT
#define PHASE_BARRIER() phase_barrier()
#define TRACE_POINT() do { } while (0)
#else
#define PHASE_BARRIER() do { __builtin_amdgcn_sched_barrier(0); trace_mark(trace_n); __builtin_amdgcn_sched_barrier(0); \
        phase_barrier(); trace_mark(trace_n); __builtin_amdgcn_sched_barrier(0); } while (0)
#define TRACE_POINT() TRACE_ALWAYS()
#endif
#else
#define PHASE_BARRIER() phase_barrier()
#define TRACE_POINT() do { } while (0)
#define TRACE_ALWAYS() do { } while (0)
#endif

// Everything one wavefront keeps across the key-block loop.
struct WaveState {
    bf16x8 qf[8];        // Q^T operand: query lane%32, d = 16*s + 8*(lane/32) .. +7
    f32x16 s[2];         // S^T of the block in flight: two 32-key tiles
    uint32_t pb[2][8];   // P^T of the previous block, BF16 pairs (the PV operand)
    f32x16 acc[4];       // O^T accumulator: four 32-d tiles
    float m;             // running maximum in log2 units (score * scale * log2 e)
    float l;             // this lane's share of the running sum
};

template <bool CAUSAL>
__global__ __launch_bounds__(NTHREADS) void attn_fwd_kernel(const Params p)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    LDS_AS unsigned char *lds = (LDS_AS unsigned char *)smem;

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
    const int tile = CAUSAL ? (p.ntile - 1 - tile_r) : tile_r;   // heavy (late) query tiles first

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31;
    const int hh = lane >> 5;

    const int head = hkv * p.G + chunk * p.pack + (wave % p.pack);
    const int q0 = tile * p.tile_pos + (wave / p.pack) * 32;   // first query row of this wave
    const int off = p.Skv - p.Sq;                               // causal: key j valid iff j <= i + off

    // ---- block counts: nblk for the workgroup (barriers), n_w computed by
    // this wave, of which the first n_unm need no mask.
    int nblk = (p.Skv + BN - 1) / BN;
    int n_w, n_unm = p.Skv / BN;
    if (CAUSAL) {
        const int qlast = min(tile * p.tile_pos + p.tile_pos, p.Sq) - 1;
        const int klast = qlast + off;
        nblk = klast < 0 ? 0 : min(nblk, klast / BN + 1);
        const int klast_w = q0 + 31 + off;
        n_w = klast_w < 0 ? 0 : min(nblk, klast_w / BN + 1);
        const int kfirst_w = q0 + off + 1;          // number of keys valid for every row of the wave
        n_unm = min(n_unm, kfirst_w <= 0 ? 0 : kfirst_w / BN);
    } else {
        n_w = nblk;
    }
    n_unm = min(n_unm, n_w);
    const int nload = min(nblk, p.Skv / BN);    // blocks below this index are full tiles inside the walk

#ifdef ATTN_TRACE
    int trace_n = 0;
#endif
    WaveState w;
    {
        const int qrow = min(q0 + l32, p.Sq - 1);
        const __bf16 *qp = p.q + ((size_t)((size_t)b * p.Sq + qrow) * p.Hq + head) * HD + 8 * hh;
#pragma unroll
        for (int s = 0; s < 8; ++s) w.qf[s] = *(const bf16x8 *)(qp + 16 * s);
    }
    w.m = -INFINITY;
    w.l = 0.0f;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) w.acc[dt][r] = 0.0f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 8; ++r) w.pb[t][r] = 0u;

    // ---- global -> LDS tile loads.  One instruction moves 1 KiB: lane L's 16
    // bytes land at (wave-uniform LDS base) + 16*L, i.e. row L/16 and physical
    // 16-byte unit L%16 of a 4-row chunk; the lane fetches the logical unit
    // that the swizzle maps there.  K: unit ^ (row & 15), so that 16 lanes
    // reading one d-range of 16 consecutive rows touch 16 different units.
    // V: unit ^ ((row & 3) << 2), so that the 4 rows x 64 bytes a half-wave
    // fetches with the transposing read cover all banks once.
    const size_t kv_row_bytes = (size_t)p.Hkv * HD * 2;
    const unsigned char *kg = (const unsigned char *)(p.k + ((size_t)b * p.Skv * p.Hkv + hkv) * HD);
    const unsigned char *vg = (const unsigned char *)(p.v + ((size_t)b * p.Skv * p.Hkv + hkv) * HD);
    const int ld_r = lane >> 4, ld_u = lane & 15;
    // Byte offset of this lane's 16 bytes from the first row of a tile, for the wave's two chunks.
    uint32_t koff[2], voff[2];
    int ld_row[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        ld_row[i] = (wave * 2 + i) * 4 + ld_r;
        koff[i] = (uint32_t)(ld_row[i] * kv_row_bytes) + ((ld_u ^ (ld_row[i] & 15)) << 4);
        voff[i] = (uint32_t)(ld_row[i] * kv_row_bytes) + ((ld_u ^ ((ld_row[i] & 3) << 2)) << 4);
    }
    auto issue_tile = [&](int blk_req, bool is_v) __attribute__((always_inline)) {
        // A request past the last block re-reads the last block into the (dead) stage it would have
        // used: the number of loads in flight stays the same in every iteration.
        const int blk = min(blk_req, nblk - 1);
        const unsigned char *g = (is_v ? vg : kg) + (size_t)blk * BN * kv_row_bytes;
        const int lbase = (is_v ? V_BASE : 0) + (blk_req % NSTAGE) * TILE_BYTES + wave * 2048;
        const bool partial = (blk + 1) * BN > p.Skv;          // rows past the end: re-read the last row
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            uint32_t o = is_v ? voff[i] : koff[i];
            if (partial) {
                const int rl = min(ld_row[i], p.Skv - 1 - blk * BN);
                o = o - (uint32_t)(ld_row[i] * kv_row_bytes) + (uint32_t)(rl * kv_row_bytes);
            }
            lds_dma16(g, o, (uint32_t)(uintptr_t)(lds + lbase + i * 1024));
        }
    };
    // Fast form for full, in-range tiles: running tile pointers and LDS stage offsets, no clamping.
    const size_t tile_gbytes = (size_t)BN * kv_row_bytes;
    auto issue_loads_fast = [&](const unsigned char *kp, const unsigned char *vp, int kstage, int vstage)
        __attribute__((always_inline)) {
#ifdef ABL_NO_DMA
        return;
#endif
        const uint32_t lb = (uint32_t)(uintptr_t)lds + wave * 2048;
        lds_dma16(kp, koff[0], lb + kstage);
        lds_dma16(kp, koff[1], lb + kstage + 1024);
        lds_dma16(vp, voff[0], lb + V_BASE + vstage);
        lds_dma16(vp, voff[1], lb + V_BASE + vstage + 1024);
    };
    // The four loads of one iteration: K(kblk) and V(vblk), this wave's eighth of each tile.
    auto issue_loads = [&](int kblk, int vblk) __attribute__((always_inline)) {
#ifdef ABL_NO_DMA
        return;
#endif
        issue_tile(kblk, false);
        issue_tile(vblk, true);
    };

    // ---- per-lane LDS read addresses
    int kaddr[8];   // K operand: row l32 (+32 per tile), logical unit 2*st + hh
#pragma unroll
    for (int st = 0; st < 8; ++st) kaddr[st] = l32 * ROW_BYTES + (((2 * st + hh) ^ (l32 & 15)) << 4);
    // V operand via the transposing read: lane (i = lane%16, g = (lane%32)/16, hh) supplies the address
    // of key row 4*hh + i/4 and d = 16*g + 4*(i%4) of a 16-key x 32-d block and receives d = 16*g + i
    // of keys 4*hh .. 4*hh+3.
    int vaddr[4];
    {
        const int i16 = lane & 15, g = (lane >> 4) & 1;
        const int row = 4 * hh + (i16 >> 2);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            const int d = 32 * dt + 16 * g + 4 * (i16 & 3);
            vaddr[dt] = V_BASE + row * ROW_BYTES + ((((d >> 3) ^ ((row & 3) << 2))) << 4) + (d & 7) * 2;
        }
    }

    // ---- the pieces of one iteration
    auto stage_off = [&](int blk) __attribute__((always_inline)) { return (blk % NSTAGE) * TILE_BYTES; };
    auto next_stage = [&](int off) __attribute__((always_inline)) {      // stage_off(blk + 1) from stage_off(blk)
        return off == (NSTAGE - 1) * TILE_BYTES ? 0 : off + TILE_BYTES;
    };
    // S^T(blk) = K(blk) Q^T alone (first block only)
    auto qk = [&](int blk) __attribute__((always_inline)) {
        const int kb = (blk % NSTAGE) * TILE_BYTES;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) w.s[t][r] = 0.0f;
#pragma unroll
        for (int st = 0; st < 8; ++st)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                bf16x8 a = *(const LDS_AS bf16x8 *)(lds + kb + t * 32 * ROW_BYTES + kaddr[st]);
                w.s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, w.qf[st], w.s[t], 0, 0, 0);
            }
    };
    // The matrix half: O^T += V(vblk)^T P^T (16 MFMAs), then S^T = K(kblk) Q^T (16 MFMAs).
    // Written as one software-pipelined sequence: the LDS reads of MFMA i+PREFETCH are issued
    // before MFMA i, so that LDS latency hides behind the matrix pipe.
    // vb / kb: byte offset of the LDS stage that holds the V / K block (stage_off(block)).
    auto mat_half = [&](int vb, int kb) __attribute__((always_inline)) {
#ifdef ABL_NO_MAT
        return;
#endif
        constexpr int PREFETCH = MAT_PREFETCH;
        bf16x8 frag[32];
        // stage offsets folded into the per-lane bases once, so every read below is base + immediate
        int va[4], ka[8];
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) va[dt] = vaddr[dt] + vb;
#pragma unroll
        for (int st = 0; st < 8; ++st) ka[st] = kaddr[st] + kb;
        // Slot i of the sequence: even slots are PV MFMA i/2, odd slots QK MFMA i/2, so that two MFMAs
        // that accumulate into the same registers are at least four slots apart.
        auto fetch = [&](int slot) __attribute__((always_inline)) -> bf16x8 {
            const int i = slot >> 1;
#ifdef ABL_NO_LDSREAD
            return w.qf[i & 7];
#endif
            if ((slot & 1) == 0) {            // V^T operand of PV MFMA i: key group i/4, d tile i%4
                const int ro = (i >> 2) * 16 * ROW_BYTES;
                s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)(lds + va[i & 3] + ro));
                s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (LDS_AS s16x4 *)(lds + va[i & 3] + (ro + 8 * ROW_BYTES)));
                s16x8 av = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                return __builtin_bit_cast(bf16x8, av);
            }
            const int st = i >> 1, t = i & 1;   // K operand of QK MFMA i: d step st, key tile t
            return *(const LDS_AS bf16x8 *)(lds + ka[st] + t * 32 * ROW_BYTES);
        };
#pragma unroll
        for (int i = 0; i < PREFETCH; ++i) frag[i] = fetch(i);
#pragma unroll
        for (int slot = 0; slot < 32; ++slot) {
            if (slot + PREFETCH < 32) frag[slot + PREFETCH] = fetch(slot + PREFETCH);
#ifdef ABL_MAT_MARKS
            if (slot == 8 || slot == 16 || slot == 24) TRACE_POINT();
#endif
            const int i = slot >> 1;
            if ((slot & 1) == 0) {
                const int g = i >> 2;         // key group: tile g/2, half g%2
                u32x4 pw = {w.pb[g >> 1][4 * (g & 1)], w.pb[g >> 1][4 * (g & 1) + 1],
                            w.pb[g >> 1][4 * (g & 1) + 2], w.pb[g >> 1][4 * (g & 1) + 3]};
                w.acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    frag[slot], __builtin_bit_cast(bf16x8, pw), w.acc[i & 3], 0, 0, 0);
            } else {
                const int st = i >> 1, t = i & 1;
                if (st == 0) {
                    f32x16 z;
#pragma unroll
                    for (int r = 0; r < 16; ++r) z[r] = 0.0f;
                    w.s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[slot], w.qf[st], z, 0, 0, 0);
                } else {
                    w.s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[slot], w.qf[st], w.s[t], 0, 0, 0);
                }
            }
        }
        schedule_matrix_half();
    };
    auto rescale = [&](float mn, float alpha) __attribute__((always_inline)) {
        w.m = mn;
        w.l *= alpha;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) w.acc[dt][r] *= alpha;
    };
    // P^T = exp2(S^T * c - m) of an unmasked block into the PV operand registers; returns this lane's
    // partial row sum (its 16 of every 32 keys), taken from the unrounded FP32 probabilities.
    auto probabilities = [&]() __attribute__((always_inline)) -> float {
        float ls0 = 0.0f, ls1 = 0.0f;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(w.s[t][r], p.c, -w.m));
                const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(w.s[t][r + 1], p.c, -w.m));
                ls0 += e0;
                ls1 += e1;
                w.pb[t][r >> 1] = pack_bf16(e0, e1);
            }
        return ls0 + ls1;
    };
    // Raise the running maximum to cover the block in w.s and rescale the accumulator and the row sum.
    auto raise_reference = [&]() __attribute__((always_inline)) {
        float mx = max3(w.s[0][0], w.s[0][1], w.s[0][2]);
#pragma unroll
        for (int i = 3; i < 31; i += 2) mx = max3(mx, w.s[i >> 4][i & 15], w.s[(i + 1) >> 4][(i + 1) & 15]);
        mx = max3(mx, w.s[1][15], w.s[1][15]);
        mx = lane32_max(mx) * p.c;
        const float mn = fmaxf(w.m, mx);
        rescale(mn, __builtin_amdgcn_exp2f(w.m - mn));
    };
    // Softmax of a block without masked keys.  Softmax is the same against any reference point, so
    // the probabilities are first formed against the running maximum as it stands, WITHOUT looking
    // for the block's maximum.  Only if some lane's partial row sum comes out above P_SUM_LIMIT (or
    // is not a number) did the scores outgrow the reference; then the whole wavefront raises the
    // reference, rescales, and forms the probabilities again.  The branch is wave-uniform and rare:
    // with scores of bounded spread the reference settles after the first blocks.
    auto softmax_fast = [&]() __attribute__((always_inline)) {
#ifdef ABL_NO_VEC
        return;
#endif
        float ls = probabilities();
        if (__builtin_amdgcn_ballot_w64(!(ls <= P_SUM_LIMIT)) != 0) {
            raise_reference();
            ls = probabilities();
        }
        w.l += ls;
    };
    auto softmax_masked = [&](int blk) __attribute__((always_inline)) {   // diagonal or tail block: key index per register, limit per lane
        int lim = p.Skv - 1;
        if (CAUSAL) lim = min(lim, q0 + l32 + off);
        const int kidx = blk * BN + 4 * hh;
        float mx = -INFINITY;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = kidx + 32 * t + 8 * (r >> 2) + (r & 3);
                mx = fmaxf(mx, key <= lim ? w.s[t][r] : -INFINITY);
            }
        mx = lane32_max(mx);
        mx = (mx == -INFINITY) ? -INFINITY : mx * p.c;
        if (__builtin_amdgcn_ballot_w64(mx > w.m + RESCALE_SLACK) != 0) {
            const float mn = fmaxf(w.m, mx);
            rescale(mn, (mn == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(w.m - mn));
        }
        const float mu = (w.m == -INFINITY) ? 0.0f : w.m;
        float ls = 0.0f;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const int key = kidx + 32 * t + 8 * (r >> 2) + (r & 3);
                float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(w.s[t][r], p.c, -mu));
                float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(w.s[t][r + 1], p.c, -mu));
                e0 = (key <= lim) ? e0 : 0.0f;
                e1 = (key + 1 <= lim) ? e1 : 0.0f;
                ls += e0 + e1;
                w.pb[t][r >> 1] = pack_bf16(e0, e1);
            }
        w.l += ls;
    };
    TRACE_ALWAYS();
    if (nblk > 0) {
        issue_tile(0, false);
        issue_loads(1, 0);
        __builtin_amdgcn_s_waitcnt(WAIT_VMCNT4);          // K(0) has landed
        PHASE_BARRIER();

        // Wavefronts 0-3 (one per SIMD) run "matrix half, vector half"; wavefronts 4-7 run the same
        // sequence half an iteration later, so the matrix pipe and the vector ALU of a SIMD are busy
        // at the same time.  Every half ends with a workgroup barrier.
        //
        // K/V tiles live in NSTAGE = 3 LDS stages.  The vector half of iteration j ends by requesting
        // K(j+3) and V(j+2) (into the stages of K(j) and V(j-1), whose last readers finished at least
        // one barrier earlier) and then waits until only those four loads are still in flight, i.e.
        // until K(j+2) and V(j+1) have landed, one barrier before their first reader.  Issuing the
        // loads from the vector half keeps the address unit's queueing delay off the matrix half.
        //
        // Blocks >= n_unm go through the masked softmax, which yields P = 0 where a key is not valid:
        // blocks that are masked out entirely for this wavefront (and the block past the end that the
        // last matrix half multiplies from a stale stage) then contribute nothing, with no branch
        // around the MFMA sequences.
        if (wave < 4) {
            qk(0);
            softmax_masked(0);
            issue_loads(2, 1);
            __builtin_amdgcn_s_waitcnt(WAIT_VMCNT4);
            PHASE_BARRIER();
            int j = 0;
            int vst = stage_off(0), kst = stage_off(1);       // stages of V(j) and K(j+1)
            // running request state of the fast loop: K(j+3) goes where K(j) was, V(j+2) where V(j-1) was
            const unsigned char *kp = kg + 3 * tile_gbytes, *vp = vg + 2 * tile_gbytes;
            int kreq = stage_off(3), vreq = stage_off(2);
#pragma nounroll
            for (; j + 1 < n_unm && j + 3 < nload; ++j) {
                MAT_PRIO(1);
                mat_half(vst, kst);
                MAT_PRIO(0);
                vst = next_stage(vst);
                kst = next_stage(kst);
                MID_BARRIER();
                softmax_fast();
                issue_loads_fast(kp, vp, kreq, vreq);
                kp += tile_gbytes;
                vp += tile_gbytes;
                kreq = next_stage(kreq);
                vreq = next_stage(vreq);
                __builtin_amdgcn_s_waitcnt(WAIT_VMCNT4);
                PHASE_BARRIER();
            }
#pragma nounroll
            for (; j < nblk; ++j) {
                MAT_PRIO(1);
                mat_half(vst, kst);
                MAT_PRIO(0);
                vst = next_stage(vst);
                kst = next_stage(kst);
                MID_BARRIER();
                softmax_masked(j + 1);
                issue_loads(j + 3, j + 2);
                __builtin_amdgcn_s_waitcnt(WAIT_VMCNT4);
                PHASE_BARRIER();
            }
        } else {
            issue_loads(2, 1);
            qk(0);
            __builtin_amdgcn_s_waitcnt(WAIT_VMCNT4);
            PHASE_BARRIER();
            int j = 0;
            int vst = stage_off(0), kst = stage_off(1);       // stages of V(j) and K(j+1)
            const unsigned char *kp = kg + 3 * tile_gbytes, *vp = vg + 2 * tile_gbytes;
            int kreq = stage_off(3), vreq = stage_off(2);
#pragma nounroll
            for (; j < n_unm && j + 3 < nload; ++j) {
                softmax_fast();
                issue_loads_fast(kp, vp, kreq, vreq);
                kp += tile_gbytes;
                vp += tile_gbytes;
                kreq = next_stage(kreq);
                vreq = next_stage(vreq);
                MID_BARRIER();
                MAT_PRIO(1);
                mat_half(vst, kst);
                MAT_PRIO(0);
                vst = next_stage(vst);
                kst = next_stage(kst);
                __builtin_amdgcn_s_waitcnt(WAIT_VMCNT4);
                PHASE_BARRIER();
            }
#pragma nounroll
            for (; j < nblk; ++j) {
                softmax_masked(j);
                issue_loads(j + 3, j + 2);
                MID_BARRIER();
                MAT_PRIO(1);
                mat_half(vst, kst);
                MAT_PRIO(0);
                vst = next_stage(vst);
                kst = next_stage(kst);
                __builtin_amdgcn_s_waitcnt(WAIT_VMCNT4);
                PHASE_BARRIER();
            }
        }
    }

    TRACE_ALWAYS();
    // ---- epilogue: O = acc / l (BF16), LSE = ln2 * (m + log2 l)
    const float lt = lane32_sum(w.l);
    const float inv = lt > 0.0f ? 1.0f / lt : 0.0f;
    const int qrow = q0 + l32;
    if (qrow < p.Sq) {
        __bf16 *op = p.o + ((size_t)((size_t)b * p.Sq + qrow) * p.Hq + head) * HD + 4 * hh;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                u32x2 ww = {pack_bf16(w.acc[dt][4 * rg] * inv, w.acc[dt][4 * rg + 1] * inv),
                            pack_bf16(w.acc[dt][4 * rg + 2] * inv, w.acc[dt][4 * rg + 3] * inv)};
                *(u32x2 *)(op + 32 * dt + 8 * rg) = ww;
            }
        if (hh == 0) {
            const float lse = lt > 0.0f ? (w.m + __builtin_amdgcn_logf(lt)) * 0.6931471805599453f : -INFINITY;
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

    // 96 KiB of dynamic LDS needs an opt-in, once per device and kernel.
    {
        static bool ready[64] = {};
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return ATTN_E_LAUNCH;
        if (!ready[dev]) {
            if (hipFuncSetAttribute((const void *)attn_fwd_kernel<true>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess ||
                hipFuncSetAttribute((const void *)attn_fwd_kernel<false>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess)
                return ATTN_E_LAUNCH;
            ready[dev] = true;
        }
    }
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
