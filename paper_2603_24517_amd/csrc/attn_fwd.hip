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
// tiles go from global memory straight into three XOR-swizzled LDS stages
// (global_load_lds_dwordx4), requested two iterations before use.  For
// grouped-query attention the 256 rows are PACK heads of one K/V group x
// 256/PACK positions, so one K/V tile in LDS serves several query heads.
//
// The key-block loop is software-pipelined three deep inside every wavefront:
// iteration j issues the MFMAs of O += P(j) V(j) and S(j+2) = K(j+2) Q^T while
// its vector instructions turn S(j+1) into P(j+1).  The two instruction kinds
// are independent within an iteration and are interleaved (one MFMA, its LDS
// reads, a few VALU), so the matrix pipe and the vector ALU run at the same
// time (the paper's section 2.2 describes the same need, met on its hardware
// by specialised warps), with one workgroup barrier per iteration.
//
// The launch has one workgroup per CU, and each works through a list of
// (batch entry, K/V head, query tile) items: while an item is in its last
// blocks it already requests the next item's first K/V tiles into the stages
// that fall free and the next item's Q into the rest of LDS, and O leaves
// through LDS as whole rows, so that the matrix pipe idles for little more
// than one short prologue per item.  The per-iteration overhead of the loop
// (stage rotation, request addresses, LDS address arithmetic) is kept out of
// the instruction stream as far as possible, because with two wavefronts per
// SIMD the issue of vector instructions, not the matrix pipe alone, is what
// an iteration's length follows.
//
// A second kernel at the end of this file serves small problems (few query
// rows, however many keys): 32-row work items whose key blocks are shared out
// among the wavefronts of a workgroup and whose partial results are merged
// through LDS.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>
#include <type_traits>
#include <atomic>

#include "../../include/attn.h"

// ---- Compile-time variants.  The shipped library defines none of these; each alternative is built
// into a library of its own and goes through the same parity tests, so that the choices below can be
// measured against what they replaced (the paper's sections 5.1 and 5.2 analyse the same two
// decisions on its hardware).
//
// ATTN_SOFTMAX: how the softmax of an unmasked key block treats the running maximum.
//   0  (shipped) probabilities against the running maximum as it stands, no search for the block's
//      maximum; the exact path runs only if a partial row sum leaves the safe range
//   1  block maximum every block, accumulator and row sums multiplied by alpha every block, no branch
//   2  block maximum every block, the multiplication skipped under a wave-uniform vote when no lane's
//      maximum rose
//   3  block maximum every block, the reference raised (and the accumulator rescaled) only where the
//      block maximum exceeds it by more than 8 in log2 units
#ifndef ATTN_SOFTMAX
#define ATTN_SOFTMAX 0
#endif
// ATTN_ITEM_OVERLAP: 1 (shipped) the last blocks of an item request the first tiles and the Q tile of the
// next one; 0 every item loads its own tiles and its Q after the epilogue of the item before.
#ifndef ATTN_ITEM_OVERLAP
#define ATTN_ITEM_OVERLAP 1
#endif
// ATTN_SMALL_PATH: which launches go to the split-key kernel for small problems (at the end of this
// file): 1 (shipped) those whose 256-row work items would occupy at most a quarter of the compute
// units; 0 none; 2 all.
#ifndef ATTN_SMALL_PATH
#define ATTN_SMALL_PATH 1
#endif
// ATTN_LDS_PREFETCH: how many MFMAs ahead of its consumer an LDS operand fragment is read (shipped: 3).
#ifndef ATTN_LDS_PREFETCH
#define ATTN_LDS_PREFETCH 3
#endif
// ATTN_WAVES_PER_SIMD (shipped: 2): the occupancy the attention kernel is compiled for, i.e. its register
// budget: 512 / n vector registers per wavefront.  3 and 4 are for compile-only builds that show what a
// smaller budget costs in spills (the paper's section 5.3 weighs register budgets on its hardware);
// such builds are not meant to be run (see wait_vmcnt below for what a spill costs in this loop).
#ifndef ATTN_WAVES_PER_SIMD
#define ATTN_WAVES_PER_SIMD 2
#endif
// ATTN_CLOCKS (undefined in the shipped library): the first wavefront of the first workgroup stamps the
// shader cycle counter and the constant 100 MHz counter when it starts and when it ends, and the cycle
// counter where the key-block loop of its second and of its third work item starts and ends; the
// library exports attn_clocks_read(), and the benchmark derives the shader clock of a launch, the
// length of an iteration and the stretch between two items from the stamps.
// ATTN_CLOCKS=2 additionally has the first and the last wavefront of that workgroup add up, over its
// second work item, the cycles each phase of an item takes (set-up, first score blocks, first softmax,
// the key-block iterations by kind, epilogue), read with attn_phases_read().  A stamp per iteration
// costs about 1.5 % of the loop, which is why the clock figures come from the build without them.
static_assert(ATTN_SOFTMAX >= 0 && ATTN_SOFTMAX <= 3, "ATTN_SOFTMAX is 0, 1, 2 or 3");
static_assert(ATTN_LDS_PREFETCH >= 1 && ATTN_LDS_PREFETCH <= 8, "ATTN_LDS_PREFETCH is 1 .. 8");

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

constexpr int HD = 128;              // head dimension
constexpr int BN = 64;               // keys per K/V block
constexpr int NWAVES = 8;            // wavefronts per workgroup; one workgroup fills a CU (registers and LDS)
constexpr int NTHREADS = NWAVES * 64;
constexpr int WG_ROWS = NWAVES * 32; // query rows per workgroup
constexpr int ROW_BYTES = HD * 2;    // one (token, head) row of BF16
constexpr int TILE_BYTES = BN * ROW_BYTES;
constexpr int NSTAGE = 3;                   // LDS stages per operand
constexpr int REQ_AHEAD = NSTAGE - 1;       // tiles are requested this many iterations before use
constexpr int LPT = 16 / NWAVES;            // 1 KiB load instructions per tile and wavefront
constexpr int V_BASE = NSTAGE * TILE_BYTES; // K stages first, V stages after them
constexpr int Q_BASE = 2 * NSTAGE * TILE_BYTES;      // after the stages: Q of the next item, 8 KiB per wavefront
constexpr int Q_WAVE_BYTES = 32 * ROW_BYTES;
constexpr int LDS_BYTES = Q_BASE + NWAVES * Q_WAVE_BYTES;   // 160 KiB, all of a CU's LDS
// Largest partial row sum (16 probabilities of one lane) the fast softmax path accepts: probabilities
// stay below 2^14 relative to the reference maximum, far inside BF16 / FP32 range.
constexpr float P_SUM_LIMIT = 16384.0f;
constexpr int MAT_PREFETCH = ATTN_LDS_PREFETCH;   // LDS reads run this many MFMAs ahead of their consumer
// s_waitcnt vmcnt(n), n < 16, other counters untouched.  The tile requests are counted by hand: "all but
// the newest n vector-memory operations have completed" stands for "the tiles of the iterations before
// have landed".  That holds whatever else is in the queue, because the loads that must have landed are
// always followed by n newer loads and loads complete in order; but it is only CHEAP while the requests
// are the only memory operations of the loop: a register spill would bring reloads of the compiler's own,
// each behind an s_waitcnt vmcnt(0) that waits for every tile request in flight (a memory latency per
// reload, in a loop whose iteration is shorter than one).  So the kernels must compile without scratch
// (a host-side test of the built code object checks that), and the epilogue's stores are issued only
// after the wait that the next item's first tiles need.
constexpr int wait_vmcnt(int n) { return 0x0F70 | n; }
constexpr int WAIT_VMCNT0 = wait_vmcnt(0);
// end of an iteration: everything but the loads of the last REQ_AHEAD-1 iterations has landed
constexpr int WAIT_ITER_END = wait_vmcnt((REQ_AHEAD - 1) * 2 * LPT);

// Exact n / d for 0 <= n < 2^31 as a multiply-high, an add and a shift; the constants come from the host.
struct Div { uint32_t mul, shift; };
__host__ __device__ inline uint32_t fast_div(uint32_t n, const Div d) {
#ifdef __HIP_DEVICE_COMPILE__
    return (__umulhi(n, d.mul) + n) >> d.shift;
#else
    return (uint32_t)((((uint64_t)n * d.mul) >> 32) + n) >> d.shift;
#endif
}
inline Div make_div(uint32_t d) {
    Div r;
    r.shift = 0;
    while ((1u << r.shift) < d) ++r.shift;
    r.mul = (uint32_t)((((uint64_t)1 << 32) * (((uint64_t)1 << r.shift) - d)) / d + 1);
    return r;
}

// How the work items are dealt out (read by the per-item code only).
struct Sched {
    int total;      // work items = B * Hkv * chunks * ntile
    int per_xcd;    // entries in the work list of one XCD (non-causal: ceil(total / 8))
    int slots;      // workgroups per XCD in this launch (one per CU); the grid is 8 * slots
    int ntile;      // ceil(Sq / tile_pos)
    // causal only: how the (group, tile) pairs are dealt to the XCDs (a group = one batch entry, K/V head and chunk)
    int split;      // every group is cut into `split` sub-groups (a power of two), sub-group r holding the tiles t = r (mod split)
    int split_log2;
    int nsub;       // tiles per sub-group = ceil(ntile / split); the padding entries are skipped
    int sgx;        // sub-groups per XCD = groups * split / 8
    int window;     // sub-groups that one XCD works through together, longest tiles of all of them first
    int per_win;    // window * nsub
    Div d_ntile, d_per_win, d_window;
};
// Tensor shape and head packing (read by the per-item code only).
struct Shape {
    int Sq, Hq;
    int G;          // Hq / Hkv
    int pack;       // query heads of one K/V group served by one workgroup (1, 2, 4 or 8)
    int pack_log2;
    int tile_pos;   // query positions per workgroup = WG_ROWS / pack
    int chunks;     // G / pack
    Div d_chunks, d_hkv;
};
struct Params {
    const __bf16 *k, *v;
    int Hkv, Skv;
    float c;        // scale * log2(e)
    int pad_;
    // the rest is read from the argument block where it is needed
    const __bf16 *q;
    __bf16 *o;
    float *lse;
    Shape shape;
    Sched sched;
};

// "Extreme" below is the raw score that maximises score * c: the largest one for c >= 0, the smallest
// for c < 0 (NEG), so that the running maximum of the scaled scores is c times the extreme.
template <bool NEG>
__device__ __forceinline__ float ext2(float a, float b) { return NEG ? fminf(a, b) : fmaxf(a, b); }
template <bool NEG>
__device__ __forceinline__ float lane32_ext(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return ext2<NEG>(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float lane32_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    bf16x2 p = __builtin_convertvector((f32x2){a, b}, bf16x2);   // v_cvt_pk_bf16_f32, nearest even
    return __builtin_bit_cast(uint32_t, p);
}
// acc + lo(p) + hi(p) for a pair of BF16 values (v_dot2c_f32_bf16 against (1, 1)).
__device__ __forceinline__ float add_bf16_pair(uint32_t p, float acc) {
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, p), ones, acc, false);
}
template <bool NEG>
__device__ __forceinline__ float ext3(float a, float b, float c) {
    float r;
    if (NEG) asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    else asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
// 16 bytes per lane from global memory straight into LDS: lane L's data lands at lds_base + 16*L.
// Issued as inline assembly so that the compiler's counter bookkeeping does not make every later
// LDS read wait for it; the caller waits with s_waitcnt vmcnt(n) before the barrier that publishes
// the tile.
// A wave-uniform pointer as a scalar-register pair, also when the compiler chose to keep it in vector registers.
__device__ __forceinline__ const unsigned char *uniform_ptr(const unsigned char *ptr) {
    const uint64_t v = (uint64_t)(uintptr_t)ptr;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const unsigned char *)(uintptr_t)(((uint64_t)hi << 32) | lo);
}
// Both forms write M0 and say so in their clobber lists: the compiler reserves M0 (it sets it itself
// right before an instruction of its own that reads it) and warns that it will not preserve it across
// the statement, which is exactly what is meant here.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void lds_dma16(const unsigned char *base, uint32_t voffset, uint32_t lds_base) {
    base = uniform_ptr(base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base), "v"(voffset), "s"(base)
                 : "memory", "m0");
}
// The same with the LDS address given as a scalar plus a compile-time constant (one scalar instruction).
template <int IMM>
__device__ __forceinline__ void lds_dma16_imm(const unsigned char *base, uint32_t voffset, uint32_t lds_base) {
    asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base), "v"(voffset), "s"(base), "n"(IMM)
                 : "memory", "scc", "m0");
}
#pragma clang diagnostic pop
// Keeps the instruction that produces x at this point of the program order (no code is emitted).
#define PIN(x) asm volatile("" : "+v"(x))
__device__ __forceinline__ void wg_barrier() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
}

#ifdef ATTN_CLOCKS
// cycle counter at start / end, 100 MHz counter at start / end; then, for the second and the third item of
// the first workgroup: cycle counter at the start and at the end of the key-block loop, and the loop's iterations
__device__ unsigned long long g_clocks[10];
#define ATTN_STAMP(k, v) do { __builtin_amdgcn_sched_barrier(0); if (bid == 0 && tid == 0 && (item_no == 1 || item_no == 2)) \
                                  g_clocks[4 + 3 * (item_no - 1) + (k)] = (v); __builtin_amdgcn_sched_barrier(0); } while (0)
#else
#define ATTN_STAMP(k, v) do { } while (0)
#endif
#if defined(ATTN_CLOCKS) && ATTN_CLOCKS >= 2
// [first / last wavefront of the first workgroup][phase]: cycles of its second work item spent in
// 0 set-up (next item's lookup, state reset, Q request; a cold item's first tile requests and wait),
// 1 the first two score blocks, 2 the first softmax, 3 the barrier and requests before the loop,
// 4 iterations in which this wavefront took the fast path, 5 their number, 6 other iterations but the
// last, 7 their number, 8 the last iteration, 9 the wait for outstanding loads, 10 the epilogue,
// 11 the whole item
__device__ unsigned long long g_phases[2][12];
__device__ __forceinline__ unsigned long long phase_now() {
    __builtin_amdgcn_sched_barrier(0);
    const unsigned long long t = __builtin_readcyclecounter();
    __builtin_amdgcn_sched_barrier(0);
    return t;
}
#define ATTN_PHASE(k) do { const unsigned long long now_ = phase_now(); ph[k] += now_ - ph_prev; ph_prev = now_; } while (0)
#define ATTN_PHASE_COUNT(k) do { ++ph[k]; } while (0)
#else
#define ATTN_PHASE(k) do { } while (0)
#define ATTN_PHASE_COUNT(k) do { } while (0)
#endif

template <bool CAUSAL, bool NEG>
__global__ __launch_bounds__(NTHREADS) __attribute__((amdgpu_waves_per_eu(ATTN_WAVES_PER_SIMD, ATTN_WAVES_PER_SIMD)))
void attn_fwd_kernel(const Params p)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    LDS_AS unsigned char *lds = (LDS_AS unsigned char *)smem;
    // Launch constants that only the per-item code needs are read from the kernel argument block where
    // they are used, instead of occupying scalar registers through the block loop.
    auto cold = [&]() __attribute__((always_inline)) -> const __attribute__((address_space(4))) Params & {
        auto cp = (const __attribute__((address_space(4))) Params *)__builtin_amdgcn_kernarg_segment_ptr();
        asm volatile("" : "+s"(cp));
        return *cp;
    };

    // ---- work distribution.  The launch has one workgroup per CU, 8 * slots of them, dealt round-robin
    // to the 8 XCDs by the hardware: workgroup (x = bid % 8, slot = bid / 8) works through entries
    // slot, slot + slots, ... of XCD x's list, one after the other, so that the loads of the next
    // entry can start while the current one finishes.
    // Non-causal: each XCD's list is a contiguous range of items (neighbours share K/V in that XCD's
    // L2).  Causal: tiles differ in length, so each XCD owns whole sub-groups of equal total work and
    // its list walks `window` of them together from their longest tiles to their shortest; odd rounds
    // run through the slots backwards, so that the workgroup that drew the longest tile of one round
    // draws the shortest of the next.
    const int bid = blockIdx.x;
    const int xcd = bid & 7, slot = bid >> 3;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31;
    const int hh = lane >> 5;
#ifdef ATTN_CLOCKS
    if (bid == 0 && tid == 0) { g_clocks[2] = wall_clock64(); g_clocks[0] = __builtin_readcyclecounter(); }
#endif
    const int off = p.Skv - cold().shape.Sq;                    // causal: key j valid iff j <= i + off
    const int nfull = p.Skv / BN;                               // tiles below this index are full
    const bool all_full = (p.Skv % BN) == 0;

    // one wide scalar load each, where the per-item code starts
    auto load_sched = [&]() __attribute__((always_inline)) -> Sched {
        Sched sc;
        __builtin_memcpy(&sc, &cold().sched, sizeof(Sched));
        return sc;
    };
    auto load_shape = [&]() __attribute__((always_inline)) -> Shape {
        Shape sh;
        __builtin_memcpy(&sh, &cold().shape, sizeof(Shape));
        return sh;
    };
    // entry j of this XCD's list -> (group, tile); false for a padding entry
    auto decode = [&](const Sched &sc, int j, int &grp, int &tile) __attribute__((always_inline)) -> bool {
        if (CAUSAL) {
            const int w = fast_div(j, sc.d_per_win);
            const int r = j - w * sc.per_win;
            const int kw = min(sc.window, sc.sgx - w * sc.window);      // the last window may be narrower
            const int st = kw == sc.window ? (int)fast_div(r, sc.d_window) : r / kw;
            const int sg = xcd * sc.sgx + w * sc.window + (r - st * kw);
            grp = sg >> sc.split_log2;
            const int tile_r = st * sc.split + (sg & (sc.split - 1));
            tile = sc.ntile - 1 - tile_r;                               // long (late) query tiles first
            return tile_r < sc.ntile;
        }
        const int item = xcd * sc.per_xcd + j;
        grp = fast_div(item, sc.d_ntile);
        tile = item - grp * sc.ntile;
        return item < sc.total;
    };
    // first round >= r in which this workgroup has a real entry; false when its list is exhausted
    auto find_item = [&](int &r, int &grp, int &tile) __attribute__((always_inline)) -> bool {
        const Sched sc = load_sched();
        for (; r * sc.slots < sc.per_xcd; ++r) {
            const int j = r * sc.slots + ((CAUSAL && (r & 1)) ? sc.slots - 1 - slot : slot);
            if (j < sc.per_xcd && decode(sc, j, grp, tile)) return true;
        }
        return false;
    };
    // what a wavefront needs to know of an item
    struct Geo {
        int b, head, q0;                 // batch entry, query head and first query row of this wavefront
        int nblk;                        // key blocks of the workgroup (one barrier each)
        const unsigned char *kg, *vg;    // first K / V row of the item's batch entry and K/V head
    };
    const size_t kv_row_bytes = (size_t)p.Hkv * HD * 2;
    const size_t tile_gbytes = (size_t)BN * kv_row_bytes;
    auto geometry = [&](int grp, int tile) __attribute__((always_inline)) -> Geo {
        const Shape sh = load_shape();
        Geo g;
        const int bh = fast_div(grp, sh.d_chunks);
        const int chunk = grp - bh * sh.chunks;
        g.b = fast_div(bh, sh.d_hkv);
        const int hkv = bh - g.b * p.Hkv;
        g.head = hkv * sh.G + chunk * sh.pack + (wave & (sh.pack - 1));
        g.q0 = tile * sh.tile_pos + (wave >> sh.pack_log2) * 32;
        g.nblk = (p.Skv + BN - 1) / BN;
        if (CAUSAL) {
            const int klast = min(tile * sh.tile_pos + sh.tile_pos, sh.Sq) - 1 + off;
            g.nblk = klast < 0 ? 0 : min(g.nblk, klast / BN + 1);
        }
        g.kg = (const unsigned char *)(p.k + ((size_t)g.b * p.Skv * p.Hkv + hkv) * HD);
        g.vg = (const unsigned char *)(p.v + ((size_t)g.b * p.Skv * p.Hkv + hkv) * HD);
        // all of it is wave-uniform: say so, so that it lives in scalar registers
        g.b = __builtin_amdgcn_readfirstlane(g.b);
        g.head = __builtin_amdgcn_readfirstlane(g.head);
        g.q0 = __builtin_amdgcn_readfirstlane(g.q0);
        g.nblk = __builtin_amdgcn_readfirstlane(g.nblk);
        g.kg = uniform_ptr(g.kg);
        g.vg = uniform_ptr(g.vg);
        return g;
    };

    // ---- the item in work and the one after it
    int b = 0, head = 0, q0 = 0;
    int nblk = 0;       // key blocks of the workgroup
    int n_w = 0;        // of those, the blocks that hold a key valid for some row of this wavefront
    int n_unm = 0;      // of those, the leading blocks that need no mask at all
    const unsigned char *kg = nullptr, *vg = nullptr;
    bool warm_next = false;             // the item after this one exists and its first tiles are requested by this one
    int nx_nblk = 0;
    const unsigned char *nx_kg = nullptr, *nx_vg = nullptr;
    int ring0 = 0;                      // LDS stage of block 0 of the item in work
    auto enter = [&](const Geo &g) __attribute__((always_inline)) {
        b = g.b; head = g.head; q0 = g.q0; nblk = g.nblk; kg = g.kg; vg = g.vg;
        n_unm = p.Skv / BN;
        n_w = nblk;
        if (CAUSAL) {
            const int klast_w = q0 + 31 + off;          // last key valid for the last row of the wave
            n_w = klast_w < 0 ? 0 : min(nblk, klast_w / BN + 1);
            const int kfirst_w = q0 + off + 1;          // number of keys valid for every row of the wave
            n_unm = min(n_unm, kfirst_w <= 0 ? 0 : kfirst_w / BN);
        }
        n_unm = min(n_unm, n_w);
    };

    // ---- everything the wavefront keeps across the key-block loop
    bf16x8 qf[8];          // Q^T operand: query lane%32, d = 16*s + 8*(lane/32) .. +7
    f32x16 sa[2], sb[2];   // S^T of two blocks in flight (two 32-key tiles each): the softmax consumes one
                           // while the MFMAs fill the other
    uint32_t pb[2][8];     // P^T of the block whose PV product comes next, BF16 pairs
    f32x16 acc[4];         // O^T accumulator: four 32-d tiles
    float m;               // running maximum in log2 units (score * scale * log2 e)
    float l;               // this lane's share of the running sum (its 16 of every 32 keys), unrounded FP32
                           // probabilities: the sum LSE is formed from
    float lr;              // the same sum over the BF16-rounded probabilities that multiply V: O is
                           // normalised by this one, so that a rounding error in a dominant weight
                           // cancels between numerator and denominator
    auto load_q = [&](const Geo &g) __attribute__((always_inline)) {
        const int Sq = cold().shape.Sq, Hq = cold().shape.Hq;
        const int qrow = min(g.q0 + l32, Sq - 1);
        const __bf16 *qp = cold().q + ((size_t)((size_t)g.b * Sq + qrow) * Hq + g.head) * HD + 8 * hh;
#pragma unroll
        for (int s = 0; s < 8; ++s) qf[s] = *(const bf16x8 *)(qp + 16 * s);
    };
    // The same through LDS: requested (wave-private region, the K swizzle) when the item before
    // starts, fetched into registers when that one's last block is done.
    auto request_q = [&](const Geo &g) __attribute__((always_inline)) {
        const int Sq = cold().shape.Sq, Hq = cold().shape.Hq;
        const size_t q_row_bytes = (size_t)Hq * HD * 2;
        const int q0c = min(g.q0, Sq - 1);          // rows past the end of Q re-read the last row
        const unsigned char *qg = (const unsigned char *)(cold().q + ((size_t)((size_t)g.b * Sq + q0c) * Hq + g.head) * HD);
        const int last = Sq - 1 - q0c;
        const uint32_t lbase = (uint32_t)(uintptr_t)lds + Q_BASE + wave * Q_WAVE_BYTES;
        int ln = lane;
        PIN(ln);            // per-lane offsets are formed here, not kept in registers across the block loop
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = 4 * i + (ln >> 4);
            const uint32_t o = (uint32_t)(min(row, last) * q_row_bytes) + (((ln & 15) ^ (row & 15)) << 4);
            lds_dma16(qg, o, lbase + i * 1024);
        }
    };
    auto reset_state = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[dt][r] = 0.0f;
        m = -INFINITY;
        l = 0.0f;
        lr = 0.0f;
    };
    // ---- global -> LDS tile loads.  One instruction moves 1 KiB: lane L's 16
    // bytes land at (wave-uniform LDS base) + 16*L, i.e. row L/16 and physical
    // 16-byte unit L%16 of a 4-row chunk; the lane fetches the logical unit
    // that the swizzle maps there.  K: unit ^ (row & 15), so that 16 lanes
    // reading one d-range of 16 consecutive rows touch 16 different units.
    // V: unit ^ ((row & 3) << 2), so that the 4 rows x 64 bytes a half-wave
    // fetches with the transposing read cover all banks once.
    const int ld_r = lane >> 4, ld_u = lane & 15;
    uint32_t koff[LPT], voff[LPT];   // byte offset of this lane's 16 bytes from the first row of a tile
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int row = (wave * LPT + i) * 4 + ld_r;
        koff[i] = (uint32_t)(row * kv_row_bytes) + ((ld_u ^ (row & 15)) << 4);
        voff[i] = (uint32_t)(row * kv_row_bytes) + ((ld_u ^ ((row & 3) << 2)) << 4);
    }
    const uint32_t lds_wave = (uint32_t)(uintptr_t)lds + wave * (LPT * 1024);
    // The three stages are a ring that runs on from one item to the next: block j of the item in work
    // lives in stage (ring0 + j) % 3, and blocks nblk, nblk+1, ... are blocks 0, 1, ... of the next item.
    auto stage_off = [&](int blk) __attribute__((always_inline)) { return ((blk + ring0) % NSTAGE) * TILE_BYTES; };
    // Global address of the tile that request `blk_req` stands for: a block of this item, or (past its
    // end) a block of the next item if that one is being warmed up; otherwise, and past the end of
    // the next item too, the last block is read again into the (dead) stage the request would have
    // used, so that the number of loads in flight is the same in every iteration.
    auto tile_ptr = [&](int blk_req, bool is_v, int &blk) __attribute__((always_inline)) -> const unsigned char * {
        const unsigned char *g = is_v ? vg : kg;
        blk = min(blk_req, nblk - 1);
        if (blk_req >= nblk && warm_next) {
            g = is_v ? nx_vg : nx_kg;
            blk = min(blk_req - nblk, nx_nblk - 1);
        }
        return g + (size_t)blk * tile_gbytes;
    };
    // General form of a tile request: rows past the end of a partial tile re-read the last row (they
    // are masked later).
    auto issue_tile = [&](int blk_req, bool is_v) __attribute__((always_inline)) {
        int blk;
        const unsigned char *g = tile_ptr(blk_req, is_v, blk);
        const uint32_t lbase = lds_wave + (is_v ? V_BASE : 0) + stage_off(blk_req);
        const bool partial = (blk + 1) * BN > p.Skv;
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            uint32_t o = is_v ? voff[i] : koff[i];
            if (partial) {
                int ln = lane;
                PIN(ln);        // formed here, not kept in a register across the block loop
                const int row = (wave * LPT + i) * 4 + (ln >> 4);
                const int rl = min(row, p.Skv - 1 - blk * BN);
                o = o - (uint32_t)(row * kv_row_bytes) + (uint32_t)(rl * kv_row_bytes);
            }
            lds_dma16(g, o, lbase + i * 1024);
        }
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

    // ---- building blocks
    // S^T = K(stage kb) Q^T alone (prologue).
    auto qk_only = [&](f32x16 (&s)[2], int kb) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[t][r] = 0.0f;
#pragma unroll
        for (int st = 0; st < 8; ++st)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                bf16x8 a = *(const LDS_AS bf16x8 *)(lds + kb + t * 32 * ROW_BYTES + kaddr[st]);
                s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[st], s[t], 0, 0, 0);
            }
    };
    // The 32 MFMAs of one iteration as one software-pipelined sequence: even slots O^T += V^T P^T
    // (V stage vb, P from pb), odd slots snxt = K Q^T (K stage kb), so that two MFMAs accumulating into
    // the same registers are four slots apart; the LDS reads of slot i+MAT_PREFETCH are issued before
    // the MFMA of slot i.  `between(slot)` is called after each MFMA and carries the caller's vector
    // work for that slot (it must not touch pb entries the remaining PV MFMAs still read).
    auto mfma_block = [&](f32x16 (&snxt)[2], int vb, int kb, auto between) __attribute__((always_inline)) {
        constexpr int PREFETCH = MAT_PREFETCH;
        bf16x8 frag[32];
        int va[4], ka[8];      // stage offsets folded into the per-lane bases: every read is base + immediate
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) va[dt] = vaddr[dt] + vb;
#pragma unroll
        for (int st = 0; st < 8; ++st) ka[st] = kaddr[st] + kb;
        auto fetch = [&](int slot) __attribute__((always_inline)) -> bf16x8 {
            const int i = slot >> 1;
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
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int slot = 0; slot < 32; ++slot) {
            if (slot + PREFETCH < 32) frag[slot + PREFETCH] = fetch(slot + PREFETCH);
            const int i = slot >> 1;
            if ((slot & 1) == 0) {
                const int g = i >> 2;         // key group: tile g/2, half g%2
                u32x4 pw = {pb[g >> 1][4 * (g & 1)], pb[g >> 1][4 * (g & 1) + 1],
                            pb[g >> 1][4 * (g & 1) + 2], pb[g >> 1][4 * (g & 1) + 3]};
                acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    frag[slot], __builtin_bit_cast(bf16x8, pw), acc[i & 3], 0, 0, 0);
            } else {
                const int st = i >> 1, t = i & 1;
                if (st == 0) {
                    f32x16 z;
#pragma unroll
                    for (int r = 0; r < 16; ++r) z[r] = 0.0f;
                    snxt[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[slot], qf[st], z, 0, 0, 0);
                } else {
                    snxt[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[slot], qf[st], snxt[t], 0, 0, 0);
                }
            }
            between(slot);
            __builtin_amdgcn_sched_barrier(0);     // keep the slot order exactly as written
        }
    };
    // O^T += V^T P^T alone: the last iteration of an item, when no further scores are wanted.
    auto pv_only = [&](int vb) __attribute__((always_inline)) {
        constexpr int PREFETCH = MAT_PREFETCH;
        bf16x8 frag[16];
        int va[4];
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) va[dt] = vaddr[dt] + vb;
        auto fetch = [&](int i) __attribute__((always_inline)) -> bf16x8 {
            const int ro = (i >> 2) * 16 * ROW_BYTES;
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)(lds + va[i & 3] + ro));
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)(lds + va[i & 3] + (ro + 8 * ROW_BYTES)));
            s16x8 av = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            return __builtin_bit_cast(bf16x8, av);
        };
#pragma unroll
        for (int i = 0; i < PREFETCH; ++i) frag[i] = fetch(i);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (i + PREFETCH < 16) frag[i + PREFETCH] = fetch(i + PREFETCH);
            const int g = i >> 2;
            u32x4 pw = {pb[g >> 1][4 * (g & 1)], pb[g >> 1][4 * (g & 1) + 1],
                        pb[g >> 1][4 * (g & 1) + 2], pb[g >> 1][4 * (g & 1) + 3]};
            acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[i], __builtin_bit_cast(bf16x8, pw), acc[i & 3], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto rescale = [&](float mn, float alpha) __attribute__((always_inline)) {
        m = mn;
        l *= alpha;
        lr *= alpha;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[dt][r] *= alpha;
    };
    // P^T = exp2(S^T * c - m) of an unmasked block into pb; returns this lane's partial row sums: over
    // the unrounded FP32 probabilities, and (through lrs) over the BF16-rounded ones.
    auto probabilities = [&](f32x16 (&s)[2], float &lrs) __attribute__((always_inline)) -> float {
        float ls0 = 0.0f, ls1 = 0.0f, r0 = 0.0f;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][r], p.c, -m));
                const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][r + 1], p.c, -m));
                ls0 += e0;
                ls1 += e1;
                pb[t][r >> 1] = pack_bf16(e0, e1);
                r0 = add_bf16_pair(pb[t][r >> 1], r0);
            }
        lrs = r0;
        return ls0 + ls1;
    };
    // Raise the running maximum to cover the unmasked block in s; rescale the accumulator and row sum.
    // Maximum of the scaled scores of an unmasked block, per query (log2 units).
    auto block_maximum = [&](f32x16 (&s)[2]) __attribute__((always_inline)) -> float {
        float mx = ext3<NEG>(s[0][0], s[0][1], s[0][2]);
#pragma unroll
        for (int i = 3; i < 31; i += 2) mx = ext3<NEG>(mx, s[i >> 4][i & 15], s[(i + 1) >> 4][(i + 1) & 15]);
        mx = ext3<NEG>(mx, s[1][15], s[1][15]);
        return lane32_ext<NEG>(mx) * p.c;
    };
    auto raise_reference = [&](f32x16 (&s)[2]) __attribute__((always_inline)) {
        const float mx = block_maximum(s);
        const float mn = fmaxf(m, mx);
        rescale(mn, __builtin_amdgcn_exp2f(m - mn));
    };
    // Softmax of a block that may hold masked keys (diagonal block, tail block, or a block that lies
    // wholly past this wavefront's rows): key index per register, limit per lane.  Masked keys get
    // P = 0 exactly, whatever the score registers hold.
    auto softmax_masked = [&](f32x16 (&s)[2], int blk) __attribute__((always_inline)) {
        int ln = lane;
        PIN(ln);                // lane-derived values are formed here, not kept across the block loop
        int lim = p.Skv - 1;
        if (CAUSAL) lim = min(lim, q0 + (ln & 31) + off);
        const int kidx = blk * BN + 4 * (ln >> 5);
        constexpr float NONE = NEG ? INFINITY : -INFINITY;      // extreme of no score at all
        float mx = NONE;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = kidx + 32 * t + 8 * (r >> 2) + (r & 3);
                mx = ext2<NEG>(mx, key <= lim ? s[t][r] : NONE);
            }
        mx = lane32_ext<NEG>(mx);
        mx = (mx == NONE) ? -INFINITY : mx * p.c;
        if (__builtin_amdgcn_ballot_w64(mx > m) != 0) {
            const float mn = fmaxf(m, mx);
            rescale(mn, (mn == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m - mn));
        }
        const float mu = (m == -INFINITY) ? 0.0f : m;
        float ls = 0.0f;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const int key = kidx + 32 * t + 8 * (r >> 2) + (r & 3);
                float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][r], p.c, -mu));
                float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][r + 1], p.c, -mu));
                e0 = (key <= lim) ? e0 : 0.0f;
                e1 = (key + 1 <= lim) ? e1 : 0.0f;
                ls += e0 + e1;
                pb[t][r >> 1] = pack_bf16(e0, e1);
                lr = add_bf16_pair(pb[t][r >> 1], lr);
            }
        l += ls;
    };

    // Fast iteration j: MFMAs of PV(j) and S(j+2) interleaved with the softmax of S(j+1) = scur.
    // Softmax is the same against any reference point, so the probabilities are formed against the
    // running maximum as it stands, WITHOUT looking for the block's maximum first.  Only if some lane's
    // partial row sum comes out above P_SUM_LIMIT (or is not a number) did the scores outgrow the
    // reference; then the whole wavefront raises the reference, rescales, and forms the probabilities
    // again.  That branch is wave-uniform and rare: with scores of bounded spread the reference
    // settles after the first blocks.
    // The iteration's four tile requests (K(j+4) from kp into stage kreq, V(j+2) from vp into stage vreq)
    // are spread over the block, one every eight slots, so that the wavefronts' requests do not queue up
    // behind each other in the address unit.
    // s0, s1, s2: stages of blocks j, j+1, j+2 (V is read from s0, K from s2; the requests go to s1 for K
    // and s2 for V).
    // The masked form (diagonal blocks, the partial last block, blocks past the end) does the same with
    // every probability whose key is not valid for the lane's row set to zero, whatever its score
    // register holds; its second pass is the masked softmax, which also copes with a row that has no
    // valid key so far (reference at minus infinity).  It issues no requests: those go through the
    // general form after the block.
    auto fused_iteration = [&](auto masked, f32x16 (&scur)[2], f32x16 (&snxt)[2], int s0, int s1, int s2,
                               const unsigned char *kp, const unsigned char *vp, int blk)
        __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked)::value;
        float ev[32];
        uint32_t pn[16];
        float ls0 = 0.0f, ls1 = 0.0f, lrn = 0.0f;
        const uint32_t klds = lds_wave + s1, vlds = lds_wave + V_BASE + s2;
        int room = 0;       // masked form: key offset c within block blk is valid for this lane's row iff c <= room
        if (MASKED) {
            int ln = lane;
            PIN(ln);
            int lim = p.Skv - 1;
            if (CAUSAL) lim = min(lim, q0 + (ln & 31) + off);
            room = lim - blk * BN - 4 * (ln >> 5);
        }
        // Variants 1..3 look for the block's maximum first (the classic running-maximum form); their
        // masked blocks take the MFMA sequence and the exact masked softmax one after the other.
        if (ATTN_SOFTMAX != 0 && MASKED) {
            mfma_block(snxt, s0, s2, [](int) __attribute__((always_inline)) {});
            softmax_masked(scur, blk);
            return;
        }
        float mref = m;     // reference point of this block's probabilities
        if (ATTN_SOFTMAX != 0) {
            const float mx = block_maximum(scur);
            mref = ATTN_SOFTMAX == 3 ? (mx > m + 8.0f ? mx : m) : fmaxf(m, mx);
        }
        mfma_block(snxt, s0, s2, [&](int slot) __attribute__((always_inline)) {
            // element `slot` of the 32 scores of this lane: exp now, row-sum add one slot later
            ev[slot] = __builtin_amdgcn_exp2f(__builtin_fmaf(scur[slot >> 4][slot & 15], p.c, -mref));
            if (MASKED) {
                const int r = slot & 15;
                ev[slot] = (32 * (slot >> 4) + 8 * (r >> 2) + (r & 3) <= room) ? ev[slot] : 0.0f;
            }
            if (slot >= 1) {
                if ((slot - 1) & 1) { ls1 += ev[slot - 1]; PIN(ls1); } else { ls0 += ev[slot - 1]; PIN(ls0); }
            }
            // BF16 pair k once the PV MFMAs that read the old pb entry k have been issued
            // (entries 4g..4g+3 are read by the even slots 8g..8g+6): pair k goes at slot 2k+9
            if (slot >= 9 && (slot & 1)) {
                const int k = (slot - 9) >> 1;
                pn[k] = pack_bf16(ev[2 * k], ev[2 * k + 1]);
                PIN(pn[k]);
            }
            if (!MASKED) {
                static_assert(LPT == 2, "request slots below are written out for two loads per tile and wavefront");
                if (slot == 4) lds_dma16_imm<0>(kp, koff[0], klds);
                if (slot == 12) lds_dma16_imm<1024>(kp, koff[1], klds);
                if (slot == 20) lds_dma16_imm<0>(vp, voff[0], vlds);
                if (slot == 28) lds_dma16_imm<1024>(vp, voff[1], vlds);
            }
        });
        ls1 += ev[31];
#pragma unroll
        for (int k = 12; k < 16; ++k) pn[k] = pack_bf16(ev[2 * k], ev[2 * k + 1]);
        // The rounded row sum, all 16 dot instructions together after the block's last MFMA: they run on
        // the matrix pipe, and one between two MFMAs stalls both (measured: spread over the slots the
        // loop is 2.5 % slower, placed before the first MFMA of the block 4.5 % slower than here).
#pragma unroll
        for (int k = 0; k < 16; ++k) lrn = add_bf16_pair(pn[k], lrn);
#pragma unroll
        for (int k = 0; k < 16; ++k) pb[k >> 3][k & 7] = pn[k];
        float ls = ls0 + ls1;
        if (ATTN_SOFTMAX != 0) {
            // the accumulator holds P(j) V(j) against the old reference: bring it to the new one
            const float alpha = __builtin_amdgcn_exp2f(m - mref);
            // Variant 1 multiplies every time.  Its test never fails; it stands there because with the 64
            // multiplications in the same basic block as the MFMA sequence the register allocator spills
            // (32 to 100 bytes per lane), and a spill inside this loop is not acceptable (see wait_vmcnt).
            const bool raise = ATTN_SOFTMAX == 1 ? __builtin_amdgcn_ballot_w64(alpha <= 1.0f) != 0
                                                 : __builtin_amdgcn_ballot_w64(mref > m) != 0;
            if (raise) rescale(mref, alpha);
            l += ls;
            lr += lrn;
            return;
        }
        if (__builtin_amdgcn_ballot_w64(!(ls <= P_SUM_LIMIT)) != 0) {
            if (MASKED) {
                softmax_masked(scur, blk);      // adds to l and lr itself
                ls = 0.0f;
                lrn = 0.0f;
            } else {
                raise_reference(scur);
                ls = probabilities(scur, lrn);
            }
        }
        l += ls;
        lr += lrn;
    };
    auto fast_iteration = [&](f32x16 (&scur)[2], f32x16 (&snxt)[2], int s0, int s1, int s2,
                              const unsigned char *kp, const unsigned char *vp) __attribute__((always_inline)) {
        fused_iteration(std::false_type{}, scur, snxt, s0, s1, s2, kp, vp, 0);
    };
    // General iteration j, unless block j (and with it every later block) is wholly masked for this
    // wavefront: the MFMAs of PV(j) and S(j+2) with the masked softmax of S(j+1) between them.
    auto general_iteration = [&](f32x16 (&scur)[2], f32x16 (&snxt)[2], int j) __attribute__((always_inline)) {
        if (j < n_w)
            fused_iteration(std::true_type{}, scur, snxt, stage_off(j), 0, stage_off(j + 2), nullptr, nullptr, j + 1);
    };

    // ---- the workgroup's items, one after the other
    int r = 0, grp = 0, tile = 0;
    bool have = find_item(r, grp, tile);
    Geo cur = {};
    if (have) {
        cur = geometry(grp, tile);
        load_q(cur);
    }
    bool warm = false;          // the first tiles of the item about to start were requested by the item before it
#ifdef ATTN_CLOCKS
    int item_no = 0;
#endif
#if defined(ATTN_CLOCKS) && ATTN_CLOCKS >= 2
    unsigned long long ph[11], ph_prev = 0, ph_item = 0;
#endif
    while (have) {
#if defined(ATTN_CLOCKS) && ATTN_CLOCKS >= 2
#pragma unroll
        for (int k = 0; k < 11; ++k) ph[k] = 0;
        ph_prev = ph_item = phase_now();
#endif
        enter(cur);
        reset_state();
        // the item after this one
        Geo nxt = cur;
        int r2 = r + 1;
        const bool have2 = find_item(r2, grp, tile);
        if (have2) nxt = geometry(grp, tile);
        // Its tiles K'(0..2), V'(0) ride on this item's last iterations (requests K(j+4), V(j+2) of
        // iterations j >= nblk-4), which takes four iterations to host them.
        warm_next = ATTN_ITEM_OVERLAP && have2 && nblk >= 2 + REQ_AHEAD && nxt.nblk > 0;
        nx_nblk = nxt.nblk; nx_kg = nxt.kg; nx_vg = nxt.vg;
        // Its Q goes into this wavefront's LDS region now (the epilogue of the item before is done with
        // it) and into registers when this item's last block is done; being the oldest request of the
        // item, it never holds up a wait for tiles.
        if (ATTN_ITEM_OVERLAP && have2) request_q(nxt);

        if (nblk > 0) {
            // Iteration j reads K(j+2) and V(j) and requests K(j+4) and V(j+2) into the stages of K(j+1)
            // and V(j-1), whose last readers finished before the previous barrier.  It ends by waiting until
            // only those four loads are still in flight, i.e. until K(j+3) and V(j+1) have landed, then the
            // barrier publishes them.
            if (!warm) {
                // Every wavefront is past the last barrier of the item before, so no stage is being read.
                issue_tile(0, false);
                issue_tile(1, false);
                issue_tile(2, false);
                issue_tile(0, true);
                __builtin_amdgcn_s_waitcnt(wait_vmcnt(2 * LPT));   // K(0), K(1) landed
                wg_barrier();
            }
            // warm: K(0), K(1) landed before the last barrier of the item before, and Q is in registers
            ATTN_PHASE(0);
            qk_only(sa, stage_off(0));
            qk_only(sb, stage_off(1));
            ATTN_PHASE(1);
            // P(0).  A first block without masked keys (every one but a causal item's diagonal start or a
            // short tail) takes its maximum as the reference and has nothing to rescale yet; the masked
            // path also handles an empty first block.
            if (n_unm > 0) {
                m = block_maximum(sa);
                l = probabilities(sa, lr);
            } else {
                softmax_masked(sa, 0);
            }
            ATTN_PHASE(2);
            // K(2), V(0) landed: a warm item waited for them before the epilogue of the item before, and
            // what it still has in flight are that epilogue's stores, which nothing here depends on
            if (!warm) __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
            wg_barrier();                                 // and every wavefront is done with K(0), K(1)
            issue_tile(3, false);                         // the requests of "iteration -1"
            issue_tile(1, true);

            // Blocks >= n_unm go through the masked softmax, which yields P = 0 where a key is not valid:
            // blocks masked out entirely for this wavefront, and the blocks past the end that the last
            // iterations multiply from stages that hold other tiles, then contribute nothing, with no
            // branch around the MFMA sequences.  Iteration j: scur = S(j+1) (sb for even j), snxt
            // receives S(j+2).
            int j = 0;
            ATTN_STAMP(0, __builtin_readcyclecounter());
            ATTN_PHASE(3);
            // Iterations j < fast_end take the fast path: S(j+1) needs no mask, and the tiles requested are
            // full ones (past the last block: of the next item, or the last block again).
            int fast_end = all_full ? n_unm - 1 : min(n_unm - 1, nfull - (2 + REQ_AHEAD));
            // Request addresses of the fast loop.  K and V have the same shape, so V's address is K's of
            // two iterations earlier plus the distance between the tensors; K's moves on by one tile per
            // iteration, except at the item's last block (on to block 0 of the next item, or stay) and,
            // if there is no next item, after it (stay).
            const ptrdiff_t dv = (const unsigned char *)p.v - (const unsigned char *)p.k;
            int unused;
            const unsigned char *kp = uniform_ptr(tile_ptr(2 + REQ_AHEAD, false, unused));
            const unsigned char *vp = uniform_ptr(tile_ptr(REQ_AHEAD, true, unused));
            const unsigned char *vp1 = uniform_ptr(tile_ptr(1 + REQ_AHEAD, true, unused));
            int kleft = nblk - 1 - (2 + REQ_AHEAD);      // whole-tile steps left before K's request reaches the last block
            const ptrdiff_t kjump = warm_next ? nx_kg - (kg + (size_t)(nblk - 1) * tile_gbytes) : 0;
            const ptrdiff_t kafter = warm_next ? (ptrdiff_t)tile_gbytes : 0;
            // (written out twice below rather than as a lambda: selecting between captured variables
            // would keep them in memory)
#define ATTN_ADVANCE_REQUESTS()                                                              \
            do {                                                                             \
                ptrdiff_t step = kleft < 0 ? kafter : kjump;                                 \
                step = kleft > 0 ? (ptrdiff_t)tile_gbytes : step;                            \
                vp = vp1;                                                                    \
                vp1 = kp + dv;                                                               \
                kp += step;                                                                  \
                --kleft;                                                                     \
            } while (0)
#define ATTN_FAST(scur, snxt, a0, a1, a2)                                                    \
            do {                                                                             \
                fast_iteration(scur, snxt, a0, a1, a2, kp, vp);                              \
                ATTN_ADVANCE_REQUESTS();                                                     \
                __builtin_amdgcn_s_waitcnt(WAIT_ITER_END);                                   \
                wg_barrier();                                                                \
                ATTN_PHASE(4);                                                               \
                ATTN_PHASE_COUNT(5);                                                         \
            } while (0)
            // The bulk of the fast iterations runs in a loop unrolled six times (two score buffers x three
            // stages), in which every LDS address is a register plus a constant.  That loop wants block j in
            // stage 0; a two-iteration loop with the stages in registers brings j there, and takes what
            // is left afterwards.
            static_assert(NSTAGE == 3, "the unrolled loop below is written for three stages");
            const int j_align = ring0 == 0 ? 0 : 2 * ring0 == 2 ? 2 : 4;     // smallest even j with (ring0 + j) % 3 == 0
#pragma nounroll
            for (int round = 0; round < 2; ++round) {
                const int lim = round == 0 ? min(fast_end, j_align) : fast_end;
                int s0 = stage_off(j), s1 = stage_off(j + 1), s2 = stage_off(j + 2);
#pragma nounroll
                for (; j + 1 < lim; j += 2) {
                    ATTN_FAST(sb, sa, s0, s1, s2);
                    ATTN_FAST(sa, sb, s1, s2, s0);
                    { const int t = s0; s0 = s2; s2 = s1; s1 = t; }
                }
                if (round == 0) {
                    constexpr int T0 = 0, T1 = TILE_BYTES, T2 = 2 * TILE_BYTES;
#pragma nounroll
                    for (; j + 5 < fast_end; j += 6) {
                        ATTN_FAST(sb, sa, T0, T1, T2);
                        ATTN_FAST(sa, sb, T1, T2, T0);
                        ATTN_FAST(sb, sa, T2, T0, T1);
                        ATTN_FAST(sa, sb, T0, T1, T2);
                        ATTN_FAST(sb, sa, T1, T2, T0);
                        ATTN_FAST(sa, sb, T2, T0, T1);
                    }
                }
            }
            // an item without masks whose last fast iteration is left over by the loops of two
            if (j == nblk - 2 && fast_end == nblk - 1) {
                ATTN_FAST(sb, sa, stage_off(j), stage_off(j + 1), stage_off(j + 2));
                ++j;
            }
#undef ATTN_FAST
#undef ATTN_ADVANCE_REQUESTS
            // The last iteration of an item that warms up the next one requests nothing (K'(3) would
            // land in the stage of K'(0), which is read only after this item's last barrier).
            auto iteration_end = [&](int jj) __attribute__((always_inline)) {
                if (!(warm_next && jj == nblk - 1)) {
                    issue_tile(jj + 2 + REQ_AHEAD, false);
                    issue_tile(jj + REQ_AHEAD, true);
                }
                __builtin_amdgcn_s_waitcnt(WAIT_ITER_END);
                wg_barrier();
                if (jj == nblk - 1) {
                    ATTN_PHASE(8);
                } else {
                    ATTN_PHASE(6);
                    ATTN_PHASE_COUNT(7);
                }
            };
#pragma nounroll
            for (; j < nblk - 1; j += 2) {
                general_iteration(sb, sa, j);
                iteration_end(j);
                if (j + 1 < nblk - 1) {
                    general_iteration(sa, sb, j + 1);
                    iteration_end(j + 1);
                }
            }
            // the last iteration has only its PV product left to do
            if (nblk - 1 < n_w) pv_only(stage_off(nblk - 1));
            iteration_end(nblk - 1);
            ATTN_STAMP(1, __builtin_readcyclecounter());
            ATTN_STAMP(2, (unsigned long long)nblk);
        }
        // Nothing may still be writing LDS at exit; the next item's Q has landed; and its K'(2), V'(0) are
        // waited for here, before the epilogue's stores join the queue, so that its first barrier can
        // publish them.
        __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
        ATTN_PHASE(9);

        // ---- Q of the next item into registers, from this wavefront's LDS region
        if (ATTN_ITEM_OVERLAP && have2) {
#pragma unroll
            for (int s = 0; s < 8; ++s)
                qf[s] = *(const LDS_AS bf16x8 *)(lds + Q_BASE + wave * Q_WAVE_BYTES + kaddr[s]);
        }
        // ---- epilogue: O = acc / lr (BF16), LSE = ln2 * (m + log2 l).  A lane holds one query's values
        // in pieces of 8 bytes; they go through the same LDS region (32 rows of 256 bytes, 16-byte units
        // swizzled by the row), so that each store instruction writes whole rows.
        const float lt = lane32_sum(l);
        const float lrt = lane32_sum(lr);
        const float inv = lrt > 0.0f ? 1.0f / lrt : 0.0f;
        {
            const int ob = Q_BASE + wave * Q_WAVE_BYTES;
            int ln = lane;
            PIN(ln);        // per-lane offsets are formed here, not kept in registers across the block loop
            const int orow = ln >> 4, ounit = ln & 15, l32 = ln & 31, hh = ln >> 5;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    u32x2 ww = {pack_bf16(acc[dt][4 * rg] * inv, acc[dt][4 * rg + 1] * inv),
                                pack_bf16(acc[dt][4 * rg + 2] * inv, acc[dt][4 * rg + 3] * inv)};
                    *(LDS_AS u32x2 *)(lds + ob + l32 * ROW_BYTES + (((4 * dt + rg) ^ (l32 & 15)) << 4) + 8 * hh) = ww;
                }
            const int Sq = cold().shape.Sq, Hq = cold().shape.Hq;
            const size_t o_row_bytes = (size_t)Hq * HD * 2;
            unsigned char *og = (unsigned char *)(cold().o + ((size_t)((size_t)b * Sq + q0) * Hq + head) * HD);
            const int rows = Sq - q0;               // rows of this wavefront that exist
            // (the row pitch is below 2^23 bytes, so the lane's first offset fits 32 bits; the rest are additions)
            unsigned char *gp = og + ((uint32_t)orow * (uint32_t)o_row_bytes + 16u * (uint32_t)ounit);
            const size_t gstep = 4 * o_row_bytes;
            if (rows >= 32) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int row = 4 * i + orow;
                    const u32x4 val = *(const LDS_AS u32x4 *)(lds + ob + row * ROW_BYTES + ((ounit ^ (row & 15)) << 4));
                    *(u32x4 *)gp = val;
                    gp += gstep;
                }
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int row = 4 * i + orow;
                    const u32x4 val = *(const LDS_AS u32x4 *)(lds + ob + row * ROW_BYTES + ((ounit ^ (row & 15)) << 4));
                    if (row < rows) *(u32x4 *)gp = val;
                    gp += gstep;
                }
            }
            if (l32 < rows && hh == 0) {
                const float lse = lt > 0.0f ? (m + __builtin_amdgcn_logf(lt)) * 0.6931471805599453f : -INFINITY;
                cold().lse[((size_t)b * Hq + head) * Sq + q0 + l32] = lse;
            }
        }

        if (!ATTN_ITEM_OVERLAP && have2) load_q(nxt);
#if defined(ATTN_CLOCKS) && ATTN_CLOCKS >= 2
        ATTN_PHASE(10);
        if (bid == 0 && item_no == 1 && (tid == 0 || tid == NTHREADS - 64)) {
#pragma unroll
            for (int k = 0; k < 11; ++k) g_phases[tid != 0][k] = ph[k];
            g_phases[tid != 0][11] = ph_prev - ph_item;
        }
#endif
#ifdef ATTN_CLOCKS
        ++item_no;
#endif
        ring0 = (ring0 + nblk) % NSTAGE;
        warm = warm_next;
        have = have2;
        r = r2;
        cur = nxt;
    }
#ifdef ATTN_CLOCKS
    if (bid == 0 && tid == 0) { g_clocks[1] = __builtin_readcyclecounter(); g_clocks[3] = wall_clock64(); }
#endif
}

// ---------------------------------------------------------------------------------------------------
// The kernel for small problems.  With 256 query rows per work item a short query sequence (or few
// heads) leaves most compute units without work, however long the key sequence is.  Here a work item
// is 32 query rows that share a K/V head -- PACK query heads of one group x 32/PACK positions, so that
// grouped-query heads share the K/V blocks here too -- and the eight wavefronts of the workgroup share its
// KEYS instead of its rows: wavefront w takes the 32-key blocks w, w + 8, ... with a running maximum and running
// sums of its own (the same online softmax, paper section 2.2), staging its K and V blocks through a
// private 16 KiB of LDS, and the eight partial results are merged through LDS at the end:
//     M = max_w m_w,  f_w = 2^(m_w - M),  O = sum_w f_w acc_w / sum_w f_w lr_w,  LSE = ln2 (M + log2 sum_w f_w l_w).
// No barrier inside the key loop, no workspace in device memory.
struct SplitParams {
    const __bf16 *q, *k, *v;
    __bf16 *o;
    float *lse;
    int Hq, Hkv, Sq, Skv, G;
    int pack, pack_log2;    // query heads of one K/V group in a work item (8, 4, 2 or 1); row r is head r % pack, position r / pack
    int chunks;             // G / pack
    int tile_pos;           // query positions per work item = 32 / pack
    int ntile;              // ceil(Sq / tile_pos)
    Div d_ntile, d_chunks, d_hkv;   // exact division by ntile, chunks, Hkv
    float c;                // scale * log2(e)
};
constexpr int SPLIT_KEYS = 32;                                  // keys per block of the split kernel
constexpr int SPLIT_TILE_BYTES = SPLIT_KEYS * ROW_BYTES;        // 8 KiB: one K or V block
constexpr int SPLIT_WAVE_BYTES = 2 * SPLIT_TILE_BYTES;          // per wavefront: its K block, then its V block
constexpr int SPLIT_STATE_BASE = NWAVES * SPLIT_WAVE_BYTES;     // after them: m, l, lr of every wavefront
constexpr int SPLIT_Q_BASE = SPLIT_STATE_BASE + NWAVES * 3 * 32 * 4;   // then the item's 32 Q rows (K's swizzle)
constexpr int SPLIT_LDS_BYTES = SPLIT_Q_BASE + 32 * ROW_BYTES;
static_assert(SPLIT_Q_BASE % 1024 == 0 && NWAVES * 4 == 32, "each wavefront requests four of the 32 Q rows, 1 KiB");
static_assert(SPLIT_WAVE_BYTES == 32 * HD * 4, "a wavefront's partial accumulator takes the place of its two blocks");
static_assert(SPLIT_LDS_BYTES <= LDS_BYTES, "the split kernel is launched with the same dynamic LDS size");

template <bool CAUSAL, bool NEG>
__global__ __launch_bounds__(NTHREADS) void attn_fwd_split_kernel(const SplitParams p)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    LDS_AS unsigned char *lds = (LDS_AS unsigned char *)smem;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hh = lane >> 5;
    const int item = blockIdx.x;
#ifdef ATTN_CLOCKS
    if (item == 0 && tid == 0) { g_clocks[2] = wall_clock64(); g_clocks[0] = __builtin_readcyclecounter(); }
#endif
    const int rest = fast_div(item, p.d_ntile), tile = item - rest * p.ntile;
    const int bh = fast_div(rest, p.d_chunks), chunk = rest - bh * p.chunks;
    const int b = fast_div(bh, p.d_hkv), hkv = bh - b * p.Hkv;
    const int q0 = tile * p.tile_pos;
    // this lane's query: head and position (rows past the end of Q compute on the last row and are not stored)
    const int head = hkv * p.G + chunk * p.pack + (l32 & (p.pack - 1));
    const int qpos = q0 + (l32 >> p.pack_log2);
    const int off = p.Skv - p.Sq;
    // keys 0 .. klast are valid for some row of the tile
    int klast = p.Skv - 1;
    if (CAUSAL) klast = min(klast, min(q0 + p.tile_pos - 1, p.Sq - 1) + off);
    const int nb = klast < 0 ? 0 : klast / SPLIT_KEYS + 1;
    const size_t kv_row_bytes = (size_t)p.Hkv * HD * 2;
    const unsigned char *kg = (const unsigned char *)(p.k + ((size_t)b * p.Skv * p.Hkv + hkv) * HD);
    const unsigned char *vg = (const unsigned char *)(p.v + ((size_t)b * p.Skv * p.Hkv + hkv) * HD);

    const uint32_t kbase = wave * SPLIT_WAVE_BYTES, vbase = kbase + SPLIT_TILE_BYTES;
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    // One block = 8 requests of 1 KiB (4 rows): lane L's 16 bytes land at base + 16 L, and the lane
    // fetches the logical 16-byte unit that the swizzle of the main kernel puts there.
    uint32_t koff[8], voff[8];      // byte offset of this lane's 16 bytes from the first row of a full block
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = 4 * i + (lane >> 4), unit = lane & 15;
        koff[i] = (uint32_t)(row * kv_row_bytes) + ((unit ^ (row & 15)) << 4);
        voff[i] = (uint32_t)(row * kv_row_bytes) + ((unit ^ ((row & 3) << 2)) << 4);
    }
    auto request = [&](int blk, bool is_v) __attribute__((always_inline)) {
        const unsigned char *g = uniform_ptr((is_v ? vg : kg) + (size_t)blk * SPLIT_KEYS * kv_row_bytes);
        const int last = p.Skv - 1 - blk * SPLIT_KEYS;      // rows past the end of K/V re-read the last row
        const uint32_t dst = lds0 + (is_v ? vbase : kbase);
        if (last >= SPLIT_KEYS - 1) {
#pragma unroll
            for (int i = 0; i < 8; ++i) lds_dma16(g, is_v ? voff[i] : koff[i], dst + i * 1024);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int row = 4 * i + (lane >> 4);
                const uint32_t o = (is_v ? voff[i] : koff[i]) - (uint32_t)(row * kv_row_bytes) + (uint32_t)(min(row, last) * kv_row_bytes);
                lds_dma16(g, o, dst + i * 1024);
            }
        }
    };
    // What the first MFMA needs goes out first, and before anything else is computed: the eight wavefronts'
    // first blocks are 128 KiB through a load path of 64 bytes a clock, the longest single stretch of a
    // small launch.  The item's 32 Q rows go through LDS as well, each wavefront requesting four of them
    // (rows past the end re-read the last row): fetched by every wavefront for itself they would be
    // another 64 KiB on that path, and as ordinary loads they would make the compiler's own count of
    // outstanding loads, which knows nothing of the requests around them, wait for V before the first MFMA.
    {
        const int r = 4 * wave + (lane >> 4), unit = lane & 15;
        const int row0 = min(q0, p.Sq - 1);
        const int drow = min(q0 + (r >> p.pack_log2), p.Sq - 1) - row0;         // 0 .. 31
        const int dhead = r & (p.pack - 1);
        const unsigned char *qg = (const unsigned char *)(p.q + ((size_t)((size_t)b * p.Sq + row0) * p.Hq + hkv * p.G + chunk * p.pack) * HD);
        // (at most 32 rows of at most 32768 heads of 256 bytes: the offset fits 32 bits)
        const uint32_t o = (uint32_t)(drow * p.Hq + dhead) * (uint32_t)(HD * 2) + ((unit ^ (r & 15)) << 4);
        lds_dma16(qg, o, lds0 + SPLIT_Q_BASE + wave * 1024);
    }
    int t = wave;
    if (t < nb) {
        request(t, false);
        request(t, true);
    }
    __builtin_amdgcn_sched_barrier(0);
    f32x16 acc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[dt][r] = 0.0f;
    float m = -INFINITY, l = 0.0f, lr = 0.0f;
    int kaddr[8];
#pragma unroll
    for (int st = 0; st < 8; ++st) kaddr[st] = kbase + l32 * ROW_BYTES + (((2 * st + hh) ^ (l32 & 15)) << 4);
    int vaddr[4];
    {
        const int i16 = lane & 15, g = (lane >> 4) & 1;
        const int row = 4 * hh + (i16 >> 2);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            const int d = 32 * dt + 16 * g + 4 * (i16 & 3);
            vaddr[dt] = vbase + row * ROW_BYTES + ((((d >> 3) ^ ((row & 3) << 2))) << 4) + (d & 7) * 2;
        }
    }

    // this wavefront's Q rows have landed (and K(t), if it has a block: both are older than V(t)'s
    // eight requests); the barrier publishes all 32 rows
    if (t < nb) __builtin_amdgcn_s_waitcnt(wait_vmcnt(8)); else __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
    wg_barrier();
    bf16x8 qf[8];           // Q^T operand: query l32, d = 16 s + 8 hh .. + 7
#pragma unroll
    for (int s = 0; s < 8; ++s)
        qf[s] = *(const LDS_AS bf16x8 *)(lds + SPLIT_Q_BASE + l32 * ROW_BYTES + (((2 * s + hh) ^ (l32 & 15)) << 4));

    // Blocks wave, wave + 8, ...: K(t) and V(t) were requested above (this wavefront's first block); K(t + 8) goes out as soon as the
    // score MFMAs have read K(t), V(t + 8) as soon as the PV MFMAs have read V(t), so that a wait is "all
    // but the newest eight requests have landed" while there is a next block and "all" at the last one.
    for (; t < nb; t += NWAVES) {
        const bool more = t + NWAVES < nb;
        __builtin_amdgcn_s_waitcnt(wait_vmcnt(8));          // K(t) has landed
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.0f;
#pragma unroll
        for (int st = 0; st < 8; ++st) {
            bf16x8 a = *(const LDS_AS bf16x8 *)(lds + kaddr[st]);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[st], s, 0, 0, 0);
        }
        // (the MFMAs above hold K(t) in registers: the compiler has waited for the LDS reads)
        __builtin_amdgcn_sched_barrier(0);
        if (more) request(t + NWAVES, false);
        // exact online softmax of the block, masked per key
        int lim = p.Skv - 1;
        if (CAUSAL) lim = min(lim, qpos + off);
        const int kidx = t * SPLIT_KEYS + 4 * hh;
        constexpr float NONE = NEG ? INFINITY : -INFINITY;
        float mx = NONE;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = kidx + 8 * (r >> 2) + (r & 3);
            mx = ext2<NEG>(mx, key <= lim ? s[r] : NONE);
        }
        mx = lane32_ext<NEG>(mx);
        mx = (mx == NONE) ? -INFINITY : mx * p.c;
        if (__builtin_amdgcn_ballot_w64(mx > m) != 0) {
            const float mn = fmaxf(m, mx);
            const float alpha = (mn == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m - mn);
            m = mn;
            l *= alpha;
            lr *= alpha;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[dt][r] *= alpha;
        }
        const float mu = (m == -INFINITY) ? 0.0f : m;
        uint32_t pb[8];
        float ls = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const int key = kidx + 8 * (r >> 2) + (r & 3);
            float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], p.c, -mu));
            float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r + 1], p.c, -mu));
            e0 = (key <= lim) ? e0 : 0.0f;
            e1 = (key + 1 <= lim) ? e1 : 0.0f;
            ls += e0 + e1;
            pb[r >> 1] = pack_bf16(e0, e1);
            lr = add_bf16_pair(pb[r >> 1], lr);
        }
        l += ls;
        // V(t) has landed: behind it in the queue are the requests of K(t + 8), if there is such a block
        if (more) __builtin_amdgcn_s_waitcnt(wait_vmcnt(8)); else __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            u32x4 pw = {pb[4 * g], pb[4 * g + 1], pb[4 * g + 2], pb[4 * g + 3]};
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                const int ro = g * 16 * ROW_BYTES;
                s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)(lds + vaddr[dt] + ro));
                s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)(lds + vaddr[dt] + (ro + 8 * ROW_BYTES)));
                s16x8 av = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av),
                                                                   __builtin_bit_cast(bf16x8, pw), acc[dt], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (more) request(t + NWAVES, true);
    }
    // nothing of this wavefront's is still on its way into LDS (the last block waited for everything),
    // and its MFMAs have read their operands
    __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);

    // ---- merge.  Each wavefront leaves its accumulator as FP32 [query][d] in its own 16 KiB (its blocks
    // are dead), the 16-byte units of a query's row swizzled by the query so that the 32 lanes of a
    // store or load touch 32 different units, and its m, l, lr in the state area; wavefront w then
    // combines d = 16 w .. 16 w + 15.
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    {
        LDS_AS unsigned char *part = lds + wave * SPLIT_WAVE_BYTES + l32 * (HD * 4);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int u = 8 * dt + 2 * rg + hh;          // d = 4 u .. 4 u + 3
                const f32x4 val = {acc[dt][4 * rg], acc[dt][4 * rg + 1], acc[dt][4 * rg + 2], acc[dt][4 * rg + 3]};
                *(LDS_AS f32x4 *)(part + ((u ^ l32) << 4)) = val;
            }
        // every lane of a query holds the same m; l and lr are the lane's share: add the two halves
        const float lt = lane32_sum(l), lrt = lane32_sum(lr);
        LDS_AS float *state = (LDS_AS float *)(lds + SPLIT_STATE_BASE) + wave * 96;
        if (hh == 0) {
            state[l32] = m;
            state[32 + l32] = lt;
            state[64 + l32] = lrt;
        }
    }
    __syncthreads();
    {
        const LDS_AS float *state = (const LDS_AS float *)(lds + SPLIT_STATE_BASE);
        float mw[NWAVES], M = -INFINITY;
#pragma unroll
        for (int w = 0; w < NWAVES; ++w) {
            mw[w] = state[w * 96 + l32];
            M = fmaxf(M, mw[w]);
        }
        float L = 0.0f, LR = 0.0f, o8[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) o8[j] = 0.0f;
#pragma unroll
        for (int w = 0; w < NWAVES; ++w) {
            const float f = (mw[w] == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(mw[w] - M);
            L += f * state[w * 96 + 32 + l32];
            LR += f * state[w * 96 + 64 + l32];
            const LDS_AS unsigned char *part = lds + w * SPLIT_WAVE_BYTES + l32 * (HD * 4);
            const int u = 4 * wave + 2 * hh;
            const f32x4 lo = *(const LDS_AS f32x4 *)(part + ((u ^ l32) << 4));
            const f32x4 hi = *(const LDS_AS f32x4 *)(part + (((u + 1) ^ l32) << 4));
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                o8[j] += f * lo[j];
                o8[4 + j] += f * hi[j];
            }
        }
        const float inv = LR > 0.0f ? 1.0f / LR : 0.0f;
        if (qpos < p.Sq) {
            u32x4 ww = {pack_bf16(o8[0] * inv, o8[1] * inv), pack_bf16(o8[2] * inv, o8[3] * inv),
                        pack_bf16(o8[4] * inv, o8[5] * inv), pack_bf16(o8[6] * inv, o8[7] * inv)};
            __bf16 *op = p.o + ((size_t)((size_t)b * p.Sq + qpos) * p.Hq + head) * HD + 16 * wave + 8 * hh;
            *(u32x4 *)op = ww;
            if (wave == 0 && hh == 0)
                p.lse[((size_t)b * p.Hq + head) * p.Sq + qpos] =
                    L > 0.0f ? (M + __builtin_amdgcn_logf(L)) * 0.6931471805599453f : -INFINITY;
        }
    }
#ifdef ATTN_CLOCKS
    if (item == 0 && tid == 0) { g_clocks[1] = __builtin_readcyclecounter(); g_clocks[3] = wall_clock64(); }
#endif
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
    if (!isfinite(scale)) return ATTN_E_SCALE;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15) return ATTN_E_ALIGN;
    if ((uintptr_t)lse & 3) return ATTN_E_ALIGN;

    Params p = {};
    p.q = (const __bf16 *)q; p.k = (const __bf16 *)k; p.v = (const __bf16 *)v;
    p.o = (__bf16 *)o; p.lse = lse;
    p.Hkv = Hkv; p.Skv = Skv;
    p.c = scale * 1.4426950408889634f;
    Shape &sh = p.shape;
    Sched &sc = p.sched;
    sh.Sq = Sq; sh.Hq = Hq;
    sh.G = Hq / Hkv;
    sh.pack = (sh.G % 8 == 0) ? 8 : (sh.G % 4 == 0) ? 4 : (sh.G % 2 == 0) ? 2 : 1;
    sh.pack_log2 = sh.pack == 8 ? 3 : sh.pack == 4 ? 2 : sh.pack == 2 ? 1 : 0;
    sh.tile_pos = WG_ROWS / sh.pack;
    sh.chunks = sh.G / sh.pack;
    sh.d_chunks = make_div((uint32_t)sh.chunks);
    sh.d_hkv = make_div((uint32_t)Hkv);
    sc.ntile = (Sq + sh.tile_pos - 1) / sh.tile_pos;
    // Key/query indices and the work-item count are 32-bit in the kernel (and below 2^31 for the divisions).
    if ((int64_t)Sq + Skv + WG_ROWS + 8 * BN >= INT32_MAX) return ATTN_E_UNSUPPORTED;
    // Byte offsets within one tile (rows x row pitch) are 32-bit in the kernel.
    if (Hq > 32768 || Hkv > 32768) return ATTN_E_UNSUPPORTED;
    const int64_t total = (int64_t)B * Hkv * sh.chunks * sc.ntile;
    if (total + 8 >= INT32_MAX / 16) return ATTN_E_UNSUPPORTED;
    sc.total = (int)total;

    // Once per device: the CU count, and the opt-in that 160 KiB of dynamic LDS needs.
    static std::atomic<int> cus[64];          // zero-initialised; threads that race here store the same value
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return ATTN_E_LAUNCH;
    if (!cus[dev].load(std::memory_order_acquire)) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0 ||
            hipFuncSetAttribute((const void *)attn_fwd_kernel<true, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess ||
            hipFuncSetAttribute((const void *)attn_fwd_kernel<false, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess ||
            hipFuncSetAttribute((const void *)attn_fwd_kernel<true, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess ||
            hipFuncSetAttribute((const void *)attn_fwd_kernel<false, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess ||
            hipFuncSetAttribute((const void *)attn_fwd_split_kernel<true, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, SPLIT_LDS_BYTES) != hipSuccess ||
            hipFuncSetAttribute((const void *)attn_fwd_split_kernel<false, false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, SPLIT_LDS_BYTES) != hipSuccess ||
            hipFuncSetAttribute((const void *)attn_fwd_split_kernel<true, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, SPLIT_LDS_BYTES) != hipSuccess ||
            hipFuncSetAttribute((const void *)attn_fwd_split_kernel<false, true>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, SPLIT_LDS_BYTES) != hipSuccess)
            return ATTN_E_LAUNCH;
        cus[dev].store(n, std::memory_order_release);
    }
    const int ncu = cus[dev].load(std::memory_order_relaxed);
    hipStream_t st = (hipStream_t)stream;
    // a negative scale turns the running maximum of the scaled scores into c times the smallest raw score
    const bool neg = scale < 0.0f;

    // Small problems: few 256-row items would leave most compute units idle; 32-row items whose keys
    // are shared out among the wavefronts of a workgroup fill the device instead.
    const int split_tile_pos = 32 / sh.pack;
    const int64_t split_items = (int64_t)B * Hkv * sh.chunks * ((Sq + split_tile_pos - 1) / split_tile_pos);
    const bool small = ATTN_SMALL_PATH == 2 || (ATTN_SMALL_PATH == 1 && total * 4 <= ncu);
    if (small && split_items < INT32_MAX) {
        SplitParams sp = {};
        sp.q = p.q; sp.k = p.k; sp.v = p.v; sp.o = p.o; sp.lse = lse;
        sp.Hq = Hq; sp.Hkv = Hkv; sp.Sq = Sq; sp.Skv = Skv; sp.G = sh.G;
        sp.pack = sh.pack; sp.pack_log2 = sh.pack_log2; sp.chunks = sh.chunks;
        sp.tile_pos = split_tile_pos;
        sp.ntile = (Sq + split_tile_pos - 1) / split_tile_pos;
        sp.d_ntile = make_div((uint32_t)sp.ntile);
        sp.d_chunks = make_div((uint32_t)sp.chunks);
        sp.d_hkv = make_div((uint32_t)Hkv);
        sp.c = p.c;
        const dim3 sgrid((unsigned)split_items), sblock(NTHREADS);
        if (causal && neg)
            hipLaunchKernelGGL((attn_fwd_split_kernel<true, true>), sgrid, sblock, SPLIT_LDS_BYTES, st, sp);
        else if (causal)
            hipLaunchKernelGGL((attn_fwd_split_kernel<true, false>), sgrid, sblock, SPLIT_LDS_BYTES, st, sp);
        else if (neg)
            hipLaunchKernelGGL((attn_fwd_split_kernel<false, true>), sgrid, sblock, SPLIT_LDS_BYTES, st, sp);
        else
            hipLaunchKernelGGL((attn_fwd_split_kernel<false, false>), sgrid, sblock, SPLIT_LDS_BYTES, st, sp);
        return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_E_LAUNCH;
    }

    // One workgroup per CU (a workgroup takes all of a CU's registers and LDS), each working through a list.
    const int cu_slots = ncu >= 8 ? ncu / 8 : 1;
    sc.per_xcd = (int)((total + 7) / 8);
    sc.split = sc.nsub = sc.sgx = sc.window = 1;
    sc.split_log2 = 0;
    if (causal) {
        const int64_t groups = (int64_t)B * Hkv * sh.chunks;
        while ((groups * sc.split) % 8 != 0) { sc.split *= 2; ++sc.split_log2; }    // 1, 2, 4 or 8
        sc.nsub = (sc.ntile + sc.split - 1) / sc.split;
        sc.sgx = (int)(groups * sc.split / 8);
        while (sc.window * 2 <= sc.sgx && sc.window * sc.nsub < cu_slots) sc.window *= 2;
        sc.per_xcd = sc.sgx * sc.nsub;          // <= total + padding, far below 2^31 after the check above
    }
    sc.per_win = sc.window * sc.nsub;
    sc.d_ntile = make_div((uint32_t)sc.ntile);
    sc.d_per_win = make_div((uint32_t)sc.per_win);
    sc.d_window = make_div((uint32_t)sc.window);
    sc.slots = sc.per_xcd < cu_slots ? sc.per_xcd : cu_slots;
    const dim3 grid((unsigned)(sc.slots * 8)), block(NTHREADS);
    if (causal && neg)
        hipLaunchKernelGGL((attn_fwd_kernel<true, true>), grid, block, LDS_BYTES, st, p);
    else if (causal)
        hipLaunchKernelGGL((attn_fwd_kernel<true, false>), grid, block, LDS_BYTES, st, p);
    else if (neg)
        hipLaunchKernelGGL((attn_fwd_kernel<false, true>), grid, block, LDS_BYTES, st, p);
    else
        hipLaunchKernelGGL((attn_fwd_kernel<false, false>), grid, block, LDS_BYTES, st, p);
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
    case ATTN_E_SCALE:       return "scale must be finite";
    case ATTN_E_LAUNCH:      return "kernel launch failed";
    default:                 return "unknown attn error code";
    }
}

int attn_version(void) { return 1001; }

#ifdef ATTN_CLOCKS
// Waits for the device, then copies the stamps of the last launch to the host (10 x 64-bit).
int attn_clocks_read(unsigned long long *out)
{
    if (!out) return ATTN_E_NULL;
    return hipMemcpyFromSymbol(out, HIP_SYMBOL(g_clocks), sizeof(g_clocks)) == hipSuccess ? ATTN_OK : ATTN_E_LAUNCH;
}
#if ATTN_CLOCKS >= 2
// Waits for the device, then copies the phase sums of the last launch to the host (2 x 12 x 64-bit).
int attn_phases_read(unsigned long long *out)
{
    if (!out) return ATTN_E_NULL;
    return hipMemcpyFromSymbol(out, HIP_SYMBOL(g_phases), sizeof(g_phases)) == hipSuccess ? ATTN_OK : ATTN_E_LAUNCH;
}
#endif
#endif

}  // extern "C"
