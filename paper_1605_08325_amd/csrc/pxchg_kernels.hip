// gfx950 kernels of libpxchg and the C-ABI calls that launch them.
//
// Every operation here is element-wise over a parameter set that is scattered
// over many separately allocated tensors, and every one is bound by HBM
// bandwidth (a handful of flops per 18..48 bytes moved).  So the design is about
// memory traffic only:
//   * one launch per call: workgroups walk a device-resident list of chunks
//     (tensor, start, length), so 16 tensors or 116 cost the same single launch;
//   * lanes move 16-byte vectors (8-byte ones for binary16 next to float32
//     operands) in one of three lane layouts, all of which make every memory
//     instruction of a wavefront cover one contiguous stretch, and issue all
//     loads of a step before the first use (k x 16 bytes in flight per lane);
//   * no LDS staging and no cross-lane traffic in the exchange kernels: lanes are
//     independent, which also makes the fixed worker order of the sum trivially
//     bit-exact (only the diagnostics kernel reduces across lanes);
//   * nothing is reused inside one launch, so loads carry the non-temporal hint
//     and stores a per-kernel streaming policy, both chosen by measurement.
// There is no matrix-core work here on purpose: there is no contraction.
//
// Floating point: compiled with -ffp-contract=off and `fp contract(off)` below,
// so every product and sum is rounded to binary32 on its own, exactly as the
// definition of each operation in pxchg.h states.  binary32 -> binary16 uses the
// hardware convert under the default round-to-nearest-even mode with binary16
// denormals enabled; the packed round-toward-zero convert is never used.
#include <atomic>
#include <shared_mutex>
#include <tuple>
#include <type_traits>

#include "pxchg_internal.h"

#pragma clang fp contract(off)

namespace {

// A workgroup takes one 512-element chunk (or half of one, in the kernels that
// run two workgroups per chunk: see take_part), and every memory instruction of a
// wavefront covers one contiguous stretch (1 KiB for 16-byte lanes).  Three lane
// layouts do that, chosen per kernel by measurement on MI355X (the rule of thumb
// behind the choices: a wavefront should have 2..4 KiB of loads in flight, and
// binary16 accesses of at least 8 bytes where binary16 is all the traffic):
//   * the binary16 reduce of one to three workers and the diagnostics of a
//     binary16 buffer: lane l of a wavefront owns elements 8l..8l+7 (one 16-byte
//     access per operand);
//   * pack, unpack, the reduces with float32 on one side and the float32 reduce
//     of up to three workers: one wavefront in the SPLIT layout, lane l owns
//     4l..4l+3 and 256+4l..256+4l+3 (float32 as two 16-byte accesses 1 KiB
//     apart, binary16 as two 8-byte accesses);
//   * everything else: 128, 256 or 512 lanes per chunk, lane l owning 4, 2 or 1
//     consecutive elements.  Four elements for the in-place float32 kernels with
//     few operands (momentum update, one elastic meeting: +3.5 % and +6 % against
//     the split layout) and the binary16 reduce of four or more workers (+5 %);
//     narrower lanes the more operands a step has (fused reduce+update, fused
//     elastic round, float32 reduce of four or more workers: see reduce_lanes,
//     fused_lanes and elastic_lanes below).
// As many small workgroups as there are chunks keep the window of addresses in
// flight narrow; larger tiles, several steps per lane and persistent grids were
// all measured slower.
template <typename... T>
constexpr bool touches_f32() {
    return (std::is_same<T, float>::value || ...);
}
static_assert(PXCHG_MAX_K <= 64, "the any-k kernel uses one lane per worker to fetch pointers");

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Data pointers come out of pointer tables in memory, so the compiler cannot
// know they are global addresses; say so, to get global (not flat) memory
// instructions.  The pointer tables themselves are read-only for the lifetime
// of a launch and uniform per workgroup: reading them through the constant
// address space turns those reads into scalar loads.
#define PX_GLOBAL __attribute__((address_space(1)))
#define PX_CONST __attribute__((address_space(4)))

template <typename T>
__device__ __forceinline__ T *table_ptr(const void *const *table, int tensor) {
    return (T *)((const void *const PX_CONST *)table)[tensor];
}
template <typename T>
__device__ __forceinline__ T *table_ptr(void *const *table, int tensor) {
    return (T *)((void *const PX_CONST *)table)[tensor];
}

// On tables of many small tensors the reduce fetches its pointers lane-parallel instead: lane i of every wavefront
// reads operand i's pointer for the chunk's tensor with ONE vector load, and the wavefront then reads lanes 0..K
// out.  A workgroup's K + 1 scalar loads become one vector load.  Where the scalar loads miss their cache for most
// chunks (few chunks per tensor) that measured 3..7 % on the reduce: 116 tensors in 7 M elements 25.5 against 26.4
// us, 128 in 13.4 M 44.7 against 46.2, 512 in 7 M 23.7 against 25.1, 2048 in 61 M 177 against 187.  With many chunks
// per tensor it is level or slower (AlexNet shapes 181 against 177, in step 171 against 168; VGGNet shapes in step
// 393 against 382), so the launch picks by the table's average (small_tensors below).  The other kernels
// keep the scalar loads at any tensor count: the same change cost the update 7 %, the meeting 18 %, the fused
// reduce+update 2..6 % and the pack 4 % (the round of 8: level, 5 % faster with 2048 tensors).
// A/B builds: PXCHG_TUNE_REDUCE_POINTERS = 0 (always scalar) or 1 (always lane-parallel).
// (The lane's table is picked with a chain of selects over the kernel's own arguments: an array of tables handed
// to a helper ends up in scratch memory and costs 15..45 %.)
__device__ __forceinline__ uintptr_t table_entry(const void *const *tab, int tensor) {  // a vector load
    return (uintptr_t)((const void *const PX_GLOBAL *)tab)[tensor];
}
template <typename T>
__device__ __forceinline__ T *lane_pointer(uintptr_t mine, int i) {  // lane i's value; i is the same in every lane
    const unsigned lo = __builtin_amdgcn_readlane((unsigned)mine, i);
    const unsigned hi = __builtin_amdgcn_readlane((unsigned)(mine >> 32), i);
    return (T *)(((uintptr_t)hi << 32) | lo);
}

template <int U>
struct FV {
    float v[U];
};

template <int NT, typename V>
__device__ __forceinline__ V ldv(const PX_GLOBAL V *p) {
    if constexpr (NT == 1 || NT == 3 || NT == 4 || NT == 5)
        return __builtin_nontemporal_load(p);
    else
        return *p;
}
// Streaming store with agent scope ("sc1 nt"): measured 1-4 % faster than the plain non-temporal store on the
// kernels that write half of their traffic.  The compiler has no builtin that sets both bits on a 16-byte
// vector store, hence the instruction is written out.  A store of more than 8 bytes reads its data registers
// over several cycles, and this chip family wants TWO wait states before a vector-ALU instruction may overwrite
// them; the compiler inserts those for its own stores but cannot see through inline assembly, hence the
// trailing `s_nop 1` (N + 1 wait states) after the 16-byte form.  (With one wait state a kernel shape tried
// during tuning, six such stores in a row, stored 16 wrong elements in 70,001; no shipped shape did, but that
// was luck.)  The 8-byte form needs none; its `s_nop 0` is a margin.
template <typename V>
__device__ __forceinline__ void store_sc1_nt(PX_GLOBAL V *p, V x) {
    static_assert(sizeof(V) == 16 || sizeof(V) == 8 || sizeof(V) == 4, "dwordx4, dwordx2 or dword");
    if constexpr (sizeof(V) == 16)
        asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"(x) : "memory");
    else if constexpr (sizeof(V) == 8)
        asm volatile("global_store_dwordx2 %0, %1, off sc1 nt\n\ts_nop 0" ::"v"(p), "v"(x) : "memory");
    else
        asm volatile("global_store_dword %0, %1, off sc1 nt" ::"v"(p), "v"(x) : "memory");
}
// Agent-scope store without the streaming hint ("sc1"): measured 3 % faster than a plain store on the reduce
// kernel, whose writes are one byte in nine of its traffic.
template <typename V>
__device__ __forceinline__ void store_sc1(PX_GLOBAL V *p, V x) {
    static_assert(sizeof(V) == 16 || sizeof(V) == 8 || sizeof(V) == 4, "dwordx4, dwordx2 or dword");
    if constexpr (sizeof(V) == 16)
        asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(x) : "memory");
    else if constexpr (sizeof(V) == 8)
        asm volatile("global_store_dwordx2 %0, %1, off sc1\n\ts_nop 0" ::"v"(p), "v"(x) : "memory");
    else
        asm volatile("global_store_dword %0, %1, off sc1" ::"v"(p), "v"(x) : "memory");
}

// NT: 0 plain, bit 0 non-temporal loads, bit 1 non-temporal stores, 4 = non-temporal loads with "sc1 nt" stores,
// 5 = non-temporal loads with "sc1" stores.
template <int NT, typename V>
__device__ __forceinline__ void stv(PX_GLOBAL V *p, V x) {
    if constexpr (NT == 4)
        store_sc1_nt(p, x);
    else if constexpr (NT == 5)
        store_sc1(p, x);
    else if constexpr (NT == 2 || NT == 3)
        __builtin_nontemporal_store(x, p);
    else
        *p = x;
}

// A lane's U elements starting at p, as binary32: U consecutive elements, or (SPLIT, U = 8) elements
// p[0..3] and p[256..259].  p is aligned to the access: 16 bytes, or 8 bytes for four halves.
constexpr int SPLIT_GAP = 256;
template <int NT, int U, bool SPLIT>
__device__ __forceinline__ FV<U> loadv(const float *p) {
    static_assert(U == 1 || U == 2 || U == 4 || U == 8, "4 or 8 bytes, or one or two 16-byte vectors");
    static_assert(!SPLIT || U == 8, "the split layout is two groups of four");
    FV<U> r;
    if constexpr (U == 1) {
        r.v[0] = ldv<NT>((const PX_GLOBAL float *)p);
    } else if constexpr (U == 2) {
        const f32x2 a = ldv<NT>((const PX_GLOBAL f32x2 *)p);
        r.v[0] = a.x; r.v[1] = a.y;
    } else {
        const f32x4 a = ldv<NT>((const PX_GLOBAL f32x4 *)p);
        r.v[0] = a.x; r.v[1] = a.y; r.v[2] = a.z; r.v[3] = a.w;
        if constexpr (U == 8) {
            const f32x4 b = ldv<NT>((const PX_GLOBAL f32x4 *)(p + (SPLIT ? SPLIT_GAP : 4)));
            r.v[4] = b.x; r.v[5] = b.y; r.v[6] = b.z; r.v[7] = b.w;
        }
    }
    return r;
}
template <int NT, int U, bool SPLIT>
__device__ __forceinline__ FV<U> loadv(const _Float16 *p) {
    static_assert(U == 2 || U == 4 || U == 8, "4, 8 or 16 bytes");
    static_assert(!SPLIT || U == 8, "the split layout is two groups of four");
    FV<U> r;
    if constexpr (U == 2) {
        const f16x2 a = ldv<NT>((const PX_GLOBAL f16x2 *)p);
        r.v[0] = (float)a[0]; r.v[1] = (float)a[1];
    } else if constexpr (U == 4 || SPLIT) {
        const f16x4 a = ldv<NT>((const PX_GLOBAL f16x4 *)p);
#pragma unroll
        for (int i = 0; i < 4; ++i) r.v[i] = (float)a[i];  // exact widening
        if constexpr (SPLIT) {
            const f16x4 b = ldv<NT>((const PX_GLOBAL f16x4 *)(p + SPLIT_GAP));
#pragma unroll
            for (int i = 0; i < 4; ++i) r.v[4 + i] = (float)b[i];
        }
    } else {
        const f16x8 h = ldv<NT>((const PX_GLOBAL f16x8 *)p);
#pragma unroll
        for (int i = 0; i < 8; ++i) r.v[i] = (float)h[i];  // exact widening
    }
    return r;
}
template <int NT, int U, bool SPLIT>
__device__ __forceinline__ void storev(float *p, const FV<U> &x) {
    static_assert(U == 1 || U == 2 || U == 4 || U == 8, "4 or 8 bytes, or one or two 16-byte vectors");
    static_assert(!SPLIT || U == 8, "the split layout is two groups of four");
    if constexpr (U == 1) {
        stv<NT>((PX_GLOBAL float *)p, x.v[0]);
    } else if constexpr (U == 2) {
        f32x2 a2;
        a2.x = x.v[0]; a2.y = x.v[1];
        stv<NT>((PX_GLOBAL f32x2 *)p, a2);
    } else {
        f32x4 a;
        a.x = x.v[0]; a.y = x.v[1]; a.z = x.v[2]; a.w = x.v[3];
        stv<NT>((PX_GLOBAL f32x4 *)p, a);
        if constexpr (U == 8) {
            f32x4 b;
            b.x = x.v[4]; b.y = x.v[5]; b.z = x.v[6]; b.w = x.v[7];
            stv<NT>((PX_GLOBAL f32x4 *)(p + (SPLIT ? SPLIT_GAP : 4)), b);
        }
    }
}
template <int NT, int U, bool SPLIT>
__device__ __forceinline__ void storev(_Float16 *p, const FV<U> &x) {
    // a lane layout with any other number of binary16 elements per lane must not compile (the 16-byte branch
    // below would store eight elements whatever U says)
    static_assert(U == 2 || U == 4 || U == 8, "4, 8 or 16 bytes");
    static_assert(!SPLIT || U == 8, "the split layout is two groups of four");
    if constexpr (U == 2) {
        f16x2 a;
        a[0] = (_Float16)x.v[0];  // round to nearest even
        a[1] = (_Float16)x.v[1];
        stv<NT>((PX_GLOBAL f16x2 *)p, a);
    } else if constexpr (U == 4 || SPLIT) {
        f16x4 a;
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = (_Float16)x.v[i];  // round to nearest even
        stv<NT>((PX_GLOBAL f16x4 *)p, a);
        if constexpr (SPLIT) {
            f16x4 b;
#pragma unroll
            for (int i = 0; i < 4; ++i) b[i] = (_Float16)x.v[4 + i];
            stv<NT>((PX_GLOBAL f16x4 *)(p + SPLIT_GAP), b);
        }
    } else {
        f16x8 h;
#pragma unroll
        for (int i = 0; i < 8; ++i) h[i] = (_Float16)x.v[i];  // round to nearest even
        stv<NT>((PX_GLOBAL f16x8 *)p, h);
    }
}
__device__ __forceinline__ float load1(const float *p) { return *(const PX_GLOBAL float *)p; }
__device__ __forceinline__ float load1(const _Float16 *p) { return (float)*(const PX_GLOBAL _Float16 *)p; }
__device__ __forceinline__ void store1(float *p, float x) { *(PX_GLOBAL float *)p = x; }
__device__ __forceinline__ void store1(_Float16 *p, float x) { *(PX_GLOBAL _Float16 *)p = (_Float16)x; }

// Number of leading elements after which `a` is 16-byte aligned.
__device__ __forceinline__ int head_of(uintptr_t a, int es) { return (int)(((16u - (unsigned)(a & 15u)) & 15u) / (unsigned)es); }
// Address bits of `a`, after skipping `head` elements, that spoil the alignment of a U-element vector access
// (16 bytes, or 8 for four halves); zero means aligned.  The kernels OR these together over a chunk's operands.
template <int U>
__device__ __forceinline__ unsigned misalign_after(uintptr_t a, int es, int head) {
    const unsigned mask = (unsigned)(U * es < 16 ? U * es : 16) - 1u;
    return (unsigned)(a + (uintptr_t)head * es) & mask;
}
// (The split layout's 8-byte binary16 accesses would be content with 8-byte alignment, but the consecutive
// 8-element steps that finish a chunk use 16-byte ones, so U = 8 always asks for 16.)

// One vector step of a lane: every load is issued before the first use, then the
// arithmetic, then the stores.
template <bool SP, class Op>
__device__ __forceinline__ void vector_step(const Op &op, int i) {
    typename Op::State st;
    op.template load<SP>(st, i);
    op.compute(st);
    op.template store<SP>(st, i);
}

// Lanes that cooperate on a chunk, out of a workgroup of THREADS of which the first WORK have vector work.  As
// shipped every lane takes part (the idle wavefronts help only where a chunk goes element by element); in the A/B
// builds with PXCHG_TUNE_IDLE_EXIT the idle wavefronts leave at kernel entry instead, before they load anything
// (1), or after they have read the chunk's descriptor and before they read any pointer (2).
#if defined(PXCHG_TUNE_IDLE_EXIT) && PXCHG_TUNE_IDLE_EXIT == 1
#define PX_IDLE_WAVEFRONTS(WORK, THREADS)                      \
    static_assert((WORK) % 64 == 0, "whole wavefronts");       \
    if ((int)threadIdx.x >= (WORK)) return;                    \
    constexpr int NTH = (WORK)
#define PX_IDLE_AFTER_DESCRIPTOR(ch)
#elif defined(PXCHG_TUNE_IDLE_EXIT) && PXCHG_TUNE_IDLE_EXIT == 2  // they read the chunk's descriptor, then leave
#define PX_IDLE_WAVEFRONTS(WORK, THREADS)                      \
    static_assert((WORK) % 64 == 0, "whole wavefronts");       \
    constexpr int PX_WORK = (WORK);                            \
    constexpr int NTH = (WORK)
#define PX_IDLE_AFTER_DESCRIPTOR(ch)                           \
    if ((int)threadIdx.x >= PX_WORK) {                         \
        asm volatile("" ::"s"((ch).len));                      \
        continue;                                              \
    }
#else
#define PX_IDLE_WAVEFRONTS(WORK, THREADS) constexpr int NTH = (THREADS)
#define PX_IDLE_AFTER_DESCRIPTOR(ch)
#endif

// Walks one chunk with NTH cooperating lanes (`tid` is the lane's index among them): an element-wise head
// until every operand is aligned, U-element vector steps, an element-wise tail.  `head` < 0 means the operands
// cannot be aligned together and the whole chunk goes element by element.  With SPLIT (U = 8) the vector part
// is cut into 512-element tiles, one split-layout step of a whole wavefront each, and what is left after the
// last full tile goes in consecutive 8-element steps.
template <int U, bool SPLIT, int NTH, class Op>
__device__ __forceinline__ void run_chunk(const Op &op, int len, int head, int tid) {
    if (head < 0 || head > len) {
        for (int i = tid; i < len; i += NTH) op.scalar(i);
        return;
    }
    for (int i = tid; i < head; i += NTH) op.scalar(i);
    const int nvec = (len - head) / U;
    int done = 0;
    if constexpr (SPLIT) {
        static_assert(U == 8 && NTH % 64 == 0, "two groups of four per lane, whole wavefronts");
        const int ntile = nvec / 64;
        for (int t = tid >> 6; t < ntile; t += NTH / 64) vector_step<true>(op, head + t * (64 * U) + (tid & 63) * 4);
        done = ntile * 64;
    }
    for (int u = done + tid; u < nvec; u += NTH) vector_step<false>(op, head + u * U);
    for (int i = head + nvec * U + tid; i < len; i += NTH) op.scalar(i);
}

__device__ __forceinline__ float scale_sum(float s, int use_div, float kf, float scale) {
    // AVG with k a power of two and SUM multiply by an exactly representable
    // factor (1/k or 1), which gives the correctly rounded quotient; other k take
    // the correctly rounded division itself.
    return use_div ? s / kf : s * scale;
}

template <int U>
__device__ __forceinline__ void scale_sumv(FV<U> &s, int use_div, float kf, float scale) {
    if (use_div) {  // uniform branch
#pragma unroll
        for (int e = 0; e < U; ++e) s.v[e] = s.v[e] / kf;
    } else {
#pragma unroll
        for (int e = 0; e < U; ++e) s.v[e] = s.v[e] * scale;
    }
}

__device__ __forceinline__ void momentum_step(float g, float &w, float &v, float lr, float mu, float wd) {
    const float dw = wd * w;
    const float gg = g + dw;
    const float mv = mu * v;
    const float lg = lr * gg;
    v = mv - lg;
    w = w + v;
}

__device__ __forceinline__ void elastic_step(float &x, float &c, float alpha) {
    const float diff = x - c;
    const float d = alpha * diff;
    x = x - d;
    c = c + d;
}

// ---------------------------------------------------------------- pack / unpack

struct ConvertArgs {
    const void *const *src[PXCHG_MAX_K];
    void *const *dst[PXCHG_MAX_K];
};

template <typename TI, typename TO, int NT, int U>
struct ConvertOp {
    const TI *src;
    TO *dst;
    __device__ __forceinline__ void scalar(int i) const { store1(dst + i, load1(src + i)); }
    struct State {
        FV<U> x;
    };
    template <bool SP>
    __device__ __forceinline__ void load(State &st, int i) const { st.x = loadv<NT, U, SP>(src + i); }
    __device__ __forceinline__ void compute(State &) const {}
    template <bool SP>
    __device__ __forceinline__ void store(const State &st, int i) const { storev<NT, U, SP>(dst + i, st.x); }
};

// The chunk list reaches every kernel as a `const PxChunk *__restrict__` parameter of its own, on purpose: the
// descriptor is then known to be read-only and uniform and comes through one scalar load.  Handed over as a member
// of a struct it came through vector loads instead, and the meeting took 187 us instead of 142, the fused
// reduce+update 366 instead of 291.  (Also measured, with no effect beyond 1 %: a second copy of the list dealt out
// so that the eight XCDs, which take every 8th chunk each, find their descriptors in cache lines of their own.)
//
// A chunk may be shared by PARTS workgroups, each taking `part_elems` consecutive elements of it (the table's
// chunk size over PARTS, a multiple of 64, so a part starts at the same offset from 16-byte alignment as its
// chunk).  Returns false for a part that lies beyond a short chunk's end.  Uniform over the workgroup.
template <int PARTS>
__device__ __forceinline__ bool take_part(PxChunk &ch, int part, int part_elems) {
    if constexpr (PARTS > 1) {
        const int off = part * part_elems;
        if (off >= ch.len) return false;
        ch.start += off;
        ch.len = ch.len - off < part_elems ? ch.len - off : part_elems;
    }
    return true;
}

// Workgroups per chunk of the kernels other than the elastic ones (the PXCHG_TUNE_* macros: A/B builds only).
// Measured with two: the update level when cold and 8 % slower inside the step, the binary16 reduce 2..3 %
// slower, the fused reduce+update 1..3 % faster on sets of 7 M to 61 M elements and 2..8 % from 100 M on.
constexpr int update_parts() {
#ifdef PXCHG_TUNE_UPDATE_PARTS
    return PXCHG_TUNE_UPDATE_PARTS;
#else
    return 1;
#endif
}
template <int K, bool F32>
constexpr int reduce_parts() {
#ifdef PXCHG_TUNE_REDUCE16_PARTS  // binary16 in and out, four to eight workers
    if (!F32 && K >= 4) return PXCHG_TUNE_REDUCE16_PARTS;
#endif
    return 1;
}
template <int K>
constexpr int fused_parts() {  // the fused reduce+update with three to eight workers runs two workgroups per chunk
#ifdef PXCHG_TUNE_FUSED_PARTS
    if (K >= 3) return PXCHG_TUNE_FUSED_PARTS;
#endif
    return K >= 3 ? 2 : 1;
}

// Converts every tensor of every worker between binary32 and binary16.  The grid covers k x n_chunks virtual
// chunks, worker-major (chunk-major, where consecutive workgroups take one chunk of consecutive workers and each
// XCD so stays with one worker's buffers, measured 2 % slower).  One wavefront in the split layout per chunk (A/B builds: other lanes, or several
// workgroups per chunk).
constexpr int convert_parts() {
#ifdef PXCHG_TUNE_CONVERT_PARTS
    return PXCHG_TUNE_CONVERT_PARTS;
#else
    return 1;
#endif
}
constexpr int convert_lanes() {  // per workgroup
#ifdef PXCHG_TUNE_CONVERT_LANES
    return PXCHG_TUNE_CONVERT_LANES;
#else
    return 64;
#endif
}
template <typename TI, typename TO, int NT>
__global__ __launch_bounds__(convert_lanes()) void pxchg_convert_kernel(const PxChunk *__restrict__ chunks, int n_chunks,
                                                                        int64_t n_virtual, ConvertArgs args, int part_elems) {
    constexpr int PARTS = convert_parts(), NTH = convert_lanes(), U = 512 / (NTH * PARTS);
    constexpr bool SPLIT = U == 8;  // float32 on one side
    const int64_t per_worker = (int64_t)n_chunks * PARTS;
    for (int64_t vc = blockIdx.x; vc < n_virtual; vc += gridDim.x) {
        const int w = (int)(vc / per_worker);
        const int rest = (int)(vc - (int64_t)w * per_worker);
        PxChunk ch = chunks[rest / PARTS];
        if (!take_part<PARTS>(ch, rest % PARTS, part_elems)) continue;
        ConvertOp<TI, TO, NT, U> op;
        op.src = table_ptr<const TI>(args.src[w], ch.tensor) + ch.start;
        op.dst = table_ptr<TO>(args.dst[w], ch.tensor) + ch.start;
        int head = head_of((uintptr_t)op.dst, sizeof(TO));
        if (misalign_after<U>((uintptr_t)op.src, sizeof(TI), head) | misalign_after<U>((uintptr_t)op.dst, sizeof(TO), head))
            head = -1;
        run_chunk<U, SPLIT, NTH>(op, ch.len, head, threadIdx.x);
    }
}

// ---------------------------------------------------------------- reduce + average

// Lanes per 512-element chunk in the reduce kernels.  Binary16 in and out with four or more workers runs as
// two wavefronts of 4-element (8-byte) lanes, measured 2..8 % faster than one wavefront of 8-element lanes and
// 6 % faster than four wavefronts of 2-element lanes;
// with fewer workers a wavefront would have too little in flight that way (k = 1: 30 % slower), so those keep
// one wavefront of 8-element lanes.  Float32 in and out with four or more workers: 2-element (8-byte) lanes,
// +1..3 % over the split layout of one wavefront, which every other combination with float32 on either side
// keeps.  K = 0 stands for the any-k kernel (more than 8 workers).
template <int K, typename TI, typename TO>
constexpr int reduce_lanes() {
    if (std::is_same<TI, float>::value && std::is_same<TO, float>::value && K >= 4) return 256;
#ifdef PXCHG_TUNE_REDUCE16_LANES  // A/B builds only (paper_1605_08325_amd/tune.py): 64, 128 or 256
    if (!touches_f32<TI, TO>() && !(K >= 1 && K <= 3)) return PXCHG_TUNE_REDUCE16_LANES;
#endif
    return (touches_f32<TI, TO>() || (K >= 1 && K <= 3)) ? 64 : 128 / reduce_parts<K, touches_f32<TI, TO>()>();
}

// How a launch of the reduce treats its table (see small_tensors and large_tensors below).
enum ReduceMode { REDUCE_PLAIN = 0, REDUCE_LANE_POINTERS = 1, REDUCE_IDLE_WAVEFRONTS = 2 };

// Workgroup size of the reduce kernels: the working lanes, and for binary16 in and out with four to eight workers
// on tables of large tensors two idle wavefronts (see update_lanes).  Measured there: 61 M in 16 tensors 171.2
// against 175.9 us cold and 164.3 against 167.6 inside the step, 138 M in 32 tensors 378 against 396 and 365 against
// 373; single tensors of 7 M to 100 M elements level to 6 % faster.  With a hundred tensors and more they cost
// 4..8 % instead (61 M in 116 tensors 177 against 170; 7 M in 116 tensors 26.8 against 25.5; 13.4 M in 128 tensors
// 48.6 against 45.0), and with 16 tensors in 7 M 2 %: hence only on tables of large tensors.
template <int K, typename TI, typename TO, int MODE>
constexpr int reduce_threads() {
#ifdef PXCHG_TUNE_REDUCE16_IDLE  // A/B builds only: that many idle wavefronts on every table
    if (!touches_f32<TI, TO>() && K >= 4) return reduce_lanes<K, TI, TO>() + 64 * PXCHG_TUNE_REDUCE16_IDLE;
#endif
    return reduce_lanes<K, TI, TO>() + (MODE == REDUCE_IDLE_WAVEFRONTS && !touches_f32<TI, TO>() && K >= 4 ? 128 : 0);
}

struct ReduceArgs {
    const void *const *contrib[PXCHG_MAX_K];
    void *const *out;
    int k;
    int use_div;
    float kf;
    float scale;
};

template <int K, typename TI, typename TO, int NT, int U>
struct ReduceOp {
    const TI *src[K];
    TO *dst;
    int use_div;
    float kf, scale;
    __device__ __forceinline__ void scalar(int i) const {
        float s = load1(src[0] + i);
#pragma unroll
        for (int w = 1; w < K; ++w) s = s + load1(src[w] + i);
        store1(dst + i, scale_sum(s, use_div, kf, scale));
    }
    struct State {
        FV<U> c[K];
    };
    template <bool SP>
    __device__ __forceinline__ void load(State &st, int i) const {
#pragma unroll
        for (int w = 0; w < K; ++w) st.c[w] = loadv<NT, U, SP>(src[w] + i);
    }
    __device__ __forceinline__ void compute(State &st) const {
#pragma unroll
        for (int w = 1; w < K; ++w)
#pragma unroll
            for (int e = 0; e < U; ++e) st.c[0].v[e] = st.c[0].v[e] + st.c[w].v[e];  // worker order
        scale_sumv(st.c[0], use_div, kf, scale);
    }
    template <bool SP>
    __device__ __forceinline__ void store(const State &st, int i) const {
        storev<NT, U, SP>(dst + i, st.c[0]);
    }
};

// Any k up to PXCHG_MAX_K: the chunk's k source pointers sit in LDS.
template <typename TI, typename TO, int NT, int U>
struct ReduceOpAnyK {
    const TI *const *src;  // LDS
    TO *dst;
    int k, use_div;
    float kf, scale;
    __device__ __forceinline__ void scalar(int i) const {
        float s = load1(src[0] + i);
        for (int w = 1; w < k; ++w) s = s + load1(src[w] + i);
        store1(dst + i, scale_sum(s, use_div, kf, scale));
    }
    struct State {
        FV<U> s;
    };
    // any k: the sum is formed while loading, four contributions at a time
    template <bool SP>
    __device__ __forceinline__ void load(State &st, int i) const {
        FV<U> s = loadv<NT, U, SP>(src[0] + i);
        int w = 1;
        for (; w + 4 <= k; w += 4) {
            FV<U> c[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) c[q] = loadv<NT, U, SP>(src[w + q] + i);
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int e = 0; e < U; ++e) s.v[e] = s.v[e] + c[q].v[e];
        }
        for (; w < k; ++w) {
            const FV<U> c = loadv<NT, U, SP>(src[w] + i);
#pragma unroll
            for (int e = 0; e < U; ++e) s.v[e] = s.v[e] + c.v[e];
        }
        st.s = s;
    }
    __device__ __forceinline__ void compute(State &st) const { scale_sumv(st.s, use_div, kf, scale); }
    template <bool SP>
    __device__ __forceinline__ void store(const State &st, int i) const { storev<NT, U, SP>(dst + i, st.s); }
};

template <int K, typename TI, typename TO, int NT, int MODE>
__global__ __launch_bounds__((reduce_threads<K, TI, TO, MODE>())) void pxchg_reduce_avg_kernel(
    const PxChunk *__restrict__ chunks, int n_chunks, ReduceArgs args, int part_elems) {
    constexpr int PARTS = reduce_parts<K, touches_f32<TI, TO>()>();
    constexpr int U = 512 / (reduce_lanes<K, TI, TO>() * PARTS);
    PX_IDLE_WAVEFRONTS((reduce_lanes<K, TI, TO>()), (reduce_threads<K, TI, TO, MODE>()));
    constexpr bool SPLIT = touches_f32<TI, TO>() && U == 8;
    for (int vc = blockIdx.x; vc < n_chunks * PARTS; vc += gridDim.x) {
        PxChunk ch = chunks[vc / PARTS];
        PX_IDLE_AFTER_DESCRIPTOR(ch)
        if (!take_part<PARTS>(ch, vc % PARTS, part_elems)) continue;
        ReduceOp<K, TI, TO, NT, U> op;
        op.use_div = args.use_div;
        op.kf = args.kf;
        op.scale = args.scale;
        if constexpr (MODE == REDUCE_LANE_POINTERS) {
            const int lane = threadIdx.x & 63;
            const void *const *tab = (const void *const *)args.out;  // lanes K.. (lane K's is the one read out)
#pragma unroll
            for (int w = 0; w < K; ++w)
                if (lane == w) tab = args.contrib[w];
            const uintptr_t mine = table_entry(tab, ch.tensor);
            op.dst = lane_pointer<TO>(mine, K) + ch.start;
#pragma unroll
            for (int w = 0; w < K; ++w) op.src[w] = lane_pointer<const TI>(mine, w) + ch.start;
        } else {
            op.dst = table_ptr<TO>(args.out, ch.tensor) + ch.start;
#pragma unroll
            for (int w = 0; w < K; ++w) op.src[w] = table_ptr<const TI>(args.contrib[w], ch.tensor) + ch.start;
        }
        int head = head_of((uintptr_t)op.dst, sizeof(TO));
        unsigned bad = misalign_after<U>((uintptr_t)op.dst, sizeof(TO), head);
#pragma unroll
        for (int w = 0; w < K; ++w) bad |= misalign_after<U>((uintptr_t)op.src[w], sizeof(TI), head);
        if (bad) head = -1;
        run_chunk<U, SPLIT, NTH>(op, ch.len, head, threadIdx.x);
    }
}

template <typename TI, typename TO, int NT>
__global__ __launch_bounds__((reduce_lanes<0, TI, TO>())) void pxchg_reduce_avg_anyk_kernel(
    const PxChunk *__restrict__ chunks, int n_chunks, ReduceArgs args) {
    constexpr bool SPLIT = touches_f32<TI, TO>();
    constexpr int NTH = reduce_lanes<0, TI, TO>(), U = NTH == 64 ? 8 : 4;
    __shared__ const TI *sp[PXCHG_MAX_K];
    __shared__ int s_head;
    for (int c = blockIdx.x; c < n_chunks; c += gridDim.x) {
        const PxChunk ch = chunks[c];
        ReduceOpAnyK<TI, TO, NT, U> op;
        op.dst = table_ptr<TO>(args.out, ch.tensor) + ch.start;
        op.k = args.k;
        op.use_div = args.use_div;
        op.kf = args.kf;
        op.scale = args.scale;
        const int head0 = head_of((uintptr_t)op.dst, sizeof(TO));
        __syncthreads();  // previous chunk's readers are done with sp
        if (threadIdx.x == 0) s_head = misalign_after<U>((uintptr_t)op.dst, sizeof(TO), head0) ? -1 : head0;
        __syncthreads();
        if ((int)threadIdx.x < args.k) {
            const TI *p = table_ptr<const TI>(args.contrib[threadIdx.x], ch.tensor) + ch.start;
            sp[threadIdx.x] = p;
            if (misalign_after<U>((uintptr_t)p, sizeof(TI), head0)) s_head = -1;  // benign race: all write -1
        }
        __syncthreads();
        op.src = sp;
        run_chunk<U, SPLIT, NTH>(op, ch.len, s_head, threadIdx.x);
    }
}

// ---------------------------------------------------------------- momentum SGD

struct UpdateArgs {
    const void *const *grad;
    void *const *param;
    void *const *vel;
    const float *mult;  // per tensor (lr multiplier, decay multiplier), or null
    float lr, mu, wd;
};

// The tensor's own learning rate and decay: the call's values times the table's per-tensor multipliers, each
// product rounded to binary32 (uniform per chunk).
__device__ __forceinline__ void tensor_rates(const float *mult, int tensor, float &lr, float &wd) {
    if (mult) {
        const float PX_CONST *m = (const float PX_CONST *)mult + 2 * tensor;
        lr = lr * m[0];
        wd = wd * m[1];
    }
}

template <typename TG, int NT, int U>
struct UpdateOp {
    const TG *g;
    float *w, *v;
    float lr, mu, wd;
    __device__ __forceinline__ void scalar(int i) const {
        float wi = load1(w + i), vi = load1(v + i);
        momentum_step(load1(g + i), wi, vi, lr, mu, wd);
        store1(v + i, vi);
        store1(w + i, wi);
    }
    struct State {
        FV<U> a, ww, vv;
    };
    template <bool SP>
    __device__ __forceinline__ void load(State &st, int i) const {
        // A binary16 gradient is read with plain loads whatever the policy: it is usually the mean that the
        // reduce has just written, and what is left of it in the memory-side cache is only found that way
        // (update 3 % faster right after the reduce, the same when the gradient is cold; a float32 gradient
        // is twice the size, gains nothing warm and loses 0.6 % cold, so it follows the policy).
        st.a = loadv<(std::is_same<TG, _Float16>::value ? 0 : NT), U, SP>(g + i);
        st.ww = loadv<NT, U, SP>(w + i);
        st.vv = loadv<NT, U, SP>(v + i);
    }
    __device__ __forceinline__ void compute(State &st) const {
#pragma unroll
        for (int e = 0; e < U; ++e) momentum_step(st.a.v[e], st.ww.v[e], st.vv.v[e], lr, mu, wd);
    }
    template <bool SP>
    __device__ __forceinline__ void store(const State &st, int i) const {
        storev<NT, U, SP>(v + i, st.vv);
        storev<NT, U, SP>(w + i, st.ww);
    }
};

// Idle wavefronts.  Several kernels run faster when their workgroups are launched with more wavefronts than have
// work.  The extra ones run the prelude like the others (the chunk's descriptor and pointers), find nothing to do
// in the vector part of a 512-element chunk and end; lanes beyond the working ones only ever take part in the
// element-wise paths.  Measured against the same kernel without them, in one run each, on sets from 7 M to 138 M
// elements: the update with a binary16 gradient (as many idle wavefronts as working ones) 1.5..2.5 %, the single
// elastic meeting (two per working one) 4..7 %, and on tables of large tensors the fused reduce+update of three
// or more workers (one) 2..3 % and the binary16 reduce of four or more (two) 2..4 %.  The counts are optima, one
// more or one less is 1..4 % slower.  Idle wavefronts that leave at kernel entry, or right after reading the
// descriptor, give about half of the gain (A/B build PXCHG_TUNE_IDLE_EXIT): what helps is that they stay for the
// prelude.  It is not a general rule: the update with a float32 gradient lost 6 % in the exchange, the pack 20 %,
// the round of 8 workers 8 %, the float32 reduce 1..6 %; the reduce and the fused kernel lose 4..11 % with them on
// tables of many tensors.  Those run without.
template <typename TG>
constexpr int update_lanes() {  // 128 working lanes; as many idle ones for a binary16 gradient
#ifdef PXCHG_TUNE_UPDATE_THREADS  // A/B builds only: workgroup size for a binary16 gradient (128 lanes work)
    if (std::is_same<TG, _Float16>::value) return PXCHG_TUNE_UPDATE_THREADS;
#endif
#ifdef PXCHG_TUNE_NO_IDLE  // A/B builds only: no idle wavefronts anywhere
    return 128 / update_parts();
#else
    return (std::is_same<TG, _Float16>::value ? 256 : 128) / update_parts();
#endif
}

template <typename TG, int NT>
__global__ __launch_bounds__((update_lanes<TG>())) void pxchg_sgd_momentum_kernel(const PxChunk *__restrict__ chunks, int n_chunks,
                                                                 UpdateArgs args, int part_elems) {
    constexpr int U = 4;  // two working wavefronts of 4-element lanes (one per workgroup in the A/B build with two parts)
    constexpr bool SPLIT = false;
    constexpr int PARTS = update_parts();
    PX_IDLE_WAVEFRONTS(128 / PARTS, update_lanes<TG>());
    for (int vc = blockIdx.x; vc < n_chunks * PARTS; vc += gridDim.x) {
        PxChunk ch = chunks[vc / PARTS];
        PX_IDLE_AFTER_DESCRIPTOR(ch)
        if (!take_part<PARTS>(ch, vc % PARTS, part_elems)) continue;
        UpdateOp<TG, NT, U> op;
        op.g = table_ptr<const TG>(args.grad, ch.tensor) + ch.start;
        op.w = table_ptr<float>(args.param, ch.tensor) + ch.start;
        op.v = table_ptr<float>(args.vel, ch.tensor) + ch.start;
        op.lr = args.lr;
        op.mu = args.mu;
        op.wd = args.wd;
        tensor_rates(args.mult, ch.tensor, op.lr, op.wd);
        int head = head_of((uintptr_t)op.g, sizeof(TG));
        if (misalign_after<U>((uintptr_t)op.g, sizeof(TG), head) | misalign_after<U>((uintptr_t)op.w, 4, head) |
            misalign_after<U>((uintptr_t)op.v, 4, head))
            head = -1;
        run_chunk<U, SPLIT, NTH>(op, ch.len, head, threadIdx.x);
    }
}

// ---------------------------------------------------------------- fused reduce + update

struct FusedArgs {
    const void *const *contrib[PXCHG_MAX_K];
    void *const *param;
    void *const *vel;
    const float *mult;  // per tensor (lr multiplier, decay multiplier), or null
    int k;
    int use_div;
    float kf, scale;
    float lr, mu, wd;
};

template <int K, typename TI, bool WIRE16, int NT, int U>
struct FusedOp {
    const TI *src[K];
    float *w, *v;
    int use_div;
    float kf, scale, lr, mu, wd;
    __device__ __forceinline__ static float wire(float a) {
        if constexpr (WIRE16)
            return (float)(_Float16)a;  // what the second transfer leg would have carried
        else
            return a;
    }
    __device__ __forceinline__ void scalar(int i) const {
        float s = load1(src[0] + i);
#pragma unroll
        for (int q = 1; q < K; ++q) s = s + load1(src[q] + i);
        float wi = load1(w + i), vi = load1(v + i);
        momentum_step(wire(scale_sum(s, use_div, kf, scale)), wi, vi, lr, mu, wd);
        store1(v + i, vi);
        store1(w + i, wi);
    }
    struct State {
        FV<U> c[K], ww, vv;
    };
    template <bool SP>
    __device__ __forceinline__ void load(State &st, int i) const {
#pragma unroll
        for (int q = 0; q < K; ++q) st.c[q] = loadv<NT, U, SP>(src[q] + i);
        st.ww = loadv<NT, U, SP>(w + i);
        st.vv = loadv<NT, U, SP>(v + i);
    }
    __device__ __forceinline__ void compute(State &st) const {
#pragma unroll
        for (int q = 1; q < K; ++q)
#pragma unroll
            for (int e = 0; e < U; ++e) st.c[0].v[e] = st.c[0].v[e] + st.c[q].v[e];  // worker order
        scale_sumv(st.c[0], use_div, kf, scale);
#pragma unroll
        for (int e = 0; e < U; ++e) momentum_step(wire(st.c[0].v[e]), st.ww.v[e], st.vv.v[e], lr, mu, wd);
    }
    template <bool SP>
    __device__ __forceinline__ void store(const State &st, int i) const {
        storev<NT, U, SP>(v + i, st.vv);
        storev<NT, U, SP>(w + i, st.ww);
    }
};

// Lanes per workgroup in the fused kernel.  Float32 contributions: 2-element (8-byte) lanes measured
// 3..6 % faster than the split layout of one wavefront for every k.  Binary16 contributions: the same
// 2-element lanes (8-byte accesses to w and v, 4-byte ones to the contributions) from k = 3 on (+1..5 %), in
// two workgroups of 128 lanes per chunk (see fused_parts); k = 2 keeps the split layout and k = 1 runs as
// two wavefronts of 4-element lanes (+4 %).
template <int K, typename TI>
constexpr int fused_lanes() {
#ifdef PXCHG_TUNE_FUSED_LANES  // A/B builds only: lanes per workgroup for three or more workers
    if (K >= 3) return PXCHG_TUNE_FUSED_LANES;
#endif
    if (std::is_same<TI, float>::value) return 256 / fused_parts<K>();
    return K == 1 ? 128 : K == 2 ? 64 : 256 / fused_parts<K>();
}

// Workgroup size of the fused kernel: the working lanes, and for three or more workers on tables of large tensors
// (IDLE; see small_tensors below) one idle wavefront (see update_lanes), measured 2..3 % faster there (61 M in 16
// tensors 293 against 299 us, in 116 tensors 292 against 301, 138 M in 32 tensors 667 against 683) and up to 11 %
// slower on tables of many small tensors (61 M in 2048 tensors), which therefore run without; two idle wavefronts
// lose 4 %.
template <int K, typename TI, bool IDLE>
constexpr int fused_threads() {
#ifdef PXCHG_TUNE_FUSED_IDLE  // A/B builds only: that many idle wavefronts on every table
    if (K >= 3) return fused_lanes<K, TI>() + 64 * PXCHG_TUNE_FUSED_IDLE;
#endif
    return fused_lanes<K, TI>() + (K >= 3 && IDLE ? 64 : 0);
}

template <int K, typename TI, bool WIRE16, int NT, bool IDLE>
__global__ __launch_bounds__((fused_threads<K, TI, IDLE>())) void pxchg_reduce_avg_sgd_momentum_kernel(
    const PxChunk *__restrict__ chunks, int n_chunks, FusedArgs args, int part_elems) {
    constexpr int PARTS = fused_parts<K>();
    constexpr int U = 512 / (fused_lanes<K, TI>() * PARTS);
    PX_IDLE_WAVEFRONTS((fused_lanes<K, TI>()), (fused_threads<K, TI, IDLE>()));
    constexpr bool SPLIT = U == 8;
    for (int vc = blockIdx.x; vc < n_chunks * PARTS; vc += gridDim.x) {
        PxChunk ch = chunks[vc / PARTS];
        PX_IDLE_AFTER_DESCRIPTOR(ch)
        if (!take_part<PARTS>(ch, vc % PARTS, part_elems)) continue;
        FusedOp<K, TI, WIRE16, NT, U> op;
        op.w = table_ptr<float>(args.param, ch.tensor) + ch.start;
        op.v = table_ptr<float>(args.vel, ch.tensor) + ch.start;
#pragma unroll
        for (int q = 0; q < K; ++q) op.src[q] = table_ptr<const TI>(args.contrib[q], ch.tensor) + ch.start;
        op.use_div = args.use_div;
        op.kf = args.kf;
        op.scale = args.scale;
        op.lr = args.lr;
        op.mu = args.mu;
        op.wd = args.wd;
        tensor_rates(args.mult, ch.tensor, op.lr, op.wd);
        int head = head_of((uintptr_t)op.src[0], sizeof(TI));
        unsigned bad = misalign_after<U>((uintptr_t)op.w, 4, head) | misalign_after<U>((uintptr_t)op.v, 4, head);
#pragma unroll
        for (int q = 0; q < K; ++q) bad |= misalign_after<U>((uintptr_t)op.src[q], sizeof(TI), head);
        if (bad) head = -1;
        run_chunk<U, SPLIT, NTH>(op, ch.len, head, threadIdx.x);
    }
}

// Any k up to PXCHG_MAX_K (more than 8 workers): the chunk's k source pointers sit in LDS and the sum is
// formed while loading, four contributions at a time, as in the any-k reduce.  Two wavefronts of 4-element
// lanes per chunk.
template <typename TI, bool WIRE16, int NT, int U>
struct FusedOpAnyK {
    const TI *const *src;  // LDS
    float *w, *v;
    int k, use_div;
    float kf, scale, lr, mu, wd;
    __device__ __forceinline__ static float wire(float a) {
        if constexpr (WIRE16)
            return (float)(_Float16)a;
        else
            return a;
    }
    __device__ __forceinline__ void scalar(int i) const {
        float s = load1(src[0] + i);
        for (int q = 1; q < k; ++q) s = s + load1(src[q] + i);
        float wi = load1(w + i), vi = load1(v + i);
        momentum_step(wire(scale_sum(s, use_div, kf, scale)), wi, vi, lr, mu, wd);
        store1(v + i, vi);
        store1(w + i, wi);
    }
    struct State {
        FV<U> s, ww, vv;
    };
    template <bool SP>
    __device__ __forceinline__ void load(State &st, int i) const {
        st.ww = loadv<NT, U, SP>(w + i);
        st.vv = loadv<NT, U, SP>(v + i);
        FV<U> s = loadv<NT, U, SP>(src[0] + i);
        int q = 1;
        for (; q + 4 <= k; q += 4) {
            FV<U> c[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) c[r] = loadv<NT, U, SP>(src[q + r] + i);
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int e = 0; e < U; ++e) s.v[e] = s.v[e] + c[r].v[e];  // worker order
        }
        for (; q < k; ++q) {
            const FV<U> c = loadv<NT, U, SP>(src[q] + i);
#pragma unroll
            for (int e = 0; e < U; ++e) s.v[e] = s.v[e] + c.v[e];
        }
        st.s = s;
    }
    __device__ __forceinline__ void compute(State &st) const {
        scale_sumv(st.s, use_div, kf, scale);
#pragma unroll
        for (int e = 0; e < U; ++e) momentum_step(wire(st.s.v[e]), st.ww.v[e], st.vv.v[e], lr, mu, wd);
    }
    template <bool SP>
    __device__ __forceinline__ void store(const State &st, int i) const {
        storev<NT, U, SP>(v + i, st.vv);
        storev<NT, U, SP>(w + i, st.ww);
    }
};

template <typename TI, bool WIRE16, int NT>
__global__ __launch_bounds__(128) void pxchg_reduce_avg_sgd_momentum_anyk_kernel(const PxChunk *__restrict__ chunks,
                                                                                 int n_chunks, FusedArgs args) {
    constexpr int NTH = 128, U = 4;
    __shared__ const TI *sp[PXCHG_MAX_K];
    __shared__ int s_head;
    for (int c = blockIdx.x; c < n_chunks; c += gridDim.x) {
        const PxChunk ch = chunks[c];
        FusedOpAnyK<TI, WIRE16, NT, U> op;
        op.w = table_ptr<float>(args.param, ch.tensor) + ch.start;
        op.v = table_ptr<float>(args.vel, ch.tensor) + ch.start;
        op.k = args.k;
        op.use_div = args.use_div;
        op.kf = args.kf;
        op.scale = args.scale;
        op.lr = args.lr;
        op.mu = args.mu;
        op.wd = args.wd;
        tensor_rates(args.mult, ch.tensor, op.lr, op.wd);
        const int head0 = head_of((uintptr_t)op.w, 4);
        __syncthreads();  // previous chunk's readers are done with sp
        if (threadIdx.x == 0)
            s_head = (misalign_after<U>((uintptr_t)op.w, 4, head0) | misalign_after<U>((uintptr_t)op.v, 4, head0)) ? -1 : head0;
        __syncthreads();
        if ((int)threadIdx.x < args.k) {
            const TI *p = table_ptr<const TI>(args.contrib[threadIdx.x], ch.tensor) + ch.start;
            sp[threadIdx.x] = p;
            if (misalign_after<U>((uintptr_t)p, sizeof(TI), head0)) s_head = -1;  // benign race: all write -1
        }
        __syncthreads();
        op.src = sp;
        run_chunk<U, false, NTH>(op, ch.len, s_head, threadIdx.x);
    }
}

// ---------------------------------------------------------------- elastic averaging

// Workgroup shape of the elastic kernels: a wavefront should load 2..4 KiB in all, so the more workers a fused
// round has, the narrower its lanes (a round of 8 with 4-byte lanes measured 7 % faster than with the split
// layout of one wavefront, and 6..9 % faster than with 8- or 16-byte lanes).  Rounds of five or more workers
// also cut every chunk into two parts, one workgroup of 256 lanes each: the same 4-byte lanes in workgroups of
// four wavefronts instead of eight measured 2 % faster (cold operands, round of 8: 710.6 against 726.2 us).
// The single meeting does the same with 16-byte lanes: one working wavefront per 256 elements instead of two per
// 512 measured 1.5..3.6 % faster on sets of 7 M to 61 M elements and on single tensors up to 300 M, and 0.7..2.5 %
// slower on the 138 M set of 32 tensors; narrower lanes in the same two parts lose 11 %.
template <int K, bool CR>
constexpr int elastic_parts() {  // workgroups per chunk
#ifdef PXCHG_TUNE_ELASTIC1_PARTS  // A/B builds only: 1, 2 or 4 for the single meeting
    if (K == 1) return PXCHG_TUNE_ELASTIC1_PARTS;
#endif
    if (K == 1) return CR ? 1 : 2;  // with the center kept cached, one workgroup per chunk is the faster shape (5 %)
#ifdef PXCHG_TUNE_ELASTIC8_PARTS  // A/B builds only: 1 or 2
    return K >= 5 ? PXCHG_TUNE_ELASTIC8_PARTS : 1;
#else
    return K >= 5 ? 2 : 1;
#endif
}
template <int K, bool CR>
constexpr int elastic_lanes() {  // working lanes per workgroup
#ifdef PXCHG_TUNE_ELASTIC8_LANES  // A/B builds only: 128, 256 or 512 lanes per chunk for rounds of five or more
    if (K >= 5) return PXCHG_TUNE_ELASTIC8_LANES / elastic_parts<K, CR>();
#endif
#ifdef PXCHG_TUNE_ELASTIC1_LANES  // A/B builds only: 64, 128 or 256 per workgroup for the single meeting
    if (K == 1) return PXCHG_TUNE_ELASTIC1_LANES;
#endif
    return K == 1 ? 128 / elastic_parts<K, CR>() : K == 2 ? 128 : K <= 4 ? 256 : 512 / elastic_parts<K, CR>();
}

// Workgroup size over working lanes.  Idle wavefronts (see update_lanes): one per working wavefront for the fused
// round of two and for the meeting with the center kept cached, two for the single meeting, whose workgroups
// then are one working wavefront and two idle ones (measured against one idle wavefront: -1.7 % at 61 M, -2.1 % at
// 138 M, -1.5 % at 7 M and 13 M; three idle ones are level at 61 M and 4 % slower at 138 M, five and more lose 40 %
// and upwards).
template <int K, bool CR>
constexpr int elastic_pad() {
#ifdef PXCHG_TUNE_ELASTIC1_PAD  // A/B builds only: 1..6 for the single meeting
    if (K == 1) return PXCHG_TUNE_ELASTIC1_PAD;
#endif
#ifdef PXCHG_TUNE_ELASTIC8_PAD  // A/B builds only: 1 or 2 for rounds of five or more
    if (K >= 5) return PXCHG_TUNE_ELASTIC8_PAD;
#endif
#ifdef PXCHG_TUNE_NO_IDLE
    return 1;
#else
    return K == 1 && !CR ? 3 : K <= 2 ? 2 : 1;
#endif
}

struct ElasticArgs {
    void *const *x[PXCHG_MAX_K];
    void *const *c;
    int k;
    float alpha;
    int part_elems;  // elements per workgroup where a chunk is cut into parts: the table's chunk size over the parts
};

// CR ("center resident"): the center is read with plain loads and written with agent-scope stores, whatever
// the policy of the worker operands, so that it stays in the memory-side cache between meetings.
template <int K, int NT, int U, bool CR>
struct ElasticOp {
    static constexpr int C_LOAD = CR ? 0 : NT, C_STORE = CR ? 5 : NT;
    float *x[K];
    float *c;
    float alpha;
    __device__ __forceinline__ void scalar(int i) const {
        float ci = load1(c + i);
#pragma unroll
        for (int q = 0; q < K; ++q) {
            float xi = load1(x[q] + i);
            elastic_step(xi, ci, alpha);
            store1(x[q] + i, xi);
        }
        store1(c + i, ci);
    }
    struct State {
        FV<U> xs[K], cc;
    };
    template <bool SP>
    __device__ __forceinline__ void load(State &st, int i) const {
#pragma unroll
        for (int q = 0; q < K; ++q) st.xs[q] = loadv<NT, U, SP>(x[q] + i);
        st.cc = loadv<C_LOAD, U, SP>(c + i);
    }
    __device__ __forceinline__ void compute(State &st) const {
#pragma unroll
        for (int q = 0; q < K; ++q)  // arrival order: the center carries over
#pragma unroll
            for (int e = 0; e < U; ++e) elastic_step(st.xs[q].v[e], st.cc.v[e], alpha);
    }
    template <bool SP>
    __device__ __forceinline__ void store(const State &st, int i) const {
#pragma unroll
        for (int q = 0; q < K; ++q) storev<NT, U, SP>(x[q] + i, st.xs[q]);
        storev<C_STORE, U, SP>(c + i, st.cc);
    }
};

template <int K, int NT, bool CR>
__global__ __launch_bounds__((elastic_lanes<K, CR>() * elastic_pad<K, CR>())) void pxchg_easgd_kernel(const PxChunk *__restrict__ chunks,
                                                                        int n_chunks, ElasticArgs args) {
    constexpr int PARTS = elastic_parts<K, CR>();
    constexpr int U = 512 / (elastic_lanes<K, CR>() * PARTS);
    PX_IDLE_WAVEFRONTS((elastic_lanes<K, CR>()), (elastic_lanes<K, CR>() * elastic_pad<K, CR>()));
    constexpr bool SPLIT = false;
    for (int vc = blockIdx.x; vc < n_chunks * PARTS; vc += gridDim.x) {
        PxChunk ch = chunks[vc / PARTS];
        PX_IDLE_AFTER_DESCRIPTOR(ch)
        if (!take_part<PARTS>(ch, vc % PARTS, args.part_elems)) continue;
        ElasticOp<K, NT, U, CR> op;
        op.alpha = args.alpha;
        op.c = table_ptr<float>(args.c, ch.tensor) + ch.start;
#pragma unroll
        for (int q = 0; q < K; ++q) op.x[q] = table_ptr<float>(args.x[q], ch.tensor) + ch.start;
        int head = head_of((uintptr_t)op.c, 4);
        unsigned bad = misalign_after<U>((uintptr_t)op.c, 4, head);
#pragma unroll
        for (int q = 0; q < K; ++q) bad |= misalign_after<U>((uintptr_t)op.x[q], 4, head);
        if (bad) head = -1;
        run_chunk<U, SPLIT, NTH>(op, ch.len, head, threadIdx.x);
    }
}

// ---------------------------------------------------------------- diagnostics

struct StatsAcc {
    unsigned bad;  // one lane's share of the count: far below 2^32 for any set that fits the device
    float mx;
    double ss;
};

// Branch-free: a non-finite element counts and then takes part as +0, which changes neither the maximum of
// magnitudes nor the sum (the accumulators are never negative, so adding +0 leaves every bit as it is).  The
// square of a binary32 value is exact in binary64, so the fused multiply-add gives the same bits as a product
// and a sum rounded one after the other.
__device__ __forceinline__ void stats_take(StatsAcc &a, float x) {
    const bool nonfinite = (__float_as_uint(x) & 0x7f800000u) == 0x7f800000u;  // infinity or NaN
    const float xf = nonfinite ? 0.0f : x;
    a.bad += nonfinite ? 1u : 0u;
    a.mx = fmaxf(a.mx, fabsf(xf));
    const double d = (double)xf;
    a.ss = __builtin_fma(d, d, a.ss);
}

// The sum of squares is defined with its order (pxchg.h): which lane of which wavefront of which block takes an
// element follows from the element's place alone, never from how a launch happens to be scheduled, and the
// partial sums are combined in a fixed tree.  So the result is the same bits on every run.
//   * block b = chunks b*BLOCK_CHUNKS .. +BLOCK_CHUNKS-1, one workgroup of WAVES wavefronts;
//   * the chunk at place j of its block belongs to wavefront j mod WAVES;
//   * element i of a chunk belongs to lane (i div P) mod 64, P = elements per 16 bytes.
// A whole 512-element chunk is therefore one 16-byte load per lane for binary16 (lane l: elements 8l..8l+7) and
// two for float32 (4l..4l+3 and 256+4l..256+4l+3, each instruction covering a contiguous 1 KiB): the owner rule
// is the coalesced layout.  A binary16 wavefront takes two of its chunks per trip (2 KiB of loads in flight;
// one chunk per trip measured 9 % slower, 4 KiB 5 % slower).  Block shape, measured on 122 MB / 14 MB of
// binary16 (both launches, microseconds): 4 wavefronts x 32 chunks 27.9 / 14.2, 4 x 64 27.9 / 18.0, 8 x 64
// 28.6 / 13.6, 8 x 32 31.0 / 11.4, 16 x 64 32.9 / 11.3, 16 x 256 28.2 / 21.1, 2 x 16 29.8 / 14.3.
constexpr int STATS_WAVES = PXCHG_STATS_WAVES, STATS_BLOCK_CHUNKS = PXCHG_STATS_BLOCK_CHUNKS;
constexpr int STATS_COMBINE_THREADS = PXCHG_STATS_COMBINE_THREADS;
static_assert(STATS_COMBINE_THREADS % 64 == 0 && STATS_COMBINE_THREADS <= 1024, "whole wavefronts, one workgroup");

// Any chunk, any alignment, in the owner order: 16-byte piece q of the chunk belongs to lane q mod 64.
template <typename T, int NT>
__device__ __forceinline__ void stats_chunk(StatsAcc &acc, const T *src, int len, int lane) {
    constexpr int P = 16 / (int)sizeof(T);
    const bool aligned = ((uintptr_t)src & 15u) == 0;
    const int pieces = (len + P - 1) / P;
    for (int q = lane; q < pieces; q += 64) {
        const int i0 = q * P;
        if (aligned && i0 + P <= len) {
            const FV<P> x = loadv<NT, P, false>(src + i0);
#pragma unroll
            for (int e = 0; e < P; ++e) stats_take(acc, x.v[e]);
        } else {
            const int i1 = i0 + P < len ? i0 + P : len;
            for (int i = i0; i < i1; ++i) stats_take(acc, load1(src + i));
        }
    }
}

// Butterfly over the 64 lanes, then the wavefronts' values in wavefront order (thread 0 holds the result).
template <int WAVES>
__device__ __forceinline__ void stats_combine_workgroup(StatsAcc &acc, unsigned long long &bad) {
    __shared__ unsigned long long s_bad[WAVES];
    __shared__ float s_mx[WAVES];
    __shared__ double s_ss[WAVES];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        bad += __shfl_xor(bad, off);
        acc.mx = fmaxf(acc.mx, __shfl_xor(acc.mx, off));
        acc.ss = acc.ss + __shfl_xor(acc.ss, off);
    }
    if (lane == 0) {
        s_bad[wave] = bad;
        s_mx[wave] = acc.mx;
        s_ss[wave] = acc.ss;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < WAVES; ++w) {
            bad += s_bad[w];
            acc.mx = fmaxf(acc.mx, s_mx[w]);
            acc.ss = acc.ss + s_ss[w];
        }
    }
}

template <typename T, int NT>
__global__ __launch_bounds__(STATS_WAVES * 64) void pxchg_stats_partial_kernel(const PxChunk *__restrict__ chunks, int n_chunks,
                                                                               const void *const *set,
                                                                               pxchg_stats *__restrict__ partials) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // the same in all 64 lanes: keep it scalar
    constexpr bool F32 = std::is_same<T, float>::value;
#ifdef PX_STATS_TRIP
    constexpr int G = PX_STATS_TRIP;  // chunks per trip (tuning)
#else
    constexpr int G = F32 ? 1 : 2;  // chunks per trip
#endif
    const int n_blocks = (n_chunks + STATS_BLOCK_CHUNKS - 1) / STATS_BLOCK_CHUNKS;
    for (int b = blockIdx.x; b < n_blocks; b += gridDim.x) {
        const int first = b * STATS_BLOCK_CHUNKS;
        const int count = n_chunks - first < STATS_BLOCK_CHUNKS ? n_chunks - first : STATS_BLOCK_CHUNKS;
        StatsAcc acc = {0u, 0.0f, 0.0};
        // this wavefront's chunks: places wave, wave + WAVES, ... of the block, G of them per trip
        for (int j0 = wave; j0 < count; j0 += STATS_WAVES * G) {
            const T *src[G];
            int len[G];
            bool whole = true;  // uniform over the wavefront
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const int j = j0 + g * STATS_WAVES;
                if (j < count) {
                    const PxChunk ch = chunks[first + j];
                    src[g] = table_ptr<const T>(set, ch.tensor) + ch.start;
                    len[g] = ch.len;
                    whole = whole && ch.len == 512 && ((uintptr_t)src[g] & 15u) == 0;
                } else {
                    len[g] = 0;
                    whole = false;
                }
            }
            if (whole) {
                FV<8> x[G];
#pragma unroll
                for (int g = 0; g < G; ++g) x[g] = loadv<NT, 8, F32>(src[g] + (F32 ? 4 : 8) * lane);
#pragma unroll
                for (int g = 0; g < G; ++g)
#pragma unroll
                    for (int e = 0; e < 8; ++e) stats_take(acc, x[g].v[e]);
            } else {
#pragma unroll
                for (int g = 0; g < G; ++g)
                    if (len[g] > 0) stats_chunk<T, NT>(acc, src[g], len[g], lane);
            }
        }
        unsigned long long bad = acc.bad;
        __syncthreads();  // the previous block's reader of the shared arrays is done
        stats_combine_workgroup<STATS_WAVES>(acc, bad);
        if (threadIdx.x == 0) {
            pxchg_stats r;
            r.nonfinite = bad;
            r.sum_sq = acc.ss;
            r.max_abs = acc.mx;
            r.reserved = 0;
            partials[b] = r;
        }
    }
}

// One workgroup: thread t takes partial results t, t + T, ... in that order, then the same tree as above.
// With no partial result at all (an empty table) it writes zeros.
__global__ __launch_bounds__(STATS_COMBINE_THREADS) void pxchg_stats_combine_kernel(const pxchg_stats *__restrict__ partials,
                                                                                    int n_partials, pxchg_stats *out) {
    StatsAcc acc = {0u, 0.0f, 0.0};
    unsigned long long bad = 0;
    for (int i = threadIdx.x; i < n_partials; i += STATS_COMBINE_THREADS) {
        const pxchg_stats p = partials[i];
        bad += p.nonfinite;
        acc.mx = fmaxf(acc.mx, p.max_abs);
        acc.ss = acc.ss + p.sum_sq;
    }
    stats_combine_workgroup<STATS_COMBINE_THREADS / 64>(acc, bad);
    if (threadIdx.x == 0) {
        pxchg_stats r;
        r.nonfinite = bad;
        r.sum_sq = acc.ss;
        r.max_abs = acc.mx;
        r.reserved = 0;
        *out = r;
    }
}

// ---------------------------------------------------------------- launch helpers

// Launches through the runtime's C entry point, whose return value is the status of THIS launch: the call
// neither reads nor clears whatever error an earlier HIP call of the process may have left behind.
template <typename... P, typename... A>
int px_launch(void (*kernel)(P...), dim3 grid, dim3 block, hipStream_t stream, A... args) {
    static_assert(sizeof...(P) == sizeof...(A), "one argument per kernel parameter");
    std::tuple<P...> params{args...};
    void *argv[sizeof...(P)];
    int i = 0;
    std::apply([&](auto &...p) { ((argv[i++] = (void *)&p), ...); }, params);
    return hipLaunchKernel((const void *)kernel, grid, block, argv, 0, stream) == hipSuccess ? PXCHG_OK : PXCHG_ERR_RUNTIME;
}

// Cache policies: 0 plain; bit 0 non-temporal loads, bit 1 non-temporal stores; 4 non-temporal loads with
// "sc1 nt" stores; 5 non-temporal loads with "sc1" stores.  Measured on MI355X (AlexNet-shaped set, k = 8),
// A/B inside one run:
//   * the non-temporal hint on loads helps every kernel (+10..17 %);
//   * the reduce (one written byte in nine) and the widening unpack are fastest with agent-scope stores without
//     the streaming hint (policy 5: +3..4 % over plain stores, +7 % over non-temporal stores);
//   * pack, the update with a binary16 gradient, the single elastic meeting and the fused elastic round of
//     three or more workers are fastest with agent-scope streaming stores (policy 4: +1..3 % over plain
//     non-temporal stores);
//   * the update with a binary32 gradient, the fused reduce+update and the fused round of two are fastest with
//     plain non-temporal stores (policy 3; policy 4 is 0..3 % slower there).
// The regular build compiles each kernel with its own policy and with policy 0; a tuning build
// (-DPXCHG_ALL_POLICIES) compiles all six for every kernel, which is what the comparisons above were made with.
constexpr int NT_BOTH = 3, NT_LOADS_SC1NT_STORES = 4, NT_LOADS_SC1_STORES = 5;

// Expands CALL(n) for the policy to use: the caller's choice (PXCHG_OPT_NONTEMPORAL) if set, else OWN.
#ifdef PXCHG_ALL_POLICIES
#define PX_DISPATCH_NT(OWN, CALL)                     \
    switch (policy_for(t, OWN)) {                     \
        case 0: return CALL(0);                       \
        case 1: return CALL(1);                       \
        case 2: return CALL(2);                       \
        case 3: return CALL(3);                       \
        case 4: return CALL(4);                       \
        default: return CALL(5);                      \
    }
#else
#define PX_DISPATCH_NT(OWN, CALL)                     \
    if (policy_for(t, OWN) == 0) return CALL(0);      \
    return CALL(OWN);
#endif

int policy_for(const pxchg_table *t, int own) {  // `t`: the table of the call (every launcher names it so)
    const int64_t nt = px_nontemporal_for(t);
    return nt < 0 ? own : (int)nt;
}

dim3 grid_for(const pxchg_table *t, int64_t n_virtual) {
    const int64_t bpc = px_options().blocks_per_cu;
    int64_t g = std::min<int64_t>(n_virtual, (int64_t)1 << 24);  // the kernels loop over what is left
    if (bpc > 0) g = std::min<int64_t>(g, (int64_t)px_cu_count(t->device) * bpc);
    return dim3((unsigned)g, 1, 1);
}

int check_table(const pxchg_table *t) {
    if (!px_valid(t)) return PXCHG_ERR_INVALID_ARG;
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device != t->device) return PXCHG_ERR_NO_DEVICE;
    return PXCHG_OK;
}

int check_set(const pxchg_table *t, const pxchg_bufset *s, int dtype /* -1: either */) {
    if (!px_valid(s)) return PXCHG_ERR_INVALID_ARG;
    const pxchg_table *root = px_root(t);  // a view takes its parent's sets
    if (s->table != root || s->table_id != root->id) return PXCHG_ERR_SHAPE_MISMATCH;
    if (dtype >= 0 && s->dtype != dtype) return PXCHG_ERR_SHAPE_MISMATCH;
    return PXCHG_OK;
}

bool is_pow2(int k) { return k > 0 && (k & (k - 1)) == 0; }

using Shared = std::shared_lock<std::shared_mutex>;

template <typename TI, typename TO>
int launch_convert(const pxchg_table *t, int k, const pxchg_bufset *const *src, pxchg_bufset *const *dst,
                   int src_dtype, int dst_dtype, hipStream_t stream) {
    Shared lock(px_registry_lock());
    int rc = check_table(t);
    if (rc) return rc;
    if (!src || !dst) return PXCHG_ERR_INVALID_ARG;
    if (k < 1 || k > PXCHG_MAX_K) return PXCHG_ERR_UNSUPPORTED;
    ConvertArgs a;
    for (int i = 0; i < k; ++i) {
        if ((rc = check_set(t, src[i], src_dtype))) return rc;
        if ((rc = check_set(t, dst[i], dst_dtype))) return rc;
        a.src[i] = (const void *const *)src[i]->d_ptrs;
        a.dst[i] = (void *const *)dst[i]->d_ptrs;
    }
    for (int i = 0; i < k; ++i)
        for (int j = i + 1; j < k; ++j)
            if (dst[i] == dst[j]) return PXCHG_ERR_INVALID_ARG;
    if (t->n_chunks == 0) return PXCHG_OK;
    const int64_t n_virtual = t->n_chunks * k * convert_parts();
    const dim3 grid = grid_for(t, n_virtual);
    const int part_elems = (int)(t->chunk_elems / convert_parts());
    constexpr int OWN = sizeof(TO) < sizeof(TI) ? NT_LOADS_SC1NT_STORES : NT_LOADS_SC1_STORES;
#define PX_CALL(N)                                                                                                      \
    px_launch(pxchg_convert_kernel<TI, TO, N>, grid, dim3(convert_lanes()), stream, (const PxChunk *)t->d_chunks, (int)t->n_chunks, \
              n_virtual, a, part_elems)
    PX_DISPATCH_NT(OWN, PX_CALL)
#undef PX_CALL
}

#ifndef PXCHG_TUNE_REDUCE_POLICY  // A/B builds only: the reduce's own store policy (3, 4 or 5)
#define PXCHG_TUNE_REDUCE_POLICY NT_LOADS_SC1_STORES
#endif

// A table (or view) of many small tensors: at most 512 chunks per tensor on average.  Two launch choices follow it.
// The reduce fetches its pointers lane-parallel on such tables (measured: better up to 204 chunks per tensor, level
// at 1027, worse from 7400 on); the fused reduce+update has an idle wavefront on the others (better from 1027
// chunks per tensor on, level at 233, worse at 58 and below).
bool small_tensors(const pxchg_table *t) { return t->n_chunks <= (int64_t)512 * t->n_tensors; }

// A table (or view) of large tensors: at least 4096 chunks per tensor on average (2 M elements at the default chunk
// size).  The binary16 reduce runs with idle wavefronts on such tables (measured: better at 7400 and 8400 chunks
// per tensor and on single tensors, worse at 1027 and below).
bool large_tensors(const pxchg_table *t) { return t->n_chunks >= (int64_t)4096 * t->n_tensors; }

int reduce_mode(const pxchg_table *t) {
#ifdef PXCHG_TUNE_REDUCE_POINTERS  // A/B builds only: 0 scalar loads on every table, 1 lane-parallel on every table
    return PXCHG_TUNE_REDUCE_POINTERS != 0 ? REDUCE_LANE_POINTERS : REDUCE_PLAIN;
#else
    return small_tensors(t) ? REDUCE_LANE_POINTERS : large_tensors(t) ? REDUCE_IDLE_WAVEFRONTS : REDUCE_PLAIN;
#endif
}

template <int K, typename TI, typename TO, int MODE>
int launch_reduce_km(const pxchg_table *t, const ReduceArgs &a, hipStream_t stream) {
    constexpr int PARTS = reduce_parts<K, touches_f32<TI, TO>()>();
    const dim3 grid = grid_for(t, t->n_chunks * PARTS);
    const int part_elems = (int)(t->chunk_elems / PARTS);
#define PX_CALL(N)                                                                                                \
    px_launch(pxchg_reduce_avg_kernel<K, TI, TO, N, MODE>, grid, dim3(reduce_threads<K, TI, TO, MODE>()), stream, \
              (const PxChunk *)t->d_chunks, (int)t->n_chunks, a, part_elems)
    PX_DISPATCH_NT(PXCHG_TUNE_REDUCE_POLICY, PX_CALL)
#undef PX_CALL
}

template <int K, typename TI, typename TO>
int launch_reduce_k(const pxchg_table *t, const ReduceArgs &a, hipStream_t stream) {
    const int mode = reduce_mode(t);
    if (mode == REDUCE_LANE_POINTERS) return launch_reduce_km<K, TI, TO, REDUCE_LANE_POINTERS>(t, a, stream);
    if constexpr (!touches_f32<TI, TO>() && K >= 4) {  // the only kernels whose shape the third mode changes
        if (mode == REDUCE_IDLE_WAVEFRONTS) return launch_reduce_km<K, TI, TO, REDUCE_IDLE_WAVEFRONTS>(t, a, stream);
    }
    return launch_reduce_km<K, TI, TO, REDUCE_PLAIN>(t, a, stream);
}

template <typename TI, typename TO>
int launch_reduce_anyk(const pxchg_table *t, const ReduceArgs &a, hipStream_t stream) {
    const dim3 grid = grid_for(t, t->n_chunks);
#define PX_CALL(N)                                                                                                            \
    px_launch(pxchg_reduce_avg_anyk_kernel<TI, TO, N>, grid, dim3(reduce_lanes<0, TI, TO>()), stream, (const PxChunk *)t->d_chunks, \
              (int)t->n_chunks, a)
    PX_DISPATCH_NT(NT_LOADS_SC1_STORES, PX_CALL)
#undef PX_CALL
}

template <typename TI, typename TO>
int launch_reduce(const pxchg_table *t, int k, const ReduceArgs &a, hipStream_t stream) {
    switch (k) {
        case 1: return launch_reduce_k<1, TI, TO>(t, a, stream);
        case 2: return launch_reduce_k<2, TI, TO>(t, a, stream);
        case 3: return launch_reduce_k<3, TI, TO>(t, a, stream);
        case 4: return launch_reduce_k<4, TI, TO>(t, a, stream);
        case 5: return launch_reduce_k<5, TI, TO>(t, a, stream);
        case 6: return launch_reduce_k<6, TI, TO>(t, a, stream);
        case 7: return launch_reduce_k<7, TI, TO>(t, a, stream);
        case 8: return launch_reduce_k<8, TI, TO>(t, a, stream);
        default: return launch_reduce_anyk<TI, TO>(t, a, stream);
    }
}

template <int K, typename TI, bool WIRE16, bool IDLE>
int launch_fused_ki(const pxchg_table *t, const FusedArgs &a, hipStream_t stream) {
    const dim3 grid = grid_for(t, t->n_chunks * fused_parts<K>());
    const int part_elems = (int)(t->chunk_elems / fused_parts<K>());
#define PX_CALL(N)                                                                                                        \
    px_launch(pxchg_reduce_avg_sgd_momentum_kernel<K, TI, WIRE16, N, IDLE>, grid, dim3(fused_threads<K, TI, IDLE>()), stream, \
              (const PxChunk *)t->d_chunks, (int)t->n_chunks, a, part_elems)
    PX_DISPATCH_NT(NT_BOTH, PX_CALL)
#undef PX_CALL
}

template <int K, typename TI, bool WIRE16>
int launch_fused_k(const pxchg_table *t, const FusedArgs &a, hipStream_t stream) {
    if constexpr (K >= 3) {
        if (!small_tensors(t)) return launch_fused_ki<K, TI, WIRE16, true>(t, a, stream);
    }
    return launch_fused_ki<K, TI, WIRE16, false>(t, a, stream);
}

template <typename TI, bool WIRE16>
int launch_fused_anyk(const pxchg_table *t, const FusedArgs &a, hipStream_t stream) {
    const dim3 grid = grid_for(t, t->n_chunks);
#define PX_CALL(N)                                                                                     \
    px_launch(pxchg_reduce_avg_sgd_momentum_anyk_kernel<TI, WIRE16, N>, grid, dim3(128), stream, \
              (const PxChunk *)t->d_chunks, (int)t->n_chunks, a)
    PX_DISPATCH_NT(NT_BOTH, PX_CALL)
#undef PX_CALL
}

template <typename TI, bool WIRE16>
int launch_fused(const pxchg_table *t, int k, const FusedArgs &a, hipStream_t stream) {
    switch (k) {
        case 1: return launch_fused_k<1, TI, WIRE16>(t, a, stream);
        case 2: return launch_fused_k<2, TI, WIRE16>(t, a, stream);
        case 3: return launch_fused_k<3, TI, WIRE16>(t, a, stream);
        case 4: return launch_fused_k<4, TI, WIRE16>(t, a, stream);
        case 5: return launch_fused_k<5, TI, WIRE16>(t, a, stream);
        case 6: return launch_fused_k<6, TI, WIRE16>(t, a, stream);
        case 7: return launch_fused_k<7, TI, WIRE16>(t, a, stream);
        case 8: return launch_fused_k<8, TI, WIRE16>(t, a, stream);
        default: return launch_fused_anyk<TI, WIRE16>(t, a, stream);
    }
}

template <int K, bool CR>
int launch_elastic_kc(const pxchg_table *t, const ElasticArgs &a, hipStream_t stream) {
    const dim3 grid = grid_for(t, t->n_chunks * elastic_parts<K, CR>());
    ElasticArgs b = a;
    b.part_elems = (int)(t->chunk_elems / elastic_parts<K, CR>());  // elements per workgroup
    constexpr int OWN = K == 2 ? NT_BOTH : NT_LOADS_SC1NT_STORES;
#define PX_CALL(N)                                                                                                      \
    px_launch(pxchg_easgd_kernel<K, N, CR>, grid, dim3(elastic_lanes<K, CR>() * elastic_pad<K, CR>()), stream, (const PxChunk *)t->d_chunks, \
              (int)t->n_chunks, b)
    PX_DISPATCH_NT(OWN, PX_CALL)
#undef PX_CALL
}

template <int K>
int launch_elastic_k(const pxchg_table *t, const ElasticArgs &a, hipStream_t stream) {
    // a center larger than the 256 MiB memory-side cache cannot stay there (measured 2.5 % slower at 553 MB)
    if (px_center_resident_for(t) && t->total * 4 <= ((int64_t)256 << 20)) return launch_elastic_kc<K, true>(t, a, stream);
    return launch_elastic_kc<K, false>(t, a, stream);
}

template <typename TG>
int launch_update(const pxchg_table *t, const UpdateArgs &a, hipStream_t stream) {
    const dim3 grid = grid_for(t, t->n_chunks * update_parts());
    const int part_elems = (int)(t->chunk_elems / update_parts());
    constexpr int OWN = std::is_same<TG, _Float16>::value ? NT_LOADS_SC1NT_STORES : NT_BOTH;
#define PX_CALL(N)                                                                                                          \
    px_launch(pxchg_sgd_momentum_kernel<TG, N>, grid, dim3(update_lanes<TG>()), stream, (const PxChunk *)t->d_chunks, (int)t->n_chunks, a, \
              part_elems)
    PX_DISPATCH_NT(OWN, PX_CALL)
#undef PX_CALL
}

void fill_scale(int k, int mode, int *use_div, float *kf, float *scale) {
    *kf = (float)k;
    if (mode == PXCHG_SUM) {
        *use_div = 0;
        *scale = 1.0f;
    } else if (is_pow2(k)) {
        *use_div = 0;
        *scale = 1.0f / (float)k;  // exact
    } else {
        *use_div = 1;
        *scale = 1.0f;
    }
}

// Partial results for pxchg_buffer_stats_static: memory that exists from the moment the code object is loaded,
// so that the call has nothing to allocate.  One copy per GPU, at its own address on each, looked up once per
// device with that device current and kept; host code never uses the array's name for anything else (the name
// is only a host-side stand-in, not a device address).
static __device__ __align__(256) pxchg_stats scratch[PXCHG_STATS_STATIC_MAX_BLOCKS];
constexpr int PX_MAX_DEVICES = 64;
std::atomic<pxchg_stats *> scratch_ptr[PX_MAX_DEVICES];

// The current device's copy of `scratch`; `device` must be the current device.
int static_scratch(int device, pxchg_stats **out) {
    if (device < 0 || device >= PX_MAX_DEVICES) return PXCHG_ERR_UNSUPPORTED;
    pxchg_stats *p = scratch_ptr[device].load(std::memory_order_acquire);
    if (!p) {
        void *addr = nullptr;
        if (hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch)) != hipSuccess || !addr) return PXCHG_ERR_RUNTIME;
        p = (pxchg_stats *)addr;
        scratch_ptr[device].store(p, std::memory_order_release);  // every thread finds the same address
    }
    *out = p;
    return PXCHG_OK;
}

// The two launches of the diagnostics; `partials` has room for one result per block of the table's chunk list.
int launch_stats(const pxchg_table *table, const pxchg_bufset *set, pxchg_stats *partials, pxchg_stats *out,
                 hipStream_t stream) {
    const int n_blocks = (int)px_stats_blocks(table->n_chunks);
    if (n_blocks > 0) {
        const void *const *ptrs = (const void *const *)set->d_ptrs;
        const dim3 grid((unsigned)n_blocks), block(STATS_WAVES * 64);
        const int rc = set->dtype == PXCHG_F32
                           ? px_launch(pxchg_stats_partial_kernel<float, 1>, grid, block, stream, (const PxChunk *)table->d_chunks,
                                       (int)table->n_chunks, ptrs, partials)
                           : px_launch(pxchg_stats_partial_kernel<_Float16, 1>, grid, block, stream,
                                       (const PxChunk *)table->d_chunks, (int)table->n_chunks, ptrs, partials);
        if (rc) return rc;
    }
    return px_launch(pxchg_stats_combine_kernel, dim3(1), dim3(STATS_COMBINE_THREADS), stream, (const pxchg_stats *)partials,
                     n_blocks, out);
}

}  // namespace

int px_prepare_static_scratch(int device) {
    pxchg_stats *p = nullptr;
    return static_scratch(device, &p);
}

int px_all_policies_built() {
#ifdef PXCHG_ALL_POLICIES
    return 1;
#else
    return 0;
#endif
}

extern "C" {

int pxchg_pack_fp16(const pxchg_table *table, int k, const pxchg_bufset *const *src_f32, pxchg_bufset *const *dst_f16,
                    void *stream) {
    return launch_convert<float, _Float16>(table, k, src_f32, dst_f16, PXCHG_F32, PXCHG_F16, (hipStream_t)stream);
}

int pxchg_unpack_fp16(const pxchg_table *table, int k, const pxchg_bufset *const *src_f16, pxchg_bufset *const *dst_f32,
                      void *stream) {
    return launch_convert<_Float16, float>(table, k, src_f16, dst_f32, PXCHG_F16, PXCHG_F32, (hipStream_t)stream);
}

int pxchg_reduce_avg(const pxchg_table *table, int k, const pxchg_bufset *const *contrib, pxchg_bufset *out, int mode,
                     void *stream) {
    Shared lock(px_registry_lock());
    int rc = check_table(table);
    if (rc) return rc;
    if (!contrib) return PXCHG_ERR_INVALID_ARG;
    if (mode != PXCHG_AVG && mode != PXCHG_SUM) return PXCHG_ERR_INVALID_ARG;
    if (k < 1 || k > PXCHG_MAX_K) return PXCHG_ERR_UNSUPPORTED;
    if ((rc = check_set(table, out, -1))) return rc;
    if ((rc = check_set(table, contrib[0], -1))) return rc;
    const int in_dtype = contrib[0]->dtype;
    ReduceArgs a;
    for (int i = 0; i < k; ++i) {
        if ((rc = check_set(table, contrib[i], in_dtype))) return rc;
        a.contrib[i] = (const void *const *)contrib[i]->d_ptrs;
    }
    a.out = (void *const *)out->d_ptrs;
    a.k = k;
    fill_scale(k, mode, &a.use_div, &a.kf, &a.scale);
    if (table->n_chunks == 0) return PXCHG_OK;
    hipStream_t s = (hipStream_t)stream;
    if (in_dtype == PXCHG_F32 && out->dtype == PXCHG_F32) return launch_reduce<float, float>(table, k, a, s);
    if (in_dtype == PXCHG_F32) return launch_reduce<float, _Float16>(table, k, a, s);
    if (out->dtype == PXCHG_F32) return launch_reduce<_Float16, float>(table, k, a, s);
    return launch_reduce<_Float16, _Float16>(table, k, a, s);
}

int pxchg_sgd_momentum(const pxchg_table *table, const pxchg_bufset *grad, pxchg_bufset *param, pxchg_bufset *vel,
                       float lr, float mu, float wd, void *stream) {
    Shared lock(px_registry_lock());
    int rc = check_table(table);
    if (rc) return rc;
    if ((rc = check_set(table, grad, -1))) return rc;
    if ((rc = check_set(table, param, PXCHG_F32))) return rc;
    if ((rc = check_set(table, vel, PXCHG_F32))) return rc;
    if (param == vel || (const pxchg_bufset *)param == grad || (const pxchg_bufset *)vel == grad)
        return PXCHG_ERR_INVALID_ARG;
    if (table->n_chunks == 0) return PXCHG_OK;
    UpdateArgs a;
    a.grad = (const void *const *)grad->d_ptrs;
    a.param = (void *const *)param->d_ptrs;
    a.vel = (void *const *)vel->d_ptrs;
    a.mult = px_root(table)->d_mult;
    a.lr = lr;
    a.mu = mu;
    a.wd = wd;
    hipStream_t s = (hipStream_t)stream;
    if (grad->dtype == PXCHG_F32) return launch_update<float>(table, a, s);
    return launch_update<_Float16>(table, a, s);
}

int pxchg_reduce_avg_sgd_momentum(const pxchg_table *table, int k, const pxchg_bufset *const *contrib, int mode,
                                  int wire_dtype, pxchg_bufset *param, pxchg_bufset *vel, float lr, float mu, float wd,
                                  void *stream) {
    Shared lock(px_registry_lock());
    int rc = check_table(table);
    if (rc) return rc;
    if (!contrib) return PXCHG_ERR_INVALID_ARG;
    if (mode != PXCHG_AVG && mode != PXCHG_SUM) return PXCHG_ERR_INVALID_ARG;
    if (wire_dtype != PXCHG_F32 && wire_dtype != PXCHG_F16) return PXCHG_ERR_INVALID_ARG;
    if (k < 1 || k > PXCHG_MAX_K) return PXCHG_ERR_UNSUPPORTED;
    if ((rc = check_set(table, param, PXCHG_F32))) return rc;
    if ((rc = check_set(table, vel, PXCHG_F32))) return rc;
    if (param == vel) return PXCHG_ERR_INVALID_ARG;
    if ((rc = check_set(table, contrib[0], -1))) return rc;
    const int in_dtype = contrib[0]->dtype;
    FusedArgs a;
    for (int i = 0; i < k; ++i) {
        if ((rc = check_set(table, contrib[i], in_dtype))) return rc;
        if (contrib[i] == (const pxchg_bufset *)param || contrib[i] == (const pxchg_bufset *)vel)
            return PXCHG_ERR_INVALID_ARG;
        a.contrib[i] = (const void *const *)contrib[i]->d_ptrs;
    }
    a.param = (void *const *)param->d_ptrs;
    a.vel = (void *const *)vel->d_ptrs;
    a.mult = px_root(table)->d_mult;
    a.k = k;
    fill_scale(k, mode, &a.use_div, &a.kf, &a.scale);
    a.lr = lr;
    a.mu = mu;
    a.wd = wd;
    if (table->n_chunks == 0) return PXCHG_OK;
    hipStream_t s = (hipStream_t)stream;
    const bool wire16 = wire_dtype == PXCHG_F16;
    if (in_dtype == PXCHG_F32) return wire16 ? launch_fused<float, true>(table, k, a, s) : launch_fused<float, false>(table, k, a, s);
    return wire16 ? launch_fused<_Float16, true>(table, k, a, s) : launch_fused<_Float16, false>(table, k, a, s);
}

int pxchg_easgd_round(const pxchg_table *table, int k, pxchg_bufset *const *x, pxchg_bufset *c, float alpha,
                      void *stream) {
    Shared lock(px_registry_lock());
    int rc = check_table(table);
    if (rc) return rc;
    if (!x) return PXCHG_ERR_INVALID_ARG;
    if (k < 1 || k > PXCHG_MAX_K) return PXCHG_ERR_UNSUPPORTED;
    if ((rc = check_set(table, c, PXCHG_F32))) return rc;
    for (int i = 0; i < k; ++i) {
        if ((rc = check_set(table, x[i], PXCHG_F32))) return rc;
        if (x[i] == c) return PXCHG_ERR_INVALID_ARG;
        for (int j = 0; j < i; ++j)
            if (x[i] == x[j]) return PXCHG_ERR_INVALID_ARG;
    }
    if (table->n_chunks == 0) return PXCHG_OK;
    hipStream_t s = (hipStream_t)stream;
    // More than 8 workers: successive launches of up to 8, the center carried
    // through memory between them (same arithmetic, same order).
    for (int i0 = 0; i0 < k; i0 += 8) {
        const int kk = std::min(8, k - i0);
        ElasticArgs a;
        for (int i = 0; i < kk; ++i) a.x[i] = (void *const *)x[i0 + i]->d_ptrs;
        a.c = (void *const *)c->d_ptrs;
        a.k = kk;
        a.alpha = alpha;
        a.part_elems = 0;  // set per kernel shape at the launch
        switch (kk) {
            case 1: rc = launch_elastic_k<1>(table, a, s); break;
            case 2: rc = launch_elastic_k<2>(table, a, s); break;
            case 3: rc = launch_elastic_k<3>(table, a, s); break;
            case 4: rc = launch_elastic_k<4>(table, a, s); break;
            case 5: rc = launch_elastic_k<5>(table, a, s); break;
            case 6: rc = launch_elastic_k<6>(table, a, s); break;
            case 7: rc = launch_elastic_k<7>(table, a, s); break;
            default: rc = launch_elastic_k<8>(table, a, s); break;
        }
        if (rc) return rc;
    }
    return PXCHG_OK;
}

int pxchg_easgd(const pxchg_table *table, pxchg_bufset *x, pxchg_bufset *c, float alpha, void *stream) {
    pxchg_bufset *xs[1] = {x};
    return pxchg_easgd_round(table, 1, xs, c, alpha, stream);
}

int pxchg_buffer_stats(const pxchg_table *table, const pxchg_bufset *set, pxchg_stats *out, void *stream) {
    Shared lock(px_registry_lock());
    int rc = check_table(table);
    if (rc) return rc;
    if ((rc = check_set(table, set, -1))) return rc;
    if (!out || ((uintptr_t)out & 7u)) return PXCHG_ERR_INVALID_ARG;
    return launch_stats(table, set, px_root(table)->d_partials, out, (hipStream_t)stream);
}

int pxchg_buffer_stats_static(const pxchg_table *table, const pxchg_bufset *set, pxchg_stats *out, void *stream) {
    Shared lock(px_registry_lock());
    int rc = check_table(table);
    if (rc) return rc;
    if ((rc = check_set(table, set, -1))) return rc;
    if (!out || ((uintptr_t)out & 7u)) return PXCHG_ERR_INVALID_ARG;
    if (px_stats_blocks(table->n_chunks) > PXCHG_STATS_STATIC_MAX_BLOCKS) return PXCHG_ERR_UNSUPPORTED;
    pxchg_stats *partials = nullptr;
    if ((rc = static_scratch(table->device, &partials))) return rc;  // the table's device is the current one
    return launch_stats(table, set, partials, out, (hipStream_t)stream);
}

}  // extern "C"
