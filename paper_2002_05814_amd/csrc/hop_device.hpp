// Device code of the gfx950 reduce and copy kernels (templates), shared by the
// library's launchers. See hop_kernels.hip for what the kernels are for.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hop_kernels.h"

namespace hop {

// ----------------------------------------------------------------------------
// element types
// ----------------------------------------------------------------------------

template <int DT> struct Traits;
template <> struct Traits<HOP_F32>  { using acc_t = float;   static constexpr int W = 4; static constexpr int ES = 4; };
template <> struct Traits<HOP_BF16> { using acc_t = float;   static constexpr int W = 8; static constexpr int ES = 2; };
template <> struct Traits<HOP_I32>  { using acc_t = int32_t; static constexpr int W = 4; static constexpr int ES = 4; };

__device__ __forceinline__ float bits_to_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t f32_to_bits(float f) { return __builtin_bit_cast(uint32_t, f); }

// binary32 -> bfloat16 bits, round to nearest, ties to even; NaN stays a quiet NaN. As a formula:
//     u = bits(f); NaN ? (u >> 16) | 0x0040 : (u + 0x7fff + ((u >> 16) & 1)) >> 16
// gfx950 has an instruction for it (v_cvt_pk_bf16_f32, which the compiler selects for a conversion
// to __bf16); it returns the formula's value for every one of the 2^32 inputs (swept on the device),
// at one instruction per two values instead of about seven per value.
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f);
}
// two values: lo in bits 0..15, hi in bits 16..31
__device__ __forceinline__ uint32_t f32x2_to_bf16x2_bits(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

template <int OP> __device__ __forceinline__ float combine(float a, float b)
{
    if (OP == HOP_SUM) return a + b;
    if (OP == HOP_MIN) return (b < a) ? b : a;
    return (b > a) ? b : a;
}
template <int OP> __device__ __forceinline__ int32_t combine(int32_t a, int32_t b)
{
    if (OP == HOP_SUM) return (int32_t)((uint32_t)a + (uint32_t)b);   // wraps mod 2^32
    if (OP == HOP_MIN) return (b < a) ? b : a;
    return (b > a) ? b : a;
}

// 16 raw bytes <-> W accumulator-typed values
template <int DT> __device__ __forceinline__ void decode(const uint4 &r, typename Traits<DT>::acc_t *x);
template <> __device__ __forceinline__ void decode<HOP_F32>(const uint4 &r, float *x)
{
    x[0] = bits_to_f32(r.x); x[1] = bits_to_f32(r.y); x[2] = bits_to_f32(r.z); x[3] = bits_to_f32(r.w);
}
template <> __device__ __forceinline__ void decode<HOP_I32>(const uint4 &r, int32_t *x)
{
    x[0] = (int32_t)r.x; x[1] = (int32_t)r.y; x[2] = (int32_t)r.z; x[3] = (int32_t)r.w;
}
template <> __device__ __forceinline__ void decode<HOP_BF16>(const uint4 &r, float *x)
{
    // element 2i is the low half of word i (little endian); widening is exact
    x[0] = bits_to_f32(r.x << 16); x[1] = bits_to_f32(r.x & 0xffff0000u);
    x[2] = bits_to_f32(r.y << 16); x[3] = bits_to_f32(r.y & 0xffff0000u);
    x[4] = bits_to_f32(r.z << 16); x[5] = bits_to_f32(r.z & 0xffff0000u);
    x[6] = bits_to_f32(r.w << 16); x[7] = bits_to_f32(r.w & 0xffff0000u);
}

template <int DT> __device__ __forceinline__ uint4 encode(const typename Traits<DT>::acc_t *x);
template <> __device__ __forceinline__ uint4 encode<HOP_F32>(const float *x)
{
    return make_uint4(f32_to_bits(x[0]), f32_to_bits(x[1]), f32_to_bits(x[2]), f32_to_bits(x[3]));
}
template <> __device__ __forceinline__ uint4 encode<HOP_I32>(const int32_t *x)
{
    return make_uint4((uint32_t)x[0], (uint32_t)x[1], (uint32_t)x[2], (uint32_t)x[3]);
}
template <> __device__ __forceinline__ uint4 encode<HOP_BF16>(const float *x)
{
    return make_uint4(f32x2_to_bf16x2_bits(x[0], x[1]), f32x2_to_bf16x2_bits(x[2], x[3]),
                      f32x2_to_bf16x2_bits(x[4], x[5]), f32x2_to_bf16x2_bits(x[6], x[7]));
}

// one element (the ragged tail of an object whose size is not a multiple of 16 bytes)
template <int DT> __device__ __forceinline__ typename Traits<DT>::acc_t load_elem(const void *p, size_t byte_off);
template <> __device__ __forceinline__ float load_elem<HOP_F32>(const void *p, size_t o) { return *(const float *)((const char *)p + o); }
template <> __device__ __forceinline__ int32_t load_elem<HOP_I32>(const void *p, size_t o) { return *(const int32_t *)((const char *)p + o); }
template <> __device__ __forceinline__ float load_elem<HOP_BF16>(const void *p, size_t o)
{
    return bits_to_f32((uint32_t)(*(const uint16_t *)((const char *)p + o)) << 16);
}
template <int DT> __device__ __forceinline__ void store_elem(void *p, size_t byte_off, typename Traits<DT>::acc_t v);
template <> __device__ __forceinline__ void store_elem<HOP_F32>(void *p, size_t o, float v) { *(float *)((char *)p + o) = v; }
template <> __device__ __forceinline__ void store_elem<HOP_I32>(void *p, size_t o, int32_t v) { *(int32_t *)((char *)p + o) = v; }
template <> __device__ __forceinline__ void store_elem<HOP_BF16>(void *p, size_t o, float v)
{
    *(uint16_t *)((char *)p + o) = (uint16_t)f32_to_bf16_bits(v);
}

// ----------------------------------------------------------------------------
// the accumulator machine: D partial results of W values each, all in VGPRs.
// Program steps are wave-uniform (scalar loads, scalar branches); every index
// into acc[][] is a compile-time constant after unrolling.
// ----------------------------------------------------------------------------

template <int DT, int OP, int D, int W>
struct Machine {
    using A = typename Traits<DT>::acc_t;
    A acc[D][W];

    __device__ __forceinline__ void step(uint32_t ctl, const A (&x)[W])
    {
        uint32_t level = ctl & 0xffu;
        const bool set = (ctl >> 8) & 1u;
        uint32_t n_fold = ctl >> 16;
#pragma unroll
        for (int L = 0; L < D; ++L) {
            if (level == (uint32_t)L) {
                if (set) {
#pragma unroll
                    for (int w = 0; w < W; ++w) acc[L][w] = x[w];
                } else {
#pragma unroll
                    for (int w = 0; w < W; ++w) acc[L][w] = combine<OP>(acc[L][w], x[w]);
                }
            }
        }
        while (n_fold) {
#pragma unroll
            for (int L = 1; L < D; ++L) {
                if (level == (uint32_t)L) {
#pragma unroll
                    for (int w = 0; w < W; ++w) acc[L - 1][w] = combine<OP>(acc[L - 1][w], acc[L][w]);
                }
            }
            --level;
            --n_fold;
        }
    }

    // The two halves of step(), for kernels that do something between a step's folds.
    __device__ __forceinline__ void combine_at(uint32_t level, bool set, const A (&x)[W])
    {
#pragma unroll
        for (int L = 0; L < D; ++L) {
            if (level == (uint32_t)L) {
                if (set) {
#pragma unroll
                    for (int w = 0; w < W; ++w) acc[L][w] = x[w];
                } else {
#pragma unroll
                    for (int w = 0; w < W; ++w) acc[L][w] = combine<OP>(acc[L][w], x[w]);
                }
            }
        }
    }
    // acc[level - 1] (op)= acc[level], count times, level by level downwards; returns the level reached
    __device__ __forceinline__ uint32_t fold_down(uint32_t level, uint32_t count)
    {
        while (count) {
#pragma unroll
            for (int L = 1; L < D; ++L) {
                if (level == (uint32_t)L) {
#pragma unroll
                    for (int w = 0; w < W; ++w) acc[L - 1][w] = combine<OP>(acc[L - 1][w], acc[L][w]);
                }
            }
            --level;
            --count;
        }
        return level;
    }

    // G values, one after the other, into the accumulator of one level
    template <int G, class Get> __device__ __forceinline__ void run(uint32_t level, Get get)
    {
#pragma unroll
        for (int L = 0; L < D; ++L) {
            if (level == (uint32_t)L) {
#pragma unroll
                for (int u = 0; u < G; ++u) {
                    A x[W];
                    get(u, x);
#pragma unroll
                    for (int w = 0; w < W; ++w) acc[L][w] = combine<OP>(acc[L][w], x[w]);
                }
            }
        }
    }
};

// All object traffic is streamed exactly once, so loads and stores carry the
// non-temporal hint: lines are not kept in L2 / the memory-side cache, which
// measurably raises sustained HBM bandwidth for this access pattern.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint4 ld16(const void *base, size_t byte_off)
{
    const u32x4 r = __builtin_nontemporal_load((const u32x4 *)((const char *)base + byte_off));
    return make_uint4(r.x, r.y, r.z, r.w);
}
__device__ __forceinline__ void st16(void *base, size_t byte_off, const uint4 &v)
{
    const u32x4 r = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(r, (u32x4 *)((char *)base + byte_off));
}

// Accumulator-typed values of one 16-byte source vector in the spill area: the
// vector at object byte offset `off` holds W elements, whose W accumulators sit at
// byte offset off / element size * 4 of a level's array (W * 4 bytes: 16 for
// 32-bit elements, 32 for bf16).
template <int DT> __device__ __forceinline__ void load_acc(const char *level_base, size_t off, typename Traits<DT>::acc_t *x)
{
    constexpr int W = Traits<DT>::W;
    const size_t o = off / Traits<DT>::ES * 4;
#pragma unroll
    for (int q = 0; q < W / 4; ++q) {
        const uint4 r = ld16(level_base, o + 16 * q);
        x[4 * q + 0] = __builtin_bit_cast(typename Traits<DT>::acc_t, r.x);
        x[4 * q + 1] = __builtin_bit_cast(typename Traits<DT>::acc_t, r.y);
        x[4 * q + 2] = __builtin_bit_cast(typename Traits<DT>::acc_t, r.z);
        x[4 * q + 3] = __builtin_bit_cast(typename Traits<DT>::acc_t, r.w);
    }
}
template <int DT> __device__ __forceinline__ void store_acc(char *level_base, size_t off, const typename Traits<DT>::acc_t *x)
{
    constexpr int W = Traits<DT>::W;
    const size_t o = off / Traits<DT>::ES * 4;
#pragma unroll
    for (int q = 0; q < W / 4; ++q) {
        const uint4 r = make_uint4(__builtin_bit_cast(uint32_t, x[4 * q + 0]), __builtin_bit_cast(uint32_t, x[4 * q + 1]),
                                   __builtin_bit_cast(uint32_t, x[4 * q + 2]), __builtin_bit_cast(uint32_t, x[4 * q + 3]));
        st16(level_base, o + 16 * q, r);
    }
}

// Layout of a kept partial result: one accumulator-typed value (4 bytes) per element of the
// object. The accumulators of 64 consecutive source vectors (the vectors the lanes of a wave hold)
// form a block of Q * 1 KiB, Q = W / 4: first the accumulators 0..3 of all 64 vectors, then 4..7 of
// all 64 (bf16: Q = 2; for 32-bit elements the layout is simply that of the object). Every store
// and load instruction of a wave then covers 1 KiB of consecutive addresses and a partial is one
// sequential stream. With a vector's W accumulators side by side instead, each instruction would
// touch every other 16 bytes of 2 KiB (measured: 10 % more bytes written to memory than stored);
// with the two halves in two planes an object's length apart, twice as many write streams (10 %
// slower).
template <int DT> __device__ __forceinline__ size_t kept_offset(size_t off, int q)
{
    constexpr size_t Q = Traits<DT>::W / 4;
    const size_t v = off >> 4;                   // index of the 16-byte source vector
    return ((v >> 6) * Q + (size_t)q) * 1024 + (v & 63) * 16;
}
template <int DT> __device__ __forceinline__ void load_kept(const char *base, size_t off, typename Traits<DT>::acc_t *x)
{
    using A = typename Traits<DT>::acc_t;
#pragma unroll
    for (int q = 0; q < Traits<DT>::W / 4; ++q) {
        const uint4 r = ld16(base, kept_offset<DT>(off, q));
        x[4 * q + 0] = __builtin_bit_cast(A, r.x);
        x[4 * q + 1] = __builtin_bit_cast(A, r.y);
        x[4 * q + 2] = __builtin_bit_cast(A, r.z);
        x[4 * q + 3] = __builtin_bit_cast(A, r.w);
    }
}
template <int DT> __device__ __forceinline__ void store_kept(char *base, size_t off, const typename Traits<DT>::acc_t *x)
{
#pragma unroll
    for (int q = 0; q < Traits<DT>::W / 4; ++q) {
        const uint4 r = make_uint4(__builtin_bit_cast(uint32_t, x[4 * q + 0]), __builtin_bit_cast(uint32_t, x[4 * q + 1]),
                                   __builtin_bit_cast(uint32_t, x[4 * q + 2]), __builtin_bit_cast(uint32_t, x[4 * q + 3]));
        st16(base, kept_offset<DT>(off, q), r);
    }
}
// where the accumulator of the single element at object byte offset off lives
template <int DT> __device__ __forceinline__ size_t kept_elem_offset(size_t off)
{
    const size_t i = (off & 15) / Traits<DT>::ES;           // element within its vector
    return kept_offset<DT>(off & ~(size_t)15, (int)(i >> 2)) + (i & 3) * 4;
}

// The program is read through the constant address space: it is never written
// while a kernel runs, so its steps can be fetched with scalar loads and held
// in SGPRs (a plain global pointer would make the compiler assume that the
// result stores may change it, and fall back to per-lane loads).
typedef const DevEntry __attribute__((address_space(4))) *prog_ptr;
// The broadcast's destination table is read the same way.
typedef void *const __attribute__((address_space(4))) *table_ptr;

// A sub-program record held by the lanes of a wave: lane 0 has the SubHeader, lane 1 + t step t
// (the 16 bytes of a DevEntry as x = address low, y = address high, z = ctl). Reading a step is
// three lane reads with a wave-uniform lane number, so the values land in SGPRs like those of a
// scalar load.
struct LaneStep {
    const void *src;
    uint32_t ctl;
};
struct LaneProg {
    uint4 mine;
    __device__ __forceinline__ static uint32_t from(uint32_t v, int lane) { return (uint32_t)__builtin_amdgcn_readlane((int)v, lane); }
    __device__ __forceinline__ LaneStep operator[](int t) const
    {
        const uint64_t p = ((uint64_t)from(mine.y, t + 1) << 32) | from(mine.x, t + 1);
        return {(const void *)(uintptr_t)p, from(mine.z, t + 1)};
    }
    __device__ __forceinline__ int n_entries() const { return (int)from(mine.z, 0); }
    __device__ __forceinline__ bool partial_out() const { return (from(mine.w, 0) & kSubStoresAccumulators) != 0; }
    __device__ __forceinline__ void *dst() const { return (void *)(uintptr_t)(((uint64_t)from(mine.y, 0) << 32) | from(mine.x, 0)); }
};

// The addresses and control words of G consecutive program steps, held in SGPRs.
template <int G> struct StepGroup {
    const void *src[G];
    uint32_t ctl[G];
};
// Steps [t, t + G) of the program, indices clamped to the last step so that a look-ahead past the
// end reads valid memory (its values are never used).
template <int G, class Prog> __device__ __forceinline__ StepGroup<G> fetch_steps(const Prog prog, int t, int n)
{
    StepGroup<G> g;
#pragma unroll
    for (int u = 0; u < G; ++u) {
        const int i = (t + u < n) ? t + u : n - 1;
        g.src[u] = prog[i].src;
        g.ctl[u] = prog[i].ctl;
    }
    return g;
}

// Keeps the scalar loads of a look-ahead where they are written (right behind the vector loads
// they are meant to overlap with): an empty statement that formally reads the fetched words.
// Without it the compiler sinks them to the end of the iteration, behind all the folds.
template <int G> __device__ __forceinline__ void pin_here(const StepGroup<G> &g)
{
#pragma unroll
    for (int u = 0; u < G; ++u) asm volatile("" : : "s"(g.src[u]), "s"(g.ctl[u]));
}

// Whether a program's result is stored as accumulator-typed values laid out like a kept partial result
// (see kept_offset) instead of as elements: a sub-program's header can say so.
template <class Prog> __device__ __forceinline__ bool stores_accumulators(const Prog &) { return false; }
__device__ __forceinline__ bool stores_accumulators(const LaneProg &p) { return p.partial_out(); }

// What the loads of G steps bring in: one 16-byte vector per step and vector of the lane. MIXED (kernels
// whose steps may read partial results of an element type with W = 8 accumulators per vector): a
// step with kPartialBit reads W accumulator-typed values, the second half of which lands in more[].
template <int G, int VPT, bool MIXED> struct Loaded {
    uint4 raw[G][VPT];
    uint4 more[MIXED ? G : 1][VPT];
};

// G consecutive program steps: all G*VPT loads are issued before the first value
// is consumed, then the values are folded in program order.
template <int DT, int G, int VPT, bool MIXED>
__device__ __forceinline__ void issue_group(const StepGroup<G> &g, const size_t (&off)[VPT], Loaded<G, VPT, MIXED> &in)
{
#pragma unroll
    for (int u = 0; u < G; ++u) {
        if constexpr (MIXED) {
            // one load that every step issues, at an offset picked by the step's kind, and a second one for
            // partial results only: two loads into the same registers on either side of a branch would make
            // the second wait for everything in flight
            const bool partial = (g.ctl[u] & kPartialBit) != 0;
#pragma unroll
            for (int j = 0; j < VPT; ++j) {
                size_t at = partial ? kept_offset<DT>(off[j], 0) : off[j];
                asm volatile("" : "+v"(at));          // the offset is picked here, so that the load is not split in two again
                in.raw[u][j] = ld16(g.src[u], at);
            }
            if (partial) {
#pragma unroll
                for (int j = 0; j < VPT; ++j) in.more[u][j] = ld16(g.src[u], kept_offset<DT>(off[j], 1));
            }
        } else {
#pragma unroll
            for (int j = 0; j < VPT; ++j) in.raw[u][j] = ld16(g.src[u], off[j]);
        }
    }
}
template <int DT, int G, int VPT, bool MIXED, class M>
__device__ __forceinline__ void fold_group(M &m, const StepGroup<G> &g, const Loaded<G, VPT, MIXED> &in)
{
    using A = typename Traits<DT>::acc_t;
    constexpr int W = Traits<DT>::W;
    if (G == kRunSteps && (g.ctl[0] & kRunBit)) {
        // a run of plain combines of objects into one level: one dispatch for the whole group
        m.template run<G>(g.ctl[0] & 0xffu, [&](int u, A *x) {
#pragma unroll
            for (int j = 0; j < VPT; ++j) decode<DT>(in.raw[u][j], &x[j * W]);
        });
        return;
    }
#pragma unroll
    for (int u = 0; u < G; ++u) {
        if constexpr (MIXED) {
            static_assert(!MIXED || W == 8, "two vectors of four accumulators per source vector");
            if (g.ctl[u] & kPartialBit) {
                A y[VPT * W];
#pragma unroll
                for (int j = 0; j < VPT; ++j) {
                    const uint4 lo = in.raw[u][j], hi = in.more[u][j];
                    y[j * W + 0] = __builtin_bit_cast(A, lo.x);
                    y[j * W + 1] = __builtin_bit_cast(A, lo.y);
                    y[j * W + 2] = __builtin_bit_cast(A, lo.z);
                    y[j * W + 3] = __builtin_bit_cast(A, lo.w);
                    y[j * W + 4] = __builtin_bit_cast(A, hi.x);
                    y[j * W + 5] = __builtin_bit_cast(A, hi.y);
                    y[j * W + 6] = __builtin_bit_cast(A, hi.z);
                    y[j * W + 7] = __builtin_bit_cast(A, hi.w);
                }
                m.step(g.ctl[u], y);
                continue;
            }
        }
        A x[VPT * W];
#pragma unroll
        for (int j = 0; j < VPT; ++j) decode<DT>(in.raw[u][j], &x[j * W]);
        m.step(g.ctl[u], x);
    }
}
template <int DT, int G, int VPT, bool MIXED, class M, class Prog>
__device__ __forceinline__ void run_group(M &m, const Prog prog, int t, int n, const size_t (&off)[VPT])
{
    const StepGroup<G> g = fetch_steps<G>(prog, t, n);
    Loaded<G, VPT, MIXED> in;
    issue_group<DT, G, VPT, MIXED>(g, off, in);
    fold_group<DT, G, VPT, MIXED>(m, g, in);
}

// One workgroup of THREADS lanes walks tiles of THREADS*VPT 16-byte vectors:
// VPT pieces of THREADS consecutive vectors (every load instruction of a wave
// covers 1 KiB of consecutive addresses), the pieces side by side or a fixed
// distance apart (piece_stride_log2, below). For each tile the program is run
// in groups of U steps: the U*VPT loads of a group are all issued before the
// first of them is consumed, then the group's values are folded in program
// order. D = accumulator levels held in registers.
//
// SEG: the launch runs only a segment of a program. Accumulator levels
// [0, n_restore) are first read back from the spill area (where the previous
// segment on these chunks left them); afterwards either levels [0, n_save) are
// written to the spill area (more steps will follow) or, when n_save is 0, the
// result is stored like in a whole-program launch. The spill area holds one
// object-sized array of accumulator-typed values per level.
//
// The pieces of a long bf16 program that was cut into sub-programs: their partial results must be
// accumulator-typed, or the bits of the result would depend on the cut. A sub-program whose header says so
// stores its result as 4 bytes per element, laid out as kept_offset says (any bf16 kernel that runs
// sub-programs can do that), and MIXED kernels take steps with kPartialBit, which read such a result.
template <int DT, int OP, int D, int VPT, int U, int THREADS, bool SEG = false, bool MIXED = false, class Prog>
__device__ __forceinline__ void reduce_body(const ReduceArgs &a, const Prog prog, const int n, void *const dst)
{
    static_assert(!(SEG && MIXED), "segments keep their accumulators in the spill area, not in partial results");
    using T = Traits<DT>;
    using A = typename T::acc_t;
    constexpr int W = T::W;
    constexpr size_t kTile = (size_t)THREADS * VPT;
    // Which vectors a workgroup owns. Contiguous: VPT * THREADS consecutive vectors. Strided
    // (piece_stride_log2 = s >= 0): the range is cut into pieces of THREADS vectors and into groups
    // of VPT << s pieces; workgroup r of a group owns pieces r, r + 2^s, r + 2 * 2^s, ... of it. A
    // wave's loads in flight then lie 2^s pieces apart instead of side by side, and consecutive
    // workgroups still cover consecutive pieces.
    const int sl = a.piece_stride_log2;
    // The grid of vectors starts lead vectors before the range (the host picks lead so that it starts
    // where the sources are 128-byte aligned: a wave's 1 KiB load then covers 8 whole lines instead of
    // parts of 9, which is worth 10 points of bandwidth for sources that are only 16-byte aligned).
    const size_t lead = (size_t)a.lead_vecs, n_all = a.n_vec + lead;
    const size_t n_tiles = sl < 0 ? (n_all + kTile - 1) / kTile : ((n_all + (kTile << sl) - 1) / (kTile << sl)) << sl;

    for (size_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        // lanes in front of the range or past its end re-read its first or last vector (always
        // inside the range) and skip the store, so control flow stays uniform across the wave
        size_t off[VPT];
        bool live[VPT];
        size_t first = tile * kTile, step = THREADS;     // vector index of piece 0, distance between pieces
        if (sl >= 0) {
            const size_t r = tile & (((size_t)1 << sl) - 1);
            first = (((tile >> sl) * VPT) << sl) * THREADS + r * THREADS;
            step = (size_t)THREADS << sl;
            if (first >= n_all) continue;                 // a workgroup of the last group with nothing to do
        }
#pragma unroll
        for (int j = 0; j < VPT; ++j) {
            const size_t v = first + (size_t)j * step + threadIdx.x;
            live[j] = v >= lead && v < n_all;
            off[j] = a.byte_begin + ((live[j] ? v : v < lead ? lead : n_all - 1) - lead) * 16;
        }
        Machine<DT, OP, D, VPT * W> m;
        if (SEG) {
#pragma unroll
            for (int L = 0; L < D; ++L) {
                if (L < a.n_restore) {
#pragma unroll
                    for (int j = 0; j < VPT; ++j) load_acc<DT>(a.spill + (size_t)L * a.level_stride, off[j], &m.acc[L][j * W]);
                }
            }
        }
        int t = 0;
        if (n >= U) {
            // the next group's addresses are fetched (scalar loads) while this group's data is in
            // flight, so that their latency does not add to the data's
            StepGroup<U> cur = fetch_steps<U>(prog, 0, n);
            for (; t + U <= n; t += U) {
                Loaded<U, VPT, MIXED> in;
                issue_group<DT, U, VPT, MIXED>(cur, off, in);
                const StepGroup<U> nxt = fetch_steps<U>(prog, t + U, n);
                pin_here(nxt);
                fold_group<DT, U, VPT, MIXED>(m, cur, in);
                cur = nxt;
            }
        }
        // what is left is taken in halving groups so that it stays in flight together too
        if (U > 8 && t + 8 <= n) { run_group<DT, 8, VPT, MIXED>(m, prog, t, n, off); t += 8; }
        if (U > 4 && t + 4 <= n) { run_group<DT, 4, VPT, MIXED>(m, prog, t, n, off); t += 4; }
        if (U > 2 && t + 2 <= n) { run_group<DT, 2, VPT, MIXED>(m, prog, t, n, off); t += 2; }
        if (U > 1 && t < n) { run_group<DT, 1, VPT, MIXED>(m, prog, t, n, off); t += 1; }
        if (SEG && a.n_save > 0) {
#pragma unroll
            for (int L = 0; L < D; ++L) {
                if (L < a.n_save) {
#pragma unroll
                    for (int j = 0; j < VPT; ++j)
                        if (live[j]) store_acc<DT>(a.spill + (size_t)L * a.level_stride, off[j], &m.acc[L][j * W]);
                }
            }
        } else if (DT == HOP_BF16 && stores_accumulators(prog)) {
#pragma unroll
            for (int j = 0; j < VPT; ++j)
                if (live[j]) store_kept<DT>((char *)dst, off[j], &m.acc[0][j * W]);
        } else {
#pragma unroll
            for (int j = 0; j < VPT; ++j) {
                const uint4 out = encode<DT>(&m.acc[0][j * W]);
                if (live[j]) st16(dst, off[j], out);
            }
        }
    }

    // ragged tail: fewer than 16 bytes at the very end of the object
    if (blockIdx.x == 0 && (int)threadIdx.x < a.n_tail) {
        const size_t off = a.byte_begin + a.n_vec * 16 + (size_t)threadIdx.x * T::ES;
        Machine<DT, OP, D, 1> m;
        const size_t acc_off = off / T::ES * sizeof(A);
        if (SEG) {
#pragma unroll
            for (int L = 0; L < D; ++L)
                if (L < a.n_restore) m.acc[L][0] = *(const A *)(a.spill + (size_t)L * a.level_stride + acc_off);
        }
        for (int t = 0; t < n; ++t) {
            const void *const src = prog[t].src;
            const uint32_t ctl = prog[t].ctl;
            A x[1];
            if (MIXED && (ctl & kPartialBit)) x[0] = *(const A *)((const char *)src + kept_elem_offset<DT>(off));
            else x[0] = load_elem<DT>(src, off);
            m.step(ctl, x);
        }
        if (SEG && a.n_save > 0) {
#pragma unroll
            for (int L = 0; L < D; ++L)
                if (L < a.n_save) *(A *)(a.spill + (size_t)L * a.level_stride + acc_off) = m.acc[L][0];
        } else if (DT == HOP_BF16 && stores_accumulators(prog)) {
            *(A *)((char *)dst + kept_elem_offset<DT>(off)) = m.acc[0][0];
        } else {
            store_elem<DT>(dst, off, m.acc[0][0]);
        }
    }
}

// ----------------------------------------------------------------------------
// a long program over a narrow column of the objects, as chains (ChainArgs)
// ----------------------------------------------------------------------------

// The value x with x (op) identity == x for every x, bit for bit: -0.0 for a floating-point sum
// (x + -0.0 is x also for x = +0.0), the infinities for min and max (combine keeps its left operand
// unless the right one is strictly better, so a NaN on the left stays too), 0 and the extreme
// integers for int32.
template <int DT, int OP> __device__ __forceinline__ typename Traits<DT>::acc_t chain_identity()
{
    using A = typename Traits<DT>::acc_t;
    if (DT == HOP_I32) return OP == HOP_SUM ? A(0) : OP == HOP_MIN ? A(INT32_MAX) : A(INT32_MIN);
    return __builtin_bit_cast(A, OP == HOP_SUM ? 0x80000000u : OP == HOP_MIN ? 0x7f800000u : 0xff800000u);
}

// One team of kChainLanes lanes per chain, one 16-byte vector (TAIL: one element) per lane. A lane
// loads its chain's whole record (one trip to the table), then everything the items name - vectors
// of the objects from memory, values of other chains from LDS - all in flight together, then folds
// in item order. The chains of the teams of one wave differ, so all of this is per-lane data, and
// what counts is how few instructions an item takes (one wave per SIMD: nothing hides them): a
// record is padded to its full length with the identity value, so neither the loads nor the folds
// look at the item count. For 32-bit elements an object's vector and a chain's value are both 16
// bytes per lane (TAIL: 4) and are fetched by the same flat load, whose address is the item plus
// either the lane's byte offset into the object or the lane's place in the LDS window.
// A value in LDS: W accumulators per lane, the value at byte offset b of the LDS array at
// [b + lane * W * 4].
//
// LANES, TEAMS: the narrow form is teams of kChainLanes lanes (64-byte columns, kChainTeams chains side by
// side: ranges up to 64 KiB); the wide form is teams of kChainWideLanes = a whole wave each (1 KiB columns,
// kChainWideTeams chains side by side: every load instruction covers 1 KiB of one object, for ranges of
// hundreds of KiB, where the narrow form would need thousands of workgroups).
template <int DT, int OP, bool TAIL, int LANES, int TEAMS, class Table>
__device__ __forceinline__ void chains_body(const ChainArgs &a, const Table table, typename Traits<DT>::acc_t *lds,
                                            const size_t off, const bool live)
{
    using T = Traits<DT>;
    using A = typename T::acc_t;
    constexpr int W = TAIL ? 1 : T::W;
    constexpr int R = kChainMaxItems;
    constexpr bool kAlike = T::ES == 4;
    static_assert(kChainRecordWords % 8 == 0 && R + 1 == kChainRecordWords, "records are read as 16-byte pairs of words, held eight at a time");
    const int lane = (int)threadIdx.x % LANES, team = (int)threadIdx.x / LANES;
    char *const mine = (char *)lds + (size_t)lane * T::W * 4;           // this lane's part of the value at offset 0
    const uint64_t mine_flat = (uint64_t)(uintptr_t)(const void *)mine;
    // the identity value sits behind the chains' values; every team writes the same bytes
    {
        A *v = (A *)(mine + a.identity_at);
#pragma unroll
        for (int w = 0; w < T::W; ++w) v[w] = chain_identity<DT, OP>();
    }
    __syncthreads();
    for (int p = 0; p < a.base.n_entries; ++p) {
        for (uint32_t c = a.pass_begin[p] + (uint32_t)team; c < a.pass_begin[p + 1]; c += TEAMS) {
            uint64_t word[kChainRecordWords];
            if constexpr (LANES == 64) {
                // a wave per chain: the record is the same for all its lanes and is fetched by scalar loads (the
                // table is in the kernel arguments or comes as a pointer into the constant address space: see
                // the kernels), so its 24 words sit in scalar registers
                const size_t at = (size_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)c) * (kChainRecordWords / 2);
#pragma unroll
                for (int j = 0; j < kChainRecordWords / 2; ++j) {
                    const u32x4 q = table[at + j];
                    word[2 * j] = ((uint64_t)q.y << 32) | q.x;
                    word[2 * j + 1] = ((uint64_t)q.w << 32) | q.z;
                }
#pragma unroll
                for (int j = 0; j < kChainRecordWords; j += 8)
                    asm volatile("" : "+s"(word[j]), "+s"(word[j + 1]), "+s"(word[j + 2]), "+s"(word[j + 3]), "+s"(word[j + 4]),
                                 "+s"(word[j + 5]), "+s"(word[j + 6]), "+s"(word[j + 7]) : : "memory");
            } else {
                const auto rec = table + (size_t)c * (kChainRecordWords / 2);
#pragma unroll
                for (int j = 0; j < kChainRecordWords / 2; ++j) {
                    const auto q = rec[j];
                    word[2 * j] = ((uint64_t)q.y << 32) | q.x;
                    word[2 * j + 1] = ((uint64_t)q.w << 32) | q.z;
                }
                // The whole record has arrived before the first item is fetched: an empty statement that formally
                // rewrites every word. (Flat loads complete out of order with other loads, so with the record
                // still on its way the compiler would wait for everything in flight before each use of a word.)
#pragma unroll
                for (int j = 0; j < kChainRecordWords; j += 8)
                    asm volatile("" : "+v"(word[j]), "+v"(word[j + 1]), "+v"(word[j + 2]), "+v"(word[j + 3]), "+v"(word[j + 4]),
                                 "+v"(word[j + 5]), "+v"(word[j + 6]), "+v"(word[j + 7]) : : "memory");
            }
            const uint32_t out = (uint32_t)word[0];
            A acc[W];
            if (kAlike) {
                u32x4 raw[R + 1];
#pragma unroll
                for (int u = 0; u < R; ++u) {
                    const uint64_t e = word[1 + u];
                    const uint64_t at = e + ((uint32_t)(e >> 32) == 0 ? mine_flat : (uint64_t)off);
                    if (TAIL) raw[u].x = *(const uint32_t *)(uintptr_t)at;
                    else raw[u] = *(const u32x4 *)(uintptr_t)at;
                }
                raw[R] = raw[R - 1];
                // Every load is issued before the first fold, and the folds start when all have arrived: an
                // empty statement that formally rewrites every loaded value. (The compiler would otherwise
                // interleave loads and folds to save registers, and the chain would wait for memory once
                // per few items instead of once.)
#pragma unroll
                for (int u = 0; u < R + 1; u += 8)
                    asm volatile("" : "+v"(raw[u]), "+v"(raw[u + 1]), "+v"(raw[u + 2]), "+v"(raw[u + 3]), "+v"(raw[u + 4]),
                                 "+v"(raw[u + 5]), "+v"(raw[u + 6]), "+v"(raw[u + 7]) : : "memory");
#pragma unroll
                for (int u = 0; u < R; ++u) {
                    const uint32_t r[4] = {raw[u].x, raw[u].y, raw[u].z, raw[u].w};
#pragma unroll
                    for (int w = 0; w < W; ++w) {
                        const A x = __builtin_bit_cast(A, r[w]);
                        acc[w] = u == 0 ? x : combine<OP>(acc[w], x);
                    }
                }
            } else {
                // bf16: an object's vector is 16 bytes of 8 elements, a value 32 bytes of 8 accumulators. The
                // objects' vectors are all fetched first (an item that is a value fetches the lane's part of the
                // identity value instead, by the same flat load, and does not use it); the values are read from LDS
                // as the fold comes to them (an item that is an object reads the identity value instead), so
                // that the registers hold 16 bytes per item, not 48, and several workgroups fit a compute unit.
                u32x4 raw[R];
                uint32_t value_at[R], values = 0;       // where each item's value is in LDS; bit u: item u is a value
#pragma unroll
                for (int u = 0; u < R; ++u) {
                    const uint64_t e = word[1 + u];
                    const bool is_value = (uint32_t)(e >> 32) == 0;
                    value_at[u] = is_value ? (uint32_t)e : a.identity_at;
                    values |= (uint32_t)is_value << u;
                    const uint64_t at = is_value ? mine_flat + a.identity_at : e + (uint64_t)off;
                    if constexpr (TAIL) raw[u].x = *(const uint16_t *)(uintptr_t)at;
                    else raw[u] = *(const u32x4 *)(uintptr_t)at;
                }
                asm volatile("" ::: "memory");
                // The value of item u + 1 is on its way from LDS while item u is folded. The empty statements
                // formally use what was read, so the reads happen whether or not the item is a value (no
                // branch around them), and being barriers for memory accesses they keep the next read ahead.
                typedef const u32x4 __attribute__((address_space(3))) *lds_vec_ptr;
                typedef const uint32_t __attribute__((address_space(3))) *lds_word_ptr;
                constexpr int Q = TAIL ? 1 : T::W / 4;
                u32x4 next[Q], cur[Q];
                const auto fetch_value = [&](int u) {
                    if constexpr (TAIL) next[0].x = *(lds_word_ptr)(mine + value_at[u]);
                    else {
#pragma unroll
                        for (int q = 0; q < Q; ++q) next[q] = ((lds_vec_ptr)(mine + value_at[u]))[q];
                    }
                };
                fetch_value(0);
#pragma unroll
                for (int u = 0; u < R; ++u) {
                    const bool is_value = (values >> u) & 1u;
#pragma unroll
                    for (int q = 0; q < Q; ++q) cur[q] = next[q];
                    if (u + 1 < R) fetch_value(u + 1);
#pragma unroll
                    for (int q = 0; q < Q; ++q) {
                        if constexpr (TAIL) asm volatile("" : "+v"(cur[q].x) : : "memory");
                        else asm volatile("" : "+v"(cur[q]) : : "memory");
                    }
                    A x[W];
                    if constexpr (TAIL) x[0] = bits_to_f32(raw[u].x << 16);
                    else decode<DT>(make_uint4(raw[u].x, raw[u].y, raw[u].z, raw[u].w), x);
#pragma unroll
                    for (int w = 0; w < W; ++w) {
                        const A y = is_value ? __builtin_bit_cast(A, (uint32_t)cur[w / 4][w % 4]) : x[w];
                        acc[w] = u == 0 ? y : combine<OP>(acc[w], y);
                    }
                }
            }
            if (out != kChainFinal) {
                A *v = (A *)(mine + out);
#pragma unroll
                for (int w = 0; w < W; ++w) v[w] = acc[w];
            } else if (live) {
                if (TAIL) store_elem<DT>(a.base.dst, off, acc[0]);
                else st16(a.base.dst, off, encode<DT>(acc));
            }
        }
        __syncthreads();       // the next pass reads what this one wrote; every lane comes by here once per pass
    }
}

// The column (or, behind the last column, the elements after the last full vector) that this workgroup owns.
template <int DT, int OP, int LANES, int TEAMS, class Table>
__device__ __forceinline__ void chains_workgroup(const ChainArgs &a, const Table table)
{
    using T = Traits<DT>;
    extern __shared__ __align__(16) unsigned char chain_values[];
    typename T::acc_t *const lds = (typename T::acc_t *)chain_values;
    const size_t n_cols = (a.base.n_vec + LANES - 1) / LANES;
    const size_t lane = threadIdx.x % LANES;
    if (blockIdx.x < n_cols) {
        size_t col = blockIdx.x;
        if constexpr (LANES * 16 < 128) {
            // Two narrow columns share a 128-byte line. Workgroups go to the chip's 8 dies in turn, each die with
            // an L2 of its own: within every whole block of 8 * kChainColumnRun workgroups, the workgroups that
            // land on one die take kChainColumnRun columns in a row, so a line is fetched from memory by one L2, once.
            constexpr size_t kBlock = 8 * kChainColumnRun;
            const size_t block0 = col / kBlock * kBlock;
            if (block0 + kBlock <= n_cols) col = block0 + (col - block0) % 8 * kChainColumnRun + (col - block0) / 8;
        }
        const size_t v = col * LANES + lane;
        const bool live = v < a.base.n_vec;
        chains_body<DT, OP, false, LANES, TEAMS>(a, table, lds, a.base.byte_begin + (live ? v : a.base.n_vec - 1) * 16, live);
    } else {
        // the workgroups after the last column: the elements behind the last full vector, one per lane
        const size_t i = (blockIdx.x - n_cols) * LANES + lane;
        const bool live = i < (size_t)a.base.n_tail;
        chains_body<DT, OP, true, LANES, TEAMS>(a, table, lds, a.base.byte_begin + a.base.n_vec * 16 + (live ? i : 0) * T::ES, live);
    }
}

// The table in device memory (a.base.prog) ...
template <int DT, int OP>
__global__ __launch_bounds__(kChainThreads) void reduce_kernel_chains(const ChainArgs a)
{
    chains_workgroup<DT, OP, kChainLanes, kChainTeams>(a, (const uint4 *)a.base.prog);
}
// ... or inside the kernel arguments: nothing is staged ahead of the launch.
template <int DT, int OP, int WORDS>
__global__ __launch_bounds__(kChainThreads) void reduce_kernel_chains_inline(const ChainArgsInline<WORDS> a)
{
    chains_workgroup<DT, OP, kChainLanes, kChainTeams>(a.base, (const uint4 *)&a.table[0]);
}
// The wide form of both. Its records are read with a wave-uniform index: from the kernel arguments that is a
// scalar load as it stands; a table in device memory is read through the constant address space for the
// same effect (like the programs of the streaming kernels: nothing writes it while the kernel runs).
template <int DT, int OP>
__global__ __launch_bounds__(kChainWideThreads) void reduce_kernel_chains_wide(const ChainArgs a)
{
    typedef const u32x4 __attribute__((address_space(4))) *uniform_table_ptr;
    chains_workgroup<DT, OP, kChainWideLanes, kChainWideTeams>(a, (uniform_table_ptr)(uintptr_t)a.base.prog);
}
template <int DT, int OP, int WORDS>
__global__ __launch_bounds__(kChainWideThreads) void reduce_kernel_chains_wide_inline(const ChainArgsInline<WORDS> a)
{
    chains_workgroup<DT, OP, kChainWideLanes, kChainWideTeams>(a.base, (const u32x4 *)&a.table[0]);
}

// The reduce that keeps and reuses partial results (failure repair, section 3.5.2: the partial
// results that do not contain the failed object survive). Same tiling as reduce_body, one step
// at a time. A step whose control word carries kPartialBit reads a kept partial instead of an
// object; a step with a save mark stores, once its folds have come down to the marked level,
// that level's accumulator as a kept partial (array q of the kept area, a.spill + q *
// a.level_stride, laid out as kept_offset says) and then finishes its folds. The next step's
// address and control words are fetched while this step's data is in flight.
template <int DT, int OP, int D, int VPT, int THREADS, class Prog>
__device__ __forceinline__ void reduce_body_kept(const ReduceArgs &a, const Prog prog, const int n, void *const dst)
{
    using T = Traits<DT>;
    using A = typename T::acc_t;
    constexpr int W = T::W;
    constexpr size_t kTile = (size_t)THREADS * VPT;
    const int sl = a.piece_stride_log2;
    const size_t lead = (size_t)a.lead_vecs, n_all = a.n_vec + lead;
    const size_t n_tiles = sl < 0 ? (n_all + kTile - 1) / kTile : ((n_all + (kTile << sl) - 1) / (kTile << sl)) << sl;

    for (size_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        size_t off[VPT];
        bool live[VPT];
        size_t first = tile * kTile, step = THREADS;
        if (sl >= 0) {
            const size_t r = tile & (((size_t)1 << sl) - 1);
            first = (((tile >> sl) * VPT) << sl) * THREADS + r * THREADS;
            step = (size_t)THREADS << sl;
            if (first >= n_all) continue;
        }
#pragma unroll
        for (int j = 0; j < VPT; ++j) {
            const size_t v = first + (size_t)j * step + threadIdx.x;
            live[j] = v >= lead && v < n_all;
            off[j] = a.byte_begin + ((live[j] ? v : v < lead ? lead : n_all - 1) - lead) * 16;
        }
        Machine<DT, OP, D, VPT * W> m;
        const void *src = prog[0].src;
        uint32_t ctl = prog[0].ctl, aux = prog[0].aux;
        for (int t = 0; t < n; ++t) {
            A x[VPT * W];
            uint4 raw[VPT];
            const bool partial = (ctl & kPartialBit) != 0;
            if (partial) {
#pragma unroll
                for (int j = 0; j < VPT; ++j) load_kept<DT>((const char *)src, off[j], &x[j * W]);
            } else {
#pragma unroll
                for (int j = 0; j < VPT; ++j) raw[j] = ld16(src, off[j]);
            }
            // look ahead (clamped to the last step, whose words are then simply read twice)
            const int nx = t + 1 < n ? t + 1 : n - 1;
            const void *src_n = prog[nx].src;
            const uint32_t ctl_n = prog[nx].ctl, aux_n = prog[nx].aux;
            asm volatile("" : : "s"(src_n), "s"(ctl_n), "s"(aux_n));
            if (!partial) {
#pragma unroll
                for (int j = 0; j < VPT; ++j) decode<DT>(raw[j], &x[j * W]);
            }
            uint32_t level = ctl & 0xffu, n_fold = ctl >> 16;
            m.combine_at(level, (ctl >> 8) & 1u, x);
            if (aux) {
                const uint32_t keep_level = aux >> 16;
                const uint32_t inner = level - keep_level;          // folds that stay inside the kept subtree
                level = m.fold_down(level, inner);
                n_fold -= inner;
                char *base = a.spill + (size_t)((aux & 0xffffu) - 1) * a.level_stride;
#pragma unroll
                for (int L = 0; L < D; ++L) {
                    if (keep_level == (uint32_t)L) {
#pragma unroll
                        for (int j = 0; j < VPT; ++j)
                            if (live[j]) store_kept<DT>(base, off[j], &m.acc[L][j * W]);
                    }
                }
            }
            m.fold_down(level, n_fold);
            src = src_n;
            ctl = ctl_n;
            aux = aux_n;
        }
#pragma unroll
        for (int j = 0; j < VPT; ++j) {
            const uint4 out = encode<DT>(&m.acc[0][j * W]);
            if (live[j]) st16(dst, off[j], out);
        }
    }

    // ragged tail: fewer than 16 bytes at the very end of the object
    if (blockIdx.x == 0 && (int)threadIdx.x < a.n_tail) {
        const size_t off = a.byte_begin + a.n_vec * 16 + (size_t)threadIdx.x * T::ES;
        const size_t acc_off = kept_elem_offset<DT>(off);
        Machine<DT, OP, D, 1> m;
        for (int t = 0; t < n; ++t) {
            const uint32_t ctl = prog[t].ctl, aux = prog[t].aux;
            A x[1];
            if (ctl & kPartialBit) x[0] = *(const A *)((const char *)prog[t].src + acc_off);
            else x[0] = load_elem<DT>(prog[t].src, off);
            uint32_t level = ctl & 0xffu, n_fold = ctl >> 16;
            m.combine_at(level, (ctl >> 8) & 1u, x);
            if (aux) {
                const uint32_t keep_level = aux >> 16;
                const uint32_t inner = level - keep_level;
                level = m.fold_down(level, inner);
                n_fold -= inner;
                char *base = a.spill + (size_t)((aux & 0xffffu) - 1) * a.level_stride;
#pragma unroll
                for (int L = 0; L < D; ++L)
                    if (keep_level == (uint32_t)L) *(A *)(base + acc_off) = m.acc[L][0];
            }
            m.fold_down(level, n_fold);
        }
        store_elem<DT>(dst, off, m.acc[0][0]);
    }
}

// Program in device memory, steps that keep or read partial results (reduce_body_kept).
template <int DT, int OP, int D, int VPT, int THREADS>
__global__ __launch_bounds__(THREADS) void reduce_kernel_kept(ReduceArgs a)
{
    reduce_body_kept<DT, OP, D, VPT, THREADS>(a, (prog_ptr)(uintptr_t)a.prog, a.n_entries, a.dst);
}
// The same with the program inside the kernel arguments.
template <int DT, int OP, int D, int VPT, int THREADS>
__global__ __launch_bounds__(THREADS) void reduce_kernel_kept_inline(ReduceArgsInline a)
{
    reduce_body_kept<DT, OP, D, VPT, THREADS>(a.base, &a.steps[0], a.base.n_entries, a.base.dst);
}

// Program in device memory (or, with sub_entries set, the records of several sub-programs).
template <int DT, int OP, int D, int VPT, int U, int THREADS, bool MIXED>
__device__ __forceinline__ void reduce_kernel_body(const ReduceArgs &a)
{
    if (a.sub_entries > 0) {
        // several independent sub-programs in one launch: blockIdx.y picks a record, lane i fetches
        // its entry i (lanes past the record's end re-read its last entry), and the steps are then
        // taken from the lanes
        const int lane = (int)threadIdx.x < a.sub_entries ? (int)threadIdx.x : a.sub_entries - 1;
        const uint4 *rec = (const uint4 *)a.prog + (size_t)blockIdx.y * (size_t)a.sub_entries;
        const LaneProg lp{rec[lane]};
        reduce_body<DT, OP, D, VPT, U, THREADS, false, MIXED>(a, lp, lp.n_entries(), lp.dst());
    } else {
        reduce_body<DT, OP, D, VPT, U, THREADS, false, MIXED>(a, (prog_ptr)(uintptr_t)a.prog, a.n_entries, a.dst);
    }
}

template <int DT, int OP, int D, int VPT, int U, int THREADS>
__global__ __launch_bounds__(THREADS) void reduce_kernel(ReduceArgs a)
{
    reduce_kernel_body<DT, OP, D, VPT, U, THREADS, false>(a);
}
// The same for programs some of whose steps read partial results (kPartialBit): see MIXED at reduce_body.
template <int DT, int OP, int D, int VPT, int U, int THREADS>
__global__ __launch_bounds__(THREADS) void reduce_kernel_mixed(ReduceArgs a)
{
    reduce_kernel_body<DT, OP, D, VPT, U, THREADS, true>(a);
}

// A segment of a program in device memory, with accumulators restored from and/or saved to the spill area.
template <int DT, int OP, int D, int VPT, int U, int THREADS>
__global__ __launch_bounds__(THREADS) void reduce_kernel_seg(ReduceArgs a)
{
    reduce_body<DT, OP, D, VPT, U, THREADS, true>(a, (prog_ptr)(uintptr_t)a.prog, a.n_entries, a.dst);
}

// Program inside the kernel arguments.
template <int DT, int OP, int D, int VPT, int U, int THREADS>
__global__ __launch_bounds__(THREADS) void reduce_kernel_inline(ReduceArgsInline a)
{
    reduce_body<DT, OP, D, VPT, U, THREADS>(a.base, &a.steps[0], a.base.n_entries, a.base.dst);
}
template <int DT, int OP, int D, int VPT, int U, int THREADS>
__global__ __launch_bounds__(THREADS) void reduce_kernel_mixed_inline(ReduceArgsInline a)
{
    reduce_body<DT, OP, D, VPT, U, THREADS, false, true>(a.base, &a.steps[0], a.base.n_entries, a.base.dst);
}

// One source, n_dst destinations: each 16-byte vector is read once (non-temporal) and
// written n_dst times. VPT vectors per lane are in flight together.
template <int VPT, int THREADS, class Table>
__device__ __forceinline__ void copy_body(const CopyArgs &a, const Table dsts)
{
    constexpr size_t kTile = (size_t)THREADS * VPT;
    // the vectors of a workgroup: contiguous, or VPT pieces 2^s pieces apart (as in reduce_body)
    const int sl = a.piece_stride_log2;
    // the grid of vectors starts lead vectors before the range, at a 128-byte boundary of the
    // destination: stores of whole lines (a destination that is only 16-byte aligned otherwise
    // costs a tenth of the bandwidth here and a third in the fan-out kernel)
    const size_t lead = (size_t)a.lead_vecs, n_all = a.n_vec + lead;
    const size_t n_tiles = sl < 0 ? (n_all + kTile - 1) / kTile : ((n_all + (kTile << sl) - 1) / (kTile << sl)) << sl;
    for (size_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        uint4 x[VPT];
        size_t off[VPT];
        bool live[VPT];
        size_t first = tile * kTile, step = THREADS;
        if (sl >= 0) {
            const size_t r = tile & (((size_t)1 << sl) - 1);
            first = (((tile >> sl) * VPT) << sl) * THREADS + r * THREADS;
            step = (size_t)THREADS << sl;
            if (first >= n_all) continue;
        }
#pragma unroll
        for (int j = 0; j < VPT; ++j) {
            const size_t v = first + (size_t)j * step + threadIdx.x;
            live[j] = v >= lead && v < n_all;
            off[j] = a.byte_begin + ((live[j] ? v : v < lead ? lead : n_all - 1) - lead) * 16;
            x[j] = ld16(a.src, off[j]);
        }
        for (int d = 0; d < a.n_dst; ++d) {
            void *dst = a.dst0 ? a.dst0 : dsts[d];
#pragma unroll
            for (int j = 0; j < VPT; ++j)
                if (live[j]) st16(dst, off[j], x[j]);
        }
    }
    if (blockIdx.x == 0 && (int)threadIdx.x < a.n_tail_bytes) {
        const size_t off = a.byte_begin + a.n_vec * 16 + threadIdx.x;
        const unsigned char b = *((const unsigned char *)a.src + off);
        for (int d = 0; d < a.n_dst; ++d) *((unsigned char *)(a.dst0 ? a.dst0 : dsts[d]) + off) = b;
    }
}
// destination table in device memory (or the single destination a.dst0)
template <int VPT, int THREADS>
__global__ __launch_bounds__(THREADS) void copy_kernel(CopyArgs a)
{
    copy_body<VPT, THREADS>(a, (table_ptr)(uintptr_t)a.dsts);
}

// One source, several destinations, the source read through the caches: a workgroup copies
// one tile to one destination and ends. The tiles of a launch are grouped into spans; within
// a span the workgroups go destination by destination, tile index fastest. Consecutive
// workgroups then store consecutive tiles of one destination (a stream of short-lived waves,
// which is what the memory system writes fastest), and a span's source tiles are read again
// for every destination from the L2 of the XCD that read them first: workgroups are dealt to
// the XCDs in turn and a span holds a multiple of 8 tiles, so a tile meets the same XCD for
// every destination, and a span is sized to leave each XCD's share well inside its L2.
template <int VPT, int THREADS, class Table>
__device__ __forceinline__ void fanout_body(const CopyArgs &a, const Table dsts)
{
    constexpr size_t kTile = (size_t)THREADS * VPT;
    const unsigned per_span = a.span_tiles * (unsigned)a.n_dst;
    const unsigned span = blockIdx.x / per_span, r = blockIdx.x - span * per_span;
    const unsigned first = span * a.span_tiles;
    const unsigned rest = a.n_tiles - first;
    const unsigned ts = rest < a.span_tiles ? rest : a.span_tiles;      // tiles in this span
    const unsigned d = r / ts, tile = first + (r - d * ts);
    void *dst = dsts[d];
    const size_t lead = (size_t)a.lead_vecs, n_all = a.n_vec + lead;    // as in copy_kernel
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        const size_t v = tile * kTile + (size_t)j * THREADS + threadIdx.x;
        if (v >= lead && v < n_all) {
            const size_t off = a.byte_begin + (v - lead) * 16;
            const u32x4 x = *(const u32x4 *)((const char *)a.src + off);
            __builtin_nontemporal_store(x, (u32x4 *)((char *)dst + off));
        }
    }
    if (blockIdx.x == 0 && (int)threadIdx.x < a.n_tail_bytes) {
        const size_t off = a.byte_begin + a.n_vec * 16 + threadIdx.x;
        const unsigned char b = *((const unsigned char *)a.src + off);
        for (int e = 0; e < a.n_dst; ++e) *((unsigned char *)dsts[e] + off) = b;
    }
}
// destination table in device memory
template <int VPT, int THREADS>
__global__ __launch_bounds__(THREADS) void fanout_kernel(CopyArgs a)
{
    fanout_body<VPT, THREADS>(a, (table_ptr)(uintptr_t)a.dsts);
}
// destination table inside the kernel arguments
template <int VPT, int THREADS>
__global__ __launch_bounds__(THREADS) void fanout_kernel_inline(CopyArgsInline a)
{
    fanout_body<VPT, THREADS>(a.base, &a.dsts[0]);
}

}  // namespace hop
