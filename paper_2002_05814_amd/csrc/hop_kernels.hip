// gfx950 kernels of the chunked N-way reduce: a bandwidth-bound multi-input
// streaming reduce that evaluates the tree expression in registers, and a
// chunked one-to-many copy.
//
// The reduce is the elementwise ReduceOp of the paper's Table 1 applied in the
// order fixed by the reduce tree of section 3.4.2; the copy is the data
// movement of the broadcast of section 3.4.1. Both are pure streaming work:
// every input byte is read once with 128-bit loads, nothing is staged through
// LDS and no matrix unit is involved.
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

// binary32 -> bfloat16 bits, round to nearest, ties to even; NaN stays a quiet NaN.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = f32_to_bits(f);
    uint32_t rounded = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    uint32_t nan = (u >> 16) | 0x0040u;
    return ((u & 0x7fffffffu) > 0x7f800000u) ? nan : rounded;
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
template <int DT> __device__ __forceinline__ void decode(const uint4 &r, typename Traits<DT>::acc_t (&x)[Traits<DT>::W]);
template <> __device__ __forceinline__ void decode<HOP_F32>(const uint4 &r, float (&x)[4])
{
    x[0] = bits_to_f32(r.x); x[1] = bits_to_f32(r.y); x[2] = bits_to_f32(r.z); x[3] = bits_to_f32(r.w);
}
template <> __device__ __forceinline__ void decode<HOP_I32>(const uint4 &r, int32_t (&x)[4])
{
    x[0] = (int32_t)r.x; x[1] = (int32_t)r.y; x[2] = (int32_t)r.z; x[3] = (int32_t)r.w;
}
template <> __device__ __forceinline__ void decode<HOP_BF16>(const uint4 &r, float (&x)[8])
{
    // element 2i is the low half of word i (little endian); widening is exact
    x[0] = bits_to_f32(r.x << 16); x[1] = bits_to_f32(r.x & 0xffff0000u);
    x[2] = bits_to_f32(r.y << 16); x[3] = bits_to_f32(r.y & 0xffff0000u);
    x[4] = bits_to_f32(r.z << 16); x[5] = bits_to_f32(r.z & 0xffff0000u);
    x[6] = bits_to_f32(r.w << 16); x[7] = bits_to_f32(r.w & 0xffff0000u);
}

template <int DT> __device__ __forceinline__ uint4 encode(const typename Traits<DT>::acc_t (&x)[Traits<DT>::W]);
template <> __device__ __forceinline__ uint4 encode<HOP_F32>(const float (&x)[4])
{
    return make_uint4(f32_to_bits(x[0]), f32_to_bits(x[1]), f32_to_bits(x[2]), f32_to_bits(x[3]));
}
template <> __device__ __forceinline__ uint4 encode<HOP_I32>(const int32_t (&x)[4])
{
    return make_uint4((uint32_t)x[0], (uint32_t)x[1], (uint32_t)x[2], (uint32_t)x[3]);
}
template <> __device__ __forceinline__ uint4 encode<HOP_BF16>(const float (&x)[8])
{
    return make_uint4(f32_to_bf16_bits(x[0]) | (f32_to_bf16_bits(x[1]) << 16),
                      f32_to_bf16_bits(x[2]) | (f32_to_bf16_bits(x[3]) << 16),
                      f32_to_bf16_bits(x[4]) | (f32_to_bf16_bits(x[5]) << 16),
                      f32_to_bf16_bits(x[6]) | (f32_to_bf16_bits(x[7]) << 16));
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
};

__device__ __forceinline__ uint4 ld16(const void *base, size_t byte_off)
{
    return *(const uint4 *)((const char *)base + byte_off);
}
__device__ __forceinline__ void st16(void *base, size_t byte_off, const uint4 &v)
{
    *(uint4 *)((char *)base + byte_off) = v;
}

// Loads issued back to back per lane before any of them is consumed.
constexpr int kUnroll = 8;
constexpr int kThreads = 256;

// The program is read through the constant address space: it is never written
// while a kernel runs, so its steps can be fetched with scalar loads and held
// in SGPRs (a plain global pointer would make the compiler assume that the
// result stores may change it, and fall back to per-lane loads).
typedef const DevEntry __attribute__((address_space(4))) *prog_ptr;

template <int DT, int OP, int D>
__global__ __launch_bounds__(kThreads) void reduce_kernel(ReduceArgs a)
{
    using T = Traits<DT>;
    using A = typename T::acc_t;
    const prog_ptr prog = (prog_ptr)(uintptr_t)a.prog;
    const int n = a.n_entries;
    const size_t stride = (size_t)gridDim.x * kThreads;

    for (size_t v = (size_t)blockIdx.x * kThreads + threadIdx.x; v < a.n_vec; v += stride) {
        const size_t off = a.byte_begin + v * 16;
        Machine<DT, OP, D, T::W> m;
        int t = 0;
        for (; t + kUnroll <= n; t += kUnroll) {
            uint4 raw[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) raw[u] = ld16(prog[t + u].src, off);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                A x[T::W];
                decode<DT>(raw[u], x);
                m.step(prog[t + u].ctl, x);
            }
        }
        for (; t < n; ++t) {
            uint4 raw = ld16(prog[t].src, off);
            A x[T::W];
            decode<DT>(raw, x);
            m.step(prog[t].ctl, x);
        }
        const uint4 out = encode<DT>(m.acc[0]);
        st16(a.dst, off, out);
        for (int j = 0; j < a.n_extra; ++j) st16(a.extra_dsts[j], off, out);
    }

    // ragged tail: fewer than 16 bytes at the very end of the object
    if (blockIdx.x == 0 && (int)threadIdx.x < a.n_tail) {
        const size_t off = a.byte_begin + a.n_vec * 16 + (size_t)threadIdx.x * T::ES;
        Machine<DT, OP, D, 1> m;
        for (int t = 0; t < n; ++t) {
            A x[1] = {load_elem<DT>(prog[t].src, off)};
            m.step(prog[t].ctl, x);
        }
        store_elem<DT>(a.dst, off, m.acc[0][0]);
        for (int j = 0; j < a.n_extra; ++j) store_elem<DT>(a.extra_dsts[j], off, m.acc[0][0]);
    }
}

// One source, n_dst destinations: each 16-byte vector is read once and
// written n_dst times.
__global__ __launch_bounds__(kThreads) void copy_kernel(CopyArgs a)
{
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t v = (size_t)blockIdx.x * kThreads + threadIdx.x; v < a.n_vec; v += stride) {
        const size_t off = a.byte_begin + v * 16;
        const uint4 x = ld16(a.src, off);
        for (int j = 0; j < a.n_dst; ++j) st16(a.dsts[j], off, x);
    }
    if (blockIdx.x == 0 && (int)threadIdx.x < a.n_tail_bytes) {
        const size_t off = a.byte_begin + a.n_vec * 16 + threadIdx.x;
        const unsigned char b = *((const unsigned char *)a.src + off);
        for (int j = 0; j < a.n_dst; ++j) *((unsigned char *)a.dsts[j] + off) = b;
    }
}

// ----------------------------------------------------------------------------
// launch helpers
// ----------------------------------------------------------------------------

typedef void (*reduce_fn)(ReduceArgs);

template <int DT, int OP> static reduce_fn pick_depth(int depth)
{
    if (depth <= 1) return reduce_kernel<DT, OP, 1>;
    if (depth <= 2) return reduce_kernel<DT, OP, 2>;
    if (depth <= 4) return reduce_kernel<DT, OP, 4>;
    if (depth <= 8) return reduce_kernel<DT, OP, 8>;
    return reduce_kernel<DT, OP, 16>;
}
template <int DT> static reduce_fn pick_op(int op, int depth)
{
    switch (op) {
    case HOP_SUM: return pick_depth<DT, HOP_SUM>(depth);
    case HOP_MIN: return pick_depth<DT, HOP_MIN>(depth);
    default:      return pick_depth<DT, HOP_MAX>(depth);
    }
}

static int grid_for(size_t n_vec, int blocks_per_cu, int n_cu)
{
    size_t tiles = (n_vec + kThreads - 1) / kThreads;
    size_t cap = (size_t)n_cu * (size_t)blocks_per_cu;
    size_t g = tiles < cap ? tiles : cap;
    return (int)(g < 1 ? 1 : g);
}

int elem_bytes(int dtype) { return dtype == HOP_BF16 ? 2 : 4; }

hipError_t launch_reduce(hipStream_t stream, int dtype, int op, int depth, const DevEntry *prog,
                         int n_entries, void *dst, void *const *extra_dsts, int n_extra,
                         size_t byte_begin, size_t byte_end, int n_cu)
{
    if (byte_end <= byte_begin || n_entries <= 0) return hipSuccess;
    ReduceArgs a;
    a.prog = prog;
    a.n_entries = n_entries;
    a.dst = dst;
    a.extra_dsts = extra_dsts;
    a.n_extra = n_extra;
    a.byte_begin = byte_begin;
    a.n_vec = (byte_end - byte_begin) / 16;
    a.n_tail = (int)(((byte_end - byte_begin) % 16) / elem_bytes(dtype));
    reduce_fn fn;
    switch (dtype) {
    case HOP_F32:  fn = pick_op<HOP_F32>(op, depth); break;
    case HOP_BF16: fn = pick_op<HOP_BF16>(op, depth); break;
    default:       fn = pick_op<HOP_I32>(op, depth); break;
    }
    const int grid = grid_for(a.n_vec, kReduceBlocksPerCu, n_cu);
    hipLaunchKernelGGL(fn, dim3(grid), dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_copy(hipStream_t stream, const void *src, void *const *dsts, int n_dst,
                       size_t byte_begin, size_t byte_end, int n_cu)
{
    if (byte_end <= byte_begin || n_dst <= 0) return hipSuccess;
    CopyArgs a;
    a.src = src;
    a.dsts = dsts;
    a.n_dst = n_dst;
    a.byte_begin = byte_begin;
    a.n_vec = (byte_end - byte_begin) / 16;
    a.n_tail_bytes = (int)((byte_end - byte_begin) % 16);
    const int grid = grid_for(a.n_vec, kCopyBlocksPerCu, n_cu);
    hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

}  // namespace hop
