// Instantiations of the reduce kernels for ONE (element type, op) pair, chosen by
// -DHOP_INST_DT=<hop_dtype_t value> -DHOP_INST_OP=<hop_op_t value>. The build compiles
// this file once per pair, in parallel, so that no single compile is long.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hop_device.hpp"
#include "hop_kernels.h"
#include "hop_launch_shape.h"

#if !defined(HOP_INST_DT) || !defined(HOP_INST_OP)
#error "compile with -DHOP_INST_DT=<0|1|2> -DHOP_INST_OP=<0|1|2>"
#endif

namespace hop {

// The small-shape kernels whose steps may read partial results: for bf16 only, whose partial results are
// not of the element type.
template <int DT, int OP, int D> struct mixed_small {
    static void (*dev())(ReduceArgs) { return nullptr; }
    static void (*inl())(ReduceArgsInline) { return nullptr; }
};
template <int OP, int D> struct mixed_small<HOP_BF16, OP, D> {
    static void (*dev())(ReduceArgs) { return reduce_kernel_mixed<HOP_BF16, OP, D, 1, kSmallUnroll, kThreads>; }
    static void (*inl())(ReduceArgsInline) { return reduce_kernel_mixed_inline<HOP_BF16, OP, D, 1, kSmallUnroll, kThreads>; }
};

template <int DT, int OP, int D> static Launcher make_launcher()
{
    constexpr int V = VecPerLane<Traits<DT>::W, D>::value;
    return {reduce_kernel<DT, OP, D, V, kUnroll, kThreads>, reduce_kernel_inline<DT, OP, D, V, kUnroll, kThreads>,
            reduce_kernel<DT, OP, D, 1, kSmallUnroll, kThreads>,
            reduce_kernel_inline<DT, OP, D, 1, kSmallUnroll, kThreads>,
            mixed_small<DT, OP, D>::dev(), mixed_small<DT, OP, D>::inl(),
            reduce_kernel<DT, OP, D, (V < kMidVecs ? V : kMidVecs), kMidUnroll, kThreads>,
            reduce_kernel_inline<DT, OP, D, (V < kMidVecs ? V : kMidVecs), kMidUnroll, kThreads>,
            reduce_kernel_seg<DT, OP, D, V, kUnroll, kThreads>, reduce_kernel_kept<DT, OP, D, V, kThreads>,
            reduce_kernel_kept_inline<DT, OP, D, V, kThreads>, reduce_kernel_chains<DT, OP>,
            reduce_kernel_chains_inline<DT, OP, kChainInlineWordsSmall>, reduce_kernel_chains_inline<DT, OP, kChainInlineWordsMid>,
            reduce_kernel_chains_inline<DT, OP, kChainInlineWordsLarge>, reduce_kernel_chains_wide<DT, OP>,
            reduce_kernel_chains_wide_inline<DT, OP, kChainInlineWordsSmall>,
            reduce_kernel_chains_wide_inline<DT, OP, kChainInlineWordsMid>,
            reduce_kernel_chains_wide_inline<DT, OP, kChainInlineWordsLarge>, V};
}

#define HOP_CAT3(a, b, c) a##b##_##c
#define HOP_LAUNCHER_NAME(dt, op) HOP_CAT3(launcher_, dt, op)

Launcher HOP_LAUNCHER_NAME(HOP_INST_DT, HOP_INST_OP)(int depth)
{
    if (depth <= 1) return make_launcher<HOP_INST_DT, HOP_INST_OP, 1>();
    if (depth <= 2) return make_launcher<HOP_INST_DT, HOP_INST_OP, 2>();
    if (depth <= 4) return make_launcher<HOP_INST_DT, HOP_INST_OP, 4>();
    if (depth <= 8) return make_launcher<HOP_INST_DT, HOP_INST_OP, 8>();
    return make_launcher<HOP_INST_DT, HOP_INST_OP, 16>();
}

}  // namespace hop
