// Instantiations of the direct filter-gradient kernel for one storage type.
// Built twice: -DOWT_INST_BF16={0,1}.
#include "dfilter.hpp"
#include "owt_host.hpp"

#ifndef OWT_INST_BF16
#error "define OWT_INST_BF16 (0 fp32 storage, 1 bf16 storage)"
#endif

namespace owt {

#if OWT_INST_BF16
typedef bf16_t TT;
#define OWT_FN owt_launch_dfilter_bf16
#else
typedef float TT;
#define OWT_FN owt_launch_dfilter_f32
#endif

template <int V>
static hipError_t go(const GemmParams &p, hipStream_t s)
{
    constexpr DFilterVariant v = kDFilterVariants[V];
    const dim3 grid(owt_split_major_grid(p.tiles_m * p.tiles_n, p.splits));
    // the low-vector-ALU form of the loader and fetch: fp32 storage, chunks cut per image, one filter row per
    // work-group, dz not masked by the call, tables and byte offsets within their ranges
    const long IP = (long)p.Hp * p.Wp, PQ = (long)p.g.P * p.g.Q;
    const bool fast = !OWT_INST_BF16 && v.aligned && p.cpi > 0 && p.groups > 1 && !p.mask && IP + v.prf <= 1152 && PQ <= 1024 &&
                      (long)p.g.N * p.g.H * p.g.W * p.g.C * 4 < 0x7fffffffL && (long)p.g.N * PQ * p.g.K * 4 < 0x7fffffffL;
    if (v.aligned && !OWT_INST_BF16 && fast)
        hipLaunchKernelGGL((dfilter_kernel<TT, v.WK, v.WC, v.tmax, v.prf, v.occ, v.aligned && !OWT_INST_BF16>), grid, dim3(64 * v.WK * v.WC), 0, s, p);
    else
        hipLaunchKernelGGL((dfilter_kernel<TT, v.WK, v.WC, v.tmax, v.prf, v.occ>), grid, dim3(64 * v.WK * v.WC), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && p.splits > 1) e = launch_splitk_reduce<EpiFilter>(p, s);
    return e;
}

hipError_t OWT_FN(int variant, const GemmParams &p, hipStream_t s)
{
    switch (variant) {
    case 0: return go<0>(p, s);
    case 1: return go<1>(p, s);
    case 2: return go<2>(p, s);
    case 3: return go<3>(p, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace owt
