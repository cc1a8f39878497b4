// Instantiations of the filter-gradient kernel with the in-work-group pixel split (fp32 storage).
#include "dfilter2.hpp"
#include "owt_host.hpp"

namespace owt {

template <int V>
static hipError_t go(const GemmParams &p, hipStream_t s)
{
    constexpr DFilter2Variant v = kDFilter2Variants[V];
    const dim3 grid(owt_split_major_grid(p.tiles_m * p.tiles_n, p.splits));
    if (p.mask) return hipErrorInvalidValue;       // the planner sends masked calls to dfilter.hpp
    hipLaunchKernelGGL((dfilter2_kernel<v.WK, v.WP, v.tmax, v.SW, v.WPC, v.prows>), grid, dim3(64 * v.WK * v.WP), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && p.splits > 1) e = launch_splitk_reduce<EpiFilter>(p, s);
    return e;
}

hipError_t owt_launch_dfilter2_f32(int variant, const GemmParams &p, hipStream_t s)
{
    switch (variant) {
    case 0: return go<0>(p, s);
    case 1: return go<1>(p, s);
    case 2: return go<2>(p, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace owt
