// Instantiations of the bf16-MFMA direct filter-gradient kernel whose operands stream straight into LDS.
#include "dfilter16b.hpp"
#include "owt_host.hpp"

namespace owt {

template <int V>
static hipError_t go(const GemmParams &p, hipStream_t s)
{
    constexpr DFilter16bVariant v = kDFilter16bVariants[V];
    const dim3 grid(owt_split_major_grid(p.tiles_m * p.tiles_n, p.splits));
    hipLaunchKernelGGL((dfilter16b_kernel<v.WK, v.WC, v.KB, v.tmax, v.SW, v.WPC, v.prf>), grid, dim3(64 * v.WK * v.WC), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && p.splits > 1) e = launch_splitk_reduce<EpiFilter>(p, s);
    return e;
}

hipError_t owt_launch_dfilter16b(int variant, const GemmParams &p, hipStream_t s)
{
    if (p.mask) return hipErrorInvalidValue;        // the kernel takes dz as it is
    switch (variant) {
    case 0: return go<0>(p, s);
    case 1: return go<1>(p, s);
    case 2: return go<2>(p, s);
    case 3: return go<3>(p, s);
    case 4: return go<4>(p, s);
    case 5: return go<5>(p, s);
    case 6: return go<6>(p, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace owt
