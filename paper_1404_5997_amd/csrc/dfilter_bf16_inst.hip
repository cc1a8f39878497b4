// Instantiations of the bf16-MFMA direct filter-gradient kernel.
#include "dfilter_bf16.hpp"
#include "owt_host.hpp"

namespace owt {

template <int WK, int WC, int KB, int TMAX, int PRF>
static hipError_t go(const GemmParams &p, hipStream_t s)
{
    const dim3 grid(p.tiles_m * p.tiles_n, p.splits);
    hipLaunchKernelGGL((dfilter16_kernel<WK, WC, KB, TMAX, PRF>), grid, dim3(64 * WK * WC), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && p.splits > 1) e = launch_splitk_reduce<EpiFilter>(p, s);
    return e;
}

hipError_t owt_launch_dfilter16(int variant, const GemmParams &p, hipStream_t s)
{
    switch (variant) {
    case 0: return go<kDFilter16Variants[0].WK, kDFilter16Variants[0].WC, kDFilter16Variants[0].KB, kDFilter16Variants[0].tmax,
                      kDFilter16Variants[0].prf>(p, s);
    case 1: return go<kDFilter16Variants[1].WK, kDFilter16Variants[1].WC, kDFilter16Variants[1].KB, kDFilter16Variants[1].tmax,
                      kDFilter16Variants[1].prf>(p, s);
    case 2: return go<kDFilter16Variants[2].WK, kDFilter16Variants[2].WC, kDFilter16Variants[2].KB, kDFilter16Variants[2].tmax,
                      kDFilter16Variants[2].prf>(p, s);
    case 3: return go<kDFilter16Variants[3].WK, kDFilter16Variants[3].WC, kDFilter16Variants[3].KB, kDFilter16Variants[3].tmax,
                      kDFilter16Variants[3].prf>(p, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace owt
