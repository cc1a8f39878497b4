// Instantiations of the small-channel strided filter-gradient kernel.
// Built twice: -DOWT_INST_BF16={0,1}.
#include "sfilter.hpp"
#include "owt_host.hpp"

#ifndef OWT_INST_BF16
#error "define OWT_INST_BF16 (0 fp32 storage, 1 bf16 storage)"
#endif

namespace owt {

#if OWT_INST_BF16
typedef bf16_t TT;
#define OWT_FN owt_launch_sfilter_bf16
#else
typedef float TT;
#define OWT_FN owt_launch_sfilter_f32
#endif

template <int ACCS>
static hipError_t go(const GemmParams &p, const SFilterGeom &sg, int ktiles, size_t lds, hipStream_t s)
{
    static bool attr_set = false;     // benign race: the attribute is idempotent
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)sfilter_kernel<TT, kSFilterNT, ACCS, kSFilterPNP, kSFilterDNP>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 152 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((sfilter_kernel<TT, kSFilterNT, ACCS, kSFilterPNP, kSFilterDNP>), dim3(ktiles, p.splits), dim3(kSFilterNT), lds, s, p, sg);
    return hipGetLastError();
}

hipError_t OWT_FN(const GemmParams &p, const SFilterGeom &sg, int ktiles, hipStream_t s)
{
    const size_t lds = ((size_t)sg.ROWS * sg.PITCH + (size_t)sg.DZP * 68) * 4 + (size_t)sg.DZP * 4;
    if (sg.NB > 4 * kSFilterACCS) return hipErrorInvalidValue;
    // three accumulator blocks per wavefront when they cover the filter (11x11x3: 12 blocks), else four
    hipError_t e = sg.NB <= 12 ? go<3>(p, sg, ktiles, lds, s) : go<kSFilterACCS>(p, sg, ktiles, lds, s);
    if (e == hipSuccess && p.splits > 1) e = launch_splitk_reduce<EpiFilter>(p, s);
    return e;
}

}  // namespace owt
