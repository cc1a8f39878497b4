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

hipError_t OWT_FN(const GemmParams &p, const SFilterGeom &sg, int ktiles, hipStream_t s)
{
    const size_t lds = ((size_t)sg.ROWS * sg.PITCH + (size_t)sg.DZP * 68) * 4 + (size_t)sg.DZP * 4;
    static bool attr_set = false;     // benign race: the attribute is idempotent
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)sfilter_kernel<TT, kSFilterNT, kSFilterACCS, kSFilterPNP, kSFilterDNP>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 152 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((sfilter_kernel<TT, kSFilterNT, kSFilterACCS, kSFilterPNP, kSFilterDNP>), dim3(ktiles, p.splits), dim3(kSFilterNT), lds, s, p, sg);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && p.splits > 1) e = launch_splitk_reduce<EpiFilter>(p, s);
    return e;
}

}  // namespace owt
