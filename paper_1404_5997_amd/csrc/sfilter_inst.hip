// Instantiations of the small-channel strided filter-gradient kernel.
// Built twice: -DOWT_INST_BF16={0,1}.
#include "sfilter2.hpp"
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

#if !OWT_INST_BF16
// The form whose units stream from global memory straight into two LDS stages (fp32 storage, unmasked dz).
template <int ACCS, int FQ, int FPITCH, int FSWC, int FSH>
static hipError_t go2(const GemmParams &p, const SFilterGeom &sg, int ktiles, size_t lds, hipStream_t s)
{
    static bool attr_set = false;     // benign race: the attribute is idempotent
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)sfilter2_kernel<ACCS, kSFilter2PNI, kSFilter2DNI, FQ, FPITCH, FSWC, FSH>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 158 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((sfilter2_kernel<ACCS, kSFilter2PNI, kSFilter2DNI, FQ, FPITCH, FSWC, FSH>), dim3(ktiles, p.splits),
                       dim3(kSFilterNT), lds, s, p, sg);
    return hipGetLastError();
}

hipError_t owt_launch_sfilter2_f32(const GemmParams &p, const SFilterGeom &sg, int ktiles, hipStream_t s)
{
    const int pan_inst = (sg.ROWS * (sg.PITCH / 4) + 63) / 64, dz_inst = (sg.DZP * 17 + 63) / 64;
    const size_t lds = (size_t)2 * (pan_inst + dz_inst) * 1024 + (size_t)sg.DZP * 4;
    if (sg.NB > 4 * kSFilterACCS || pan_inst > 8 * kSFilter2PNI || dz_inst > 8 * kSFilter2DNI || lds > 158 * 1024 || p.mask)
        return hipErrorInvalidValue;
    // the Section 5 model's first layer (224x224x3 images, 11x11 filters, stride 4, pad 2: 55 windows per row, 12 floats
    // apart, panel rows of 684 floats) has an instantiation with its geometry at compile time
    const bool paper = p.g.Q == 55 && sg.PITCH == 684 && p.g.sw * p.g.C == 12 && p.g.sh == 4 && sg.NB <= 12;
    hipError_t e = paper ? go2<3, 55, 684, 12, 4>(p, sg, ktiles, lds, s)
                 : sg.NB <= 12 ? go2<3, 0, 0, 0, 0>(p, sg, ktiles, lds, s) : go2<kSFilterACCS, 0, 0, 0, 0>(p, sg, ktiles, lds, s);
    if (e == hipSuccess && p.splits > 1) e = launch_splitk_reduce<EpiFilter>(p, s);
    return e;
}
#endif

}  // namespace owt
