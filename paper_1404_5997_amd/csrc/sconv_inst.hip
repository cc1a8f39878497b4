// Instantiations of the small-channel strided forward kernel.
// Built twice: -DOWT_INST_BF16={0,1}.
#include "sconv.hpp"
#include "owt_host.hpp"

#ifndef OWT_INST_BF16
#error "define OWT_INST_BF16 (0 fp32 storage, 1 bf16 storage)"
#endif
#include "sconv2.hpp"

namespace owt {

#if OWT_INST_BF16
typedef bf16_t TT;
#define OWT_FN owt_launch_sconv_bf16
#else
typedef float TT;
#define OWT_FN owt_launch_sconv_f32
#endif

hipError_t OWT_FN(const GemmParams &p, const SConvGeom &sg, int ktiles, int nwg, float *w2, hipStream_t s)
{
    const size_t lds = ((size_t)2 * 64 * (kSConvBK + 4) + (size_t)sg.ZROWS * sg.PITCH) * 4;
    static bool attr_set = false;     // benign race: the attribute is idempotent
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)sconv_fwd_kernel<TT>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 152 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int total = p.g.K * sg.KSLOTS;
    hipLaunchKernelGGL((sconv_pack_filters_kernel<TT>), dim3((total + 255) / 256), dim3(256), 0, s,
                       (const TT *)p.b, w2, p.g.K, p.g.R, sg);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((sconv_fwd_kernel<TT>), dim3(ktiles, nwg), dim3(kSConvNT), lds, s, p, sg, (const float *)w2);
    return hipGetLastError();
}

#if !OWT_INST_BF16
// The filters-in-LDS form: ktiles tiles of 32 filters x nwg band groups, as a 1-D grid whose work-groups 8j .. 8j+7
// (one per XCD) take the same filter tile of eight neighbouring band groups.
hipError_t owt_launch_sconv2_f32(const GemmParams &p, const SConvGeom &sg, int ktiles, int nwg, float *w2, hipStream_t s)
{
    const size_t lds = ((size_t)kSConv2KB * (sg.KSLOTS + 4) + (size_t)sg.ZROWS * sg.PITCH) * 4;
    static bool attr_set = false;     // benign race: the attribute is idempotent
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)sconv2_fwd_kernel<10>, hipFuncAttributeMaxDynamicSharedMemorySize, 157 * 1024);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void *)sconv2_fwd_kernel<0>, hipFuncAttributeMaxDynamicSharedMemorySize, 157 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    if (lds > 157 * 1024) return hipErrorInvalidValue;
    const int total = p.g.K * sg.KSLOTS;
    hipLaunchKernelGGL((sconv_pack_filters_kernel<float>), dim3((total + 255) / 256), dim3(256), 0, s,
                       (const float *)p.b, w2, p.g.K, p.g.R, sg);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const dim3 grid(ktiles * ((nwg + 7) / 8) * 8);
    if (sg.KSTEPS == 10) hipLaunchKernelGGL(sconv2_fwd_kernel<10>, grid, dim3(kSConvNT), lds, s, p, sg, (const float *)w2, ktiles, nwg);
    else hipLaunchKernelGGL(sconv2_fwd_kernel<0>, grid, dim3(kSConvNT), lds, s, p, sg, (const float *)w2, ktiles, nwg);
    return hipGetLastError();
}
#endif

}  // namespace owt
