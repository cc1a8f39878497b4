// Instantiations of the small-channel strided forward kernel.
// Built twice: -DOWT_INST_BF16={0,1}.
#include "sconv.hpp"
#include "owt_host.hpp"

#ifndef OWT_INST_BF16
#error "define OWT_INST_BF16 (0 fp32 storage, 1 bf16 storage)"
#endif

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

}  // namespace owt
