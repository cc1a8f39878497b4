// Launcher of the bf16-MFMA small-channel strided forward kernel.
#include "sconv_bf16.hpp"
#include "owt_host.hpp"

namespace owt {

hipError_t owt_launch_sconv16(const GemmParams &p, const SConv16Geom &sg, int ktiles, int nwg, void *w2, hipStream_t s)
{
    const size_t lds = ((size_t)sg.BIAS + 128 + (sg.STAGE > 0 ? kSConv16StageValues : 0)) * 2;
    static bool attr_set = false;     // benign race: the attribute is idempotent
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)sconv16_fwd_kernel<0>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int total = p.g.K * sg.KSLOTS;
    hipLaunchKernelGGL(sconv16_pack_filters_kernel<0>, dim3((total + 255) / 256), dim3(256), 0, s, (const uint16_t *)p.b,
                       (uint16_t *)w2, p.g.K, p.g.R, sg);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(sconv16_fwd_kernel<0>, dim3(ktiles, nwg), dim3(kSConv16NT), lds, s, p, sg, (const uint16_t *)w2);
    return hipGetLastError();
}

}  // namespace owt
