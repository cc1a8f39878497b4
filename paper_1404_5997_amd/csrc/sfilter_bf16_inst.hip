// Launcher of the bf16-MFMA small-channel strided filter-gradient kernel.
#include "sfilter16b.hpp"
#include "owt_host.hpp"

namespace owt {

hipError_t owt_launch_sfilter16(const GemmParams &p, const SFilter16Geom &sg, int ktiles, hipStream_t s)
{
    size_t lds = ((size_t)sg.ROWS * sg.PITCH + (size_t)sg.DZP * 80) * 2 + (size_t)sg.DZP * 4;
    const size_t scratch = (size_t)(kSFilter16NT / 8) * 64 * 4;      // the bias-gradient reduction reuses the start of LDS
    if (lds < scratch) lds = scratch;
    static bool attr_set = false;     // benign race: the attribute is idempotent
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)sfilter16_kernel<0>, hipFuncAttributeMaxDynamicSharedMemorySize, 152 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(sfilter16_kernel<0>, dim3(ktiles, p.splits), dim3(kSFilter16NT), lds, s, p, sg);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && p.splits > 1) e = launch_splitk_reduce<EpiFilter>(p, s);
    return e;
}

// The form whose units stream from global memory straight into two LDS stages (unmasked dz).
hipError_t owt_launch_sfilter16b(const GemmParams &p, const SFilter16Geom &sg, int ktiles, hipStream_t s)
{
    const int pp8 = ((sg.PITCH + 7) & ~7) / 8, pan_inst = (sg.ROWS * pp8 + 63) / 64, dz_inst = sg.DZP / 8;
    size_t lds = (size_t)2 * (pan_inst + dz_inst) * 1024 + (size_t)sg.DZP * 4;
    if (lds < 32 * 1024) lds = 32 * 1024;     // the sum of the two pixel halves stages 4 column groups x 8 KB at the start of LDS
    if (pan_inst > 8 * kSFilter16bPNI || dz_inst > 8 * kSFilter16bDNI || lds > 158 * 1024 || p.mask) return hipErrorInvalidValue;
    static bool attr_set = false;     // benign race: the attribute is idempotent
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)sfilter16b_kernel<kSFilter16bPNI, kSFilter16bDNI>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 158 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((sfilter16b_kernel<kSFilter16bPNI, kSFilter16bDNI>), dim3(ktiles, p.splits), dim3(kSFilter16NT), lds, s, p, sg);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && p.splits > 1) e = launch_splitk_reduce<EpiFilter>(p, s);
    return e;
}

}  // namespace owt
