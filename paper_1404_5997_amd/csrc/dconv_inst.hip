// Instantiations of the panel-resident stride-1 kernel for one (pass, storage type) pair.
// Built four times: -DOWT_INST_PASS={0,1} -DOWT_INST_BF16={0,1}.
#include "dconv.hpp"
#include "owt_host.hpp"

#ifndef OWT_INST_PASS
#error "define OWT_INST_PASS (0 fwd, 1 bwd-data)"
#endif
#ifndef OWT_INST_BF16
#error "define OWT_INST_BF16 (0 fp32 storage, 1 bf16 storage)"
#endif

namespace owt {

#if OWT_INST_BF16
typedef bf16_t TT;
#define OWT_SFX(n) n##_bf16
#else
typedef float TT;
#define OWT_SFX(n) n##_f32
#endif

#if OWT_INST_PASS == 0
typedef EpiFwd<TT> OE;
constexpr bool kBwd = false;
#define OWT_FN OWT_SFX(owt_launch_dconv_fwd)
#else
typedef EpiData<TT> OE;
constexpr bool kBwd = true;
#define OWT_FN OWT_SFX(owt_launch_dconv_data)
#endif

template <int WM, int WN, int PR, int BK, int MB = 2, int OCC = 2>
static hipError_t go(const GemmParams &p, hipStream_t s)
{
    const dim3 grid(p.tiles_m * p.tiles_n, p.splits);
    hipLaunchKernelGGL((dconv_kernel<TT, OE, kBwd, WM, WN, PR, BK, MB, OCC>), grid, dim3(64 * WM * WN), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && p.splits > 1) e = launch_splitk_reduce<OE>(p, s);
    return e;
}

hipError_t OWT_FN(int tile, int pr, const GemmParams &p, hipStream_t s)
{
    // 128x128: 32-channel chunks; 128x64 (two wavefronts): 16-channel chunks keep LDS small
    // enough for five work-groups per CU
    if (tile == TILE_128x128) {
        if (pr <= 160) return go<2, 2, 160, 32>(p, s);
        if (pr <= 256) return go<2, 2, 256, 32>(p, s);
    } else if (tile == TILE_128x64) {
        if (pr <= 160) return go<2, 1, 160, 16>(p, s);
        if (pr <= 256) return go<2, 1, 256, 16>(p, s);
    } else if (tile == TILE_128x64H) {
        if (pr <= 160) return go<4, 1, 160, 32, 1, 3>(p, s);     // 42 KB of LDS, 126 registers: three per CU
        if (pr <= 244) return go<4, 1, 244, 32, 1, 3>(p, s);     // 53 KB of LDS: three work-groups per CU
        if (pr <= 256) return go<4, 1, 256, 32, 1>(p, s);
    } else if (tile == TILE_128x128H) {
        if (pr <= 160) return go<4, 2, 160, 32, 1>(p, s);
        if (pr <= 256) return go<4, 2, 256, 32, 1>(p, s);
    } else if (tile == TILE_256x64) {
        if (pr <= 288) return go<4, 1, 288, 32>(p, s);
        if (pr <= 384) return go<4, 1, 384, 32>(p, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace owt
