// Instantiations of the implicit-GEMM kernel for one (pass, storage type) pair.
// Built six times: -DOWT_INST_PASS={0,1,2} -DOWT_INST_BF16={0,1}.
#include "igemm.hpp"
#include "owt_host.hpp"

#ifndef OWT_INST_PASS
#error "define OWT_INST_PASS (0 fwd, 1 bwd-data, 2 bwd-filter)"
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
typedef FwdA<TT> OA; typedef FwdB<TT> OB; typedef EpiFwd<TT> OE;
#define OWT_FN OWT_SFX(owt_launch_fwd)
#elif OWT_INST_PASS == 1
typedef DataA<TT> OA; typedef DataB<TT> OB; typedef EpiData<TT> OE;
#define OWT_FN OWT_SFX(owt_launch_data)
#else
typedef FilterA<TT> OA; typedef FilterB<TT> OB; typedef EpiFilter OE;
#define OWT_FN OWT_SFX(owt_launch_filter)
#endif

template <int VA, int VB, int WM, int WN, int BK>
static hipError_t go(const GemmParams &p, hipStream_t s)
{
    const dim3 grid(p.tiles_m * p.tiles_n, p.splits);
    hipLaunchKernelGGL((igemm_kernel<OA, OB, OE, VA, VB, WM, WN, BK>), grid, dim3(64 * WM * WN), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && p.splits > 1) e = launch_splitk_reduce<OE>(p, s);
    return e;
}

hipError_t OWT_FN(int tile, int va, int vb, const GemmParams &p, hipStream_t s)
{
    if (va == 4 && vb == 4) {
        switch (tile) {
        case TILE_128x128: return go<4, 4, 2, 2, 32>(p, s);
        case TILE_128x64: return go<4, 4, 2, 1, 16>(p, s);
        case TILE_64x128: return go<4, 4, 1, 2, 16>(p, s);
        case TILE_64x64: return go<4, 4, 1, 1, 16>(p, s);
        default: return hipErrorInvalidValue;
        }
    }
    if (tile != TILE_64x64) return hipErrorInvalidValue;
#if OWT_INST_PASS == 0
    // both forward operands run along (r,s,c): one flag decides both
    return go<1, 1, 1, 1, 16>(p, s);
#else
    if (va == 1 && vb == 1) return go<1, 1, 1, 1, 16>(p, s);
    if (va == 1 && vb == 4) return go<1, 4, 1, 1, 16>(p, s);
    return go<4, 1, 1, 1, 16>(p, s);
#endif
}

}  // namespace owt
