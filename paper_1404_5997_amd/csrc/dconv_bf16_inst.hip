// Instantiations of the bf16-MFMA stride-1 kernel for one pass.
// Built twice: -DOWT_INST_PASS={0,1}.
#include "dconv_bf16p.hpp"
#include "owt_host.hpp"

#ifndef OWT_INST_PASS
#error "define OWT_INST_PASS (0 fwd, 1 bwd-data)"
#endif

namespace owt {

#if OWT_INST_PASS == 0
typedef EpiFwd<bf16_t> OE;
constexpr bool kBwd = false;
#else
typedef EpiData<bf16_t> OE;
constexpr bool kBwd = true;
#endif

template <int WM, int WN, int PR>
static hipError_t go(const GemmParams &p, hipStream_t s)
{
    const dim3 grid(p.tiles_m * p.tiles_n, p.splits);
    hipLaunchKernelGGL((dconv_bf16_kernel<OE, kBwd, WM, WN, PR>), grid, dim3(64 * WM * WN), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && p.splits > 1) e = launch_splitk_reduce<OE>(p, s);
    return e;
}

template <int PR, int MB, int OCC>
static hipError_t go_pipelined(const GemmParams &p, hipStream_t s)
{
    const dim3 grid(p.tiles_m * p.tiles_n, p.splits);
    hipLaunchKernelGGL((dconv16p_kernel<OE, kBwd, PR, MB, OCC>), grid, dim3(256), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && p.splits > 1) e = launch_splitk_reduce<OE>(p, s);
    return e;
}

static hipError_t dispatch(int tile, int pr, const GemmParams &p, hipStream_t s)
{
    if (tile == TILE_128x128) {
        if (pr <= 160) return go<2, 2, 160>(p, s);
        if (pr <= 256) return go<2, 2, 256>(p, s);
    } else if (tile == TILE_128x64) {
        if (pr <= 160) return go<2, 1, 160>(p, s);
        if (pr <= 256) return go<2, 1, 256>(p, s);
    } else if (tile == TILE_256x64) {
        if (pr <= 288) return go<4, 1, 288>(p, s);
        if (pr <= 384) return go<4, 1, 384>(p, s);
    } else if ((tile == TILE_512x64 || tile == TILE_256x64P) && p.Ncols % 4 == 0 && p.Cred % 32 == 0 &&
               p.g.R * p.g.S >= 2 && p.g.R * p.g.S <= 32) {
        if (tile == TILE_512x64) {
            if (pr <= 544) return go_pipelined<544, 4, 2>(p, s);
            if (pr <= 624) return go_pipelined<624, 4, 2>(p, s);
        } else {
            if (pr <= 288) return go_pipelined<288, 2, 3>(p, s);
            if (pr <= 384) return go_pipelined<384, 2, 3>(p, s);
        }
    }
    return hipErrorInvalidValue;
}

#if OWT_INST_PASS == 0
hipError_t owt_launch_dconv16_fwd(int tile, int pr, const GemmParams &p, hipStream_t s) { return dispatch(tile, pr, p, s); }
#else
hipError_t owt_launch_dconv16_data(int tile, int pr, const GemmParams &p0, void *ws, hipStream_t s)
{
    const Geom &g = p0.g;
    const int total = g.K * g.R * g.S * g.C;
    hipLaunchKernelGGL(flip_transpose_filters_kernel<uint16_t>, dim3((total + 255) / 256 > 4096 ? 4096 : (total + 255) / 256), dim3(256),
                       0, s, (const uint16_t *)p0.b, (uint16_t *)ws, g.K, g.R * g.S, g.C);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    GemmParams p = p0;
    p.b = ws;
    return dispatch(tile, pr, p, s);
}
#endif

}  // namespace owt
