// Instantiations of the dense GEMM kernel of the fully-connected shard (fp32 storage).
#include "fcgemm.hpp"
#include "owt_host.hpp"

namespace owt {

template <int PASS, int T>
static hipError_t go(const GemmParams &p, hipStream_t s)
{
    constexpr FcTile t = kFcTiles[T];
    constexpr bool AKM = PASS != OWT_PASS_BWD_FILTER, BKM = PASS == OWT_PASS_FWD;
    typedef typename std::conditional<PASS == OWT_PASS_FWD, EpiFwd<float>,
            typename std::conditional<PASS == OWT_PASS_BWD_DATA, EpiData<float>, EpiFilter>::type>::type Epi;
    const dim3 grid(p.tiles_m * p.tiles_n, p.splits);
    hipLaunchKernelGGL((fcgemm_kernel<AKM, BKM, Epi, t.WM, t.WN, t.MB, t.NB, t.occ>), grid, dim3(64 * t.WM * t.WN), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && p.splits > 1) e = launch_splitk_reduce<Epi>(p, s);
    return e;
}

template <int PASS>
static hipError_t by_tile(int tile, const GemmParams &p, hipStream_t s)
{
    switch (tile) {
    case 0: return go<PASS, 0>(p, s);
    case 1: return go<PASS, 1>(p, s);
    case 2: return go<PASS, 2>(p, s);
    case 3: return go<PASS, 3>(p, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t owt_launch_fcgemm(int pass, int tile, const GemmParams &p0, float *dz, hipStream_t s)
{
    GemmParams p = p0;
    // what the kernel takes for granted
    if (p.M < 1 || p.Ncols < 1 || p.Kd < 1 || p.splits < 1 || p.ksteps != (p.Kd + 31) / 32 ||
        (long)(p.splits - 1) * p.ksteps_per_split >= p.ksteps || (long)p.splits * p.ksteps_per_split < p.ksteps ||
        (pass == OWT_PASS_FWD ? p.Kd % 32 != 0 : p.Ncols % 4 != 0))
        return hipErrorInvalidValue;
    p.kvalid = p.Kd;
    if (pass == OWT_PASS_FWD) {
        p.lda = p.ldb = p.Kd;
    } else {
        // dz[n][o]: n = rows of A in the data pass, reduction index in the filter pass
        const int N = pass == OWT_PASS_BWD_DATA ? p.M : p.Kd, O = pass == OWT_PASS_BWD_DATA ? p.Kd : p.M;
        const bool copy = p.mask || N % 32 || O % 32, db = pass == OWT_PASS_BWD_FILTER && p.dbias;
        const int Np = (N + 31) & ~31, Op = (O + 31) & ~31;
        if (copy || db) {
            hipLaunchKernelGGL(fc_dz_kernel, dim3(Op / 32), dim3(256), 0, s, (const float *)p.a, (const float *)p.mask,
                               copy ? dz : nullptr, db ? p.dbias : nullptr, p.alpha, p.beta, N, O, Np, Op);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        if (copy) p.a = dz;
        p.mask = nullptr; p.dbias = nullptr;
        p.lda = copy ? Op : O;
        p.ldb = p.Ncols;
    }
    switch (pass) {
    case OWT_PASS_FWD: return by_tile<OWT_PASS_FWD>(tile, p, s);
    case OWT_PASS_BWD_DATA: return by_tile<OWT_PASS_BWD_DATA>(tile, p, s);
    case OWT_PASS_BWD_FILTER: return by_tile<OWT_PASS_BWD_FILTER>(tile, p, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace owt
