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
    hipLaunchKernelGGL((fcgemm_kernel<AKM, BKM, Epi, t.WM, t.WN, t.MB, t.NB, t.NS, t.occ>), grid, dim3(64 * t.WM * t.WN), 0, s, p);
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

// Checks what the kernel takes for granted and sets the operand pitches; `prepared` = a already points at
// the padded dz copy (or at dy when no copy is needed) and the bias gradient is done.
static bool frame(int pass, GemmParams &p)
{
    if (p.M < 1 || p.Ncols < 1 || p.Kd < 1 || p.splits < 1 || p.ksteps != (p.Kd + 31) / 32 ||
        (long)(p.splits - 1) * p.ksteps_per_split >= p.ksteps || (long)p.splits * p.ksteps_per_split < p.ksteps ||
        (pass == OWT_PASS_FWD ? p.Kd % 32 != 0 : p.Ncols % 4 != 0))
        return false;
    p.kvalid = p.Kd;
    p.ldb = pass == OWT_PASS_FWD ? p.Kd : p.Ncols;
    if (pass == OWT_PASS_FWD) p.lda = p.Kd;
    return true;
}

// dz[n][o] of a backward pass: n = rows of A in the data pass, reduction index in the filter pass.  Runs
// fc_dz_kernel when a masked or zero-padded copy or the bias gradient is wanted and points p at the result.
static hipError_t prepare_dz(int pass, GemmParams &p, float *dz, float *dbias, hipStream_t s)
{
    const int N = pass == OWT_PASS_BWD_DATA ? p.M : p.Kd, O = pass == OWT_PASS_BWD_DATA ? p.Kd : p.M;
    const bool copy = p.mask || N % 32 || O % 32;
    const int Np = (N + 31) & ~31, Op = (O + 31) & ~31;
    if (copy || dbias) {
        hipLaunchKernelGGL(fc_dz_kernel, dim3(Op / 16), dim3(256), 0, s, (const float *)p.a, (const float *)p.mask,
                           copy ? dz : nullptr, dbias, p.alpha, p.beta, N, O, Np, Op);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (copy) p.a = dz;
    p.mask = nullptr; p.dbias = nullptr;
    p.lda = copy ? Op : O;
    return hipSuccess;
}

hipError_t owt_launch_fcgemm(int pass, int tile, const GemmParams &p0, float *dz, hipStream_t s)
{
    GemmParams p = p0;
    if (!frame(pass, p)) return hipErrorInvalidValue;
    if (pass != OWT_PASS_FWD) {
        hipError_t e = prepare_dz(pass, p, dz, pass == OWT_PASS_BWD_FILTER ? p.dbias : nullptr, s);
        if (e != hipSuccess) return e;
    }
    switch (pass) {
    case OWT_PASS_FWD: return by_tile<OWT_PASS_FWD>(tile, p, s);
    case OWT_PASS_BWD_DATA: return by_tile<OWT_PASS_BWD_DATA>(tile, p, s);
    case OWT_PASS_BWD_FILTER: return by_tile<OWT_PASS_BWD_FILTER>(tile, p, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t owt_launch_fcgemm_bwd(int tile_d, int tile_f, bool fused, const GemmParams &pd0, const GemmParams &pf0, float *dz,
                                 hipStream_t s)
{
    GemmParams pd = pd0, pf = pf0;
    if (!frame(OWT_PASS_BWD_DATA, pd) || !frame(OWT_PASS_BWD_FILTER, pf)) return hipErrorInvalidValue;
    if (fused && (tile_d != kFcPairTile || tile_f != kFcPairTile || pd.splits != 1 || pf.splits != 1)) return hipErrorInvalidValue;
    // one dz for both products (the filter pass's view decides the bias gradient)
    hipError_t e = prepare_dz(OWT_PASS_BWD_FILTER, pf, dz, pf.dbias, s);
    if (e != hipSuccess) return e;
    pd.a = pf.a; pd.lda = pf.lda; pd.mask = nullptr;
    if (!fused) {
        e = by_tile<OWT_PASS_BWD_DATA>(tile_d, pd, s);
        return e != hipSuccess ? e : by_tile<OWT_PASS_BWD_FILTER>(tile_f, pf, s);
    }
    constexpr FcTile t = kFcTiles[kFcPairTile];
    const dim3 grid(pd.tiles_m * pd.tiles_n + pf.tiles_m * pf.tiles_n);
    hipLaunchKernelGGL((fcgemm_bwd_pair_kernel<t.WM, t.WN, t.MB, t.NB, t.NS, t.occ>), grid, dim3(64 * t.WM * t.WN), 0, s, pd, pf);
    return hipGetLastError();
}

}  // namespace owt
