// C ABI entry points of libowt: descriptor checks, planning, launches.
#include "owt_host.hpp"

namespace owt {

static thread_local char g_err[512] = "";

owt_status fail(owt_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}
void clear_error() { g_err[0] = 0; }

const TileInfo kTiles[NUM_TILES] = {
    {TILE_128x128, 2, 2, 32, 1.00f},
    {TILE_128x64, 2, 1, 16, 0.85f},
    {TILE_64x128, 1, 2, 16, 0.85f},
    {TILE_64x64, 1, 1, 16, 0.70f},
};

static inline long cdiv(long a, long b) { return (a + b - 1) / b; }

// Cost model in arbitrary time units: every CU works through ceil(WGs/256)
// work-groups of BM*BN*Kd/splits MACs each at the tile's relative efficiency; a
// split adds one write and one read of the partial results plus a launch.
Plan plan_gemm(long M, long Ncols, long Kd, bool vec_ok, bool want_dbias)
{
    static const int kSplits[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128, 192, 256};
    int force_tile = -1, force_split = -1;
    if (const char *e = getenv("OWT_TILE")) force_tile = atoi(e);
    if (const char *e = getenv("OWT_SPLITK")) force_split = atoi(e);
    Plan best; memset(&best, 0, sizeof(best));
    double best_cost = 1e300;
    for (int t = 0; t < NUM_TILES; t++) {
        if (!vec_ok && t != TILE_64x64) continue;
        if (vec_ok && force_tile >= 0 && force_tile < NUM_TILES && t != force_tile) continue;
        const TileInfo &ti = kTiles[t];
        const long BM = 64 * ti.WM, BN = 64 * ti.WN;
        const long tm = cdiv(M, BM), tn = cdiv(Ncols, BN), ksteps = cdiv(Kd, ti.BK);
        for (int s0 : kSplits) {
            long s = s0;
            if (force_split > 0) {           // tuning/test override: take it as given, capped by the steps there are
                if (s0 != 1) break;
                s = force_split < ksteps ? force_split : ksteps;
            } else if (s > 1 && ksteps / s < 4) {
                break;
            }
            const long per = cdiv(ksteps, s);
            const long splits = cdiv(ksteps, per);        // drop empty trailing splits
            const long wgs = tm * tn * splits;
            const double macs_per_wg = (double)BM * BN * ti.BK * per;
            double cost = (double)cdiv(wgs, 256) * macs_per_wg / (128.0 * ti.eff);   // ~clocks
            if (splits > 1) cost += 12000.0 + (double)(splits + 1) * M * Ncols * 4.0 / 1200.0;
            if (cost < best_cost) {
                best_cost = cost;
                best.tile = t; best.splits = (int)splits; best.ksteps = (int)ksteps;
                best.ksteps_per_split = (int)per; best.tiles_m = (int)tm; best.tiles_n = (int)tn;
            }
        }
    }
    if (best.splits > 1) {
        best.partial_bytes = (((size_t)best.splits * M * Ncols * 4) + 255) & ~(size_t)255;
        best.dbias_partial_bytes = want_dbias ? ((((size_t)best.splits * M * 4) + 255) & ~(size_t)255) : 0;
    }
    return best;
}

bool fill_geom(Geom &g, int N, int C, int H, int W, int K, int R, int S, int sh, int sw, int ph, int pw)
{
    g.N = N; g.C = C; g.H = H; g.W = W; g.K = K; g.R = R; g.S = S;
    g.sh = sh; g.sw = sw; g.ph = ph; g.pw = pw;
    g.P = (H + 2 * ph - R) / sh + 1;
    g.Q = (W + 2 * pw - S) / sw + 1;
    if (H + 2 * ph - R < 0 || W + 2 * pw - S < 0) return false;
    g.dC.set(C); g.dS.set(S); g.dK.set(K); g.dQ.set(g.Q); g.dPQ.set(g.P * g.Q);
    g.dW.set(W); g.dHW.set(H * W); g.dsh.set(sh); g.dsw.set(sw);
    return true;
}

owt_status run_pass(int pass, owt_dtype dt, int va, int vb, GemmParams &p, const Plan &pl,
                    void *ws, hipStream_t s)
{
    static const LaunchFn table[3][2] = {
        {owt_launch_fwd_f32, owt_launch_fwd_bf16},
        {owt_launch_data_f32, owt_launch_data_bf16},
        {owt_launch_filter_f32, owt_launch_filter_bf16},
    };
    p.splits = pl.splits; p.ksteps = pl.ksteps; p.ksteps_per_split = pl.ksteps_per_split;
    p.tiles_m = pl.tiles_m; p.tiles_n = pl.tiles_n;
    p.partial = pl.splits > 1 ? (float *)ws : nullptr;
    p.dbias_partial = (pl.splits > 1 && pl.dbias_partial_bytes) ? (float *)((char *)ws + pl.partial_bytes) : nullptr;
    const hipError_t e = table[pass][dt == OWT_BF16 ? 1 : 0](pl.tile, va, vb, p, s);
    if (e != hipSuccess) return fail(OWT_ELAUNCH, "HIP launch failed: %s", hipGetErrorString(e));
    return OWT_OK;
}

// ----------------------------------------------------------------- checking
static const long kMaxElems = 0x7fffffffL;   // tensors are indexed with 32-bit offsets

static owt_status check_conv(const owt_conv_desc *d, Geom &g)
{
    if (!d) return fail(OWT_EINVAL, "descriptor is NULL");
    if (d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0)
        return fail(OWT_EINVAL, "N,C,H,W,K,R,S must be positive");
    if (d->stride_h < 1 || d->stride_w < 1) return fail(OWT_EINVAL, "strides must be >= 1");
    if (d->pad_h < 0 || d->pad_w < 0 || d->pad_h >= d->R || d->pad_w >= d->S)
        return fail(OWT_EINVAL, "need 0 <= pad_h < R and 0 <= pad_w < S");
    if (d->dtype != OWT_F32 && d->dtype != OWT_BF16) return fail(OWT_EINVAL, "unknown dtype %d", (int)d->dtype);
    if (d->flags & ~(unsigned)(OWT_BIAS | OWT_RELU)) return fail(OWT_EINVAL, "unknown flag bits 0x%x", d->flags);
    if (!fill_geom(g, d->N, d->C, d->H, d->W, d->K, d->R, d->S, d->stride_h, d->stride_w, d->pad_h, d->pad_w))
        return fail(OWT_EINVAL, "filter larger than the padded input: no output");
    const long xe = (long)d->N * d->H * d->W * d->C, ye = (long)d->N * g.P * g.Q * d->K,
               we = (long)d->K * d->R * d->S * d->C;
    if (xe > kMaxElems || ye > kMaxElems || we > kMaxElems)
        return fail(OWT_EUNSUPPORTED, "tensor with more than 2^31-1 elements");
    return OWT_OK;
}

struct PassDims { long M, Ncols, Kd; bool va, vb; };

static PassDims conv_dims(const Geom &g, int pass)
{
    PassDims r;
    const bool c4 = g.C % 4 == 0, k4 = g.K % 4 == 0;
    if (pass == OWT_PASS_FWD) {
        r.M = (long)g.N * g.P * g.Q; r.Ncols = g.K; r.Kd = (long)g.R * g.S * g.C; r.va = r.vb = c4;
    } else if (pass == OWT_PASS_BWD_DATA) {
        r.M = (long)g.N * g.H * g.W; r.Ncols = g.C; r.Kd = (long)g.R * g.S * g.K; r.va = k4; r.vb = c4;
    } else {
        r.M = g.K; r.Ncols = (long)g.R * g.S * g.C; r.Kd = (long)g.N * g.P * g.Q; r.va = k4; r.vb = c4;
    }
    return r;
}

static owt_status check_ptr(const void *p, const char *name)
{
    if (!p) return fail(OWT_EINVAL, "%s is NULL", name);
    if (!aligned16(p)) return fail(OWT_EINVAL, "%s is not 16-byte aligned", name);
    return OWT_OK;
}

#define OWT_TRY(expr) do { owt_status st_ = (expr); if (st_ != OWT_OK) return st_; } while (0)

static owt_status conv_pass(const Geom &g, int pass, owt_dtype dt, GemmParams &p, bool want_db,
                            void *ws, size_t ws_bytes, hipStream_t s)
{
    const PassDims dm = conv_dims(g, pass);
    const Plan pl = plan_gemm(dm.M, dm.Ncols, dm.Kd, dm.va && dm.vb, want_db);
    if (pl.total_bytes() > ws_bytes)
        return fail(OWT_EWORKSPACE, "workspace too small: need %zu bytes, got %zu", pl.total_bytes(), ws_bytes);
    if (pl.total_bytes() && (!ws || !aligned16(ws))) return fail(OWT_EINVAL, "ws is NULL or misaligned");
    if ((long)pl.splits * dm.M * dm.Ncols > kMaxElems * 4L)
        return fail(OWT_EUNSUPPORTED, "split-K partials too large");
    p.g = g; p.M = (int)dm.M; p.Ncols = (int)dm.Ncols; p.Kd = (int)dm.Kd;
    return run_pass(pass, dt, dm.va ? 4 : 1, dm.vb ? 4 : 1, p, pl, ws, s);
}

}  // namespace owt

using namespace owt;

extern "C" {

const char *owt_last_error(void) { return g_err; }
int owt_abi_version(void) { return 1; }

int owt_selftest_host(void)
{
    // exact-division constants: every divisor up to 4100 plus large ones, against n around
    // multiples of d, small n and the top of the 31-bit range
    static const uint32_t big[] = {9216, 21632, 93312, 387200, 3097600, 50176, 0x7fffffffu, 0x40000001u};
    for (uint32_t i = 1; i <= 4100 + sizeof(big) / sizeof(big[0]); i++) {
        const uint32_t d = i <= 4100 ? i : big[i - 4101];
        FastDiv f; f.set(d);
        for (uint32_t j = 0; j < 64; j++) {
            const uint64_t mul = (uint64_t)d * (j * 0x01000193u % 100000u);
            const uint32_t cand[] = {j, (uint32_t)(mul & 0x7fffffffu), (uint32_t)((mul + d - 1) & 0x7fffffffu),
                                     0x7fffffffu - j, 0x7fffffffu / (j + 1)};
            for (uint32_t n : cand)
                if (f.div(n) != n / d) { fail(OWT_EINVAL, "FastDiv wrong: %u / %u", n, d); return 1; }
        }
    }
    // the planner never asks for more splits than there are BK steps and covers all of them
    for (long M : {1L, 64L, 125L, 21632L, 387200L})
        for (long Nc : {1L, 64L, 363L, 3456L})
            for (long Kd : {1L, 27L, 363L, 9216L, 387200L}) {
                const Plan pl = plan_gemm(M, Nc, Kd, true, true);
                if (pl.splits < 1 || (long)pl.splits * pl.ksteps_per_split < pl.ksteps ||
                    (long)(pl.splits - 1) * pl.ksteps_per_split >= pl.ksteps) {
                    fail(OWT_EINVAL, "bad plan for %ld x %ld x %ld", M, Nc, Kd); return 2;
                }
            }
    return 0;
}

size_t owt_conv_workspace_bytes(const owt_conv_desc *d, int pass)
{
    Geom g;
    if (pass < 0 || pass > 2) { fail(OWT_EINVAL, "pass must be 0, 1 or 2"); return (size_t)-1; }
    if (check_conv(d, g) != OWT_OK) return (size_t)-1;
    const PassDims dm = conv_dims(g, pass);
    return plan_gemm(dm.M, dm.Ncols, dm.Kd, dm.va && dm.vb, pass == OWT_PASS_BWD_FILTER).total_bytes();
}

int owt_conv_plan_describe(const owt_conv_desc *d, int pass, char *buf, size_t buf_bytes)
{
    Geom g;
    if (pass < 0 || pass > 2 || !buf || buf_bytes == 0) { fail(OWT_EINVAL, "bad pass or buffer"); return -1; }
    if (check_conv(d, g) != OWT_OK) return -1;
    const PassDims dm = conv_dims(g, pass);
    const Plan pl = plan_gemm(dm.M, dm.Ncols, dm.Kd, dm.va && dm.vb, pass == OWT_PASS_BWD_FILTER);
    static const char *pn[3] = {"fwd", "bwd_data", "bwd_filter"};
    const TileInfo &ti = kTiles[pl.tile];
    return snprintf(buf, buf_bytes, "igemm %s %s tile%dx%dx%d vec%d/%d splitk%d grid%dx%d", pn[pass],
                    d->dtype == OWT_BF16 ? "bf16" : "f32", 64 * ti.WM, 64 * ti.WN, ti.BK, dm.va ? 4 : 1,
                    dm.vb ? 4 : 1, pl.splits, pl.tiles_m * pl.tiles_n, pl.splits);
}

owt_status owt_conv_fwd(const owt_conv_desc *d, const void *x, const void *w, const float *bias,
                        void *y, void *ws, size_t ws_bytes, void *hip_stream)
{
    Geom g;
    OWT_TRY(check_conv(d, g));
    OWT_TRY(check_ptr(x, "x")); OWT_TRY(check_ptr(w, "w")); OWT_TRY(check_ptr(y, "y"));
    if (d->flags & OWT_BIAS) OWT_TRY(check_ptr(bias, "bias"));
    GemmParams p; memset(&p, 0, sizeof(p));
    p.a = x; p.b = w; p.out = y; p.bias = bias; p.flags = d->flags;
    return conv_pass(g, OWT_PASS_FWD, d->dtype, p, false, ws, ws_bytes, (hipStream_t)hip_stream);
}

owt_status owt_conv_bwd_data(const owt_conv_desc *d, const void *dy, const void *y_or_null,
                             const void *w, void *dx, void *ws, size_t ws_bytes, void *hip_stream)
{
    Geom g;
    OWT_TRY(check_conv(d, g));
    OWT_TRY(check_ptr(dy, "dy")); OWT_TRY(check_ptr(w, "w")); OWT_TRY(check_ptr(dx, "dx"));
    if (d->flags & OWT_RELU) OWT_TRY(check_ptr(y_or_null, "y (needed for the ReLU mask)"));
    GemmParams p; memset(&p, 0, sizeof(p));
    p.a = dy; p.b = w; p.out = dx; p.flags = d->flags;
    p.mask = (d->flags & OWT_RELU) ? y_or_null : nullptr;
    return conv_pass(g, OWT_PASS_BWD_DATA, d->dtype, p, false, ws, ws_bytes, (hipStream_t)hip_stream);
}

owt_status owt_conv_bwd_filter(const owt_conv_desc *d, const void *x, const void *dy,
                               const void *y_or_null, float alpha, float beta, float *dw,
                               float *dbias_or_null, void *ws, size_t ws_bytes, void *hip_stream)
{
    Geom g;
    OWT_TRY(check_conv(d, g));
    OWT_TRY(check_ptr(x, "x")); OWT_TRY(check_ptr(dy, "dy")); OWT_TRY(check_ptr(dw, "dw"));
    if (dbias_or_null) OWT_TRY(check_ptr(dbias_or_null, "dbias"));
    if (d->flags & OWT_RELU) OWT_TRY(check_ptr(y_or_null, "y (needed for the ReLU mask)"));
    GemmParams p; memset(&p, 0, sizeof(p));
    p.a = dy; p.b = x; p.out = dw; p.flags = d->flags; p.alpha = alpha; p.beta = beta;
    p.dbias = dbias_or_null;
    p.mask = (d->flags & OWT_RELU) ? y_or_null : nullptr;
    return conv_pass(g, OWT_PASS_BWD_FILTER, d->dtype, p, true, ws, ws_bytes, (hipStream_t)hip_stream);
}

// ------------------------------------------------------- fully-connected shard
static owt_status check_fc(const owt_fc_desc *d, Geom &g, int &o_local)
{
    if (!d) return fail(OWT_EINVAL, "descriptor is NULL");
    if (d->N <= 0 || d->I <= 0 || d->O_total <= 0 || d->workers <= 0)
        return fail(OWT_EINVAL, "N, I, O_total, workers must be positive");
    if (d->rank < 0 || d->rank >= d->workers) return fail(OWT_EINVAL, "need 0 <= rank < workers");
    if (d->O_total % d->workers) return fail(OWT_EINVAL, "O_total must be divisible by workers");
    if (d->dtype != OWT_F32 && d->dtype != OWT_BF16) return fail(OWT_EINVAL, "unknown dtype %d", (int)d->dtype);
    if (d->flags & ~(unsigned)(OWT_BIAS | OWT_RELU)) return fail(OWT_EINVAL, "unknown flag bits 0x%x", d->flags);
    o_local = d->O_total / d->workers;
    if ((long)d->N * d->I > kMaxElems || (long)o_local * d->I > kMaxElems)
        return fail(OWT_EUNSUPPORTED, "tensor with more than 2^31-1 elements");
    fill_geom(g, d->N, d->I, 1, 1, o_local, 1, 1, 1, 1, 0, 0);
    return OWT_OK;
}

size_t owt_fc_workspace_bytes(const owt_fc_desc *d, int pass)
{
    Geom g; int ol;
    if (pass < 0 || pass > 2) { fail(OWT_EINVAL, "pass must be 0, 1 or 2"); return (size_t)-1; }
    if (check_fc(d, g, ol) != OWT_OK) return (size_t)-1;
    if (pass == OWT_PASS_FWD) {
        const PassDims dm = conv_dims(g, OWT_PASS_FWD);
        return plan_gemm(dm.M, dm.Ncols, dm.Kd, dm.va && dm.vb, false).total_bytes();
    }
    // the backward call runs the data pass, then the filter pass, on one scratch area
    const PassDims d1 = conv_dims(g, OWT_PASS_BWD_DATA), d2 = conv_dims(g, OWT_PASS_BWD_FILTER);
    const size_t a = plan_gemm(d1.M, d1.Ncols, d1.Kd, d1.va && d1.vb, false).total_bytes();
    const size_t b = plan_gemm(d2.M, d2.Ncols, d2.Kd, d2.va && d2.vb, true).total_bytes();
    return a > b ? a : b;
}

owt_status owt_fc_shard_fwd(const owt_fc_desc *d, const void *x, const void *w, const float *bias,
                            void *y, void *ws, size_t ws_bytes, void *hip_stream)
{
    Geom g; int ol;
    OWT_TRY(check_fc(d, g, ol));
    OWT_TRY(check_ptr(x, "x")); OWT_TRY(check_ptr(w, "w")); OWT_TRY(check_ptr(y, "y"));
    if (d->flags & OWT_BIAS) OWT_TRY(check_ptr(bias, "bias"));
    GemmParams p; memset(&p, 0, sizeof(p));
    p.a = x; p.b = w; p.out = y; p.bias = bias; p.flags = d->flags;
    return conv_pass(g, OWT_PASS_FWD, d->dtype, p, false, ws, ws_bytes, (hipStream_t)hip_stream);
}

owt_status owt_fc_shard_bwd(const owt_fc_desc *d, const void *x, const void *w, const void *y_or_null,
                            const void *dy, float alpha, float beta, void *dx_partial_or_null,
                            float *dw, float *dbias_or_null, void *ws, size_t ws_bytes,
                            void *hip_stream)
{
    Geom g; int ol;
    OWT_TRY(check_fc(d, g, ol));
    OWT_TRY(check_ptr(x, "x")); OWT_TRY(check_ptr(w, "w")); OWT_TRY(check_ptr(dy, "dy"));
    OWT_TRY(check_ptr(dw, "dw"));
    if (dx_partial_or_null) OWT_TRY(check_ptr(dx_partial_or_null, "dx_partial"));
    if (dbias_or_null) OWT_TRY(check_ptr(dbias_or_null, "dbias"));
    if (d->flags & OWT_RELU) OWT_TRY(check_ptr(y_or_null, "y (needed for the ReLU mask)"));
    if (ws_bytes < owt_fc_workspace_bytes(d, OWT_PASS_BWD_DATA))
        return fail(OWT_EWORKSPACE, "workspace too small: need %zu bytes, got %zu",
                    owt_fc_workspace_bytes(d, OWT_PASS_BWD_DATA), ws_bytes);
    const void *mask = (d->flags & OWT_RELU) ? y_or_null : nullptr;
    if (dx_partial_or_null) {
        GemmParams p; memset(&p, 0, sizeof(p));
        p.a = dy; p.b = w; p.out = dx_partial_or_null; p.flags = d->flags; p.mask = mask;
        OWT_TRY(conv_pass(g, OWT_PASS_BWD_DATA, d->dtype, p, false, ws, ws_bytes, (hipStream_t)hip_stream));
    }
    GemmParams p; memset(&p, 0, sizeof(p));
    p.a = dy; p.b = x; p.out = dw; p.flags = d->flags; p.alpha = alpha; p.beta = beta;
    p.dbias = dbias_or_null; p.mask = mask;
    return conv_pass(g, OWT_PASS_BWD_FILTER, d->dtype, p, true, ws, ws_bytes, (hipStream_t)hip_stream);
}

}  // extern "C"
