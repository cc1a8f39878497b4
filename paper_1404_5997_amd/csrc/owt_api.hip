// C ABI entry points of libowt: descriptor checks, launch planning, tuning, launches.
#include <algorithm>
#include <array>
#include <atomic>
#include <map>
#include <mutex>
#include <vector>

#include "owt_host.hpp"
#include "sconv.hpp"
#include "sconv_bf16.hpp"
#include "sfilter.hpp"
#include "sfilter_bf16.hpp"

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

const TileInfo kTiles[NUM_TILES + 5] = {
    {TILE_128x128, 2, 2, 32, 1.00f, 128},
    {TILE_128x64, 2, 1, 16, 0.90f, 128},
    {TILE_64x128, 1, 2, 16, 0.90f, 64},
    {TILE_64x64, 1, 1, 16, 0.75f, 64},
    {TILE_256x64, 4, 1, 32, 1.00f, 256},
    {TILE_128x64H, 4, 1, 32, 1.00f, 128},
    {TILE_128x128H, 4, 2, 32, 1.00f, 128},
    {TILE_512x64, 4, 1, 32, 1.00f, 512},
    {TILE_256x64P, 4, 1, 32, 1.00f, 256},
};

static inline long cdiv(long a, long b) { return (a + b - 1) / b; }
static inline size_t pad256(size_t n) { return (n + 255) & ~(size_t)255; }

bool fill_geom(Geom &g, int N, int C, int H, int W, int K, int R, int S, int sh, int sw, int ph, int pw)
{
    g.N = N; g.C = C; g.H = H; g.W = W; g.K = K; g.R = R; g.S = S;
    g.sh = sh; g.sw = sw; g.ph = ph; g.pw = pw; g.bf16 = 0; g.masked = 0;
    g.P = (H + 2 * ph - R) / sh + 1;
    g.Q = (W + 2 * pw - S) / sw + 1;
    if (H + 2 * ph - R < 0 || W + 2 * pw - S < 0) return false;
    g.dC.set(C); g.dS.set(S); g.dK.set(K); g.dQ.set(g.Q); g.dPQ.set(g.P * g.Q);
    g.dW.set(W); g.dHW.set(H * W); g.dsh.set(sh); g.dsw.set(sw);
    return true;
}

// ------------------------------------------------------------ launch planning
// A pass can run as the gather kernel (igemm.hpp; any shape) or, for stride-1
// forward / backward-data, as the panel-resident kernel (dconv.hpp).  Every
// (kernel, tile, split) that fits is a candidate; a cost model picks one unless
// owt_conv_autotune has timed them for this descriptor.
enum { KIND_GATHER = 0, KIND_DIRECT = 1, KIND_DFILTER = 2, KIND_SFILTER = 3, KIND_SCONV = 4, KIND_DIRECT16 = 5, KIND_DFILTER16 = 6, KIND_SCONV16 = 7, KIND_SFILTER16 = 8, KIND_FCGEMM = 9, KIND_DFILTER2 = 10, KIND_SCONV2 = 11, KIND_SFILTER2 = 12, KIND_DFILTER16B = 13, KIND_SFILTER16B = 14 };

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

static void dconv_frame(const Geom &g, int pass, GemmParams &p)
{
    if (pass == OWT_PASS_FWD) {
        p.Hi = g.H; p.Wi = g.W; p.Ho = g.P; p.Wo = g.Q; p.pah = g.ph; p.paw = g.pw; p.Cred = g.C;
    } else {
        p.Hi = g.P; p.Wi = g.Q; p.Ho = g.H; p.Wo = g.W; p.pah = g.R - 1 - g.ph; p.paw = g.S - 1 - g.pw; p.Cred = g.K;
    }
    p.dWo.set(p.Wo); p.dHoWo.set(p.Ho * p.Wo);
}

// LDS panel rows the direct kernel needs for BM-row tiles, or -1 when the pass does not qualify.
static long direct_panel_rows(const Geom &g, int pass, const PassDims &dm, long BM = 128)
{
    if (pass == OWT_PASS_BWD_FILTER || g.sh != 1 || g.sw != 1 || g.R * g.S == 1) return -1;
    GemmParams f; memset(&f, 0, sizeof(f));
    dconv_frame(g, pass, f);
    if (f.Ho > f.Hi || f.Wo > f.Wi || f.Cred % 4 || (pass == OWT_PASS_BWD_DATA && dm.Ncols % 4)) return -1;
    auto pin = [&](long m) {
        const long n = m / (f.Ho * f.Wo), rem = m % (f.Ho * f.Wo);
        return n * f.Hi * f.Wi + (rem / f.Wo - f.pah) * f.Wi + (rem % f.Wo - f.paw);
    };
    long need = 0;
    for (long m0 = 0; m0 < dm.M; m0 += BM) {
        const long last = (m0 + BM < dm.M ? m0 + BM : dm.M) - 1;
        const long rows = pin(last) - pin(m0) + (g.R - 1) * f.Wi + g.S;
        if (rows > need) need = rows;
    }
    return need;
}

// Geometry of the bf16-MFMA small-channel strided forward kernel; false when it does not apply (bf16
// storage, window starts and image rows that are multiples of 4 values, K a multiple of 4, the filter
// bank of 64 filters plus one band of rows within 150 KB of LDS).
static bool sconv16_geom(const Geom &g, SConv16Geom &sg)
{
    if (!g.bf16 || (g.sw * g.C) % 4 || (g.W * g.C) % 4 || g.C > 16 || g.K % 4 || (g.sh == 1 && g.sw == 1)) return false;
    sg.SEG = g.S * g.C;
    sg.LPAD = (4 - (g.pw * g.C) % 4) % 4;
    sg.SLOTS = (sg.SEG + sg.LPAD + 7) & ~7;
    sg.OCT = sg.SLOTS / 8;
    sg.NG = ((g.R * sg.OCT + 3) / 4) * 2;          // groups of 16 slots, an even number of them
    sg.KSLOTS = sg.NG * 16;
    sg.WP = sg.KSLOTS + 8;
    const int a = g.pw * g.C + sg.LPAD + g.W * g.C, b = (g.Q - 1) * g.sw * g.C + sg.SLOTS;
    sg.PITCH = ((a > b ? a : b) + 7) & ~7;
    sg.ROWS = (kSConv16TP - 1) * g.sh + g.R;
    // the padded tail of the reduction (up to 3 octets) reads past filter row R-1: those panel rows exist and stay zero
    sg.ZROWS = sg.ROWS + 1 + (3 + sg.OCT - 1) / sg.OCT;
    sg.MPIX = kSConv16TP * g.Q;
    sg.units_per_image = (g.P + kSConv16TP - 1) / kSConv16TP;
    sg.units = g.N * sg.units_per_image;
    sg.BIAS = 64 * sg.WP + 2 * sg.ZROWS * sg.PITCH;
    const size_t lds = ((size_t)sg.BIAS + 128) * 2;                  // filter bank + two bands + 64 fp32 biases
    // the output staging blocks follow when the 160 KB of a CU still hold them
    sg.STAGE = lds + (size_t)kSConv16StageValues * 2 <= 160 * 1024 ? (int)(lds / 2) : 0;
    return sg.OCT >= 2 && sg.MPIX <= 256 && lds <= 150 * 1024 && sg.ROWS < 256 &&
           (long)sg.ROWS * (g.W * g.C / 4) <= (long)(kSConv16NT / 2) * kSConv16PNP;
}

// Tap grouping and panel size of the direct filter-gradient kernel for one variant; false when it
// does not apply (needs stride 1, P == H, Q == W, C and K multiples of 4, R*S or S equal to the variant's tap count, and a
// 32-pixel chunk whose padded-coordinate span fits the variant's LDS panel).
static bool dfilter_fits(const Geom &g, int variant, int &taps, int &groups)
{
    const DFilterVariant &v = kDFilterVariants[variant];
    if (g.sh != 1 || g.sw != 1 || g.P != g.H || g.Q != g.W || g.C % 4 || g.K % 4) return false;
    if (g.R * g.S == v.tmax) { taps = g.R * g.S; groups = 1; }
    else if (g.S == v.tmax) { taps = g.S; groups = g.R; }
    else return false;
    const long Wp = g.W + 2 * g.pw, Hp = g.H + 2 * g.ph, PQ = (long)g.P * g.Q;
    long span = 31 + (31 / g.Q + 1) * (Wp - g.Q);
    if (v.aligned) {        // chunks cut per image: worth it only when the short last chunk wastes little
        if (((PQ + 31) / 32) * 32 * 100 > PQ * 104) return false;
    } else {
        span += (31 / PQ + 1) * (Hp - g.P) * Wp;
    }
    const long rows = span + (groups > 1 ? 0 : g.R - 1) * Wp + g.S;
    return rows <= v.prf && (long)g.N * Hp * Wp < 0x7fffffffL;
}

// The same for the kernel with the in-work-group pixel split (fp32 storage; chunks of 32*WP pixels).
static bool dfilter2_fits(const Geom &g, int variant, int &taps, int &groups)
{
    const DFilter2Variant &v = kDFilter2Variants[variant];
    if (g.bf16 || g.masked || g.sh != 1 || g.sw != 1 || g.P != g.H || g.Q != g.W || g.C % 4 || g.K % 4) return false;
    const long Wp = g.W + 2 * g.pw, Hp = g.H + 2 * g.ph, PQ = (long)g.P * g.Q, last = 32 * v.WP - 1;
    if (v.SW > 0) {
        if (g.S != v.SW || g.R * g.S != v.tmax || Wp != v.WPC) return false;
        taps = v.tmax; groups = 1;
    } else {
        if (g.S != v.tmax) return false;
        taps = g.S; groups = g.R;
    }
    // buffer descriptors hold byte counts in 32 bits, and bit 31 of an offset marks "reads as zero"
    if ((long)g.N * g.H * g.W * g.C * 4 >= 0x7fffffffL || (long)g.N * PQ * g.K * 4 >= 0x7fffffffL) return false;
    // the loaders' two LDS tables have 1024 entries, and a chunk may touch two images at most
    if (Hp * Wp > 1024 || PQ > 1024 || 32 * v.WP > PQ) return false;
    const long span = last + (last / g.Q + 1) * (Wp - g.Q) + (last / PQ + 1) * (Hp - g.P) * Wp;
    const long rows = span + (groups > 1 ? 0 : g.R - 1) * Wp + g.S;
    return rows <= v.prows && (long)g.N * Hp * Wp < 0x7fffffffL;
}

// The same for the bf16-MFMA variant (64-pixel chunks, 16-byte pieces: C and K multiples of 8).
static bool dfilter16_fits(const Geom &g, int variant, int &taps, int &groups)
{
    const DFilter16Variant &v = kDFilter16Variants[variant];
    if (!g.bf16 || g.sh != 1 || g.sw != 1 || g.P != g.H || g.Q != g.W || g.C % 8 || g.K % 8) return false;
    if (g.R * g.S == v.tmax) { taps = g.R * g.S; groups = 1; }
    else if (g.S == v.tmax) { taps = g.S; groups = g.R; }
    else return false;
    const long Wp = g.W + 2 * g.pw, Hp = g.H + 2 * g.ph, PQ = (long)g.P * g.Q, last = kDFilter16BP - 1;
    const long span = last + (last / g.Q + 1) * (Wp - g.Q) + (last / PQ + 1) * (Hp - g.P) * Wp;
    const long rows = span + (groups > 1 ? 0 : g.R - 1) * Wp + g.S;
    return rows <= v.prf && (long)g.N * Hp * Wp < 0x7fffffffL;
}

// The bf16 filter-gradient kernel whose operands stream straight into LDS: as above, plus dz taken as it is, loader
// tables of 1024 entries, chunks that touch at most two images, and 32-bit byte offsets into x.
static bool dfilter16b_fits(const Geom &g, int variant, int &taps, int &groups)
{
    const DFilter16bVariant &v = kDFilter16bVariants[variant];
    if (!g.bf16 || g.masked || g.sh != 1 || g.sw != 1 || g.P != g.H || g.Q != g.W || g.C % 8 || g.K % 8) return false;
    const long Wp = g.W + 2 * g.pw, Hp = g.H + 2 * g.ph, PQ = (long)g.P * g.Q, last = kDFilter16BP - 1;
    if (v.SW > 0) {
        if (g.S != v.SW || g.R * g.S != v.tmax || Wp != v.WPC) return false;
        taps = v.tmax; groups = 1;
    } else {
        if (g.S != v.tmax) return false;
        taps = g.S; groups = g.R;
    }
    if (Hp * Wp > 1024 || PQ > 1024 || kDFilter16BP > PQ) return false;
    if ((size_t)g.N * g.H * g.W * g.C * 2 >= 0x7fffffffull || (size_t)g.N * PQ * g.K * 2 >= 0x7fffffffull) return false;
    const long span = last + (last / g.Q + 1) * (Wp - g.Q) + (Hp - g.P) * Wp;      // 64 pixels, their row ends, one image end
    const long rows = span + (groups > 1 ? 0 : g.R - 1) * Wp + g.S;
    return rows <= v.prf;
}

// Geometry of the small-channel strided filter-gradient kernel; false when it does not apply
// (needs window starts and image rows that are multiples of 4 floats, at most 16 blocks of 32
// slots (four accumulators per wavefront in each of four column groups), at most 150 KB of LDS).
static bool sfilter_geom(const Geom &g, SFilterGeom &sg)
{
    if ((g.sw * g.C) % 4 || (g.W * g.C) % 4 || g.K % 4) return false;
    sg.SEG = g.S * g.C;
    sg.LPAD = (4 - (g.pw * g.C) % 4) % 4;
    sg.SLOTS = (sg.SEG + sg.LPAD + 3) & ~3;
    const int a = g.pw * g.C + sg.LPAD + g.W * g.C, b = (g.Q - 1) * g.sw * g.C + sg.SLOTS;
    sg.PITCH = ((a > b ? a : b) + 3) & ~3;
    sg.ROWS = g.sh + g.R;                         // two output rows
    sg.NB = (g.R * sg.SEG + 31) / 32;             // blocks of 32 densely packed (r, s, c) slots
    sg.DZP = (2 * g.Q + 1) & ~1;
    sg.units_per_image = (g.P + 1) / 2;
    sg.units = g.N * sg.units_per_image;
    const size_t lds = ((size_t)sg.ROWS * sg.PITCH + (size_t)sg.DZP * 68) * 4 + (size_t)sg.DZP * 4;
    return sg.NB <= 4 * kSFilterACCS && lds <= 150 * 1024 && g.C <= 16 &&
           sg.ROWS < 256 && g.Q < 65536 &&
           (long)sg.ROWS * (g.W * g.C / 4) <= (long)kSFilterNT * kSFilterPNP && (long)sg.DZP * 16 <= (long)kSFilterNT * kSFilterDNP;
}

// Geometry of the bf16-MFMA small-channel strided filter-gradient kernel; false when it does not apply
// (bf16 storage, K a multiple of 8, window starts and image rows that are multiples of 4 values, at
// most 16 blocks of 32 columns, one band of rows + its dz values within 150 KB of LDS).
static bool sfilter16_geom(const Geom &g, SFilter16Geom &sg)
{
    if (!g.bf16 || (g.sw * g.C) % 4 || (g.W * g.C) % 4 || g.K % 8 || g.C > 16) return false;
    sg.SEG = g.S * g.C;
    sg.LPAD = (4 - (g.pw * g.C) % 4) % 4;
    sg.SLOTS = (sg.SEG + sg.LPAD + 3) & ~3;
    const int a = g.pw * g.C + sg.LPAD + g.W * g.C, b = (g.Q - 1) * g.sw * g.C + sg.SLOTS;
    sg.PITCH = ((a > b ? a : b) + 3) & ~3;
    sg.ROWS = (kSFilter16TP - 1) * g.sh + g.R;
    sg.NB = (g.R * sg.SLOTS + 31) / 32;
    sg.MPIX = kSFilter16TP * g.Q;
    sg.NGP = ((sg.MPIX + 31) / 32) * 2;            // groups of 16 pixels, an even number of them
    sg.DZP = sg.NGP * 16;
    sg.units_per_image = (g.P + kSFilter16TP - 1) / kSFilter16TP;
    sg.units = g.N * sg.units_per_image;
    const size_t lds = ((size_t)sg.ROWS * sg.PITCH + (size_t)sg.DZP * 80) * 2 + (size_t)sg.DZP * 4;
    return sg.NB <= (kSFilter16NT / 64) * kSFilter16CB && lds <= 150 * 1024 && sg.ROWS < 256 &&
           (long)sg.ROWS * (g.W * g.C / 4) <= (long)kSFilter16NT * kSFilter16PNP &&
           sg.DZP <= (kSFilter16NT / 8) * kSFilter16DNP;
}

// The bf16 first-layer filter-gradient kernel whose units stream straight into two LDS stages: dz taken as it is,
// 16-byte aligned row data in the panel, both stages within LDS, the loaders' instruction counts, 32-bit byte
// offsets inside one image.
static bool sfilter16b_fits(const Geom &g, const SFilter16Geom &sg)
{
    const long pp8 = ((sg.PITCH + 7) & ~7) / 8, pan_inst = ((long)sg.ROWS * pp8 + 63) / 64, dz_inst = sg.DZP / 8;
    const size_t lds = (size_t)2 * (pan_inst + dz_inst) * 1024 + (size_t)sg.DZP * 4;
    return !g.masked && (g.pw * g.C + sg.LPAD) % 8 == 0 && (g.W * g.C) % 8 == 0 && pan_inst <= 8 * kSFilter16bPNI &&
           dz_inst <= 8 * kSFilter16bDNI && lds <= 158 * 1024 && (size_t)g.H * g.W * g.C * 2 < 0x40000000ull &&
           (size_t)g.P * g.Q * g.K * 2 < 0x40000000ull;
}

// Geometry of the small-channel strided forward kernel; false when it does not apply.
static bool sconv_geom(const Geom &g, SConvGeom &sg)
{
    if ((g.sw * g.C) % 4 || (g.W * g.C) % 4 || g.C > 16 || (g.sh == 1 && g.sw == 1)) return false;
    sg.SEG = g.S * g.C;
    sg.LPAD = (4 - (g.pw * g.C) % 4) % 4;
    sg.SLOTS = (sg.SEG + sg.LPAD + 3) & ~3;
    const int a = g.pw * g.C + sg.LPAD + g.W * g.C, b = (g.Q - 1) * g.sw * g.C + sg.SLOTS;
    sg.PITCH = ((a > b ? a : b) + 3) & ~3;
    // output rows that kSConvBand consecutive pixels can touch, and the input rows under them
    int orows = (g.Q + kSConvBand - 2) / g.Q + 1;
    if (orows > g.P) orows = g.P;
    sg.ROWS = (orows - 1) * g.sh + g.R;
    sg.KSTEPS = (g.R * sg.SLOTS + kSConvBK - 1) / kSConvBK;
    sg.KSLOTS = sg.KSTEPS * kSConvBK;
    sg.MPIX = kSConvBand;
    sg.units_per_image = (g.P * g.Q + kSConvBand - 1) / kSConvBand;
    sg.units = g.N * sg.units_per_image;
    // the padded tail of the reduction runs past filter row R-1: those panel rows exist and stay zero
    const int zr = (orows - 1) * g.sh + (sg.KSLOTS - 1) / sg.SLOTS + 1;
    sg.ZROWS = zr > sg.ROWS + 1 ? zr : sg.ROWS + 1;
    const size_t lds = ((size_t)2 * 64 * (kSConvBK + 4) + (size_t)sg.ZROWS * sg.PITCH) * 4;
    return sg.MPIX <= 256 && lds <= 150 * 1024 && sg.ROWS < 256 && sg.SLOTS >= 8 && sg.KSLOTS <= 2048 &&
           (long)sg.ROWS * (g.W * g.C / 4) <= (long)kSConvNT * kSConvPNP;
}

// The first-layer forward kernel that keeps 32 filters' whole bank in LDS beside the band: fp32 storage, LDS
// capacity, and 32-bit byte offsets into x and y for its buffer descriptors.
static bool sconv2_fits(const Geom &g, const SConvGeom &sg)
{
    const size_t lds = ((size_t)kSConv2KB * (sg.KSLOTS + 4) + (size_t)sg.ZROWS * sg.PITCH) * 4;
    const size_t xb = (size_t)g.N * g.H * g.W * g.C * 4, yb = (size_t)g.N * g.P * g.Q * g.K * 4;
    return lds <= 157 * 1024 && xb < 0x7fffffffull && yb < 0x7fffffffull && sg.KSTEPS * (kSConvBK / 4) <= 512;
}

// The first-layer filter-gradient kernel whose units stream straight into two LDS stages: fp32 storage, dz taken
// as it is, both stages within LDS, the loaders' instruction counts, 32-bit byte offsets inside one image.
static bool sfilter2_fits(const Geom &g, const SFilterGeom &sg)
{
    const long pan_inst = ((long)sg.ROWS * (sg.PITCH / 4) + 63) / 64, dz_inst = ((long)sg.DZP * 17 + 63) / 64;
    const size_t lds = (size_t)2 * (pan_inst + dz_inst) * 1024 + (size_t)sg.DZP * 4;
    return !g.bf16 && !g.masked && pan_inst <= 8 * kSFilter2PNI && dz_inst <= 8 * kSFilter2DNI && lds <= 158 * 1024 &&
           (size_t)g.H * g.W * g.C * 4 < 0x40000000ull && (size_t)g.P * g.Q * g.K * 4 < 0x40000000ull;
}

struct Launch {
    int kind, tile, splits, steps, steps_per_split, tiles_m, tiles_n, pr, taps, groups, ctiles;
    size_t partial_bytes, dbias_bytes;
    size_t pre_bytes;   // workspace in front of the partials (re-laid-out filters of the bf16 backward-data kernel)
    double cost;   // model estimate, ~clocks
    size_t ws_bytes() const { return pre_bytes + partial_bytes + dbias_bytes; }
};

// Model: the launch's MACs spread over 256 CUs at the tile's relative efficiency, derated when fewer
// than two wavefronts per SIMD are resident (nothing hides load latency then) and by the unevenness
// of the last round of work-groups; a split adds a write+read of the partials and a launch.
static double model_cost(long wgs, int waves_per_wg, int occ, double macs_per_wg, double eff, long splits,
                         long M, long Ncols)
{
    const double per_cu = (double)wgs / 256.0;
    const double resident = (per_cu < occ ? per_cu : occ) * waves_per_wg / 4.0;
    const double lat = resident >= 2.0 ? 1.0 : (resident >= 1.0 ? 0.62 + 0.38 * (resident - 1.0) : 0.62 * resident);
    const double rounds = (double)wgs / (256.0 * occ);
    const double tail = rounds > 1.0 ? 0.5 + 0.5 * rounds / (double)cdiv(wgs, 256L * occ) : 1.0;
    double cost = (double)wgs * macs_per_wg / 256.0 / (128.0 * eff * lat * tail);
    if (splits > 1) cost += 14000.0 + (double)(splits + 1) * M * Ncols * 4.0 / 1300.0;
    return cost;
}

static const size_t kMaxPartialBytes = (size_t)192 << 20;

// What owt_test_force_variant asked for (tests only; -1 / 0 = the planner decides).
static std::atomic<int> g_force_tile{-1}, g_force_split{-1};
static std::atomic<unsigned> g_force_flags{0};
static inline bool forced(unsigned bit) { return (g_force_flags.load(std::memory_order_relaxed) & bit) != 0; }

static void enumerate(const Geom &g, int pass, const PassDims &dm, bool want_db, std::vector<Launch> &out)
{
    const int force_tile = g_force_tile.load(std::memory_order_relaxed);
    const int force_split = g_force_split.load(std::memory_order_relaxed);
    const bool no_direct = forced(OWT_FORCE_NO_DIRECT);
    const bool vec = dm.va && dm.vb;

    auto add = [&](int kind, int tile, int pr, long steps, long s, double macs_per_step_wg, int occ, double eff) {
        if (force_split > 0) s = force_split < steps ? force_split : steps;
        const long per = cdiv(steps, s), splits = cdiv(steps, per);     // drops empty trailing splits
        const TileInfo &ti = kTiles[tile];
        const long tm = cdiv(dm.M, ti.BM), tn = cdiv(dm.Ncols, 64 * ti.WN);
        Launch l; memset(&l, 0, sizeof(l));
        l.kind = kind; l.tile = tile; l.pr = pr; l.splits = (int)splits; l.steps = (int)steps;
        l.steps_per_split = (int)per; l.tiles_m = (int)tm; l.tiles_n = (int)tn;
        if (splits > 1) {
            l.partial_bytes = pad256((size_t)splits * dm.M * dm.Ncols * 4);
            l.dbias_bytes = want_db ? pad256((size_t)splits * dm.M * 4) : 0;
            if (l.partial_bytes > kMaxPartialBytes && force_split <= 0) return;
        }
        l.cost = model_cost(tm * tn * splits, ti.WM * ti.WN, occ, macs_per_step_wg * per, eff, splits, dm.M, dm.Ncols);
        for (const Launch &o : out)
            if (o.kind == l.kind && o.tile == l.tile && o.splits == l.splits) return;
        out.push_back(l);
    };

    static const long kSplits[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128, 192, 256};
    // split counts to try for `tiles` output tiles: the fixed ladder plus the counts that fill one, two
    // or three rounds of the chip's work-group slots exactly (256 CUs x 2 resident work-groups)
    auto split_ladder = [&](long tiles, long slots = 512) {
        std::vector<long> v(kSplits, kSplits + sizeof(kSplits) / sizeof(kSplits[0]));
        for (long rounds = 1; rounds <= 3; rounds++)
            if (slots * rounds / tiles >= 1) v.push_back(slots * rounds / tiles);
        std::sort(v.begin(), v.end());
        v.erase(std::unique(v.begin(), v.end()), v.end());
        return v;
    };
    const long cred = pass == OWT_PASS_FWD ? g.C : g.K;
    for (int t : {TILE_128x128, TILE_128x64, TILE_256x64, TILE_128x64H, TILE_128x128H}) {
        if (no_direct || (force_tile >= 0 && force_tile != t)) continue;
        const long BM = kTiles[t].BM, rows = direct_panel_rows(g, pass, dm, BM);
        int pr;                                        // panel sizes the kernel is instantiated for
        if (t == TILE_256x64) { if (rows < 0 || rows > 384) continue; pr = rows <= 288 ? 288 : 384; }
        else { if (rows < 0 || rows > 256) continue; pr = rows <= 160 ? 160 : ((t == TILE_128x64H && rows <= 244) ? 244 : 256); }
        const long bk = t == TILE_128x64 ? 16 : 32, chunks = cdiv(cred, bk);
        const double macs = (double)BM * 64 * kTiles[t].WN * bk * g.R * g.S;
        for (long s : kSplits) {
            if (s > 1 && (chunks / s < 2 || s > 8)) break;
            add(KIND_DIRECT, t, pr, chunks, s, macs, t == TILE_128x64 ? 5 : (t == TILE_128x64H ? 3 : 2),
                t == TILE_128x64 ? 1.1 : 1.25);
            if (force_split > 0) break;
        }
    }
    if (g.bf16 && cred % 8 == 0 && !forced(OWT_FORCE_NO_BF16_MFMA)) {      // the bf16 MFMA: 64-channel chunks, or 32 in the 512x64 tile
        for (int t : {TILE_128x128, TILE_128x64, TILE_256x64, TILE_512x64, TILE_256x64P}) {
            if (no_direct || (force_tile >= 0 && force_tile != t)) continue;
            const long BM = kTiles[t].BM, rows = direct_panel_rows(g, pass, dm, BM);
            int pr;
            const bool pipelined = t == TILE_512x64 || t == TILE_256x64P;
            if (pipelined && (dm.Ncols % 4 || cred % 32 || g.R * g.S > 32)) continue;
            if (t == TILE_512x64) { if (rows < 0 || rows > 624) continue; pr = rows <= 544 ? 544 : 624; }
            else if (t == TILE_256x64 || t == TILE_256x64P) { if (rows < 0 || rows > 384) continue; pr = rows <= 288 ? 288 : 384; }
            else { if (rows < 0 || rows > 256) continue; pr = rows <= 160 ? 160 : 256; }
            const long bk = pipelined ? 32 : 64, chunks = cdiv(cred, bk);
            // ~6x the fp32 MFMA rate; the pipelined tile keeps the matrix unit about 1.5x busier
            const double macs = (double)BM * 64 * kTiles[t].WN * bk * g.R * g.S / (pipelined ? 9.0 : 6.0);
            const size_t n0 = out.size();
            for (long s : kSplits) {
                if (s > 1 && (chunks / s < 1 || s > 8 || s > chunks)) break;
                add(KIND_DIRECT16, t, pr, chunks, s, macs, t == TILE_256x64P ? 3 : 2, 1.25);
                if (force_split > 0) break;
            }
            if (pass == OWT_PASS_BWD_DATA)
                for (size_t i = n0; i < out.size(); i++) out[i].pre_bytes = pad256((size_t)g.K * g.R * g.S * g.C * 2);
        }
    }
    SConvGeom scg;
    // test hook: tile 20 = only the filter-streaming first-layer forward kernel, 21 = only the filters-in-LDS one
    const bool sconv_ok = pass == OWT_PASS_FWD && !no_direct && sconv_geom(g, scg);
    if (sconv_ok && force_tile != 20 && !g.bf16 && sconv2_fits(g, scg)) {
        const long ktiles = cdiv(g.K, kSConv2KB);
        for (long target : {256L, 512L}) {
            long wgs = target / ktiles > 0 ? target / ktiles : 1;
            if (force_split > 0) wgs = force_split;
            if (wgs > scg.units) wgs = scg.units;
            const long per = cdiv(scg.units, wgs), n = cdiv(scg.units, per);
            Launch l; memset(&l, 0, sizeof(l));
            l.kind = KIND_SCONV2; l.splits = 1; l.steps = scg.units; l.steps_per_split = (int)per;
            l.tiles_m = (int)ktiles; l.tiles_n = (int)n;
            l.partial_bytes = pad256((size_t)g.K * scg.KSLOTS * 4);          // the re-laid-out filters
            l.cost = model_cost(ktiles * n, 8, 1, 256.0 * kSConv2KB * scg.KSLOTS * per, 1.2, 1, dm.M, dm.Ncols);
            bool dup = false;
            for (const Launch &o : out) dup |= o.kind == l.kind && o.tiles_n == l.tiles_n;
            if (!dup) out.push_back(l);
            if (force_split > 0) break;
        }
    }
    if (sconv_ok && force_tile != 21) {
        const long ktiles = cdiv(g.K, 64);
        for (long target : {256L, 512L}) {
            long wgs = target / ktiles > 0 ? target / ktiles : 1;
            if (force_split > 0) wgs = force_split;
            if (wgs > scg.units) wgs = scg.units;
            const long per = cdiv(scg.units, wgs), n = cdiv(scg.units, per);
            Launch l; memset(&l, 0, sizeof(l));
            l.kind = KIND_SCONV; l.splits = 1; l.steps = scg.units; l.steps_per_split = (int)per;
            l.tiles_m = (int)ktiles; l.tiles_n = (int)n;
            l.partial_bytes = pad256((size_t)g.K * scg.KSLOTS * 4);          // the re-laid-out filters
            // (bf16 storage: the bf16-MFMA kernel below, when it applies, is the faster one)
            l.cost = model_cost(ktiles * n, 8, 1, 256.0 * 64 * scg.KSLOTS * per, 1.0, 1, dm.M, dm.Ncols) * (g.bf16 ? 2.0 : 1.0);
            bool dup = false;
            for (const Launch &o : out) dup |= o.kind == l.kind && o.tiles_n == l.tiles_n;
            if (!dup) out.push_back(l);
            if (force_split > 0) break;
        }
    }
    SConv16Geom s16g;
    if (pass == OWT_PASS_FWD && !no_direct && !forced(OWT_FORCE_NO_BF16_MFMA) && sconv16_geom(g, s16g)) {
        const long ktiles = cdiv(g.K, 64);
        for (long target : {256L, 512L}) {
            long wgs = target / ktiles > 0 ? target / ktiles : 1;
            if (force_split > 0) wgs = force_split;
            if (wgs > s16g.units) wgs = s16g.units;
            const long per = cdiv(s16g.units, wgs), n = cdiv(s16g.units, per);
            Launch l; memset(&l, 0, sizeof(l));
            l.kind = KIND_SCONV16; l.splits = 1; l.steps = s16g.units; l.steps_per_split = (int)per;
            l.tiles_m = (int)ktiles; l.tiles_n = (int)n;
            l.partial_bytes = pad256((size_t)g.K * s16g.KSLOTS * 2);        // the re-laid-out filters
            l.cost = model_cost(ktiles * n, 4, 1, 256.0 * 64 * s16g.KSLOTS * per / 6.0, 1.0, 1, dm.M, dm.Ncols);
            bool dup = false;
            for (const Launch &o : out) dup |= o.kind == l.kind && o.tiles_n == l.tiles_n;
            if (!dup) out.push_back(l);
            if (force_split > 0) break;
        }
    }
    // test hook: tile 22 = only the register-staged first-layer filter-gradient kernel, 23 = only the one that streams
    // its units straight into LDS
    SFilterGeom sfg;
    const bool sfilter_ok = pass == OWT_PASS_BWD_FILTER && !no_direct && (g.sh > 1 || g.sw > 1) && sfilter_geom(g, sfg);
    for (int form = 0; form < 2 && sfilter_ok; form++) {
        if (form == 0 ? force_tile == 23 : (force_tile == 22 || !sfilter2_fits(g, sfg))) continue;
        const long ktiles = cdiv(g.K, 64);
        for (long target : {256L, 512L, 1024L}) {
            long wgs = target / ktiles > 0 ? target / ktiles : 1;
            if (force_split > 0) wgs = force_split;
            if (wgs > sfg.units) wgs = sfg.units;
            const long per = cdiv(sfg.units, wgs), splits = cdiv(sfg.units, per);
            Launch l; memset(&l, 0, sizeof(l));
            l.kind = form ? KIND_SFILTER2 : KIND_SFILTER; l.tile = 0; l.splits = (int)splits; l.steps = sfg.units; l.steps_per_split = (int)per;
            l.tiles_m = (int)ktiles; l.tiles_n = 1;
            if (splits > 1) {
                l.partial_bytes = pad256((size_t)splits * dm.M * dm.Ncols * 4);
                l.dbias_bytes = want_db ? pad256((size_t)splits * dm.M * 4) : 0;
            }
            l.cost = model_cost(ktiles * splits, 8, form ? 1 : 2, 64.0 * sfg.NB * 32 * sfg.DZP * per, form ? 1.15 : 1.0, splits, dm.M, dm.Ncols);
            bool dup = false;
            for (const Launch &o : out) dup |= o.kind == l.kind && o.splits == l.splits;
            if (!dup) out.push_back(l);
            if (force_split > 0) break;
        }
    }
    // test hook: tile 24 = only the register-staged bf16 first-layer filter-gradient kernel, 25 = only the one that
    // streams its units straight into LDS
    SFilter16Geom sf16g;
    const bool sf16_ok = pass == OWT_PASS_BWD_FILTER && !no_direct && !forced(OWT_FORCE_NO_BF16_MFMA) && (g.sh > 1 || g.sw > 1) &&
                         sfilter16_geom(g, sf16g);
    for (int form = 0; form < 2 && sf16_ok; form++) {
        if (form == 0 ? force_tile == 25 : (force_tile == 24 || !sfilter16b_fits(g, sf16g))) continue;
        const long ktiles = cdiv(g.K, 64);
        for (long target : {256L, 512L, 1024L}) {
            long wgs = target / ktiles > 0 ? target / ktiles : 1;
            if (force_split > 0) wgs = force_split;
            if (wgs > sf16g.units) wgs = sf16g.units;
            const long per = cdiv(sf16g.units, wgs), splits = cdiv(sf16g.units, per);
            Launch l; memset(&l, 0, sizeof(l));
            l.kind = form ? KIND_SFILTER16B : KIND_SFILTER16; l.tile = 0; l.splits = (int)splits; l.steps = sf16g.units; l.steps_per_split = (int)per;
            l.tiles_m = (int)ktiles; l.tiles_n = 1;
            if (splits > 1) {
                l.partial_bytes = pad256((size_t)splits * dm.M * dm.Ncols * 4);
                l.dbias_bytes = want_db ? pad256((size_t)splits * dm.M * 4) : 0;
            }
            l.cost = model_cost(ktiles * splits, 8, 1, 64.0 * sf16g.NB * 32 * sf16g.DZP * per / 5.0, form ? 1.3 : 1.0, splits, dm.M, dm.Ncols);
            bool dup = false;
            for (const Launch &o : out) dup |= o.kind == l.kind && o.splits == l.splits;
            if (!dup) out.push_back(l);
            if (force_split > 0) break;
        }
    }
    if (pass == OWT_PASS_BWD_FILTER && !no_direct) {
        for (int v = 0; v < kNumDFilterVariants; v++) {
            int taps, groups;
            if (force_tile >= 0 && force_tile != v) continue;
            if (!dfilter_fits(g, v, taps, groups)) continue;
            if (v == 2 && g.K % 128 == 0) continue;                  // variant 0 covers it with the same accumulators
            const DFilterVariant &dv = kDFilterVariants[v];
            const long KT = 32 * dv.WK, CT = 32 * dv.WC;
            const long tm = cdiv(g.K, KT), ctl = cdiv(g.C, CT);
            const long steps = dv.aligned ? (long)g.N * cdiv((long)g.P * g.Q, 32) : cdiv(dm.Kd, 32);
            for (long s0 : split_ladder(tm * ctl * groups, 256 * dv.occ)) {
                long s = s0;
                if (force_split > 0) s = force_split < steps ? force_split : steps;
                else if (s > 1 && (steps / s < 2 || tm * ctl * groups * s > 2560)) break;
                const long per = cdiv(steps, s), splits = cdiv(steps, per);
                Launch l; memset(&l, 0, sizeof(l));
                l.kind = KIND_DFILTER; l.tile = v; l.splits = (int)splits; l.steps = (int)steps;
                l.steps_per_split = (int)per; l.tiles_m = (int)tm; l.tiles_n = (int)(ctl * groups);
                l.taps = taps; l.groups = groups; l.ctiles = (int)ctl;
                if (splits > 1) {
                    l.partial_bytes = pad256((size_t)splits * dm.M * dm.Ncols * 4);
                    l.dbias_bytes = want_db ? pad256((size_t)splits * dm.M * 4) : 0;
                }
                l.cost = model_cost(tm * ctl * groups * splits, dv.WK * dv.WC, dv.occ, (double)KT * CT * 32 * taps * per, 1.2, splits,
                                    dm.M, dm.Ncols);
                bool dup = false;
                for (const Launch &o : out) dup |= o.kind == l.kind && o.tile == l.tile && o.splits == l.splits;
                if (!dup && (l.partial_bytes <= kMaxPartialBytes || force_split > 0) &&
                    (force_split > 0 || tm * ctl * groups * splits >= 128 || s0 == 256)) out.push_back(l);
                if (force_split > 0) break;
            }
        }
    }
    if (pass == OWT_PASS_BWD_FILTER && !no_direct) {
        for (int v = 0; v < kNumDFilter2Variants; v++) {
            int taps, groups;
            if (force_tile >= 0 && force_tile != kDFilter2FirstTile + v) continue;
            if (!dfilter2_fits(g, v, taps, groups)) continue;
            const DFilter2Variant &dv = kDFilter2Variants[v];
            const long KT = 32 * dv.WK, CT = 32, BP = 32 * dv.WP;
            const long tm = cdiv(g.K, KT), ctl = cdiv(g.C, CT), steps = cdiv(dm.Kd, BP);
            for (long s0 : split_ladder(tm * ctl * groups, 256)) {
                long s = s0;
                if (force_split > 0) s = force_split < steps ? force_split : steps;
                else if (s > 1 && (steps / s < 2 || tm * ctl * groups * s > 1280)) break;
                const long per = cdiv(steps, s), splits = cdiv(steps, per);
                Launch l; memset(&l, 0, sizeof(l));
                l.kind = KIND_DFILTER2; l.tile = v; l.splits = (int)splits; l.steps = (int)steps;
                l.steps_per_split = (int)per; l.tiles_m = (int)tm; l.tiles_n = (int)(ctl * groups);
                l.taps = taps; l.groups = groups; l.ctiles = (int)ctl;
                if (splits > 1) {
                    l.partial_bytes = pad256((size_t)splits * dm.M * dm.Ncols * 4);
                    l.dbias_bytes = want_db ? pad256((size_t)splits * dm.M * 4) : 0;
                }
                l.cost = model_cost(tm * ctl * groups * splits, dv.WK * dv.WP, 1, (double)KT * CT * BP * taps * per, 1.3, splits,
                                    dm.M, dm.Ncols);
                bool dup = false;
                for (const Launch &o : out) dup |= o.kind == l.kind && o.tile == l.tile && o.splits == l.splits;
                if (!dup && (l.partial_bytes <= kMaxPartialBytes || force_split > 0) &&
                    (force_split > 0 || tm * ctl * groups * splits >= 64 || s0 == 256)) out.push_back(l);
                if (force_split > 0) break;
            }
        }
    }
    if (pass == OWT_PASS_BWD_FILTER && !no_direct && !forced(OWT_FORCE_NO_BF16_MFMA)) {
        for (int v = 0; v < kNumDFilter16bVariants; v++) {
            int taps, groups;
            if (force_tile >= 0 && force_tile != kDFilter16bFirstTile + v) continue;
            if (!dfilter16b_fits(g, v, taps, groups)) continue;
            const DFilter16bVariant &dv = kDFilter16bVariants[v];
            const long KT = 32 * dv.KB * dv.WK, CT = 32 * dv.WC;
            const long tm = cdiv(g.K, KT), ctl = cdiv(g.C, CT), steps = cdiv(dm.Kd, kDFilter16BP);
            for (long s0 : split_ladder(tm * ctl * groups, 256)) {
                long s = s0;
                if (force_split > 0) s = force_split < steps ? force_split : steps;
                else if (s > 1 && (steps / s < 2 || tm * ctl * groups * s > 1280)) break;
                const long per = cdiv(steps, s), splits = cdiv(steps, per);
                if (per > kDFilter16bMaxChunks) { if (force_split > 0) break; continue; }
                Launch l; memset(&l, 0, sizeof(l));
                l.kind = KIND_DFILTER16B; l.tile = v; l.splits = (int)splits; l.steps = (int)steps;
                l.steps_per_split = (int)per; l.tiles_m = (int)tm; l.tiles_n = (int)(ctl * groups);
                l.taps = taps; l.groups = groups; l.ctiles = (int)ctl;
                if (splits > 1) {
                    l.partial_bytes = pad256((size_t)splits * dm.M * dm.Ncols * 4);
                    l.dbias_bytes = want_db ? pad256((size_t)splits * dm.M * 4) : 0;
                }
                l.cost = model_cost(tm * ctl * groups * splits, dv.WK * dv.WC, 1,
                                    (double)KT * CT * kDFilter16BP * taps * per / 5.0, 1.5, splits, dm.M, dm.Ncols);
                bool dup = false;
                for (const Launch &o : out) dup |= o.kind == l.kind && o.tile == l.tile && o.splits == l.splits;
                if (!dup && (l.partial_bytes <= kMaxPartialBytes || force_split > 0) &&
                    (force_split > 0 || tm * ctl * groups * splits >= 64 || s0 == 256)) out.push_back(l);
                if (force_split > 0) break;
            }
        }
        for (int v = 0; v < kNumDFilter16Variants; v++) {
            int taps, groups;
            if (force_tile >= 0 && force_tile != v) continue;
            if (!dfilter16_fits(g, v, taps, groups)) continue;
            const DFilter16Variant &dv = kDFilter16Variants[v];
            const long KT = 32 * dv.KB * dv.WK, CT = 32 * dv.WC;
            const long tm = cdiv(g.K, KT), ctl = cdiv(g.C, CT), steps = cdiv(dm.Kd, kDFilter16BP);
            for (long s0 : split_ladder(tm * ctl * groups, 256)) {            // one or two work-groups per CU
                long s = s0;
                if (force_split > 0) s = force_split < steps ? force_split : steps;
                else if (s > 1 && (steps / s < 2 || tm * ctl * groups * s > 1280)) break;
                const long per = cdiv(steps, s), splits = cdiv(steps, per);
                Launch l; memset(&l, 0, sizeof(l));
                l.kind = KIND_DFILTER16; l.tile = v; l.splits = (int)splits; l.steps = (int)steps;
                l.steps_per_split = (int)per; l.tiles_m = (int)tm; l.tiles_n = (int)(ctl * groups);
                l.taps = taps; l.groups = groups; l.ctiles = (int)ctl;
                if (splits > 1) {
                    l.partial_bytes = pad256((size_t)splits * dm.M * dm.Ncols * 4);
                    l.dbias_bytes = want_db ? pad256((size_t)splits * dm.M * 4) : 0;
                }
                l.cost = model_cost(tm * ctl * groups * splits, dv.WK * dv.WC, dv.occ,
                                    (double)KT * CT * kDFilter16BP * taps * per / 5.0, 1.2,
                                    splits, dm.M, dm.Ncols);
                bool dup = false;
                for (const Launch &o : out) dup |= o.kind == l.kind && o.tile == l.tile && o.splits == l.splits;
                if (!dup && (l.partial_bytes <= kMaxPartialBytes || force_split > 0) &&
                    (force_split > 0 || tm * ctl * groups * splits >= 64 || s0 == 256)) out.push_back(l);
                if (force_split > 0) break;
            }
        }
    }
    // plain matrix product (the fully-connected shard), fp32 storage: the dense kernel with operands streamed
    // straight into LDS; needs 16-byte aligned operand rows and, in the forward pass, whole 32-deep
    // reduction steps (the backward passes can read a zero-padded copy of dz instead)
    if (!no_direct && !g.bf16 && g.H == 1 && g.W == 1 && g.R == 1 && g.S == 1 &&
        (pass == OWT_PASS_FWD ? dm.Kd % 32 == 0 : dm.Ncols % 4 == 0)) {
        for (int t = 0; t < kNumFcTiles; t++) {
            if (force_tile >= 0 && force_tile != 16 + t) continue;
            const FcTile &ft = kFcTiles[t];
            const long BM = 32 * ft.MB * ft.WM, BN = 32 * ft.NB * ft.WN;
            const long steps = cdiv(dm.Kd, 32), tm = cdiv(dm.M, BM), tn = cdiv(dm.Ncols, BN);
            for (long s0 : split_ladder(tm * tn, 256 * ft.occ)) {
                long s = s0;
                if (force_split > 0) s = force_split < steps ? force_split : steps;
                if (force_split <= 0 && s > 1 && (steps / s < 2 || tm * tn * s > 2048)) break;
                const long per = cdiv(steps, s), splits = cdiv(steps, per);
                Launch l; memset(&l, 0, sizeof(l));
                l.kind = KIND_FCGEMM; l.tile = t; l.splits = (int)splits; l.steps = (int)steps; l.steps_per_split = (int)per;
                l.tiles_m = (int)tm; l.tiles_n = (int)tn;
                if (splits > 1) l.partial_bytes = pad256((size_t)splits * dm.M * dm.Ncols * 4);
                if (pass != OWT_PASS_FWD) l.pre_bytes = pad256((size_t)((g.N + 31) & ~31) * ((g.K + 31) & ~31) * 4);     // padded dz
                l.cost = model_cost(tm * tn * splits, 4, ft.occ, (double)BM * BN * 32 * per, 1.6, splits, dm.M, dm.Ncols);
                bool dup = l.partial_bytes > kMaxPartialBytes && force_split <= 0;
                for (const Launch &o : out) dup |= o.kind == l.kind && o.tile == l.tile && o.splits == l.splits;
                if (!dup) out.push_back(l);
                if (force_split > 0) break;
            }
        }
    }
    // the gather kernel is the fallback of the stride-1 forward / backward-data kernel, and an
    // alternative worth timing next to the direct filter-gradient kernel
    const bool have_direct = !out.empty() && (out[0].kind == KIND_DIRECT || out[0].kind == KIND_DIRECT16);
    for (int t = 0; t < NUM_TILES && !have_direct; t++) {
        if (!vec && t != TILE_64x64) continue;
        if (force_tile >= kDFilter2FirstTile && !out.empty()) continue;
        if (vec && force_tile >= 0 && force_tile < NUM_TILES && t != force_tile) continue;
        const TileInfo &ti = kTiles[t];
        const long ksteps = cdiv(dm.Kd, ti.BK);
        const long tiles = cdiv(dm.M, ti.BM) * cdiv(dm.Ncols, 64 * ti.WN);
        const double macs = (double)ti.BM * 64 * ti.WN * ti.BK;
        for (long s : split_ladder(tiles)) {
            if (s > 1 && (ksteps / s < 4 || tiles * s > 4096)) break;
            add(KIND_GATHER, t, 0, ksteps, s, macs, t == TILE_128x128 ? 2 : 5, ti.eff);
            if (force_split > 0) break;
        }
    }
}

typedef std::array<int, 15> PlanKey;
static std::map<PlanKey, Launch> g_tuned;
static std::mutex g_tuned_mutex;

static PlanKey plan_key(const Geom &g, int pass, owt_dtype dt)
{
    return PlanKey{g.N, g.C, g.H, g.W, g.K, g.R, g.S, g.sh, g.sw, g.ph, g.pw, pass, (int)dt, g.masked, 0};
}

static bool variants_forced()
{
    return g_force_tile.load(std::memory_order_relaxed) >= 0 || g_force_split.load(std::memory_order_relaxed) > 0 ||
           g_force_flags.load(std::memory_order_relaxed) != 0;
}

static std::map<PlanKey, Launch> g_modelled;   // the cost model's choice per geometry (untimed), so that a call plans once

static Launch choose(const Geom &g, int pass, owt_dtype dt, const PassDims &dm, bool want_db, bool use_cache)
{
    const bool cached = use_cache && !variants_forced();
    if (cached) {
        std::lock_guard<std::mutex> lk(g_tuned_mutex);
        auto it = g_tuned.find(plan_key(g, pass, dt));
        if (it != g_tuned.end()) return it->second;
        it = g_modelled.find(plan_key(g, pass, dt));
        if (it != g_modelled.end()) return it->second;
    }
    std::vector<Launch> c;
    enumerate(g, pass, dm, want_db, c);
    bool only_direct = forced(OWT_FORCE_ONLY_DIRECT), any_direct = false;   // test hook
    for (const Launch &l : c) any_direct |= l.kind != KIND_GATHER;
    size_t best = c.size();
    for (size_t i = 0; i < c.size(); i++) {
        if (only_direct && any_direct && c[i].kind == KIND_GATHER) continue;
        if (best == c.size() || c[i].cost < c[best].cost) best = i;
    }
    if (cached) {
        std::lock_guard<std::mutex> lk(g_tuned_mutex);
        g_modelled[plan_key(g, pass, dt)] = c[best];
    }
    return c[best];
}

// Workspace every candidate fits in (so a tuned choice never outgrows the caller's buffer).
static size_t max_workspace(const Geom &g, int pass, const PassDims &dm, bool want_db)
{
    // with and without the ReLU' mask flag: a caller may size its buffer with one descriptor of a layer and call
    // with the other (the kernels that take dz as it is are only candidates for the unmasked one)
    size_t m = 0;
    for (int masked = 0; masked < 2; masked++) {
        Geom gm = g;
        gm.masked = masked != 0;
        std::vector<Launch> c;
        enumerate(gm, pass, dm, want_db, c);
        for (const Launch &l : c) m = l.ws_bytes() > m ? l.ws_bytes() : m;
    }
    return m;
}

// The part of the kernel parameters that the chosen launch decides.
static void frame_params(const Geom &g, const PassDims &dm, const Launch &l, void *ws, GemmParams &p)
{
    p.g = g; p.M = (int)dm.M; p.Ncols = (int)dm.Ncols; p.Kd = (int)dm.Kd;
    p.splits = l.splits; p.ksteps = l.steps; p.ksteps_per_split = l.steps_per_split;
    p.tiles_m = l.tiles_m; p.tiles_n = l.tiles_n;
    p.partial = l.splits > 1 ? (float *)((char *)ws + l.pre_bytes) : nullptr;
    p.dbias_partial = (l.splits > 1 && l.dbias_bytes) ? (float *)((char *)ws + l.pre_bytes + l.partial_bytes) : nullptr;
}

static owt_status launch(const Geom &g, int pass, owt_dtype dt, const PassDims &dm, GemmParams p, const Launch &l,
                         void *ws, hipStream_t s)
{
    frame_params(g, dm, l, ws, p);
    const bool bf = dt == OWT_BF16;
    hipError_t e;
    if (l.kind == KIND_FCGEMM) {
        e = owt_launch_fcgemm(pass, l.tile, p, (float *)ws, s);
    } else if (l.kind == KIND_DIRECT16) {
        dconv_frame(g, pass, p);
        e = pass == OWT_PASS_FWD ? owt_launch_dconv16_fwd(l.tile, l.pr, p, s) : owt_launch_dconv16_data(l.tile, l.pr, p, ws, s);
    } else if (l.kind == KIND_SCONV16) {
        SConv16Geom sg;
        sconv16_geom(g, sg);
        sg.units_per_wg = l.steps_per_split;
        p.splits = 1; p.partial = nullptr;
        e = owt_launch_sconv16(p, sg, l.tiles_m, l.tiles_n, ws, s);
    } else if (l.kind == KIND_SCONV2) {
        SConvGeom sg;
        sconv_geom(g, sg);
        sg.units_per_wg = l.steps_per_split;
        p.splits = 1; p.partial = nullptr;
        e = owt_launch_sconv2_f32(p, sg, l.tiles_m, l.tiles_n, (float *)ws, s);
    } else if (l.kind == KIND_SCONV) {
        SConvGeom sg;
        sconv_geom(g, sg);
        sg.units_per_wg = l.steps_per_split;
        p.splits = 1; p.partial = nullptr;
        e = bf ? owt_launch_sconv_bf16(p, sg, l.tiles_m, l.tiles_n, (float *)ws, s)
               : owt_launch_sconv_f32(p, sg, l.tiles_m, l.tiles_n, (float *)ws, s);
    } else if (l.kind == KIND_SFILTER16B) {
        SFilter16Geom sg;
        sfilter16_geom(g, sg);
        sg.units_per_wg = l.steps_per_split;
        e = owt_launch_sfilter16b(p, sg, l.tiles_m, s);
    } else if (l.kind == KIND_SFILTER16) {
        SFilter16Geom sg;
        sfilter16_geom(g, sg);
        sg.units_per_wg = l.steps_per_split;
        e = owt_launch_sfilter16(p, sg, l.tiles_m, s);
    } else if (l.kind == KIND_SFILTER2) {
        SFilterGeom sg;
        sfilter_geom(g, sg);
        sg.units_per_wg = l.steps_per_split;
        e = owt_launch_sfilter2_f32(p, sg, l.tiles_m, s);
    } else if (l.kind == KIND_SFILTER) {
        SFilterGeom sg;
        sfilter_geom(g, sg);
        sg.units_per_wg = l.steps_per_split;
        e = bf ? owt_launch_sfilter_bf16(p, sg, l.tiles_m, s) : owt_launch_sfilter_f32(p, sg, l.tiles_m, s);
    } else if (l.kind == KIND_DFILTER16B) {
        p.Hp = g.H + 2 * g.ph; p.Wp = g.W + 2 * g.pw; p.taps = l.taps; p.groups = l.groups; p.ctiles = l.ctiles;
        p.dWp.set(p.Wp); p.dHpWp.set(p.Hp * p.Wp);
        e = owt_launch_dfilter16b(l.tile, p, s);
    } else if (l.kind == KIND_DFILTER16) {
        p.Hp = g.H + 2 * g.ph; p.Wp = g.W + 2 * g.pw; p.taps = l.taps; p.groups = l.groups; p.ctiles = l.ctiles;
        p.dWp.set(p.Wp); p.dHpWp.set(p.Hp * p.Wp);
        e = owt_launch_dfilter16(l.tile, p, s);
    } else if (l.kind == KIND_DFILTER2) {
        p.Hp = g.H + 2 * g.ph; p.Wp = g.W + 2 * g.pw; p.taps = l.taps; p.groups = l.groups; p.ctiles = l.ctiles;
        p.dWp.set(p.Wp); p.dHpWp.set(p.Hp * p.Wp);
        e = owt_launch_dfilter2_f32(l.tile, p, s);
    } else if (l.kind == KIND_DFILTER) {
        p.Hp = g.H + 2 * g.ph; p.Wp = g.W + 2 * g.pw; p.taps = l.taps; p.groups = l.groups; p.ctiles = l.ctiles;
        p.dWp.set(p.Wp); p.dHpWp.set(p.Hp * p.Wp);
        if (kDFilterVariants[l.tile].aligned) { p.cpi = (int)cdiv((long)g.P * g.Q, 32); p.dCpi.set(p.cpi); }
        e = bf ? owt_launch_dfilter_bf16(l.tile, p, s) : owt_launch_dfilter_f32(l.tile, p, s);
    } else if (l.kind == KIND_DIRECT) {
        dconv_frame(g, pass, p);
        if (pass == OWT_PASS_FWD) e = bf ? owt_launch_dconv_fwd_bf16(l.tile, l.pr, p, s) : owt_launch_dconv_fwd_f32(l.tile, l.pr, p, s);
        else e = bf ? owt_launch_dconv_data_bf16(l.tile, l.pr, p, s) : owt_launch_dconv_data_f32(l.tile, l.pr, p, s);
    } else {
        static const LaunchFn table[3][2] = {
            {owt_launch_fwd_f32, owt_launch_fwd_bf16},
            {owt_launch_data_f32, owt_launch_data_bf16},
            {owt_launch_filter_f32, owt_launch_filter_bf16},
        };
        e = table[pass][bf ? 1 : 0](l.tile, dm.va ? 4 : 1, dm.vb ? 4 : 1, p, s);
    }
    if (e != hipSuccess) return fail(OWT_ELAUNCH, "HIP launch failed: %s", hipGetErrorString(e));
    return OWT_OK;
}

static int describe(char *buf, size_t n, int pass, owt_dtype dt, const PassDims &dm, const Launch &l)
{
    // "... gridAxB threadsT": A x B work-groups, T = total threads of the main kernel's launch (the
    // figure profilers list as its grid size)
    static const char *pn[3] = {"fwd", "bwd_data", "bwd_filter"};
    const char *ds = dt == OWT_BF16 ? "bf16" : "f32";
    if (l.kind == KIND_FCGEMM) {
        const FcTile &ft = kFcTiles[l.tile];
        return snprintf(buf, n, "fcgemm %s %s tile%dx%dx32 splitk%d grid%dx%d threads%ld", pn[pass], ds, 32 * ft.MB * ft.WM,
                        32 * ft.NB * ft.WN, l.splits, l.tiles_m * l.tiles_n, l.splits,
                        (long)l.tiles_m * l.tiles_n * l.splits * 64 * ft.WM * ft.WN);
    }
    if (l.kind == KIND_SCONV16)
        return snprintf(buf, n, "sconv16 %s %s rows%d grid%dx%d threads%ld", pn[pass], ds, kSConv16TP, l.tiles_m, l.tiles_n,
                        (long)l.tiles_m * l.tiles_n * kSConv16NT);
    if (l.kind == KIND_SCONV2)
        return snprintf(buf, n, "sconv2 %s %s band%d filters%d grid%dx%d threads%ld", pn[pass], ds, kSConvBand, kSConv2KB, l.tiles_m,
                        l.tiles_n, (long)l.tiles_m * ((l.tiles_n + 7) / 8) * 8 * kSConvNT);
    if (l.kind == KIND_SCONV)
        return snprintf(buf, n, "sconv %s %s band%d grid%dx%d threads%ld", pn[pass], ds, kSConvBand, l.tiles_m, l.tiles_n,
                        (long)l.tiles_m * l.tiles_n * kSConvNT);
    if (l.kind == KIND_SFILTER16B)
        return snprintf(buf, n, "sfilter16b %s %s rows%d splitk%d grid%dx%d threads%ld", pn[pass], ds, kSFilter16TP, l.splits,
                        l.tiles_m, l.splits, (long)l.tiles_m * l.splits * kSFilter16NT);
    if (l.kind == KIND_SFILTER16)
        return snprintf(buf, n, "sfilter16 %s %s rows%d splitk%d grid%dx%d threads%ld", pn[pass], ds, kSFilter16TP, l.splits,
                        l.tiles_m, l.splits, (long)l.tiles_m * l.splits * kSFilter16NT);
    if (l.kind == KIND_SFILTER2)
        return snprintf(buf, n, "sfilter2 %s %s rows2 splitk%d grid%dx%d threads%ld", pn[pass], ds, l.splits, l.tiles_m,
                        l.splits, (long)l.tiles_m * l.splits * kSFilterNT);
    if (l.kind == KIND_SFILTER)
        return snprintf(buf, n, "sfilter %s %s rows2 splitk%d grid%dx%d threads%ld", pn[pass], ds, l.splits, l.tiles_m,
                        l.splits, (long)l.tiles_m * l.splits * kSFilterNT);
    if (l.kind == KIND_DFILTER16B) {
        const DFilter16bVariant &v = kDFilter16bVariants[l.tile];
        return snprintf(buf, n, "dfilter16b %s %s tile%dx%d taps%dx%d splitk%d grid%dx%d threads%ld", pn[pass], ds,
                        32 * v.KB * v.WK, 32 * v.WC, l.taps, l.groups, l.splits, l.tiles_m * l.tiles_n, l.splits,
                        (long)l.tiles_m * l.tiles_n * l.splits * 64 * v.WK * v.WC);
    }
    if (l.kind == KIND_DFILTER16) {
        const DFilter16Variant &v = kDFilter16Variants[l.tile];
        return snprintf(buf, n, "dfilter16 %s %s tile%dx%d taps%dx%d splitk%d grid%dx%d threads%ld", pn[pass], ds,
                        32 * v.KB * v.WK, 32 * v.WC, l.taps, l.groups, l.splits, l.tiles_m * l.tiles_n, l.splits,
                        (long)l.tiles_m * l.tiles_n * l.splits * 64 * v.WK * v.WC);
    }
    if (l.kind == KIND_DFILTER2) {
        const DFilter2Variant &v = kDFilter2Variants[l.tile];
        return snprintf(buf, n, "dfilter2 %s %s tile%dx32 pixelparts%d taps%dx%d splitk%d grid%dx%d threads%ld", pn[pass], ds, 32 * v.WK,
                        v.WP, l.taps, l.groups, l.splits, l.tiles_m * l.tiles_n, l.splits,
                        (long)l.tiles_m * l.tiles_n * l.splits * 64 * v.WK * v.WP);
    }
    if (l.kind == KIND_DFILTER) {
        const DFilterVariant &v = kDFilterVariants[l.tile];
        return snprintf(buf, n, "dfilter %s %s tile%dx%d taps%dx%d%s splitk%d grid%dx%d threads%ld", pn[pass], ds, 32 * v.WK,
                        32 * v.WC, l.taps, l.groups, v.aligned ? " chunks-per-image" : "", l.splits, l.tiles_m * l.tiles_n, l.splits,
                        (long)l.tiles_m * l.tiles_n * l.splits * 64 * v.WK * v.WC);
    }
    const TileInfo &ti = kTiles[l.tile];
    const long threads = (long)l.tiles_m * l.tiles_n * l.splits * 64 * ti.WM * ti.WN;
    if (l.kind == KIND_DIRECT16)
        return snprintf(buf, n, "dconv16 %s %s tile%dx%dx%d waves%dx%d panel%d splitk%d grid%dx%d threads%ld", pn[pass], ds,
                        ti.BM, 64 * ti.WN, (l.tile == TILE_512x64 || l.tile == TILE_256x64P) ? 32 : 64, ti.WM, ti.WN, l.pr, l.splits,
                        l.tiles_m * l.tiles_n, l.splits, threads);
    if (l.kind == KIND_DIRECT)
        return snprintf(buf, n, "dconv %s %s tile%dx%dx%d waves%dx%d panel%d splitk%d grid%dx%d threads%ld", pn[pass], ds,
                        ti.BM, 64 * ti.WN, l.tile == TILE_128x64 ? 16 : 32, ti.WM, ti.WN, l.pr, l.splits,
                        l.tiles_m * l.tiles_n, l.splits, threads);
    return snprintf(buf, n, "igemm %s %s tile%dx%dx%d vec%d/%d splitk%d grid%dx%d threads%ld", pn[pass], ds, ti.BM,
                    64 * ti.WN, ti.BK, dm.va ? 4 : 1, dm.vb ? 4 : 1, l.splits, l.tiles_m * l.tiles_n, l.splits, threads);
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
    g.bf16 = d->dtype == OWT_BF16;
    g.masked = (d->flags & OWT_RELU) ? 1 : 0;       // backward calls then mask dy by y > 0 themselves
    const long xe = (long)d->N * d->H * d->W * d->C, ye = (long)d->N * g.P * g.Q * d->K,
               we = (long)d->K * d->R * d->S * d->C;
    if (xe > kMaxElems || ye > kMaxElems || we > kMaxElems)
        return fail(OWT_EUNSUPPORTED, "tensor with more than 2^31-1 elements");
    return OWT_OK;
}

static owt_status check_ptr(const void *p, const char *name)
{
    if (!p) return fail(OWT_EINVAL, "%s is NULL", name);
    if (!aligned16(p)) return fail(OWT_EINVAL, "%s is not 16-byte aligned", name);
    return OWT_OK;
}

#define OWT_TRY(expr) do { owt_status st_ = (expr); if (st_ != OWT_OK) return st_; } while (0)

static owt_status check_ws(const Launch &l, void *ws, size_t ws_bytes)
{
    if (l.ws_bytes() > ws_bytes)
        return fail(OWT_EWORKSPACE, "workspace too small: need %zu bytes, got %zu", l.ws_bytes(), ws_bytes);
    if (l.ws_bytes() && (!ws || !aligned16(ws))) return fail(OWT_EINVAL, "ws is NULL or misaligned");
    return OWT_OK;
}

static owt_status conv_pass(const Geom &g, int pass, owt_dtype dt, const GemmParams &p, bool want_db,
                            void *ws, size_t ws_bytes, hipStream_t s, bool use_cache)
{
    const PassDims dm = conv_dims(g, pass);
    const Launch l = choose(g, pass, dt, dm, want_db, use_cache);
    OWT_TRY(check_ws(l, ws, ws_bytes));
    return launch(g, pass, dt, dm, p, l, ws, s);
}

static GemmParams fwd_params(const owt_conv_desc *d, const void *x, const void *w, const float *bias, void *y)
{
    GemmParams p; memset(&p, 0, sizeof(p));
    p.a = x; p.b = w; p.out = y; p.bias = bias; p.flags = d->flags;
    return p;
}
static GemmParams data_params(const owt_conv_desc *d, const void *dy, const void *y, const void *w, void *dx,
                              const void *xmask = nullptr)
{
    GemmParams p; memset(&p, 0, sizeof(p));
    p.a = dy; p.b = w; p.out = dx; p.flags = d->flags; p.xmask = xmask;
    p.mask = (d->flags & OWT_RELU) ? y : nullptr;
    return p;
}
static GemmParams filter_params(const owt_conv_desc *d, const void *x, const void *dy, const void *y, float alpha,
                                float beta, float *dw, float *db)
{
    GemmParams p; memset(&p, 0, sizeof(p));
    p.a = dy; p.b = x; p.out = dw; p.flags = d->flags; p.alpha = alpha; p.beta = beta; p.dbias = db;
    p.mask = (d->flags & OWT_RELU) ? y : nullptr;
    return p;
}

// Backward pass of a fully-connected shard when both of its products run on the dense kernel.
struct FcPair { Launch ld, lf; bool fused; };
static std::map<PlanKey, int> g_fc_fused;      // timed by owt_fc_autotune: 1 = one launch for both products

static bool find_fc_launch(const Geom &g, int pass, int tile, Launch &out)
{
    std::vector<Launch> c;
    enumerate(g, pass, conv_dims(g, pass), pass == OWT_PASS_BWD_FILTER, c);
    for (const Launch &l : c)
        if (l.kind == KIND_FCGEMM && l.tile == tile && l.splits == 1) { out = l; return true; }
    return false;
}

static std::map<PlanKey, std::pair<bool, FcPair>> g_fc_pairs;     // planned once per geometry; owt_fc_autotune erases its entry

static bool fc_pair_plan(const Geom &g, owt_dtype dt, FcPair &fp)
{
    const bool cached = !variants_forced();
    if (cached) {
        std::lock_guard<std::mutex> lk(g_tuned_mutex);
        auto it = g_fc_pairs.find(plan_key(g, 3, dt));
        if (it != g_fc_pairs.end()) { fp = it->second.second; return it->second.first; }
    }
    bool ok = false;
    fp.fused = false;
    fp.ld = choose(g, OWT_PASS_BWD_DATA, dt, conv_dims(g, OWT_PASS_BWD_DATA), false, true);
    fp.lf = choose(g, OWT_PASS_BWD_FILTER, dt, conv_dims(g, OWT_PASS_BWD_FILTER), true, true);
    if (fp.ld.kind == KIND_FCGEMM && fp.lf.kind == KIND_FCGEMM) {
        ok = true;
        Launch fd, ff;
        if (!forced(OWT_FORCE_FC_TWO_LAUNCHES) && find_fc_launch(g, OWT_PASS_BWD_DATA, kFcPairTile, fd) &&
            find_fc_launch(g, OWT_PASS_BWD_FILTER, kFcPairTile, ff)) {
            int fused = 1;                       // untimed: one launch
            {
                std::lock_guard<std::mutex> lk(g_tuned_mutex);
                auto it = g_fc_fused.find(plan_key(g, 3, dt));
                if (it != g_fc_fused.end()) fused = it->second;
            }
            if (forced(OWT_FORCE_FC_ONE_LAUNCH)) fused = 1;
            if (fused) { fp.ld = fd; fp.lf = ff; fp.fused = true; }
        }
    }
    if (cached) {
        std::lock_guard<std::mutex> lk(g_tuned_mutex);
        g_fc_pairs[plan_key(g, 3, dt)] = std::make_pair(ok, fp);
    }
    return ok;
}

static owt_status launch_fc_pair(const Geom &g, const FcPair &fp, GemmParams pd, GemmParams pf, void *ws, hipStream_t s)
{
    frame_params(g, conv_dims(g, OWT_PASS_BWD_DATA), fp.ld, ws, pd);
    frame_params(g, conv_dims(g, OWT_PASS_BWD_FILTER), fp.lf, ws, pf);
    const hipError_t e = owt_launch_fcgemm_bwd(fp.ld.tile, fp.lf.tile, fp.fused, pd, pf, (float *)ws, s);
    if (e != hipSuccess) return fail(OWT_ELAUNCH, "HIP launch failed: %s", hipGetErrorString(e));
    return OWT_OK;
}

// ---------------------------------------------------------------- static scratch
// Device memory for owt_conv_bwd_filter_static: lives in the code object, one copy per GPU that loads
// the library, held until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the device address it yields (per device) is what kernels and launchers get.
static constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

static owt_status static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(OWT_ELAUNCH, "hipGetDevice failed: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(OWT_EUNSUPPORTED, "device ordinal %d out of range", dev);
    std::lock_guard<std::mutex> lk(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(OWT_ELAUNCH, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return OWT_OK;
}

}  // namespace owt

using namespace owt;

extern "C" {

const char *owt_last_error(void) { return g_err; }
int owt_abi_version(void) { return 3; }

void owt_test_force_variant(int tile, int splitk, unsigned flags)
{
    g_force_tile.store(tile < 0 ? -1 : tile);
    g_force_split.store(splitk > 0 ? splitk : -1);
    g_force_flags.store(flags);
}

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
    // every candidate launch covers all reduction steps with no empty split, and fits its workspace bound
    static const int shapes[][7] = {{128, 3, 224, 64, 11, 4, 2}, {128, 64, 27, 192, 5, 1, 2}, {128, 192, 13, 384, 3, 1, 1},
                                    {128, 384, 13, 256, 3, 1, 1}, {8, 3, 32, 16, 5, 1, 2}, {2, 8, 7, 4, 7, 1, 0},
                                    {1024, 256, 13, 256, 3, 1, 1}, {128, 9216, 1, 512, 1, 1, 0}, {1, 1, 3, 1, 3, 1, 1}};
    for (const auto &sh : shapes) {
        Geom g;
        if (!fill_geom(g, sh[0], sh[1], sh[2], sh[2], sh[3], sh[4], sh[4], sh[5], sh[5], sh[6], sh[6])) return 2;
        for (int pass = 0; pass < 3; pass++) {
            const PassDims dm = conv_dims(g, pass);
            std::vector<Launch> c;
            enumerate(g, pass, dm, pass == OWT_PASS_BWD_FILTER, c);
            if (c.empty()) { fail(OWT_EINVAL, "no candidate for shape N=%d C=%d pass %d", sh[0], sh[1], pass); return 3; }
            const size_t bound = max_workspace(g, pass, dm, pass == OWT_PASS_BWD_FILTER);
            for (const Launch &l : c) {
                const long parts = (l.kind == KIND_SCONV || l.kind == KIND_SCONV2 || l.kind == KIND_SCONV16) ? l.tiles_n : l.splits;   // who shares the steps
                if (l.splits < 1 || parts * l.steps_per_split < l.steps ||
                    (parts - 1) * l.steps_per_split >= l.steps || l.ws_bytes() > bound ||
                    ((l.kind == KIND_DIRECT || l.kind == KIND_DIRECT16) && (l.pr > 624 || direct_panel_rows(g, pass, dm, kTiles[l.tile].BM) > l.pr))) {
                    fail(OWT_EINVAL, "bad candidate for shape N=%d C=%d pass %d", sh[0], sh[1], pass); return 4;
                }
            }
        }
    }
    return 0;
}

size_t owt_conv_workspace_bytes(const owt_conv_desc *d, int pass)
{
    Geom g;
    if (pass < 0 || pass > 2) { fail(OWT_EINVAL, "pass must be 0, 1 or 2"); return (size_t)-1; }
    if (check_conv(d, g) != OWT_OK) return (size_t)-1;
    return max_workspace(g, pass, conv_dims(g, pass), pass == OWT_PASS_BWD_FILTER);
}

int owt_conv_plan_describe(const owt_conv_desc *d, int pass, char *buf, size_t buf_bytes)
{
    Geom g;
    if (pass < 0 || pass > 2 || !buf || buf_bytes == 0) { fail(OWT_EINVAL, "bad pass or buffer"); return -1; }
    if (check_conv(d, g) != OWT_OK) return -1;
    const PassDims dm = conv_dims(g, pass);
    return describe(buf, buf_bytes, pass, d->dtype, dm, choose(g, pass, d->dtype, dm, pass == OWT_PASS_BWD_FILTER, true));
}

owt_status owt_conv_fwd(const owt_conv_desc *d, const void *x, const void *w, const float *bias,
                        void *y, void *ws, size_t ws_bytes, void *hip_stream)
{
    Geom g;
    OWT_TRY(check_conv(d, g));
    OWT_TRY(check_ptr(x, "x")); OWT_TRY(check_ptr(w, "w")); OWT_TRY(check_ptr(y, "y"));
    if (d->flags & OWT_BIAS) OWT_TRY(check_ptr(bias, "bias"));
    return conv_pass(g, OWT_PASS_FWD, d->dtype, fwd_params(d, x, w, bias, y), false, ws, ws_bytes,
                     (hipStream_t)hip_stream, true);
}

owt_status owt_conv_bwd_data(const owt_conv_desc *d, const void *dy, const void *y_or_null,
                             const void *w, void *dx, void *ws, size_t ws_bytes, void *hip_stream)
{
    Geom g;
    OWT_TRY(check_conv(d, g));
    OWT_TRY(check_ptr(dy, "dy")); OWT_TRY(check_ptr(w, "w")); OWT_TRY(check_ptr(dx, "dx"));
    if (d->flags & OWT_RELU) OWT_TRY(check_ptr(y_or_null, "y (needed for the ReLU mask)"));
    return conv_pass(g, OWT_PASS_BWD_DATA, d->dtype, data_params(d, dy, y_or_null, w, dx), false, ws, ws_bytes,
                     (hipStream_t)hip_stream, true);
}

owt_status owt_conv_bwd_data_relu_in(const owt_conv_desc *d, const void *dy, const void *y_or_null,
                                     const void *w, const void *x, void *dx, void *ws, size_t ws_bytes,
                                     void *hip_stream)
{
    Geom g;
    OWT_TRY(check_conv(d, g));
    OWT_TRY(check_ptr(dy, "dy")); OWT_TRY(check_ptr(w, "w")); OWT_TRY(check_ptr(dx, "dx")); OWT_TRY(check_ptr(x, "x"));
    if (d->flags & OWT_RELU) OWT_TRY(check_ptr(y_or_null, "y (needed for the ReLU mask)"));
    return conv_pass(g, OWT_PASS_BWD_DATA, d->dtype, data_params(d, dy, y_or_null, w, dx, x), false, ws, ws_bytes,
                     (hipStream_t)hip_stream, true);
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
    return conv_pass(g, OWT_PASS_BWD_FILTER, d->dtype, filter_params(d, x, dy, y_or_null, alpha, beta, dw, dbias_or_null),
                     true, ws, ws_bytes, (hipStream_t)hip_stream, true);
}

size_t owt_static_scratch_bytes(void) { return kStaticScratchBytes; }

owt_status owt_conv_bwd_filter_static(const owt_conv_desc *d, const void *x, const void *dy, const void *y_or_null,
                                      float alpha, float beta, float *dw, float *dbias_or_null, void *hip_stream)
{
    Geom g;
    OWT_TRY(check_conv(d, g));
    OWT_TRY(check_ptr(x, "x")); OWT_TRY(check_ptr(dy, "dy")); OWT_TRY(check_ptr(dw, "dw"));
    if (dbias_or_null) OWT_TRY(check_ptr(dbias_or_null, "dbias"));
    if (d->flags & OWT_RELU) OWT_TRY(check_ptr(y_or_null, "y (needed for the ReLU mask)"));
    const PassDims dm = conv_dims(g, OWT_PASS_BWD_FILTER);
    // the variant owt_conv_bwd_filter would run if its partial sums fit the static array, else the
    // cheapest (by the cost model) of those that do
    Launch l = choose(g, OWT_PASS_BWD_FILTER, d->dtype, dm, true, true);
    if (l.ws_bytes() > kStaticScratchBytes) {
        std::vector<Launch> c;
        enumerate(g, OWT_PASS_BWD_FILTER, dm, true, c);
        size_t best = c.size(), least = (size_t)-1;
        for (size_t i = 0; i < c.size(); i++) {
            least = c[i].ws_bytes() < least ? c[i].ws_bytes() : least;
            if (c[i].ws_bytes() <= kStaticScratchBytes && (best == c.size() || c[i].cost < c[best].cost)) best = i;
        }
        if (best == c.size())
            return fail(OWT_EWORKSPACE, "this filter gradient needs at least %zu bytes of scratch; the static buffer holds %zu "
                        "(use owt_conv_bwd_filter with a caller workspace)", least, kStaticScratchBytes);
        l = c[best];
    }
    void *ws = nullptr;
    OWT_TRY(static_scratch(&ws));
    return launch(g, OWT_PASS_BWD_FILTER, d->dtype, dm, filter_params(d, x, dy, y_or_null, alpha, beta, dw, dbias_or_null), l, ws,
                  (hipStream_t)hip_stream);
}

owt_status owt_conv_autotune(const owt_conv_desc *d, int pass, const void *x, const void *w, const float *bias,
                             void *y, const void *dy, void *dx, float *dw, float *dbias_or_null, void *ws,
                             size_t ws_bytes, void *hip_stream)
{
    Geom g;
    if (pass < 0 || pass > 2) return fail(OWT_EINVAL, "pass must be 0, 1 or 2");
    OWT_TRY(check_conv(d, g));
    OWT_TRY(check_ptr(w, "w"));
    GemmParams p;
    if (pass == OWT_PASS_FWD) {
        OWT_TRY(check_ptr(x, "x")); OWT_TRY(check_ptr(y, "y"));
        if (d->flags & OWT_BIAS) OWT_TRY(check_ptr(bias, "bias"));
        p = fwd_params(d, x, w, bias, y);
    } else {
        OWT_TRY(check_ptr(dy, "dy"));
        if (d->flags & OWT_RELU) OWT_TRY(check_ptr(y, "y (needed for the ReLU mask)"));
        if (pass == OWT_PASS_BWD_DATA) { OWT_TRY(check_ptr(dx, "dx")); p = data_params(d, dy, y, w, dx); }
        else { OWT_TRY(check_ptr(x, "x")); OWT_TRY(check_ptr(dw, "dw")); p = filter_params(d, x, dy, y, 1.f, 0.f, dw, dbias_or_null); }
    }
    const PassDims dm = conv_dims(g, pass);
    std::vector<Launch> c;
    enumerate(g, pass, dm, pass == OWT_PASS_BWD_FILTER, c);
    for (const Launch &l : c) OWT_TRY(check_ws(l, ws, ws_bytes));
    hipStream_t s = (hipStream_t)hip_stream;
    if (c.empty()) return fail(OWT_EUNSUPPORTED, "no kernel variant for this geometry");
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return fail(OWT_ELAUNCH, "hipEventCreate failed");
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return fail(OWT_ELAUNCH, "hipEventCreate failed"); }
    int best = -1; float best_ms = 0.f;
    owt_status st = OWT_OK;
    for (size_t i = 0; i < c.size() && st == OWT_OK; i++) {
        st = launch(g, pass, d->dtype, dm, p, c[i], ws, s);                       // warm-up
        if (st != OWT_OK) break;
        // 3 launches; a variant that takes under 50 us is timed again over 12 (launch jitter is a few us)
        float ms = 0.f;
        bool ok = true;
        for (int reps = 3; ok && st == OWT_OK; reps = 12) {
            ok = hipEventRecord(e0, s) == hipSuccess;
            for (int r = 0; r < reps && st == OWT_OK; r++) st = launch(g, pass, d->dtype, dm, p, c[i], ws, s);
            if (st != OWT_OK) break;
            ok = ok && hipEventRecord(e1, s) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
                 hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
            ms /= (float)reps;
            if (reps == 12 || ms > 0.05f) break;
        }
        if (st != OWT_OK) break;
        if (!ok) { st = fail(OWT_ELAUNCH, "timing a kernel variant failed: %s", hipGetErrorString(hipGetLastError())); break; }
        if (best < 0 || ms < best_ms) { best = (int)i; best_ms = ms; }
    }
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    if (st != OWT_OK) return st;
    std::lock_guard<std::mutex> lk(g_tuned_mutex);
    g_tuned[plan_key(g, pass, d->dtype)] = c[best];
    g_fc_pairs.erase(plan_key(g, 3, d->dtype));      // a pair plan built on the old choice is stale
    return OWT_OK;
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
    g.bf16 = d->dtype == OWT_BF16;
    return OWT_OK;
}

// Workspace every candidate of the shard's passes fits in, remembered per geometry: the backward call checks
// it on every launch, and listing the candidates costs microseconds on a path whose kernels take ten.
static std::map<PlanKey, size_t> g_fc_ws;

static size_t fc_workspace(const Geom &g, owt_dtype dt, int pass)
{
    const PlanKey key = plan_key(g, 4 + (pass == OWT_PASS_FWD ? 0 : 1), dt);
    if (!variants_forced()) {
        std::lock_guard<std::mutex> lk(g_tuned_mutex);
        auto it = g_fc_ws.find(key);
        if (it != g_fc_ws.end()) return it->second;
    }
    size_t need;
    if (pass == OWT_PASS_FWD) need = max_workspace(g, OWT_PASS_FWD, conv_dims(g, OWT_PASS_FWD), false);
    else {      // the backward call runs the data pass, then the filter pass, on one scratch area
        const size_t a = max_workspace(g, OWT_PASS_BWD_DATA, conv_dims(g, OWT_PASS_BWD_DATA), false);
        const size_t b = max_workspace(g, OWT_PASS_BWD_FILTER, conv_dims(g, OWT_PASS_BWD_FILTER), true);
        need = a > b ? a : b;
    }
    if (!variants_forced()) {
        std::lock_guard<std::mutex> lk(g_tuned_mutex);
        g_fc_ws[key] = need;
    }
    return need;
}

size_t owt_fc_workspace_bytes(const owt_fc_desc *d, int pass)
{
    Geom g; int ol;
    if (pass < 0 || pass > 2) { fail(OWT_EINVAL, "pass must be 0, 1 or 2"); return (size_t)-1; }
    if (check_fc(d, g, ol) != OWT_OK) return (size_t)-1;
    return fc_workspace(g, d->dtype, pass);
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
    return conv_pass(g, OWT_PASS_FWD, d->dtype, p, false, ws, ws_bytes, (hipStream_t)hip_stream, true);
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
    const size_t need = fc_workspace(g, d->dtype, OWT_PASS_BWD_DATA);
    if (ws_bytes < need) return fail(OWT_EWORKSPACE, "workspace too small: need %zu bytes, got %zu", need, ws_bytes);
    if (need && (!ws || !aligned16(ws))) return fail(OWT_EINVAL, "ws is NULL or misaligned");
    const void *mask = (d->flags & OWT_RELU) ? y_or_null : nullptr;
    GemmParams pd; memset(&pd, 0, sizeof(pd));
    pd.a = dy; pd.b = w; pd.out = dx_partial_or_null; pd.flags = d->flags; pd.mask = mask;
    GemmParams p; memset(&p, 0, sizeof(p));
    p.a = dy; p.b = x; p.out = dw; p.flags = d->flags; p.alpha = alpha; p.beta = beta;
    p.dbias = dbias_or_null; p.mask = mask;
    if (dx_partial_or_null) {
        // both products on the dense kernel: one dz for the two, and one launch for both when that is faster
        FcPair fp;
        if (fc_pair_plan(g, d->dtype, fp)) {
            OWT_TRY(check_ws(fp.ld, ws, ws_bytes)); OWT_TRY(check_ws(fp.lf, ws, ws_bytes));
            return launch_fc_pair(g, fp, pd, p, ws, (hipStream_t)hip_stream);
        }
        OWT_TRY(conv_pass(g, OWT_PASS_BWD_DATA, d->dtype, pd, false, ws, ws_bytes, (hipStream_t)hip_stream, true));
    }
    return conv_pass(g, OWT_PASS_BWD_FILTER, d->dtype, p, true, ws, ws_bytes, (hipStream_t)hip_stream, true);
}

owt_status owt_fc_autotune(const owt_fc_desc *d, const void *x, const void *w, const float *bias, void *y,
                           const void *dy, void *dx_partial, float *dw, float *dbias_or_null, void *ws,
                           size_t ws_bytes, void *hip_stream)
{
    // the shard is the convolution with H = W = R = S = 1 on [N, I] -> [N, O_local]: tune that geometry
    Geom g; int ol;
    OWT_TRY(check_fc(d, g, ol));
    owt_conv_desc c;
    memset(&c, 0, sizeof(c));
    c.N = d->N; c.C = d->I; c.H = c.W = 1; c.K = ol; c.R = c.S = 1; c.stride_h = c.stride_w = 1;
    c.dtype = d->dtype; c.flags = d->flags;
    const size_t need_f = owt_fc_workspace_bytes(d, OWT_PASS_FWD), need_b = owt_fc_workspace_bytes(d, OWT_PASS_BWD_DATA);
    if (ws_bytes < (need_f > need_b ? need_f : need_b))
        return fail(OWT_EWORKSPACE, "workspace too small: need %zu bytes, got %zu", need_f > need_b ? need_f : need_b, ws_bytes);
    OWT_TRY(owt_conv_autotune(&c, OWT_PASS_FWD, x, w, bias, y, nullptr, nullptr, nullptr, nullptr, ws, ws_bytes, hip_stream));
    OWT_TRY(owt_conv_autotune(&c, OWT_PASS_BWD_DATA, nullptr, w, nullptr, y, dy, dx_partial, nullptr, nullptr, ws, ws_bytes,
                              hip_stream));
    OWT_TRY(owt_conv_autotune(&c, OWT_PASS_BWD_FILTER, x, w, nullptr, y, dy, nullptr, dw, dbias_or_null, ws, ws_bytes,
                              hip_stream));
    // both backward products on the dense kernel: two launches (the tiles just timed) or one for both?
    Launch fd, ff;
    if (variants_forced() || !find_fc_launch(g, OWT_PASS_BWD_DATA, kFcPairTile, fd) || !find_fc_launch(g, OWT_PASS_BWD_FILTER, kFcPairTile, ff))
        return OWT_OK;
    FcPair two;
    two.ld = choose(g, OWT_PASS_BWD_DATA, d->dtype, conv_dims(g, OWT_PASS_BWD_DATA), false, true);
    two.lf = choose(g, OWT_PASS_BWD_FILTER, d->dtype, conv_dims(g, OWT_PASS_BWD_FILTER), true, true);
    two.fused = false;
    if (two.ld.kind != KIND_FCGEMM || two.lf.kind != KIND_FCGEMM) return OWT_OK;
    FcPair one; one.ld = fd; one.lf = ff; one.fused = true;
    const void *mask = (d->flags & OWT_RELU) ? y : nullptr;
    GemmParams pd; memset(&pd, 0, sizeof(pd));
    pd.a = dy; pd.b = w; pd.out = dx_partial; pd.flags = d->flags; pd.mask = mask;
    GemmParams pf; memset(&pf, 0, sizeof(pf));
    pf.a = dy; pf.b = x; pf.out = dw; pf.flags = d->flags; pf.alpha = 1.f; pf.beta = 0.f; pf.dbias = dbias_or_null; pf.mask = mask;
    hipStream_t s = (hipStream_t)hip_stream;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return fail(OWT_ELAUNCH, "hipEventCreate failed");
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return fail(OWT_ELAUNCH, "hipEventCreate failed"); }
    float ms[2] = {0.f, 0.f};
    owt_status st = OWT_OK;
    for (int v = 0; v < 2 && st == OWT_OK; v++) {
        const FcPair &fp = v ? one : two;
        st = launch_fc_pair(g, fp, pd, pf, ws, s);                                 // warm-up
        bool ok = st == OWT_OK && hipEventRecord(e0, s) == hipSuccess;
        for (int r = 0; r < 12 && st == OWT_OK; r++) st = launch_fc_pair(g, fp, pd, pf, ws, s);
        if (st != OWT_OK) break;
        ok = ok && hipEventRecord(e1, s) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
             hipEventElapsedTime(&ms[v], e0, e1) == hipSuccess;
        if (!ok) st = fail(OWT_ELAUNCH, "timing the backward pair failed: %s", hipGetErrorString(hipGetLastError()));
    }
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    if (st != OWT_OK) return st;
    std::lock_guard<std::mutex> lk(g_tuned_mutex);
    g_fc_fused[plan_key(g, 3, d->dtype)] = ms[1] < ms[0] ? 1 : 0;
    g_fc_pairs.erase(plan_key(g, 3, d->dtype));
    return OWT_OK;
}

}  // extern "C"
