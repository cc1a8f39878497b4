// Forward pass of a strided convolution with few input channels (the first layer of the
// Section 5 model: 3 channels, 11x11 filters, stride 4), fp32 storage on the fp32 MFMA, with
// the filters resident in LDS.
//
// Same view of the data as sconv.hpp (a window row is SLOTS consecutive floats of the NHWC
// image; a work-group keeps the input rows under a band of 256 consecutive output pixels in
// LDS and walks the reduction index t = r*SLOTS + jj), but a work-group owns 32 filters
// instead of 64 and keeps their whole re-laid-out bank w2[k][t] in LDS next to the band.
// The reduction loop then contains no global load, no filter-slice staging and no barrier:
// per four MFMAs a lane reads one table entry and two 16-byte fragments.  With nothing in
// the loop waiting on the vector-memory counter, the results of a band are not stored at its
// end (where every work-group of the chip would write at once and stall on the write path)
// but during the next band: one store at a time between its MFMA groups when the number of
// reduction steps is a template parameter (the loop is then unrolled completely), else
// behind its first MFMA group.  Each band is read by
// the work-groups of all filter tiles; they are numbered so that they run on the same XCD
// and share its L2.  Stores go through a buffer descriptor that ends with the band's image,
// so pixels past the end of the image and filters past K are dropped by the range check.
#pragma once
#include "sconv.hpp"

namespace owt {

// KS: the number of 40-slot reduction steps when it is known at compile time (10 for the 11x11x3 layer), else 0.
template <int KS>
__global__ void __launch_bounds__(kSConvNT, 1) sconv2_fwd_kernel(const GemmParams p, const SConvGeom sg, const float *w2,
                                                                 const int ktiles, const int nwg)
{
    constexpr int NT = kSConvNT, BAND = kSConvBand, BK = kSConvBK, KB = kSConv2KB, PNP = kSConvPNP;
    constexpr int BQ = BK / 4;                                  // quads per step
    constexpr unsigned OOB = 0x80000000u;
    extern __shared__ __attribute__((aligned(16))) float slds[];
    const int BP = sg.KSLOTS + 4;                               // bank row pitch: an odd number of 16-byte pieces
    float *bank = slds;                                         // KB x BP
    float *panel = slds + KB * BP;                              // ZROWS x PITCH; rows >= ROWS stay zero
    __shared__ int qoff[512];                                   // panel offset (floats) of reduction quad Q

    const Geom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    // work-group b runs on XCD b % 8: the filter tiles of one band group follow each other there
    const int xcd = blockIdx.x & 7, jb = blockIdx.x >> 3;
    const int kt = jb % ktiles, wg = (jb / ktiles) * 8 + xcd;
    if (wg >= nwg) return;
    const int k0 = kt * KB;

    const int PQ = g.P * g.Q;
    const int qpr = sg.SLOTS / 4;                               // quads per filter row

    for (int i = tid; i < sg.ZROWS * sg.PITCH; i += NT) panel[i] = 0.f;
    for (int i = tid; i < sg.KSTEPS * BQ; i += NT) qoff[i] = (i / qpr) * sg.PITCH + (i % qpr) * 4;
    const int kq = sg.KSLOTS / 4;
    for (int i = tid; i < KB * kq; i += NT) {
        const int line = i / kq, q = i - line * kq;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (k0 + line < g.K) v = *(const float4 *)(w2 + (size_t)(k0 + line) * sg.KSLOTS + q * 4);
        *(float4 *)(bank + line * BP + q * 4) = v;
    }

    const int row_f4 = g.W * g.C / 4, panel_f4 = sg.ROWS * row_f4;
    const int img_off = g.pw * g.C + sg.LPAD;
    float4 preg[PNP];
    // piece `it` of this thread is (row, float4 f4) of the band, the same for every band (row | f4 << 8, or -1 past it)
    int prf[PNP];
#pragma unroll
    for (int it = 0; it < PNP; it++) {
        const int i = tid + it * NT;
        const int row = i / row_f4, f4 = i - row * row_f4;
        prf[it] = i < panel_f4 ? (row | (f4 << 8)) : -1;
    }
    const __amdgpu_buffer_rsrc_t x_rsrc = owt_make_rsrc(p.a, (unsigned)g.N * g.H * g.W * g.C * 4u);
    auto load_band = [&](int u) {
        const int n = u / sg.units_per_image, p0 = g.dQ.div((u - n * sg.units_per_image) * BAND);
        const int h0 = p0 * g.sh - g.ph;                        // first input row of the band's first output row
        const int img = n * g.H * row_f4 * 16;                  // byte offset of the image
#pragma unroll
        for (int it = 0; it < PNP; it++) {
            const int row = prf[it] & 255, f4 = prf[it] >> 8, h = h0 + row;
            const bool ok = prf[it] >= 0 && (unsigned)h < (unsigned)g.H;
            preg[it] = buffer_load4(x_rsrc, ok ? (unsigned)(img + (h * row_f4 + f4) * 16) : OOB);
        }
    };
    auto store_band = [&]() {
#pragma unroll
        for (int it = 0; it < PNP; it++)
            if (prf[it] >= 0) *(float4 *)(panel + (prf[it] & 255) * sg.PITCH + img_off + (prf[it] >> 8) * 4) = preg[it];
    };

    const int u_beg = wg * sg.units_per_wg, u_end = min(sg.units, u_beg + sg.units_per_wg);
    if (u_beg < u_end) { load_band(u_beg); store_band(); }
    __syncthreads();

    const int k = k0 + li;
    const float bias = ((p.flags & 1u) && k < g.K) ? p.bias[k] : 0.f;
    const bool relu = (p.flags & 2u) != 0;
    const int K4 = g.K * 4;                                     // bytes per output pixel
    const float *bl = bank + li * BP + lh * 4;
    const int *qt = qoff + lh;

    float prev[16];
#pragma unroll
    for (int r = 0; r < 16; r++) prev[r] = 0.f;
    bool have_prev = false;
    unsigned prev_voff = OOB;
    __amdgpu_buffer_rsrc_t prev_rsrc = owt_make_rsrc(p.out, 0u);
    auto store_prev = [&](int r) {
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(prev[r]), prev_rsrc, (int)(prev_voff + (unsigned)((8 * (r / 4) + r % 4) * K4)), 0, 0);
    };

    for (int u = u_beg; u < u_end; u++) {
        const bool more_u = u + 1 < u_end;
        // the pixel this lane feeds to the MFMA: slot wave*32 + li of the band, relative to the band's first row
        // (a lane past the end of the image computes on the image's last pixel; its results are never stored)
        const int n = u / sg.units_per_image, m0 = (u - n * sg.units_per_image) * BAND;
        const int m = min(m0 + wave * 32 + li, PQ - 1), pr = g.dQ.div(m), pl = pr - (int)g.dQ.div(m0), q = m - pr * g.Q;
        const float *ap = panel + pl * g.sh * sg.PITCH + q * g.sw * g.C;
        float16v acc[2];
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][r] = 0.f;
        if (more_u) load_band(u + 1);                            // held in registers until the band is done
        // this lane's quad of pair j is Q = 2*j + lh (step j / 5 of the table); its panel offsets come from the
        // table, read one step ahead
        if constexpr (KS > 0) {
            // compile-time step count: the whole reduction unrolled, the fragments of pair j+1 requested before
            // the MFMAs of pair j, and store r of the previous band behind pair 3r+1
            constexpr int NP = KS * (BQ / 2);
            int ot[2][BQ / 2];
            float4 fa[2], fb[2];
#pragma unroll
            for (int cc = 0; cc < BQ / 2; cc++) ot[0][cc] = qt[2 * cc];
            fa[0] = *(const float4 *)(ap + ot[0][0]);
            fb[0] = *(const float4 *)bl;
#pragma unroll
            for (int j = 0; j < NP; j++) {
                const int step = j / (BQ / 2), cc = j % (BQ / 2);
                if (cc == 0 && step + 1 < KS) {
#pragma unroll
                    for (int c2 = 0; c2 < BQ / 2; c2++) ot[(step + 1) & 1][c2] = qt[(step + 1) * BQ + 2 * c2];
                }
                if (j + 1 < NP) {
                    fa[(j + 1) & 1] = *(const float4 *)(ap + ot[((j + 1) / (BQ / 2)) & 1][(j + 1) % (BQ / 2)]);
                    fb[(j + 1) & 1] = *(const float4 *)(bl + (j + 1) * 8);
                }
                __builtin_amdgcn_sched_barrier(0);
                const float4 a = fa[j & 1], b = fb[j & 1];
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc[1], 0, 0, 0);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc[1], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (j % 3 == 1 && j / 3 < 16 && have_prev) store_prev(j / 3);
            }
            static_assert(3 * 15 + 1 < NP, "all sixteen stores of the previous band fit between the pairs");
        } else {
            int onext[BQ / 2];
#pragma unroll
            for (int cc = 0; cc < BQ / 2; cc++) onext[cc] = qt[2 * cc];
            for (int step = 0; step < sg.KSTEPS; step++) {
                const bool last = step + 1 == sg.KSTEPS;
                int ocur[BQ / 2];
#pragma unroll
                for (int cc = 0; cc < BQ / 2; cc++) ocur[cc] = onext[cc];
                const int *qn = qt + (last ? 0 : (step + 1) * BQ);
#pragma unroll
                for (int cc = 0; cc < BQ / 2; cc++) onext[cc] = qn[2 * cc];
                const float *bs = bl + step * BK;
#pragma unroll
                for (int cc = 0; cc < BQ / 2; cc++) {
                    const float4 a = *(const float4 *)(ap + ocur[cc]);
                    const float4 b = *(const float4 *)(bs + cc * 8);
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc[1], 0, 0, 0);
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc[1], 0, 0, 0);
                }
                if (have_prev && step == 0) {                    // behind the first MFMAs of this band
#pragma unroll
                    for (int r = 0; r < 16; r++) store_prev(r);
                }
            }
        }
        // ---- this band's results: register r of lane (li, lh) is pixel slot 8*(r/4) + 4*lh + r%4 of the
        // wavefront's 32, filter k0 + li.  They leave during the next band (or below, after the last one).
#pragma unroll
        for (int r = 0; r < 16; r++) {
            float v = acc[0][r] + acc[1][r] + bias;
            prev[r] = relu ? fmaxf(v, 0.f) : v;
        }
        have_prev = true;
        prev_rsrc = owt_make_rsrc(p.out, (unsigned)(n + 1) * (unsigned)PQ * (unsigned)K4);
        prev_voff = k < g.K ? ((unsigned)(n * PQ + m0 + wave * 32 + 4 * lh) * (unsigned)g.K + (unsigned)k) * 4u : OOB;
        if (more_u) {
            __syncthreads();                                     // every wave is done with this band's rows
            store_band();
            __syncthreads();
        }
    }
    if (have_prev) {
#pragma unroll
        for (int r = 0; r < 16; r++) store_prev(r);
    }
}

}  // namespace owt
