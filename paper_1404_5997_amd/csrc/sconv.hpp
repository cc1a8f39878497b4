// Forward pass of a strided convolution with few input channels (the first layer
// of the Section 5 model: 3 channels, 11x11 filters, stride 4), fp32 MFMA.
//
// For a fixed filter row r the S*C inputs of one window are one contiguous run of
// floats in the NHWC image, so a window row is read as SLOTS = round4(S*C + LPAD)
// consecutive floats starting LPAD floats left of the window (16-byte aligned for
// every window because stride_w*C is a multiple of 4); the extra slots meet zero
// weights.  A work-group takes a band of 256 consecutive output pixels of one image
// (row-major, so a band starts and ends anywhere in a row: whole rows of 55 pixels
// would leave 36 of 256 MFMA rows empty), keeps the input rows those pixels touch in
// LDS, zero padding included, and walks the reduction index t = r*SLOTS + jj in
// steps of 40 slots, streaming the matching slice of the re-laid-out filters
// w2[k][t] through a double-buffered LDS tile.  Eight wavefronts each own 32 output
// pixels x 64 filters.  Work-groups loop over (image, band) units with the next
// band prefetched into registers.
#pragma once
#include <type_traits>

#include "igemm.hpp"

namespace owt {

struct SConvGeom {
    int SEG, LPAD, SLOTS, PITCH, ROWS, ZROWS, KSLOTS, KSTEPS, units_per_image, units, units_per_wg, MPIX;
};
constexpr int kSConvNT = 512, kSConvBand = 256, kSConvBK = 40, kSConvPNP = 11;
constexpr int kSConv2KB = 32;      // filters per work-group of the filters-in-LDS form (sconv2.hpp)

// w2[k][t] = w[k][r][jj - LPAD] for t = r*SLOTS + jj inside the filter, else 0 (fp32, K x KSLOTS)
template <class T>
__global__ void __launch_bounds__(256) sconv_pack_filters_kernel(const T *__restrict__ w, float *__restrict__ w2,
                                                                 int K, int R, SConvGeom sg)
{
    const int total = K * sg.KSLOTS;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < total; i += gridDim.x * 256) {
        const int k = i / sg.KSLOTS, t = i - k * sg.KSLOTS;
        const int r = t / sg.SLOTS, j = t - r * sg.SLOTS - sg.LPAD;
        w2[i] = (r < R && j >= 0 && j < sg.SEG) ? load1(w, (k * R + r) * sg.SEG + j) : 0.f;
    }
}

template <class T>
__global__ void __launch_bounds__(kSConvNT, 2) sconv_fwd_kernel(const GemmParams p, const SConvGeom sg, const float *w2)
{
    constexpr int NT = kSConvNT, BAND = kSConvBand, BK = kSConvBK, WP = BK + 4, KB = 64, PNP = kSConvPNP;
    constexpr int BQ = BK / 4;                                  // quads per step
    extern __shared__ __attribute__((aligned(16))) float slds[];
    float *Bs = slds;                                           // 2 x KB x WP
    float *panel = slds + 2 * KB * WP;                          // ZROWS x PITCH; rows >= ROWS stay zero
    // qoff[Q]: panel offset (floats) of reduction quad Q = (filter row Q / qpr, quad Q % qpr of that row).  Looked
    // up instead of being tracked with compares, selects and a multiply per group of eight MFMAs: vector-ALU
    // instructions take MFMA time on this chip, LDS reads next to none.
    __shared__ int qoff[512];

    const Geom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int k0 = blockIdx.x * KB;

    const int PQ = g.P * g.Q;
    const int qpr = sg.SLOTS / 4;                               // quads per filter row

    for (int i = tid; i < sg.ZROWS * sg.PITCH; i += NT) panel[i] = 0.f;
    for (int i = tid; i < sg.KSTEPS * BQ; i += NT) qoff[i] = (i / qpr) * sg.PITCH + (i % qpr) * 4;
    __syncthreads();

    const T *xsrc = (const T *)p.a;
    const int row_f4 = g.W * g.C / 4, panel_f4 = sg.ROWS * row_f4;
    const int img_off = g.pw * g.C + sg.LPAD;
    constexpr int BPASS = (KB + NT / BQ - 1) / (NT / BQ);       // passes of the filter-slice loader
    float4 preg[PNP], breg[BPASS];
    const int bq = tid % BQ, bl0 = tid / BQ;                    // filter-slice loader: quad, filter line
    constexpr int BLPP = NT / BQ;                               // lines per pass (51 for 512 threads)

    // piece `it` of this thread is (row, float4 f4) of the band, the same for every band: the divisions
    // happen once (row | f4 << 8, or -1 past the band)
    int prf[PNP];
#pragma unroll
    for (int it = 0; it < PNP; it++) {
        const int i = tid + it * NT;
        const int row = i / row_f4, f4 = i - row * row_f4;
        prf[it] = i < panel_f4 ? (row | (f4 << 8)) : -1;
    }
    // fp32 storage: loads go through buffer descriptors (an offset outside the descriptor reads as zeros), so a
    // piece that does not exist costs no branch, no exec masking and no zeroing
    constexpr unsigned OOB = 0x80000000u;
    const bool fast = std::is_same<T, float>::value && (size_t)g.N * g.H * g.W * g.C * 4 < OOB;
    const __amdgpu_buffer_rsrc_t x_rsrc = owt_make_rsrc(p.a, (unsigned)g.N * g.H * g.W * g.C * 4u);
    const __amdgpu_buffer_rsrc_t w2_rsrc = owt_make_rsrc(w2, (unsigned)g.K * sg.KSLOTS * 4u);
    auto load_band = [&](int u) {
        const int n = u / sg.units_per_image, p0 = g.dQ.div((u - n * sg.units_per_image) * BAND);
        const int h0 = p0 * g.sh - g.ph;                        // first input row of the band's first output row
        if (fast) {
            const int img = n * g.H * row_f4 * 16;                // byte offset of the image
#pragma unroll
            for (int it = 0; it < PNP; it++) {
                const int row = prf[it] & 255, f4 = prf[it] >> 8, h = h0 + row;
                const bool ok = prf[it] >= 0 && (unsigned)h < (unsigned)g.H;
                preg[it] = buffer_load4(x_rsrc, ok ? (unsigned)(img + (h * row_f4 + f4) * 16) : OOB);
            }
            return;
        }
#pragma unroll
        for (int it = 0; it < PNP; it++) {
            const int row = prf[it] & 255, f4 = prf[it] >> 8, h = h0 + row;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (prf[it] >= 0 && (unsigned)h < (unsigned)g.H) v = load4(xsrc, ((n * g.H + h) * g.W) * g.C + f4 * 4);
            preg[it] = v;
        }
    };
    auto store_band = [&]() {
#pragma unroll
        for (int it = 0; it < PNP; it++)
            if (prf[it] >= 0) *(float4 *)(panel + (prf[it] & 255) * sg.PITCH + img_off + (prf[it] >> 8) * 4) = preg[it];
    };
    unsigned bvoff[BPASS];             // byte offset of this thread's filter-slice pieces at step 0, or OOB
#pragma unroll
    for (int it = 0; it < BPASS; it++) {
        const int line = bl0 + it * BLPP, k = k0 + line;
        bvoff[it] = (line < KB && k < g.K) ? (unsigned)((k * sg.KSLOTS + bq * 4) * 4) : OOB;
    }
    auto load_b = [&](int step) {
#pragma unroll
        for (int it = 0; it < BPASS; it++) breg[it] = buffer_load4(w2_rsrc, __builtin_elementwise_add_sat(bvoff[it], (unsigned)(step * BK * 4)));
    };
    auto store_b = [&](float *buf) {
#pragma unroll
        for (int it = 0; it < BPASS; it++) {
            const int line = bl0 + it * BLPP;
            if (line < KB) *(float4 *)(buf + line * WP + bq * 4) = breg[it];
        }
    };

    const int u_beg = blockIdx.y * sg.units_per_wg, u_end = min(sg.units, u_beg + sg.units_per_wg);
    if (u_beg < u_end) { load_band(u_beg); store_band(); }
    load_b(0);
    store_b(Bs);
    __syncthreads();

    typedef typename EpiFwd<T>::TOut TOut;
    TOut *out = (TOut *)p.out;
    int cur = 0;
    for (int u = u_beg; u < u_end; u++) {
        const bool more_u = u + 1 < u_end;
        // the pixel this lane feeds to the MFMA: slot wave*32 + li of the band, relative to the band's first row
        const int n = u / sg.units_per_image, m0 = (u - n * sg.units_per_image) * BAND;
        const int m = m0 + wave * 32 + li, pr = g.dQ.div(m), pl = pr - (int)g.dQ.div(m0), q = m - pr * g.Q;
        const bool mvalid = m < PQ;
        const int abase = mvalid ? pl * g.sh * sg.PITCH + q * g.sw * g.C : sg.ROWS * sg.PITCH;
        float16v acc[2];
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][r] = 0.f;
        // this lane's quad of group cc in step `step` is Q = step*BQ + 2*cc + lh; its panel offsets come from the table,
        // read one step ahead, and are masked to zero for a lane without a pixel (its base is the row of zeros)
        const int omask = mvalid ? -1 : 0;
        const int *qt = qoff + lh;
        int onext[BQ / 2];
#pragma unroll
        for (int cc = 0; cc < BQ / 2; cc++) onext[cc] = qt[2 * cc];
        for (int step = 0; step < sg.KSTEPS; step++) {
            const bool last = step + 1 == sg.KSTEPS;
            if (!last || more_u) load_b(last ? 0 : step + 1);
            if (step == 0 && more_u) load_band(u + 1);          // held in registers until the band is done
            const float *Bc = Bs + cur * KB * WP;
            int ocur[BQ / 2];
#pragma unroll
            for (int cc = 0; cc < BQ / 2; cc++) ocur[cc] = onext[cc];
            const int *qn = qt + (last ? 0 : (step + 1) * BQ);
#pragma unroll
            for (int cc = 0; cc < BQ / 2; cc++) onext[cc] = qn[2 * cc];
#pragma unroll
            for (int cc = 0; cc < BQ / 2; cc++) {
                const float4 a = *(const float4 *)(panel + abase + (ocur[cc] & omask));
                const float4 b0 = *(const float4 *)(Bc + li * WP + (2 * cc + lh) * 4);
                const float4 b1 = *(const float4 *)(Bc + (32 + li) * WP + (2 * cc + lh) * 4);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b0.x, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b1.x, acc[1], 0, 0, 0);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b0.y, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b1.y, acc[1], 0, 0, 0);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b0.z, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b1.z, acc[1], 0, 0, 0);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b0.w, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b1.w, acc[1], 0, 0, 0);
            }
            if (!last || more_u) store_b(Bs + (cur ^ 1) * KB * WP);
            if (last && more_u) {
                __syncthreads();                                 // every wave is done with this band's rows
                store_band();
            }
            __syncthreads();
            cur ^= 1;
        }
        // ---- epilogue of this band: register r of lane (li, lh) is pixel slot 8*(r/4) + 4*lh + r%4 of
        // the wavefront's 32, filter li (+32 for the second accumulator)
#pragma unroll
        for (int r = 0; r < 16; r++) {
            const int mm = m0 + wave * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
            if (mm >= PQ) continue;
            const size_t row = (size_t)n * PQ + mm;
#pragma unroll
            for (int i = 0; i < 2; i++) {
                const int k = k0 + 32 * i + li;
                if (k < g.K) store1(out, row * g.K + k, EpiFwd<T>::op(p, 0, k, acc[i][r]));
            }
        }
    }
}

}  // namespace owt
