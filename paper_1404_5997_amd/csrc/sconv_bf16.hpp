// Forward pass of a strided convolution with few input channels and bf16 storage (the first
// layer of the Section 5 model at bf16: 3 channels, 11x11 filters, stride 4) on the bf16 MFMA.
//
// Same view of the data as sconv.hpp: for a fixed filter row r the S*C inputs of a window are
// one contiguous run of an NHWC image row, so a window row is read as SLOTS = round8(S*C + LPAD)
// consecutive values starting LPAD values left of the window (8-byte aligned for every window
// because stride_w*C is a multiple of 4); the extra slots meet zero weights.  The reduction
// index t = r*SLOTS + j is walked in groups of 16; a lane's 8 consecutive slots never cross a
// filter row because SLOTS is a multiple of 8.
//
// A work-group keeps the WHOLE re-laid-out filter bank of its 64 filters, w2[k][t], in LDS (57 KB
// for 11x11x3) and, beside it, two bands of input rows: the (TP-1)*stride_h + R rows that TP = 4
// output rows touch.  Its eight wavefronts form two halves that share the filter bank and work on
// two different bands at a time (two wavefronts per SIMD cover each other's LDS latency).
// Nothing is staged per reduction step; the only barriers are the two around the swap of the
// bands.  The MFMA computes the transposed tile D[filter][pixel] (filters as the A operand),
// so a lane ends up with four consecutive filters of one pixel per register quad and the
// output leaves in 8-byte pieces.  Work-groups loop over (image, 4-row band) units with the
// next band prefetched into registers.
#pragma once
#include "igemm.hpp"

namespace owt {

struct SConv16Geom {
    int SEG, LPAD, SLOTS, OCT, NG, KSLOTS, WP, PITCH, ROWS, ZROWS, MPIX, units_per_image, units, units_per_wg;
    int BIAS;       // LDS offset (values) of the 64 fp32 biases of the work-group's filters
    int STAGE;      // LDS offset (values) of the output staging blocks, 0 when they do not fit
};
constexpr int kSConv16NT = 512, kSConv16TP = 4, kSConv16PNP = 16;
constexpr int kSConv16EP = 64 + 4;                               // staging row of one pixel: 136 bytes, conflict-free 8-byte writes
constexpr int kSConv16StageValues = (kSConv16NT / 64) * 32 * kSConv16EP;    // one 32-pixel block per wavefront

typedef __bf16 sc16_bf16x8 __attribute__((ext_vector_type(8)));

// (The kernels are templates only so that this header can be included from several translation units.)
// w2[k][t] = w[k][r][j - LPAD] for t = r*SLOTS + j inside the filter, else 0 (bf16 bits, K x KSLOTS)
template <int UNUSED = 0>
__global__ void __launch_bounds__(256) sconv16_pack_filters_kernel(const uint16_t *__restrict__ w, uint16_t *__restrict__ w2,
                                                                   int K, int R, SConv16Geom sg)
{
    const int total = K * sg.KSLOTS;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < total; i += gridDim.x * 256) {
        const int k = i / sg.KSLOTS, t = i - k * sg.KSLOTS;
        const int r = t / sg.SLOTS, j = t - r * sg.SLOTS - sg.LPAD;
        w2[i] = (r < R && j >= 0 && j < sg.SEG) ? w[(k * R + r) * sg.SEG + j] : (uint16_t)0;
    }
}

template <int UNUSED = 0>
__global__ void __launch_bounds__(kSConv16NT, 1) sconv16_fwd_kernel(const GemmParams p, const SConv16Geom sg, const uint16_t *w2)
{
    constexpr int NT = kSConv16NT, TP = kSConv16TP, KB = 64, PNP = kSConv16PNP;
    extern __shared__ __attribute__((aligned(16))) uint16_t s16[];
    const int half = threadIdx.x >> 8;                           // which of the two bands in flight this wavefront works on
    uint16_t *Bs = s16;                                          // KB x WP: the filter bank of this work-group
    uint16_t *panels = s16 + KB * sg.WP;                         // 2 x ZROWS x PITCH; rows >= ROWS stay zero
    uint16_t *panel = panels + half * sg.ZROWS * sg.PITCH;

    const Geom &g = p.g;
    const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;     // position inside the half
    const int li = lane & 31, lh = lane >> 5;
    const int k0 = blockIdx.x * KB;

    // ---- one-time set-up: zero the panel, bring the filter bank in
    for (int i = threadIdx.x; i < sg.ZROWS * sg.PITCH; i += NT) ((uint32_t *)panels)[i] = 0u;     // both bands
    {
        const int octs = sg.KSLOTS / 8;                          // 16-byte pieces per filter
        for (int i = threadIdx.x; i < KB * octs; i += NT) {
            const int line = i / octs, o = i - line * octs, k = k0 + line;
            const uint4 v = k < g.K ? *(const uint4 *)(w2 + (size_t)k * sg.KSLOTS + o * 8) : make_uint4(0u, 0u, 0u, 0u);
            *(uint4 *)(Bs + line * sg.WP + o * 8) = v;
        }
    }
    // the biases of the 64 filters wait in LDS for the epilogues (32 registers per lane otherwise)
    float *biasl = (float *)(s16 + sg.BIAS);
    if (threadIdx.x < KB) biasl[threadIdx.x] = ((p.flags & 1u) && k0 + (int)threadIdx.x < g.K) ? p.bias[k0 + threadIdx.x] : 0.f;
    __syncthreads();

    // the two pixels this lane feeds to the MFMA (B operand): slots m of the band's TP*Q pixels.
    // Lanes past the band read pixel 0 instead; their columns of the result are never stored.
    int abase[2];
#pragma unroll
    for (int bm = 0; bm < 2; bm++) {
        const int m = wave * 64 + bm * 32 + li;
        const int pl = m / g.Q, q = m - pl * g.Q;
        abase[bm] = m < sg.MPIX ? pl * g.sh * sg.PITCH + q * g.sw * g.C : 0;
    }

    const uint16_t *xsrc = (const uint16_t *)p.a;
    const int row_q = g.W * g.C / 4, panel_q = sg.ROWS * row_q;  // 8-byte pieces per image row / per band
    const int img_off = g.pw * g.C + sg.LPAD;
    uint2 preg[PNP];
    // piece `it` of this thread is (row, 8-byte piece f) of the band, the same for every band: the
    // divisions happen once.  prow[it] < 0 marks pieces past the band.
    int prow[PNP], pgoff[PNP], ploff[PNP];
#pragma unroll
    for (int it = 0; it < PNP; it++) {
        const int i = tid + it * (NT / 2);
        const int row = i / row_q, f = i - row * row_q;
        prow[it] = i < panel_q ? row : -1;
        pgoff[it] = row * g.W * g.C + f * 4;                     // from the first value of the band's first row
        ploff[it] = row * sg.PITCH + img_off + f * 4;
    }

    auto load_band = [&](int u) {
        const int n = u / sg.units_per_image, p0 = (u - n * sg.units_per_image) * TP;
        const int h0 = p0 * g.sh - g.ph;
        const uint16_t *src = xsrc + ((long)n * g.H + h0) * g.W * g.C;     // may point before the image: rows are checked
#pragma unroll
        for (int it = 0; it < PNP; it++) {
            uint2 v = make_uint2(0u, 0u);
            if (prow[it] >= 0 && (unsigned)(h0 + prow[it]) < (unsigned)g.H) v = *(const uint2 *)(src + pgoff[it]);
            preg[it] = v;
        }
    };
    auto store_band = [&]() {
#pragma unroll
        for (int it = 0; it < PNP; it++)
            if (prow[it] >= 0) *(uint2 *)(panel + ploff[it]) = preg[it];
    };

    const int u_beg = blockIdx.y * sg.units_per_wg, u_end = min(sg.units, u_beg + sg.units_per_wg);
    if (u_beg + half < u_end) { load_band(u_beg + half); store_band(); }
    __syncthreads();

    uint16_t *out = (uint16_t *)p.out;
    constexpr int EP = kSConv16EP;
    const bool staged = sg.STAGE > 0 && (g.K & 7) == 0;          // 16-byte output pieces need K % 8 == 0
    uint16_t *stage = s16 + sg.STAGE + (threadIdx.x >> 6) * 32 * EP;
    const bool relu = (p.flags & 2u) != 0;
    // both halves run the same number of rounds (the barriers are work-group wide); a half without a
    // band in the last round computes on its stale rows and stores nothing
    for (int u0 = u_beg; u0 < u_end; u0 += 2) {
        const int u = u0 + half;
        const bool have = u < u_end, more_u = u + 2 < u_end;
        if (more_u) load_band(u + 2);                            // held in registers until the band is done
        float16v acc[2][2];                                      // [filter block][pixel block]
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
            for (int j = 0; j < 2; j++)
#pragma unroll
                for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

        // this lane's 8 slots of group gi are octet 2*gi + lh of the reduction: filter row oct / OCT,
        // octet oct % OCT of that row.  The fragments of group gi+1 are read before the MFMAs of group
        // gi are issued (two register sets), so the LDS latency hides behind the matrix pipe.
        int orow = 0, ocol = lh;                                 // OCT >= 2
        if (ocol >= sg.OCT) { ocol -= sg.OCT; orow++; }
        auto fetch = [&](int gi, sc16_bf16x8 (&xf)[2], sc16_bf16x8 (&wf)[2]) {
            const int xoff = orow * sg.PITCH + ocol * 8;
#pragma unroll
            for (int bm = 0; bm < 2; bm++) {
                const uint2 lo = *(const uint2 *)(panel + abase[bm] + xoff);
                const uint2 hi = *(const uint2 *)(panel + abase[bm] + xoff + 4);
                xf[bm] = __builtin_bit_cast(sc16_bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
            }
#pragma unroll
            for (int bk = 0; bk < 2; bk++)
                wf[bk] = __builtin_bit_cast(sc16_bf16x8, *(const uint4 *)(Bs + (bk * 32 + li) * sg.WP + gi * 16 + lh * 8));
            ocol += 2;
            if (ocol >= sg.OCT) { ocol -= sg.OCT; orow++; }
        };
        auto mma = [&](const sc16_bf16x8 (&xf)[2], const sc16_bf16x8 (&wf)[2]) {
#pragma unroll
            for (int bk = 0; bk < 2; bk++)
#pragma unroll
                for (int bm = 0; bm < 2; bm++)
                    acc[bk][bm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[bk], xf[bm], acc[bk][bm], 0, 0, 0);
        };
        sc16_bf16x8 xf0[2], wf0[2], xf1[2], wf1[2];
        fetch(0, xf0, wf0);
        for (int gi = 0; gi < sg.NG; gi += 2) {                  // NG is even (host)
            fetch(gi + 1, xf1, wf1);
            __builtin_amdgcn_sched_barrier(0);
            mma(xf0, wf0);
            __builtin_amdgcn_sched_barrier(0);
            if (gi + 2 < sg.NG) fetch(gi + 2, xf0, wf0);
            __builtin_amdgcn_sched_barrier(0);
            mma(xf1, wf1);
            __builtin_amdgcn_sched_barrier(0);
        }

        // ---- epilogue of this band.  Output rows p0..p0+TP-1 are consecutive in NHWC, so pixel slot m
        // of the band is output pixel (n*P + p0)*Q + m.  Register r of lane (li, lh) of block (bk, bm)
        // is filter 32*bk + 8*(r/4) + 4*lh + r%4 of pixel slot wave*64 + 32*bm + li.
        const int n = u / sg.units_per_image, p0 = (u - n * sg.units_per_image) * TP;
        const int mlim = have ? min(sg.MPIX, (g.P - p0) * g.Q) : 0;
        const size_t pix0 = ((size_t)n * g.P + p0) * g.Q;
        if (staged) {
            // Results leave through LDS, 32 pixels x 64 filters per wavefront and pass: a lane writes its
            // 8-byte pieces, then the wavefront reads the block back pixel by pixel and stores 16 bytes per
            // lane, eight lanes to the 128-byte line of a pixel (stored straight from the accumulators a
            // store instruction touches 32 lines with 16 bytes each).  Each wavefront stages in a block of
            // its own, so program order is all the synchronisation this needs.
#pragma unroll
            for (int bm = 0; bm < 2; bm++) {
#pragma unroll
                for (int bk = 0; bk < 2; bk++)
#pragma unroll
                    for (int rq = 0; rq < 4; rq++) {
                        float v[4];
#pragma unroll
                        for (int j = 0; j < 4; j++) v[j] = acc[bk][bm][4 * rq + j];
                        const float4 b4 = *(const float4 *)(biasl + 32 * bk + 8 * rq + 4 * lh);
                        v[0] += b4.x; v[1] += b4.y; v[2] += b4.z; v[3] += b4.w;
                        if (relu) {
#pragma unroll
                            for (int j = 0; j < 4; j++) v[j] = v[j] > 0.f ? v[j] : 0.f;
                        }
                        *(uint2 *)(stage + li * EP + 32 * bk + 8 * rq + 4 * lh) =
                            make_uint2(f32x2_to_bf16x2(v[0], v[1]), f32x2_to_bf16x2(v[2], v[3]));
                    }
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const int row = q * 8 + (lane >> 3), kl = (lane & 7) * 8;
                    const int m = wave * 64 + bm * 32 + row;
                    const uint4 v = *(const uint4 *)(stage + row * EP + kl);
                    if (m < mlim && k0 + kl < g.K) *(uint4 *)(out + (pix0 + m) * g.K + k0 + kl) = v;
                }
            }
        } else {
#pragma unroll
            for (int bm = 0; bm < 2; bm++) {
                const int m = wave * 64 + bm * 32 + li;
                if (m >= mlim) continue;
#pragma unroll
                for (int bk = 0; bk < 2; bk++)
#pragma unroll
                    for (int rq = 0; rq < 4; rq++) {
                        const int k = k0 + 32 * bk + 8 * rq + 4 * lh;
                        if (k >= g.K) continue;                      // K is a multiple of 4: whole quads are in or out
                        float v[4];
#pragma unroll
                        for (int j = 0; j < 4; j++) v[j] = acc[bk][bm][4 * rq + j];
                        const float4 b4 = *(const float4 *)(biasl + 32 * bk + 8 * rq + 4 * lh);
                        v[0] += b4.x; v[1] += b4.y; v[2] += b4.z; v[3] += b4.w;
                        if (relu) {
#pragma unroll
                            for (int j = 0; j < 4; j++) v[j] = v[j] > 0.f ? v[j] : 0.f;
                        }
                        uint2 o;
                        o.x = f32x2_to_bf16x2(v[0], v[1]);
                        o.y = f32x2_to_bf16x2(v[2], v[3]);
                        *(uint2 *)(out + (pix0 + m) * g.K + k) = o;
                    }
            }
        }

        if (u0 + 2 < u_end) {                                    // uniform over the work-group
            __syncthreads();                                     // every wave is done with its band's rows
            if (more_u) store_band();
            __syncthreads();
        }
    }
}

}  // namespace owt
