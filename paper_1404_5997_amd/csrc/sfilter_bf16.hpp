// Filter gradient of a strided convolution with few input channels and bf16 storage (the first
// layer of the Section 5 model at bf16) on the bf16 MFMA.
//
//   dw[k][r][(s,c)] = sum over (n,p,q) of dz[n,p,q,k] * x[n, p*sh-ph+r, (q*sw-pw)*C + (s,c)]
//
// Same view of the data as sfilter.hpp: for a fixed filter row r the S*C inputs of a window are
// one contiguous run of an NHWC image row, so column t = r*SLOTS + jj of the result reads the
// value jj places right of the window's (aligned) start in panel row r.  A work-group keeps the
// input rows that TP = 4 output rows touch and the dz values of those 4*Q pixels in LDS, in their
// natural [pixel][channel] / [row][value] order.  The reduction runs over pixels, which are NOT
// contiguous for either operand; both fragments are read with ds_read_b64_tr_b16 (lane mapping in
// dfilter_bf16.hpp): for dz a lane of a 16-lane group points at (pixel s/4, filters 4*(s%4)..+3),
// for x at (pixel s/4, columns 4*(s%4)..+3 of its 16-column group), i.e. four consecutive values
// of one panel row.  Each of the eight wavefronts owns 64 filters x up to two 32-column blocks
// (4 accumulators, 8 transposing reads per 4 MFMAs).  Units (image, 4-row band) are split over the
// grid and summed by splitk_reduce_kernel.
#pragma once
#include "dfilter_bf16.hpp"

namespace owt {

struct SFilter16Geom {
    int SEG, LPAD, SLOTS, PITCH, ROWS, NB, MPIX, NGP, DZP, units_per_image, units, units_per_wg;
};
constexpr int kSFilter16NT = 512, kSFilter16TP = 4, kSFilter16PNP = 8, kSFilter16DNP = 4, kSFilter16CB = 2;

// direct-to-LDS instructions per wavefront and unit (panel, dz) of the form that streams its units into LDS (sfilter16b.hpp)
constexpr int kSFilter16bPNI = 6, kSFilter16bDNI = 4;

template <int UNUSED = 0>
__global__ void __launch_bounds__(kSFilter16NT, 1) sfilter16_kernel(const GemmParams p, const SFilter16Geom sg)
{
    constexpr int NT = kSFilter16NT, TP = kSFilter16TP, KB = 64, DZPITCH = KB + 16, PNP = kSFilter16PNP, DNP = kSFilter16DNP;
    constexpr int CB = kSFilter16CB;
    extern __shared__ __attribute__((aligned(16))) uint16_t sf16[];
    uint16_t *panel = sf16;                                      // ROWS x PITCH
    uint16_t *dzs = panel + sg.ROWS * sg.PITCH;                  // DZP x DZPITCH (DZP = 16 * NGP pixels)
    int *pbase = (int *)(dzs + sg.DZP * DZPITCH);                // DZP

    const Geom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int grp16 = lane >> 4, i16 = lane & 15;
    const int k0 = blockIdx.x * KB;
    const int split = blockIdx.y;

    // source position of this lane inside a transposing read: (pixel pixsel, values colsel..colsel+3)
    const int colsel = 16 * (grp16 & 1) + 4 * (i16 & 3);
    const int pixsel = 8 * (grp16 >> 1) + (i16 >> 2);
    // panel offset of this lane's four source columns of column block a (relative to the pixel's base)
    int toff[CB];
    bool blk_ok[CB];
#pragma unroll
    for (int a = 0; a < CB; a++) {
        const int nb = wave + (NT / 64) * a, t = 32 * nb + colsel;
        const int r = t / sg.SLOTS, jj = t - r * sg.SLOTS;
        blk_ok[a] = nb < sg.NB;                                  // uniform over the wavefront
        toff[a] = (nb < sg.NB && r < g.R) ? r * sg.PITCH + jj : 0;
    }
    float16v acc[2][CB];
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int a = 0; a < CB; a++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[kb][a][r] = 0.f;

    // constant parts of LDS: zero padding of the panel rows, pixel -> base table
    for (int i = tid; i < sg.ROWS * sg.PITCH / 2; i += NT) ((uint32_t *)panel)[i] = 0u;
    for (int i = tid; i < sg.DZP; i += NT) {
        const int pl = i / g.Q, q = i - pl * g.Q;
        pbase[i] = i < sg.MPIX ? pl * g.sh * sg.PITCH + q * g.sw * g.C : 0;
    }

    const uint16_t *dzsrc = (const uint16_t *)p.a, *xsrc = (const uint16_t *)p.b, *mask = (const uint16_t *)p.mask;
    const int row_q = g.W * g.C / 4, panel_q = sg.ROWS * row_q;  // 8-byte pieces per image row / per band
    const int img_off = g.pw * g.C + sg.LPAD;
    // piece `it` of this thread: the same (row, piece) / (pixel, filter octet) for every unit
    int prf[PNP];                                                // row | piece << 8, or -1 past the band
#pragma unroll
    for (int it = 0; it < PNP; it++) {
        const int i = tid + it * NT;
        const int row = i / row_q, f = i - row * row_q;
        prf[it] = i < panel_q ? (row | (f << 8)) : -1;
    }
    const int dko = tid & 7, dpix0 = tid >> 3;                   // dz piece: filters k0 + 8*dko.., pixels dpix0 + 32*it
    const bool dk_ok = k0 + dko * 8 < g.K;
    __syncthreads();

    uint2 preg[PNP];
    uint4 dreg[DNP];
    float dbacc[8];
#pragma unroll
    for (int j = 0; j < 8; j++) dbacc[j] = 0.f;
    const bool do_db = p.dbias != nullptr;
    const uint4 zero4 = make_uint4(0u, 0u, 0u, 0u);

    auto load_unit = [&](int u) {
        const int n = u / sg.units_per_image, p0 = (u - n * sg.units_per_image) * TP;
        const int h0 = p0 * g.sh - g.ph;
        const uint16_t *src = xsrc + ((long)n * g.H + h0) * g.W * g.C;      // may point before the image: rows are checked
#pragma unroll
        for (int it = 0; it < PNP; it++) {
            uint2 v = make_uint2(0u, 0u);
            const int row = prf[it] & 255, f = prf[it] >> 8;
            if (prf[it] >= 0 && (unsigned)(h0 + row) < (unsigned)g.H) v = *(const uint2 *)(src + row * g.W * g.C + f * 4);
            preg[it] = v;
        }
        // the unit's dz values are one contiguous run: output rows p0.. are consecutive in NHWC
        const int mlim = min(sg.MPIX, (g.P - p0) * g.Q);
        const size_t dz0 = ((size_t)n * g.P + p0) * g.Q * g.K + k0 + dko * 8;
#pragma unroll
        for (int it = 0; it < DNP; it++) {
            const int pix = dpix0 + it * (NT / 8);
            uint4 v = zero4;
            if (pix < mlim && dk_ok) {
                const size_t off = dz0 + (size_t)pix * g.K;
                v = *(const uint4 *)(dzsrc + off);
                if (mask) {
                    const uint4 y = *(const uint4 *)(mask + off);
                    v.x = relu_mask_pair(v.x, y.x); v.y = relu_mask_pair(v.y, y.y);
                    v.z = relu_mask_pair(v.z, y.z); v.w = relu_mask_pair(v.w, y.w);
                }
            }
            dreg[it] = v;
        }
    };
    auto store_unit = [&]() {
#pragma unroll
        for (int it = 0; it < PNP; it++)
            if (prf[it] >= 0) *(uint2 *)(panel + (prf[it] & 255) * sg.PITCH + img_off + (prf[it] >> 8) * 4) = preg[it];
#pragma unroll
        for (int it = 0; it < DNP; it++) {
            const int pix = dpix0 + it * (NT / 8);
            if (pix < sg.DZP) {
                *(uint4 *)(dzs + pix * DZPITCH + dko * 8) = dreg[it];
                if (do_db) {
                    const uint32_t w4[4] = {dreg[it].x, dreg[it].y, dreg[it].z, dreg[it].w};
#pragma unroll
                    for (int j = 0; j < 4; j++) {
                        dbacc[2 * j] += __uint_as_float(w4[j] << 16);
                        dbacc[2 * j + 1] += __uint_as_float(w4[j] & 0xffff0000u);
                    }
                }
            }
        }
    };

    const int u_beg = split * sg.units_per_wg, u_end = min(sg.units, u_beg + sg.units_per_wg);
    if (u_beg < u_end) { load_unit(u_beg); store_unit(); }
    __syncthreads();
    for (int u = u_beg; u < u_end; u++) {
        const bool more = u + 1 < u_end;
        if (more) load_unit(u + 1);          // in flight while this unit's MFMAs run
        // fragments of one 16-pixel group: dz for the two filter blocks, x for this wavefront's column
        // blocks, two transposing reads each; two register sets ping-pong
        auto fetch = [&](int gp, short8_t (&a)[2], short8_t (&b)[CB]) {
            const int px0 = 16 * gp + pixsel, px1 = px0 + 4;
            const int b0 = pbase[px0], b1 = pbase[px1];
#pragma unroll
            for (int kb = 0; kb < 2; kb++) {
                const short4_t lo = lds_read_tr16(dzs + px0 * DZPITCH + kb * 32 + colsel);
                const short4_t hi = lds_read_tr16(dzs + px1 * DZPITCH + kb * 32 + colsel);
                a[kb] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
            for (int i = 0; i < CB; i++) {
                if (!blk_ok[i]) continue;
                const short4_t lo = lds_read_tr16(panel + b0 + toff[i]);
                const short4_t hi = lds_read_tr16(panel + b1 + toff[i]);
                b[i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        };
        auto mma = [&](const short8_t (&a)[2], const short8_t (&b)[CB]) {
#pragma unroll
            for (int i = 0; i < CB; i++) {
                if (!blk_ok[i]) continue;
#pragma unroll
                for (int kb = 0; kb < 2; kb++)
                    acc[kb][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a[kb]),
                                                                        __builtin_bit_cast(bf16x8_t, b[i]), acc[kb][i], 0, 0, 0);
            }
        };
        short8_t a0[2], a1[2], b0[CB], b1[CB];
#pragma unroll
        for (int i = 0; i < CB; i++) { b0[i] = (short8_t)0; b1[i] = (short8_t)0; }
        fetch(0, a0, b0);
        for (int gp = 0; gp < sg.NGP; gp += 2) {                 // NGP is even (host)
            fetch(gp + 1, a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            mma(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            if (gp + 2 < sg.NGP) fetch(gp + 2, a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            mma(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
        if (more) store_unit();
        __syncthreads();
    }

    // ---- epilogue: column t = r*SLOTS + jj holds dw[k][r][jj - LPAD] when 0 <= jj - LPAD < S*C.
    // Register rr of lane (li, lh) of block (kb, a) is filter 32*kb + 8*(rr/4) + 4*lh + rr%4, column 32*nb + li.
    const bool part = p.splits > 1;
    float *pout = part ? p.partial + (size_t)split * p.M * p.Ncols : nullptr;
    float *out = (float *)p.out;
#pragma unroll
    for (int a = 0; a < CB; a++) {
        const int nb = wave + (NT / 64) * a, t = 32 * nb + li;
        const int r = t / sg.SLOTS, j = t - r * sg.SLOTS - sg.LPAD;
        if (nb >= sg.NB || r >= g.R || j < 0 || j >= sg.SEG) continue;
#pragma unroll
        for (int kb = 0; kb < 2; kb++)
#pragma unroll
            for (int rr = 0; rr < 16; rr++) {
                const int k = k0 + kb * 32 + 8 * (rr / 4) + 4 * lh + (rr % 4);
                if (k >= g.K) continue;
                const size_t o = ((size_t)k * g.R + r) * sg.SEG + j;
                if (part) pout[o] = acc[kb][a][rr];
                else out[o] = p.alpha * acc[kb][a][rr] + (p.beta != 0.f ? p.beta * out[o] : 0.f);
            }
    }

    if (do_db) {   // every thread summed the dz octets it staged; threads with equal tid % 8 share an octet
        float *red = (float *)sf16;                              // NT/8 x 64 floats; the launch sizes LDS for it
#pragma unroll
        for (int j = 0; j < 8; j++) red[dpix0 * KB + dko * 8 + j] = dbacc[j];
        __syncthreads();
        if (tid < KB && k0 + tid < g.K) {
            float s = 0.f;
            for (int j = 0; j < NT / 8; j++) s += red[j * KB + tid];
            const int k = k0 + tid;
            if (part) p.dbias_partial[(size_t)split * p.M + k] = s;
            else p.dbias[k] = p.alpha * s + (p.beta != 0.f ? p.beta * p.dbias[k] : 0.f);
        }
    }
}

}  // namespace owt
