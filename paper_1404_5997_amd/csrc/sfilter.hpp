// Filter gradient of a strided convolution with few input channels (the first
// layer of the Section 5 model: 3 channels, 11x11 filters, stride 4), fp32 MFMA.
//
//   dw[k][r][(s,c)] = sum over (n,p,q) of dz[n,p,q,k] * x[n, p*sh-ph+r, (q*sw-pw)*C + (s,c)]
//
// For a fixed filter row r the S*C inputs of one window are ONE contiguous run
// of floats in the NHWC image.  A work-group therefore keeps the input rows that
// TP = 2 output rows touch ((TP-1)*sh + R rows) in LDS, each row laid out with
// its zero padding, plus the dz values of those 2*Q pixels, and computes
//   acc[k][t] += dz[pix][k] * row[base(pix) + off(t)],   t = r*(S*C) + j
// The window values are gathered with 4-byte LDS reads, one per lane, so the slots t are packed
// densely (no alignment slots between filter rows: 363 slots = 12 blocks of 32 for 11x11x3, where a
// layout with 16-byte aligned rows needs 13 and leaves a quarter of the MFMAs on empty blocks).
// The 2 x NB accumulator blocks (64 filters x 32-slot blocks) are dealt to the eight wavefronts of the
// work-group, ACCS (3 or 4) each.  The pixel range is split over the grid and summed by
// splitk_reduce_kernel.
#pragma once
#include "igemm.hpp"

namespace owt {

struct SFilterGeom {
    int SEG, LPAD, SLOTS, PITCH, ROWS, NB, units_per_image, units, units_per_wg, DZP;
};
// float4 staged per thread and unit: input rows (kSFilterPNP) and dz rows (kSFilterDNP)
constexpr int kSFilterNT = 512, kSFilterACCS = 4, kSFilterPNP = 5, kSFilterDNP = 4;      // ACCS: the larger of the two instantiations

// direct-to-LDS instructions per wavefront and unit of the form that streams its units into LDS (sfilter2.hpp)
constexpr int kSFilter2PNI = 6, kSFilter2DNI = 4;

template <class T, int NT, int ACCS, int PNP, int DNP>
__global__ void __launch_bounds__(NT, 2) sfilter_kernel(const GemmParams p, const SFilterGeom sg)
{
    constexpr int TP = 2, KB = 64, DZPITCH = KB + 4;
    extern __shared__ __attribute__((aligned(16))) float slds[];
    float *panel = slds;                                   // ROWS x PITCH
    float *dzs = panel + sg.ROWS * sg.PITCH;               // DZP x DZPITCH   (DZP = TP*Q rounded up to even)
    int *pbase = (int *)(dzs + sg.DZP * DZPITCH);          // DZP

    const Geom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int k0 = blockIdx.x * KB;
    const int split = blockIdx.y;
    const int mb = wave & 1;                               // which 32 of the 64 filters this wavefront owns
    const int nb0 = wave >> 1;                             // its slot blocks: nb0, nb0 + NT/128, ...

    // per-lane offset of slot t = 32*nb + li inside the panel (relative to the pixel's base)
    int toff[ACCS];
#pragma unroll
    for (int a = 0; a < ACCS; a++) {
        const int t = 32 * (nb0 + (NT / 128) * a) + li;
        const int r = t / sg.SEG, j = t - r * sg.SEG;
        toff[a] = (nb0 + (NT / 128) * a < sg.NB && r < g.R) ? r * sg.PITCH + sg.LPAD + j : 0;
    }
    float16v acc[ACCS];
#pragma unroll
    for (int a = 0; a < ACCS; a++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[a][r] = 0.f;

    // constant parts of LDS: zero padding of the panel rows, pixel -> base table
    for (int i = tid; i < sg.ROWS * sg.PITCH; i += NT) panel[i] = 0.f;
    for (int i = tid; i < sg.DZP; i += NT) {
        const int pl = i / g.Q, q = i - pl * g.Q;
        pbase[i] = pl < TP ? pl * g.sh * sg.PITCH + q * g.sw * g.C : 0;
    }
    __syncthreads();

    const T *dzsrc = (const T *)p.a, *xsrc = (const T *)p.b, *mask = (const T *)p.mask;
    const int row_f4 = g.W * g.C / 4;                      // float4 per image row (W*C is a multiple of 4)
    const int panel_f4 = sg.ROWS * row_f4, dz_f4 = sg.DZP * (KB / 4);
    const int img_off = g.pw * g.C + sg.LPAD;              // panel float of image float 0
    float4 dbacc = make_float4(0.f, 0.f, 0.f, 0.f);
    const bool do_db = p.dbias != nullptr;

    // global -> registers for one unit (two output rows of one image), registers -> LDS
    float4 preg[PNP], dreg[DNP];
    // the pieces a thread stages are the same (row, float4) / (pixel, filter quad) for every unit:
    // the divisions happen once (row | f4 << 8 and pixel-in-row | output row << 16, or -1 when unused)
    int prf[PNP], dpq[DNP];
#pragma unroll
    for (int it = 0; it < PNP; it++) {
        const int i = tid + it * NT;
        const int row = i / row_f4, f4 = i - row * row_f4;
        prf[it] = i < panel_f4 ? (row | (f4 << 8)) : -1;
    }
#pragma unroll
    for (int it = 0; it < DNP; it++) {
        const int i = tid + it * NT;
        const int pix = i / (KB / 4), pl = pix / g.Q, q = pix - pl * g.Q;
        dpq[it] = (i < dz_f4 && pl < TP) ? (q | (pl << 16)) : -1;
    }
    const int dkq = tid % (KB / 4);                                  // NT is a multiple of KB/4: the same quad every time
    auto load_unit = [&](int u) {
        const int n = u / sg.units_per_image, p0 = (u - n * sg.units_per_image) * TP;
        const int h0 = p0 * g.sh - g.ph;
#pragma unroll
        for (int it = 0; it < PNP; it++) {
            const int row = prf[it] & 255, f4 = prf[it] >> 8, h = h0 + row;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (prf[it] >= 0 && (unsigned)h < (unsigned)g.H) v = load4(xsrc, ((n * g.H + h) * g.W) * g.C + f4 * 4);
            preg[it] = v;
        }
#pragma unroll
        for (int it = 0; it < DNP; it++) {
            const int q = dpq[it] & 0xffff, pp = p0 + (dpq[it] >> 16), k = k0 + dkq * 4;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (dpq[it] >= 0 && pp < g.P && k < g.K) {
                const int off = ((n * g.P + pp) * g.Q + q) * g.K + k;
                v = load4(dzsrc, off);
                if (mask) {
                    const float4 y = load4(mask, off);
                    v.x = y.x > 0.f ? v.x : 0.f; v.y = y.y > 0.f ? v.y : 0.f;
                    v.z = y.z > 0.f ? v.z : 0.f; v.w = y.w > 0.f ? v.w : 0.f;
                }
            }
            dreg[it] = v;
        }
    };
    auto store_unit = [&]() {
#pragma unroll
        for (int it = 0; it < PNP; it++)
            if (prf[it] >= 0) *(float4 *)(panel + (prf[it] & 255) * sg.PITCH + img_off + (prf[it] >> 8) * 4) = preg[it];
#pragma unroll
        for (int it = 0; it < DNP; it++) {
            const int i = tid + it * NT;
            if (i < dz_f4) {
                *(float4 *)(dzs + (i / (KB / 4)) * DZPITCH + dkq * 4) = dreg[it];
                if (do_db) { dbacc.x += dreg[it].x; dbacc.y += dreg[it].y; dbacc.z += dreg[it].z; dbacc.w += dreg[it].w; }
            }
        }
    };

    const int u_beg = split * sg.units_per_wg, u_end = min(sg.units, u_beg + sg.units_per_wg);
    if (u_beg < u_end) { load_unit(u_beg); store_unit(); }
    __syncthreads();
    for (int u = u_beg; u < u_end; u++) {
        const bool more = u + 1 < u_end;
        if (more) load_unit(u + 1);          // in flight while this unit's MFMAs run
        // ---- dz^T * windows: two pixels per MFMA.  Two fragment sets ping-pong so that the LDS
        // reads of the next pixel pair are issued before the MFMAs of the current one.
        const int npair = sg.DZP / 2;
        // fetch(pair, base, ...) reads the fragments of `pair` at the panel offset `base` looked up one
        // call earlier, and looks up the offset of pair + 2 for the call after next
        auto fetch = [&](int pair, int &base, float &a, float (&b)[ACCS]) {
            const int pix = 2 * pair + lh;
            a = dzs[pix * DZPITCH + mb * 32 + li];
#pragma unroll
            for (int i = 0; i < ACCS; i++) b[i] = panel[base + toff[i]];
            base = pbase[min(pix + 4, sg.DZP - 1)];
        };
        auto mma = [&](float a, const float (&b)[ACCS]) {
#pragma unroll
            for (int i = 0; i < ACCS; i++) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b[i], acc[i], 0, 0, 0);
        };
        float a0, a1, b0[ACCS], b1[ACCS];
        int base0 = pbase[lh], base1 = pbase[min(2 + lh, sg.DZP - 1)];
        fetch(0, base0, a0, b0);
        int j = 0;
        for (; j + 1 < npair; j += 2) {
            fetch(j + 1, base1, a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            mma(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            fetch(min(j + 2, npair - 1), base0, a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            mma(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (j < npair) mma(a0, b0);
        __syncthreads();
        if (more) store_unit();
        __syncthreads();
    }

    // ---- epilogue: slot t = r*(S*C) + j holds dw[k][r][j], which is element t of filter k
    const bool part = p.splits > 1;
    float *pout = part ? p.partial + (size_t)split * p.M * p.Ncols : nullptr;
    float *out = (float *)p.out;
#pragma unroll
    for (int a = 0; a < ACCS; a++) {
        const int nb = nb0 + (NT / 128) * a, t = 32 * nb + li;
        if (nb >= sg.NB || t >= g.R * sg.SEG) continue;
#pragma unroll
        for (int rr = 0; rr < 16; rr++) {
            const int k = k0 + mb * 32 + 8 * (rr / 4) + 4 * lh + (rr % 4);
            if (k >= g.K) continue;
            const size_t o = (size_t)k * g.R * sg.SEG + t;
            if (part) pout[o] = acc[a][rr];
            else out[o] = p.alpha * acc[a][rr] + (p.beta != 0.f ? p.beta * out[o] : 0.f);
        }
    }

    if (do_db) {   // every thread summed the dz quads it staged; threads with equal tid % 16 share a quad
        float *red = panel;
        *(float4 *)(red + tid * 4) = dbacc;
        __syncthreads();
        if (tid < KB && k0 + tid < g.K) {
            float s = 0.f;
            for (int j = 0; j < NT / 16; j++) s += red[(j * 16 + tid / 4) * 4 + (tid & 3)];
            const int k = k0 + tid;
            if (part) p.dbias_partial[(size_t)split * p.M + k] = s;
            else p.dbias[k] = p.alpha * s + (p.beta != 0.f ? p.beta * p.dbias[k] : 0.f);
        }
    }
}

}  // namespace owt
