// Filter gradient of a strided convolution with few input channels (the first layer of the
// Section 5 model: 3 channels, 11x11 filters, stride 4), fp32 storage on the fp32 MFMA, with
// the operands streamed from global memory straight into LDS.
//
//   dw[k][r][(s,c)] = sum over (n,p,q) of dz[n,p,q,k] * x[n, p*sh-ph+r, (q*sw-pw)*C + (s,c)]
//
// Same decomposition as sfilter.hpp (a unit is two output rows of one image: the input rows
// under them, laid out with their zero padding, and the dz values of those 2*Q pixels; eight
// wavefronts share 64 filters x NB blocks of 32 densely packed (r,s,c) slots).  What differs
// is how a unit reaches LDS.  There the next unit waits in registers and every wavefront
// stops between two units to write it (two barriers, the loads' address arithmetic and
// predicates on the vector ALU).  Here LDS holds two stages and buffer loads write the next
// unit into the other stage while this one is multiplied, 16 bytes per lane and 1 KB per
// wavefront instruction, with one barrier per unit.  A stage is a flat run of 16-byte pieces:
// piece f of the panel is (row f / (PITCH/4), position f % (PITCH/4)) and piece f of dz is
// (pixel f / 17, filter quad f % 17); a lane's pieces are the same for every unit, so their
// offsets are per-lane constants and a unit adds one scalar.  Pieces that must read as zero
// (the padding left and right of a row, the pad quad of a dz row, rows above or below the
// image, pixels past its last row, filters past K) get an offset outside the descriptor of
// the unit's image, which the hardware turns into zeros: the padding is rewritten with every
// unit and nothing has to be cleared.  The kernel takes dz as it is (no ReLU' mask).
#pragma once
#include <type_traits>
#include <utility>

#include "sfilter.hpp"

namespace owt {

// PNI, DNI: direct-to-LDS instructions per wavefront and unit for the panel and for dz (kSFilter2PNI, kSFilter2DNI).
// FQ > 0: the geometry is known at compile time (Q == FQ output pixels per row, panel rows FPITCH floats apart,
// windows FSWC = stride_w * C floats apart, output rows FSH = stride_h panel rows apart).  The pixel loop of a unit
// is then unrolled completely and every LDS address in it is a per-lane base plus an immediate: vector-ALU
// instructions take MFMA time on this chip, and the run-time form spends ten of them per three MFMAs on addresses.
template <int ACCS, int PNI, int DNI, int FQ = 0, int FPITCH = 0, int FSWC = 0, int FSH = 0>
__global__ void __launch_bounds__(kSFilterNT, 1) sfilter2_kernel(const GemmParams p, const SFilterGeom sg)
{
    constexpr int NT = kSFilterNT, NW = NT / 64, TP = 2, KB = 64, DZPITCH = KB + 4, DQ = DZPITCH / 4;
    constexpr unsigned OOB = 0x80000000u;
    extern __shared__ __attribute__((aligned(1024))) float slds[];
    const int pp4 = sg.PITCH / 4;                                   // 16-byte pieces per panel row
    const int pan_inst = (sg.ROWS * pp4 + 63) / 64, dz_inst = (sg.DZP * DQ + 63) / 64;
    const int stage_f = (pan_inst + dz_inst) * 256;                 // floats per stage: panel pieces, then dz pieces
    int *pbase = (int *)(slds + 2 * stage_f);                       // DZP

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

    for (int i = tid; i < sg.DZP; i += NT) {               // pixel -> panel offset of its window's first row
        const int pl = i / g.Q, q = i - pl * g.Q;
        pbase[i] = pl < TP ? pl * g.sh * sg.PITCH + q * g.sw * g.C : 0;
    }

    // ---- per-lane constants of the loaders: instruction i of this wavefront is number wave + NW*i of the stage
    const int row_f4 = g.W * g.C / 4, rowbytes = row_f4 * 16;
    const int io4 = (g.pw * g.C + sg.LPAD) / 4;            // pieces of zero padding in front of a row's data
    unsigned pvoff[PNI], dvoff[DNI];
#pragma unroll
    for (int i = 0; i < PNI; i++) {
        const int f = (wave + NW * i) * 64 + lane, r = f / pp4, c = f - r * pp4 - io4;
        pvoff[i] = (r < sg.ROWS && (unsigned)c < (unsigned)row_f4) ? (unsigned)(r * rowbytes + c * 16) : OOB;
    }
#pragma unroll
    for (int i = 0; i < DNI; i++) {
        const int f = (wave + NW * i) * 64 + lane, pix = f / DQ, c = f - pix * DQ;
        dvoff[i] = (pix < TP * g.Q && c < KB / 4 && k0 + 4 * c < g.K) ? (unsigned)((pix * g.K + k0 + 4 * c) * 4) : OOB;
    }
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) float *)slds;
    const unsigned img_bytes = (unsigned)g.H * (unsigned)rowbytes, dzimg_bytes = (unsigned)(g.P * g.Q * g.K) * 4u;

    // All loads of unit u (two output rows of one image) into stage `stage`.  Nothing is waited for here.
    // Offsets are relative to the unit's image: a row above the image gives a negative offset, which as an
    // unsigned number is out of range like one below it; OOB plus or minus a unit's scalar stays out of range.
    auto issue_unit = [&](int u, int stage) {
        const int n = u / sg.units_per_image, p0 = (u - n * sg.units_per_image) * TP;
        const int h0 = p0 * g.sh - g.ph;
        const unsigned sbase = lds_base + (unsigned)stage * (unsigned)(stage_f * 4);
        const owt_i32x4 xrsrc = make_rsrc((const float *)p.b + (size_t)n * g.H * g.W * g.C, img_bytes);
        const unsigned xs = (unsigned)(h0 * rowbytes);
#pragma unroll
        for (int i = 0; i < PNI; i++)
            if (wave + NW * i < pan_inst) buffer_load16_to_lds(xrsrc, pvoff[i] + xs, sbase + (unsigned)(wave + NW * i) * 1024u);
        const owt_i32x4 drsrc = make_rsrc((const float *)p.a + (size_t)n * g.P * g.Q * g.K, dzimg_bytes);
        const unsigned ds = (unsigned)(p0 * g.Q * g.K) * 4u;
#pragma unroll
        for (int i = 0; i < DNI; i++)
            if (wave + NW * i < dz_inst)
                buffer_load16_to_lds(drsrc, dvoff[i] + ds, sbase + (unsigned)(pan_inst + wave + NW * i) * 1024u);
    };

    float dbacc = 0.f;
    const bool do_db = p.dbias != nullptr;
    const int u_beg = split * sg.units_per_wg, u_end = min(sg.units, u_beg + sg.units_per_wg);
    if (u_beg < u_end) issue_unit(u_beg, 0);
    int cur = 0;
    for (int u = u_beg; u < u_end; u++) {
        // this wavefront's pieces of unit u have landed (and its table writes); behind the barrier everybody's have,
        // and nobody reads the other stage (unit u-1) any more
        __builtin_amdgcn_s_waitcnt(0x0070);
        __builtin_amdgcn_s_barrier();
        if (u + 1 < u_end) issue_unit(u + 1, cur ^ 1);
        const float *panel = slds + cur * stage_f, *dzs = panel + pan_inst * 256;
        if (do_db)                                        // column sums of the unit's dz rows (rows past the image are zero)
            for (int pix = wave; pix < sg.DZP; pix += NW) dbacc += dzs[pix * DZPITCH + lane];
        auto mma = [&](float a, const float (&b)[ACCS]) {
#pragma unroll
            for (int i = 0; i < ACCS; i++) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b[i], acc[i], 0, 0, 0);
        };
        if constexpr (FQ > 0) {
            // ---- dz^T * windows, two pixels per MFMA, pairs taken inside an output row: pair i of row pl is pixels
            // (pl, 2i) and (pl, 2i + 1), one per half-wave; an odd row length leaves one pixel per row, and the two
            // leftovers of the unit's two rows make the last pair.  Fragment sets ping-pong one pair ahead.
            constexpr int RP = FQ / 2, NPAIR = 2 * RP + (FQ & 1);
            const float *ain = dzs + lh * DZPITCH + mb * 32 + li;            // in-row pairs: + (pl*FQ + 2i) * DZPITCH
            const float *ax = dzs + lh * (FQ * DZPITCH) + mb * 32 + li;      // leftover pair: + (FQ-1) * DZPITCH
            const float *bin[ACCS], *bx[ACCS];
#pragma unroll
            for (int i = 0; i < ACCS; i++) {
                bin[i] = panel + toff[i] + lh * FSWC;                        // + pl*FSH*FPITCH + 2i*FSWC
                bx[i] = panel + toff[i] + lh * (FSH * FPITCH);               // + (FQ-1)*FSWC
            }
            float fa[2], fb[2][ACCS];
            auto fetchc = [&](auto jc, float &a, float (&b)[ACCS]) {
                constexpr int j = decltype(jc)::value;
                if constexpr (j < 2 * RP) {
                    constexpr int pl = j / RP, i2 = 2 * (j % RP);
                    a = ain[(pl * FQ + i2) * DZPITCH];
#pragma unroll
                    for (int i = 0; i < ACCS; i++) b[i] = bin[i][pl * FSH * FPITCH + i2 * FSWC];
                } else {
                    a = ax[(FQ - 1) * DZPITCH];
#pragma unroll
                    for (int i = 0; i < ACCS; i++) b[i] = bx[i][(FQ - 1) * FSWC];
                }
            };
            fetchc(std::integral_constant<int, 0>{}, fa[0], fb[0]);
            auto body = [&](auto jc) {
                constexpr int j = decltype(jc)::value;
                if constexpr (j + 1 < NPAIR) fetchc(std::integral_constant<int, j + 1>{}, fa[(j + 1) & 1], fb[(j + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
                mma(fa[j & 1], fb[j & 1]);
                __builtin_amdgcn_sched_barrier(0);
            };
            [&]<int... J>(std::integer_sequence<int, J...>) { (body(std::integral_constant<int, J>{}), ...); }(std::make_integer_sequence<int, NPAIR>{});
        } else {
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
        }
        cur ^= 1;
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

    if (do_db) {   // wavefront w summed pixels w, w + 8, ... of every unit for filter k0 + lane
        __syncthreads();                                  // every wavefront is done with the stages
        float *red = slds;
        red[wave * 64 + lane] = dbacc;
        __syncthreads();
        if (tid < KB && k0 + tid < g.K) {
            float s = 0.f;
            for (int j = 0; j < NW; j++) s += red[j * 64 + tid];
            const int k = k0 + tid;
            if (part) p.dbias_partial[(size_t)split * p.M + k] = s;
            else p.dbias[k] = p.alpha * s + (p.beta != 0.f ? p.beta * p.dbias[k] : 0.f);
        }
    }
}

}  // namespace owt
