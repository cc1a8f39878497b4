// Direct filter-gradient kernel for stride-1 "same" convolutions with bf16 storage on the bf16 MFMA
// (v_mfma_f32_32x32x16_bf16, fp32 accumulate), with the operands streamed from global memory straight
// into LDS and next to no vector-ALU work in the chunk loop.
//
//   dw[k][r][s][c] = sum over pixels (n,p,q) of dz[n,p,q,k] * x[n, p+r-pad_h, q+s-pad_w, c]
//
// (Section 4 of the paper, backward step 2: the weight gradients of the data-parallel convolution
// layers.)  Same decomposition and the same transposing fragment reads as dfilter_bf16.hpp: a
// work-group owns KT filters x CT channels x the taps of a tap group, walks over the pixels in chunks
// of 64, and keeps the dz rows and the x pixels of a chunk in LDS in zero-padded image coordinates, so
// tap (r,s) of a pixel is a fixed row offset; a wavefront holds KB x TAPS accumulators of 32 x 32.
//
// What differs is everything around the MFMAs, because a bf16 MFMA takes 32 cycles and a vector-ALU
// instruction costs the SIMD about four of them, whichever wavefront issues it: the register-staged
// kernel spends about ten vector instructions per MFMA (loader address arithmetic with divisions,
// predicates, LDS stores, fragment addresses) and keeps the matrix pipe a third busy.  Here
//  * LDS is laid out per block of 32 channels: [block][pixel][32 values], 64 bytes per pixel.  The
//    four consecutive pixel rows that a transposing read touches per half-wave are then 256
//    contiguous bytes (all 64 banks, no conflict, no padding, no swizzle), and a fragment's address
//    is a per-lane constant plus compile-time terms (block, 16-pixel group, tap), i.e. an immediate;
//  * buffer loads write LDS directly (16 bytes per lane, 1 KB = 16 pixel rows of one block per
//    wavefront instruction): no staging registers, no LDS stores, two stages, one barrier per chunk;
//    what must read as zero (pixels past the end, channels or filters past a ragged tile, padding
//    positions) gets an offset outside its descriptor;
//  * the loaders take a chunk's geometry from two LDS tables filled once (padded position -> pixel
//    offset, output pixel -> padded position) instead of divisions.  A chunk may straddle two images.
// The kernel takes dz as it is (no ReLU' mask).
#pragma once
#include <type_traits>

#include "dfilter_bf16.hpp"

namespace owt {

// SW > 0: all R x SW taps in one work-group (TAPS == R*SW), padded rows WPC pixels wide.
// SW == 0: one filter row of TAPS taps per work-group (any row width).
// PRF: panel rows per stage, a multiple of 16.  A work-group walks at most kDFilter16bMaxChunks chunks (host-checked).
template <int WK, int WC, int KB, int TAPS, int SW, int WPC, int PRF>
__global__ void __launch_bounds__(64 * WK * WC, 1) dfilter16b_kernel(const GemmParams p)
{
    constexpr int NW = WK * WC, NT = 64 * NW, KBLK = KB * WK, KT = 32 * KBLK, CT = 32 * WC, BP = 64, NG = BP / 16;
    constexpr int SUBS = PRF / 16;                                   // 16-row sets of the panel
    constexpr int DZI = KBLK * (BP / 16), PNI = WC * SUBS;           // 1 KB instructions per stage: dz, panel
    constexpr int DZB = DZI * 1024, PNB = PNI * 1024, STAGEB = DZB + PNB + 1024;   // bytes; the last KB holds the row table
    constexpr int AI = (DZI + NW - 1) / NW, RSETS = (SUBS + NW - 1) / NW;
    constexpr int CPAIRS = KBLK * 16, NPG = NT / CPAIRS;            // bias gradient: filter pairs x pixel groups
    static_assert(PRF % 16 == 0, "the panel is loaded in sets of 16 rows");
    static_assert(NPG >= 1, "the bias-gradient sums give a thread one pair of filters");
    static_assert(SW == 0 || TAPS % SW == 0, "taps = filter rows x filter width");
    constexpr unsigned OOB = 0x80000000u;                            // a byte offset no descriptor here reaches
    constexpr int TABMAX = 1024;                                     // entries of each of the two loader tables

    __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * STAGEB];
    __shared__ unsigned xoff_tab[TABMAX];
    __shared__ int prow_tab[TABMAX];
    __shared__ int4 cinfo[kDFilter16bMaxChunks][2];                  // per chunk of this work-group, see below

    const Geom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int grp16 = lane >> 4, i16 = lane & 15;                // 16-lane group and position in it
    const int wkw = wave / WC, wcw = wave % WC;

    int logical, split;
    if (!owt_split_major_wg(p.tiles_m * p.tiles_n, p.splits, logical, split)) return;
    const int kt = logical / p.tiles_n, rem = logical - kt * p.tiles_n;
    const int grp = rem / p.ctiles, ct = rem - grp * p.ctiles;
    const int k0 = kt * KT, c0 = ct * CT;
    const int ch_beg = split * p.ksteps_per_split, ch_end = min(p.ksteps, ch_beg + p.ksteps_per_split);

    const int RS = g.R * g.S, Wp = p.Wp, npix = p.Kd;
    const int r0 = p.groups > 1 ? grp : 0, rows_g = p.groups > 1 ? 1 : g.R;
    const int tap_first = p.groups > 1 ? grp * g.S : 0;

    // ---- loader tables, filled once:
    //   xoff_tab[pos], pos < Hp*Wp: byte offset inside an image of the pixel that padded position pos shows, or OOB;
    //   prow_tab[pq],  pq < P*Q:    64 (bytes per panel row) times the padded position of output pixel pq's window corner.
    // A chunk touches at most two images (host-checked: 64 <= P*Q and PRF <= Hp*Wp).
    const int IP = p.Hp * Wp, PQ = g.P * g.Q;
    for (int pos = tid; pos < IP; pos += NT) {
        const int hp = p.dWp.div(pos), wp = pos - hp * Wp, h = hp - g.ph, w = wp - g.pw;
        xoff_tab[pos] = ((unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W) ? (unsigned)((h * g.W + w) * g.C) * 2u : OOB;
    }
    for (int pq = tid; pq < PQ; pq += NT) {
        const int pp = g.dQ.div(pq), q = pq - pp * g.Q;
        prow_tab[pq] = (pp * Wp + q) * 64;
    }

    // ---- per-lane constants of the loaders.  An instruction writes 16 pixel rows of one 32-value block: lane l is
    // row l / 4, 16-byte piece l % 4.  dz instruction q = wave + NW*i is block q / 4, rows 16 (q % 4) ..; the panel's
    // 16-row set `sub` is loaded for all WC blocks by wavefront sub % NW (one table lookup serves the WC loads).
    const int lrow = lane >> 2, lpiece = lane & 3;
    unsigned davoff[AI];                  // byte offset of this lane's piece inside the chunk's dz rows, or OOB
#pragma unroll
    for (int i = 0; i < AI; i++) {
        const int q = wave + NW * i, blk = q / (BP / 16), px = (q % (BP / 16)) * 16 + lrow, k = k0 + blk * 32 + lpiece * 8;
        davoff[i] = (q < DZI && k < g.K) ? (unsigned)((px * g.K + k) * 2) : OOB;
    }
    unsigned bcoff[WC];                   // this lane's piece inside a pixel, per channel block, or OOB
#pragma unroll
    for (int w = 0; w < WC; w++) {
        const int c = c0 + w * 32 + lpiece * 8;
        bcoff[w] = c < g.C ? (unsigned)(c * 2) : OOB;
    }
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)lds;
    const owt_i32x4 xrsrc = make_rsrc(p.b, (unsigned)g.N * g.H * g.W * g.C * 2u);
    const unsigned img_bytes = (unsigned)(g.H * g.W * g.C) * 2u;

    // ---- what the loaders need to know about each of this work-group's chunks, worked out once, in parallel, and kept
    // in LDS: the scalar unit is shared by the CU's wavefronts, and a dozen of them repeating two divisions and the
    // row arithmetic per chunk cost as much as the chunk's MFMAs.
    //   x: first panel row's padded position in image n0, panel rows needed, byte offsets of images n0 and n0 + 1 (or OOB)
    //   y: byte offset of the chunk's first dz row, first pixel's index in image n0, pixels in the chunk
    for (int ci = tid; ci < ch_end - ch_beg; ci += NT) {
        const int pix0 = (ch_beg + ci) * BP, lim = min(pix0 + BP, npix);
        const int n0 = g.dPQ.div(pix0), pq0 = pix0 - n0 * PQ;
        const int pp0 = g.dQ.div(pq0), q0 = pq0 - pp0 * g.Q;
        const int pos0 = (pp0 + r0) * Wp + q0;
        const int nl = g.dPQ.div(lim - 1), pql = lim - 1 - nl * PQ;
        const int ppl = g.dQ.div(pql), ql = pql - ppl * g.Q;
        const int nrows = (nl - n0) * IP + (ppl + r0 + rows_g - 1) * Wp + ql + g.S - pos0;   // <= PRF (host-checked)
        const unsigned img0 = (unsigned)n0 * img_bytes, img1 = n0 + 1 < g.N ? img0 + img_bytes : OOB;
        cinfo[ci][0] = make_int4(pos0, nrows, (int)img0, (int)img1);
        cinfo[ci][1] = make_int4(pix0 * g.K * 2, pq0, lim - pix0, 0);
    }
    const owt_i32x4 arsrc = make_rsrc(p.a, (unsigned)npix * g.K * 2u);

    // All loads of this work-group's chunk ci, into stage `stage`.  Nothing is waited for here.
    // part 0: the dz rows and the row table; part 1: the panel; part < 0: both
    auto issue_chunk = [&](int ci, int stage, int part) {
        const int4 cx = cinfo[ci][0], cy = cinfo[ci][1];          // the same address in every lane
        const unsigned sbase = lds_base + (unsigned)stage * STAGEB;
        // dz rows of the chunk; rows past the last pixel are past the descriptor
        if (part != 1) {
#pragma unroll
        for (int i = 0; i < AI; i++)
            if (wave + NW * i < DZI) buffer_load16_to_lds(arsrc, davoff[i] + (unsigned)cy.x, sbase + (unsigned)(wave + NW * i) * 1024u);
        }
        // panel row -> padded position in image n0 or n0 + 1 -> the pixel it shows, or none (padding, past the rows
        // this chunk needs, past the last image)
        if (part != 0) {
#pragma unroll
        for (int j = 0; j < RSETS; j++) {
            const int sub = wave + NW * j;
            if (sub < SUBS) {
                const int row = sub * 16 + lrow, pos = cx.x + row;
                const unsigned t = xoff_tab[min((unsigned)pos, (unsigned)(pos - IP))];
                const unsigned pixoff = row < cx.y ? t + (unsigned)(pos >= IP ? cx.w : cx.z) : OOB;   // OOB + an image offset stays >= OOB
#pragma unroll
                for (int w = 0; w < WC; w++)
                    buffer_load16_to_lds(xrsrc, __builtin_elementwise_add_sat(pixoff, bcoff[w]),
                                         sbase + (unsigned)DZB + (unsigned)(w * SUBS + sub) * 1024u);
            }
        }
        }
        if (part != 1 && tid < BP) {       // byte offset of each pixel's panel row relative to the chunk's first
            const int pq = cy.y + tid;
            const int v = prow_tab[min((unsigned)pq, (unsigned)(pq - PQ))] + ((pq >= PQ ? IP : 0) + r0 * Wp - cx.x) * 64;
            ((int *)(lds + stage * STAGEB + DZB + PNB))[tid] = tid < cy.z ? v : 0;
        }
    };

    float16v acc[KB][TAPS];
#pragma unroll
    for (int kb = 0; kb < KB; kb++)
#pragma unroll
        for (int t = 0; t < TAPS; t++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[kb][t][r] = 0.f;
    float db0 = 0.f, db1 = 0.f;
    const bool do_db = ct == 0 && grp == 0 && p.dbias != nullptr;

    // byte offsets this lane passes to the transposing reads: source position (pixel row i16/4 of its quarter of
    // the 16-pixel group, values 4*(i16%4)..+3 of its half of the 32-value block)
    const int colb = 32 * (grp16 & 1) + 8 * (i16 & 3);
    const int pixsel = 8 * (grp16 >> 1) + (i16 >> 2);                // + 16*group (+ 4 for the second read)
    const int dz_l = (KB * wkw) * (BP * 64) + pixsel * 64 + colb;   // + kb*BP*64 + group*1024 (+ 256)
    const int pn_l = DZB + wcw * (PRF * 64) + colb;                  // + row table entry + tap*64
    const int tab_l = DZB + PNB + pixsel * 4;                        // + group*64 (+ 16)

    typedef __attribute__((address_space(3))) short4_t *lds_frag_ptr;
    auto tr = [](unsigned byte_addr) {                   // transposing read at an LDS byte address
        return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_frag_ptr)(size_t)byte_addr);
    };
    // The loads of the work-group's chunk `next` (if >= 0) are issued behind the MFMAs of the first two 16-pixel groups.
    auto compute = [&](int stage, int next) {
        const unsigned sb = lds_base + (unsigned)stage * STAGEB;
        const unsigned dzp = sb + (unsigned)dz_l;
        const unsigned char *tabp = lds + stage * STAGEB + tab_l;
        constexpr int sw = SW > 0 ? SW : 1;
        auto tapoff = [](int t) { return (SW > 0 ? (t / sw) * WPC + t % sw : t) * 64; };
        auto frag_a = [&](int gi, int kb) {
            const short4_t lo = tr(dzp + kb * (BP * 64) + gi * 1024), hi = tr(dzp + kb * (BP * 64) + gi * 1024 + 256);
            return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        };
        auto frag_b = [&](unsigned p0, unsigned p1, int t) {
            const short4_t lo = tr(p0 + tapoff(t)), hi = tr(p1 + tapoff(t));
            return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        };
        auto mfma = [&](int kb, int t, const short8_t &a, const short8_t &bq) {
            acc[kb][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, bq),
                                                                 acc[kb][t], 0, 0, 0);
        };
        if constexpr (KB * TAPS >= 12 && 64 * WK * WC > 256) {
            // Large accumulator tiles at two wavefronts per SIMD leave registers for one set of fragments only: a
            // fragment is read again for the next 16-pixel group right behind its last MFMA of this one (the x
            // fragment of a tap after the tap's KB MFMAs, the dz fragments during the last tap), and the SIMD's
            // other wavefront covers what latency that leaves.
            short8_t af[KB], bq[TAPS];
            unsigned p0 = sb + (unsigned)pn_l + *(const unsigned *)tabp, p1 = sb + (unsigned)pn_l + *(const unsigned *)(tabp + 16);
#pragma unroll
            for (int kb = 0; kb < KB; kb++) af[kb] = frag_a(0, kb);
#pragma unroll
            for (int t = 0; t < TAPS; t++) bq[t] = frag_b(p0, p1, t);
#pragma unroll
            for (int gi = 0; gi < NG; gi++) {
                if (gi + 1 < NG) {
                    p0 = sb + (unsigned)pn_l + *(const unsigned *)(tabp + (gi + 1) * 64);
                    p1 = sb + (unsigned)pn_l + *(const unsigned *)(tabp + (gi + 1) * 64 + 16);
                }
#pragma unroll
                for (int t = 0; t < TAPS; t++) {
#pragma unroll
                    for (int kb = 0; kb < KB; kb++) {
                        mfma(kb, t, af[kb], bq[t]);
                        if (t == TAPS - 1 && gi + 1 < NG) af[kb] = frag_a(gi + 1, kb);
                    }
                    if (gi + 1 < NG) bq[t] = frag_b(p0, p1, t);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (gi < 2 && next >= 0) issue_chunk(next, stage ^ 1, gi);
            }
        } else {
            // panel rows of this lane's pixels in all four groups: read first, so no fragment read waits for the table
            unsigned pb[NG][2];
#pragma unroll
            for (int gi = 0; gi < NG; gi++) {
                pb[gi][0] = sb + (unsigned)pn_l + *(const unsigned *)(tabp + gi * 64);
                pb[gi][1] = sb + (unsigned)pn_l + *(const unsigned *)(tabp + gi * 64 + 16);
            }
            // two fragment sets: the reads of group gi + 1 are issued before the MFMAs of group gi
            short8_t af[2][KB], bf[2][TAPS];
#pragma unroll
            for (int kb = 0; kb < KB; kb++) af[0][kb] = frag_a(0, kb);
#pragma unroll
            for (int t = 0; t < TAPS; t++) bf[0][t] = frag_b(pb[0][0], pb[0][1], t);
#pragma unroll
            for (int gi = 0; gi < NG; gi++) {
                __builtin_amdgcn_sched_barrier(0);
                if (gi + 1 < NG) {
#pragma unroll
                    for (int kb = 0; kb < KB; kb++) af[(gi + 1) & 1][kb] = frag_a(gi + 1, kb);
#pragma unroll
                    for (int t = 0; t < TAPS; t++) bf[(gi + 1) & 1][t] = frag_b(pb[gi + 1][0], pb[gi + 1][1], t);
                }
#pragma unroll
                for (int t = 0; t < TAPS; t++)
#pragma unroll
                    for (int kb = 0; kb < KB; kb++) mfma(kb, t, af[gi & 1][kb], bf[gi & 1][t]);
                // issue order: the next group's reads trickle out between this group's MFMAs.  Issued in one burst
                // (which is what the compiler does by itself) every wavefront of the CU stalls on the LDS queue at
                // the same time and the matrix pipe idles meanwhile: measured, read time and MFMA time then add up.
                if (gi + 1 < NG) {
                    constexpr int NM = KB * TAPS, NR = 2 * (KB + TAPS), RPM = (NR + NM - 1) / NM;
#pragma unroll
                    for (int i = 0; i < NM; i++) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, RPM, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                if (gi < 2 && next >= 0) issue_chunk(next, stage ^ 1, gi);
            }
        }
    };

    __syncthreads();                                    // the loader tables are complete
    if (ch_beg < ch_end) issue_chunk(0, 0, -1);

    int cur = 0;
    for (int ch = ch_beg; ch < ch_end; ch++) {
        // this lane's pieces of chunk ch have landed and its row-table entry is written; after the barrier that
        // holds for the whole work-group, and every wavefront is done reading the other stage (chunk ch - 1)
        __builtin_amdgcn_s_waitcnt(0x0070);             // vmcnt(0) lgkmcnt(0), expcnt untouched
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");                  // no LDS read of this stage moves above the barrier
        compute(cur, ch + 1 < ch_end ? ch + 1 - ch_beg : -1);
        if (do_db && tid < NPG * CPAIRS) {          // bias gradient: column sums of the chunk's dz rows, a pair of filters per thread
            const unsigned char *col = lds + cur * STAGEB + (tid % CPAIRS / 16) * (BP * 64) + (tid % 16) * 4;
            for (int px = tid / CPAIRS; px < BP; px += NPG) {
                const uint32_t v = *(const uint32_t *)(col + px * 64);
                db0 += __uint_as_float(v << 16);
                db1 += __uint_as_float(v & 0xffff0000u);
            }
        }
        cur ^= 1;
    }

    // ---- epilogue: dw[k][tap][c]; accumulator register r of lane (li, lh) holds
    // filter k = 8*(r/4) + 4*lh + r%4 of its 32-filter block, channel li.
    const bool part = p.splits > 1;
    float *pout = part ? p.partial + (size_t)split * p.M * p.Ncols : nullptr;
    float *out = (float *)p.out;
    const int c = c0 + wcw * 32 + li;
#pragma unroll
    for (int kb = 0; kb < KB; kb++)
#pragma unroll
        for (int t = 0; t < TAPS; t++) {
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int k = k0 + (KB * wkw + kb) * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
                if (k >= g.K || c >= g.C) continue;
                const size_t o = ((size_t)k * RS + tap_first + t) * g.C + c;
                if (part) pout[o] = acc[kb][t][r];
                else out[o] = p.alpha * acc[kb][t][r] + (p.beta != 0.f ? p.beta * out[o] : 0.f);
            }
        }

    if (do_db) {   // uniform over the work-group
        __syncthreads();                                // every wavefront is done with the stages
        float *red = (float *)lds;                      // [pixel group][filter]
        static_assert(2 * STAGEB >= NPG * KT * 4, "bias-gradient scratch must fit the stages");
        const int cp = tid % CPAIRS;
        if (tid < NPG * CPAIRS) {
            red[(tid / CPAIRS) * KT + (cp / 16) * 32 + 2 * (cp % 16)] = db0;
            red[(tid / CPAIRS) * KT + (cp / 16) * 32 + 2 * (cp % 16) + 1] = db1;
        }
        __syncthreads();
        if (tid < KT && k0 + tid < g.K) {
            float s = 0.f;
            for (int j = 0; j < NPG; j++) s += red[j * KT + tid];
            const int k = k0 + tid;
            if (part) p.dbias_partial[(size_t)split * p.M + k] = s;
            else p.dbias[k] = p.alpha * s + (p.beta != 0.f ? p.beta * p.dbias[k] : 0.f);
        }
    }
}

}  // namespace owt
