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
// two different bands, half a round apart: while one half runs its MFMA loop (one wavefront per
// SIMD, fragments read two groups ahead, reads and MFMAs issued alternately), the other stores
// its results, writes its next band into its LDS rows and issues the loads of the band after
// that.  Run in step, both wavefronts of a SIMD were in the same phase, and the vector and memory
// instructions of the phases without MFMAs (more than half of a round) had nothing to hide
// behind.  Nothing is staged per reduction step; a round has two barriers, which wait for LDS
// traffic only.  The MFMA computes the transposed tile D[filter][pixel] (filters as the A
// operand), so a lane ends up with four consecutive filters of one pixel per register quad; the
// accumulators start from the biases, and the results leave through per-wavefront LDS staging
// blocks as whole 128-byte lines.  Work-groups loop over (image, 4-row band) units with the
// band after the next in registers.
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
    // which of the two bands in flight this wavefront works on (the same for all its lanes: kept in a scalar register)
    const int half = __builtin_amdgcn_readfirstlane(threadIdx.x >> 8);
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
    const int wc = g.W * g.C;
    const int row_q = wc / 4, panel_q = sg.ROWS * row_q;         // 8-byte pieces per image row / per band
    const int img_off = g.pw * g.C + sg.LPAD;
    uint2 preg[PNP];
    // Piece `it` of this thread is (row, 8-byte piece f) of the band, the same for every band: the
    // divisions happen once.  The pieces past the band repeat earlier ones (the same value goes to the
    // same place twice), so neither the loads nor the LDS writes need a predicate.
    int pcol[PNP], ploff[PNP];                                   // ploff: LDS place (values) | row << 20
#pragma unroll
    for (int it = 0; it < PNP; it++) {
        const int i = (tid + it * (NT / 2)) % panel_q;
        const int row = i / row_q, f = i - row * row_q;
        pcol[it] = 2 * (row * wc + f * 4);                       // bytes from the first value of the band's first row
        ploff[it] = (row * sg.PITCH + img_off + f * 4) | (row << 20);
    }

    // A band whose rows all lie inside the image is loaded from one scalar base plus the fixed offsets
    // above.  A band that sticks out takes every piece from its image row clamped into the image (a load
    // inside a bounds branch would wait for the one before it); pvalid remembers which pieces are real,
    // the others become zeros on their way into LDS.
    unsigned pvalid = 0xffffffffu;
    auto load_band = [&](int u) {
        const int n = u / sg.units_per_image, p0 = (u - n * sg.units_per_image) * TP;
        const int h0 = p0 * g.sh - g.ph;
        const char *img = (const char *)(xsrc + (long)n * g.H * wc);       // scalar
        if (h0 >= 0 && h0 + sg.ROWS <= g.H) {
            const char *src = img + (long)h0 * wc * 2;
            pvalid = 0xffffffffu;
#pragma unroll
            for (int it = 0; it < PNP; it++) preg[it] = *(const uint2 *)(src + (unsigned)pcol[it]);
        } else {
            pvalid = 0u;
#pragma unroll
            for (int it = 0; it < PNP; it++) {
                const int row = ploff[it] >> 20, h = h0 + row;
                if ((unsigned)h < (unsigned)g.H) pvalid |= 1u << it;
                const unsigned off = (unsigned)(pcol[it] + (min(max(h, 0), g.H - 1) - row) * wc * 2);
                preg[it] = *(const uint2 *)(img + off);
            }
        }
    };
    auto store_band = [&]() {
        if (pvalid == 0xffffffffu) {
#pragma unroll
            for (int it = 0; it < PNP; it++) *(uint2 *)(panel + (ploff[it] & 0xfffff)) = preg[it];
        } else {
#pragma unroll
            for (int it = 0; it < PNP; it++)
                *(uint2 *)(panel + (ploff[it] & 0xfffff)) = ((pvalid >> it) & 1u) ? preg[it] : make_uint2(0u, 0u);
        }
    };
    // A barrier that waits for this wavefront's LDS traffic only: global loads and stores stay in flight
    // across it (the compiler waits for a load where its registers are used).
    auto lds_barrier = [&]() {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xc07f);                      // lgkmcnt(0), vmcnt and expcnt untouched
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    const int u_beg = blockIdx.y * sg.units_per_wg, u_end = min(sg.units, u_beg + sg.units_per_wg);
    if (u_beg + half < u_end) { load_band(u_beg + half); store_band(); }
    if (u_beg + half + 2 < u_end) load_band(u_beg + half + 2);   // in flight during the first band's MFMAs
    __syncthreads();

    uint16_t *out = (uint16_t *)p.out;
    constexpr int EP = kSConv16EP;
    const bool staged = sg.STAGE > 0 && (g.K & 7) == 0;          // 16-byte output pieces need K % 8 == 0
    uint16_t *stage = s16 + sg.STAGE + (int)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6) * 32 * EP;
    uint16_t *stw = stage + li * EP + 4 * lh;                    // this lane's pixel row of the staging block
    const uint16_t *str = stage + (lane >> 3) * EP + (lane & 7) * 8;
    const int mrow = wave * 64 + (lane >> 3);                    // pixel slot of this lane's first 16-byte piece
    const bool kok = k0 + (lane & 7) * 8 < g.K;
    const unsigned ooff = (unsigned)(mrow * g.K + (lane & 7) * 8) * 2u;      // its byte offset from the band's first result
    // ReLU on packed bf16 pairs: a signed 16-bit max with 0 clears the negative values; with -32768 it is the identity
    typedef short sc16_short2 __attribute__((ext_vector_type(2)));
    const short relu_lo = (p.flags & 2u) ? (short)0 : (short)-32768;
    const sc16_short2 relu2 = {relu_lo, relu_lo};
    auto relu_pair = [&](uint32_t v) {
        return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(sc16_short2, v), relu2));
    };

    // The two halves run half a round apart: while one is in its MFMA loop, the other stores its results,
    // writes the next band into its LDS rows and issues the loads of the band after that, so the vector
    // and memory work of one hides behind the matrix work of the other.  Every wavefront meets the same
    // number of barriers: the second half takes one before its first band, the first half one after its last.
    const bool fast5 = sg.OCT == 5 && (g.R & 1) && sg.NG == 5 * (g.R >> 1) + 3;
    if (half == 1) lds_barrier();
    for (int u0 = u_beg; u0 < u_end; u0 += 2) {
        const int u = u0 + half;
        const bool have = u < u_end, more_u = u + 2 < u_end;
        // the accumulators start from the biases (register 4*rq + j of block bk is filter 32*bk + 8*rq + 4*lh + j)
        float16v acc[2][2];                                      // [filter block][pixel block]
#pragma unroll
        for (int bk = 0; bk < 2; bk++)
#pragma unroll
            for (int rq = 0; rq < 4; rq++) {
                const float4 b4 = *(const float4 *)(biasl + 32 * bk + 8 * rq + 4 * lh);
#pragma unroll
                for (int bm = 0; bm < 2; bm++) {
                    acc[bk][bm][4 * rq] = b4.x; acc[bk][bm][4 * rq + 1] = b4.y;
                    acc[bk][bm][4 * rq + 2] = b4.z; acc[bk][bm][4 * rq + 3] = b4.w;
                }
            }

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
        if (have && fast5) {
            // Five octets to a filter row, an odd number of rows: two rows are five groups whose slots sit at
            // fixed places, so the reads take immediate offsets from three bases per pixel block (pa: before
            // the row change, pc: after it, pb: the group in which only the upper half of the lanes has
            // changed rows).  The fragments of a group are read two groups ahead of its MFMAs, and reads
            // and MFMAs are issued alternately: this wavefront has its SIMD's matrix pipe to itself.
            const int wrap = sg.PITCH - 40;
            const uint16_t *pa[2], *pb[2], *pc[2], *pw[2];
#pragma unroll
            for (int i = 0; i < 2; i++) {
                pa[i] = panel + abase[i] + 8 * lh;
                pb[i] = pa[i] + (lh ? wrap : 0);
                pc[i] = pa[i] + wrap;
                pw[i] = Bs + (i * 32 + li) * sg.WP + lh * 8;
            }
            auto rd = [&](const uint16_t *const (&px)[2], int xo, int wo, sc16_bf16x8 (&xf)[2], sc16_bf16x8 (&wf)[2]) {
#pragma unroll
                for (int bm = 0; bm < 2; bm++) {
                    const uint2 lo = *(const uint2 *)(px[bm] + xo);
                    const uint2 hi = *(const uint2 *)(px[bm] + xo + 4);
                    xf[bm] = __builtin_bit_cast(sc16_bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
                }
#pragma unroll
                for (int bk = 0; bk < 2; bk++) wf[bk] = __builtin_bit_cast(sc16_bf16x8, *(const uint4 *)(pw[bk] + wo));
            };
            auto interleave = [&]() {                            // MFMA, LDS read, MFMA, LDS read, ...
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
            };
            sc16_bf16x8 ax0[2], aw0[2], ax1[2], aw1[2], x2[2], w2f[2], x3[2], w3[2], x4[2], w4[2];
            rd(pa, 0, 0, ax0, aw0);
            rd(pa, 16, 16, ax1, aw1);
            const int units2 = g.R >> 1;
            for (int t = 0; t < units2; t++) {
                rd(pb, 32, 32, x2, w2f); mma(ax0, aw0); interleave();
                rd(pc, 48, 48, x3, w3);  mma(ax1, aw1); interleave();
                rd(pc, 64, 64, x4, w4);  mma(x2, w2f);  interleave();
#pragma unroll
                for (int i = 0; i < 2; i++) {
                    pa[i] += 2 * sg.PITCH; pb[i] += 2 * sg.PITCH; pc[i] += 2 * sg.PITCH; pw[i] += 80;
                }
                rd(pa, 0, 0, ax0, aw0);   mma(x3, w3);  interleave();
                rd(pa, 16, 16, ax1, aw1); mma(x4, w4);  interleave();
            }
            rd(pb, 32, 32, x2, w2f);
            mma(ax0, aw0);
            mma(ax1, aw1);
            mma(x2, w2f);
        } else if (have) {
            sc16_bf16x8 xf0[2], wf0[2], xf1[2], wf1[2];
            fetch(0, xf0, wf0);
            for (int gi = 0; gi < sg.NG; gi += 2) {              // NG is even (host)
                fetch(gi + 1, xf1, wf1);
                __builtin_amdgcn_sched_barrier(0);
                mma(xf0, wf0);
                __builtin_amdgcn_sched_barrier(0);
                if (gi + 2 < sg.NG) fetch(gi + 2, xf0, wf0);
                __builtin_amdgcn_sched_barrier(0);
                mma(xf1, wf1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        lds_barrier();                                           // every wavefront of the half is done with the band's rows

        // ---- the other phase: the next band goes into the rows, the loads of the one after it start,
        // and the results of this band leave.
        if (more_u) store_band();
        if (u + 4 < u_end) load_band(u + 4);

        // Output rows p0..p0+TP-1 are consecutive in NHWC, so pixel slot m of the band is output pixel
        // (n*P + p0)*Q + m.  Register r of lane (li, lh) of block (bk, bm) is filter
        // 32*bk + 8*(r/4) + 4*lh + r%4 of pixel slot wave*64 + 32*bm + li.
        const int n = u / sg.units_per_image, p0 = (u - n * sg.units_per_image) * TP;
        const int mlim = have ? min(sg.MPIX, (g.P - p0) * g.Q) : 0;
        const size_t pix0 = ((size_t)n * g.P + p0) * g.Q;
        if (staged) {
            // Results leave through LDS, 32 pixels x 64 filters per wavefront and pass: a lane writes its
            // 8-byte pieces, then the wavefront reads the block back pixel by pixel and stores 16 bytes per
            // lane, eight lanes to the 128-byte line of a pixel (stored straight from the accumulators a
            // store instruction touches 32 lines with 16 bytes each).  Each wavefront stages in a block of
            // its own, so program order is all the synchronisation this needs.
            char *outb = (char *)(out + pix0 * g.K + k0);        // scalar
            // (LDS runs a wavefront's accesses in order: the second block is written right behind the reads
            // of the first, and only then does the wavefront wait for what it read.)
            uint4 back[2][4];
#pragma unroll
            for (int bm = 0; bm < 2; bm++) {
#pragma unroll
                for (int bk = 0; bk < 2; bk++)
#pragma unroll
                    for (int rq = 0; rq < 4; rq++)
                        *(uint2 *)(stw + 32 * bk + 8 * rq) =
                            make_uint2(f32x2_to_bf16x2(acc[bk][bm][4 * rq], acc[bk][bm][4 * rq + 1]),
                                       f32x2_to_bf16x2(acc[bk][bm][4 * rq + 2], acc[bk][bm][4 * rq + 3]));
#pragma unroll
                for (int q = 0; q < 4; q++) back[bm][q] = *(const uint4 *)(str + q * 8 * EP);
                asm volatile("" ::: "memory");                   // keeps the block order: write, read, write, read
            }
#pragma unroll
            for (int bm = 0; bm < 2; bm++)
#pragma unroll
                for (int q = 0; q < 4; q++)
                    asm volatile("" : "+v"(back[bm][q].x), "+v"(back[bm][q].y), "+v"(back[bm][q].z), "+v"(back[bm][q].w));
#pragma unroll
            for (int bm = 0; bm < 2; bm++)
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    uint4 v = back[bm][q];
                    v.x = relu_pair(v.x); v.y = relu_pair(v.y); v.z = relu_pair(v.z); v.w = relu_pair(v.w);
                    const int mo = bm * 32 + q * 8;
                    if (kok && mrow < mlim - mo) *(uint4 *)(outb + (size_t)mo * g.K * 2 + ooff) = v;
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
                        if (k >= g.K) continue;                  // K is a multiple of 4: whole quads are in or out
                        uint2 o;
                        o.x = relu_pair(f32x2_to_bf16x2(acc[bk][bm][4 * rq], acc[bk][bm][4 * rq + 1]));
                        o.y = relu_pair(f32x2_to_bf16x2(acc[bk][bm][4 * rq + 2], acc[bk][bm][4 * rq + 3]));
                        *(uint2 *)(out + (pix0 + m) * g.K + k) = o;
                    }
            }
        }
        lds_barrier();                                           // the next band is in place
    }
    if (half == 0) lds_barrier();
}

}  // namespace owt
