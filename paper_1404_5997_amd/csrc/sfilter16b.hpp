// Filter gradient of a strided convolution with few input channels and bf16 storage (the first
// layer of the Section 5 model at bf16) on the bf16 MFMA, with the operands streamed from global
// memory straight into LDS.
//
//   dw[k][r][(s,c)] = sum over (n,p,q) of dz[n,p,q,k] * x[n, p*sh-ph+r, (q*sw-pw)*C + (s,c)]
//
// Same view of the data and the same transposing fragment reads as sfilter_bf16.hpp (a unit is four
// output rows of one image).  The eight wavefronts are four column groups x two pixel halves: a
// wavefront owns 64 filters x up to four 32-column blocks (8 accumulators) and takes every other
// 16-pixel group of a unit, 12 transposing reads per 8 MFMAs instead of the 8 per 4 of two column
// blocks per wavefront (the kernel is bound by LDS reads and by HBM: a unit is 59 KB for 26 x 14
// MFMAs), requested one group ahead and issued between the MFMAs; the two halves add their
// accumulators up through LDS at the end, in a fixed order.
// The other difference is how a unit reaches LDS.  Knocking the loader out of that kernel (global loads
// into registers with predicates and address arithmetic, then a store phase between two barriers)
// took 39 % off its run time, the fragment reads 20 %.  Here LDS holds two stages and buffer loads
// write the next unit into the other stage while this one is multiplied (16 bytes per lane, 1 KB
// per wavefront instruction, one barrier per unit).  A stage is a flat run of 16-byte pieces: the
// panel rows with their zero padding (piece f = row f / pieces-per-row), then the dz values as
// [32-filter block][pixel][32 values], 64 bytes per pixel, so that the four consecutive pixel rows
// a transposing read touches are 256 contiguous bytes.  A lane's pieces are the same for every
// unit: their offsets are per-lane constants and a unit adds one scalar; pieces that must read as
// zero (row padding, rows outside the image, pixels past its last row, filters past K) get an
// offset outside the descriptor of the unit's image.  The kernel takes dz as it is (no ReLU' mask).
#pragma once
#include "sfilter_bf16.hpp"

namespace owt {

template <int PNI, int DNI>
__global__ void __launch_bounds__(kSFilter16NT, 1) sfilter16b_kernel(const GemmParams p, const SFilter16Geom sg)
{
    constexpr int NT = kSFilter16NT, NW = NT / 64, TP = kSFilter16TP, KB = 64, CB = 4, CG = 4;
    static_assert(CG * 2 == NW, "wavefronts = column groups x two pixel halves");
    constexpr unsigned OOB = 0x80000000u;
    extern __shared__ __attribute__((aligned(1024))) unsigned char sf16b[];
    const int PP = (sg.PITCH + 7) & ~7, pp8 = PP / 8;             // panel row pitch in values / in 16-byte pieces
    const int pan_inst = (sg.ROWS * pp8 + 63) / 64, dz_inst = sg.DZP / 8;      // 1 KB instructions per stage
    const int stage_b = (pan_inst + dz_inst) * 1024;
    int *pbase = (int *)(sf16b + 2 * stage_b);                   // DZP: byte offset of a pixel's window in the panel

    const Geom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int grp16 = lane >> 4, i16 = lane & 15;
    const int k0 = blockIdx.x * KB;
    const int split = blockIdx.y;
    const int cg = wave % CG, half = wave / CG;                   // column group (blocks cg, cg + CG, ...), pixel half

    // source position of this lane inside a transposing read: (pixel pixsel, values colsel..colsel+3)
    const int colsel = 16 * (grp16 & 1) + 4 * (i16 & 3);
    const int pixsel = 8 * (grp16 >> 1) + (i16 >> 2);
    // byte offset of this lane's four source columns of column block a (relative to the pixel's window)
    int toff[CB];
    bool blk_ok[CB];
#pragma unroll
    for (int a = 0; a < CB; a++) {
        const int nb = cg + CG * a, t = 32 * nb + colsel;
        const int r = t / sg.SLOTS, jj = t - r * sg.SLOTS;
        blk_ok[a] = nb < sg.NB;                                  // uniform over the wavefront
        toff[a] = (nb < sg.NB && r < g.R) ? (r * PP + jj) * 2 : 0;
    }
    float16v acc[2][CB];
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int a = 0; a < CB; a++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[kb][a][r] = 0.f;

    for (int i = tid; i < sg.DZP; i += NT) {
        const int pl = i / g.Q, q = i - pl * g.Q;
        pbase[i] = i < sg.MPIX ? (pl * g.sh * PP + q * g.sw * g.C) * 2 : 0;
    }

    // ---- per-lane constants of the loaders: instruction i of this wavefront is number wave + NW*i of the stage
    const int row_p8 = g.W * g.C / 8, rowbytes = row_p8 * 16;
    const int io8 = (g.pw * g.C + sg.LPAD) / 8;                  // pieces of zero padding in front of a row's data
    unsigned pvoff[PNI], dvoff[DNI];
#pragma unroll
    for (int i = 0; i < PNI; i++) {
        const int f = (wave + NW * i) * 64 + lane, r = f / pp8, c = f - r * pp8 - io8;
        pvoff[i] = (r < sg.ROWS && (unsigned)c < (unsigned)row_p8) ? (unsigned)(r * rowbytes + c * 16) : OOB;
    }
#pragma unroll
    for (int i = 0; i < DNI; i++) {
        const int f = (wave + NW * i) * 64 + lane, kb = f / (sg.DZP * 4), px = (f >> 2) - kb * sg.DZP, k = k0 + kb * 32 + (f & 3) * 8;
        dvoff[i] = (kb < 2 && px < sg.MPIX && k < g.K) ? (unsigned)((px * g.K + k) * 2) : OOB;
    }
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)sf16b;
    const unsigned img_bytes = (unsigned)g.H * (unsigned)rowbytes, dzimg_bytes = (unsigned)(g.P * g.Q * g.K) * 2u;

    // All loads of unit u (four output rows of one image) into stage `stage`.  Nothing is waited for here.
    // Offsets are relative to the unit's image: a row above the image gives a negative offset, which as an
    // unsigned number is out of range like one below it; OOB plus or minus a unit's scalar stays out of range.
    auto issue_unit = [&](int u, int stage) {
        const int n = u / sg.units_per_image, p0 = (u - n * sg.units_per_image) * TP;
        const int h0 = p0 * g.sh - g.ph;
        const unsigned sbase = lds_base + (unsigned)stage * (unsigned)stage_b;
        const owt_i32x4 xrsrc = make_rsrc((const uint16_t *)p.b + (size_t)n * g.H * g.W * g.C, img_bytes);
        const unsigned xs = (unsigned)(h0 * rowbytes);
#pragma unroll
        for (int i = 0; i < PNI; i++)
            if (wave + NW * i < pan_inst) buffer_load16_to_lds(xrsrc, pvoff[i] + xs, sbase + (unsigned)(wave + NW * i) * 1024u);
        const owt_i32x4 drsrc = make_rsrc((const uint16_t *)p.a + (size_t)n * g.P * g.Q * g.K, dzimg_bytes);
        const unsigned ds = (unsigned)(p0 * g.Q * g.K) * 2u;
#pragma unroll
        for (int i = 0; i < DNI; i++)
            if (wave + NW * i < dz_inst)
                buffer_load16_to_lds(drsrc, dvoff[i] + ds, sbase + (unsigned)(pan_inst + wave + NW * i) * 1024u);
    };

    typedef __attribute__((address_space(3))) short4_t *lds_frag_ptr;
    auto tr = [](unsigned byte_addr) { return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_frag_ptr)(size_t)byte_addr); };
    const int colb = colsel * 2;
    const int dz_l = pan_inst * 1024 + pixsel * 64 + colb;        // + kb * DZP * 64 + group * 1024 (+ 256)
    const int kbstep = sg.DZP * 64;

    float db0 = 0.f, db1 = 0.f;
    const bool do_db = p.dbias != nullptr;
    const int u_beg = split * sg.units_per_wg, u_end = min(sg.units, u_beg + sg.units_per_wg);
    if (u_beg < u_end) issue_unit(u_beg, 0);
    int cur = 0;
    for (int u = u_beg; u < u_end; u++) {
        // this wavefront's pieces of unit u have landed (and its table writes); behind the barrier everybody's have,
        // and nobody reads the other stage (unit u-1) any more
        __builtin_amdgcn_s_waitcnt(0x0070);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (u + 1 < u_end) issue_unit(u + 1, cur ^ 1);
        const unsigned sb = lds_base + (unsigned)cur * (unsigned)stage_b;
        if (do_db) {          // column sums of the unit's dz rows (rows past the image are zero), a pair of filters per thread
            const unsigned char *col = sf16b + cur * stage_b + pan_inst * 1024 + ((tid & 31) >> 4) * kbstep + (tid & 15) * 4;
            for (int px = tid >> 5; px < sg.DZP; px += NT / 32) {
                const uint32_t v = *(const uint32_t *)(col + px * 64);
                db0 += __uint_as_float(v << 16);
                db1 += __uint_as_float(v & 0xffff0000u);
            }
        }
        // fragments of one 16-pixel group: dz for the two filter blocks, x for this wavefront's column
        // blocks, two transposing reads each; two register sets ping-pong
        auto fetch = [&](int gp, short8_t (&a)[2], short8_t (&b)[CB]) {
            const int *tb = pbase + 16 * gp + pixsel;
            const unsigned b0 = sb + (unsigned)tb[0], b1 = sb + (unsigned)tb[4];
            const unsigned da = sb + (unsigned)dz_l + (unsigned)gp * 1024u;
#pragma unroll
            for (int kb = 0; kb < 2; kb++) {
                const short4_t lo = tr(da + kb * kbstep), hi = tr(da + kb * kbstep + 256);
                a[kb] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
            for (int i = 0; i < CB; i++) {
                if (!blk_ok[i]) continue;
                const short4_t lo = tr(b0 + toff[i]), hi = tr(b1 + toff[i]);
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
        // this half's groups are half, half + 2, ...: NGP / 2 of them (NGP is even, host); the next group's
        // fragments are requested before this group's MFMAs
        const int nk = sg.NGP / 2;
        fetch(half, a0, b0);
        for (int k = 0; k < nk; k += 2) {
            if (k + 1 < nk) fetch(2 * (k + 1) + half, a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            mma(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            if (k + 2 < nk) fetch(2 * (k + 2) + half, a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            if (k + 1 < nk) mma(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
        }
        cur ^= 1;
    }

    // ---- the two pixel halves add up through LDS, one column block (two accumulators) per round
    __syncthreads();                                              // every wavefront is done with the stages
    {
        float *red = (float *)sf16b + (size_t)cg * (2 * 16 * 64) + lane * 4;     // [column group][kb][r/4][lane][4]
#pragma unroll
        for (int a = 0; a < CB; a++) {
            if (half == 1) {
#pragma unroll
                for (int kb = 0; kb < 2; kb++)
#pragma unroll
                    for (int r = 0; r < 16; r += 4)
                        *(float4 *)(red + (kb * 4 + r / 4) * 256) = make_float4(acc[kb][a][r], acc[kb][a][r + 1], acc[kb][a][r + 2], acc[kb][a][r + 3]);
            }
            __syncthreads();
            if (half == 0) {
#pragma unroll
                for (int kb = 0; kb < 2; kb++)
#pragma unroll
                    for (int r = 0; r < 16; r += 4) {
                        const float4 v = *(const float4 *)(red + (kb * 4 + r / 4) * 256);
                        acc[kb][a][r] += v.x; acc[kb][a][r + 1] += v.y; acc[kb][a][r + 2] += v.z; acc[kb][a][r + 3] += v.w;
                    }
            }
            __syncthreads();
        }
    }

    // ---- epilogue: column t = r*SLOTS + jj holds dw[k][r][jj - LPAD] when 0 <= jj - LPAD < S*C.
    // Register rr of lane (li, lh) of block (kb, a) is filter 32*kb + 8*(rr/4) + 4*lh + rr%4, column 32*nb + li.
    const bool part = p.splits > 1;
    float *pout = part ? p.partial + (size_t)split * p.M * p.Ncols : nullptr;
    float *out = (float *)p.out;
#pragma unroll
    for (int a = 0; a < CB; a++) {
        const int nb = cg + CG * a, t = 32 * nb + li;
        const int r = t / sg.SLOTS, j = t - r * sg.SLOTS - sg.LPAD;
        if (half != 0 || nb >= sg.NB || r >= g.R || j < 0 || j >= sg.SEG) continue;
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

    if (do_db) {   // thread (pixel group tid / 32, filter pair tid % 32) summed its pixels of every unit; the tree ended with a barrier
        float *red = (float *)sf16b;                              // [pixel group][64 filters]
        const int cp = tid & 31;
        red[(tid >> 5) * KB + (cp >> 4) * 32 + 2 * (cp & 15)] = db0;
        red[(tid >> 5) * KB + (cp >> 4) * 32 + 2 * (cp & 15) + 1] = db1;
        __syncthreads();
        if (tid < KB && k0 + tid < g.K) {
            float s = 0.f;
            for (int j = 0; j < NT / 32; j++) s += red[j * KB + tid];
            const int k = k0 + tid;
            if (part) p.dbias_partial[(size_t)split * p.M + k] = s;
            else p.dbias[k] = p.alpha * s + (p.beta != 0.f ? p.beta * p.dbias[k] : 0.f);
        }
    }
}

}  // namespace owt
