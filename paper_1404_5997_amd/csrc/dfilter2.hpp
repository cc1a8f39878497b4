// Direct filter-gradient kernel for stride-1 "same" convolutions (P == H, Q == W), fp32 storage and
// fp32 MFMA, with the pixel reduction split INSIDE the work-group, operands streamed from global memory
// straight into LDS, and as few vector-ALU instructions per MFMA as the data layout allows.
//
//   dw[k][r][s][c] = sum over pixels (n,p,q) of dz[n,p,q,k] * x[n, p+r-pad_h, q+s-pad_w, c]
//
// (Section 4 of the paper, backward step 2: the weight gradients of the data-parallel convolution
// layers.)  Same view as dfilter.hpp: the work-group keeps the dz rows of a chunk of consecutive pixels
// and the x pixels those positions touch in LDS, in ZERO-PADDED image coordinates, where tap (r,s) of a
// pixel is a fixed row offset; each wavefront holds one 32 x 32 accumulator per tap (<= 9) and feeds all
// of them from one dz fragment.
//
// Who shares what.  In dfilter.hpp every wavefront of the chip owns accumulators of its own, so the
// chip's whole register file (75 MB of accumulators at two wavefronts per SIMD) goes to HBM as partial
// sums and comes back in the reduction pass.  Here a work-group is WK x WP wavefronts: WK filter blocks
// of 32, and WP wavefronts per block that take 32 pixels each of a 32*WP-pixel chunk.  The WP wavefronts
// of a block add their accumulators up through LDS at the end (a fixed tree, so the result is the same
// bits every run), and only one of them stores: the partial sums that leave the CU, and the number of
// splits of the pixel range across work-groups, shrink WP times.
//
// What the chunk loop avoids, and why (in-kernel cycle counters on this chip):
//  * Vector-ALU instructions.  The fp32 MFMA does not run beside vector-ALU work of the same SIMD,
//    whichever wavefront issues it: a wavefront's address arithmetic took three times as long while the
//    SIMD's other wavefront was in its MFMA phase, and a chunk took the MFMA time plus the vector-ALU time
//    of both wavefronts whatever the order of their phases.  So the padded row width WPC and the filter
//    width SW are template parameters (the LDS address of tap (r,s) is a per-pixel base, read from a table
//    of byte offsets, plus an immediate), the loaders take what they need to know about a chunk from two
//    small LDS tables instead of divisions, and whatever must read as zero (rows past the end of the
//    tensor, filters or channels past the end of a ragged tile, padding pixels) gets a buffer offset beyond
//    its descriptor's range, which the hardware turns into zeros without touching memory.
//  * Staging through registers.  Writing a chunk into LDS from registers took a tenth of the kernel: all
//    wavefronts wait for their loads, push 60 KB through ds_write and wait again before the next fragment
//    read.  Here buffer loads write LDS directly (16 bytes per lane, 1 KB per wavefront instruction, lane l
//    at base + 16 l): the next chunk lands in the other stage while this one is multiplied, with one
//    barrier per chunk.  Rows are unpadded (a fragment read runs along a row).
#pragma once
#include <type_traits>

#include "igemm.hpp"

namespace owt {

// SW > 0: all R x SW taps in one work-group (TAPS == R*SW), padded rows WPC pixels wide.
// SW == 0: one filter row of TAPS taps per work-group (any row width).
// PROWS: panel rows per stage, a multiple of 64.
template <int WK, int WP, int TAPS, int SW, int WPC, int PROWS>
__global__ void __launch_bounds__(64 * WK * WP, 1) dfilter2_kernel(const GemmParams p)
{
    constexpr int NW = WK * WP, NT = 64 * NW, KT = 32 * WK, CT = 32, BP = 32 * WP;
    constexpr int ALPR = KT / 4, ARPI = 64 / ALPR, AI = BP / ARPI / NW;     // dz: lanes per row, rows per instruction, instructions per wavefront
    constexpr int BI = PROWS / 8 / NW;                                      // panel: 8 rows of 128 bytes per instruction
    static_assert(BP % (ARPI * NW) == 0 && PROWS % (8 * NW) == 0, "a stage must split into whole 1 KB instructions per wavefront");
    static_assert((WP & (WP - 1)) == 0 && WP >= 2, "the pixel parts are added up in a binary tree");
    static_assert(SW == 0 || TAPS % SW == 0, "taps = filter rows x filter width");
    static_assert(BP * KT == 16 * NT, "the bias-gradient sums take 16 rows per thread");
    constexpr int STAGE = BP * KT + PROWS * CT + BP;                     // floats: dz rows, panel, row table
    // taps per round of the final tree: the writers' accumulators of one round must fit the two stages
    constexpr int RED_SLOTS = WK * WP / 2, TG_MAX = (2 * STAGE) / (RED_SLOTS * 16 * 64);
    constexpr int TG = TG_MAX < TAPS ? TG_MAX : TAPS;
    static_assert(TG >= 1, "LDS too small for the reduction tree");
    constexpr unsigned OOB = 0x80000000u;                                // a byte offset no descriptor here reaches
    constexpr int TABMAX = 1024;                                         // entries of each of the two loader tables

    __shared__ __attribute__((aligned(1024))) float lds[2 * STAGE];
    __shared__ unsigned xoff_tab[TABMAX];
    __shared__ int prow_tab[TABMAX];

    const Geom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int kb = wave / WP, part = wave % WP;
    const int wk0 = kb * 32, pbase = part * 32;

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
    //   prow_tab[pq],  pq < P*Q:    128 (bytes per panel row) times the padded position of output pixel pq's window corner.
    // A chunk touches at most two images (host-checked: BP <= P*Q and PROWS <= Hp*Wp), so a lane only has to
    // decide which of the two it is in: compare, conditional subtract, table read.
    const int IP = p.Hp * Wp, PQ = g.P * g.Q;
    for (int pos = tid; pos < IP; pos += NT) {
        const int hp = p.dWp.div(pos), wp = pos - hp * Wp, h = hp - g.ph, w = wp - g.pw;
        xoff_tab[pos] = ((unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W) ? (unsigned)((h * g.W + w) * g.C) * 4u : OOB;
    }
    for (int pq = tid; pq < PQ; pq += NT) {
        const int pp = g.dQ.div(pq), q = pq - pp * g.Q;
        prow_tab[pq] = (pp * Wp + q) * (CT * 4);
    }

    // ---- per-lane constants of the loaders.  Instruction i of this wavefront is number q = wave + NW*i of the
    // stage: dz instruction q covers rows ARPI*q .. of the chunk, panel instruction q rows 8q .. 8q+7.
    unsigned avoff[AI];                   // byte offset of this lane's piece inside the chunk's dz rows, or OOB
#pragma unroll
    for (int i = 0; i < AI; i++) {
        const int row = (wave + NW * i) * ARPI + lane / ALPR, k = k0 + (lane % ALPR) * 4;
        avoff[i] = k < g.K ? (unsigned)((row * g.K + k) * 4) : OOB;
    }
    const unsigned bcoff = c0 + (lane & 7) * 4 < g.C ? (unsigned)((c0 + (lane & 7) * 4) * 4) : OOB;   // this lane's piece inside a pixel
    const int brow_l = wave * 8 + (lane >> 3);                       // its panel row in instruction 0; instruction i: + 8*NW*i
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) float *)lds;
    const owt_i32x4 xrsrc = make_rsrc(p.b, (unsigned)g.N * g.H * g.W * g.C * 4u);
    const unsigned img_bytes = (unsigned)(g.H * g.W * g.C) * 4u;

    // All loads of chunk ch, into stage `stage`.  Nothing is waited for here.
    auto issue_chunk = [&](int ch, int stage) {
        // wavefront-uniform bookkeeping of the chunk (scalar unit)
        const int pix0 = ch * BP, lim = min(pix0 + BP, npix);
        const int n0 = g.dPQ.div(pix0), pq0 = pix0 - n0 * PQ;
        const int pp0 = g.dQ.div(pq0), q0 = pq0 - pp0 * g.Q;
        const int pos0 = (pp0 + r0) * Wp + q0;                    // first panel row's padded position in image n0
        const int nl = g.dPQ.div(lim - 1), pql = lim - 1 - nl * PQ;
        const int ppl = g.dQ.div(pql), ql = pql - ppl * g.Q;
        const int nrows = (nl - n0) * IP + (ppl + r0 + rows_g - 1) * Wp + ql + g.S - pos0;   // <= PROWS (host-checked)
        const unsigned img0 = (unsigned)n0 * img_bytes, img1 = n0 + 1 < g.N ? img0 + img_bytes : OOB;
        const unsigned sbase = lds_base + (unsigned)stage * (STAGE * 4);
        // dz rows pix0 .. pix0 + BP - 1: the descriptor starts at the chunk and ends with the tensor
        const owt_i32x4 arsrc = make_rsrc((const float *)p.a + (size_t)pix0 * g.K, (unsigned)(npix - pix0) * g.K * 4u);
#pragma unroll
        for (int i = 0; i < AI; i++) buffer_load16_to_lds(arsrc, avoff[i], sbase + (unsigned)(wave + NW * i) * 1024u);
        // panel row -> padded position in image n0 or n0 + 1 -> the pixel it shows, or none (padding, past the rows
        // this chunk needs, past the last image)
        unsigned bvoff[BI];
#pragma unroll
        for (int i = 0; i < BI; i++) {
            const int row = brow_l + 8 * NW * i, pos = pos0 + row;
            const unsigned t = xoff_tab[min((unsigned)pos, (unsigned)(pos - IP))];
            const unsigned pixoff = row < nrows ? t + (pos >= IP ? img1 : img0) : OOB;        // OOB + an image offset stays >= OOB
            bvoff[i] = __builtin_elementwise_add_sat(pixoff, bcoff);
        }
#pragma unroll
        for (int i = 0; i < BI; i++) buffer_load16_to_lds(xrsrc, bvoff[i], sbase + (unsigned)(BP * KT * 4) + (unsigned)(wave + NW * i) * 1024u);
        if (tid < BP) {       // byte offset of each pixel's panel row relative to the chunk's first
            const int pq = pq0 + tid;
            const int v = prow_tab[min((unsigned)pq, (unsigned)(pq - PQ))] + ((pq >= PQ ? IP : 0) + r0 * Wp - pos0) * (CT * 4);
            ((int *)(lds + stage * STAGE + BP * KT + PROWS * CT))[tid] = pix0 + tid < lim ? v : 0;
        }
    };

    float16v acc[TAPS];
#pragma unroll
    for (int t = 0; t < TAPS; t++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[t][r] = 0.f;
    float dbacc = 0.f;
    const bool do_db = ct == 0 && grp == 0 && p.dbias != nullptr;

    // Sixteen pixels (eight MFMA steps of two) of this wavefront's 32, from one LDS stage.  Two fragment sets
    // ping-pong so the LDS reads of the next pixel pair are issued before the MFMAs of the current one; a
    // pair's panel row is looked up one fetch ahead of its use.  Every address below is a per-lane base that
    // is set up once per call plus an immediate offset.
    auto compute16 = [&](int stage, int pfirst) {
        const float *dzs = lds + stage * STAGE, *panel = dzs + BP * KT;
        const int *tab = (const int *)(panel + PROWS * CT) + pfirst + lh;         // this lane's pixels: tab[2 * pair]
        const float *abase = dzs + (pfirst + lh) * KT + wk0 + li;                 // a of pair: abase[2 * pair * KT]
        const char *pbase_l = (const char *)(panel + li);
        auto fetch = [&](auto pair_c, int &prow, float &a, float (&bb)[TAPS]) {
            constexpr int pair = decltype(pair_c)::value;
            const float *pb = (const float *)(pbase_l + prow);
            a = abase[2 * pair * KT];
#pragma unroll
            for (int t = 0; t < TAPS; t++) {
                constexpr int sw = SW > 0 ? SW : 1;
                bb[t] = pb[(SW > 0 ? (t / sw) * WPC + t % sw : t) * CT];
            }
            prow = tab[2 * pair + 4 <= 14 ? 2 * pair + 4 : 14];
        };
        auto mma = [&](float a, const float (&bb)[TAPS]) {
#pragma unroll
            for (int t = 0; t < TAPS; t++) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bb[t], acc[t], 0, 0, 0);
        };
        float a0, a1, b0[TAPS], b1[TAPS];
        int prow0 = tab[0], prow1 = tab[2];
        fetch(std::integral_constant<int, 0>{}, prow0, a0, b0);
#define OWT_DF2_STEP(J)                                                                    \
        fetch(std::integral_constant<int, (J) + 1>{}, prow1, a1, b1);                      \
        __builtin_amdgcn_sched_barrier(0);                                                 \
        mma(a0, b0);                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                 \
        fetch(std::integral_constant<int, ((J) + 2 < 7 ? (J) + 2 : 7)>{}, prow0, a0, b0);  \
        __builtin_amdgcn_sched_barrier(0);                                                 \
        mma(a1, b1);                                                                       \
        __builtin_amdgcn_sched_barrier(0);
        OWT_DF2_STEP(0) OWT_DF2_STEP(2) OWT_DF2_STEP(4) OWT_DF2_STEP(6)
#undef OWT_DF2_STEP
    };

    __syncthreads();                                    // the loader tables are complete
    if (ch_beg < ch_end) issue_chunk(ch_beg, 0);

    int cur = 0;
    for (int ch = ch_beg; ch < ch_end; ch++) {
        // this lane's pieces of chunk ch have landed and its row-table entry is written; after the barrier that
        // holds for the whole work-group, and every wavefront is done reading the other stage (chunk ch - 1)
        __builtin_amdgcn_s_waitcnt(0x0070);             // vmcnt(0) lgkmcnt(0), expcnt untouched
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");                  // no LDS read of this stage moves above the barrier
        if (ch + 1 < ch_end) issue_chunk(ch + 1, cur ^ 1);
        compute16(cur, pbase);
        compute16(cur, pbase + 16);
        if (do_db) {          // bias gradient: column sums of the chunk's dz rows, 16 rows per thread
            const float *col = lds + cur * STAGE + (tid / KT) * 16 * KT + tid % KT;
#pragma unroll
            for (int j = 0; j < 16; j++) dbacc += col[j * KT];
        }
        cur ^= 1;
    }
    __syncthreads();                                    // every wavefront is done with the stages

    // ---- the WP pixel parts of a filter block add up through LDS: in every round the upper half of the
    // remaining parts writes TG taps at a time, the lower half adds.
#pragma unroll
    for (int stride = WP / 2; stride >= 1; stride >>= 1) {
#pragma unroll
        for (int t0 = 0; t0 < TAPS; t0 += TG) {
            if (part >= stride && part < 2 * stride) {
                float *red = lds + (size_t)(kb * stride + part - stride) * (TG * 16 * 64) + lane * 4;
#pragma unroll
                for (int t = t0; t < (t0 + TG < TAPS ? t0 + TG : TAPS); t++)
#pragma unroll
                    for (int r = 0; r < 16; r += 4)
                        *(float4 *)(red + ((t - t0) * 4 + r / 4) * 256) = make_float4(acc[t][r], acc[t][r + 1], acc[t][r + 2], acc[t][r + 3]);
            }
            __syncthreads();
            if (part < stride) {
                const float *red = lds + (size_t)(kb * stride + part) * (TG * 16 * 64) + lane * 4;
#pragma unroll
                for (int t = t0; t < (t0 + TG < TAPS ? t0 + TG : TAPS); t++)
#pragma unroll
                    for (int r = 0; r < 16; r += 4) {
                        const float4 v = *(const float4 *)(red + ((t - t0) * 4 + r / 4) * 256);
                        acc[t][r] += v.x; acc[t][r + 1] += v.y; acc[t][r + 2] += v.z; acc[t][r + 3] += v.w;
                    }
            }
            __syncthreads();
        }
    }

    // ---- epilogue: dw[k][tap][c]; accumulator register r of lane (li, lh) holds
    // filter k = 8*(r/4) + 4*lh + r%4 of the wavefront's 32, channel li.
    const bool parts = p.splits > 1;
    if (part == 0) {
        float *pout = parts ? p.partial + (size_t)split * p.M * p.Ncols : nullptr;
        float *out = (float *)p.out;
        const int c = c0 + li;
#pragma unroll
        for (int t = 0; t < TAPS; t++) {
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int k = k0 + wk0 + 8 * (r / 4) + 4 * lh + (r % 4);
                if (k >= g.K || c >= g.C) continue;
                const size_t o = ((size_t)k * RS + tap_first + t) * g.C + c;
                if (parts) pout[o] = acc[t][r];
                else out[o] = p.alpha * acc[t][r] + (p.beta != 0.f ? p.beta * out[o] : 0.f);
            }
        }
    }

    if (do_db) {   // uniform over the work-group; the tree above ended with a barrier
        float *red = lds;
        red[tid] = dbacc;                               // [row group][filter]
        __syncthreads();
        if (tid < KT && k0 + tid < g.K) {
            float s = 0.f;
            for (int j = 0; j < NT / KT; j++) s += red[j * KT + tid];
            const int k = k0 + tid;
            if (parts) p.dbias_partial[(size_t)split * p.M + k] = s;
            else p.dbias[k] = p.alpha * s + (p.beta != 0.f ? p.beta * p.dbias[k] : 0.f);
        }
    }
}

}  // namespace owt
