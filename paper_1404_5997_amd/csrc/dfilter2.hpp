// Direct filter-gradient kernel for stride-1 "same" convolutions (P == H, Q == W), fp32 storage and
// fp32 MFMA, with the pixel reduction split INSIDE the work-group and as few vector-ALU instructions
// per MFMA as the data layout allows.
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
// splits of the pixel range across work-groups, shrink WP times.  LDS is double buffered: one barrier
// per chunk.
//
// Vector-ALU instructions.  In-kernel cycle counters showed that on this chip the fp32 MFMA does not run
// beside vector-ALU work of the same SIMD, whichever wavefront issues it: a wavefront's address
// arithmetic took three times as long while the SIMD's other wavefront was in its MFMA phase, and a
// chunk took the MFMA time plus the vector-ALU time of both wavefronts whatever the order of their
// phases.  So every vector instruction in the chunk loop costs matrix time, and the loop is written to
// have almost none:
//  * the padded row width WPC and the filter width SW are template parameters, so the LDS address of
//    tap (r,s) is one per-pixel base (read from a table of byte offsets) plus an immediate offset;
//  * what the loaders need to know about a chunk (which pixel a panel row shows, where a pixel's panel row
//    is) comes from two small LDS tables instead of divisions;
//  * global loads are buffer loads: a thread's offsets into the dz chunk are constants, the chunk's
//    base goes into the buffer descriptor (scalar arithmetic), and whatever must read as zero (rows past
//    the end of the tensor, filters or channels past the end of a ragged tile, padding pixels) gets an
//    offset beyond the descriptor's range, which the hardware turns into zeros without touching memory.
#pragma once
#include <type_traits>

#include "igemm.hpp"

namespace owt {

typedef unsigned int owt_u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float4 buffer_load4(__amdgpu_buffer_rsrc_t rsrc, unsigned voffset_bytes)
{
    const owt_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voffset_bytes, 0, 0);
    return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}

// SW > 0: all R x SW taps in one work-group (TAPS == R*SW), padded rows WPC pixels wide.
// SW == 0: one filter row of TAPS taps per work-group (any row width).
template <int WK, int WP, int TAPS, int SW, int WPC, int PRF, bool MASKED>
__global__ void __launch_bounds__(64 * WK * WP, 1) dfilter2_kernel(const GemmParams p)
{
    constexpr int NT = 64 * WK * WP, KT = 32 * WK, CT = 32, BP = 32 * WP;
    constexpr int PA = KT + 4, PB = CT + 4;
    constexpr int KQ = KT / 4, ARPP = NT / KQ, ANP = BP / ARPP;          // dz loader
    // x panel loader: a thread fetches the LPT 16-byte pieces bq, bq + TPR, ... of one panel row
    constexpr int CQ = CT / 4, LPT = 4, TPR = CQ / LPT, BRPP = NT / TPR, BNP = (PRF + BRPP - 1) / BRPP;
    static_assert(CQ % LPT == 0 && NT % TPR == 0, "panel rows must split evenly over the threads");
    static_assert(BP % ARPP == 0 && NT % KQ == 0, "dz chunk must split evenly over the threads");
    static_assert((WP & (WP - 1)) == 0 && WP >= 2, "the pixel parts are added up in a binary tree");
    static_assert(SW == 0 || TAPS % SW == 0, "taps = filter rows x filter width");
    constexpr int STAGE = BP * PA + PRF * PB + BP;                       // floats: dz rows, panel, row table
    // taps per round of the final tree: the writers' accumulators of one round must fit the two stages
    constexpr int RED_SLOTS = WK * WP / 2, TG_MAX = (2 * STAGE) / (RED_SLOTS * 16 * 64);
    constexpr int TG = TG_MAX < TAPS ? TG_MAX : TAPS;
    static_assert(TG >= 1, "LDS too small for the reduction tree");
    static_assert(ARPP * KT <= 2 * STAGE, "LDS too small for the bias-gradient sums");
    constexpr unsigned OOB = 0x80000000u;                                // a byte offset no descriptor here reaches
    constexpr int TABMAX = 1024;                                         // entries of each of the two loader tables

    __shared__ __attribute__((aligned(16))) float lds[2 * STAGE];

    const Geom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int kb = wave / WP, part = wave % WP;
    const int wk0 = kb * 32, pbase = part * 32;

    const int ntiles = p.tiles_m * p.tiles_n;
    const int b = blockIdx.x, xcd = b & 7;
    const int logical = xcd * (ntiles >> 3) + min(xcd, ntiles & 7) + (b >> 3);
    const int kt = logical / p.tiles_n, rem = logical - kt * p.tiles_n;
    const int grp = rem / p.ctiles, ct = rem - grp * p.ctiles;
    const int k0 = kt * KT, c0 = ct * CT;
    const int split = blockIdx.y;
    const int ch_beg = split * p.ksteps_per_split, ch_end = min(p.ksteps, ch_beg + p.ksteps_per_split);

    const int RS = g.R * g.S, Wp = p.Wp, npix = p.Kd;
    const int r0 = p.groups > 1 ? grp : 0, rows_g = p.groups > 1 ? 1 : g.R;
    const int tap_first = p.groups > 1 ? grp * g.S : 0;

    // padded linear index of the window's top-left corner of pixel pix
    auto ppad = [&](int pix) {
        const int n = g.dPQ.div(pix), pq = pix - n * g.P * g.Q;
        const int pp = g.dQ.div(pq), q = pq - pp * g.Q;
        return (n * p.Hp + pp) * Wp + q;
    };

    // ---- loaders.  Two tables in LDS, filled once, replace the per-chunk divisions (integer multiplies run at
    // a quarter of the vector rate, and vector instructions cost matrix time here):
    //   xoff_tab[pos], pos < Hp*Wp: byte offset inside an image of the pixel that padded position pos shows, or OOB;
    //   prow_tab[pq],  pq < P*Q:    PB*4 times the padded position of output pixel pq's window corner.
    // A chunk touches at most two images (host-checked: BP <= P*Q and PRF <= Hp*Wp), so a thread only has to
    // decide which of the two it is in: compare, conditional subtract, table read.
    __shared__ unsigned xoff_tab[TABMAX];
    __shared__ int prow_tab[TABMAX];
    const int IP = p.Hp * Wp, PQ = g.P * g.Q;
    for (int pos = threadIdx.x; pos < IP; pos += NT) {
        const int hp = p.dWp.div(pos), wp = pos - hp * Wp, h = hp - g.ph, w = wp - g.pw;
        xoff_tab[pos] = ((unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W) ? (unsigned)((h * g.W + w) * g.C) * 4u : OOB;
    }
    for (int pq = threadIdx.x; pq < PQ; pq += NT) {
        const int pp = g.dQ.div(pq), q = pq - pp * g.Q;
        prow_tab[pq] = (pp * Wp + q) * (PB * 4);
    }
    __syncthreads();
    // Per-thread constants: byte offsets of the thread's ANP pieces inside a dz chunk, the panel pieces it owns,
    // and which of its pieces exist at all (ragged last filter / channel tile).
    const int akq = tid % KQ, arow0 = tid / KQ;
    const int bq = tid % TPR, brow0 = tid / TPR;
    unsigned avoff[ANP];
#pragma unroll
    for (int i = 0; i < ANP; i++)
        avoff[i] = k0 + akq * 4 < g.K ? (unsigned)(((arow0 + i * ARPP) * g.K + k0 + akq * 4) * 4) : OOB;
    unsigned bpiece[LPT];                 // byte offset of piece j inside the pixel, or OOB
#pragma unroll
    for (int j = 0; j < LPT; j++) bpiece[j] = c0 + (bq + j * TPR) * 4 < g.C ? (unsigned)((c0 + (bq + j * TPR) * 4) * 4) : OOB;
    const bool c_full = c0 + CT <= g.C;   // uniform: every piece of the channel tile exists
    const __amdgpu_buffer_rsrc_t xrsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.b, 0, (int)((unsigned)g.N * g.H * g.W * g.C * 4u), 0x00020000);
    const unsigned img_bytes = (unsigned)(g.H * g.W * g.C) * 4u;

    float4 areg[ANP], breg[BNP][LPT];
    int tab_next = 0;

    auto load_chunk = [&](int ch) {
        // wavefront-uniform bookkeeping of the chunk (scalar unit)
        const int pix0 = ch * BP, lim = min(pix0 + BP, npix);
        const int n0 = g.dPQ.div(pix0), pq0 = pix0 - n0 * PQ;
        const int pp0 = g.dQ.div(pq0), q0 = pq0 - pp0 * g.Q;
        const int pos0 = (pp0 + r0) * Wp + q0;                    // first panel row's padded position in image n0
        const int nl = g.dPQ.div(lim - 1), pql = lim - 1 - nl * PQ;
        const int ppl = g.dQ.div(pql), ql = pql - ppl * g.Q;
        const int nrows = (nl - n0) * IP + (ppl + r0 + rows_g - 1) * Wp + ql + g.S - pos0;   // <= PRF (host-checked)
        const unsigned img0 = (unsigned)n0 * img_bytes, img1 = n0 + 1 < g.N ? img0 + img_bytes : OOB;
        // dz rows pix0 .. pix0 + BP - 1: the descriptor starts at the chunk and ends with the tensor
        const unsigned left = (unsigned)(npix - pix0) * g.K * 4u;
        const __amdgpu_buffer_rsrc_t arsrc =
            __builtin_amdgcn_make_buffer_rsrc((void *)((const float *)p.a + (size_t)pix0 * g.K), 0, (int)left, 0x00020000);
#pragma unroll
        for (int i = 0; i < ANP; i++) areg[i] = buffer_load4(arsrc, avoff[i]);
        if constexpr (MASKED) {           // dz = dy * [y > 0]: applied on arrival (this variant waits for its loads here)
            const __amdgpu_buffer_rsrc_t mrsrc =
                __builtin_amdgcn_make_buffer_rsrc((void *)((const float *)p.mask + (size_t)pix0 * g.K), 0, (int)left, 0x00020000);
#pragma unroll
            for (int i = 0; i < ANP; i++) {
                const float4 y = buffer_load4(mrsrc, avoff[i]);
                areg[i].x = y.x > 0.f ? areg[i].x : 0.f; areg[i].y = y.y > 0.f ? areg[i].y : 0.f;
                areg[i].z = y.z > 0.f ? areg[i].z : 0.f; areg[i].w = y.w > 0.f ? areg[i].w : 0.f;
            }
        }
#pragma unroll
        for (int i = 0; i < BNP; i++) {
            // panel row -> padded position in image n0 or n0 + 1 -> the pixel it shows, or none (padding, past the
            // rows this chunk needs, past the last image)
            const int row = brow0 + i * BRPP, pos = pos0 + row;
            const bool second = pos >= IP;
            const unsigned t = xoff_tab[min((unsigned)pos, (unsigned)(pos - IP))];
            const unsigned pixoff = row < nrows ? t + (second ? img1 : img0) : OOB;      // OOB + anything stays >= OOB
            if (c_full) {
                const unsigned v0 = pixoff + (unsigned)((c0 + bq * 4) * 4);
#pragma unroll
                for (int j = 0; j < LPT; j++) breg[i][j] = buffer_load4(xrsrc, v0 + j * TPR * 16);
            } else {
#pragma unroll
                for (int j = 0; j < LPT; j++) breg[i][j] = buffer_load4(xrsrc, (pixoff | bpiece[j]) >= OOB ? OOB : pixoff + bpiece[j]);
            }
        }
        if (tid < BP) {       // byte offset of each pixel's panel row relative to the chunk's first
            const int pq = pq0 + tid;
            const bool second = pq >= PQ;
            const int v = prow_tab[min((unsigned)pq, (unsigned)(pq - PQ))] + ((second ? IP : 0) + r0 * Wp - pos0) * (PB * 4);
            tab_next = pix0 + tid < lim ? v : 0;
        }
    };
    float4 dbacc = make_float4(0.f, 0.f, 0.f, 0.f);
    const bool do_db = ct == 0 && grp == 0 && p.dbias != nullptr;
    auto store_chunk = [&](int stage) {
        float *dzs = lds + stage * STAGE, *panel = dzs + BP * PA;
        int *tab = (int *)(panel + PRF * PB);
#pragma unroll
        for (int i = 0; i < ANP; i++)
            *(float4 *)(dzs + (arow0 + i * ARPP) * PA + akq * 4) = areg[i];
        if (do_db) {
#pragma unroll
            for (int i = 0; i < ANP; i++) {
                dbacc.x += areg[i].x; dbacc.y += areg[i].y; dbacc.z += areg[i].z; dbacc.w += areg[i].w;
            }
        }
#pragma unroll
        for (int i = 0; i < BNP; i++) {
            const int row = brow0 + i * BRPP;
            if (BNP * BRPP <= PRF || row < PRF) {
#pragma unroll
                for (int j = 0; j < LPT; j++) *(float4 *)(panel + row * PB + (bq + j * TPR) * 4) = breg[i][j];
            }
        }
        if (tid < BP) tab[tid] = tab_next;
    };

    float16v acc[TAPS];
#pragma unroll
    for (int t = 0; t < TAPS; t++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[t][r] = 0.f;

    // Sixteen pixels (eight MFMA steps of two) of this wavefront's 32, from one LDS stage.  Two fragment sets
    // ping-pong so the LDS reads of the next pixel pair are issued before the MFMAs of the current one; a
    // pair's panel row is looked up one fetch ahead of its use.  Every address below is a per-lane base that
    // is set up once per call plus an immediate offset.
    auto compute16 = [&](int stage, int pfirst) {
        const float *dzs = lds + stage * STAGE, *panel = dzs + BP * PA;
        const int *tab = (const int *)(panel + PRF * PB) + pfirst + lh;           // this lane's pixels: tab[2 * pair]
        const float *abase = dzs + (pfirst + lh) * PA + wk0 + li;                 // a of pair: abase[2 * pair * PA]
        const char *pbase_l = (const char *)(panel + li);
        auto fetch = [&](auto pair_c, int &prow, float &a, float (&bb)[TAPS]) {
            constexpr int pair = decltype(pair_c)::value;
            const float *pb = (const float *)(pbase_l + prow);
            a = abase[2 * pair * PA];
#pragma unroll
            for (int t = 0; t < TAPS; t++) {
                constexpr int sw = SW > 0 ? SW : 1;
                bb[t] = pb[(SW > 0 ? (t / sw) * WPC + t % sw : t) * PB];
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

    if (ch_beg < ch_end) { load_chunk(ch_beg); store_chunk(0); }
    __syncthreads();

    int cur = 0;
    for (int ch = ch_beg; ch < ch_end; ch++) {
        const bool more = ch + 1 < ch_end;
        if (more) load_chunk(ch + 1);
        compute16(cur, pbase);
        // the other stage was last read before the barrier that ended the previous chunk
        if (more) store_chunk(cur ^ 1);
        compute16(cur, pbase + 16);
        __syncthreads();
        cur ^= 1;
    }

    // ---- the WP pixel parts of a filter block add up through LDS: in every round the upper half of the
    // remaining parts writes TG taps at a time, the lower half adds.  (All stage memory is free: every
    // wavefront has passed the loop's last barrier.)
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
        *(float4 *)(red + arow0 * KT + akq * 4) = dbacc;
        __syncthreads();
        if (tid < KT && k0 + tid < g.K) {
            float s = 0.f;
            for (int j = 0; j < ARPP; j++) s += red[j * KT + tid];
            const int k = k0 + tid;
            if (parts) p.dbias_partial[(size_t)split * p.M + k] = s;
            else p.dbias[k] = p.alpha * s + (p.beta != 0.f ? p.beta * p.dbias[k] : 0.f);
        }
    }
}

}  // namespace owt
