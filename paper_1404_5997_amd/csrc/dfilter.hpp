// Direct filter-gradient kernel for stride-1 "same" convolutions (P == H, Q == W), fp32 MFMA.
//
//   dw[k][r][s][c] = sum over pixels (n,p,q) of dz[n,p,q,k] * x[n, p+r-pad_h, q+s-pad_w, c]
//
// (Section 4 of the paper, backward step 2: the weight gradients of the
// data-parallel convolution layers.)  A gather-style GEMM re-reads dz for every
// 128 columns of (r,s,c) and x for every tap.  Here a work-group owns
// 32*WK filters x 32*WC channels x ALL taps of a tap group and walks over the
// pixels in chunks of 32: per chunk it loads the dz rows once and the x pixels
// those 32 positions touch once, into LDS, laid out in ZERO-PADDED image
// coordinates (Hp x Wp per image), where tap (r,s) of pixel (p,q) is simply
// row ppad(p,q) + r*Wp + s: no bounds checks in the inner loop.  Each wavefront
// keeps one 32 x 32 accumulator per tap (<= 9) and feeds all of them from one
// dz fragment.
//
// Tap groups: all R*S taps at once when R*S == TAPS, else one filter row per
// work-group when S == TAPS (the tap count is a compile-time constant so the
// inner loop is branch-free; other filter sizes use the gather kernel).  The pixel range is split over work-groups (numbered so that the tiles of a split share an L2); partial sums are
// reduced by splitk_reduce_kernel (deterministic, no atomics).
#pragma once
#include "igemm.hpp"

namespace owt {

// OCC = work-groups per CU the register budget is cut for.
// FAST (fp32 storage, chunks cut per image, one filter row per work-group; the launcher checks what it needs):
// the chunk loader and the fragment fetch are written for few vector-ALU instructions, which take MFMA time
// on this chip.  Loads go through buffer descriptors (what must read as zero gets an offset outside the
// descriptor), the position of a panel row in the image and of a pixel's window come from two LDS tables
// instead of divisions, and the taps of a filter row are immediate offsets from one address.
template <class T, int WK, int WC, int TAPS, int PRF, int OCC, bool FAST = false>
__global__ void __launch_bounds__(64 * WK * WC, OCC) dfilter_kernel(const GemmParams p)
{
    constexpr int NT = 64 * WK * WC, KT = 32 * WK, CT = 32 * WC, BP = 32;
    constexpr int PA = KT + 4, PB = CT + 4;
    constexpr int KQ = KT / 4, ARPP = NT / KQ, ANP = BP / ARPP;          // dz loader
    // x panel loader: a thread fetches LPT 16-byte pieces of one panel row (pieces bq, bq + TPR, ...), so the
    // row's position in the padded image is worked out once per LPT loads
    constexpr int CQ = CT / 4, LPT = 4, TPR = CQ / LPT, BRPP = NT / TPR, BNP = (PRF + BRPP - 1) / BRPP;
    static_assert(CQ % LPT == 0 && NT % TPR == 0, "panel rows must split evenly over the threads");
    static_assert(BP % ARPP == 0, "dz chunk must split evenly over the threads");

    __shared__ __attribute__((aligned(16))) float dzs[BP * PA];
    __shared__ __attribute__((aligned(16))) float panel[PRF * PB];
    __shared__ int prow_tab[BP];
    constexpr int XTAB = FAST ? 1152 : 1, QTAB = FAST ? 1024 : 1;
    __shared__ unsigned xoff_tab[XTAB];      // padded position in an image -> byte offset of the pixel it shows, or OOB
    __shared__ int win_tab[QTAB];            // output pixel of an image -> padded position of its window's corner
    constexpr unsigned OOB = 0x80000000u;

    const Geom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int wk0 = (wave / WC) * 32, wc0 = (wave % WC) * 32;

    int logical, split;
    if (!owt_split_major_wg(p.tiles_m * p.tiles_n, p.splits, logical, split)) return;
    const int kt = logical / p.tiles_n, rem = logical - kt * p.tiles_n;
    const int grp = rem / p.ctiles, ct = rem - grp * p.ctiles;
    const int k0 = kt * KT, c0 = ct * CT;
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

    const T *dzsrc = (const T *)p.a, *xsrc = (const T *)p.b, *mask = (const T *)p.mask;
    const int akq = tid % KQ, arow0 = tid / KQ;
    const int bq = tid % TPR, brow0 = tid / TPR;
    float4 areg[ANP], breg[BNP][LPT];
    int tab_next = 0;
    const int pad_pix_total = g.N * p.Hp * Wp;

    // Pixels [pix0, lim) of chunk ch.  With p.cpi the chunks are cut per image (the last chunk of an image is
    // short), so a chunk never spans the padding rows between two images and its panel stays small.
    auto chunk_range = [&](int ch, int &pix0, int &lim) {
        if (p.cpi) {
            const int n = p.dCpi.div(ch), cw = ch - n * p.cpi;
            pix0 = n * g.P * g.Q + cw * BP;
            lim = min(pix0 + BP, (n + 1) * g.P * g.Q);
        } else {
            pix0 = ch * BP;
            lim = min(pix0 + BP, npix);
        }
    };
    // ---- FAST loader state: per-thread constant offsets, descriptors
    unsigned avoff[ANP], bcoff[LPT];
    __amdgpu_buffer_rsrc_t xrsrc = owt_make_rsrc(p.b, 0);
    if constexpr (FAST) {
        const int IPt = p.Hp * Wp, PQt = g.P * g.Q;
        for (int pos = tid; pos < XTAB; pos += NT) {
            const int hp = p.dWp.div(pos), wp = pos - hp * Wp, h = hp - g.ph, w = wp - g.pw;
            xoff_tab[pos] = (pos < IPt && (unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W)
                                ? (unsigned)((h * g.W + w) * g.C) * 4u : OOB;
        }
        for (int pq = tid; pq < PQt; pq += NT) {
            const int pp = g.dQ.div(pq), q = pq - pp * g.Q;
            win_tab[pq] = pp * Wp + q;
        }
#pragma unroll
        for (int i = 0; i < ANP; i++)
            avoff[i] = k0 + akq * 4 < g.K ? (unsigned)(((arow0 + i * ARPP) * g.K + k0 + akq * 4) * 4) : OOB;
#pragma unroll
        for (int j = 0; j < LPT; j++)
            bcoff[j] = c0 + (bq + j * TPR) * 4 < g.C ? (unsigned)((c0 + (bq + j * TPR) * 4) * 4) : OOB;
        xrsrc = owt_make_rsrc(p.b, (unsigned)g.N * g.H * g.W * g.C * 4u);
        __syncthreads();
    }
    auto load_chunk_fast = [&](int ch) {
        // chunk ch = pixels [pq0, pql] of image n (uniform, scalar unit)
        const int n = p.dCpi.div(ch), pq0 = (ch - n * p.cpi) * BP, PQt = g.P * g.Q, pql = min(pq0 + BP, PQt) - 1;
        const int pp0 = g.dQ.div(pq0), ppl = g.dQ.div(pql);
        const int pos0 = (pp0 + r0) * Wp + (pq0 - pp0 * g.Q);                               // first panel row: padded position in the image
        const int nrows = (ppl + r0 + rows_g - 1) * Wp + (pql - ppl * g.Q) + g.S - pos0;     // <= PRF (host-checked)
        const __amdgpu_buffer_rsrc_t arsrc =
            owt_make_rsrc(dzsrc + (size_t)(n * PQt + pq0) * g.K, (unsigned)(pql + 1 - pq0) * g.K * 4u);   // ends with the chunk
        const unsigned img = (unsigned)n * (unsigned)(g.H * g.W * g.C) * 4u;
#pragma unroll
        for (int i = 0; i < ANP; i++) areg[i] = buffer_load4(arsrc, avoff[i]);
#pragma unroll
        for (int i = 0; i < BNP; i++) {
            const int row = brow0 + i * BRPP;
            const unsigned t = xoff_tab[min(pos0 + row, XTAB - 1)];
            const unsigned pixoff = row < nrows ? t + img : OOB;               // OOB + an image offset stays >= OOB
#pragma unroll
            for (int j = 0; j < LPT; j++) breg[i][j] = buffer_load4(xrsrc, __builtin_elementwise_add_sat(pixoff, bcoff[j]));
        }
        if (tid < BP) tab_next = pq0 + tid <= pql ? win_tab[pq0 + tid] + r0 * Wp - pos0 : 0;
    };
    auto load_chunk = [&](int ch) {
        if constexpr (FAST) { load_chunk_fast(ch); return; }
        int pix0, lim;
        chunk_range(ch, pix0, lim);
        const int ps = ppad(pix0) + r0 * Wp;
        const int nrows = ppad(lim - 1) + (r0 + rows_g - 1) * Wp + g.S - ps;   // <= PRF (host-checked)
#pragma unroll
        for (int i = 0; i < ANP; i++) {
            const int pix = pix0 + arow0 + i * ARPP, k = k0 + akq * 4;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (pix < lim && k < g.K) {
                const int off = pix * g.K + k;
                v = load4(dzsrc, off);
                if (mask) {
                    const float4 y = load4(mask, off);
                    v.x = y.x > 0.f ? v.x : 0.f; v.y = y.y > 0.f ? v.y : 0.f;
                    v.z = y.z > 0.f ? v.z : 0.f; v.w = y.w > 0.f ? v.w : 0.f;
                }
            }
            areg[i] = v;
        }
#pragma unroll
        for (int i = 0; i < BNP; i++) {
            const int row = brow0 + i * BRPP, idx = ps + row;
            int off = -1;
            if (row < nrows && idx < pad_pix_total) {
                const int n = p.dHpWp.div(idx), r2 = idx - n * p.Hp * Wp;
                const int hp = p.dWp.div(r2), wp = r2 - hp * Wp;
                const int h = hp - g.ph, w = wp - g.pw;
                if ((unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W)
                    off = ((n * g.H + h) * g.W + w) * g.C + c0 + bq * 4;
            }
#pragma unroll
            for (int j = 0; j < LPT; j++) {
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (off >= 0 && c0 + (bq + j * TPR) * 4 < g.C) v = load4(xsrc, off + j * TPR * 4);
                breg[i][j] = v;
            }
        }
        if (tid < BP) {
            const int pix = pix0 + tid;
            tab_next = pix < lim ? ppad(pix) + r0 * Wp - ps : 0;
        }
    };
    auto store_chunk = [&]() {
#pragma unroll
        for (int i = 0; i < ANP; i++)
            *(float4 *)(dzs + (arow0 + i * ARPP) * PA + akq * 4) = areg[i];
#pragma unroll
        for (int i = 0; i < BNP; i++) {
            const int row = brow0 + i * BRPP;
            if (row < PRF) {
#pragma unroll
                for (int j = 0; j < LPT; j++) *(float4 *)(panel + row * PB + (bq + j * TPR) * 4) = breg[i][j];
            }
        }
        if (tid < BP) prow_tab[tid] = tab_next;
    };

    float16v acc[TAPS];
#pragma unroll
    for (int t = 0; t < TAPS; t++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[t][r] = 0.f;
    int toff[TAPS];
#pragma unroll
    for (int t = 0; t < TAPS; t++) {
        const int r = p.groups > 1 ? 0 : t / g.S, s = p.groups > 1 ? t : t - (t / g.S) * g.S;
        toff[t] = (r * Wp + s) * PB + wc0 + li;
    }

    float4 dbacc = make_float4(0.f, 0.f, 0.f, 0.f);
    const bool do_db = ct == 0 && grp == 0 && p.dbias != nullptr;

    if (ch_beg < ch_end) { load_chunk(ch_beg); store_chunk(); }
    __syncthreads();

    for (int ch = ch_beg; ch < ch_end; ch++) {
        if (do_db) {
#pragma unroll
            for (int i = 0; i < ANP; i++) {
                dbacc.x += areg[i].x; dbacc.y += areg[i].y; dbacc.z += areg[i].z; dbacc.w += areg[i].w;
            }
        }
        const bool more = ch + 1 < ch_end;
        if (more) load_chunk(ch + 1);
        // Two fragment sets ping-pong so the LDS reads of the next pixel pair are issued before the
        // MFMAs of the current one; a pair's panel row is looked up one fetch ahead of its use.
        auto fetch = [&](int pair, int &prow, float &a, float (&b)[TAPS]) {
            const int pix = 2 * pair + lh;
            const int base = prow * PB;
            a = dzs[pix * PA + wk0 + li];
            if constexpr (FAST) {            // one filter row: tap t is t pixels to the right of tap 0
                const float *pb = panel + base + wc0 + li;
#pragma unroll
                for (int t = 0; t < TAPS; t++) b[t] = pb[t * PB];
            } else {
#pragma unroll
                for (int t = 0; t < TAPS; t++) b[t] = panel[base + toff[t]];
            }
            prow = prow_tab[min(pix + 4, BP - 1)];
        };
        auto mma = [&](float a, const float (&b)[TAPS]) {
#pragma unroll
            for (int t = 0; t < TAPS; t++) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b[t], acc[t], 0, 0, 0);
        };
        float a0, a1, b0[TAPS], b1[TAPS];
        int prow0 = prow_tab[lh], prow1 = prow_tab[2 + lh];
        fetch(0, prow0, a0, b0);
#pragma unroll
        for (int j = 0; j < BP / 2; j += 2) {
            fetch(j + 1, prow1, a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            mma(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            fetch(min(j + 2, BP / 2 - 1), prow0, a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            mma(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
        if (more) store_chunk();
        __syncthreads();
    }

    // ---- epilogue: dw[k][tap][c]; accumulator register r of lane (li, lh) holds
    // filter k = 8*(r/4) + 4*lh + r%4 of the wavefront's 32, channel li.
    const bool part = p.splits > 1;
    float *pout = part ? p.partial + (size_t)split * p.M * p.Ncols : nullptr;
    float *out = (float *)p.out;
    const int c = c0 + wc0 + li;
#pragma unroll
    for (int t = 0; t < TAPS; t++) {
#pragma unroll
        for (int r = 0; r < 16; r++) {
            const int k = k0 + wk0 + 8 * (r / 4) + 4 * lh + (r % 4);
            if (k >= g.K || c >= g.C) continue;
            const size_t o = ((size_t)k * RS + tap_first + t) * g.C + c;
            if (part) pout[o] = acc[t][r];
            else out[o] = p.alpha * acc[t][r] + (p.beta != 0.f ? p.beta * out[o] : 0.f);
        }
    }

    if (do_db) {   // uniform over the work-group; every wave has passed the loop's last barrier
        float *red = panel;
        *(float4 *)(red + arow0 * KT + akq * 4) = dbacc;
        __syncthreads();
        if (tid < KT && k0 + tid < g.K) {
            float s = 0.f;
            for (int j = 0; j < ARPP; j++) s += red[j * KT + tid];
            const int k = k0 + tid;
            if (part) p.dbias_partial[(size_t)split * p.M + k] = s;
            else p.dbias[k] = p.alpha * s + (p.beta != 0.f ? p.beta * p.dbias[k] : 0.f);
        }
    }
}

}  // namespace owt
