// Direct stride-1 convolution on fp32 MFMA with the activation panel resident in LDS.
//
// Used for the forward and backward-data passes of stride-1 layers (Section 4 of
// the paper, forward step 2 / backward step 2; four of the five layers of the
// Section 5 model).  An im2col-style gather re-reads every activation R*S times
// from L2; here a work-group loads the pixels its 64*WM output rows touch ONCE per
// 32-channel chunk into LDS (its rows plus a halo of (R-1)*Wi + S-1 pixels) and
// every filter tap reads its MFMA fragments from that panel at a shifted row.
// Only the filter slice of the current (chunk, tap) is streamed, double buffered.
//
//   out[m][n] = sum_{chunk} sum_{tap=(r,s)} sum_{c in chunk} in[pix(m) + r*Wi + s][c] * wt[tap][c][n]
//
// forward:  in = x,            wt[tap][c][k] = w[k][r][s][c]          (filter slice K-major)
// bwd-data: in = dy*[y > 0],   wt[tap][k][c] = w[k][R-1-r][S-1-s][c]  (filter slice N-major)
//           with the top-left offset pah = R-1-pad_h, paw = S-1-pad_w.
//
// Linear pixel index pin(m) = n*Hi*Wi + (ho-pah)*Wi + (wo-paw) grows with m when
// Ho <= Hi and Wo <= Wi, so the pixels of a row tile form one contiguous range;
// taps that fall outside the image read a row of zeros instead.
#pragma once
#include <type_traits>

#include "igemm.hpp"

namespace owt {

// MB = 32-row MFMA blocks per wavefront along M (2: 64 x 64 per wavefront; 1: 32 x 64, twice the
// wavefronts for the same tile, for layers too small to fill the chip otherwise).
// OCC = work-groups the register budget is cut for per CU (waves per SIMD when a work-group has four).
template <class T, class Epi, bool BWD, int WM, int WN, int PR, int BK, int MB, int OCC = 2>
__global__ void __launch_bounds__(64 * WM * WN, OCC) dconv_kernel(const GemmParams p)
{
    constexpr int NT = 64 * WM * WN, BM = 32 * MB * WM, BN = 64 * WN, PITCH = BK + 4;
    constexpr bool BKM = !BWD;                                   // filter slice K-major in forward
    constexpr int BPITCH = BKM ? PITCH : BN + 4;
    constexpr int BT = BKM ? BN * PITCH : BK * BPITCH;           // floats per filter-slice buffer
    constexpr int BQUADS = BKM ? BK / 4 : BN / 4;                // float4 per line of the slice
    constexpr int BLINES = BKM ? BN : BK;
    constexpr int BRPP = NT / BQUADS;
    constexpr int BNP = (BLINES + BRPP - 1) / BRPP;
    constexpr int PRPP = NT / (BK / 4);                          // panel rows per load pass
    constexpr int PNP = (PR + PRPP - 1) / PRPP;
    static_assert(NT % BQUADS == 0 && BLINES % BRPP == 0, "filter slice must split evenly over the threads");

    __shared__ __attribute__((aligned(16))) float lds[2 * BT + (PR + 1) * PITCH];
    float *panel = lds + 2 * BT;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int wm0 = (wave / WN) * 32 * MB, wn0 = (wave % WN) * 64;

    const int ntiles = p.tiles_m * p.tiles_n;
    const int b = blockIdx.x, xcd = b & 7;
    const int logical = xcd * (ntiles >> 3) + min(xcd, ntiles & 7) + (b >> 3);
    const int tm = logical / p.tiles_n, tn = logical - tm * p.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const int split = blockIdx.y;
    const int ch_beg = split * p.ksteps_per_split;               // here a "k step" is a BK-channel chunk
    const int ch_end = min(p.ksteps, ch_beg + p.ksteps_per_split);

    const int R = p.g.R, S = p.g.S, RS = R * S, Hi = p.Hi, Wi = p.Wi, Cred = p.Cred;
    const int HoWo = p.Ho * p.Wo, npix_in = p.g.N * Hi * Wi;

    // first input pixel of the tile's first row and of its last row
    auto pin = [&](int m, int &hh, int &ww) {
        const int n = p.dHoWo.div(m), rem = m - n * HoWo;
        const int ho = p.dWo.div(rem), wo = rem - ho * p.Wo;
        hh = ho - p.pah; ww = wo - p.paw;
        return n * Hi * Wi + hh * Wi + ww;
    };
    int th, tw;
    const int ps = pin(m0, th, tw);
    const int nrows = pin(min(m0 + BM, p.M) - 1, th, tw) + (R - 1) * Wi + S - ps;   // <= PR (host-checked)

    // rows this lane feeds to the MFMA
    int hh[MB], ww[MB], prow[MB];
#pragma unroll
    for (int bm = 0; bm < MB; bm++) {
        const int m = m0 + wm0 + bm * 32 + li;
        if (m < p.M) prow[bm] = pin(m, hh[bm], ww[bm]) - ps;
        else { hh[bm] = kInvalidLo; ww[bm] = 0; prow[bm] = 0; }
    }

    const T *in = (const T *)p.a, *wsrc = (const T *)p.b, *mask = (const T *)p.mask;
    const int pquad = tid % (BK / 4), prow0 = tid / (BK / 4);
    const int bquad = tid % BQUADS, bline0 = tid / BQUADS;
    float4 preg[PNP], breg[BNP];

    // fp32 storage with whole chunks (Cred a multiple of BK; tensors under 2 GiB): loads go through buffer
    // descriptors.  What must read as zero gets an offset outside the descriptor (panel rows past the tile's
    // range or outside the tensor, filters past the last one), so a load costs one vector add for its address
    // and nothing else: on this chip vector-ALU work and fp32 MFMAs of a SIMD do not overlap.
    constexpr unsigned OOB = 0x80000000u;
    const bool fast = std::is_same<T, float>::value && Cred % BK == 0 &&
                      (size_t)npix_in * Cred * 4 < OOB && (size_t)p.g.K * RS * p.g.C * 4 < OOB;
    const __amdgpu_buffer_rsrc_t in_rsrc = owt_make_rsrc(p.a, (unsigned)npix_in * Cred * 4u);
    const __amdgpu_buffer_rsrc_t mask_rsrc = owt_make_rsrc(p.mask ? p.mask : p.a, (unsigned)npix_in * Cred * 4u);
    const __amdgpu_buffer_rsrc_t w_rsrc = owt_make_rsrc(p.b, (unsigned)p.g.K * RS * p.g.C * 4u);
    unsigned pvoff[PNP], bvoff[BNP];          // per-thread constants: byte offset inside the panel / the filter slice, or OOB
#pragma unroll
    for (int i = 0; i < PNP; i++) {
        const int row = prow0 + i * PRPP;
        pvoff[i] = row < nrows ? (unsigned)((row * Cred + pquad * 4) * 4) : OOB;
    }
#pragma unroll
    for (int i = 0; i < BNP; i++) {
        const int line = bline0 + i * BRPP;
        if (BKM) bvoff[i] = n0 + line < p.Ncols ? (unsigned)((((n0 + line) * RS) * Cred + bquad * 4) * 4) : OOB;
        else bvoff[i] = n0 + bquad * 4 < p.Ncols ? (unsigned)(((line * RS) * p.Ncols + n0 + bquad * 4) * 4) : OOB;
    }

    auto load_panel = [&](int ch) {
        if (fast) {
            // rows of pixels before the tensor's first wrap to offsets near 2^32: outside the descriptor as well
            const unsigned base = (unsigned)((ps * Cred + ch * BK) * 4);
#pragma unroll
            for (int i = 0; i < PNP; i++) {
                const unsigned vo = pvoff[i] >= OOB ? OOB : pvoff[i] + base;
                float4 v = buffer_load4(in_rsrc, vo);
                if (BWD && mask) {
                    const float4 y = buffer_load4(mask_rsrc, vo);
                    v.x = y.x > 0.f ? v.x : 0.f; v.y = y.y > 0.f ? v.y : 0.f;
                    v.z = y.z > 0.f ? v.z : 0.f; v.w = y.w > 0.f ? v.w : 0.f;
                }
                preg[i] = v;
            }
            return;
        }
        const int c = ch * BK + pquad * 4;
#pragma unroll
        for (int i = 0; i < PNP; i++) {
            const int row = prow0 + i * PRPP, pix = ps + row;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < nrows && (unsigned)pix < (unsigned)npix_in && c < Cred) {
                const int off = pix * Cred + c;
                v = load4(in, off);
                if (BWD && mask) {
                    const float4 y = load4(mask, off);
                    v.x = y.x > 0.f ? v.x : 0.f; v.y = y.y > 0.f ? v.y : 0.f;
                    v.z = y.z > 0.f ? v.z : 0.f; v.w = y.w > 0.f ? v.w : 0.f;
                }
            }
            preg[i] = v;
        }
    };
    auto store_panel = [&]() {
#pragma unroll
        for (int i = 0; i < PNP; i++) {
            const int row = prow0 + i * PRPP;
            if (row < PR) *(float4 *)(panel + row * PITCH + pquad * 4) = preg[i];
        }
    };
    auto load_b = [&](int ch, int tap) {
        if (fast) {
            const unsigned base = BKM ? (unsigned)((tap * Cred + ch * BK) * 4)
                                      : (unsigned)(((ch * BK * RS + (RS - 1 - tap)) * p.Ncols) * 4);
#pragma unroll
            for (int i = 0; i < BNP; i++) breg[i] = buffer_load4(w_rsrc, bvoff[i] >= OOB ? OOB : bvoff[i] + base);
            return;
        }
#pragma unroll
        for (int i = 0; i < BNP; i++) {
            const int line = bline0 + i * BRPP;
            int off = -1;
            if (BKM) {       // line = output channel, quad runs along the reduction channels
                const int n = n0 + line, c = ch * BK + bquad * 4;
                if (n < p.Ncols && c < Cred) off = (n * RS + tap) * Cred + c;
            } else {         // line = reduction channel, quad runs along the output channels
                const int k = ch * BK + line, c = n0 + bquad * 4;
                if (k < Cred && c < p.Ncols) off = (k * RS + (RS - 1 - tap)) * p.Ncols + c;
            }
            breg[i] = off < 0 ? make_float4(0.f, 0.f, 0.f, 0.f) : load4(wsrc, off);
        }
    };
    auto store_b = [&](float *buf) {
#pragma unroll
        for (int i = 0; i < BNP; i++)
            *(float4 *)(buf + (bline0 + i * BRPP) * BPITCH + bquad * 4) = breg[i];
    };

    float16v acc[MB][2];
#pragma unroll
    for (int i = 0; i < MB; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

    if (tid < PITCH) panel[PR * PITCH + tid] = 0.f;              // the row of zeros
    if (ch_beg < ch_end) {
        load_panel(ch_beg);
        load_b(ch_beg, 0);
        store_panel();
        store_b(lds);
    }
    __syncthreads();

    int cur = 0;
    for (int ch = ch_beg; ch < ch_end; ch++) {
        const bool next_chunk = ch + 1 < ch_end;
        int r = 0, s = 0;
        for (int tap = 0; tap < RS; tap++) {
            const bool last_tap = tap == RS - 1;
            const bool more = !last_tap || next_chunk;
            if (more) load_b(last_tap ? ch + 1 : ch, last_tap ? 0 : tap + 1);
            if (tap == 0 && next_chunk) load_panel(ch + 1);      // held in registers until the last tap

            int aoff[MB];
#pragma unroll
            for (int bm = 0; bm < MB; bm++) {
                const bool ok = (unsigned)(hh[bm] + r) < (unsigned)Hi && (unsigned)(ww[bm] + s) < (unsigned)Wi;
                aoff[bm] = (ok ? prow[bm] + r * Wi + s : PR) * PITCH + lh * 4;
            }
            const float *Bs = lds + cur * BT;
#pragma unroll
            for (int kc = 0; kc < BK / 8; kc++) {
                float af[MB][4], bf[2][4];
#pragma unroll
                for (int bm = 0; bm < MB; bm++) {
                    const float4 v = *(const float4 *)(panel + aoff[bm] + kc * 8);
                    af[bm][0] = v.x; af[bm][1] = v.y; af[bm][2] = v.z; af[bm][3] = v.w;
                }
                if (BKM) {
#pragma unroll
                    for (int bn = 0; bn < 2; bn++) {
                        const float4 v = *(const float4 *)(Bs + (wn0 + bn * 32 + li) * BPITCH + kc * 8 + lh * 4);
                        bf[bn][0] = v.x; bf[bn][1] = v.y; bf[bn][2] = v.z; bf[bn][3] = v.w;
                    }
                } else {
#pragma unroll
                    for (int jj = 0; jj < 4; jj++) {
                        const float2 v = *(const float2 *)(Bs + (kc * 8 + lh * 4 + jj) * BPITCH + wn0 + 2 * li);
                        bf[0][jj] = v.x; bf[1][jj] = v.y;
                    }
                }
#pragma unroll
                for (int jj = 0; jj < 4; jj++)
#pragma unroll
                    for (int bm = 0; bm < MB; bm++)
#pragma unroll
                        for (int bn = 0; bn < 2; bn++)
                            acc[bm][bn] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[bm][jj], bf[bn][jj], acc[bm][bn], 0, 0, 0);
            }
            if (more) store_b(lds + (cur ^ 1) * BT);
            if (last_tap && next_chunk) {
                __syncthreads();                                 // every wave is done with the old panel
                store_panel();
            }
            __syncthreads();
            cur ^= 1;
            if (++s == S) { s = 0; r++; }
        }
    }

    tile_epilogue<Epi, true, BKM, MB>(p, acc, m0 + wm0, n0 + wn0, li, lh, split);
}

}  // namespace owt
