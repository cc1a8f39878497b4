// Direct stride-1 convolution for bf16 storage on the bf16 MFMA
// (v_mfma_f32_32x32x16_bf16, fp32 accumulate): forward and backward-data of the
// stride-1 layers (Section 4 of the paper, forward step 2 / backward step 2) at
// 16x the fp32 matrix rate.
//
// Same scheme as dconv.hpp: the pixels a row tile touches stay resident in LDS
// for a 64-channel chunk (bf16, 144-byte rows: 128 B of data + 16 B pad, which
// keeps the 16-byte fragment reads bank-conflict free), every filter tap reads
// its A fragments from that panel at a shifted row, and the filter slice of the
// current (chunk, tap) streams through a double-buffered tile.  Both operands
// must be contiguous along the reduction channels, because one MFMA lane holds
// 8 consecutive reduction elements: the forward filters w[k][r][s][c] already
// are; backward-data uses a re-laid-out copy wt[c][r'][s'][k] = w[k][R-1-r'][S-1-s'][c]
// that owt_api writes into the workspace first.
#pragma once
#include "igemm.hpp"

namespace owt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// zero the bf16 lanes of v whose mask value (bf16 bits in y) is not > 0
__device__ __forceinline__ uint32_t mask_pair(uint32_t v, uint32_t y)
{
    const uint32_t lo = y & 0xffffu, hi = y >> 16;
    const bool plo = lo != 0u && lo < 0x8000u, phi = hi != 0u && hi < 0x8000u;   // positive, non-zero
    return (plo ? (v & 0xffffu) : 0u) | (phi ? (v & 0xffff0000u) : 0u);
}

template <class Epi, bool BWD, int WM, int WN, int PR>
__global__ void __launch_bounds__(64 * WM * WN, (WM * WN >= 4 ? 2 : 1)) dconv_bf16_kernel(const GemmParams p)
{
    constexpr int BK = 64, NT = 64 * WM * WN, BM = 64 * WM, BN = 64 * WN, PITCH = BK + 8;   // in bf16 elements
    constexpr int OCTS = BK / 8;                                 // 16-byte pieces per row
    constexpr int BT = BN * PITCH;                               // elements per filter-slice buffer
    constexpr int RPP = NT / OCTS;                               // rows per load pass
    constexpr int BNP = BN / RPP, PNP = (PR + RPP - 1) / RPP;
    static_assert(BN % RPP == 0, "filter slice must split evenly over the threads");

    __shared__ __attribute__((aligned(16))) uint16_t lds[2 * BT + (PR + 1) * PITCH];
    uint16_t *panel = lds + 2 * BT;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int wm0 = (wave / WN) * 64, wn0 = (wave % WN) * 64;

    const int ntiles = p.tiles_m * p.tiles_n;
    const int b = blockIdx.x, xcd = b & 7;
    const int logical = xcd * (ntiles >> 3) + min(xcd, ntiles & 7) + (b >> 3);
    const int tm = logical / p.tiles_n, tn = logical - tm * p.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const int split = blockIdx.y;
    const int ch_beg = split * p.ksteps_per_split, ch_end = min(p.ksteps, ch_beg + p.ksteps_per_split);

    const int R = p.g.R, S = p.g.S, RS = R * S, Hi = p.Hi, Wi = p.Wi, Cred = p.Cred;
    const int HoWo = p.Ho * p.Wo, npix_in = p.g.N * Hi * Wi;

    auto pin = [&](int m, int &hh, int &ww) {
        const int n = p.dHoWo.div(m), rem = m - n * HoWo;
        const int ho = p.dWo.div(rem), wo = rem - ho * p.Wo;
        hh = ho - p.pah; ww = wo - p.paw;
        return n * Hi * Wi + hh * Wi + ww;
    };
    int th, tw;
    const int ps = pin(m0, th, tw);
    const int nrows = pin(min(m0 + BM, p.M) - 1, th, tw) + (R - 1) * Wi + S - ps;   // <= PR (host-checked)

    int hh[2], ww[2], prow[2];
#pragma unroll
    for (int bm = 0; bm < 2; bm++) {
        const int m = m0 + wm0 + bm * 32 + li;
        if (m < p.M) prow[bm] = pin(m, hh[bm], ww[bm]) - ps;
        else { hh[bm] = kInvalidLo; ww[bm] = 0; prow[bm] = 0; }
    }

    const uint16_t *in = (const uint16_t *)p.a, *wsrc = (const uint16_t *)p.b, *mask = (const uint16_t *)p.mask;
    const int oct = tid % OCTS, line0 = tid / OCTS;
    uint4 preg[PNP], breg[BNP];
    const uint4 zero4 = make_uint4(0u, 0u, 0u, 0u);

    auto load_panel = [&](int ch) {
        const int c = ch * BK + oct * 8;
#pragma unroll
        for (int i = 0; i < PNP; i++) {
            const int row = line0 + i * RPP, pix = ps + row;
            uint4 v = zero4;
            if (row < nrows && (unsigned)pix < (unsigned)npix_in && c < Cred) {
                const int off = pix * Cred + c;
                v = *(const uint4 *)(in + off);
                if (BWD && mask) {
                    const uint4 y = *(const uint4 *)(mask + off);
                    v.x = mask_pair(v.x, y.x); v.y = mask_pair(v.y, y.y);
                    v.z = mask_pair(v.z, y.z); v.w = mask_pair(v.w, y.w);
                }
            }
            preg[i] = v;
        }
    };
    auto store_panel = [&]() {
#pragma unroll
        for (int i = 0; i < PNP; i++) {
            const int row = line0 + i * RPP;
            if (row < PR) *(uint4 *)(panel + row * PITCH + oct * 8) = preg[i];
        }
    };
    auto load_b = [&](int ch, int tap) {    // both passes: line = output channel, oct runs along the reduction
        const int c = ch * BK + oct * 8;
#pragma unroll
        for (int i = 0; i < BNP; i++) {
            const int n = n0 + line0 + i * RPP;
            uint4 v = zero4;
            if (n < p.Ncols && c < Cred) v = *(const uint4 *)(wsrc + ((size_t)n * RS + tap) * Cred + c);
            breg[i] = v;
        }
    };
    auto store_b = [&](uint16_t *buf) {
#pragma unroll
        for (int i = 0; i < BNP; i++) *(uint4 *)(buf + (line0 + i * RPP) * PITCH + oct * 8) = breg[i];
    };

    float16v acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

    if (tid < PITCH) panel[PR * PITCH + tid] = 0;                // the row of zeros
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

            int aoff[2];
#pragma unroll
            for (int bm = 0; bm < 2; bm++) {
                const bool ok = (unsigned)(hh[bm] + r) < (unsigned)Hi && (unsigned)(ww[bm] + s) < (unsigned)Wi;
                aoff[bm] = (ok ? prow[bm] + r * Wi + s : PR) * PITCH + lh * 8;
            }
            const uint16_t *Bs = lds + cur * BT;
#pragma unroll
            for (int kc = 0; kc < BK / 16; kc++) {
                bf16x8 af[2], bf[2];
#pragma unroll
                for (int bm = 0; bm < 2; bm++)
                    af[bm] = __builtin_bit_cast(bf16x8, *(const uint4 *)(panel + aoff[bm] + kc * 16));
#pragma unroll
                for (int bn = 0; bn < 2; bn++)
                    bf[bn] = __builtin_bit_cast(bf16x8, *(const uint4 *)(Bs + (wn0 + bn * 32 + li) * PITCH + kc * 16 + lh * 8));
#pragma unroll
                for (int bm = 0; bm < 2; bm++)
#pragma unroll
                    for (int bn = 0; bn < 2; bn++)
                        acc[bm][bn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[bm], bf[bn], acc[bm][bn], 0, 0, 0);
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

    tile_epilogue<Epi, true, true>(p, acc, m0 + wm0, n0 + wn0, li, lh, split);
}

}  // namespace owt
