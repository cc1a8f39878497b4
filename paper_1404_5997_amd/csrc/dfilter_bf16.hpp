// Direct filter-gradient kernel for stride-1 "same" convolutions with bf16 storage, on the
// bf16 MFMA (v_mfma_f32_32x32x16_bf16, fp32 accumulate):
//
//   dw[k][r][s][c] = sum over pixels (n,p,q) of dz[n,p,q,k] * x[n, p+r-pad_h, q+s-pad_w, c]
//
// (Section 4 of the paper, backward step 2: the weight gradients of the data-parallel
// convolution layers.)  Same decomposition as dfilter.hpp: a work-group owns KT filters x
// CT channels x all taps of a tap group, walks over the pixels in chunks, and keeps the dz
// rows and the x pixels of a chunk in LDS in zero-padded image coordinates, so tap (r,s)
// of a pixel is a fixed row offset.  What differs is the reduction index: the bf16 MFMA
// wants 8 consecutive REDUCTION elements (here: pixels) per lane, but NHWC keeps channels
// contiguous.  LDS stays in the natural [pixel][channel] order and the fragments are read
// with ds_read_b64_tr_b16, which transposes across a 16-lane group: when lane s of the group
// points at four consecutive values (row s/4, columns 4*(s%4)..+3 of a 4 x 16 block), lane i
// receives column i of rows 0..3.  Two such reads give a lane its 8 pixels of one channel.
//
// A wavefront holds KB x TAPS accumulators of 32 x 32 (filter blocks x the taps of one filter row), so one
// dz fragment feeds TAPS MFMAs and one x fragment KB of them: (2 KB + 2 TAPS) transposing reads per
// KB x TAPS MFMAs.  The host's variant table pairs each work-group tile with two splits of it: few
// wavefronts with KB = 4 (or 2 for five taps; 192 / 160 accumulator registers, one wavefront per SIMD, fewest
// LDS reads per MFMA), or twice / three times the wavefronts with half / a quarter of the filter blocks each.
// The second kind is faster by 15-20 %: at the bf16 MFMA rate a wavefront's waits (fragments, the chunk
// barrier, address arithmetic) are only filled by another wavefront on the same SIMD; sixteen wavefronts of
// one block each lose again to the LDS read rate.  LDS is double buffered: one barrier per 64-pixel chunk.
#pragma once
#include "igemm.hpp"

namespace owt {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef short short8_t __attribute__((ext_vector_type(8)));

// zero the bf16 halves of v whose mask value (bf16 bits in y) is not > 0
__device__ __forceinline__ uint32_t relu_mask_pair(uint32_t v, uint32_t y)
{
    const uint32_t lo = y & 0xffffu, hi = y >> 16;
    const bool plo = lo != 0u && lo < 0x8000u, phi = hi != 0u && hi < 0x8000u;
    return (plo ? (v & 0xffffu) : 0u) | (phi ? (v & 0xffff0000u) : 0u);
}

__device__ __forceinline__ short4_t lds_read_tr16(const uint16_t *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_t *)p);
}

// OCC = work-groups per CU; the second launch bound is wavefronts per SIMD.
template <int WK, int WC, int KB, int TAPS, int PRF, int OCC>
__global__ void __launch_bounds__(64 * WK * WC, (OCC * WK * WC >= 4 ? OCC * WK * WC / 4 : 1)) dfilter16_kernel(const GemmParams p)
{
    constexpr int NT = 64 * WK * WC, KT = 32 * KB * WK, CT = 32 * WC, BP = 64;
    // Row pitches in elements.  A transposing read touches 64 bytes of each of four consecutive rows per
    // half-wave: with rows 64 bytes (mod 256) apart the four pieces fall on disjoint banks.  The two variants
    // that run two work-groups per CU have no LDS to spare and keep a 32-byte pad (two-way conflicts).
    constexpr int PAD = OCC >= 2 ? 16 : 32, PA = KT + PAD, PB = CT + PAD;
    static_assert(OCC >= 2 || ((2 * PA) % 256 == 64 || (2 * PA) % 256 == 192), "dz rows must fall on disjoint banks");
    static_assert(OCC >= 2 || ((2 * PB) % 256 == 64 || (2 * PB) % 256 == 192), "panel rows must fall on disjoint banks");
    constexpr int KO = KT / 8, ARPP = NT / KO, ANP = (BP + ARPP - 1) / ARPP;     // dz loader (16-byte pieces); the last pass may be partial
    // x panel loader: a thread fetches LPT 16-byte pieces of one panel row (pieces bq, bq + TPR, ...), so the
    // row's position in the padded image is worked out once per LPT loads (one piece per thread where the
    // rounding up to whole passes would cost the six-wavefront variant staging registers it does not have)
    constexpr int CO = CT / 8, LPT = CO >= 16 ? 4 : (NT % 256 == 0 ? 2 : 1), TPR = CO / LPT, BRPP = NT / TPR,
                  BNP = (PRF + BRPP - 1) / BRPP;
    constexpr int NG = BP / 16;                                  // 16-pixel MFMA groups per chunk
    static_assert(CO % LPT == 0 && NT % TPR == 0 && NT % KO == 0, "tiles must split evenly over the threads");

    __shared__ __attribute__((aligned(16))) uint16_t dzs[2][BP * PA];
    __shared__ __attribute__((aligned(16))) uint16_t panel[2][PRF * PB];
    __shared__ int prow_tab[2][BP];

    const Geom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int grp16 = lane >> 4, i16 = lane & 15;                // 16-lane group and position in it
    const int wk0 = (wave / WC) * 32 * KB, wc0 = (wave % WC) * 32;

    int logical, split;
    if (!owt_split_major_wg(p.tiles_m * p.tiles_n, p.splits, logical, split)) return;
    const int kt = logical / p.tiles_n, rem = logical - kt * p.tiles_n;
    const int grp = rem / p.ctiles, ct = rem - grp * p.ctiles;
    const int k0 = kt * KT, c0 = ct * CT;
    const int ch_beg = split * p.ksteps_per_split, ch_end = min(p.ksteps, ch_beg + p.ksteps_per_split);

    const int RS = g.R * g.S, Wp = p.Wp, npix = p.Kd;
    const int r0 = p.groups > 1 ? grp : 0, rows_g = p.groups > 1 ? 1 : g.R;
    const int tap_first = p.groups > 1 ? grp * g.S : 0;

    auto ppad = [&](int pix) {       // padded linear index of the window's top-left corner of pixel pix
        const int n = g.dPQ.div(pix), pq = pix - n * g.P * g.Q;
        const int pp = g.dQ.div(pq), q = pq - pp * g.Q;
        return (n * p.Hp + pp) * Wp + q;
    };

    const uint16_t *dzsrc = (const uint16_t *)p.a, *xsrc = (const uint16_t *)p.b, *mask = (const uint16_t *)p.mask;
    const int ako = tid % KO, arow0 = tid / KO;
    const int bq = tid % TPR, brow0 = tid / TPR;
    uint4 areg[ANP], breg[BNP][LPT];
    int tab_next = 0;
    const int pad_pix_total = g.N * p.Hp * Wp;
    const uint4 zero4 = make_uint4(0u, 0u, 0u, 0u);

    auto load_chunk = [&](int ch) {
        const int pix0 = ch * BP;
        const int ps = ppad(pix0) + r0 * Wp;
        const int nrows = ppad(min(pix0 + BP, npix) - 1) + (r0 + rows_g - 1) * Wp + g.S - ps;   // <= PRF (host-checked)
#pragma unroll
        for (int i = 0; i < ANP; i++) {
            const int pix = pix0 + arow0 + i * ARPP, k = k0 + ako * 8;
            uint4 v = zero4;
            if ((BP % ARPP == 0 || arow0 + i * ARPP < BP) && pix < npix && k < g.K) {
                const int off = pix * g.K + k;
                v = *(const uint4 *)(dzsrc + off);
                if (mask) {
                    const uint4 y = *(const uint4 *)(mask + off);
                    v.x = relu_mask_pair(v.x, y.x); v.y = relu_mask_pair(v.y, y.y);
                    v.z = relu_mask_pair(v.z, y.z); v.w = relu_mask_pair(v.w, y.w);
                }
            }
            areg[i] = v;
        }
#pragma unroll
        for (int i = 0; i < BNP; i++) {
            const int row = brow0 + i * BRPP, idx = ps + row;
            const uint16_t *src = nullptr;
            if (row < nrows && idx < pad_pix_total) {
                const int n = p.dHpWp.div(idx), r2 = idx - n * p.Hp * Wp;
                const int hp = p.dWp.div(r2), wp = r2 - hp * Wp;
                const int h = hp - g.ph, w = wp - g.pw;
                if ((unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W)
                    src = xsrc + ((size_t)(n * g.H + h) * g.W + w) * g.C + c0 + bq * 8;
            }
#pragma unroll
            for (int j = 0; j < LPT; j++) {
                uint4 v = zero4;
                if (src && c0 + (bq + j * TPR) * 8 < g.C) v = *(const uint4 *)(src + j * TPR * 8);
                breg[i][j] = v;
            }
        }
        if (tid < BP) {
            const int pix = pix0 + tid;
            tab_next = pix < npix ? ppad(pix) + r0 * Wp - ps : 0;
        }
    };
    auto store_chunk = [&](int buf) {
#pragma unroll
        for (int i = 0; i < ANP; i++)
            if (BP % ARPP == 0 || arow0 + i * ARPP < BP) *(uint4 *)(dzs[buf] + (arow0 + i * ARPP) * PA + ako * 8) = areg[i];
#pragma unroll
        for (int i = 0; i < BNP; i++) {
            const int row = brow0 + i * BRPP;
            if (row < PRF) {
#pragma unroll
                for (int j = 0; j < LPT; j++) *(uint4 *)(panel[buf] + row * PB + (bq + j * TPR) * 8) = breg[i][j];
            }
        }
        if (tid < BP) prow_tab[buf][tid] = tab_next;
    };

    float16v acc[KB][TAPS];
#pragma unroll
    for (int kb = 0; kb < KB; kb++)
#pragma unroll
        for (int t = 0; t < TAPS; t++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[kb][t][r] = 0.f;

    // element offsets this lane passes to the transposing reads: source position (row i16/4,
    // columns 4*(i16%4)..+3) inside the 16-column block of its half-wave
    const int colsel = 16 * (grp16 & 1) + 4 * (i16 & 3);
    const int aoff = wk0 + colsel;                               // + kb*32 + pixel*PA
    int toff[TAPS];
#pragma unroll
    for (int t = 0; t < TAPS; t++) {
        const int r = p.groups > 1 ? 0 : t / g.S, s = p.groups > 1 ? t : t - (t / g.S) * g.S;
        toff[t] = (r * Wp + s) * PB + wc0 + colsel;
    }
    const int pixsel = 8 * (grp16 >> 1) + (i16 >> 2);            // + 16*group + 4*half

    float dbacc[8];
#pragma unroll
    for (int j = 0; j < 8; j++) dbacc[j] = 0.f;
    const bool do_db = ct == 0 && grp == 0 && p.dbias != nullptr;

    if (ch_beg < ch_end) { load_chunk(ch_beg); store_chunk(0); }
    __syncthreads();

    int cur = 0;
    for (int ch = ch_beg; ch < ch_end; ch++) {
        if (do_db) {
#pragma unroll
            for (int i = 0; i < ANP; i++) {
                const uint32_t w4[4] = {areg[i].x, areg[i].y, areg[i].z, areg[i].w};
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    dbacc[2 * j] += __uint_as_float(w4[j] << 16);
                    dbacc[2 * j + 1] += __uint_as_float(w4[j] & 0xffff0000u);
                }
            }
        }
        const bool more = ch + 1 < ch_end;
        if (more) load_chunk(ch + 1);

        const uint16_t *dzc = dzs[cur], *pnc = panel[cur];
        const int *tabc = prow_tab[cur];
        // Fragments of one 16-pixel group: KB dz fragments and TAPS x fragments, two reads each.  The x
        // fragment of a tap is refilled for the next group right after its MFMAs have been issued, so
        // one register set serves both groups and the reads run a whole group ahead of their use.
        int px0, px1, pr0, pr1;
        auto locate = [&](int gi) {
            px0 = 16 * gi + pixsel; px1 = px0 + 4;
            pr0 = tabc[px0] * PB; pr1 = tabc[px1] * PB;
        };
        auto read_a = [&](short8_t (&a)[KB]) {
#pragma unroll
            for (int kb = 0; kb < KB; kb++) {
                const short4_t lo = lds_read_tr16(dzc + px0 * PA + aoff + kb * 32);
                const short4_t hi = lds_read_tr16(dzc + px1 * PA + aoff + kb * 32);
                a[kb] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        };
        auto read_b = [&](int t) {
            const short4_t lo = lds_read_tr16(pnc + pr0 + toff[t]);
            const short4_t hi = lds_read_tr16(pnc + pr1 + toff[t]);
            return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        };
        short8_t af[2][KB], bf[TAPS];
        locate(0);
        read_a(af[0]);
#pragma unroll
        for (int t = 0; t < TAPS; t++) bf[t] = read_b(t);
#pragma unroll
        for (int gi = 0; gi < NG; gi++) {
            const bool next = gi + 1 < NG;
            if (next) { locate(gi + 1); read_a(af[(gi + 1) & 1]); }
#pragma unroll
            for (int t = 0; t < TAPS; t++) {
#pragma unroll
                for (int kb = 0; kb < KB; kb++)
                    acc[kb][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, af[gi & 1][kb]),
                                                                         __builtin_bit_cast(bf16x8_t, bf[t]), acc[kb][t], 0, 0, 0);
                if (next) bf[t] = read_b(t);
            }
        }
        if (more) store_chunk(cur ^ 1);
        __syncthreads();
        cur ^= 1;
    }

    // ---- epilogue: dw[k][tap][c]; accumulator register r of lane (li, lh) holds
    // filter k = 8*(r/4) + 4*lh + r%4 of its 32-filter block, channel li.
    const bool part = p.splits > 1;
    float *pout = part ? p.partial + (size_t)split * p.M * p.Ncols : nullptr;
    float *out = (float *)p.out;
    const int c = c0 + wc0 + li;
#pragma unroll
    for (int kb = 0; kb < KB; kb++)
#pragma unroll
        for (int t = 0; t < TAPS; t++) {
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int k = k0 + wk0 + kb * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
                if (k >= g.K || c >= g.C) continue;
                const size_t o = ((size_t)k * RS + tap_first + t) * g.C + c;
                if (part) pout[o] = acc[kb][t][r];
                else out[o] = p.alpha * acc[kb][t][r] + (p.beta != 0.f ? p.beta * out[o] : 0.f);
            }
        }

    if (do_db) {   // uniform over the work-group; every wave has passed the loop's last barrier
        float *red = (float *)&panel[0][0];                      // ARPP x KT floats
        static_assert(sizeof(panel) >= sizeof(float) * ARPP * KT, "bias-gradient scratch must fit the panel");
#pragma unroll
        for (int j = 0; j < 8; j++) red[arow0 * KT + ako * 8 + j] = dbacc[j];
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
