// Direct stride-1 convolution for bf16 storage on the bf16 MFMA, 512 x 64 tile, software pipelined.
//
// Forward and backward-data of the stride-1 layers (Section 4 of the paper, forward step 2 /
// backward step 2), same panel-resident scheme as dconv_bf16.hpp.  At the bf16 matrix rate the
// 64 x 64 wavefront tile of that kernel needs one 16-byte LDS fragment read per MFMA, which is all
// the LDS can deliver, and its reads are only one MFMA group ahead.  Here
//   * a wavefront owns 128 pixels x 64 filters (4 x 2 accumulators): 6 fragment reads per 8 MFMAs;
//   * the reduction runs in 32-channel chunks, two 16-channel MFMA phases per filter tap; during a
//     phase every pixel fragment is re-read for the NEXT phase right after its last use, and the
//     filter fragments of the next phase are read at the start of the phase, so a fragment is
//     requested about six MFMAs before it is needed;
//   * the filter slice of a tap goes from global memory straight into LDS (global_load_lds, 16 bytes
//     per lane, a wavefront's 64 pieces land back to back): no staging registers, no LDS store.  The
//     slice is therefore unpadded (64-byte lines) and the 16-byte piece c of line n sits at position
//     c ^ ((n >> 2) & 3), which keeps the fragment reads free of bank conflicts.  The two slice
//     buffers and the panel are separate __shared__ arrays and the tap loop is unrolled by two: the
//     compiler then knows which array a transfer in flight writes and does not make the fragment
//     reads of the other arrays wait for it;
//   * the one barrier per tap sits between the two phases: the transfer of the slice of tap t+1 is
//     waited for before it, the first fragments of tap t+1 are read after it, and the transfer of
//     the slice of tap t+2 is issued after it, into the buffer whose last reads ended before it.
// The accumulators hold the TRANSPOSED tile (filters along MFMA rows, pixels along columns): a lane
// then owns four consecutive filters of one pixel and stores 8 bytes at a time.
// Needs the reduction channels to be a multiple of 32 and at most 32 filter taps (host-checked).
#pragma once
#include "dconv_bf16.hpp"

namespace owt {

// MB = 32-pixel blocks per wavefront (4: the 512 x 64 tile, two work-groups per CU; 2: 256 x 64, fewer
// registers, three work-groups per CU), OCC = work-groups per CU the register budget is cut for.
template <class Epi, bool BWD, int PR, int MB, int OCC>
__global__ void __launch_bounds__(256, OCC) dconv16p_kernel(const GemmParams p)
{
    constexpr int BK = 32, NT = 256, BM = 128 * MB, BN = 64, PITCH = BK + 8;      // panel rows: 80 bytes
    constexpr int OCTS = BK / 8, RPP = NT / OCTS, PNP = (PR + RPP - 1) / RPP;
    constexpr int BT = BN * BK;                                  // bf16 elements per filter-slice buffer
    static_assert(BN * OCTS == NT, "one 16-byte piece of the filter slice per thread");
    static_assert(MB == 2 || MB == 4, "two or four 32-pixel blocks per wavefront");

    __shared__ __attribute__((aligned(16))) uint16_t slice0[BT];
    __shared__ __attribute__((aligned(16))) uint16_t slice1[BT];
    __shared__ __attribute__((aligned(16))) uint16_t panel[(PR + 1) * PITCH];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int wm0 = wave * 32 * MB;

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

    // per 32-pixel block of this lane: element offset of its panel row at tap (0,0), and one bit per
    // tap telling whether the tap falls inside the image (else the row of zeros is read)
    constexpr int ZOFF = PR * PITCH;
    int poff[MB];
    unsigned inside[MB];
#pragma unroll
    for (int bm = 0; bm < MB; bm++) {
        const int m = m0 + wm0 + bm * 32 + li;
        poff[bm] = lh * 8;
        inside[bm] = 0u;
        if (m < p.M) {
            int hh, ww;
            poff[bm] += (pin(m, hh, ww) - ps) * PITCH;
            for (int r = 0, tap = 0; r < R; r++)
                for (int s = 0; s < S; s++, tap++)
                    if ((unsigned)(hh + r) < (unsigned)Hi && (unsigned)(ww + s) < (unsigned)Wi) inside[bm] |= 1u << tap;
        }
    }

    const uint16_t *in = (const uint16_t *)p.a, *wsrc = (const uint16_t *)p.b, *mask = (const uint16_t *)p.mask;
    const int oct = tid % OCTS, line0 = tid / OCTS;
    uint4 preg[PNP];
    const uint4 zero4 = make_uint4(0u, 0u, 0u, 0u);

    auto load_panel = [&](int ch) __attribute__((always_inline)) {
        const int c = ch * BK + oct * 8;
#pragma unroll
        for (int i = 0; i < PNP; i++) {
            const int row = line0 + i * RPP, pix = ps + row;
            uint4 v = zero4;
            if (row < nrows && (unsigned)pix < (unsigned)npix_in) {
                const size_t off = (size_t)pix * Cred + c;
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
    auto store_panel = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < PNP; i++) {
            const int row = line0 + i * RPP;
            if (row < PR) *(uint4 *)(panel + row * PITCH + oct * 8) = preg[i];
        }
    };
    // Filter slice: line = output column (a filter in forward, an input channel in backward-data).  This
    // lane's piece lands at line0, position oct, so it fetches piece oct ^ ((line0 >> 2) & 3) of that line;
    // columns past the end re-read the last line (those output columns are never stored).
    const uint16_t *bsrc = wsrc + (size_t)min(n0 + line0, p.Ncols - 1) * RS * Cred + ((oct ^ ((line0 >> 2) & 3)) * 8);
    auto fetch_slice = [&](int ch, int tap, uint16_t *buf) __attribute__((always_inline)) {
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(bsrc + tap * Cred + ch * BK),
                                         (__attribute__((address_space(3))) void *)(buf + wave * 512), 16, 0, 0);
    };
    auto frag = [&](const uint16_t *q) { return __builtin_bit_cast(bf16x8, *(const uint4 *)q); };
    // element offsets of this lane's filter fragments: [32-filter block][16-channel phase]
    int boff[2][2];
#pragma unroll
    for (int bn = 0; bn < 2; bn++)
#pragma unroll
        for (int kc = 0; kc < 2; kc++) {
            const int row = bn * 32 + li;
            boff[bn][kc] = row * BK + (((kc * 2 + lh) ^ ((row >> 2) & 3)) * 8);
        }
    auto tap_offsets = [&](int tap, int r, int s, int (&aoff)[MB]) __attribute__((always_inline)) {
        const int shift = (r * Wi + s) * PITCH;
#pragma unroll
        for (int bm = 0; bm < MB; bm++) aoff[bm] = ((inside[bm] >> tap) & 1u) ? poff[bm] + shift : ZOFF + lh * 8;
    };

    // order of a phase as the hardware should see it: `lead` fragment reads, then four times (two MFMAs,
    // one fragment read; `first` reads after the first pair); the compiler's own order bunches the reads
    // behind the MFMAs
#define OWT_PIN_PHASE(LEAD, FIRST)                                           \
    do {                                                                    \
        if (LEAD) __builtin_amdgcn_sched_group_barrier(0x100, LEAD, 0);     \
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                  \
        __builtin_amdgcn_sched_group_barrier(0x100, FIRST, 0);              \
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                  \
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                  \
        if (MB > 2) {                                                       \
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);              \
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);              \
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);              \
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);              \
        }                                                                   \
    } while (0)

    float16v acc[MB][2];
#pragma unroll
    for (int i = 0; i < MB; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

    const int nsteps = (ch_end - ch_beg) * RS;                  // one step per (chunk, tap)
    if (tid < PITCH) panel[ZOFF + tid] = 0;                     // the row of zeros
    if (nsteps > 0) {
        load_panel(ch_beg);
        fetch_slice(ch_beg, 0, slice0);
        fetch_slice(ch_beg, 1, slice1);                         // at least two taps (host-checked)
        store_panel();
        __builtin_amdgcn_s_waitcnt(0x0F70);                     // vmcnt(0): both slices have landed
    }
    __syncthreads();

    if (nsteps > 0) {
        bf16x8 af[MB], bf[2][2];
        int aoff[MB];
        tap_offsets(0, 0, 0, aoff);
#pragma unroll
        for (int bm = 0; bm < MB; bm++) af[bm] = frag(panel + aoff[bm]);
        bf[0][0] = frag(slice0 + boff[0][0]);
        bf[0][1] = frag(slice0 + boff[1][0]);
        int ch = ch_beg, tap = 0, r = 0, s = 0;

        // one (chunk, tap) step on the slice in `cur`; `nxt` holds the slice of the following step.  Forced inline:
        // called out of line, everything it captures would live in scratch memory.
        auto step = [&](int t, uint16_t *cur, uint16_t *nxt) __attribute__((always_inline)) {
            const bool swap_panel = tap == RS - 1 && t + 1 < nsteps;    // the next step starts a new chunk

            // phase 0: channels 0..15 of the chunk; fetch the fragments of channels 16..31.  The first MFMAs
            // wait for the fragments requested a phase ago only: this phase's reads are issued behind them.
#pragma unroll
            for (int bm = 0; bm < MB; bm++) {
                acc[bm][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[0][0], af[bm], acc[bm][0], 0, 0, 0);
                acc[bm][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[0][1], af[bm], acc[bm][1], 0, 0, 0);
                af[bm] = frag(panel + aoff[bm] + 16);
                if (bm == 0) {
                    bf[1][0] = frag(cur + boff[0][1]);
                    bf[1][1] = frag(cur + boff[1][1]);
                }
            }
            OWT_PIN_PHASE(0, 3);
            if (swap_panel) {
                __syncthreads();                                 // every wave has its last fragments of the old panel
                store_panel();
            }
            __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): this wave's pieces of `nxt` have landed
            __syncthreads();

            // coordinates of steps t+1 and t+2
            int tap1 = tap + 1, ch1 = ch, r1 = r, s1 = s + 1;
            if (s1 == S) { s1 = 0; r1++; }
            if (tap1 == RS) { tap1 = 0; ch1++; r1 = 0; s1 = 0; }
            int tap2 = tap1 + 1, ch2 = ch1;
            if (tap2 == RS) { tap2 = 0; ch2++; }

            // phase 1: channels 16..31; fetch the first fragments of step t+1; the slice of step t+2
            // goes into `cur`, whose last reads ended before the barrier
            if (t + 2 < nsteps) fetch_slice(ch2, tap2, cur);
            if (tap == 0 && ch + 1 < ch_end) load_panel(ch + 1);  // held in registers until the last tap
            tap_offsets(tap1, r1, s1, aoff);
            bf[0][0] = frag(nxt + boff[0][0]);
            bf[0][1] = frag(nxt + boff[1][0]);
#pragma unroll
            for (int bm = 0; bm < MB; bm++) {
                acc[bm][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[1][0], af[bm], acc[bm][0], 0, 0, 0);
                acc[bm][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[1][1], af[bm], acc[bm][1], 0, 0, 0);
                af[bm] = frag(panel + aoff[bm]);
            }
            OWT_PIN_PHASE(2, 1);
            tap = tap1; ch = ch1; r = r1; s = s1;
        };
        for (int t = 0; t < nsteps; t += 2) {
            step(t, slice0, slice1);
            if (t + 1 < nsteps) step(t + 1, slice1, slice0);
        }
    }

    // epilogue: register 4j+i of accumulator (bm, bn) is pixel 32*bm + li, filter 32*bn + 8j + 4*lh + i
    const bool part = p.splits > 1;
    float *pout = part ? p.partial + (size_t)split * p.M * p.Ncols : nullptr;
    uint16_t *out = (uint16_t *)p.out;
    if (!part && (p.Ncols & 7) == 0) {
        // Results leave through LDS, 32 pixels x 64 filters per wavefront and pass: a lane writes its 8-byte
        // pieces (bias and ReLU applied), then the wavefront reads the block back row-wise and stores 16 bytes
        // per lane, eight lanes to a 128-byte line (stored straight from the accumulators a store instruction
        // would touch 32 lines with 16 bytes each).  The panel is free: after the last barrier of the loop no
        // wavefront reads anything from it that it still uses; each wavefront stages in its own part, so
        // program order is all the synchronisation this needs.  The ReLU' mask of backward-data is applied
        // on the way out, with the same 16-byte accesses.
        constexpr int EP = 64 + 4;                               // 136-byte rows: conflict-free 8-byte writes
        static_assert(4 * 32 * EP <= (PR + 1) * PITCH, "the staging blocks must fit the panel");
        uint16_t *stage = panel + wave * 32 * EP;
        const uint16_t *xm = BWD ? (const uint16_t *)p.xmask : nullptr;
#pragma unroll
        for (int bm = 0; bm < MB; bm++) {
#pragma unroll
            for (int bn = 0; bn < 2; bn++)
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    const int nl = bn * 32 + 8 * j + 4 * lh, n = n0 + nl;
                    float v0 = acc[bm][bn][4 * j], v1 = acc[bm][bn][4 * j + 1], v2 = acc[bm][bn][4 * j + 2], v3 = acc[bm][bn][4 * j + 3];
                    if (!BWD) {
                        if ((p.flags & 1u) && n < p.Ncols) { v0 += p.bias[n]; v1 += p.bias[n + 1]; v2 += p.bias[n + 2]; v3 += p.bias[n + 3]; }
                        if (p.flags & 2u) {
                            v0 = v0 > 0.f ? v0 : 0.f; v1 = v1 > 0.f ? v1 : 0.f;
                            v2 = v2 > 0.f ? v2 : 0.f; v3 = v3 > 0.f ? v3 : 0.f;
                        }
                    }
                    *(uint2 *)(stage + li * EP + nl) = make_uint2(f32x2_to_bf16x2(v0, v1), f32x2_to_bf16x2(v2, v3));
                }
#pragma unroll
            for (int q = 0; q < 4; q++) {
                const int row = q * 8 + (lane >> 3), nl = (lane & 7) * 8;
                const int m = m0 + wm0 + bm * 32 + row, n = n0 + nl;
                uint4 v = *(const uint4 *)(stage + row * EP + nl);
                if (m < p.M && n < p.Ncols) {
                    const size_t o = (size_t)m * p.Ncols + n;
                    if (BWD && xm) {
                        const uint4 x = *(const uint4 *)(xm + o);
                        v.x = mask_pair(v.x, x.x); v.y = mask_pair(v.y, x.y);
                        v.z = mask_pair(v.z, x.z); v.w = mask_pair(v.w, x.w);
                    }
                    *(uint4 *)(out + o) = v;
                }
            }
        }
        return;
    }
#pragma unroll
    for (int bn = 0; bn < 2; bn++) {
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int n = n0 + bn * 32 + 8 * j + 4 * lh;
            if (n >= p.Ncols) continue;                          // Ncols is a multiple of 4 (host-checked)
            float b0 = 0.f, b1 = 0.f, b2 = 0.f, b3 = 0.f;
            if (!BWD && !part && (p.flags & 1u)) { b0 = p.bias[n]; b1 = p.bias[n + 1]; b2 = p.bias[n + 2]; b3 = p.bias[n + 3]; }
#pragma unroll
            for (int bm = 0; bm < MB; bm++) {
                const int m = m0 + wm0 + bm * 32 + li;
                if (m >= p.M) continue;
                const size_t o = (size_t)m * p.Ncols + n;
                float v0 = acc[bm][bn][4 * j], v1 = acc[bm][bn][4 * j + 1], v2 = acc[bm][bn][4 * j + 2], v3 = acc[bm][bn][4 * j + 3];
                if (part) {
                    *(float4 *)(pout + o) = make_float4(v0, v1, v2, v3);
                    continue;
                }
                if (!BWD) {
                    v0 += b0; v1 += b1; v2 += b2; v3 += b3;
                    if (p.flags & 2u) {
                        v0 = v0 > 0.f ? v0 : 0.f; v1 = v1 > 0.f ? v1 : 0.f;
                        v2 = v2 > 0.f ? v2 : 0.f; v3 = v3 > 0.f ? v3 : 0.f;
                    }
                } else if (p.xmask) {
                    const uint2 x = *(const uint2 *)((const uint16_t *)p.xmask + o);
                    if (!(bf16_to_f32((uint16_t)(x.x & 0xffffu)) > 0.f)) v0 = 0.f;
                    if (!(bf16_to_f32((uint16_t)(x.x >> 16)) > 0.f)) v1 = 0.f;
                    if (!(bf16_to_f32((uint16_t)(x.y & 0xffffu)) > 0.f)) v2 = 0.f;
                    if (!(bf16_to_f32((uint16_t)(x.y >> 16)) > 0.f)) v3 = 0.f;
                }
                *(uint2 *)(out + o) = make_uint2(f32x2_to_bf16x2(v0, v1), f32x2_to_bf16x2(v2, v3));
            }
        }
    }
}

#undef OWT_PIN_PHASE

}  // namespace owt
