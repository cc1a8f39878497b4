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
//   * the one barrier per tap sits between the two phases: the filter slice of tap t+1 is stored
//     before it, the first fragments of tap t+1 are read after it, the global load of the slice of
//     tap t+2 is issued after it and has a whole tap to arrive.
// The accumulators hold the TRANSPOSED tile (filters along MFMA rows, pixels along columns): a lane
// then owns four consecutive filters of one pixel and stores 8 bytes at a time.
#pragma once
#include "dconv_bf16.hpp"

namespace owt {

template <class Epi, bool BWD, int PR>
__global__ void __launch_bounds__(256, 2) dconv16p_kernel(const GemmParams p)
{
    constexpr int BK = 32, NT = 256, MB = 4, BM = 512, BN = 64, PITCH = BK + 8;   // bf16 elements: 80-byte rows
    constexpr int OCTS = BK / 8, RPP = NT / OCTS, PNP = (PR + RPP - 1) / RPP;
    constexpr int BT = BN * PITCH;
    static_assert(BN * OCTS == NT, "one 16-byte piece of the filter slice per thread");

    __shared__ __attribute__((aligned(16))) uint16_t lds[2 * BT + (PR + 1) * PITCH];
    uint16_t *panel = lds + 2 * BT;

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

    int hh[MB], ww[MB], prow[MB];
#pragma unroll
    for (int bm = 0; bm < MB; bm++) {
        const int m = m0 + wm0 + bm * 32 + li;
        if (m < p.M) prow[bm] = pin(m, hh[bm], ww[bm]) - ps;
        else { hh[bm] = kInvalidLo; ww[bm] = 0; prow[bm] = 0; }
    }

    const uint16_t *in = (const uint16_t *)p.a, *wsrc = (const uint16_t *)p.b, *mask = (const uint16_t *)p.mask;
    const int oct = tid % OCTS, line0 = tid / OCTS;
    uint4 preg[PNP], breg;
    const uint4 zero4 = make_uint4(0u, 0u, 0u, 0u);

    auto load_panel = [&](int ch) {
        const int c = ch * BK + oct * 8;
#pragma unroll
        for (int i = 0; i < PNP; i++) {
            const int row = line0 + i * RPP, pix = ps + row;
            uint4 v = zero4;
            if (row < nrows && (unsigned)pix < (unsigned)npix_in && c < Cred) {
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
    auto store_panel = [&]() {
#pragma unroll
        for (int i = 0; i < PNP; i++) {
            const int row = line0 + i * RPP;
            if (row < PR) *(uint4 *)(panel + row * PITCH + oct * 8) = preg[i];
        }
    };
    // line = output column (a filter in forward, an input channel in backward-data), oct along the reduction
    const bool bline_ok = n0 + line0 < p.Ncols;
    const uint16_t *bsrc = wsrc + (size_t)(bline_ok ? n0 + line0 : 0) * RS * Cred + oct * 8;
    auto load_b = [&](int ch, int tap) {
        uint4 v = zero4;
        if (bline_ok && ch * BK + oct * 8 < Cred) v = *(const uint4 *)(bsrc + tap * Cred + ch * BK);
        breg = v;
    };
    const int bst = line0 * PITCH + oct * 8;
    auto frag = [&](const uint16_t *q) { return __builtin_bit_cast(bf16x8, *(const uint4 *)q); };
    auto tap_offsets = [&](int r, int s, int (&aoff)[MB]) {
#pragma unroll
        for (int bm = 0; bm < MB; bm++) {
            const bool ok = (unsigned)(hh[bm] + r) < (unsigned)Hi && (unsigned)(ww[bm] + s) < (unsigned)Wi;
            aoff[bm] = (ok ? prow[bm] + r * Wi + s : PR) * PITCH + lh * 8;
        }
    };

    // order of a phase as the hardware should see it: the two filter-fragment reads, then four times
    // (two MFMAs, one pixel-fragment read); the compiler's own order bunches the reads behind the MFMAs
    auto pin_schedule = [&]() {
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
        for (int bm = 0; bm < MB; bm++) {
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
    };

    float16v acc[MB][2];
#pragma unroll
    for (int i = 0; i < MB; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

    const int nsteps = (ch_end - ch_beg) * RS;                  // one step per (chunk, tap)
    if (tid < PITCH) panel[PR * PITCH + tid] = 0;               // the row of zeros
    if (nsteps > 0) {
        load_panel(ch_beg);
        load_b(ch_beg, 0);
        store_panel();
        *(uint4 *)(lds + bst) = breg;
    }
    __syncthreads();

    if (nsteps > 0) {
        const int boff0 = li * PITCH + lh * 8, boff1 = boff0 + 32 * PITCH;
        bf16x8 af[MB], bf[2][2];
        int aoff[MB];
        tap_offsets(0, 0, aoff);
#pragma unroll
        for (int bm = 0; bm < MB; bm++) af[bm] = frag(panel + aoff[bm]);
        bf[0][0] = frag(lds + boff0);
        bf[0][1] = frag(lds + boff1);
        // the slice of step 1 (guards inside load_b keep a step past the end harmless)
        int ch = ch_beg, tap = 0, r = 0, s = 0;
        load_b(RS > 1 ? ch : ch + 1, RS > 1 ? 1 : 0);

        int cur = 0;
        for (int t = 0; t < nsteps; t++) {
            const bool swap_panel = tap == RS - 1 && t + 1 < nsteps;    // the next step starts a new chunk
            const uint16_t *Bs = lds + cur * BT;
            uint16_t *Bn = lds + (cur ^ 1) * BT;

            // phase 0: channels 0..15 of the chunk; fetch the fragments of channels 16..31
            bf[1][0] = frag(Bs + boff0 + 16);
            bf[1][1] = frag(Bs + boff1 + 16);
#pragma unroll
            for (int bm = 0; bm < MB; bm++) {
                acc[bm][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[0][0], af[bm], acc[bm][0], 0, 0, 0);
                acc[bm][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[0][1], af[bm], acc[bm][1], 0, 0, 0);
                af[bm] = frag(panel + aoff[bm] + 16);
            }
            pin_schedule();
            if (swap_panel) {
                __syncthreads();                                 // every wave has its last fragments of the old panel
                store_panel();
            }
            *(uint4 *)(Bn + bst) = breg;                         // slice of step t+1
            __syncthreads();

            // coordinates of steps t+1 and t+2
            int tap1 = tap + 1, ch1 = ch, r1 = r, s1 = s + 1;
            if (s1 == S) { s1 = 0; r1++; }
            if (tap1 == RS) { tap1 = 0; ch1++; r1 = 0; s1 = 0; }
            int tap2 = tap1 + 1, ch2 = ch1;
            if (tap2 == RS) { tap2 = 0; ch2++; }

            // phase 1: channels 16..31; fetch the first fragments of step t+1
            load_b(ch2, tap2);
            if (tap == 0 && ch + 1 < ch_end) load_panel(ch + 1);  // held in registers until the last tap
            tap_offsets(r1, s1, aoff);
            bf[0][0] = frag(Bn + boff0);
            bf[0][1] = frag(Bn + boff1);
#pragma unroll
            for (int bm = 0; bm < MB; bm++) {
                acc[bm][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[1][0], af[bm], acc[bm][0], 0, 0, 0);
                acc[bm][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[1][1], af[bm], acc[bm][1], 0, 0, 0);
                af[bm] = frag(panel + aoff[bm]);
            }
            pin_schedule();
            cur ^= 1; tap = tap1; ch = ch1; r = r1; s = s1;
        }
    }

    // epilogue: register 4j+i of accumulator (bm, bn) is pixel 32*bm + li, filter 32*bn + 8j + 4*lh + i
    const bool part = p.splits > 1;
    float *pout = part ? p.partial + (size_t)split * p.M * p.Ncols : nullptr;
    uint16_t *out = (uint16_t *)p.out;
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

}  // namespace owt
