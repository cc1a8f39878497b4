// Dense fp32 GEMM kernel of the fully-connected column shard (Section 4 of the paper: forward step 3,
// backward step 1; the shard of Section 4's model-parallel dense layers is a plain matrix product).
//
//   pass        C[M x N]            A                          B
//   forward     y[n][o]             x[n][i]   (K-major)        w[o][i]  (K-major)
//   bwd-data    dx[n][i]            dz[n][o]  (K-major)        w[o][i]  (MN-major: i contiguous)
//   bwd-filter  dw[o][i]            dz[n][o]  (MN-major)       x[n][i]  (MN-major)
//
// With a batch of 128 rows these products have few output tiles, so one work-group per CU has to hide
// the memory latency by itself: the operand tiles of a 32-deep reduction step go from global memory
// straight into LDS (global_load_lds, 16 bytes per lane, no register staging) into a ring of NS
// stages, NS - 1 steps ahead of the MFMAs, with one bare s_barrier per step and explicit counter waits (a
// __syncthreads() would wait for the loads in flight as well).  The load is written as inline assembly:
// the compiler keeps its own books on direct-to-LDS loads issued through the builtin and, with several
// stages in flight, puts a wait for all of them in front of the LDS reads of the stage that has landed.
//
// LDS layout.  A wavefront's direct-to-LDS load writes 1 KB contiguously in lane order, so padding is not
// available; the lanes permute what they fetch instead:
//   K-major tile   [row][32 values]: 16-byte piece c of a row sits in slot c ^ ((row >> 1) & 7), which
//                  spreads the ds_read_b128 of a fragment (32 rows, one piece) over all banks;
//   MN-major tile  [32 k][W values]: rows k with (k >> 2) & 1 set keep their 64-value groups with the
//                  halves swapped, so the two lane halves of a fragment read (rows k and k + 4, the
//                  same 32 columns) hit different banks.
// v_mfma_f32_32x32x2f32 takes one A and one B value per lane: lane (li, lh) supplies row / column li at
// reduction index 8*kc + 4*lh + jj for the jj-th of four MFMAs, for both layouts.
//
// Rows or columns past the end of an operand re-read its last row (last four columns): those results
// are never stored.  The host guarantees 16-byte aligned rows (pitches lda, ldb).  The reduction runs over
// whole steps of 32; when its true length kvalid is not a multiple of 32 (backward passes only: there A
// is the copy of dz that fc_dz_kernel pads with zeros) B's rows past kvalid re-read row kvalid - 1,
// which meets zeros of A.
#pragma once
#include "igemm.hpp"

namespace owt {

// One output tile (`tile` = tm * tiles_n + tn) over the reduction steps of `split`; lds holds NS stages.
template <bool AKM, bool BKM, class Epi, int WM, int WN, int MB, int NB, int NS>
__device__ __forceinline__ void fcgemm_tile(const GemmParams &p, int tile, int split, float *lds)
{
    constexpr int NW = WM * WN, BM = 32 * MB * WM, BN = 32 * NB * WN, BK = 32;
    constexpr int AI = BM / 8 / NW, BI = BN / 8 / NW;      // direct-to-LDS loads per lane and stage (1 KB per wavefront each)
    constexpr int L = AI + BI;
    static_assert((BM / 8) % NW == 0 && (BN / 8) % NW == 0, "every wavefront issues the same number of loads");
    static_assert(NS >= 3 && NS <= 5 && (NS - 2) * L <= 63, "the wait counter has six bits");
    constexpr int STAGE = (BM + BN) * BK;                  // floats: the A tile, then the B tile

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, lh = lane >> 5;
    const int wm0 = (wave / WN) * 32 * MB, wn0 = (wave % WN) * 32 * NB;
    const int tm = tile / p.tiles_n, tn = tile - tm * p.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const int ks_beg = split * p.ksteps_per_split;
    const int nst = min(p.ksteps, ks_beg + p.ksteps_per_split) - ks_beg;

    const float *ag = (const float *)p.a, *bg = (const float *)p.b;
    const int lda = p.lda, ldb = p.ldb;

    // element offsets of this lane's pieces of a stage (reduction step 0); kstep advances them
    int asrc[AI], bsrc[BI], btail[BKM ? 1 : BI];      // btail: B's pieces in the last step of the whole reduction
    const int klast = (p.ksteps - 1) * BK;
#pragma unroll
    for (int i = 0; i < AI; i++) {
        const int q = wave + NW * i;
        if (AKM) {
            const int row = 8 * q + (lane >> 3), piece = (lane & 7) ^ ((row >> 1) & 7);
            asrc[i] = min(m0 + row, p.M - 1) * lda + 4 * piece;
        } else {
            const int idx = q * 256 + 4 * lane, k = idx / BM, col = (idx % BM) ^ (((k >> 2) & 1) * 32);
            asrc[i] = k * lda + min(m0 + col, lda - 4);
        }
    }
#pragma unroll
    for (int i = 0; i < BI; i++) {
        const int q = wave + NW * i;
        if (BKM) {
            const int row = 8 * q + (lane >> 3), piece = (lane & 7) ^ ((row >> 1) & 7);
            bsrc[i] = min(n0 + row, p.Ncols - 1) * ldb + 4 * piece;
        } else {
            const int idx = q * 256 + 4 * lane, k = idx / BN, col = (idx % BN) ^ (((k >> 2) & 1) * 32);
            const int c = min(n0 + col, p.Ncols - 4);
            bsrc[i] = k * ldb + c;
            btail[i] = (min(klast + k, p.kvalid - 1) - klast) * ldb + c;
        }
    }
    const int astep = AKM ? BK : BK * lda, bstep = BKM ? BK : BK * ldb;

    // lane l's 16 bytes land at LDS byte address `dst` (wave-uniform, in m0) + 16 * l; the s_nop is the wait
    // state the hardware wants between a scalar write of m0 and a direct-to-LDS load that reads it
    auto dma16 = [&](const float *src, unsigned dst) __attribute__((always_inline)) {
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(dst) : "memory", "m0");
    };
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) float *)lds + wave * 1024;
    auto issue = [&](int ks, int buf) __attribute__((always_inline)) {
        const float *ap = ag + (size_t)ks * astep, *bp = bg + (size_t)ks * bstep;
        const unsigned da = lds0 + buf * (STAGE * 4), db = da + BM * BK * 4;
#pragma unroll
        for (int i = 0; i < AI; i++) dma16(ap + asrc[i], da + NW * i * 1024);
#pragma unroll
        for (int i = 0; i < BI; i++) dma16(bp + ((!BKM && ks == p.ksteps - 1) ? btail[i] : bsrc[i]), db + NW * i * 1024);
    };

    // fragment offsets (floats) of this lane within a stage
    int afr[AKM ? 4 : MB], bfr[BKM ? 4 : NB];
    if (AKM) {
#pragma unroll
        for (int kc = 0; kc < 4; kc++) afr[kc] = (wm0 + li) * BK + 4 * ((2 * kc + lh) ^ ((li >> 1) & 7));
    } else {
#pragma unroll
        for (int bm = 0; bm < MB; bm++) afr[bm] = 4 * lh * BM + ((wm0 + bm * 32 + li) ^ (32 * lh));
    }
    if (BKM) {
#pragma unroll
        for (int kc = 0; kc < 4; kc++) bfr[kc] = (wn0 + li) * BK + 4 * ((2 * kc + lh) ^ ((li >> 1) & 7));
    } else {
#pragma unroll
        for (int bn = 0; bn < NB; bn++) bfr[bn] = 4 * lh * BN + ((wn0 + bn * 32 + li) ^ (32 * lh));
    }

    float16v acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; i++)
#pragma unroll
        for (int j = 0; j < NB; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

    auto compute = [&](const float *sa, const float *sb) __attribute__((always_inline)) {
#pragma unroll
        for (int kc = 0; kc < 4; kc++) {
            float af[MB][4], bf[NB][4];
#pragma unroll
            for (int bm = 0; bm < MB; bm++) {
                if (AKM) {
                    const float4 v = *(const float4 *)(sa + afr[kc] + bm * 32 * BK);
                    af[bm][0] = v.x; af[bm][1] = v.y; af[bm][2] = v.z; af[bm][3] = v.w;
                } else {
#pragma unroll
                    for (int jj = 0; jj < 4; jj++) af[bm][jj] = sa[afr[bm] + (8 * kc + jj) * BM];
                }
            }
#pragma unroll
            for (int bn = 0; bn < NB; bn++) {
                if (BKM) {
                    const float4 v = *(const float4 *)(sb + bfr[kc] + bn * 32 * BK);
                    bf[bn][0] = v.x; bf[bn][1] = v.y; bf[bn][2] = v.z; bf[bn][3] = v.w;
                } else {
#pragma unroll
                    for (int jj = 0; jj < 4; jj++) bf[bn][jj] = sb[bfr[bn] + (8 * kc + jj) * BN];
                }
            }
#pragma unroll
            for (int jj = 0; jj < 4; jj++)
#pragma unroll
                for (int bm = 0; bm < MB; bm++)
#pragma unroll
                    for (int bn = 0; bn < NB; bn++)
                        acc[bm][bn] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[bm][jj], bf[bn][jj], acc[bm][bn], 0, 0, 0);
        }
    };

    // s_waitcnt vmcnt(n) lgkmcnt(0), expcnt untouched; n = this lane's loads of the stages that may stay in flight
#define OWT_WAIT_STAGES(k) __builtin_amdgcn_s_waitcnt((((k) * L) & 15) | ((((k) * L) >> 4) << 14) | (7 << 4))
#pragma unroll
    for (int i = 0; i < NS - 1; i++)
        if (i < nst) issue(ks_beg + i, i);
    int cur = 0, fill = NS - 1;                // stage s lives in buffer s % NS; `fill` is the buffer of stage s + NS - 1
    for (int s = 0; s < nst; s++) {
        // this lane's pieces of stage s have landed (up to NS - 2 later stages may still be in flight) and its
        // LDS reads of stage s - 1 are done; after the barrier that holds for the whole work-group, so stage s
        // can be read and the buffer of stage s - 1 refilled
        const int ahead = min(NS - 2, nst - 1 - s);
        if (ahead == 0) OWT_WAIT_STAGES(0);
        else if (ahead == 1) OWT_WAIT_STAGES(1);
        else if (ahead == 2) OWT_WAIT_STAGES(NS >= 4 ? 2 : 1);
        else OWT_WAIT_STAGES(NS >= 5 ? 3 : 1);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");         // no LDS read of stage s moves above the barrier
        if (s + NS - 1 < nst) issue(ks_beg + s + NS - 1, fill);
        compute(lds + cur * STAGE, lds + cur * STAGE + BM * BK);
        cur = cur == NS - 1 ? 0 : cur + 1;
        fill = fill == NS - 1 ? 0 : fill + 1;
    }
#undef OWT_WAIT_STAGES

    // accumulator register r of lane (li, lh): row 8*(r/4) + 4*lh + r%4, column li of its 32 x 32 block
    typedef typename Epi::TOut TOut;
    const bool part = p.splits > 1;
    float *pout = part ? p.partial + (size_t)split * p.M * p.Ncols : nullptr;
    TOut *out = (TOut *)p.out;
#pragma unroll
    for (int bm = 0; bm < MB; bm++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
            const int row = m0 + wm0 + bm * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
            if (row >= p.M) continue;
#pragma unroll
            for (int bn = 0; bn < NB; bn++) {
                const int col = n0 + wn0 + bn * 32 + li;
                if (col >= p.Ncols) continue;
                const size_t o = (size_t)row * p.Ncols + col;
                if (part) pout[o] = acc[bm][bn][r];
                else store1(out, o, Epi::op(p, row, col, acc[bm][bn][r]));
            }
        }
}

template <bool AKM, bool BKM, class Epi, int WM, int WN, int MB, int NB, int NS, int OCC>
__global__ void __launch_bounds__(64 * WM * WN, (OCC * WM * WN + 3) / 4) fcgemm_kernel(const GemmParams p)
{
    __shared__ __attribute__((aligned(16))) float lds[NS * 32 * (MB * WM + NB * WN) * 32];
    fcgemm_tile<AKM, BKM, Epi, WM, WN, MB, NB, NS>(p, blockIdx.x, blockIdx.y, lds);
}

// Both backward products of a shard in one launch (neither split): the first tiles_m * tiles_n work-groups
// of pd's grid compute dx, the rest dw.  Each product alone leaves CUs idle in its last round of
// work-groups; together the long dx tiles start first and the short dw tiles fill the gaps.
template <int WM, int WN, int MB, int NB, int NS, int OCC>
__global__ void __launch_bounds__(64 * WM * WN, (OCC * WM * WN + 3) / 4) fcgemm_bwd_pair_kernel(const GemmParams pd, const GemmParams pf)
{
    __shared__ __attribute__((aligned(16))) float lds[NS * 32 * (MB * WM + NB * WN) * 32];
    const int nd = pd.tiles_m * pd.tiles_n;
    if ((int)blockIdx.x < nd) fcgemm_tile<true, false, EpiData<float>, WM, WN, MB, NB, NS>(pd, blockIdx.x, 0, lds);
    else fcgemm_tile<false, false, EpiFilter, WM, WN, MB, NB, NS>(pf, blockIdx.x - nd, 0, lds);
}

// dz = dy where y > 0, else 0 (when y is given), written as an [Np][Op] array whose rows past N and columns
// past O are zero (when dz is given), and the bias gradient alpha * (column sums of dz) + beta * dbias (when
// dbias is given): 16 columns x 16 row phases per work-group, the phases added in a fixed order.  The whole
// array is a few hundred KB, so the kernel is one round trip to memory long: every thread has its (up to 8)
// rows in flight at once, and narrow column strips make enough work-groups for that.
__global__ void __launch_bounds__(256) fc_dz_kernel(const float *__restrict__ dy, const float *__restrict__ y,
                                                    float *__restrict__ dz, float *dbias, float alpha, float beta, int N, int O,
                                                    int Np, int Op)
{
    __shared__ float red[16][16];
    const int cl = threadIdx.x & 15, ph = threadIdx.x >> 4, c = blockIdx.x * 16 + cl;
    float s = 0.f;
    for (int n0 = ph; n0 < Np; n0 += 128) {
        float v[8], m[8];
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const int n = n0 + 16 * j;
            const bool in = n < N && c < O;
            v[j] = in ? dy[(size_t)n * O + c] : 0.f;
            m[j] = (in && y) ? y[(size_t)n * O + c] : 1.f;
        }
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const int n = n0 + 16 * j;
            const float t = m[j] > 0.f ? v[j] : 0.f;
            if (dz && n < Np && c < Op) dz[(size_t)n * Op + c] = t;
            s += t;
        }
    }
    red[ph][cl] = s;
    __syncthreads();
    if (ph == 0 && c < O && dbias) {
        float t = red[0][cl];
#pragma unroll
        for (int j = 1; j < 16; j++) t += red[j][cl];
        dbias[c] = alpha * t + (beta != 0.f ? beta * dbias[c] : 0.f);
    }
}

}  // namespace owt
