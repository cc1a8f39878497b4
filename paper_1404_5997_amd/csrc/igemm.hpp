// Implicit-GEMM convolution kernel for gfx950 (CDNA4), fp32 MFMA.
//
// One kernel template serves the three passes of a convolution layer
// (Section 4 of the paper: forward step 2, backward step 2) and, as the
// H = W = R = S = 1 case, the fully-connected column shard (forward step 3,
// backward step 1).  Each pass is C[M x N] = sum_kd A[m][kd] * B[kd][n] where
// the A and B elements are gathered straight from the NHWC / KRSC tensors:
//
//   pass        M        N        kd         A[m][kd]                B[kd][n]
//   forward     (n,p,q)  k        (r,s,c)    x[n,p*sh-ph+r,..,c]     w[k,r,s,c]
//   bwd-data    (n,h,w)  c        (r,s,k)    dz[n,(h+ph-r)/sh,..,k]  w[k,r,s,c]
//   bwd-filter  k        (r,s,c)  (n,p,q)    dz[n,p,q,k]             x[n,p*sh-ph+r,..,c]
//
// An operand is "K-major" when its 4-element vector loads run along kd and
// "MN-major" when they run along m (or n); the LDS tile keeps the direction of
// the global load, and the MFMA fragments are read with 16-byte (K-major) or
// 8-byte (MN-major) LDS reads.  v_mfma_f32_32x32x2f32 only needs A and B to
// agree on which kd a lane half supplies and lets rows/columns be any
// permutation, so both layouts feed it without a transpose.
//
// Work-group = WM x WN wavefronts of 64 lanes, each owning a 64 x 64 block of C
// (2 x 2 MFMA accumulators of 32 x 32).  Global -> register -> LDS staging is
// double buffered with one barrier per BK step.
#pragma once
#include "owt_common.hpp"

namespace owt {

typedef float float16v __attribute__((ext_vector_type(16)));

enum { kInvalidLo = -(1 << 29), kInvalidHi = (1 << 28) };

// ------------------------------------------------------------------ accessors
// fix(): state of the M (or N) index, computed once per thread.
// red(): state of the reduction index kd, computed every BK step.
// addr(): element offset of the (first of 4 contiguous) element(s), or -1 for a zero.

template <class T_> struct FwdA {   // A of the forward pass: im2col of x
    typedef T_ T;
    static constexpr bool KMAJOR = true;
    static constexpr bool MASKED = false;
    struct Fix { int base, h0, w0; };
    struct Red { int r, s, c; };
    static __device__ __forceinline__ Fix fix(const GemmParams &p, int m)
    {
        const Geom &g = p.g;
        Fix f;
        if (m >= p.M) { f.base = 0; f.h0 = kInvalidLo; f.w0 = 0; return f; }
        const int n = g.dPQ.div(m), pq = m - n * g.P * g.Q;
        const int pp = g.dQ.div(pq), q = pq - pp * g.Q;
        f.base = n * g.H * g.W * g.C;
        f.h0 = pp * g.sh - g.ph;
        f.w0 = q * g.sw - g.pw;
        return f;
    }
    static __device__ __forceinline__ Red red(const GemmParams &p, int kd)
    {
        const Geom &g = p.g;
        Red r;
        if (kd >= p.Kd) { r.r = kInvalidHi; r.s = 0; r.c = 0; return r; }
        const int rs = g.dC.div(kd);
        r.c = kd - rs * g.C;
        r.r = g.dS.div(rs);
        r.s = rs - r.r * g.S;
        return r;
    }
    static __device__ __forceinline__ int addr(const GemmParams &p, const Fix &f, const Red &r)
    {
        const Geom &g = p.g;
        const int h = f.h0 + r.r, w = f.w0 + r.s;
        if ((unsigned)h >= (unsigned)g.H || (unsigned)w >= (unsigned)g.W) return -1;
        return f.base + (h * g.W + w) * g.C + r.c;
    }
};

template <class T_> struct FwdB {   // B of the forward pass: filters, kd contiguous
    typedef T_ T;
    static constexpr bool KMAJOR = true;
    static constexpr bool MASKED = false;
    struct Fix { int base; };
    struct Red { int kd; };
    static __device__ __forceinline__ Fix fix(const GemmParams &p, int n)
    {
        Fix f; f.base = n < p.Ncols ? n * p.Kd : -1; return f;
    }
    static __device__ __forceinline__ Red red(const GemmParams &p, int kd)
    {
        Red r; r.kd = kd < p.Kd ? kd : -1; return r;
    }
    static __device__ __forceinline__ int addr(const GemmParams &, const Fix &f, const Red &r)
    {
        return (f.base | r.kd) < 0 ? -1 : f.base + r.kd;
    }
};

template <class T_> struct DataA {  // A of bwd-data: dz gathered at ((h+ph-r)/sh, (w+pw-s)/sw)
    typedef T_ T;
    static constexpr bool KMAJOR = true;
    static constexpr bool MASKED = true;
    struct Fix { int base, hp, wp; };
    struct Red { int r, s, k; };
    static __device__ __forceinline__ Fix fix(const GemmParams &p, int m)
    {
        const Geom &g = p.g;
        Fix f;
        if (m >= p.M) { f.base = 0; f.hp = kInvalidLo; f.wp = 0; return f; }
        const int n = g.dHW.div(m), hw = m - n * g.H * g.W;
        const int h = g.dW.div(hw), w = hw - h * g.W;
        f.base = n * g.P * g.Q * g.K;
        f.hp = h + g.ph;
        f.wp = w + g.pw;
        return f;
    }
    static __device__ __forceinline__ Red red(const GemmParams &p, int kd)
    {
        const Geom &g = p.g;
        Red r;
        if (kd >= p.Kd) { r.r = kInvalidHi; r.s = 0; r.k = 0; return r; }
        const int rs = g.dK.div(kd);
        r.k = kd - rs * g.K;
        r.r = g.dS.div(rs);
        r.s = rs - r.r * g.S;
        return r;
    }
    static __device__ __forceinline__ int addr(const GemmParams &p, const Fix &f, const Red &r)
    {
        const Geom &g = p.g;
        const int hh = f.hp - r.r, ww = f.wp - r.s;
        if ((hh | ww) < 0) return -1;
        int pp = hh, q = ww;
        if (g.sh != 1) { pp = g.dsh.div(hh); if (pp * g.sh != hh) return -1; }
        if (g.sw != 1) { q = g.dsw.div(ww); if (q * g.sw != ww) return -1; }
        if (pp >= g.P || q >= g.Q) return -1;
        return f.base + (pp * g.Q + q) * g.K + r.k;
    }
};

template <class T_> struct DataB {  // B of bwd-data: filters, c contiguous
    typedef T_ T;
    static constexpr bool KMAJOR = false;
    static constexpr bool MASKED = false;
    struct Fix { int c; };
    struct Red { int off; };
    static __device__ __forceinline__ Fix fix(const GemmParams &p, int n)
    {
        Fix f; f.c = n < p.Ncols ? n : -1; return f;
    }
    static __device__ __forceinline__ Red red(const GemmParams &p, int kd)
    {
        const Geom &g = p.g;
        Red r;
        if (kd >= p.Kd) { r.off = -1; return r; }
        const int rs = g.dK.div(kd);
        const int k = kd - rs * g.K;
        r.off = (k * g.R * g.S + rs) * g.C;
        return r;
    }
    static __device__ __forceinline__ int addr(const GemmParams &, const Fix &f, const Red &r)
    {
        return (f.c | r.off) < 0 ? -1 : r.off + f.c;
    }
};

template <class T_> struct FilterA {  // A of bwd-filter: dz, k contiguous
    typedef T_ T;
    static constexpr bool KMAJOR = false;
    static constexpr bool MASKED = true;
    struct Fix { int k; };
    struct Red { int off; };
    static __device__ __forceinline__ Fix fix(const GemmParams &p, int m)
    {
        Fix f; f.k = m < p.M ? m : -1; return f;
    }
    static __device__ __forceinline__ Red red(const GemmParams &p, int kd)
    {
        Red r; r.off = kd < p.Kd ? kd * p.g.K : -1; return r;
    }
    static __device__ __forceinline__ int addr(const GemmParams &, const Fix &f, const Red &r)
    {
        return (f.k | r.off) < 0 ? -1 : r.off + f.k;
    }
};

template <class T_> struct FilterB {  // B of bwd-filter: im2col of x, c contiguous
    typedef T_ T;
    static constexpr bool KMAJOR = false;
    static constexpr bool MASKED = false;
    struct Fix { int r, s, c; };
    struct Red { int base, h0, w0; };
    static __device__ __forceinline__ Fix fix(const GemmParams &p, int n)
    {
        const Geom &g = p.g;
        Fix f;
        if (n >= p.Ncols) { f.r = kInvalidHi; f.s = 0; f.c = 0; return f; }
        const int rs = g.dC.div(n);
        f.c = n - rs * g.C;
        f.r = g.dS.div(rs);
        f.s = rs - f.r * g.S;
        return f;
    }
    static __device__ __forceinline__ Red red(const GemmParams &p, int kd)
    {
        const Geom &g = p.g;
        Red r;
        if (kd >= p.Kd) { r.base = 0; r.h0 = kInvalidLo; r.w0 = 0; return r; }
        const int n = g.dPQ.div(kd), pq = kd - n * g.P * g.Q;
        const int pp = g.dQ.div(pq), q = pq - pp * g.Q;
        r.base = n * g.H * g.W * g.C;
        r.h0 = pp * g.sh - g.ph;
        r.w0 = q * g.sw - g.pw;
        return r;
    }
    static __device__ __forceinline__ int addr(const GemmParams &p, const Fix &f, const Red &r)
    {
        const Geom &g = p.g;
        const int h = r.h0 + f.r, w = r.w0 + f.s;
        if ((unsigned)h >= (unsigned)g.H || (unsigned)w >= (unsigned)g.W) return -1;
        return r.base + (h * g.W + w) * g.C + f.c;
    }
};

// ------------------------------------------------------------------ epilogues
template <class TOut_> struct EpiFwd {     // y = act(acc + bias)
    typedef TOut_ TOut;
    static constexpr bool DBIAS = false;
    static __device__ __forceinline__ float op(const GemmParams &p, int, int col, float v)
    {
        if (p.flags & 1u) v += p.bias[col];
        if (p.flags & 2u) v = v > 0.f ? v : 0.f;
        return v;
    }
};
template <class TOut_> struct EpiData {    // dx = acc, optionally zeroed where the layer's input is <= 0
    typedef TOut_ TOut;
    static constexpr bool DBIAS = false;
    static __device__ __forceinline__ float op(const GemmParams &p, int row, int col, float v)
    {
        if (p.xmask && !(load1((const TOut *)p.xmask, row * p.Ncols + col) > 0.f)) v = 0.f;
        return v;
    }
};
struct EpiFilter {                         // dw = alpha*acc + beta*dw
    typedef float TOut;
    static constexpr bool DBIAS = true;
    static __device__ __forceinline__ float op(const GemmParams &p, int row, int col, float v)
    {
        v *= p.alpha;
        if (p.beta != 0.f) v += p.beta * ((const float *)p.out)[(size_t)row * p.Ncols + col];
        return v;
    }
};

// --------------------------------------------------------------- tile loaders
// Register staging of one operand tile for one BK step.
template <class Acc, int VEC, int ROWS, int BK, int NT> struct TileLoader {
    typedef typename Acc::T T;
    static constexpr bool KMAJOR = Acc::KMAJOR;
    // K-major: tile is ROWS x BK, a thread owns quad kq of rows row0 + i*RPP.
    // MN-major: tile is BK x ROWS, a thread owns quad cq of k-rows krow0 + i*RPP.
    static constexpr int QUADS = KMAJOR ? BK / 4 : ROWS / 4;   // float4 per tile line
    static constexpr int RPP = NT / QUADS;                     // tile lines per pass
    static constexpr int LINES = KMAJOR ? ROWS : BK;
    static constexpr int NPASS = (LINES + RPP - 1) / RPP;
    static constexpr bool EXACT = (LINES % RPP) == 0;
    static constexpr int PITCH = KMAJOR ? BK + 4 : ROWS + 4;
    static constexpr int LDS_FLOATS = LINES * PITCH;
    static constexpr int NFIX = KMAJOR ? NPASS : 1;            // fixed-index states per thread
    static constexpr int NV = VEC == 4 ? 1 : 4;
    static_assert(NT % QUADS == 0, "thread count must be a multiple of the quads per line");

    typename Acc::Fix fx[NFIX][KMAJOR ? 1 : NV];
    float4 reg[NPASS];
    int line0, quad;

    __device__ __forceinline__ void init(const GemmParams &p, int origin, int tid)
    {
        quad = tid % QUADS;
        line0 = tid / QUADS;
        if constexpr (KMAJOR) {
#pragma unroll
            for (int i = 0; i < NPASS; i++) fx[i][0] = Acc::fix(p, origin + line0 + i * RPP);
        } else {
#pragma unroll
            for (int j = 0; j < NV; j++) fx[0][j] = Acc::fix(p, origin + quad * 4 + j);
        }
    }

    __device__ __forceinline__ float4 fetch4(const GemmParams &p, const T *src, int off)
    {
        if (off < 0) return make_float4(0.f, 0.f, 0.f, 0.f);
        float4 v = load4(src, off);
        if (Acc::MASKED && p.mask) {
            const float4 y = load4((const T *)p.mask, off);
            v.x = y.x > 0.f ? v.x : 0.f; v.y = y.y > 0.f ? v.y : 0.f;
            v.z = y.z > 0.f ? v.z : 0.f; v.w = y.w > 0.f ? v.w : 0.f;
        }
        return v;
    }
    __device__ __forceinline__ float fetch1(const GemmParams &p, const T *src, int off)
    {
        if (off < 0) return 0.f;
        float v = load1(src, off);
        if (Acc::MASKED && p.mask) v = load1((const T *)p.mask, off) > 0.f ? v : 0.f;
        return v;
    }

    // global -> registers for the BK step starting at reduction index k0
    __device__ __forceinline__ void load(const GemmParams &p, const T *src, int k0)
    {
        if constexpr (KMAJOR) {
            typename Acc::Red rd[NV];
#pragma unroll
            for (int j = 0; j < NV; j++) rd[j] = Acc::red(p, k0 + quad * 4 + j);
#pragma unroll
            for (int i = 0; i < NPASS; i++) {
                if (!EXACT && line0 + i * RPP >= LINES) { reg[i] = make_float4(0, 0, 0, 0); continue; }
                if (VEC == 4) {
                    reg[i] = fetch4(p, src, Acc::addr(p, fx[i][0], rd[0]));
                } else {
                    reg[i].x = fetch1(p, src, Acc::addr(p, fx[i][0], rd[0]));
                    reg[i].y = fetch1(p, src, Acc::addr(p, fx[i][0], rd[NV > 1 ? 1 : 0]));
                    reg[i].z = fetch1(p, src, Acc::addr(p, fx[i][0], rd[NV > 1 ? 2 : 0]));
                    reg[i].w = fetch1(p, src, Acc::addr(p, fx[i][0], rd[NV > 1 ? 3 : 0]));
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < NPASS; i++) {
                const int kl = line0 + i * RPP;
                if (!EXACT && kl >= LINES) { reg[i] = make_float4(0, 0, 0, 0); continue; }
                const typename Acc::Red rd = Acc::red(p, k0 + kl);
                if (VEC == 4) {
                    reg[i] = fetch4(p, src, Acc::addr(p, fx[0][0], rd));
                } else {
                    reg[i].x = fetch1(p, src, Acc::addr(p, fx[0][0], rd));
                    reg[i].y = fetch1(p, src, Acc::addr(p, fx[0][NV > 1 ? 1 : 0], rd));
                    reg[i].z = fetch1(p, src, Acc::addr(p, fx[0][NV > 1 ? 2 : 0], rd));
                    reg[i].w = fetch1(p, src, Acc::addr(p, fx[0][NV > 1 ? 3 : 0], rd));
                }
            }
        }
    }

    // registers -> LDS tile
    __device__ __forceinline__ void store(float *tile) const
    {
#pragma unroll
        for (int i = 0; i < NPASS; i++) {
            const int line = line0 + i * RPP;
            if (!EXACT && line >= LINES) continue;
            *(float4 *)(tile + line * PITCH + quad * 4) = reg[i];
        }
    }
};

// ------------------------------------------------------------------ epilogue
// Stores one wavefront's 64 x 64 block.  Accumulator register r of lane (li, lh) is
// row slot 8*(r/4) + 4*lh + r%4, column slot li of its 32 x 32 block; a K-major operand
// maps block b, slot t to index 32*b + t, an MN-major one to 2*t + b.
template <class Epi, bool AKM, bool BKM, int MB = 2>
__device__ __forceinline__ void tile_epilogue(const GemmParams &p, const float16v (&acc)[MB][2], int row0,
                                              int col0, int li, int lh, int split)
{
    typedef typename Epi::TOut TOut;
    const bool part = p.splits > 1;
    float *pout = part ? p.partial + (size_t)split * p.M * p.Ncols : nullptr;
    TOut *out = (TOut *)p.out;
    static_assert(AKM || MB == 2, "an MN-major A operand pairs its two row blocks");
#pragma unroll
    for (int bm = 0; bm < MB; bm++) {
#pragma unroll
        for (int r = 0; r < 16; r++) {
            const int rho = 8 * (r / 4) + 4 * lh + (r % 4);
            const int row = row0 + (AKM ? bm * 32 + rho : 2 * rho + bm);
            if (row >= p.M) continue;
            if (BKM) {
#pragma unroll
                for (int bn = 0; bn < 2; bn++) {
                    const int col = col0 + bn * 32 + li;
                    if (col >= p.Ncols) continue;
                    const size_t o = (size_t)row * p.Ncols + col;
                    if (part) pout[o] = acc[bm][bn][r];
                    else store1(out, o, Epi::op(p, row, col, acc[bm][bn][r]));
                }
            } else {
                const int col = col0 + 2 * li;
                const size_t o = (size_t)row * p.Ncols + col;
                const float v0 = acc[bm][0][r], v1 = acc[bm][1][r];
                if (col + 1 < p.Ncols && (p.Ncols & 1) == 0) {
                    if (part) *(float2 *)(pout + o) = make_float2(v0, v1);
                    else store2(out, o, Epi::op(p, row, col, v0), Epi::op(p, row, col + 1, v1));
                } else {
                    if (col < p.Ncols) {
                        if (part) pout[o] = v0; else store1(out, o, Epi::op(p, row, col, v0));
                    }
                    if (col + 1 < p.Ncols) {
                        if (part) pout[o + 1] = v1; else store1(out, o + 1, Epi::op(p, row, col + 1, v1));
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------- kernel
template <class A, class B, class Epi, int VA, int VB, int WM, int WN, int BK>
__global__ void __launch_bounds__(64 * WM * WN, 2) igemm_kernel(const GemmParams p)
{
    constexpr int NT = 64 * WM * WN, BM = 64 * WM, BN = 64 * WN;
    typedef TileLoader<A, VA, BM, BK, NT> LA;
    typedef TileLoader<B, VB, BN, BK, NT> LB;
    constexpr int STAGE = LA::LDS_FLOATS + LB::LDS_FLOATS;
    __shared__ __attribute__((aligned(16))) float lds[2 * STAGE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int wm0 = (wave / WN) * 64, wn0 = (wave % WN) * 64;

    // Work-groups are handed to the 8 XCDs round-robin; renumber them so that each
    // XCD walks a contiguous run of tiles (N tiles fastest) and its L2 sees one
    // A row panel at a time.
    const int ntiles = p.tiles_m * p.tiles_n;
    const int b = blockIdx.x, xcd = b & 7;
    const int logical = xcd * (ntiles >> 3) + min(xcd, ntiles & 7) + (b >> 3);
    const int tm = logical / p.tiles_n, tn = logical - tm * p.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const int split = blockIdx.y;
    const int ks_beg = split * p.ksteps_per_split;
    const int ks_end = min(p.ksteps, ks_beg + p.ksteps_per_split);

    LA la; LB lb;
    la.init(p, m0, tid);
    lb.init(p, n0, tid);
    const typename A::T *asrc = (const typename A::T *)p.a;
    const typename B::T *bsrc = (const typename B::T *)p.b;

    float16v acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

    float4 dbacc = make_float4(0.f, 0.f, 0.f, 0.f);
    const bool do_db = Epi::DBIAS && tn == 0 && p.dbias != nullptr;

    if (ks_beg < ks_end) {
        la.load(p, asrc, ks_beg * BK);
        lb.load(p, bsrc, ks_beg * BK);
        la.store(lds);
        lb.store(lds + LA::LDS_FLOATS);
    }
    __syncthreads();

    int cur = 0;
    for (int ks = ks_beg; ks < ks_end; ks++) {
        if (Epi::DBIAS && do_db) {
#pragma unroll
            for (int i = 0; i < LA::NPASS; i++) {
                dbacc.x += la.reg[i].x; dbacc.y += la.reg[i].y;
                dbacc.z += la.reg[i].z; dbacc.w += la.reg[i].w;
            }
        }
        const bool more = ks + 1 < ks_end;
        if (more) {
            la.load(p, asrc, (ks + 1) * BK);
            lb.load(p, bsrc, (ks + 1) * BK);
        }
        const float *As = lds + cur * STAGE;
        const float *Bs = As + LA::LDS_FLOATS;
#pragma unroll
        for (int kc = 0; kc < BK / 8; kc++) {
            float af[2][4], bf[2][4];
            if (A::KMAJOR) {
#pragma unroll
                for (int bm = 0; bm < 2; bm++) {
                    const float4 v = *(const float4 *)(As + (wm0 + bm * 32 + li) * LA::PITCH + kc * 8 + lh * 4);
                    af[bm][0] = v.x; af[bm][1] = v.y; af[bm][2] = v.z; af[bm][3] = v.w;
                }
            } else {
#pragma unroll
                for (int jj = 0; jj < 4; jj++) {
                    const float2 v = *(const float2 *)(As + (kc * 8 + lh * 4 + jj) * LA::PITCH + wm0 + 2 * li);
                    af[0][jj] = v.x; af[1][jj] = v.y;
                }
            }
            if (B::KMAJOR) {
#pragma unroll
                for (int bn = 0; bn < 2; bn++) {
                    const float4 v = *(const float4 *)(Bs + (wn0 + bn * 32 + li) * LB::PITCH + kc * 8 + lh * 4);
                    bf[bn][0] = v.x; bf[bn][1] = v.y; bf[bn][2] = v.z; bf[bn][3] = v.w;
                }
            } else {
#pragma unroll
                for (int jj = 0; jj < 4; jj++) {
                    const float2 v = *(const float2 *)(Bs + (kc * 8 + lh * 4 + jj) * LB::PITCH + wn0 + 2 * li);
                    bf[0][jj] = v.x; bf[1][jj] = v.y;
                }
            }
#pragma unroll
            for (int jj = 0; jj < 4; jj++)
#pragma unroll
                for (int bm = 0; bm < 2; bm++)
#pragma unroll
                    for (int bn = 0; bn < 2; bn++)
                        acc[bm][bn] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[bm][jj], bf[bn][jj], acc[bm][bn], 0, 0, 0);
        }
        if (more) {
            float *nxt = lds + (cur ^ 1) * STAGE;
            la.store(nxt);
            lb.store(nxt + LA::LDS_FLOATS);
        }
        __syncthreads();
        cur ^= 1;
    }

    tile_epilogue<Epi, A::KMAJOR, B::KMAJOR>(p, acc, m0 + wm0, n0 + wn0, li, lh, split);

    if (Epi::DBIAS) {
        // Column sums of the dz tile: threads sharing a quad add up through LDS.
        if (do_db) {   // uniform over the work-group
            constexpr int G = LA::RPP;   // threads per quad
            float *red = lds;            // all waves passed the last barrier of the k loop
            *(float4 *)(red + la.line0 * BM + la.quad * 4) = dbacc;
            __syncthreads();
            if (tid < BM && m0 + tid < p.M) {
                float s = 0.f;
                for (int j = 0; j < G; j++) s += red[j * BM + tid];
                const int k = m0 + tid;
                if (p.splits > 1) p.dbias_partial[(size_t)split * p.M + k] = s;
                else p.dbias[k] = p.alpha * s + (p.beta != 0.f ? p.beta * p.dbias[k] : 0.f);
            }
        }
    }
}

// Sum the split-K partials and apply the epilogue: out[i] = op(sum_s partial[s][i]).
// The sum over splits always runs in the same order, so results are bit-identical run to run.
// Four consecutive results per thread (16-byte loads of every partial), SG threads per group of
// four, each summing every SG-th split with several loads in flight and combined through LDS in a
// fixed order: SG = 1 for few splits of a big result, 4 / 16 for the many splits of a small one
// (a filter gradient reduced over hundreds of work-groups).  The bias-gradient partials are summed
// by one work-group per filter.  Needs M*N to be a multiple of 4; SG == 0 is the scalar kernel for
// the other shapes.
template <class Epi, int SG>
__global__ void __launch_bounds__(256) splitk_reduce_kernel(const GemmParams p)
{
    typedef typename Epi::TOut TOut;
    const size_t total = (size_t)p.M * p.Ncols;
    if constexpr (SG == 0) {
        for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
            float s = 0.f;
            for (int sp = 0; sp < p.splits; sp++) s += p.partial[(size_t)sp * total + i];
            const int row = (int)(i / p.Ncols), col = (int)(i - (size_t)row * p.Ncols);
            store1((TOut *)p.out, i, Epi::op(p, row, col, s));
        }
    } else {
        constexpr int EPB = 256 / SG;                          // groups of four results per block
        __shared__ float4 red[SG][EPB];
        const size_t nvec = total >> 2;
        const int e = threadIdx.x % EPB, sg = threadIdx.x / EPB;
        for (size_t v0 = (size_t)blockIdx.x * EPB; v0 < nvec; v0 += (size_t)gridDim.x * EPB) {
            const size_t v = v0 + e;
            float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
            if (v < nvec) {
#pragma unroll 4
                for (int sp = sg; sp < p.splits; sp += SG) {
                    const float4 t = *(const float4 *)(p.partial + (size_t)sp * total + 4 * v);
                    s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
                }
            }
            if (SG > 1) {
                red[sg][e] = s;
                __syncthreads();
                if (sg == 0) {
                    s = red[0][e];
#pragma unroll
                    for (int j = 1; j < SG; j++) { const float4 t = red[j][e]; s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w; }
                }
            }
            if (sg == 0 && v < nvec) {
                const float r[4] = {s.x, s.y, s.z, s.w};
                const size_t i = 4 * v;
                int row = (int)(i / p.Ncols), col = (int)(i - (size_t)row * p.Ncols);
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    store1((TOut *)p.out, i + j, Epi::op(p, row, col, r[j]));
                    if (++col == p.Ncols) { col = 0; row++; }
                }
            }
            if (SG > 1) __syncthreads();
        }
    }
    if (Epi::DBIAS && p.dbias) {
        __shared__ float rb[256];
        for (int k = blockIdx.x; k < p.M; k += gridDim.x) {
            float s = 0.f;
            for (int sp = threadIdx.x; sp < p.splits; sp += 256) s += p.dbias_partial[(size_t)sp * p.M + k];
            rb[threadIdx.x] = s;
            __syncthreads();
#pragma unroll
            for (int d = 128; d >= 1; d >>= 1) {
                if ((int)threadIdx.x < d) rb[threadIdx.x] += rb[threadIdx.x + d];
                __syncthreads();
            }
            if (threadIdx.x == 0) p.dbias[k] = p.alpha * rb[0] + (p.beta != 0.f ? p.beta * p.dbias[k] : 0.f);
            __syncthreads();
        }
    }
}

template <class Epi>
static inline hipError_t launch_splitk_reduce(const GemmParams &p, hipStream_t s)
{
    const size_t total = (size_t)p.M * p.Ncols;
    if (total % 4 != 0) {
        size_t blocks = (total + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL((splitk_reduce_kernel<Epi, 0>), dim3((unsigned)blocks), dim3(256), 0, s, p);
        return hipGetLastError();
    }
    const size_t nvec = total / 4;
    auto blocks_for = [&](int epb) { const size_t b = (nvec + epb - 1) / epb; return (unsigned)(b > 16384 ? 16384 : b); };
    if (p.splits <= 6) hipLaunchKernelGGL((splitk_reduce_kernel<Epi, 1>), dim3(blocks_for(256)), dim3(256), 0, s, p);
    else if (p.splits <= 32) hipLaunchKernelGGL((splitk_reduce_kernel<Epi, 4>), dim3(blocks_for(64)), dim3(256), 0, s, p);
    else hipLaunchKernelGGL((splitk_reduce_kernel<Epi, 16>), dim3(blocks_for(16)), dim3(256), 0, s, p);
    return hipGetLastError();
}

// Filters re-laid-out for a backward-data pass that wants them contiguous along its reduction
// index k, with the taps flipped:  wt[(c*RS + t)*K + k] = w[(k*RS + RS-1-t)*C + c]
template <class T>
__global__ void __launch_bounds__(256) flip_transpose_filters_kernel(const T *__restrict__ w, T *__restrict__ wt, int K,
                                                                     int RS, int C)
{
    const int total = K * RS * C;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < total; i += gridDim.x * 256) {
        const int k = i % K, ct = i / K, t = ct % RS, c = ct / RS;
        wt[i] = w[(k * RS + (RS - 1 - t)) * C + c];
    }
}

}  // namespace owt
