// Max pooling forward/backward, NHWC, HBM-bound: one thread per 4 channels (or 1
// when C is not a multiple of 4), consecutive threads on consecutive channels.
#include "owt_host.hpp"

namespace owt {

// WS = 0: window and stride at run time; WS = 3: the 3x3 stride-2 pooling of the Section 5 model, with the
// nine loads of a window unrolled (all in flight before the first comparison).
template <class T, int V, int WS = 0>
__global__ void __launch_bounds__(256) maxpool_fwd_kernel(const T *__restrict__ x, T *__restrict__ y,
                                                          unsigned char *__restrict__ am, int N, int H, int W,
                                                          int C, int win_, int st_, int P, int Q, FastDiv dCv,
                                                          FastDiv dQ, FastDiv dP)
{
    const int win = WS ? 3 : win_, st = WS ? 2 : st_;
    const int Cv = C / V;
    const long total = (long)N * P * Q * Cv;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int pix = dCv.div((uint32_t)i), cv = (int)i - pix * Cv;
        const int np = dQ.div(pix), q = pix - np * Q;
        const int n = dP.div(np), p = np - n * P;
        const int c = cv * V;
        float best[V]; int bi[V];
        const int base = ((n * H + p * st) * W + q * st) * C + c;
        if constexpr (WS == 3 && V == 4) {
            float4 t[9];
#pragma unroll
            for (int rs = 0; rs < 9; rs++) t[rs] = load4(x, base + ((rs / 3) * W + rs % 3) * C);
#pragma unroll
            for (int rs = 0; rs < 9; rs++) {
                const float v[4] = {t[rs].x, t[rs].y, t[rs].z, t[rs].w};
#pragma unroll
                for (int j = 0; j < 4; j++)
                    if (rs == 0 || v[j] > best[j]) { best[j] = v[j]; bi[j] = rs; }
            }
        } else {
            for (int r = 0; r < win; r++)
                for (int s = 0; s < win; s++) {
                    const int off = base + (r * W + s) * C;
                    float v[V];
                    if constexpr (V == 4) { const float4 t = load4(x, off); v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w; }
                    else v[0] = load1(x, off);
#pragma unroll
                    for (int j = 0; j < V; j++)
                        if ((r | s) == 0 || v[j] > best[j]) { best[j] = v[j]; bi[j] = r * win + s; }
                }
        }
        const size_t o = (size_t)pix * C + c;
#pragma unroll
        for (int j = 0; j < V; j++) store1(y, o + j, best[j]);
        if constexpr (V == 4)       // c is a multiple of 4 and so is C: one aligned 4-byte store of the four arg-max codes
            *(uint32_t *)(am + o) = (uint32_t)bi[0] | ((uint32_t)bi[1] << 8) | ((uint32_t)bi[2] << 16) | ((uint32_t)bi[3] << 24);
        else
            am[o] = (unsigned char)bi[0];
    }
}

template <class T, int V>
__global__ void __launch_bounds__(256) maxpool_bwd_kernel(const T *__restrict__ dy,
                                                          const unsigned char *__restrict__ am,
                                                          const T *__restrict__ yp, T *__restrict__ dx,
                                                          int N, int H, int W, int C, int win, int st, int P, int Q,
                                                          FastDiv dCv, FastDiv dW, FastDiv dH, FastDiv dst)
{
    const int Cv = C / V;
    const long total = (long)N * H * W * Cv;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int pix = dCv.div((uint32_t)i), cv = (int)i - pix * Cv;
        const int nh = dW.div(pix), w = pix - nh * W;
        const int n = dH.div(nh), h = nh - n * H;
        const int c = cv * V;
        // windows p with p*st <= h <= p*st + win - 1
        const int p_hi = min(P - 1, (int)dst.div(h)), q_hi = min(Q - 1, (int)dst.div(w));
        const int p_lo = h >= win ? (int)dst.div(h - win + st) : 0;   // ceil((h-win+1)/st)
        const int q_lo = w >= win ? (int)dst.div(w - win + st) : 0;
        float acc[V];
#pragma unroll
        for (int j = 0; j < V; j++) acc[j] = 0.f;
        for (int p = p_lo; p <= p_hi; p++)
            for (int q = q_lo; q <= q_hi; q++) {
                const int code = (h - p * st) * win + (w - q * st);
                const int off = ((n * P + p) * Q + q) * C + c;
                if constexpr (V == 4) {
                    const uint32_t a4 = *(const uint32_t *)(am + off);
                    float4 g = load4(dy, off);
                    if (yp) {   // fused ReLU backward: a window whose maximum is <= 0 passes nothing
                        const float4 y = load4(yp, off);
                        g.x = y.x > 0.f ? g.x : 0.f; g.y = y.y > 0.f ? g.y : 0.f;
                        g.z = y.z > 0.f ? g.z : 0.f; g.w = y.w > 0.f ? g.w : 0.f;
                    }
                    if ((int)(a4 & 255u) == code) acc[0] += g.x;
                    if ((int)((a4 >> 8) & 255u) == code) acc[1] += g.y;
                    if ((int)((a4 >> 16) & 255u) == code) acc[2] += g.z;
                    if ((int)(a4 >> 24) == code) acc[3] += g.w;
                } else if ((int)am[off] == code) {
                    if (!yp || load1(yp, off) > 0.f) acc[0] += load1(dy, off);
                }
            }
        const size_t o = (size_t)pix * C + c;
#pragma unroll
        for (int j = 0; j < V; j++) store1(dx, o + j, acc[j]);
    }
}

// bf16 storage with C a multiple of 8: eight channels per thread, 16-byte accesses (8 bytes of arg-max).
__device__ __forceinline__ void unpack8(const uint4 v, float (&f)[8])
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; j++) { f[2 * j] = __uint_as_float(w[j] << 16); f[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u); }
}

template <int WS>
__global__ void __launch_bounds__(256) maxpool_fwd_bf16x8_kernel(const uint16_t *__restrict__ x, uint16_t *__restrict__ y,
                                                                 unsigned char *__restrict__ am, int N, int H, int W, int C,
                                                                 int win_, int st_, int P, int Q, FastDiv dCv, FastDiv dQ, FastDiv dP)
{
    const int win = WS ? 3 : win_, st = WS ? 2 : st_;
    const int Cv = C / 8;
    const long total = (long)N * P * Q * Cv;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int pix = dCv.div((uint32_t)i), cv = (int)i - pix * Cv;
        const int np = dQ.div(pix), q = pix - np * Q;
        const int n = dP.div(np), p = np - n * P;
        const int c = cv * 8;
        float best[8]; uint32_t bits[8]; int bi[8];
        const int base = ((n * H + p * st) * W + q * st) * C + c;
        if constexpr (WS == 3) {
            uint4 raw[9];
#pragma unroll
            for (int rs = 0; rs < 9; rs++) raw[rs] = *(const uint4 *)(x + base + ((rs / 3) * W + rs % 3) * C);
#pragma unroll
            for (int rs = 0; rs < 9; rs++) {
                float v[8];
                unpack8(raw[rs], v);
#pragma unroll
                for (int j = 0; j < 8; j++)
                    if (rs == 0 || v[j] > best[j]) { best[j] = v[j]; bi[j] = rs; bits[j] = __float_as_uint(v[j]) >> 16; }
            }
        } else {
            for (int r = 0; r < win; r++)
                for (int s = 0; s < win; s++) {
                    const uint4 raw = *(const uint4 *)(x + base + (r * W + s) * C);
                    float v[8];
                    unpack8(raw, v);
#pragma unroll
                    for (int j = 0; j < 8; j++)
                        if ((r | s) == 0 || v[j] > best[j]) { best[j] = v[j]; bi[j] = r * win + s; bits[j] = __float_as_uint(v[j]) >> 16; }
                }
        }
        const size_t o = (size_t)pix * C + c;
        uint4 out;                       // the maxima are input values: their bf16 bits are copied, not re-rounded
        out.x = bits[0] | (bits[1] << 16); out.y = bits[2] | (bits[3] << 16);
        out.z = bits[4] | (bits[5] << 16); out.w = bits[6] | (bits[7] << 16);
        *(uint4 *)(y + o) = out;
        uint2 a;
        a.x = (uint32_t)bi[0] | ((uint32_t)bi[1] << 8) | ((uint32_t)bi[2] << 16) | ((uint32_t)bi[3] << 24);
        a.y = (uint32_t)bi[4] | ((uint32_t)bi[5] << 8) | ((uint32_t)bi[6] << 16) | ((uint32_t)bi[7] << 24);
        *(uint2 *)(am + o) = a;
    }
}

__global__ void __launch_bounds__(256) maxpool_bwd_bf16x8_kernel(const uint16_t *__restrict__ dy, const unsigned char *__restrict__ am,
                                                                 const uint16_t *__restrict__ yp, uint16_t *__restrict__ dx,
                                                                 int N, int H, int W, int C, int win, int st, int P, int Q,
                                                                 FastDiv dCv, FastDiv dW, FastDiv dH, FastDiv dst)
{
    const int Cv = C / 8;
    const long total = (long)N * H * W * Cv;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int pix = dCv.div((uint32_t)i), cv = (int)i - pix * Cv;
        const int nh = dW.div(pix), w = pix - nh * W;
        const int n = dH.div(nh), h = nh - n * H;
        const int c = cv * 8;
        const int p_hi = min(P - 1, (int)dst.div(h)), q_hi = min(Q - 1, (int)dst.div(w));
        const int p_lo = h >= win ? (int)dst.div(h - win + st) : 0;
        const int q_lo = w >= win ? (int)dst.div(w - win + st) : 0;
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; j++) acc[j] = 0.f;
        for (int p = p_lo; p <= p_hi; p++)
            for (int q = q_lo; q <= q_hi; q++) {
                const int code = (h - p * st) * win + (w - q * st);
                const int off = ((n * P + p) * Q + q) * C + c;
                const uint2 a8 = *(const uint2 *)(am + off);
                float gv[8];
                unpack8(*(const uint4 *)(dy + off), gv);
                if (yp) {   // fused ReLU backward: a window whose maximum is <= 0 passes nothing
                    float yv[8];
                    unpack8(*(const uint4 *)(yp + off), yv);
#pragma unroll
                    for (int j = 0; j < 8; j++) gv[j] = yv[j] > 0.f ? gv[j] : 0.f;
                }
#pragma unroll
                for (int j = 0; j < 8; j++) {
                    const uint32_t aw = j < 4 ? a8.x : a8.y;
                    if ((int)((aw >> (8 * (j & 3))) & 255u) == code) acc[j] += gv[j];
                }
            }
        uint4 out;
        out.x = f32x2_to_bf16x2(acc[0], acc[1]); out.y = f32x2_to_bf16x2(acc[2], acc[3]);
        out.z = f32x2_to_bf16x2(acc[4], acc[5]); out.w = f32x2_to_bf16x2(acc[6], acc[7]);
        *(uint4 *)(dx + (size_t)pix * C + c) = out;
    }
}

// Backward pass specialised for the 3x3 window, stride 2 pooling of the Section 5 model.  A thread
// owns a 2x2 block of dx (rows 2a, 2a+1, columns 2b, 2b+1) and V channels: only the four windows
// (a-1..a, b-1..b) can route a gradient into it, so every window is read once per block instead of
// once per input element (2.25x less cache traffic than the gather above).  Window (p, q) with
// arg-max code 3r+s sends its gradient to input (2p+r, 2q+s).
template <class T, int V> struct PoolVec;
template <> struct PoolVec<float, 4> {
    static __device__ __forceinline__ void load(const float *p, size_t off, float (&f)[4])
    {
        const float4 v = *(const float4 *)(p + off);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
    static __device__ __forceinline__ void store(float *p, size_t off, const float (&f)[4])
    {
        *(float4 *)(p + off) = make_float4(f[0], f[1], f[2], f[3]);
    }
    static __device__ __forceinline__ void codes(const unsigned char *am, size_t off, int (&c)[4])
    {
        const uint32_t a = *(const uint32_t *)(am + off);
        c[0] = a & 255u; c[1] = (a >> 8) & 255u; c[2] = (a >> 16) & 255u; c[3] = a >> 24;
    }
};
template <> struct PoolVec<bf16_t, 8> {
    static __device__ __forceinline__ void load(const bf16_t *p, size_t off, float (&f)[8])
    {
        unpack8(*(const uint4 *)((const uint16_t *)p + off), f);
    }
    static __device__ __forceinline__ void store(bf16_t *p, size_t off, const float (&f)[8])
    {
        uint4 o;
        o.x = f32x2_to_bf16x2(f[0], f[1]); o.y = f32x2_to_bf16x2(f[2], f[3]);
        o.z = f32x2_to_bf16x2(f[4], f[5]); o.w = f32x2_to_bf16x2(f[6], f[7]);
        *(uint4 *)((uint16_t *)p + off) = o;
    }
    static __device__ __forceinline__ void codes(const unsigned char *am, size_t off, int (&c)[8])
    {
        const uint2 a = *(const uint2 *)(am + off);
#pragma unroll
        for (int j = 0; j < 8; j++) c[j] = ((j < 4 ? a.x : a.y) >> (8 * (j & 3))) & 255u;
    }
};

template <class T, int V>
__global__ void __launch_bounds__(256) maxpool_bwd_w3s2_kernel(const T *__restrict__ dy, const unsigned char *__restrict__ am,
                                                               const T *__restrict__ yp, T *__restrict__ dx, int N, int H, int W,
                                                               int C, int P, int Q, FastDiv dCv, FastDiv dWb, FastDiv dHb)
{
    const int Cv = C / V, Hb = (H + 1) / 2, Wb = (W + 1) / 2;
    const long total = (long)N * Hb * Wb * Cv;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int blk = dCv.div((uint32_t)i), cv = (int)i - blk * Cv;
        const int na = dWb.div(blk), b = blk - na * Wb;
        const int n = dHb.div(na), a = na - n * Hb;
        const int c = cv * V;
        float acc[2][2][V];
#pragma unroll
        for (int hr = 0; hr < 2; hr++)
#pragma unroll
            for (int wc = 0; wc < 2; wc++)
#pragma unroll
                for (int j = 0; j < V; j++) acc[hr][wc][j] = 0.f;
        // the (up to) four windows that reach into this 2x2 block; a window outside the pooled map is read at a
        // clamped position and its gradient zeroed, so that all loads are issued before the first use
        int code[2][2][V];
        float g[2][2][V];
        size_t off[2][2];
        bool ok[2][2];
#pragma unroll
        for (int dp = 0; dp < 2; dp++)
#pragma unroll
            for (int dq = 0; dq < 2; dq++) {
                const int p = a - 1 + dp, q = b - 1 + dq;
                ok[dp][dq] = (unsigned)p < (unsigned)P && (unsigned)q < (unsigned)Q;
                off[dp][dq] = ((size_t)(n * P + min(max(p, 0), P - 1)) * Q + min(max(q, 0), Q - 1)) * C + c;
                PoolVec<T, V>::codes(am, off[dp][dq], code[dp][dq]);
                PoolVec<T, V>::load(dy, off[dp][dq], g[dp][dq]);
            }
        if (yp) {   // fused ReLU backward: a window whose maximum is <= 0 passes nothing
            float y[2][2][V];
#pragma unroll
            for (int dp = 0; dp < 2; dp++)
#pragma unroll
                for (int dq = 0; dq < 2; dq++) PoolVec<T, V>::load(yp, off[dp][dq], y[dp][dq]);
#pragma unroll
            for (int dp = 0; dp < 2; dp++)
#pragma unroll
                for (int dq = 0; dq < 2; dq++)
#pragma unroll
                    for (int j = 0; j < V; j++) g[dp][dq][j] = y[dp][dq][j] > 0.f ? g[dp][dq][j] : 0.f;
        }
#pragma unroll
        for (int dp = 0; dp < 2; dp++)
#pragma unroll
            for (int dq = 0; dq < 2; dq++) {
                // window row r lands on block row (dp == 1 ? r : r - 2), likewise for columns
#pragma unroll
                for (int hr = 0; hr < 2; hr++)
#pragma unroll
                    for (int wc = 0; wc < 2; wc++) {
                        const int r = dp ? hr : hr + 2, sc = dq ? wc : wc + 2;
                        if (r > 2 || sc > 2) continue;           // compile-time: that element is outside this window
#pragma unroll
                        for (int j = 0; j < V; j++)
                            if (ok[dp][dq] && code[dp][dq][j] == 3 * r + sc) acc[hr][wc][j] += g[dp][dq][j];
                    }
            }
#pragma unroll
        for (int hr = 0; hr < 2; hr++)
#pragma unroll
            for (int wc = 0; wc < 2; wc++) {
                const int h = 2 * a + hr, w = 2 * b + wc;
                if (h < H && w < W) PoolVec<T, V>::store(dx, ((size_t)(n * H + h) * W + w) * C + c, acc[hr][wc]);
            }
    }
}

static owt_status check_pool(int N, int H, int W, int C, int win, int st, owt_dtype dt, int &P, int &Q)
{
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0) return fail(OWT_EINVAL, "N,H,W,C must be positive");
    if (win < 2 || win > 15) return fail(OWT_EINVAL, "win must be in 2..15");
    if (st < 1) return fail(OWT_EINVAL, "stride must be >= 1");
    if (H < win || W < win) return fail(OWT_EINVAL, "window larger than the input");
    if (dt != OWT_F32 && dt != OWT_BF16) return fail(OWT_EINVAL, "unknown dtype %d", (int)dt);
    if ((long)N * H * W * C > 0x7fffffffL) return fail(OWT_EUNSUPPORTED, "tensor with more than 2^31-1 elements");
    P = (H - win) / st + 1; Q = (W - win) / st + 1;
    return OWT_OK;
}

static int grid_for(long total) { long b = (total + 255) / 256; return (int)(b > 65536 ? 65536 : (b < 1 ? 1 : b)); }

}  // namespace owt

using namespace owt;

extern "C" {

owt_status owt_maxpool_fwd(int N, int H, int W, int C, int win, int stride, owt_dtype dtype,
                           const void *x, void *y, unsigned char *argmax, void *hip_stream)
{
    int P, Q;
    owt_status st = check_pool(N, H, W, C, win, stride, dtype, P, Q);
    if (st != OWT_OK) return st;
    if (!x || !y || !argmax) return fail(OWT_EINVAL, "x, y or argmax is NULL");
    if (!aligned16(x) || !aligned16(y) || !aligned16(argmax)) return fail(OWT_EINVAL, "misaligned pointer");
    const int V = (dtype == OWT_BF16 && C % 8 == 0) ? 8 : (C % 4 == 0 ? 4 : 1);
    FastDiv dCv, dQ, dP; dCv.set(C / V); dQ.set(Q); dP.set(P);
    const long total = (long)N * P * Q * (C / V);
    hipStream_t s = (hipStream_t)hip_stream;
    const bool w3s2 = win == 3 && stride == 2;
#define OWT_POOL_F(T, VV, WS) hipLaunchKernelGGL((maxpool_fwd_kernel<T, VV, WS>), dim3(grid_for(total)), dim3(256), 0, s, \
        (const T *)x, (T *)y, argmax, N, H, W, C, win, stride, P, Q, dCv, dQ, dP)
    if (V == 8) {
        if (w3s2) hipLaunchKernelGGL(maxpool_fwd_bf16x8_kernel<3>, dim3(grid_for(total)), dim3(256), 0, s, (const uint16_t *)x, (uint16_t *)y,
                                     argmax, N, H, W, C, win, stride, P, Q, dCv, dQ, dP);
        else hipLaunchKernelGGL(maxpool_fwd_bf16x8_kernel<0>, dim3(grid_for(total)), dim3(256), 0, s, (const uint16_t *)x, (uint16_t *)y,
                                argmax, N, H, W, C, win, stride, P, Q, dCv, dQ, dP);
    } else if (dtype == OWT_F32) {
        if (V == 4) { if (w3s2) OWT_POOL_F(float, 4, 3); else OWT_POOL_F(float, 4, 0); }
        else OWT_POOL_F(float, 1, 0);
    } else { if (V == 4) OWT_POOL_F(bf16_t, 4, 0); else OWT_POOL_F(bf16_t, 1, 0); }
#undef OWT_POOL_F
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(OWT_ELAUNCH, "HIP launch failed: %s", hipGetErrorString(e));
    return OWT_OK;
}

static owt_status pool_bwd(int N, int H, int W, int C, int win, int stride, owt_dtype dtype, const void *dy,
                           const unsigned char *argmax, const void *yp, void *dx, void *hip_stream)
{
    int P, Q;
    owt_status st = check_pool(N, H, W, C, win, stride, dtype, P, Q);
    if (st != OWT_OK) return st;
    if (!dy || !dx || !argmax) return fail(OWT_EINVAL, "dy, dx or argmax is NULL");
    if (!aligned16(dy) || !aligned16(dx) || !aligned16(argmax)) return fail(OWT_EINVAL, "misaligned pointer");
    const int V = (dtype == OWT_BF16 && C % 8 == 0) ? 8 : (C % 4 == 0 ? 4 : 1);
    FastDiv dCv, dW, dH, dst; dCv.set(C / V); dW.set(W); dH.set(H); dst.set(stride);
    const long total = (long)N * H * W * (C / V);
    hipStream_t s = (hipStream_t)hip_stream;
    if (win == 3 && stride == 2 && ((dtype == OWT_F32 && V == 4) || (dtype == OWT_BF16 && V == 8))) {
        FastDiv dWb, dHb; dWb.set((W + 1) / 2); dHb.set((H + 1) / 2);
        const long blocks = (long)N * ((H + 1) / 2) * ((W + 1) / 2) * (C / V);
        if (dtype == OWT_F32)
            hipLaunchKernelGGL((maxpool_bwd_w3s2_kernel<float, 4>), dim3(grid_for(blocks)), dim3(256), 0, s, (const float *)dy,
                               argmax, (const float *)yp, (float *)dx, N, H, W, C, P, Q, dCv, dWb, dHb);
        else
            hipLaunchKernelGGL((maxpool_bwd_w3s2_kernel<bf16_t, 8>), dim3(grid_for(blocks)), dim3(256), 0, s, (const bf16_t *)dy,
                               argmax, (const bf16_t *)yp, (bf16_t *)dx, N, H, W, C, P, Q, dCv, dWb, dHb);
    } else if (V == 8)
        hipLaunchKernelGGL(maxpool_bwd_bf16x8_kernel, dim3(grid_for(total)), dim3(256), 0, s, (const uint16_t *)dy, argmax,
                           (const uint16_t *)yp, (uint16_t *)dx, N, H, W, C, win, stride, P, Q, dCv, dW, dH, dst);
#define OWT_POOL_B(T, VV) hipLaunchKernelGGL((maxpool_bwd_kernel<T, VV>), dim3(grid_for(total)), dim3(256), 0, s, \
        (const T *)dy, argmax, (const T *)yp, (T *)dx, N, H, W, C, win, stride, P, Q, dCv, dW, dH, dst)
    else if (dtype == OWT_F32) { if (V == 4) OWT_POOL_B(float, 4); else OWT_POOL_B(float, 1); }
    else { if (V == 4) OWT_POOL_B(bf16_t, 4); else OWT_POOL_B(bf16_t, 1); }
#undef OWT_POOL_B
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(OWT_ELAUNCH, "HIP launch failed: %s", hipGetErrorString(e));
    return OWT_OK;
}

owt_status owt_maxpool_bwd(int N, int H, int W, int C, int win, int stride, owt_dtype dtype,
                           const void *dy, const unsigned char *argmax, void *dx, void *hip_stream)
{
    return pool_bwd(N, H, W, C, win, stride, dtype, dy, argmax, nullptr, dx, hip_stream);
}

owt_status owt_maxpool_bwd_relu(int N, int H, int W, int C, int win, int stride, owt_dtype dtype,
                                const void *dy, const unsigned char *argmax, const void *y_pooled, void *dx,
                                void *hip_stream)
{
    if (!y_pooled || !aligned16(y_pooled)) return fail(OWT_EINVAL, "y_pooled is NULL or misaligned");
    return pool_bwd(N, H, W, C, win, stride, dtype, dy, argmax, y_pooled, dx, hip_stream);
}

}  // extern "C"
