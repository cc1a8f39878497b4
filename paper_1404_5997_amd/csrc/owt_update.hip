// The two elementwise pieces of Section 5 that complete one worker's training
// step: the momentum / weight-decay update rule, and the output layer of
// independent logistic units under cross-entropy (this worker's columns).
// Both are HBM-bound: 16-byte accesses, consecutive lanes on consecutive
// addresses, no atomics.
#include <cmath>

#include "owt_host.hpp"

namespace owt {

// vel := mu*vel + eps*(gscale*g - omega*w);  w := w + vel        (Section 5)
// 20 bytes of HBM traffic per weight (3 reads, 2 writes) + 2 for the optional bf16 copy of w.
template <bool COPY>
__global__ void __launch_bounds__(256) sgd_momentum_kernel(float *__restrict__ w, float *__restrict__ vel,
                                                           const float *__restrict__ g, uint16_t *__restrict__ wb,
                                                           size_t n, float mu, float eps, float omega, float gscale)
{
    const size_t n4 = n >> 2, stride = (size_t)gridDim.x * 256;
    auto upd = [&](float &wv, float &vv, float gv) {
        vv = fmaf(mu, vv, eps * fmaf(gscale, gv, -omega * wv));
        wv += vv;
    };
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
        float4 a = ((const float4 *)w)[i], v = ((const float4 *)vel)[i];
        const float4 d = ((const float4 *)g)[i];
        upd(a.x, v.x, d.x); upd(a.y, v.y, d.y); upd(a.z, v.z, d.z); upd(a.w, v.w, d.w);
        ((float4 *)vel)[i] = v;
        ((float4 *)w)[i] = a;
        if (COPY) {
            uint2 o;
            o.x = f32_to_bf16(a.x) | ((uint32_t)f32_to_bf16(a.y) << 16);
            o.y = f32_to_bf16(a.z) | ((uint32_t)f32_to_bf16(a.w) << 16);
            ((uint2 *)wb)[i] = o;
        }
    }
    for (size_t i = (n4 << 2) + (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {   // ragged tail
        float a = w[i], v = vel[i];
        upd(a, v, g[i]);
        vel[i] = v; w[i] = a;
        if (COPY) wb[i] = f32_to_bf16(a);
    }
}

// One wavefront per sample: lanes stride over the shard's O columns, the loss is
// summed over the lanes in a fixed order (butterfly), so results repeat bit for bit.
//   s = 1/(1+exp(-z)), t = [label == col0 + j]
//   loss[n] = sum_j max(z,0) - z*t + log1p(exp(-|z|));   dz = scale*(s - t)
template <class T>
__global__ void __launch_bounds__(256) logistic_xent_kernel(const T *z, const int *__restrict__ label,
                                                            float *__restrict__ loss, T *dz, int N, int O,
                                                            int col0, float scale)
{
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;                                          // whole wavefronts leave together
    const int tj = label[n] - col0;
    float e = 0.f;
    for (int j = lane; j < O; j += 64) {
        const size_t o = (size_t)n * O + j;
        const float v = load1(z, o), t = j == tj ? 1.f : 0.f;
        const float ex = expf(-fabsf(v));                        // in (0, 1]
        const float s = v >= 0.f ? 1.f / (1.f + ex) : ex / (1.f + ex);
        e += fmaxf(v, 0.f) - v * t + log1pf(ex);
        store1(dz, o, scale * (s - t));
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) e += __shfl_xor(e, d, 64);
    if (lane == 0) loss[n] = e;
}

}  // namespace owt

using namespace owt;

extern "C" {

owt_status owt_sgd_momentum_update(size_t n, float *w, float *vel, const float *g, float mu, float eps, float omega,
                                   float gscale, void *w_bf16_or_null, void *hip_stream)
{
    if (n == 0) return OWT_OK;
    if (!w || !vel || !g) return fail(OWT_EINVAL, "w, vel and g are required");
    if (!aligned16(w) || !aligned16(vel) || !aligned16(g) || !aligned16(w_bf16_or_null))
        return fail(OWT_EINVAL, "pointers must be 16-byte aligned");
    if (!std::isfinite(mu) || !std::isfinite(eps) || !std::isfinite(omega) || !std::isfinite(gscale))
        return fail(OWT_EINVAL, "mu, eps, omega and gscale must be finite");
    const size_t want = (n / 4 + 255) / 256 + 1;
    const dim3 grid((unsigned)(want < 4096 ? want : 4096));
    hipStream_t s = (hipStream_t)hip_stream;
    if (w_bf16_or_null)
        hipLaunchKernelGGL(sgd_momentum_kernel<true>, grid, dim3(256), 0, s, w, vel, g, (uint16_t *)w_bf16_or_null, n, mu,
                           eps, omega, gscale);
    else
        hipLaunchKernelGGL(sgd_momentum_kernel<false>, grid, dim3(256), 0, s, w, vel, g, (uint16_t *)nullptr, n, mu, eps,
                           omega, gscale);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(OWT_ELAUNCH, "HIP launch failed: %s", hipGetErrorString(e));
    return OWT_OK;
}

owt_status owt_logistic_xent(int N, int O_local, int col_offset, owt_dtype dtype, const void *z, const int *labels,
                             float scale, float *loss, void *dz, void *hip_stream)
{
    if (N <= 0 || O_local <= 0 || col_offset < 0) return fail(OWT_EINVAL, "N, O_local must be positive, col_offset >= 0");
    if (dtype != OWT_F32 && dtype != OWT_BF16) return fail(OWT_EINVAL, "unknown dtype");
    if (!z || !labels || !loss || !dz) return fail(OWT_EINVAL, "z, labels, loss and dz are required");
    if (!aligned16(z) || !aligned16(dz) || !aligned16(loss) || !aligned16(labels))
        return fail(OWT_EINVAL, "pointers must be 16-byte aligned");
    if ((long)N * O_local > 0x7fffffffL) return fail(OWT_EUNSUPPORTED, "more than 2^31-1 elements");
    if (!std::isfinite(scale)) return fail(OWT_EINVAL, "scale must be finite");
    const dim3 grid((N + 3) / 4);
    hipStream_t s = (hipStream_t)hip_stream;
    if (dtype == OWT_F32)
        hipLaunchKernelGGL(logistic_xent_kernel<float>, grid, dim3(256), 0, s, (const float *)z, labels, loss, (float *)dz,
                           N, O_local, col_offset, scale);
    else
        hipLaunchKernelGGL(logistic_xent_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t *)z, labels, loss,
                           (bf16_t *)dz, N, O_local, col_offset, scale);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(OWT_ELAUNCH, "HIP launch failed: %s", hipGetErrorString(e));
    return OWT_OK;
}

owt_status owt_scale_hyperparameters(double k, double eps, double omega, double *eps_out, double *omega_out)
{
    if (!(k > 0.0) || !(eps > 0.0) || !std::isfinite(k) || !std::isfinite(eps) || !std::isfinite(omega))
        return fail(OWT_EINVAL, "k and eps must be positive and finite");
    if (!eps_out || !omega_out) return fail(OWT_EINVAL, "output pointers are required");
    *eps_out = std::sqrt(k) * eps;
    *omega_out = (1.0 - std::pow(1.0 - eps * omega, k)) / *eps_out;
    return OWT_OK;
}

}  // extern "C"
