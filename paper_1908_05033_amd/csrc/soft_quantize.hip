// Training-mode DSQ kernels: the differentiable soft quantization function of
// the paper (Sec. 3.2: phi(x) = s*tanh(k*(x - m_i)) inside interval P_i and
// Q_S(x) = l + Delta*(i + (phi+1)/2), clipped to [l, u]) with its shape tied to
// the characteristic variable alpha (Sec. 3.3: k = log(2/alpha - 1)/Delta,
// s = 1/(1 - alpha); Sec. 4.3: k <= 1000), and the back-propagation of
// Algorithm 1 for one tensor: dL/dx elementwise and the sums dL/dalpha, dL/dl,
// dL/du (Sec. 3.3 and 3.4).  Elementwise, binary32 arithmetic; the three sums
// are accumulated in binary64.  Both kernels stream their tensors once
// (8 and 12 bytes per element) and are bound by HBM bandwidth.
#include "dsq_kernels.h"

namespace {

// tanh(z) and 1 - tanh(z)^2 from e = exp(-2|z|): accurate in the saturated
// tails, where 1 - t*t computed from a rounded t would lose all its digits.
__device__ __forceinline__ void tanh_sech2(float z, float &t, float &sech2)
{
    const float e = __expf(-2.0f * fabsf(z));
    const float r = 1.0f / (1.0f + e);
    t = copysignf((1.0f - e) * r, z);
    sech2 = 4.0f * e * r * r;
}

__device__ __forceinline__ float soft_fwd(float x, const DsqSoftArgs &p)
{
    if (x < p.l) return p.l;
    if (x > p.u) return p.u;
    const float i = fminf(floorf((x - p.l) * p.inv_delta), p.last_interval);
    const float m = p.l + (i + 0.5f) * p.delta;
    float t, sech2;
    tanh_sech2(p.k * (x - m), t, sech2);
    return p.l + p.delta * (i + 0.5f * (p.s * t + 1.0f));
}

__global__ __launch_bounds__(256) void soft_fwd_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                       size_t n, DsqSoftArgs p)
{
    const size_t n4 = n / 4;
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t v = (size_t)blockIdx.x * 256 + threadIdx.x; v < n4; v += stride) {
        const float4 a = reinterpret_cast<const float4 *>(x)[v];
        reinterpret_cast<float4 *>(y)[v] =
            make_float4(soft_fwd(a.x, p), soft_fwd(a.y, p), soft_fwd(a.z, p), soft_fwd(a.w, p));
    }
    const size_t tail = n4 * 4 + (size_t)blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.x == 0 && tail < n) y[tail] = soft_fwd(x[tail], p);
}

// One element of the backward pass: returns dL/dx, adds to the three sums.
__device__ __forceinline__ float soft_bwd(float x, float g, const DsqSoftArgs &p, double &sa, double &sl,
                                          double &su)
{
    if (x < p.l) { sl += (double)g; return 0.0f; }
    if (x > p.u) { su += (double)g; return 0.0f; }
    const float i = fminf(floorf((x - p.l) * p.inv_delta), p.last_interval);
    const float m = p.l + (i + 0.5f) * p.delta;
    const float xm = x - m;
    float t, sech2;
    tanh_sech2(p.k * xm, t, sech2);
    const float q_over_levels = (i + 0.5f * (p.s * t + 1.0f)) * p.inv_levels;
    const float m_u = (i + 0.5f) * p.inv_levels, m_l = 1.0f - m_u;
    const float ss = p.s * sech2;
    const float phi_a = p.s_a * t + ss * (p.k_a * xm);
    const float phi_l = p.s_l * t + ss * (p.k_l * xm - p.k * m_l);
    const float phi_u = p.s_u * t + ss * (p.k_u * xm - p.k * m_u);
    const float half_delta = 0.5f * p.delta;
    sa += (double)(g * (half_delta * phi_a));
    sl += (double)(g * (1.0f - q_over_levels + half_delta * phi_l));
    su += (double)(g * (q_over_levels + half_delta * phi_u));
    return g * (half_delta * ss * p.k);
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off);
    return v;
}

// Few, large workgroups (1024 threads, two vectors in flight per thread): every
// workgroup ends with three binary64 atomics on one cache line, which the memory
// system serialises at a few ns each, so their number has to stay small next to
// the streaming time.
constexpr int BWD_THREADS = 1024;

__global__ __launch_bounds__(BWD_THREADS) void soft_bwd_kernel(const float *__restrict__ x,
                                                               const float *__restrict__ gy,
                                                               float *__restrict__ gx, size_t n, DsqSoftArgs p,
                                                               double *__restrict__ sums)
{
    __shared__ double part[3][BWD_THREADS / 64];
    double sa = 0.0, sl = 0.0, su = 0.0;
    const size_t n4 = n / 4;
    const size_t stride = (size_t)gridDim.x * BWD_THREADS;
    auto four = [&](const float4 a, const float4 g) {
        float4 r;
        r.x = soft_bwd(a.x, g.x, p, sa, sl, su);
        r.y = soft_bwd(a.y, g.y, p, sa, sl, su);
        r.z = soft_bwd(a.z, g.z, p, sa, sl, su);
        r.w = soft_bwd(a.w, g.w, p, sa, sl, su);
        return r;
    };
    size_t v = (size_t)blockIdx.x * BWD_THREADS + threadIdx.x;
    for (; v + stride < n4; v += 2 * stride) {
        const float4 a0 = reinterpret_cast<const float4 *>(x)[v];
        const float4 g0 = reinterpret_cast<const float4 *>(gy)[v];
        const float4 a1 = reinterpret_cast<const float4 *>(x)[v + stride];
        const float4 g1 = reinterpret_cast<const float4 *>(gy)[v + stride];
        reinterpret_cast<float4 *>(gx)[v] = four(a0, g0);
        reinterpret_cast<float4 *>(gx)[v + stride] = four(a1, g1);
    }
    if (v < n4)
        reinterpret_cast<float4 *>(gx)[v] =
            four(reinterpret_cast<const float4 *>(x)[v], reinterpret_cast<const float4 *>(gy)[v]);
    const size_t tail = n4 * 4 + threadIdx.x;
    if (blockIdx.x == 0 && tail < n) gx[tail] = soft_bwd(x[tail], gy[tail], p, sa, sl, su);

    sa = wave_sum(sa); sl = wave_sum(sl); su = wave_sum(su);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { part[0][wave] = sa; part[1][wave] = sl; part[2][wave] = su; }
    __syncthreads();
    if (threadIdx.x < 3) {
        double s = 0.0;
        for (int w = 0; w < BWD_THREADS / 64; ++w) s += part[threadIdx.x][w];
        atomicAdd(&sums[threadIdx.x], s);       // binary64: the order of the workgroups moves the sum by ~1e-16 relative
    }
}

unsigned grid_for(size_t n, size_t vectors_per_thread, size_t most)
{
    const size_t want = (n / 4 + 256 * vectors_per_thread - 1) / (256 * vectors_per_thread);
    return (unsigned)(want < 1 ? 1 : want > most ? most : want);
}

}  // namespace

hipError_t dsq_launch_soft_fwd(const float *x, float *y, size_t n, const DsqSoftArgs &p, hipStream_t stream)
{
    soft_fwd_kernel<<<grid_for(n, 1, 8192), 256, 0, stream>>>(x, y, n, p);
    return hipGetLastError();
}

hipError_t dsq_launch_soft_bwd(const float *x, const float *gy, float *gx, size_t n, const DsqSoftArgs &p,
                               double *sums, hipStream_t stream)
{
    hipError_t e = dsq_launch_fill_zero(reinterpret_cast<int32_t *>(sums), 6, stream);
    if (e != hipSuccess) return e;
    const size_t want = (n / 4 + BWD_THREADS - 1) / BWD_THREADS;
    const unsigned grid = (unsigned)(want < 1 ? 1 : want > 512 ? 512 : want);
    soft_bwd_kernel<<<grid, BWD_THREADS, 0, stream>>>(x, gy, gx, n, p, sums);
    return hipGetLastError();
}
