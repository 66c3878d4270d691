// Plain fp32 kernels (true fp32 FMA on the vector ALUs) for the reference-precision
// path: one thread per output element for forward / backward-data, one wavefront per
// filter element for backward-filter.  Small correctness configuration, no tiling.
#include "dp_kernels.h"

namespace {

__global__ __launch_bounds__(256) void k_f32_fwd(ConvGeom g, unsigned flags, const float *x, const float *w,
                                                   const float *bias, float *y)
{
    const long long total = (long long)g.N * g.Ho * g.Wo * g.K;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (long long)gridDim.x * blockDim.x) {
        int k = (int)(e % g.K);
        long long m = e / g.K;
        int q = (int)(m % g.Wo), p = (int)((m / g.Wo) % g.Ho), n = (int)(m / ((long long)g.Wo * g.Ho));
        float acc = (flags & KF_BIAS) ? bias[k] : 0.f;
        for (int r = 0; r < g.R; ++r) {
            int ih = p * g.sh - g.ph + r;
            if ((unsigned)ih >= (unsigned)g.H) continue;
            for (int s = 0; s < g.S; ++s) {
                int iw = q * g.sw - g.pw + s;
                if ((unsigned)iw >= (unsigned)g.W) continue;
                const float *xp = x + (((size_t)n * g.H + ih) * g.W + iw) * g.C;
                const float *wp = w + (((size_t)k * g.R + r) * g.S + s) * g.C;
                for (int c = 0; c < g.C; ++c) acc = fmaf(xp[c], wp[c], acc);
            }
        }
        if ((flags & KF_RELU) && !(acc > 0.f)) acc = 0.f;
        y[e] = acc;
    }
}

__device__ __forceinline__ float gm(const float *dy, const float *ym, size_t i)
{
    return (ym != nullptr && !(ym[i] > 0.f)) ? 0.f : dy[i];
}

__global__ __launch_bounds__(256) void k_f32_dgrad(ConvGeom g, const float *dy, const float *ym, const float *w, const float *xin, float *dx)
{
    const long long total = (long long)g.N * g.H * g.W * g.C;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (long long)gridDim.x * blockDim.x) {
        int c = (int)(e % g.C);
        long long m = e / g.C;
        int wi = (int)(m % g.W), h = (int)((m / g.W) % g.H), n = (int)(m / ((long long)g.W * g.H));
        float acc = 0.f;
        for (int r = 0; r < g.R; ++r) {
            int hp = h + g.ph - r;
            if (hp < 0 || hp % g.sh != 0) continue;
            int p = hp / g.sh;
            if (p >= g.Ho) continue;
            for (int s = 0; s < g.S; ++s) {
                int wq = wi + g.pw - s;
                if (wq < 0 || wq % g.sw != 0) continue;
                int q = wq / g.sw;
                if (q >= g.Wo) continue;
                size_t gb = (((size_t)n * g.Ho + p) * g.Wo + q) * g.K;
                for (int k = 0; k < g.K; ++k)
                    acc = fmaf(gm(dy, ym, gb + k), w[(((size_t)k * g.R + r) * g.S + s) * g.C + c], acc);
            }
        }
        dx[e] = (xin == nullptr || xin[e] > 0.f) ? acc : 0.f;   // backward of the ReLU that produced the layer's input
    }
}

// one wavefront per dw element; lanes stride over the output pixels, then a shuffle tree
__global__ __launch_bounds__(256) void k_f32_wgrad(ConvGeom g, const float *x, const float *dy, const float *ym, float *dw)
{
    const long long total = (long long)g.K * g.R * g.S * g.C;
    const int lane = threadIdx.x & 63;
    const long long e = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (e >= total) return;
    int c = (int)(e % g.C);
    int s = (int)((e / g.C) % g.S);
    int r = (int)((e / ((long long)g.C * g.S)) % g.R);
    int k = (int)(e / ((long long)g.C * g.S * g.R));
    const int M = g.N * g.Ho * g.Wo;
    float acc = 0.f;
    for (int m = lane; m < M; m += 64) {
        int q = m % g.Wo, p = (m / g.Wo) % g.Ho, n = m / (g.Wo * g.Ho);
        int ih = p * g.sh - g.ph + r, iw = q * g.sw - g.pw + s;
        if ((unsigned)ih >= (unsigned)g.H || (unsigned)iw >= (unsigned)g.W) continue;
        acc = fmaf(gm(dy, ym, (size_t)m * g.K + k), x[(((size_t)n * g.H + ih) * g.W + iw) * g.C + c], acc);
    }
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_down(acc, o, 64);
    if (lane == 0) dw[e] = acc;
}

unsigned blocks_for(long long total)
{
    long long nb = (total + 255) / 256;
    if (nb > 65536) nb = 65536;
    if (nb < 1) nb = 1;
    return (unsigned)nb;
}

}  // namespace

hipError_t f32_conv_fwd(const ConvGeom &g, unsigned flags, const float *x, const float *w, const float *bias,
                        float *y, hipStream_t st)
{
    hipLaunchKernelGGL(k_f32_fwd, dim3(blocks_for((long long)g.N * g.Ho * g.Wo * g.K)), dim3(256), 0, st, g, flags, x, w, bias, y);
    return hipGetLastError();
}

hipError_t f32_conv_dgrad(const ConvGeom &g, const float *dy, const float *ymask, const float *w, const float *xin, float *dx, hipStream_t st)
{
    hipLaunchKernelGGL(k_f32_dgrad, dim3(blocks_for((long long)g.N * g.H * g.W * g.C)), dim3(256), 0, st, g, dy, ymask, w, xin, dx);
    return hipGetLastError();
}

hipError_t f32_conv_wgrad(const ConvGeom &g, const float *x, const float *dy, const float *ymask, float *dw, hipStream_t st)
{
    long long total = (long long)g.K * g.R * g.S * g.C;
    hipLaunchKernelGGL(k_f32_wgrad, dim3((unsigned)((total + 3) / 4)), dim3(256), 0, st, g, x, dy, ymask, dw);
    return hipGetLastError();
}
