// Layers with very few input channels (the RGB first layer, 7x7 stems): their reduction length
// R*S*C (27, 147) is shorter than one reduction step of the tiled kernels and C is not a multiple
// of 8, so no 16-byte load is aligned.  These layers are bound by the output activation traffic,
// not by the matrix cores; the cheapest correct way to put them on the fast kernels is an explicit
// im2col of x into [pixels][Kpad] (Kpad = R*S*C rounded up to 32, zero filled) and zero-padded weights
// [K][Kpad]: forward and backward-filter then are 1x1 convolutions with Kpad input channels.
// The im2col buffer is R*S*C/ C * ... small next to the output (Kpad*2 bytes per pixel against K*2).
#include "dp_kernels.h"

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

namespace {

// one thread = one 16-byte chunk (8 reduction elements) of one output pixel's im2col row
__global__ __launch_bounds__(256) void k_im2col_small(ConvGeom g, int kpad, const bf16_t *x, bf16_t *xcol)
{
    const int cpr = kpad / 8;
    const long long total = (long long)g.N * g.Ho * g.Wo * cpr;
    const int rsc = g.R * g.S * g.C;
    for (long long id = (long long)blockIdx.x * blockDim.x + threadIdx.x; id < total; id += (long long)gridDim.x * blockDim.x) {
        const int ch = (int)(id % cpr);
        const long long m = id / cpr;
        const int q = (int)(m % g.Wo), p = (int)((m / g.Wo) % g.Ho), n = (int)(m / ((long long)g.Wo * g.Ho));
        const int hb = p * g.sh - g.ph, wb = q * g.sw - g.pw;
        unsigned v[4] = {0, 0, 0, 0};
        // decode the first element of the chunk once, then step (c, s, r) like an odometer
        int kk = ch * 8;
        int rs = kk / g.C, c = kk - rs * g.C, r = rs / g.S, s = rs - r * g.S;
        const bf16_t *img = x + (size_t)n * g.H * g.W * g.C;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            unsigned val = 0;
            const int ih = hb + r, iw = wb + s;
            if (kk + e < rsc && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W) val = img[(ih * g.W + iw) * g.C + c];
            v[e >> 1] |= val << ((e & 1) * 16);
            if (++c == g.C) { c = 0; if (++s == g.S) { s = 0; ++r; } }
        }
        *reinterpret_cast<u32x4 *>(xcol + (size_t)m * kpad + ch * 8) = u32x4{v[0], v[1], v[2], v[3]};
    }
}

__global__ __launch_bounds__(256) void k_pad_rows_bf16(int rows, int len, int lpad, const bf16_t *src, bf16_t *dst)
{
    const int total = rows * lpad;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        const int r = i / lpad, c = i - r * lpad;
        dst[i] = c < len ? src[(size_t)r * len + c] : (bf16_t)0;
    }
}

__global__ __launch_bounds__(256) void k_unpad_rows_f32(int rows, int len, int lpad, const float *src, float *dst)
{
    const int total = rows * len;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        const int r = i / len, c = i - r * len;
        dst[i] = src[(size_t)r * lpad + c];
    }
}

unsigned blocks_for(long long total)
{
    long long nb = (total + 255) / 256;
    if (nb > 16384) nb = 16384;
    return (unsigned)(nb < 1 ? 1 : nb);
}

}  // namespace

int small_c_kpad(const ConvGeom &g)
{
    if ((g.C % 8) == 0) return 0;
    const int rsc = g.R * g.S * g.C;
    const int kpad = (rsc + 31) / 32 * 32;
    return kpad <= 256 ? kpad : 0;
}

hipError_t small_c_im2col(const ConvGeom &g, int kpad, const bf16_t *x, bf16_t *xcol, hipStream_t st)
{
    hipLaunchKernelGGL(k_im2col_small, dim3(blocks_for((long long)g.N * g.Ho * g.Wo * (kpad / 8))), dim3(256), 0, st, g, kpad, x, xcol);
    return hipGetLastError();
}

hipError_t small_c_pad_weights(const ConvGeom &g, int kpad, const bf16_t *w, bf16_t *wpad, hipStream_t st)
{
    hipLaunchKernelGGL(k_pad_rows_bf16, dim3(blocks_for((long long)g.K * kpad)), dim3(256), 0, st, g.K, g.R * g.S * g.C, kpad, w, wpad);
    return hipGetLastError();
}

hipError_t small_c_unpad_dw(const ConvGeom &g, int kpad, const float *dwpad, float *dw, hipStream_t st)
{
    hipLaunchKernelGGL(k_unpad_rows_f32, dim3(blocks_for((long long)g.K * g.R * g.S * g.C)), dim3(256), 0, st, g.K, g.R * g.S * g.C, kpad, dwpad, dw);
    return hipGetLastError();
}
