// Glue layers of a whole training step: 2x2 max pooling (forward / backward), softmax cross-entropy,
// SGD with momentum.  All pointwise and bound by HBM: 16-byte accesses, one pass over the data.
#include "../../include/dp.h"
#include <hip/hip_runtime.h>
#include <stdint.h>

void dp_set_error(const char *fmt, ...);   // dp_api.hip

namespace {

typedef unsigned short bf16_t;

template <typename T> __device__ __forceinline__ float as_f32(T v);
template <> __device__ __forceinline__ float as_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float as_f32<bf16_t>(bf16_t v) { return __uint_as_float((unsigned)v << 16); }

template <typename T, int V> struct alignas(sizeof(T) * V) Pack { T v[V]; };

// Thread = V channels of one window (window grid ceil(h/2) x ceil(w/2) so that backward also reaches a
// trailing odd row / column, which it zeroes).  BWD = false: y = first maximum; true: dx.
template <typename T, int V, bool BWD>
__global__ __launch_bounds__(256) void k_pool(int n, int h, int w, int c, const T *__restrict__ x, const T *__restrict__ dy, T *__restrict__ out)
{
    typedef Pack<T, V> P;
    const int ho = h / 2, wo = w / 2, hg = BWD ? (h + 1) / 2 : ho, wg = BWD ? (w + 1) / 2 : wo, cv = c / V;
    const long long total = (long long)n * hg * wg * cv;
    const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
    if (id >= total) return;
    const int ci = (int)(id % cv) * V;
    long long r = id / cv;
    const int q = (int)(r % wg);
    r /= wg;
    const int p = (int)(r % hg), ni = (int)(r / hg);
    const size_t row0 = ((size_t)ni * h + 2 * p) * w + 2 * q;   // pixel index of window position (0, 0)
    if (BWD && (p >= ho || q >= wo)) {                           // partial window: no gradient reaches it
        P z;
#pragma unroll
        for (int e = 0; e < V; ++e) z.v[e] = (T)0;
        for (int dh = 0; dh < 2; ++dh)
            for (int dw = 0; dw < 2; ++dw)
                if (2 * p + dh < h && 2 * q + dw < w) *reinterpret_cast<P *>(out + (row0 + (size_t)dh * w + dw) * c + ci) = z;
        return;
    }
    P win[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) win[k] = *reinterpret_cast<const P *>(x + (row0 + (size_t)(k >> 1) * w + (k & 1)) * c + ci);
    int first[V];
    P best = win[0];
#pragma unroll
    for (int e = 0; e < V; ++e) {
        first[e] = 0;
#pragma unroll
        for (int k = 1; k < 4; ++k)
            if (as_f32<T>(win[k].v[e]) > as_f32<T>(best.v[e])) { best.v[e] = win[k].v[e]; first[e] = k; }
    }
    if (!BWD) {
        *reinterpret_cast<P *>(out + (((size_t)ni * ho + p) * wo + q) * c + ci) = best;
        return;
    }
    const P g = *reinterpret_cast<const P *>(dy + (((size_t)ni * ho + p) * wo + q) * c + ci);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        P d;
#pragma unroll
        for (int e = 0; e < V; ++e) d.v[e] = first[e] == k ? g.v[e] : (T)0;
        *reinterpret_cast<P *>(out + (row0 + (size_t)(k >> 1) * w + (k & 1)) * c + ci) = d;
    }
}

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return __builtin_bit_cast(bf16_t, (__bf16)v); }

// One block of 16 wavefronts; wavefront w takes rows w, w+16, ...  A row is read once into registers
// (lane-strided, up to 64*CACHE classes; longer rows re-read the tail); maximum, exponential sum and
// gradient are reduced by shuffles.  Row losses add up per wavefront in row order, the 16 wavefront sums in
// wavefront order.
template <typename T>
__global__ __launch_bounds__(1024) void k_softmax_xent(int n, int classes, const T *__restrict__ z, const int *__restrict__ labels,
                                                        float *__restrict__ loss, T *__restrict__ dz)
{
    constexpr int CACHE = 16;
    __shared__ float part[16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float inv_n = 1.0f / (float)n;
    float wsum = 0.f;
    for (int r = wave; r < n; r += 16) {
        const T *zr = z + (size_t)r * classes;
        float zc[CACHE];
#pragma unroll
        for (int k = 0; k < CACHE; ++k) {
            const int c = lane + 64 * k;
            zc[k] = c < classes ? as_f32<T>(zr[c]) : -INFINITY;
        }
        float mx = -INFINITY;
#pragma unroll
        for (int k = 0; k < CACHE; ++k) mx = fmaxf(mx, zc[k]);
        for (int c = lane + 64 * CACHE; c < classes; c += 64) mx = fmaxf(mx, as_f32<T>(zr[c]));
        for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
        float se = 0.f;
#pragma unroll
        for (int k = 0; k < CACHE; ++k) se += expf(zc[k] - mx);   // exp(-inf) = 0 past the row's end
        for (int c = lane + 64 * CACHE; c < classes; c += 64) se += expf(as_f32<T>(zr[c]) - mx);
        for (int o = 32; o >= 1; o >>= 1) se += __shfl_xor(se, o, 64);
        const float lse = mx + logf(se);
        const int lab = labels[r];
        const bool ok = lab >= 0 && lab < classes;
        wsum += lse - (ok ? as_f32<T>(zr[lab]) : 0.f);
        if (dz != nullptr) {
            T *dr = dz + (size_t)r * classes;
#pragma unroll
            for (int k = 0; k < CACHE; ++k) {
                const int c = lane + 64 * k;
                if (c < classes) dr[c] = from_f32<T>((expf(zc[k] - lse) - (ok && c == lab ? 1.f : 0.f)) * inv_n);
            }
            for (int c = lane + 64 * CACHE; c < classes; c += 64)
                dr[c] = from_f32<T>((expf(as_f32<T>(zr[c]) - lse) - (ok && c == lab ? 1.f : 0.f)) * inv_n);
        }
    }
    if (lane == 0) part[wave] = wsum;
    __syncthreads();
    if (threadIdx.x == 0) {
        float s = 0.f;
        for (int i = 0; i < 16; ++i) s += part[i];
        *loss = s * inv_n;
    }
}

// U vectors of 4 elements per thread, all loads issued before the first store; the last count % 4 elements
// go to the first threads of block 0.
template <int U>
__global__ __launch_bounds__(256) void k_sgd(long long count, float lr, float mu, const float *__restrict__ grad, float *__restrict__ mom,
                                             float *__restrict__ w32, bf16_t *__restrict__ w16)
{
    const long long nvec = count / 4;
    const long long i0 = ((long long)blockIdx.x * U) * 256 + threadIdx.x;
    float4 g[U], m[U], w[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const long long i = i0 + u * 256;
        if (i < nvec) {
            g[u] = reinterpret_cast<const float4 *>(grad)[i];
            m[u] = reinterpret_cast<const float4 *>(mom)[i];
            w[u] = reinterpret_cast<const float4 *>(w32)[i];
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const long long i = i0 + u * 256;
        if (i >= nvec) continue;
        m[u].x = fmaf(mu, m[u].x, g[u].x); m[u].y = fmaf(mu, m[u].y, g[u].y); m[u].z = fmaf(mu, m[u].z, g[u].z); m[u].w = fmaf(mu, m[u].w, g[u].w);
        w[u].x = fmaf(-lr, m[u].x, w[u].x); w[u].y = fmaf(-lr, m[u].y, w[u].y); w[u].z = fmaf(-lr, m[u].z, w[u].z); w[u].w = fmaf(-lr, m[u].w, w[u].w);
        reinterpret_cast<float4 *>(mom)[i] = m[u];
        reinterpret_cast<float4 *>(w32)[i] = w[u];
        if (w16 != nullptr) {
            Pack<bf16_t, 4> o;
            o.v[0] = from_f32<bf16_t>(w[u].x); o.v[1] = from_f32<bf16_t>(w[u].y); o.v[2] = from_f32<bf16_t>(w[u].z); o.v[3] = from_f32<bf16_t>(w[u].w);
            reinterpret_cast<Pack<bf16_t, 4> *>(w16)[i] = o;
        }
    }
    const long long t = nvec * 4 + threadIdx.x;
    if (blockIdx.x == 0 && t < count) {
        const float mt = fmaf(mu, mom[t], grad[t]), wt = fmaf(-lr, mt, w32[t]);
        mom[t] = mt;
        w32[t] = wt;
        if (w16 != nullptr) w16[t] = from_f32<bf16_t>(wt);
    }
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

dp_status launched(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) return DP_OK;
    dp_set_error("%s launch: %s", what, hipGetErrorString(e));
    return DP_ERR_HIP;
}

// a / b / d: the pointers this call dereferences (pass one twice where fewer are needed)
dp_status check_pool(int n, int h, int w, int c, int dtype, const void *a, const void *b, const void *d)
{
    if (a == nullptr || b == nullptr || d == nullptr) { dp_set_error("max-pool: null pointer"); return DP_ERR_NULL; }
    if (dtype != DP_F32 && dtype != DP_BF16) { dp_set_error("max-pool: unknown io_dtype %d", dtype); return DP_ERR_UNSUPPORTED; }
    if (n < 1 || h < 1 || w < 1 || c < 1) { dp_set_error("max-pool: n, h, w, c must be positive"); return DP_ERR_BAD_DESC; }
    if ((long long)n * h * w * c > (1ll << 40)) { dp_set_error("max-pool: tensor too large"); return DP_ERR_BAD_DESC; }
    if (!aligned16(a) || !aligned16(b) || !aligned16(d)) { dp_set_error("max-pool: pointers must be 16-byte aligned"); return DP_ERR_BAD_DESC; }
    return DP_OK;
}

template <bool BWD>
dp_status run_pool(int n, int h, int w, int c, int dtype, const void *x, const void *dy, void *out, hipStream_t st)
{
    const int hg = BWD ? (h + 1) / 2 : h / 2, wg = BWD ? (w + 1) / 2 : w / 2;
    if (hg == 0 || wg == 0) return DP_OK;   // forward of a 1-pixel-high image: empty output
    const bool bf = dtype == DP_BF16;
    const int v = bf ? (c % 8 == 0 ? 8 : 1) : (c % 4 == 0 ? 4 : 1);
    const long long total = (long long)n * hg * wg * (c / v);
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (bf && v == 8) hipLaunchKernelGGL((k_pool<bf16_t, 8, BWD>), dim3(blocks), dim3(256), 0, st, n, h, w, c, (const bf16_t *)x, (const bf16_t *)dy, (bf16_t *)out);
    else if (bf) hipLaunchKernelGGL((k_pool<bf16_t, 1, BWD>), dim3(blocks), dim3(256), 0, st, n, h, w, c, (const bf16_t *)x, (const bf16_t *)dy, (bf16_t *)out);
    else if (v == 4) hipLaunchKernelGGL((k_pool<float, 4, BWD>), dim3(blocks), dim3(256), 0, st, n, h, w, c, (const float *)x, (const float *)dy, (float *)out);
    else hipLaunchKernelGGL((k_pool<float, 1, BWD>), dim3(blocks), dim3(256), 0, st, n, h, w, c, (const float *)x, (const float *)dy, (float *)out);
    return launched(BWD ? "max-pool backward" : "max-pool forward");
}

}  // namespace

extern "C" dp_status dp_maxpool2x2_fwd(int32_t n, int32_t h, int32_t w, int32_t c, int32_t io_dtype, const void *x, void *y, void *hip_stream)
{
    const bool empty = h / 2 == 0 || w / 2 == 0;   // no window: y has no elements and may be NULL
    dp_status s = check_pool(n, h, w, c, io_dtype, x, empty ? x : y, empty ? x : y);
    if (s != DP_OK) return s;
    return run_pool<false>(n, h, w, c, io_dtype, x, nullptr, y, (hipStream_t)hip_stream);
}

extern "C" dp_status dp_maxpool2x2_bwd(int32_t n, int32_t h, int32_t w, int32_t c, int32_t io_dtype, const void *x, const void *dy, void *dx,
                                       void *hip_stream)
{
    const bool empty = h / 2 == 0 || w / 2 == 0;   // no window: dy has no elements and may be NULL; dx is zeroed
    dp_status s = check_pool(n, h, w, c, io_dtype, x, empty ? x : dy, dx);
    if (s != DP_OK) return s;
    return run_pool<true>(n, h, w, c, io_dtype, x, dy, dx, (hipStream_t)hip_stream);
}

extern "C" dp_status dp_softmax_xent(int32_t n, int32_t classes, int32_t io_dtype, const void *z, const int32_t *labels, float *loss, void *dz,
                                     void *hip_stream)
{
    if (z == nullptr || labels == nullptr || loss == nullptr) { dp_set_error("softmax cross-entropy: null pointer"); return DP_ERR_NULL; }
    if (io_dtype != DP_F32 && io_dtype != DP_BF16) { dp_set_error("softmax cross-entropy: unknown io_dtype %d", io_dtype); return DP_ERR_UNSUPPORTED; }
    if (n < 1 || classes < 1) { dp_set_error("softmax cross-entropy: n and classes must be positive"); return DP_ERR_BAD_DESC; }
    hipStream_t st = (hipStream_t)hip_stream;
    if (io_dtype == DP_BF16) hipLaunchKernelGGL(k_softmax_xent<bf16_t>, dim3(1), dim3(1024), 0, st, n, classes, (const bf16_t *)z, labels, loss, (bf16_t *)dz);
    else hipLaunchKernelGGL(k_softmax_xent<float>, dim3(1), dim3(1024), 0, st, n, classes, (const float *)z, labels, loss, (float *)dz);
    return launched("softmax cross-entropy");
}

extern "C" dp_status dp_sgd_update(int64_t count, float lr, float momentum, const float *grad, float *mom, float *w32, void *w_bf16, void *hip_stream)
{
    if (grad == nullptr || mom == nullptr || w32 == nullptr) { dp_set_error("SGD update: null pointer"); return DP_ERR_NULL; }
    if (count < 0) { dp_set_error("SGD update: negative count"); return DP_ERR_BAD_DESC; }
    if (!aligned16(grad) || !aligned16(mom) || !aligned16(w32) || !aligned16(w_bf16)) { dp_set_error("SGD update: pointers must be 16-byte aligned"); return DP_ERR_BAD_DESC; }
    if (count == 0) return DP_OK;
    constexpr int U = 2;
    long long blocks = (count / 4 + 256 * U - 1) / (256 * U);
    if (blocks < 1) blocks = 1;
    if (blocks > 0x7fffffffll) { dp_set_error("SGD update: count too large"); return DP_ERR_BAD_DESC; }
    hipLaunchKernelGGL(k_sgd<U>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream, (long long)count, lr, momentum, grad, mom, w32, (bf16_t *)w_bf16);
    return launched("SGD update");
}
