// Layers with very few input channels (the RGB first layer, 7x7 stems): their reduction length
// R*S*C (27, 147) is shorter than one reduction step of the tiled kernels and C is not a multiple
// of 8, so no 16-byte load is aligned.  These layers are bound by the output activation traffic,
// not by the matrix cores; the cheapest correct way to put them on the fast kernels is an explicit
// im2col of x into [pixels][Kpad] (Kpad = R*S*C rounded up to 32, zero filled) and zero-padded weights
// [K][Kpad]: forward and backward-filter then are 1x1 convolutions with Kpad input channels
// (the im2col matrix costs Kpad*2 bytes per output pixel next to the output's K*2).
//
// When the whole reduction fits one 32-wide slice pair (R*S*C <= 32: the 3x3 RGB stems) the im2col
// matrix never goes to memory: k_fwd_direct copies the input patch of an 8 x 32 pixel tile into LDS,
// gathers the 256 x 32 im2col tile from it (one thread per output pixel), multiplies it with weight
// fragments that stay in registers, and stores the output tile through LDS with 16-byte rows;
// k_wgrad_direct does the same for the filter gradient with both operands transposed on their way into
// LDS (and, when asked, the ReLU mask applied and the bias gradient summed on the way), one fp32 partial
// per block, and k_wgrad_direct_sum adds the partials in block order.  Both passes then move little more
// than the output activation / the upstream gradient once, which is what bounds these layers.
#include "tile_common.h"

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

// ---- direct kernels for R*S*C <= 32 ---------------------------------------------------------------
constexpr int DT = 256;          // output pixels per tile (forward)
constexpr int DLB = 40;          // im2col row pitch in bf16 (32 + 8: 80-byte rows keep 16-byte alignment, spread banks)
constexpr int DLO = 72;          // staged output row pitch in bf16 (64 channels + 8)

// element kk = (r*S + s)*C + c of the im2col row of output pixel (n, p, q), 0 outside the image
DEVFN unsigned im2col_elem(const ConvGeom &g, const bf16_t *img, int hb, int wb, int r, int s, int c)
{
    const int ih = hb + r, iw = wb + s;
    return ((unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W) ? img[(ih * g.W + iw) * g.C + c] : 0u;
}

// Forward.  A tile is 8 x 32 output pixels of one image.  Its input patch ((7*sh + R) rows of
// (31*sw + S)*C elements) is copied once into LDS with coalesced loads (zero outside the image); every
// thread then gathers the 32-element im2col row of its pixel from the patch.
// grid = (persistent blocks over tiles, 64-row tiles of c_out); 4 waves, wave tile 64 c_out x 64 pixels.
// patch offset r*PWE + s*C + c of reduction element kk (0 beyond R*S*C), passed by value: it lives in scalar registers
struct TapTable { unsigned short off[32]; };
constexpr int DPF = 16;          // patch elements per thread (prefetched in registers)
constexpr int DPATCH = DPF * 256;   // patch elements; they fit beside the im2col tile (<= 8192)
__global__ __launch_bounds__(256, 3) void k_fwd_direct(ConvGeom g, unsigned flags, const bf16_t *x, const bf16_t *w, const float *bias,
                                                    bf16_t *y, int tiles, int tiles_x, int tiles_y, unsigned inv_c, TapTable taps)
{
    // [0, 20 KB): im2col tile [256][40]; [20 KB, 36 KB): input patch; afterwards the whole array is the output tile [256][72]
    __shared__ __attribute__((aligned(16))) bf16_t lds[DT * DLO];
    __shared__ float bias_lds[64];
    bf16_t *patch = lds + DT * DLB;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int a0 = blockIdx.y * 64, rsc = g.R * g.S * g.C;
    const int PH = 7 * g.sh + g.R, PWE = (31 * g.sw + g.S) * g.C, PN = PH * PWE;
    if (tid < 64) bias_lds[tid] = ((flags & KF_BIAS) && a0 + tid < g.K) ? bias[a0 + tid] : 0.f;
    // weight fragments: row a0 + i*32 + lane%32, reduction elements ks*16 + 8*(lane/32) .. +7
    bf16x8 afr[2][2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = a0 + i * 32 + (lane & 31), kb = ks * 16 + 8 * (lane >> 5);
            unsigned v[4] = {0, 0, 0, 0};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned val = (row < g.K && kb + e < rsc) ? w[(size_t)row * rsc + kb + e] : 0u;
                v[e >> 1] |= val << ((e & 1) * 16);
            }
            afr[ks][i] = __builtin_bit_cast(bf16x8, u32x4{v[0], v[1], v[2], v[3]});
        }
    const int py = tid >> 5, px = tid & 31;
    const int goff = (py * g.sh) * PWE + (px * g.sw) * g.C;   // patch element of this pixel's tap (0, 0), channel 0
    // the patch of the next tile is fetched into registers while the current tile is processed
    unsigned short pf[DPF];
    auto fetch = [&](int tile) {
        const int n = tile / (tiles_x * tiles_y), trem = tile - n * (tiles_x * tiles_y), ty = trem / tiles_x, tx = trem - ty * tiles_x;
        const int h0 = ty * 8 * g.sh - g.ph, w0 = tx * 32 * g.sw - g.pw;
        int pr = tid / PWE, pe = tid - pr * PWE;   // element idx = pr*PWE + pe holds x[n][h0 + pr][w0 + pe / C][pe % C]
#pragma unroll
        for (int e = 0; e < DPF; ++e) {
            const int wrel = inv_c != 0 ? (int)__umulhi((unsigned)pe, inv_c) : pe, c = pe - wrel * g.C;   // inv_c == 0: one channel
            const int ih = h0 + pr, iw = w0 + wrel;
            unsigned short val = 0;
            if (tid + e * 256 < PN && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W)
                val = x[((size_t)(n * g.H + ih) * g.W + iw) * g.C + c];
            pf[e] = val;
            pe += 256;
            while (pe >= PWE) { pe -= PWE; ++pr; }
        }
    };
    if ((int)blockIdx.x < tiles) fetch(blockIdx.x);
    for (int tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const int n = tile / (tiles_x * tiles_y), trem = tile - n * (tiles_x * tiles_y), ty = trem / tiles_x, tx = trem - ty * tiles_x;
        const int p0 = ty * 8, q0 = tx * 32;
#pragma unroll
        for (int e = 0; e < DPF; ++e)
            if (tid + e * 256 < PN) patch[tid + e * 256] = pf[e];
        __syncthreads();
        if (tile + (int)gridDim.x < tiles) fetch(tile + gridDim.x);
        {   // im2col row of pixel (py, px): 32 independent LDS reads at wave-uniform offsets, no control flow
            unsigned v[16];
            int gl = goff;
            asm volatile("" : "+v"(gl));   // keeps the 32 addresses from being hoisted out of the tile loop (they would spill)
#pragma unroll
            for (int kk = 0; kk < 32; kk += 2) {
                const unsigned lo = patch[gl + taps.off[kk]] & (kk < rsc ? 0xffffu : 0u);
                const unsigned hi = patch[gl + taps.off[kk + 1]] & (kk + 1 < rsc ? 0xffffu : 0u);
                v[kk >> 1] = lo | (hi << 16);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
                *reinterpret_cast<u32x4 *>(lds + tid * DLB + j * 8) = u32x4{v[4 * j], v[4 * j + 1], v[4 * j + 2], v[4 * j + 3]};
        }
        __syncthreads();
        f32x16 acc[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const bf16x8 b = *reinterpret_cast<const bf16x8 *>(lds + (wave * 64 + j * 32 + (lane & 31)) * DLB + ks * 16 + 8 * (lane >> 5));
#pragma unroll
                for (int i = 0; i < 2; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afr[ks][i], b, acc[i][j], 0, 0, 0);
            }
        __syncthreads();   // im2col tile and patch have been read: their memory now takes the output tile
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int ch = i * 32 + 8 * gq + 4 * (lane >> 5);
                const f32x4 bv = *reinterpret_cast<const f32x4 *>(bias_lds + ch);
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    float v0 = acc[i][j][4 * gq] + bv.x, v1 = acc[i][j][4 * gq + 1] + bv.y;
                    float v2 = acc[i][j][4 * gq + 2] + bv.z, v3 = acc[i][j][4 * gq + 3] + bv.w;
                    if (flags & KF_RELU) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f); }
                    const int pix = wave * 64 + j * 32 + (lane & 31);
                    *reinterpret_cast<u32x2 *>(lds + pix * DLO + ch) = u32x2{pack_bf16(v0, v1), pack_bf16(v2, v3)};
                }
            }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int id = tid + it * 256, pix = id >> 3, cc = id & 7;
            const int p = p0 + (pix >> 5), q = q0 + (pix & 31), gc = a0 + cc * 8;
            if (p < g.Ho && q < g.Wo && gc < g.K)
                *reinterpret_cast<u32x4 *>(y + ((size_t)(n * g.Ho + p) * g.Wo + q) * g.K + gc) = *reinterpret_cast<const u32x4 *>(lds + pix * DLO + cc * 8);
        }
        __syncthreads();   // the output tile has been read before the next patch overwrites it
    }
}

// Filter gradient: block b sums pixels [b*ppb, (b+1)*ppb) in steps of 64; LDS holds both operands
// reduction-contiguous: gT[64 c_out][64 + 8 pixels], xT[32 taps][64 + 8 pixels].  Wave w multiplies the
// 16-pixel slice w of every step; the four waves' sums are added through LDS at the end.
constexpr int WLS = 72;
__global__ __launch_bounds__(256) void k_wgrad_direct(ConvGeom g, const bf16_t *x, const bf16_t *dy, const bf16_t *ym, float *partial,
                                                      float *db_partial, int steps_per_block)
{
    __shared__ __attribute__((aligned(16))) bf16_t gT[64 * WLS];
    __shared__ __attribute__((aligned(16))) bf16_t xT[32 * WLS];
    __shared__ float red[4][64][33];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int a0 = blockIdx.y * 64, rsc = g.R * g.S * g.C, M = g.N * g.Ho * g.Wo;
    const int steps_total = (M + 63) / 64;
    const int sbeg = blockIdx.x * steps_per_block, send = min(sbeg + steps_per_block, steps_total);
    // loader roles: thread -> (pixel, 16 c_out) of the gradient tile, (pixel, 8 taps) of the im2col tile
    const int gp = tid >> 2, gc = (tid & 3) * 16;
    const int xp = tid & 63, xt = (tid >> 6) * 8;
    int xr = 0, xs = 0, xc = 0;   // (r, s, c) of tap xt
    { const int rs = xt / g.C; xc = xt - rs * g.C; xr = rs / g.S; xs = rs - xr * g.S; }
    f32x16 acc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    // two register sets: the loads of steps s+1 and s+2 are in flight while step s is multiplied
    struct Regs { u32x4 gv[2], yv[2]; unsigned xv[8]; };
    Regs ra, rb;
    float dbacc[16];   // bias gradient: this thread's 16 channels over its pixels
#pragma unroll
    for (int e = 0; e < 16; ++e) dbacc[e] = 0.f;
    auto load = [&](int step, Regs &rg) {
        const int m = step * 64 + gp;
        rg.gv[0] = rg.gv[1] = u32x4{0, 0, 0, 0};
        rg.yv[0] = rg.yv[1] = u32x4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};   // "positive": keeps everything
        if (m < M) {
            const bf16_t *src = dy + (size_t)m * g.K + a0 + gc;
            if (a0 + gc + 8 <= g.K) rg.gv[0] = *reinterpret_cast<const u32x4 *>(src);
            if (a0 + gc + 16 <= g.K) rg.gv[1] = *reinterpret_cast<const u32x4 *>(src + 8);
            if (ym != nullptr) {   // ReLU gradient fused: the mask is applied when the registers go to LDS
                const bf16_t *ys = ym + (size_t)m * g.K + a0 + gc;
                if (a0 + gc + 8 <= g.K) rg.yv[0] = *reinterpret_cast<const u32x4 *>(ys);
                if (a0 + gc + 16 <= g.K) rg.yv[1] = *reinterpret_cast<const u32x4 *>(ys + 8);
            }
        }
        const int mx = step * 64 + xp;
#pragma unroll
        for (int e = 0; e < 8; ++e) rg.xv[e] = 0;
        if (mx < M) {
            const int n = mx / (g.Ho * g.Wo), rem = mx - n * (g.Ho * g.Wo), p = rem / g.Wo, q = rem - p * g.Wo;
            const int hb = p * g.sh - g.ph, wb = q * g.sw - g.pw;
            const bf16_t *img = x + (size_t)n * g.H * g.W * g.C;
            int r = xr, s = xs, c = xc;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (xt + e < rsc) {
                    rg.xv[e] = im2col_elem(g, img, hb, wb, r, s, c);
                    if (++c == g.C) { c = 0; if (++s == g.S) { s = 0; ++r; } }
                }
            }
        }
    };
    auto stash = [&](Regs &rg) {   // registers -> LDS, transposed; mask and bias gradient on the way
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const u32x4 mv = apply_mask(rg.gv[h], rg.yv[h]);
            const unsigned wv[4] = {mv.x, mv.y, mv.z, mv.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) gT[(gc + h * 8 + e) * WLS + gp] = (bf16_t)((wv[e >> 1] >> ((e & 1) * 16)) & 0xffffu);
            if (db_partial != nullptr) {
#pragma unroll
                for (int e = 0; e < 8; ++e) dbacc[h * 8 + e] += __uint_as_float((e & 1) ? (wv[e >> 1] & 0xffff0000u) : (wv[e >> 1] << 16));
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) xT[(xt + e) * WLS + xp] = (bf16_t)rg.xv[e];
    };
    auto multiply = [&]() {
        const bf16x8 b = *reinterpret_cast<const bf16x8 *>(xT + (lane & 31) * WLS + wave * 16 + 8 * (lane >> 5));
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const bf16x8 a = *reinterpret_cast<const bf16x8 *>(gT + (i * 32 + (lane & 31)) * WLS + wave * 16 + 8 * (lane >> 5));
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
        }
    };
    if (sbeg < send) load(sbeg, ra);
    if (sbeg + 1 < send) load(sbeg + 1, rb);
    for (int step = sbeg; step < send; step += 2) {
        stash(ra);
        __syncthreads();
        if (step + 2 < send) load(step + 2, ra);
        multiply();
        __syncthreads();
        if (step + 1 < send) {
            stash(rb);
            __syncthreads();
            if (step + 3 < send) load(step + 3, rb);
            multiply();
            __syncthreads();
        }
    }
    // D element v of lane l: row 8*(v/4) + 4*(l/32) + v%4 (c_out), column l%32 (tap)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[wave][i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)][lane & 31] = acc[i][v];
    __syncthreads();
    float *out = partial + ((size_t)blockIdx.x * gridDim.y + blockIdx.y) * 64 * 32;
    for (int id = tid; id < 64 * 32; id += 256) {
        const int k = id >> 5, t = id & 31;
        out[id] = (red[0][k][t] + red[1][k][t]) + (red[2][k][t] + red[3][k][t]);
    }
    if (db_partial != nullptr) {
        // 64 threads (one per pixel slot) hold sums for the same 16 channels: add them in slot order
        __syncthreads();
        float *flat = &red[0][0][0];   // [64 pixel slots][64 channels]
#pragma unroll
        for (int e = 0; e < 16; ++e) flat[gp * 64 + gc + e] = dbacc[e];
        __syncthreads();
        if (tid < 64) {
            float s = 0.f;
            for (int slot = 0; slot < 64; ++slot) s += flat[slot * 64 + tid];
            db_partial[((size_t)blockIdx.x * gridDim.y + blockIdx.y) * 64 + tid] = s;
        }
    }
}

// dw[k][t] = sum over blocks of partial[b][ktile][k % 64][t] in a fixed order; grid = c_out, 1024 threads:
// thread (t, part) adds every 32nd block with four loads in flight, the 32 parts are then added in order
// blocks K .. K + ktiles - 1 (present when the bias gradient is wanted) add db_partial[b][ktile][64] the same way
__global__ __launch_bounds__(1024) void k_wgrad_direct_sum(int K, int rsc, int nblocks, int ktiles, const float *partial, float *dw,
                                                           const float *db_partial, float *db)
{
    __shared__ float sm[32][33];
    if ((int)blockIdx.x >= K) {
        __shared__ float sd[16][64];
        const int kt = blockIdx.x - K, ch = threadIdx.x & 63, part = threadIdx.x >> 6;   // 16 parts
        float s = 0.f;
        for (int b = part; b < nblocks; b += 16) s += db_partial[((size_t)b * ktiles + kt) * 64 + ch];
        sd[part][ch] = s;
        __syncthreads();
        if (part == 0 && kt * 64 + ch < K) {
            float tot = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) tot += sd[i][ch];
            db[kt * 64 + ch] = tot;
        }
        return;
    }
    const int k = blockIdx.x, t = threadIdx.x & 31, part = threadIdx.x >> 5;
    const size_t bstride = (size_t)ktiles * 64 * 32;
    const float *src = partial + ((size_t)(k >> 6) * 64 + (k & 63)) * 32 + t;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    int b = part;
    for (; b + 96 < nblocks; b += 128) {
        s0 += src[(size_t)b * bstride];
        s1 += src[(size_t)(b + 32) * bstride];
        s2 += src[(size_t)(b + 64) * bstride];
        s3 += src[(size_t)(b + 96) * bstride];
    }
    for (; b < nblocks; b += 32) s0 += src[(size_t)b * bstride];
    sm[part][t] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (part == 0 && t < rsc) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 32; ++i) s += sm[i][t];
        dw[(size_t)k * rsc + t] = s;
    }
}

unsigned blocks_for(long long total)
{
    long long nb = (total + 255) / 256;
    if (nb > 16384) nb = 16384;
    return (unsigned)(nb < 1 ? 1 : nb);
}

// ---------------------------------------------------------------------------------------
// Forward for strided few-channel stems (7x7 stride 2 on RGB): no im2col matrix and no im2col tile.
// For a fixed filter row r the S*C inputs of an output pixel are CONTIGUOUS in NHWC (a "run", 21 elements
// for 7x7x3), so the reduction is laid out as R runs padded to 24 = three 8-element groups, and the pixel
// operand of a matrix instruction (8 consecutive reduction elements per lane) is read straight from the
// input patch in LDS: run r, group part of output pixel (pr, pc) starts at patch row pr*sh + r, element
// pc*sw*C + 8*part.  With sw*C even that address is 4-byte aligned, so a group is four dword reads; the
// elements of a group past the end of the run belong to the neighbouring pixel and are masked to zero.
// The weights (64 c_out x R*24, zero padded) stay in registers; blocks are persistent over 8x32-pixel tiles
// and fetch the next tile's patch into registers while the current one is multiplied.
// ---------------------------------------------------------------------------------------
constexpr int ST_PITCH = 512;        // bytes per patch row in LDS (data + 48 bytes that the last group of a row may over-read)
constexpr int ST_ROWS = 24;          // patch rows in LDS (rows past the real patch stay zero)
constexpr int ST_MAXSL = 12;         // reduction slices of 16 (R * 24 <= 192)

template <int NSL>
__global__ __launch_bounds__(256, 2) void k_fwd_stem(const ConvGeom g, unsigned flags, const bf16_t *__restrict__ x, const bf16_t *__restrict__ w,
                                                  const float *__restrict__ bias, bf16_t *__restrict__ y, int tiles, int tiles_x, int tiles_y)
{
    __shared__ __attribute__((aligned(16))) char patch[2][ST_ROWS * ST_PITCH];
    __shared__ __attribute__((aligned(16))) bf16_t wlds[64 * ST_MAXSL * 16];   // [c_out][R*24 padded to the slices], zero where no weight
    __shared__ float bias_lds[64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hsel = lane >> 5;
    const int a0 = blockIdx.y * 64;
    const int run = g.S * g.C;                       // elements of one filter row
    const int prow = 7 * g.sh + g.R, pwe = (31 * g.sw + g.S) * g.C;   // real patch: rows, elements per row
    for (int i = tid; i < 2 * ST_ROWS * ST_PITCH / 4; i += 256) reinterpret_cast<unsigned *>(&patch[0][0])[i] = 0u;
    for (int i = tid; i < 64 * ST_MAXSL * 16 / 2; i += 256) reinterpret_cast<unsigned *>(wlds)[i] = 0u;
    if (tid < 64) bias_lds[tid] = ((flags & KF_BIAS) && a0 + tid < g.K) ? bias[a0 + tid] : 0.f;
    __syncthreads();
    // weights: coalesced 2-byte loads into the padded LDS layout (reduction element 24*r + j holds w[ch][r][j]), then
    // one 16-byte read per fragment: slice ks, channel half i; lane (channel i*32 + l%32, elements ks*16 + 8*(l/32) ..+7)
    {
        const int per_ch = g.R * run, total = 64 * per_ch;
        for (int e0 = 0; e0 < total; e0 += 256 * 8) {
            unsigned short v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int e = e0 + u * 256 + tid, ch = e / per_ch;
                v[u] = (e < total && a0 + ch < g.K) ? w[(size_t)a0 * per_ch + e] : (unsigned short)0;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int e = e0 + u * 256 + tid, ch = e / per_ch, rem = e - ch * per_ch, r = rem / run, j = rem - r * run;
                if (e < total) wlds[ch * (ST_MAXSL * 16) + r * 24 + j] = v[u];
            }
        }
    }
    __syncthreads();
    u32x4 wfr[NSL][2];
#pragma unroll
    for (int ks = 0; ks < NSL; ++ks)
#pragma unroll
        for (int i = 0; i < 2; ++i)
            wfr[ks][i] = *reinterpret_cast<const u32x4 *>(wlds + (i * 32 + (lane & 31)) * (ST_MAXSL * 16) + ks * 16 + 8 * hsel);

    // patch elements of this thread: element e = tid + 256*i -> (row, column element); fetched as 2-byte loads
    // patch fetch: thread t takes column element t of every patch row (a row is at most 232 elements), two rows per register
    auto fetch = [&](int tile, unsigned (&v)[ST_ROWS / 2]) {
        const int n = tile / (tiles_x * tiles_y), trem = tile - n * (tiles_x * tiles_y), ty = trem / tiles_x, tx = trem - ty * tiles_x;
        const int ih0 = ty * 8 * g.sh - g.ph, ie = (tx * 32 * g.sw - g.pw) * g.C + tid;
        const bool okc = tid < pwe && (unsigned)ie < (unsigned)(g.W * g.C);
        const bf16_t *src = x + ((size_t)n * g.H + ih0) * g.W * g.C + ie;
#pragma unroll
        for (int r = 0; r < ST_ROWS; ++r) {
            const bool ok = okc && r < prow && (unsigned)(ih0 + r) < (unsigned)g.H;
            const unsigned val = ok ? src[(size_t)r * g.W * g.C] : 0u;
            v[r >> 1] = (r & 1) ? v[r >> 1] | (val << 16) : val;
        }
    };
    auto stash = [&](int buf, const unsigned (&v)[ST_ROWS / 2]) {
        if (tid >= pwe) return;
#pragma unroll
        for (int r = 0; r < ST_ROWS; ++r)
            if (r < prow) *reinterpret_cast<unsigned short *>(&patch[buf][r * ST_PITCH + tid * 2]) = (unsigned short)((r & 1) ? v[r >> 1] >> 16 : v[r >> 1] & 0xffffu);
    };
    unsigned pv[ST_ROWS / 2];
    int tile = blockIdx.x;
    __syncthreads();   // zero fill done
    if (tile < tiles) { fetch(tile, pv); stash(0, pv); }
    __syncthreads();

    // per slice: which run / group this lane reads, and how many of its 8 elements are inside the run
    int pc_off = (lane & 31) * g.sw * g.C * 2, run_v = run;
    for (int it = 0; tile < tiles; tile += gridDim.x, ++it) {
        const bool more = tile + (int)gridDim.x < tiles;
        if (more) fetch(tile + gridDim.x, pv);
        const char *pb = &patch[it & 1][0];
        asm volatile("" : "+v"(pc_off), "+v"(run_v));   // keeps the per-slice addresses and masks from being computed ahead of the tile loop
        f32x16 acc[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        // the pixel fragments of slice ks + 1 are read before the matrix instructions of slice ks
        auto read_b = [&](int ks, u32x4 (&bf)[2]) {
            const int gidx = 2 * ks + hsel, r = gidx / 3, part = gidx - 3 * r;
            int nval = run_v - 8 * part;
            nval = r < g.R ? (nval < 0 ? 0 : nval > 8 ? 8 : nval) : 0;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int prr = (2 * wave + j) * g.sh + r;   // < 7*sh + R + 1 <= ST_ROWS
                const unsigned *src = reinterpret_cast<const unsigned *>(__builtin_assume_aligned(pb + prr * ST_PITCH + pc_off + part * 16, 4));
                unsigned d[4] = {src[0], src[1], src[2], src[3]};
#pragma unroll
                for (int q = 0; q < 4; ++q) d[q] &= nval > 2 * q + 1 ? 0xffffffffu : nval > 2 * q ? 0x0000ffffu : 0u;
                bf[j] = u32x4{d[0], d[1], d[2], d[3]};
            }
        };
        u32x4 bfr[2][2];
        read_b(0, bfr[0]);
#pragma unroll
        for (int ks = 0; ks < NSL; ++ks) {
            if (ks + 1 < NSL) read_b(ks + 1, bfr[(ks + 1) & 1]);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wfr[ks][i]), __builtin_bit_cast(bf16x8, bfr[ks & 1][j]), acc[i][j], 0, 0, 0);
        }
        // accumulator element v of lane l: channel i*32 + 8*(v/4) + 4*(l/32) + v%4, pixel l%32 of row 2*wave + j; lanes l and l+32
        // swap halves of two channel groups so that each stores 8 consecutive channels
        {
            const int n = tile / (tiles_x * tiles_y), trem = tile - n * (tiles_x * tiles_y), ty = trem / tiles_x, tx = trem - ty * tiles_x;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int pr = ty * 8 + 2 * wave + j, qc = tx * 32 + (lane & 31);
                const bool okp = pr < g.Ho && qc < g.Wo;
                bf16_t *orow = y + ((size_t)(n * g.Ho + pr) * g.Wo + qc) * g.K + a0;
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int gp = 0; gp < 2; ++gp) {
                        unsigned pkd[2][2];
#pragma unroll
                        for (int e = 0; e < 2; ++e) {
                            const int gq = 2 * gp + e;
                            const f32x4 bv = *reinterpret_cast<const f32x4 *>(bias_lds + i * 32 + 8 * gq + 4 * hsel);
                            float v0 = acc[i][j][4 * gq] + bv.x, v1 = acc[i][j][4 * gq + 1] + bv.y, v2 = acc[i][j][4 * gq + 2] + bv.z,
                                  v3 = acc[i][j][4 * gq + 3] + bv.w;
                            if (flags & KF_RELU) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f); }
                            pkd[e][0] = pack_bf16(v0, v1);
                            pkd[e][1] = pack_bf16(v2, v3);
                        }
                        const auto s0 = __builtin_amdgcn_permlane32_swap(pkd[0][0], pkd[1][0], false, false);
                        const auto s1 = __builtin_amdgcn_permlane32_swap(pkd[0][1], pkd[1][1], false, false);
                        const int ch = i * 32 + 8 * (2 * gp + hsel);
                        if (okp && a0 + ch < g.K) *reinterpret_cast<u32x4 *>(orow + ch) = u32x4{s0[0], s1[0], s0[1], s1[1]};
                    }
            }
        }
        if (more) stash((it + 1) & 1, pv);   // the other buffer was last read two tiles ago, before the previous barrier
        __syncthreads();
    }
}

}  // namespace

int small_c_kpad(const ConvGeom &g)
{
    if ((g.C % 8) == 0) return 0;
    const int rsc = g.R * g.S * g.C;
    const int kpad = (rsc + 31) / 32 * 32;
    return kpad <= 256 ? kpad : 0;
}

bool small_c_direct(const ConvGeom &g)
{
    if ((g.C % 8) == 0 || g.R * g.S * g.C > 32 || (g.K % 8) != 0) return false;
    return (long long)(7 * g.sh + g.R) * ((31 * g.sw + g.S) * g.C) <= DPATCH;   // the forward kernel's input patch fits its LDS slot
}

hipError_t small_c_fwd_direct(const ConvGeom &g, unsigned flags, const bf16_t *x, const bf16_t *w, const float *bias, bf16_t *y,
                              hipStream_t st)
{
    const int tiles_x = (g.Wo + 31) / 32, tiles_y = (g.Ho + 7) / 8, ktiles = (g.K + 63) / 64;
    const long long tiles = (long long)g.N * tiles_x * tiles_y;
    const int nb = (int)(tiles < 2048 ? tiles : 2048);   // persistent beyond eight blocks per CU
    const unsigned inv_c = g.C == 1 ? 0u : (unsigned)((0x100000000ull + g.C - 1) / g.C);   // __umulhi(e, inv_c) == e / C for e < 65536
    TapTable taps;
    const int pwe = (31 * g.sw + g.S) * g.C;
    for (int kk = 0; kk < 32; ++kk) {
        const int rs = kk / g.C, c = kk - rs * g.C, r = rs / g.S, s2 = rs - r * g.S;
        taps.off[kk] = kk < g.R * g.S * g.C ? (unsigned short)(r * pwe + s2 * g.C + c) : (unsigned short)0;
    }
    hipLaunchKernelGGL(k_fwd_direct, dim3((unsigned)nb, (unsigned)ktiles), dim3(256), 0, st, g, flags, x, w, bias, y, (int)tiles,
                       tiles_x, tiles_y, inv_c, taps);
    return hipGetLastError();
}

// blocks along the pixel range of the direct filter-gradient kernel, and the bytes of its fp32 partials
int small_c_wgrad_blocks(const ConvGeom &g)
{
    const long long steps = ((long long)g.N * g.Ho * g.Wo + 63) / 64;
    long long nb = (steps + 3) / 4;   // at least four 64-pixel steps per block
    if (nb > 1024) nb = 1024;
    const long long spb = (steps + nb - 1) / nb;
    return (int)((steps + spb - 1) / spb);
}
size_t small_c_wgrad_partial_bytes(const ConvGeom &g)   // filter-gradient partials, then bias-gradient partials
{
    return (size_t)small_c_wgrad_blocks(g) * ((g.K + 63) / 64) * 64 * (32 + 1) * sizeof(float);
}

hipError_t small_c_wgrad_direct(const ConvGeom &g, const bf16_t *x, const bf16_t *dy, const bf16_t *ymask, float *partial, float *dw,
                                float *db, hipStream_t st)
{
    const long long steps = ((long long)g.N * g.Ho * g.Wo + 63) / 64;
    const int nb = small_c_wgrad_blocks(g), ktiles = (g.K + 63) / 64;
    const int spb = (int)((steps + nb - 1) / nb);
    float *dbp = db != nullptr ? partial + (size_t)nb * ktiles * 64 * 32 : nullptr;
    hipLaunchKernelGGL(k_wgrad_direct, dim3((unsigned)nb, (unsigned)ktiles), dim3(256), 0, st, g, x, dy, ymask, partial, dbp, spb);
    dp_trace_main_kernel_done(st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_wgrad_direct_sum, dim3((unsigned)(g.K + (db != nullptr ? ktiles : 0))), dim3(1024), 0, st, g.K, g.R * g.S * g.C, nb,
                       ktiles, partial, dw, dbp, db);
    return hipGetLastError();
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

// Strided few-channel stems take the row-run kernel: filter rows of at most 24 elements whose pixel step is a whole
// number of dwords, at most 8 rows, an 8x32 tile's patch within the LDS slot, 64-aligned c_out tiles of 8 channels.
bool small_c_stem(const ConvGeom &g)
{
    if ((g.C % 8) == 0 || g.S * g.C > 24 || ((g.sw * g.C * 2) % 4) != 0 || g.R * 24 > ST_MAXSL * 16 || (g.K % 8) != 0) return false;
    if (g.R * g.S * g.C <= 32) return false;   // the one-slice kernels above are the better fit
    const int prow = 7 * g.sh + g.R, pwe = (31 * g.sw + g.S) * g.C;
    return prow + 1 <= ST_ROWS && pwe * 2 + 48 <= ST_PITCH && pwe <= 256;
}

hipError_t small_c_fwd_stem(const ConvGeom &g, unsigned flags, const bf16_t *x, const bf16_t *w, const float *bias, bf16_t *y, hipStream_t st)
{
    const int tiles_x = (g.Wo + 31) / 32, tiles_y = (g.Ho + 7) / 8, ktiles = (g.K + 63) / 64;
    const long long tiles = (long long)g.N * tiles_x * tiles_y;
    const int nb = (int)(tiles < 512 ? tiles : 512);   // persistent beyond two blocks per CU (each block stages the weights once)
    const int nsl = (g.R * 24 + 15) / 16;
    dim3 grid((unsigned)nb, (unsigned)ktiles), block(256);
#define STEM_CASE(N) case N: hipLaunchKernelGGL(k_fwd_stem<N>, grid, block, 0, st, g, flags, x, w, bias, y, (int)tiles, tiles_x, tiles_y); break;
    switch (nsl) {
        STEM_CASE(2) STEM_CASE(3) STEM_CASE(4) STEM_CASE(5) STEM_CASE(6) STEM_CASE(7) STEM_CASE(8) STEM_CASE(9) STEM_CASE(10) STEM_CASE(11) STEM_CASE(12)
    default: return hipErrorInvalidValue;
    }
#undef STEM_CASE
    return hipGetLastError();
}
