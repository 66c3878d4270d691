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
// k_wgrad_direct does the same for the filter gradient with both operands stored pixel-major in LDS and
// transposed by the LDS transpose read (and, when asked, the ReLU mask applied and the bias gradient summed
// on the way), one fp32 partial per block, and k_wgrad_direct_sum adds the partials in block order.  Both
// passes then move little more than the output activation / the upstream gradient once, which is what
// bounds these layers.  The 3x3 / stride 1 / pad 1 RGB stem whose rows are whole 32-pixel segments (the
// first layer of VGG-16) has kernels of its own, k_fwd_rgb3 and k_wgrad_rgb3: per-wave pipelines of
// direct-to-LDS loads without block barriers, the tap operand read straight from three input-row strips.
#include "dma_common.h"
#include <algorithm>

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

// Filter gradient: block b sums pixels [b*ppb, (b+1)*ppb) in steps of 64.  Both operands go to LDS as they come from
// memory, pixel-major: gN[64 pixels][64 c_out], xN[64 pixels][32 taps], 16 bytes per thread and store; the matrix
// cores want them reduction-contiguous, which the LDS transpose read delivers (lane l of a 16-lane group points at
// pixel row 8*(l>>5) + (l&15)/4 (+4 for the second half), operand rows 16*((l>>4)&1) + 4*(l&3) .. +3).  Row pitches
// of 160 and 96 bytes put the four pixel rows one 16-lane group reads into distinct bank octets.  The tiles are
// double-buffered, so a step costs one barrier.  Wave w multiplies the 16-pixel slice w of every step; the four
// waves' sums are added through LDS at the end.
constexpr int WGP = 80, WXP = 48;   // row pitches in bf16
DEVFN u32x2 lds_tr_read(unsigned addr)
{
    u32x2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(v) : "v"(addr) : "memory");
    return v;
}
__global__ __launch_bounds__(256) void k_wgrad_direct(ConvGeom g, const bf16_t *x, const bf16_t *dy, const bf16_t *ym, float *partial,
                                                      float *db_partial, int steps_per_block)
{
    __shared__ __attribute__((aligned(16))) char lds[2 * 64 * (WGP + WXP) * 2];   // 32 KiB: the tiles, then the waves' sums
    static_assert(sizeof(lds) >= 4 * 64 * 32 * sizeof(float), "the four waves' sums fit the tile buffers");
    bf16_t (*gN)[64 * WGP] = reinterpret_cast<bf16_t (*)[64 * WGP]>(lds);
    bf16_t (*xN)[64 * WXP] = reinterpret_cast<bf16_t (*)[64 * WXP]>(lds + 2 * 64 * WGP * 2);
    float (*red)[64][32] = reinterpret_cast<float (*)[64][32]>(lds);
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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
    auto stash = [&](Regs &rg, int buf) {   // registers -> LDS rows; mask and bias gradient on the way
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const u32x4 mv = apply_mask(rg.gv[h], rg.yv[h]);
            *reinterpret_cast<u32x4 *>(&gN[buf][gp * WGP + gc + h * 8]) = mv;
            if (db_partial != nullptr) {
                const unsigned wv[4] = {mv.x, mv.y, mv.z, mv.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) dbacc[h * 8 + e] += __uint_as_float((e & 1) ? (wv[e >> 1] & 0xffff0000u) : (wv[e >> 1] << 16));
            }
        }
        *reinterpret_cast<u32x4 *>(&xN[buf][xp * WXP + xt]) =
            u32x4{rg.xv[0] | (rg.xv[1] << 16), rg.xv[2] | (rg.xv[3] << 16), rg.xv[4] | (rg.xv[5] << 16), rg.xv[6] | (rg.xv[7] << 16)};
    };
    const int i16 = lane & 15, tl = wave * 16 + (lane >> 5) * 8 + (i16 >> 2), cl = ((lane >> 4) & 1) * 16 + (i16 & 3) * 4;
    const unsigned fg = (unsigned)(size_t)(__attribute__((address_space(3))) const char *)&gN[0][tl * WGP + cl];
    const unsigned fx = (unsigned)(size_t)(__attribute__((address_space(3))) const char *)&xN[0][tl * WXP + cl];
    auto multiply = [&](int buf) {
        const unsigned pg = fg + buf * (64 * WGP * 2), px = fx + buf * (64 * WXP * 2);
        u32x2 v[6];
        v[0] = lds_tr_read(px);
        v[1] = lds_tr_read(px + 4 * WXP * 2);
        v[2] = lds_tr_read(pg);
        v[3] = lds_tr_read(pg + 4 * WGP * 2);
        v[4] = lds_tr_read(pg + 64);
        v[5] = lds_tr_read(pg + 64 + 4 * WGP * 2);
        asm volatile("s_waitcnt lgkmcnt(0)");
#pragma unroll
        for (int i = 0; i < 6; ++i) asm volatile("" : "+v"(v[i]));   // the products below depend on the wait
        const bf16x8 b = __builtin_bit_cast(bf16x8, u32x4{v[0].x, v[0].y, v[1].x, v[1].y});
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const bf16x8 a = __builtin_bit_cast(bf16x8, u32x4{v[2 + 2 * i].x, v[2 + 2 * i].y, v[3 + 2 * i].x, v[3 + 2 * i].y});
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
        }
    };
    if (sbeg < send) load(sbeg, ra);
    if (sbeg + 1 < send) load(sbeg + 1, rb);
    // a buffer is written again two steps later, after the barrier of the step between: by then every wave has
    // left the multiply that read it
    for (int step = sbeg; step < send; step += 2) {
        stash(ra, 0);
        __syncthreads();
        if (step + 2 < send) load(step + 2, ra);
        multiply(0);
        if (step + 1 < send) {
            stash(rb, 1);
            __syncthreads();
            if (step + 3 < send) load(step + 3, rb);
            multiply(1);
        }
    }
    __syncthreads();   // every wave has left its last multiply: the tiles give way to the sums
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

// ---------------------------------------------------------------------------------------
// Filter gradient of the 3x3 / stride 1 / pad 1 RGB stem (C = 3, W a multiple of 32), bound by reading dy once.
// The unit of work is a segment: 32 consecutive pixels of one output row.  Every WAVE walks its own contiguous range of
// segments through its own LDS stages, so the loop has no block barrier; both operands arrive by direct-to-LDS loads:
//   * dy tile [32 pixels][64 c_out] (4 KiB, four loads), 64-byte halves of a row swapped on odd row pairs so that the
//     LDS transpose read of the c_out x pixel fragments is conflict free;
//   * the three input rows the segment's taps touch, each as 14 aligned 16-byte chunks starting 16 bytes before the
//     segment's first pixel (one load; lanes of rows outside the image or of the chunk beyond a row end fetch zeros).
// The tap x pixel operand needs no im2col tile: lane l (tap t = l % 32 = (r, s, c), pixels 8*(l/32) .. +7 of a 16-pixel
// slice) reads its eight elements straight from row r of the strips, 6 bytes apart, at immediate offsets from one
// address; lanes of the five padding taps read a part of the stage that the load always fills with zeros.
// The bias gradient is one more matrix instruction per dy fragment (multiplied with ones).
// Per segment a wave issues 5 loads, 24 LDS reads, 6 matrix instructions and a handful of vector instructions.
// ---------------------------------------------------------------------------------------
constexpr int RG_NS = 3, RG_DY = 4096, RG_STAGE = RG_DY + 1024, RG_XPITCH = 224, RG_ZERO = 700;
DEVFN void dma16s(__amdgpu_buffer_rsrc_t r, unsigned lds_base, unsigned voff, unsigned soff)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_void)(size_t)lds_base, 16, voff, soff, 0, 0);
}
DEVFN void dma16s_nt(__amdgpu_buffer_rsrc_t r, unsigned lds_base, unsigned voff, unsigned soff)   // non-temporal: data that is read once
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_void)(size_t)lds_base, 16, voff, soff, 0, 2);
}
template <int OFF> DEVFN unsigned lds_read_u16(unsigned addr)
{
    unsigned v;
    asm volatile("ds_read_u16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int OFF> DEVFN u32x2 lds_tr_read_off(unsigned addr)
{
    u32x2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <bool DB>   // DB: also sum the bias gradient
__global__ __launch_bounds__(256) void k_wgrad_rgb3(ConvGeom g, const bf16_t *x, const bf16_t *dy, float *partial, float *db_partial,
                                                    int segs_total, int segs_per_wave)
{
    __shared__ __attribute__((aligned(1024))) char lds[4 * RG_NS * RG_STAGE];   // 60 KiB: per-wave stages, then the waves' sums
    static_assert(sizeof(lds) >= 4 * 64 * 33 * sizeof(float), "the four waves' sums fit the stages");
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int a0 = blockIdx.y * 64;
    const int spr = g.W / 32;                                     // segments per image row
    const int sbeg = min((int)(blockIdx.x * 4 + wave) * segs_per_wave, segs_total), send = min(sbeg + segs_per_wave, segs_total);
    __amdgpu_buffer_rsrc_t rdy = make_rsrc(dy, (size_t)g.N * g.H * g.W * g.K * 2);
    __amdgpu_buffer_rsrc_t rx = make_rsrc(x, (size_t)g.N * g.H * g.W * 3 * 2);
    const unsigned base = lds_offset(lds) + wave * (RG_NS * RG_STAGE);

    // dy loads: lane l of load q fills 16-byte position l%8 of tile row q*8 + l/8 with global chunk (l%8) ^ 4*swz(row)
    unsigned voffA[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int t = q * 8 + lane / 8, c = (lane % 8) ^ (seg_swz<64>(t) << 2);
        voffA[q] = ((unsigned)t * g.K + a0 + c * 8) * 2u;
    }
    // x load: lane l < 42 fetches chunk l%14 of strip row l/14 (input row h - 1 + l/14), relative to the segment's first pixel
    const int xr = lane / 14, xc = lane - xr * 14;
    const int xlane = (xr - 1) * g.W * 6 + xc * 16 - 16;
    // bit 0: row above the image when h == 0; 1: row below when h == H-1; 2: chunk before the row start; 3: chunk past its end
    const unsigned xflags = lane >= 42 ? 0x10u : (xr == 0 ? 1u : 0u) | (xr == 2 ? 2u : 0u) | (xc == 0 ? 4u : 0u) | (xc == 13 ? 8u : 0u);

    int seg = sbeg, row = 0, qs = 0, h = 0;   // position of the next segment to issue: flat row n*H + h, segment in the row
    if (sbeg < send) { row = sbeg / spr; qs = sbeg - row * spr; h = row % g.H; }
    auto issue = [&](unsigned st) {   // st: byte offset of the stage
        const unsigned m = (unsigned)(row * g.W + qs * 32);   // first pixel of the segment, flat
        const unsigned soff = m * (unsigned)g.K * 2u;
#pragma unroll
        for (int q = 0; q < 4; ++q) dma16s_nt(rdy, base + st + q * 1024, voffA[q], soff);
        const unsigned cond = 0x10u | (h == 0 ? 1u : 0u) | (h == g.H - 1 ? 2u : 0u) | (qs == 0 ? 4u : 0u) | (qs == spr - 1 ? 8u : 0u);
        dma16s(rx, base + st + RG_DY, (xflags & cond) ? OOR : (unsigned)(xlane + (int)(m * 6u)), 0);
        ++seg;
        if (++qs == spr) { qs = 0; ++row; if (++h == g.H) h = 0; }
    };

    f32x16 acc[2], accdb[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) { acc[i][e] = 0.f; accdb[i][e] = 0.f; }

    // transpose-read addresses of the dy fragments (c_out block i, pixel slice ks): lane l of a 16-lane group points at pixel
    // row 16*ks + 8*(l>>5) + (l&15)/4 (+4 for the second half), c_out 32*i + 16*((l>>4)&1) + 4*(l&3) .. +3
    const int i16 = lane & 15, tl = (lane >> 5) * 8 + (i16 >> 2), cl = ((lane >> 4) & 1) * 16 + (i16 & 3) * 4;
    unsigned fa[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) fa[i] = base + tl * 128 + (((i ^ seg_swz<64>(tl)) << 6) | (cl << 1));
    // tap operand: element j of lane l is input pixel (p0 + 8*(l>>5) + j) - 1 + s of strip row r, channel c
    const int tap = lane & 31, tr_ = tap / 9, ts_ = (tap - tr_ * 9) / 3, tc_ = tap - tr_ * 9 - ts_ * 3;
    const unsigned fx = base + RG_DY + (tap < 27 ? tr_ * RG_XPITCH + 10 + ts_ * 6 + tc_ * 2 + (lane >> 5) * 48 : RG_ZERO);

    const int nseg = send - sbeg;
    if (nseg > 0) issue(0);
    if (nseg > 1) issue(RG_STAGE);
    unsigned sb = 0, sfill = 2 * RG_STAGE;   // stage of segment i; stage that segment i+2 goes to
    for (int i = 0; i < nseg; ++i) {
        if (i + 1 < nseg) wait_vmcnt<5>(); else wait_vmcnt<0>();
        if (i + 2 < nseg) issue(sfill);   // that stage was read two segments ago, and those reads have returned
        const unsigned pa0 = fa[0] + sb, pa1 = fa[1] + sb, px = fx + sb;
        unsigned xe[16];
        u32x2 av[8];
        xe[0] = lds_read_u16<0>(px);   xe[1] = lds_read_u16<6>(px);   xe[2] = lds_read_u16<12>(px);  xe[3] = lds_read_u16<18>(px);
        xe[4] = lds_read_u16<24>(px);  xe[5] = lds_read_u16<30>(px);  xe[6] = lds_read_u16<36>(px);  xe[7] = lds_read_u16<42>(px);
        xe[8] = lds_read_u16<96>(px);  xe[9] = lds_read_u16<102>(px); xe[10] = lds_read_u16<108>(px); xe[11] = lds_read_u16<114>(px);
        xe[12] = lds_read_u16<120>(px); xe[13] = lds_read_u16<126>(px); xe[14] = lds_read_u16<132>(px); xe[15] = lds_read_u16<138>(px);
        av[0] = lds_tr_read_off<0>(pa0);    av[1] = lds_tr_read_off<512>(pa0);         // slice 0, c_out block 0
        av[2] = lds_tr_read_off<0>(pa1);    av[3] = lds_tr_read_off<512>(pa1);         // slice 0, block 1
        av[4] = lds_tr_read_off<2048>(pa0); av[5] = lds_tr_read_off<2048 + 512>(pa0);  // slice 1, block 0
        av[6] = lds_tr_read_off<2048>(pa1); av[7] = lds_tr_read_off<2048 + 512>(pa1);  // slice 1, block 1
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int e = 0; e < 16; ++e) asm volatile("" : "+v"(xe[e]));   // what follows depends on the wait
#pragma unroll
        for (int e = 0; e < 8; ++e) asm volatile("" : "+v"(av[e]));
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const unsigned *e = xe + 8 * ks;
            const bf16x8 b = __builtin_bit_cast(bf16x8, u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)});
#pragma unroll
            for (int ii = 0; ii < 2; ++ii) {
                const u32x2 lo = av[4 * ks + 2 * ii], hi = av[4 * ks + 2 * ii + 1];
                const bf16x8 a = __builtin_bit_cast(bf16x8, u32x4{lo.x, lo.y, hi.x, hi.y});
                acc[ii] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[ii], 0, 0, 0);
                if constexpr (DB) accdb[ii] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, ones_bf16(), accdb[ii], 0, 0, 0);
            }
        }
        sfill = sb;
        sb = sb + RG_STAGE == RG_NS * RG_STAGE ? 0u : sb + RG_STAGE;
    }
    __syncthreads();   // every wave is done with its stages: they give way to the sums
    float (*red)[64][33] = reinterpret_cast<float (*)[64][33]>(lds);
    // D element v of lane l: row 8*(v/4) + 4*(l/32) + v%4 (c_out), column l%32 (tap)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[wave][i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)][lane & 31] = acc[i][v];
    if (DB && (lane & 31) == 0) {   // every column of the ones product holds the same sums
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) red[wave][i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)][32] = accdb[i][v];
    }
    __syncthreads();
    float *out = partial + ((size_t)blockIdx.x * gridDim.y + blockIdx.y) * 64 * 32;
    for (int id = tid; id < 64 * 32; id += 256) {
        const int k = id >> 5, t = id & 31;
        out[id] = (red[0][k][t] + red[1][k][t]) + (red[2][k][t] + red[3][k][t]);
    }
    if (DB && tid < 64)
        db_partial[((size_t)blockIdx.x * gridDim.y + blockIdx.y) * 64 + tid] = (red[0][tid][32] + red[1][tid][32]) + (red[2][tid][32] + red[3][tid][32]);
}

// ---------------------------------------------------------------------------------------
// Forward of the same stem, bound by writing y once: the segment walk and the strip loads of k_wgrad_rgb3, no dy.
// The 27 taps are laid out as three slices of 16 (one per filter row r): the first eight reduction slots of a slice
// are the taps (r, 0..7) in (s, c) order, contiguous elements of strip row r starting at the pixel's left neighbour,
// the ninth slot is tap (r, 8) and the rest is padding.  Lane l of the pixel operand (pixel l % 32, slots
// 8*(l/32) .. +7) therefore reads eight consecutive elements at immediate offsets from one address; the upper half
// keeps only its first element (the others belong to the neighbouring pixel and are cleared; the weights there are
// zero as well).  The weight fragments stay in registers.  The 64 x 32 sums of a segment get bias and ReLU, go to the
// wave's LDS tile [32 pixels][64 + 8] as bf16 and leave as whole 128-byte pixel rows.
// Loads and stores share one in-order counter: behind the strip load of segment i were issued, per later segment, one
// load and four stores, which gives the wait counts in the loop (a load is issued for every slot, past the wave's range
// one that fetches nothing, so the counts hold to the end).
// ---------------------------------------------------------------------------------------
constexpr int RF_NS = 3, RF_OPITCH = 144, RF_WAVE = RF_NS * 1024 + 32 * RF_OPITCH;
template <int OFF> DEVFN void lds_write8(unsigned addr, u32x2 v)
{
    asm volatile("ds_write_b64 %0, %1 offset:%2" ::"v"(addr), "v"(v), "n"(OFF) : "memory");
}
__global__ __launch_bounds__(256) void k_fwd_rgb3(ConvGeom g, unsigned flags, const bf16_t *x, const bf16_t *w, const float *bias, bf16_t *y,
                                                  int segs_total, int segs_per_wave)
{
    __shared__ __attribute__((aligned(1024))) char lds[4 * RF_WAVE];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int a0 = blockIdx.y * 64, half = lane >> 5;
    const int spr = g.W / 32;
    const int sbeg = min((int)(blockIdx.x * 4 + wave) * segs_per_wave, segs_total), send = min(sbeg + segs_per_wave, segs_total);
    __amdgpu_buffer_rsrc_t rx = make_rsrc(x, (size_t)g.N * g.H * g.W * 3 * 2);
    __amdgpu_buffer_rsrc_t ry = make_rsrc(y, (size_t)g.N * g.H * g.W * g.K * 2);
    const unsigned base = lds_offset(lds) + wave * RF_WAVE, obase = base + RF_NS * 1024;

    // weight fragments: row a0 + 32*i + l%32; slice r, slot 8*half + j: tap (r, j) for the lower half, tap (r, 8) in slot 8, zero elsewhere
    bf16x8 afr[3][2];
    f32x4 bv[2][4];   // bias of the channels of accumulator elements 4*gq .. 4*gq+3 of block i
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int wrow = a0 + i * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            unsigned v[4] = {0, 0, 0, 0};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const unsigned val = (half == 0 || j == 0) ? w[(size_t)wrow * 27 + r * 9 + (half ? 8 : j)] : 0u;
                v[j >> 1] |= val << ((j & 1) * 16);
            }
            afr[r][i] = __builtin_bit_cast(bf16x8, u32x4{v[0], v[1], v[2], v[3]});
        }
#pragma unroll
        for (int gq = 0; gq < 4; ++gq)
            bv[i][gq] = (flags & KF_BIAS) ? *reinterpret_cast<const f32x4 *>(bias + a0 + i * 32 + 8 * gq + 4 * half) : f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const int xr = lane / 14, xc = lane - xr * 14;
    const int xlane = (xr - 1) * g.W * 6 + xc * 16 - 16;
    const unsigned xflags = lane >= 42 ? 0x10u : (xr == 0 ? 1u : 0u) | (xr == 2 ? 2u : 0u) | (xc == 0 ? 4u : 0u) | (xc == 13 ? 8u : 0u);
    int row = 0, qs = 0, h = 0;   // position of the next segment to issue
    if (sbeg < send) { row = sbeg / spr; qs = sbeg - row * spr; h = row % g.H; }
    auto issue = [&](unsigned st, bool live) {
        const unsigned m = (unsigned)(row * g.W + qs * 32);
        const unsigned cond = (live ? 0x10u : 0x1fu) | (h == 0 ? 1u : 0u) | (h == g.H - 1 ? 2u : 0u) | (qs == 0 ? 4u : 0u) | (qs == spr - 1 ? 8u : 0u);
        dma16s(rx, base + st, (xflags & cond) ? OOR : (unsigned)(xlane + (int)(m * 6u)), 0);
        if (live && ++qs == spr) { qs = 0; ++row; if (++h == g.H) h = 0; }
    };
    // pixel operand: pixel l%32 of strip row r (+224*r); the lower half starts at the left neighbour's channel 0, the upper half 16 bytes on
    const unsigned fx = base + 10 + (lane & 31) * 6 + half * 16;
    const unsigned keep0 = half ? 0x0000ffffu : 0xffffffffu, keep = half ? 0u : 0xffffffffu;
    // accumulator element 4*gq + e of block i is channel 32*i + 8*gq + 4*half + e of pixel l%32
    const unsigned ostage = obase + (lane & 31) * RF_OPITCH + half * 8;
    // copy-out: lane l moves 16 bytes: pixel row 8*it + l/8, chunk l%8
    const unsigned orow = obase + (lane >> 3) * RF_OPITCH + (lane & 7) * 16;
    const unsigned yoff = ((unsigned)(lane >> 3) * g.K + a0) * 2u + (lane & 7) * 16, ystep = 8u * g.K * 2u;

    const int nseg = send - sbeg;
    issue(0, 0 < nseg);
    issue(1024, 1 < nseg);
    unsigned sb = 0, sfill = 2 * 1024;
    for (int i = 0; i < nseg; ++i) {
        if (i == 0) wait_vmcnt<1>(); else if (i == 1) wait_vmcnt<5>(); else wait_vmcnt<9>();
        issue(sfill, i + 2 < nseg);
        const unsigned px = fx + sb;
        unsigned xe[24];
#define DP_RD8(R) xe[8 * R + 0] = lds_read_u16<224 * R + 0>(px); xe[8 * R + 1] = lds_read_u16<224 * R + 2>(px); \
                  xe[8 * R + 2] = lds_read_u16<224 * R + 4>(px); xe[8 * R + 3] = lds_read_u16<224 * R + 6>(px); \
                  xe[8 * R + 4] = lds_read_u16<224 * R + 8>(px); xe[8 * R + 5] = lds_read_u16<224 * R + 10>(px); \
                  xe[8 * R + 6] = lds_read_u16<224 * R + 12>(px); xe[8 * R + 7] = lds_read_u16<224 * R + 14>(px);
        DP_RD8(0) DP_RD8(1) DP_RD8(2)
#undef DP_RD8
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int e = 0; e < 24; ++e) asm volatile("" : "+v"(xe[e]));   // what follows depends on the wait
        f32x16 acc[2];
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[ii][e] = 0.f;
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const unsigned *e = xe + 8 * r;
            const bf16x8 b = __builtin_bit_cast(bf16x8, u32x4{(e[0] | (e[1] << 16)) & keep0, (e[2] | (e[3] << 16)) & keep, (e[4] | (e[5] << 16)) & keep,
                                                              (e[6] | (e[7] << 16)) & keep});
#pragma unroll
            for (int ii = 0; ii < 2; ++ii) acc[ii] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afr[r][ii], b, acc[ii], 0, 0, 0);
        }
        // the tile is free: the copy-out reads of the previous segment had returned before its stores were issued
        auto packed = [&](int ii, int gq) {
            float v0 = acc[ii][4 * gq] + bv[ii][gq].x, v1 = acc[ii][4 * gq + 1] + bv[ii][gq].y;
            float v2 = acc[ii][4 * gq + 2] + bv[ii][gq].z, v3 = acc[ii][4 * gq + 3] + bv[ii][gq].w;
            if (flags & KF_RELU) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f); }
            return u32x2{pack_bf16(v0, v1), pack_bf16(v2, v3)};
        };
        lds_write8<0>(ostage, packed(0, 0));  lds_write8<16>(ostage, packed(0, 1));  lds_write8<32>(ostage, packed(0, 2));  lds_write8<48>(ostage, packed(0, 3));
        lds_write8<64>(ostage, packed(1, 0)); lds_write8<80>(ostage, packed(1, 1));  lds_write8<96>(ostage, packed(1, 2));  lds_write8<112>(ostage, packed(1, 3));
        u32x4 o[4];
        o[0] = lds_read16<0>(orow); o[1] = lds_read16<8 * RF_OPITCH>(orow); o[2] = lds_read16<16 * RF_OPITCH>(orow); o[3] = lds_read16<24 * RF_OPITCH>(orow);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int it = 0; it < 4; ++it) asm volatile("" : "+v"(o[it]));
        const unsigned soff = (unsigned)(sbeg + i) * 32u * g.K * 2u;   // segment s starts at flat pixel 32*s
#pragma unroll
        for (int it = 0; it < 4; ++it) __builtin_amdgcn_raw_buffer_store_b128(o[it], ry, yoff + it * ystep, soff, 0);
        sfill = sb;
        sb = sb + 1024 == RF_NS * 1024 ? 0u : sb + 1024;
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
    float sa[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) sa[u] = 0.f;
    int b = part;
    for (; b + 224 < nblocks; b += 256) {   // eight loads in flight
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[(size_t)(b + 32 * u) * bstride];
#pragma unroll
        for (int u = 0; u < 8; ++u) sa[u] += v[u];
    }
    for (; b < nblocks; b += 32) sa[0] += src[(size_t)b * bstride];
    sm[part][t] = ((sa[0] + sa[1]) + (sa[2] + sa[3])) + ((sa[4] + sa[5]) + (sa[6] + sa[7]));
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

// shapes the 3x3 RGB stem kernels take (byte offsets into y / dy stay below 2^31)
static bool rgb3_shape(const ConvGeom &g)
{
    return g.C == 3 && g.R == 3 && g.S == 3 && g.sh == 1 && g.sw == 1 && g.ph == 1 && g.pw == 1 && g.W % 32 == 0 && g.K % 64 == 0 &&
           (unsigned long long)g.N * g.H * g.W * g.K * 2 < (1ull << 31);
}

bool small_c_direct(const ConvGeom &g)
{
    if ((g.C % 8) == 0 || g.R * g.S * g.C > 32 || (g.K % 8) != 0) return false;
    return (long long)(7 * g.sh + g.R) * ((31 * g.sw + g.S) * g.C) <= DPATCH;   // the forward kernel's input patch fits its LDS slot
}

hipError_t small_c_fwd_direct(const ConvGeom &g, unsigned flags, const bf16_t *x, const bf16_t *w, const float *bias, bf16_t *y,
                              hipStream_t st)
{
    if (rgb3_shape(g)) {
        const long long total = (long long)g.N * g.H * (g.W / 32);
        long long waves = (total + 3) / 4;   // at least four segments per wave
        if (waves > 4096) waves = 4096;      // four resident blocks of four waves per compute unit
        const long long spw = (total + waves - 1) / waves;
        const int nb = (int)(((total + spw - 1) / spw + 3) / 4);
        hipLaunchKernelGGL(k_fwd_rgb3, dim3((unsigned)nb, (unsigned)(g.K / 64)), dim3(256), 0, st, g, flags, x, w, bias, y, (int)total, (int)spw);
        return hipGetLastError();
    }
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

// blocks along the pixel range of the direct filter-gradient kernels, and the bytes of their fp32 partials
static int wgrad_blocks_direct(const ConvGeom &g)
{
    const long long steps = ((long long)g.N * g.Ho * g.Wo + 63) / 64;
    long long nb = (steps + 3) / 4;   // at least four 64-pixel steps per block
    if (nb > 1024) nb = 1024;
    const long long spb = (steps + nb - 1) / nb;
    return (int)((steps + spb - 1) / spb);
}
// segments per wave and blocks of four waves of the stem's filter-gradient kernel
static void wgrad_rgb3_split(const ConvGeom &g, int *segs, int *per_wave, int *blocks)
{
    const long long total = (long long)g.N * g.H * (g.W / 32);
    long long waves = (total + 3) / 4;   // at least four segments per wave
    if (waves > 2048) waves = 2048;      // two resident blocks of four waves per compute unit
    const long long spw = (total + waves - 1) / waves;
    *segs = (int)total; *per_wave = (int)spw; *blocks = (int)(((total + spw - 1) / spw + 3) / 4);
}
const char *small_c_fwd_kernel(const ConvGeom &g) { return rgb3_shape(g) ? "k_fwd_rgb3" : "k_fwd_direct"; }
const char *small_c_wgrad_kernel(const ConvGeom &g, bool masked, bool with_db)
{
    return masked || !rgb3_shape(g) ? "k_wgrad_direct" : with_db ? "k_wgrad_rgb3<true>" : "k_wgrad_rgb3<false>";
}
int small_c_wgrad_blocks(const ConvGeom &g, bool masked)
{
    if (!masked && rgb3_shape(g)) {
        int segs, spw, nb;
        wgrad_rgb3_split(g, &segs, &spw, &nb);
        return nb;
    }
    return wgrad_blocks_direct(g);
}
size_t small_c_wgrad_partial_bytes(const ConvGeom &g)   // filter-gradient partials, then bias-gradient partials; fits either kernel
{
    const int nb = std::max(small_c_wgrad_blocks(g, false), small_c_wgrad_blocks(g, true));
    return (size_t)nb * ((g.K + 63) / 64) * 64 * (32 + 1) * sizeof(float);
}

hipError_t small_c_wgrad_direct(const ConvGeom &g, const bf16_t *x, const bf16_t *dy, const bf16_t *ymask, float *partial, float *dw,
                                float *db, hipStream_t st)
{
    const long long steps = ((long long)g.N * g.Ho * g.Wo + 63) / 64;
    const int nb = small_c_wgrad_blocks(g, ymask != nullptr), ktiles = (g.K + 63) / 64;
    float *dbp = db != nullptr ? partial + (size_t)nb * ktiles * 64 * 32 : nullptr;
    if (ymask == nullptr && rgb3_shape(g)) {
        int segs, spw, nb2;
        wgrad_rgb3_split(g, &segs, &spw, &nb2);
        if (db != nullptr) hipLaunchKernelGGL(k_wgrad_rgb3<true>, dim3((unsigned)nb, (unsigned)ktiles), dim3(256), 0, st, g, x, dy, partial, dbp, segs, spw);
        else hipLaunchKernelGGL(k_wgrad_rgb3<false>, dim3((unsigned)nb, (unsigned)ktiles), dim3(256), 0, st, g, x, dy, partial, dbp, segs, spw);
    } else {
        const int spb = (int)((steps + nb - 1) / nb);
        hipLaunchKernelGGL(k_wgrad_direct, dim3((unsigned)nb, (unsigned)ktiles), dim3(256), 0, st, g, x, dy, ymask, partial, dbp, spb);
    }
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
