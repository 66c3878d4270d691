// Fast-path bf16 implicit-GEMM kernels for the common layer shapes (channel counts that are
// multiples of the reduction step).  Same GEMM view as conv_mfma.hip:
//
//   pass    A rows (i)   B rows (j)            reduction t
//   fwd     c_out        output pixel (n,p,q)  (r,s,c)     c_in  % BK == 0
//   dgrad   c_in         input pixel (n,h,w)   (r,s,k)     c_out % BK == 0, stride 1
//   wgrad   c_out        filter tap (r,s,c)    output pixel
//
// What makes them fast is that almost no vector-ALU work is spent per 16-byte load:
//  * all global reads are raw buffer loads: a 32-bit byte offset per lane, out-of-range
//    offsets return zero, so padding taps and tensor tails need no branches;
//  * with the channel count a multiple of BK, one reduction step lies inside one filter tap,
//    so the tap offset is wave-uniform (scalar registers); a pixel row contributes
//    offset = row_base + tap_offset, valid iff bit `tap` of a per-row mask computed once is
//    set, else the offset is replaced by an out-of-range one;
//  * operands whose reduction index is the slow memory index (dgrad weights, both wgrad
//    operands) are copied to LDS as they lie in memory, [reduction][operand row], and the
//    matrix-core fragments are fetched with the LDS transpose read (ds_read_b64_tr_b16):
//    no register transposes.  In a block of 16 lanes, lane i receives, from the four lanes
//    4u + i/4 (u = 0..3), their element i%4; with lane l pointing at (reduction t0 + l/4,
//    operand rows c0 + 4*(l%4) ..+3), lane i gets operand row c0 + i at reductions t0..t0+3.
//  * backward-filter needs per-pixel offsets that change every step: one wavefront keeps a
//    small LDS table {row_base, tap mask} for the pixels of the next steps.
#include "tile_common.h"
#include <cstdio>
#include <cstdlib>

typedef __attribute__((ext_vector_type(4))) short s16x4;

namespace {

constexpr unsigned OOR = 0xFFFFFFFFu;  // a byte offset beyond any buffer: the load returns zero

DEVFN __amdgpu_buffer_rsrc_t make_rsrc(const void *p, size_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)(unsigned)bytes, 0x00020000);
}
DEVFN u32x4 bload(__amdgpu_buffer_rsrc_t r, unsigned off) { return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0); }

// fragment of 8 reduction elements for operand row (row0 + lane%32) from a K-major tile [row][BK+8]
template <int BK>
DEVFN bf16x8 frag_direct(const bf16_t *tile, int row0, int ks, int lane)
{
    return *reinterpret_cast<const bf16x8 *>(tile + (row0 + (lane & 31)) * (BK + 8) + ks * 16 + (lane >> 5) * 8);
}
// same fragment from a reduction-major tile [BK][T+32] through the LDS transpose read
template <int T>
DEVFN bf16x8 frag_tr(const bf16_t *tile, int row0, int ks, int lane)
{
    constexpr int LS = T + 32;
    const int i = lane & 15;
    const bf16_t *p = tile + (ks * 16 + (lane >> 5) * 8 + (i >> 2)) * LS + row0 + ((lane >> 4) & 1) * 16 + (i & 3) * 4;
    typedef __attribute__((address_space(3))) s16x4 *lds_ptr;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * LS));
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

template <int FA, int FB, int BK, int TA, int TB, bool TRA, bool TRB>
DEVFN void mma_fast(const bf16_t *As, const bf16_t *Bs, int arow, int brow, int lane, f32x16 (&acc)[FA][FB])
{
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
        bf16x8 a[FA], b[FB];
#pragma unroll
        for (int i = 0; i < FA; ++i) a[i] = TRA ? frag_tr<TA>(As, arow + i * 32, ks, lane) : frag_direct<BK>(As, arow + i * 32, ks, lane);
#pragma unroll
        for (int j = 0; j < FB; ++j) b[j] = TRB ? frag_tr<TB>(Bs, brow + j * 32, ks, lane) : frag_direct<BK>(Bs, brow + j * 32, ks, lane);
#pragma unroll
        for (int i = 0; i < FA; ++i)
#pragma unroll
            for (int j = 0; j < FB; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
}

template <int T, int BK, bool TR>
constexpr int tile_elems() { return TR ? BK * (T + 32) : T * (BK + 8); }

// ---------------------------------------------------------------------------------------
// forward and backward-data (stride 1): B rows are pixels with a per-row tap mask
// ---------------------------------------------------------------------------------------

// Valid-tap mask of a pixel row: bit r*S+s is set iff lo_h <= hb + sg*r < H' and the same for w.
DEVFN unsigned tap_mask(int hb, int wb, int sg, int R, int S, int Hlim, int Wlim)
{
    unsigned smask = 0;
    for (int s = 0; s < S; ++s) smask |= ((unsigned)(wb + sg * s) < (unsigned)Wlim) ? 1u << s : 0u;
    unsigned mask = 0;
    for (int r = 0; r < R; ++r) mask |= ((unsigned)(hb + sg * r) < (unsigned)Hlim) ? smask << (r * S) : 0u;
    return mask;
}

// Epilogue of the pixel-major passes through LDS: bias / ReLU / bf16 rounding in registers, the
// tile is staged as [pixel][channel] and leaves with 16-byte stores, 16 lanes per pixel row.
// Needs rowsA % 8 == 0 and no split; the caller has passed the last barrier of the main loop.
template <int FA, int FB, int TA, int TB, int NT>
DEVFN void store_pixel_major_staged(const KArgs &p, const f32x16 (&acc)[FA][FB], bf16_t *stage, const float *bias_lds,
                                    int a0, int b0, int arow, int brow, int tid)
{
    constexpr int LSO = TA + 8;
    const int lane = tid & 63;
#pragma unroll
    for (int i = 0; i < FA; ++i)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const int ch = arow + i * 32 + 8 * gq + 4 * (lane >> 5);
            f32x4 bv = {0.f, 0.f, 0.f, 0.f};
            if (p.flags & KF_BIAS) bv = *reinterpret_cast<const f32x4 *>(bias_lds + ch);
#pragma unroll
            for (int j = 0; j < FB; ++j) {
                float v0 = acc[i][j][4 * gq] + bv.x, v1 = acc[i][j][4 * gq + 1] + bv.y;
                float v2 = acc[i][j][4 * gq + 2] + bv.z, v3 = acc[i][j][4 * gq + 3] + bv.w;
                if (p.flags & KF_RELU) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f); }
                const int pix = brow + j * 32 + (lane & 31);
                *reinterpret_cast<u32x2 *>(stage + pix * LSO + ch) =
                    u32x2{pack_bf16(v0, v1), pack_bf16(v2, v3)};
            }
        }
    constexpr int CPR = TA / 8;
    bf16_t *out = reinterpret_cast<bf16_t *>(p.out);
    if (p.flags & KF_MASK_IN) {
        // fused backward of the input ReLU: the saved-input vectors are requested in groups of eight before
        // they are needed (the first group before the staging barrier), so that their latency overlaps
        constexpr int ITERS = (TB * CPR + NT - 1) / NT, GRP = ITERS < 8 ? ITERS : 8;
        static_assert(ITERS % GRP == 0, "copy-out iterations come in whole groups");
        u32x4 xm[GRP];
        auto fetch = [&](int g0) {
#pragma unroll
            for (int u = 0; u < GRP; ++u) {
                const int id = tid + (g0 + u) * NT, pix = id / CPR, cc = id % CPR;
                const int gp = b0 + pix, gc = a0 + cc * 8;
                xm[u] = (id < TB * CPR && gp < p.rowsB && gc < p.rowsA) ? ldg16(p.x + (size_t)gp * p.rowsA + gc) : u32x4{0, 0, 0, 0};
            }
        };
        fetch(0);
        __syncthreads();
#pragma unroll
        for (int g0 = 0; g0 < ITERS; g0 += GRP) {
            if (g0 > 0) fetch(g0);
#pragma unroll
            for (int u = 0; u < GRP; ++u) {
                const int id = tid + (g0 + u) * NT, pix = id / CPR, cc = id % CPR;
                const int gp = b0 + pix, gc = a0 + cc * 8;
                if (id < TB * CPR && gp < p.rowsB && gc < p.rowsA)
                    *reinterpret_cast<u32x4 *>(out + (size_t)gp * p.rowsA + gc) =
                        apply_mask(*reinterpret_cast<const u32x4 *>(stage + pix * LSO + cc * 8), xm[u]);
            }
        }
        return;
    }
    __syncthreads();
#pragma unroll
    for (int id = tid; id < TB * CPR; id += NT) {
        const int pix = id / CPR, cc = id % CPR;
        const int gp = b0 + pix, gc = a0 + cc * 8;
        if (gp < p.rowsB && gc < p.rowsA)
            *reinterpret_cast<u32x4 *>(out + (size_t)gp * p.rowsA + gc) = *reinterpret_cast<const u32x4 *>(stage + pix * LSO + cc * 8);
    }
}

template <int PASS, int TA, int TB, int BK, int WA, int WB>
__global__ __launch_bounds__(64 * WA * WB) void k_conv_fast(const KArgs p)
{
    static_assert(PASS == PASS_FWD || PASS == PASS_DGRAD, "pixel-row kernel");
    constexpr int NT = 64 * WA * WB, CH = BK / 8;
    constexpr int FA = TA / WA / 32, FB = TB / WB / 32;
    constexpr bool TRA = PASS == PASS_DGRAD;
    constexpr int NA = TA * CH / NT, NB = TB * CH / NT;
    static_assert(NA * NT == TA * CH && NB * NT == TB * CH, "tile must divide evenly over the threads");
    static_assert(TB <= NT, "one thread per pixel row fills the row table");
    constexpr int A_ELEMS = tile_elems<TA, BK, TRA>(), B_ELEMS = tile_elems<TB, BK, false>();
    static_assert(2 * (A_ELEMS + B_ELEMS) >= TB * (TA + 8), "staged epilogue must fit in the tile buffers");
    extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
    bf16_t *As = lds, *Bs = lds + 2 * A_ELEMS;
    unsigned *rowtab = reinterpret_cast<unsigned *>(lds + 2 * (A_ELEMS + B_ELEMS));  // [TB][2] = {row base bytes, tap mask}
    float *bias_lds = reinterpret_cast<float *>(rowtab + 2 * TB);                     // [TA]

    const ConvGeom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tile = logical_block(blockIdx.x, gridDim.x);
    const int a0 = (tile % p.tilesA) * TA, b0 = (tile / p.tilesA) * TB;
    const int split = blockIdx.y;
    const int kbeg = split * p.steps_per_split, kend = min(kbeg + p.steps_per_split, p.steps_total);

    // chan = channels of the pixel tensor (inner extent of the reduction)
    const int chan = PASS == PASS_FWD ? g.C : g.K;
    const int RSC = g.R * g.S * g.C;
    __amdgpu_buffer_rsrc_t rw = make_rsrc(p.w, (size_t)g.K * RSC * 2);
    __amdgpu_buffer_rsrc_t rp = PASS == PASS_FWD ? make_rsrc(p.x, (size_t)g.N * g.H * g.W * g.C * 2)
                                                 : make_rsrc(p.dy, (size_t)g.N * g.Ho * g.Wo * g.K * 2);

    // --- row table: one thread per pixel row of the tile --------------------------------------
    if (tid < TB) {
        const int m = b0 + tid;
        unsigned base, mask = 0;
        if constexpr (PASS == PASS_FWD) {
            const int n = m / (g.Ho * g.Wo), rem = m - n * (g.Ho * g.Wo), pp = rem / g.Wo, qq = rem - pp * g.Wo;
            const int hb = pp * g.sh - g.ph, wb = qq * g.sw - g.pw;
            if (m < p.rowsB) mask = tap_mask(hb, wb, 1, g.R, g.S, g.H, g.W);
            base = (unsigned)(((n * g.H + hb) * g.W + wb) * g.C) * 2u;
        } else {
            const int n = m / (g.H * g.W), rem = m - n * (g.H * g.W), hh = rem / g.W, ww = rem - hh * g.W;
            const int hb = hh + g.ph, wb = ww + g.pw;   // the output pixel of tap (r,s) is (hb - r, wb - s)
            if (m < p.rowsB) mask = tap_mask(hb, wb, -1, g.R, g.S, g.Ho, g.Wo);
            base = (unsigned)(((n * g.Ho + hb) * g.Wo + wb) * g.K) * 2u;
        }
        rowtab[2 * tid] = base;
        rowtab[2 * tid + 1] = mask;
    }
    if (PASS == PASS_FWD && (p.flags & KF_BIAS))
        for (int i = tid; i < TA; i += NT) bias_lds[i] = a0 + i < p.rowsA ? p.bias[a0 + i] : 0.f;

    // --- per-thread constants -------------------------------------------------------------
    // A rows beyond the tensor (tail of the last tile) may load anything the buffer returns:
    // they only feed accumulator rows that the epilogue never stores.
    unsigned voffA[NA], ldsA[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int id = tid + i * NT;
        if constexpr (PASS == PASS_FWD) {
            const int row = id / CH, ch = id % CH;           // weights row (c_out), K-major
            voffA[i] = ((unsigned)(a0 + row) * RSC + ch * 8) * 2u;
            ldsA[i] = row * (BK + 8) + ch * 8;
        } else {
            const int t = id / (TA / 8), cch = id % (TA / 8);  // reduction row k, 8 input channels
            voffA[i] = ((unsigned)t * RSC + a0 + cch * 8) * 2u;
            ldsA[i] = t * (TA + 32) + cch * 8;
        }
    }
    __syncthreads();
    unsigned voffB[NB], maskB[NB], ldsB[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int id = tid + i * NT, row = id / CH, ch = id % CH;
        ldsB[i] = row * (BK + 8) + ch * 8;
        const u32x2 e = *reinterpret_cast<const u32x2 *>(rowtab + 2 * row);
        voffB[i] = e.x + ch * 16;
        maskB[i] = e.y;
    }

    // --- wave-uniform reduction position --------------------------------------------------
    int kk = kbeg * BK;
    int tap = kk / chan, c0 = kk - tap * chan;
    int tr = tap / g.S, ts = tap - tr * g.S;

    u32x4 ra[NA], rb[NB];
    auto load = [&]() {
        unsigned ua, ub;  // uniform byte offsets of this step
        if constexpr (PASS == PASS_FWD) {
            ua = (unsigned)(tap * g.C + c0) * 2u;
            ub = (unsigned)((tr * g.W + ts) * g.C + c0) * 2u;
        } else {
            ua = ((unsigned)c0 * RSC + (unsigned)tap * g.C) * 2u;
            ub = (unsigned)(c0 - (tr * g.Wo + ts) * g.K) * 2u;
        }
        const unsigned bit = 1u << tap;
#pragma unroll
        for (int i = 0; i < NA; ++i) ra[i] = bload(rw, voffA[i] + ua);
#pragma unroll
        for (int i = 0; i < NB; ++i) rb[i] = bload(rp, (maskB[i] & bit) ? voffB[i] + ub : OOR);
        c0 += BK;
        if (c0 >= chan) { c0 = 0; ++tap; if (++ts == g.S) { ts = 0; ++tr; } }
    };
    auto store = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<u32x4 *>(As + buf * A_ELEMS + ldsA[i]) = ra[i];
#pragma unroll
        for (int i = 0; i < NB; ++i) *reinterpret_cast<u32x4 *>(Bs + buf * B_ELEMS + ldsB[i]) = rb[i];
    };

    f32x16 acc[FA][FB];
#pragma unroll
    for (int i = 0; i < FA; ++i)
#pragma unroll
        for (int j = 0; j < FB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    const int arow = (wave % WA) * FA * 32, brow = (wave / WA) * FB * 32;

    if (kbeg < kend) {
        load();
        store(0);
        __syncthreads();
        for (int step = kbeg; step < kend; ++step) {
            const int buf = (step - kbeg) & 1;
            const bool more = step + 1 < kend;
            if (more) load();
            mma_fast<FA, FB, BK, TA, TB, TRA, false>(As + buf * A_ELEMS, Bs + buf * B_ELEMS, arow, brow, lane, acc);
            if (more) store(buf ^ 1);
            __syncthreads();
        }
    }
    if (p.splits == 1 && !(p.flags & KF_OUT_F32) && (p.rowsA & 7) == 0)
        store_pixel_major_staged<FA, FB, TA, TB, NT>(p, acc, lds, bias_lds, a0, b0, arow, brow, tid);
    else
        store_pixel_major<FA, FB>(p, acc, a0 + arow, b0 + brow, lane, split);
}

// ---------------------------------------------------------------------------------------
// backward-filter: both operands reduction-major in LDS, per-step pixel table for x
// ---------------------------------------------------------------------------------------
template <int TA, int TB, int BK, int WA, int WB>
__global__ __launch_bounds__(64 * WA * WB) void k_wgrad_fast(const KArgs p)
{
    constexpr int NT = 64 * WA * WB;
    constexpr int FA = TA / WA / 32, FB = TB / WB / 32;
    constexpr int NA = BK * (TA / 8) / NT, NB = BK * (TB / 8) / NT;
    static_assert(NA * NT == BK * (TA / 8) && NB * NT == BK * (TB / 8), "tile must divide evenly over the threads");
    static_assert(BK <= 64, "one wavefront fills the pixel table");
    constexpr int A_ELEMS = tile_elems<TA, BK, true>(), B_ELEMS = tile_elems<TB, BK, true>();
    extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
    bf16_t *As = lds, *Bs = lds + 2 * A_ELEMS;
    int *tab = reinterpret_cast<int *>(lds + 2 * A_ELEMS + 2 * B_ELEMS);  // [2][BK][2] = {row_base bytes, tap mask}

    const ConvGeom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tile = logical_block(blockIdx.x, gridDim.x);
    const int a0 = (tile % p.tilesA) * TA, b0 = (tile / p.tilesA) * TB;
    const int split = blockIdx.y;
    const int kbeg = split * p.steps_per_split, kend = min(kbeg + p.steps_per_split, p.steps_total);
    const int M = p.red;

    __amdgpu_buffer_rsrc_t rdy = make_rsrc(p.dy, (size_t)M * g.K * 2);
    __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, (size_t)g.N * g.H * g.W * g.C * 2);

    unsigned voffA[NA], ldsA[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int id = tid + i * NT, t = id / (TA / 8), cch = id % (TA / 8);
        voffA[i] = a0 + cch * 8 < g.K ? ((unsigned)t * g.K + a0 + cch * 8) * 2u : OOR;
        ldsA[i] = t * (TA + 32) + cch * 8;
    }
    unsigned coffB[NB], bitB[NB], ldsB[NB];
    int tB[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int id = tid + i * NT, t = id / (TB / 8), cch = id % (TB / 8);
        const int col = b0 + cch * 8;
        const int tapi = col / g.C, c = col - tapi * g.C, r = tapi / g.S, s = tapi - r * g.S;
        coffB[i] = (unsigned)((r * g.W + s) * g.C + c) * 2u;
        bitB[i] = col < p.rowsB ? 1u << tapi : 0u;
        ldsB[i] = t * (TB + 32) + cch * 8;
        tB[i] = t;
    }

    // pixel table: thread t < BK owns pixel (step*BK + t); (n,pp,qq) advance by BK per step
    int pn = 0, pp = 0, pq = 0;
    if (tid < BK) {
        const int m = kbeg * BK + tid;
        pn = m / (g.Ho * g.Wo);
        const int rem = m - pn * (g.Ho * g.Wo);
        pp = rem / g.Wo; pq = rem - pp * g.Wo;
    }
    auto fill_table = [&](int slot, int step) {
        if (tid < BK) {
            const int m = step * BK + tid;
            const int hb = pp * g.sh - g.ph, wb = pq * g.sw - g.pw;
            unsigned mask = 0;
            if (m < M)
                for (int r = 0; r < g.R; ++r)
                    for (int s = 0; s < g.S; ++s)
                        if ((unsigned)(hb + r) < (unsigned)g.H && (unsigned)(wb + s) < (unsigned)g.W) mask |= 1u << (r * g.S + s);
            tab[(slot * BK + tid) * 2] = (int)((unsigned)(((pn * g.H + hb) * g.W + wb) * g.C) * 2u);
            tab[(slot * BK + tid) * 2 + 1] = (int)mask;
            pq += BK;
            while (pq >= g.Wo) { pq -= g.Wo; if (++pp == g.Ho) { pp = 0; ++pn; } }
        }
    };

    u32x4 ra[NA], rb[NB];
    auto load = [&](int step) {
        const unsigned ua = (unsigned)step * BK * g.K * 2u;
        const int slot = (step - kbeg) & 1;
#pragma unroll
        for (int i = 0; i < NA; ++i) ra[i] = bload(rdy, voffA[i] == OOR ? OOR : voffA[i] + ua);
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const u32x2 e = *reinterpret_cast<const u32x2 *>(tab + (slot * BK + tB[i]) * 2);
            rb[i] = bload(rx, (e.y & bitB[i]) ? e.x + coffB[i] : OOR);
        }
    };
    auto store = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<u32x4 *>(As + buf * A_ELEMS + ldsA[i]) = ra[i];
#pragma unroll
        for (int i = 0; i < NB; ++i) *reinterpret_cast<u32x4 *>(Bs + buf * B_ELEMS + ldsB[i]) = rb[i];
    };

    f32x16 acc[FA][FB];
#pragma unroll
    for (int i = 0; i < FA; ++i)
#pragma unroll
        for (int j = 0; j < FB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    const int arow = (wave % WA) * FA * 32, brow = (wave / WA) * FB * 32;

    if (kbeg < kend) {
        fill_table(0, kbeg);
        fill_table(1, kbeg + 1);
        __syncthreads();
        load(kbeg);
        store(0);
        __syncthreads();
        for (int step = kbeg; step < kend; ++step) {
            const int buf = (step - kbeg) & 1;
            const bool more = step + 1 < kend;
            if (more) load(step + 1);             // reads table slot buf^1
            mma_fast<FA, FB, BK, TA, TB, true, true>(As + buf * A_ELEMS, Bs + buf * B_ELEMS, arow, brow, lane, acc);
            if (more) store(buf ^ 1);
            fill_table(buf, step + 2);             // slot buf was last read before the previous barrier
            __syncthreads();
        }
    }
    store_row_major<FA, FB>(p, acc, a0 + arow, b0 + brow, lane, split);
}

// ---------------------------------------------------------------------------------------
// variants and dispatch
// ---------------------------------------------------------------------------------------
struct FastVariant { int TA, TB, WA, WB; };
const FastVariant kFast[] = {{128, 128, 2, 2}, {64, 128, 2, 2}, {128, 64, 2, 2}, {64, 64, 2, 2}};
constexpr int kNumFast = 4;

typedef void (*KernelFn)(const KArgs);

template <int PASS, int BK>
KernelFn pick_pix(int v)
{
    switch (v) {
    case 0: return k_conv_fast<PASS, 128, 128, BK, 2, 2>;
    case 1: return k_conv_fast<PASS, 64, 128, BK, 2, 2>;
    case 2: return k_conv_fast<PASS, 128, 64, BK, 2, 2>;
    default: return k_conv_fast<PASS, 64, 64, BK, 2, 2>;
    }
}
template <int BK>
KernelFn pick_wg(int v)
{
    switch (v) {
    case 0: return k_wgrad_fast<128, 128, BK, 2, 2>;
    case 1: return k_wgrad_fast<64, 128, BK, 2, 2>;
    case 2: return k_wgrad_fast<128, 64, BK, 2, 2>;
    default: return k_wgrad_fast<64, 64, BK, 2, 2>;
    }
}
KernelFn pick_fast(int pass, int v, int bk)
{
    if (pass == PASS_FWD) return bk == 64 ? pick_pix<PASS_FWD, 64>(v) : pick_pix<PASS_FWD, 32>(v);
    if (pass == PASS_DGRAD) return bk == 64 ? pick_pix<PASS_DGRAD, 64>(v) : pick_pix<PASS_DGRAD, 32>(v);
    return bk == 64 ? pick_wg<64>(v) : pick_wg<32>(v);
}
size_t fast_lds_bytes(int pass, int TA, int TB, int BK)
{
    size_t a, b, extra = 0;
    if (pass == PASS_FWD) { a = (size_t)TA * (BK + 8); b = (size_t)TB * (BK + 8); extra = (size_t)TB * 8 + (size_t)TA * 4; }
    else if (pass == PASS_DGRAD) { a = (size_t)BK * (TA + 32); b = (size_t)TB * (BK + 8); extra = (size_t)TB * 8 + (size_t)TA * 4; }
    else { a = (size_t)BK * (TA + 32); b = (size_t)BK * (TB + 32); extra = (size_t)2 * BK * 2 * sizeof(int); }
    return 2 * (a + b) * sizeof(bf16_t) + extra;
}

void extents(const ConvGeom &g, int pass, int *rowsA, int *rowsB, int *red)
{
    if (pass == PASS_FWD) { *rowsA = g.K; *rowsB = g.N * g.Ho * g.Wo; *red = g.R * g.S * g.C; }
    else if (pass == PASS_DGRAD) { *rowsA = g.C; *rowsB = g.N * g.H * g.W; *red = g.R * g.S * g.K; }
    else { *rowsA = g.K; *rowsB = g.R * g.S * g.C; *red = g.N * g.Ho * g.Wo; }
}

}  // namespace

hipError_t fast_init()
{
    for (int pass = 0; pass < 3; ++pass)
        for (int v = 0; v < kNumFast; ++v)
            for (int bk = 32; bk <= 64; bk += 32) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pick_fast(pass, v, bk)),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize,
                                                   (int)fast_lds_bytes(pass, kFast[v].TA, kFast[v].TB, bk));
                if (e != hipSuccess) return e;
            }
    return hipSuccess;
}

bool fast_plan(const ConvGeom &g, int pass, int force_variant, int force_splits, GemmPlan *pl)
{
    if (g.R * g.S > 32) return false;
    int bk;
    if (pass == PASS_FWD) {
        if (g.C % 32) return false;
        bk = g.C % 64 == 0 ? 64 : 32;
    } else if (pass == PASS_DGRAD) {
        if (g.K % 32 || g.C % 8 || g.sh != 1 || g.sw != 1) return false;
        bk = g.K % 64 == 0 ? 64 : 32;
    } else {
        if (g.K % 8 || g.C % 8) return false;
        bk = 32;
    }
    int rowsA, rowsB, red;
    extents(g, pass, &rowsA, &rowsB, &red);
    int v;
    if (force_variant >= 100 && force_variant < 100 + kNumFast) v = force_variant - 100;
    else {
        const bool narrowA = rowsA <= 64, narrowB = rowsB <= 64;
        long long big = (long long)((rowsA + 127) / 128) * ((rowsB + 127) / 128);
        if (narrowA && narrowB) v = 3;
        else if (narrowA) v = 1;
        else if (narrowB) v = 2;
        else if (pass == PASS_WGRAD) v = 0;
        else v = big >= 128 ? 0 : 3;
    }
    const FastVariant &fv = kFast[v];
    pl->fast = true; pl->dma = false; pl->variant = v; pl->TA = fv.TA; pl->TB = fv.TB; pl->BK = bk;
    pl->vecA = pl->vecB = true;
    pl->tilesA = (rowsA + fv.TA - 1) / fv.TA;
    pl->tilesB = (rowsB + fv.TB - 1) / fv.TB;
    pl->steps_total = (red + bk - 1) / bk;
    long long tiles = (long long)pl->tilesA * pl->tilesB;
    int splits;
    if (force_splits > 0) splits = force_splits;
    else {
        const long long target = 512;
        splits = tiles >= target ? 1 : (int)((target + tiles - 1) / tiles);
        const int min_steps = 8;
        int max_splits = pl->steps_total / min_steps;
        if (max_splits < 1) max_splits = 1;
        if (splits > max_splits) splits = max_splits;
    }
    if (splits > pl->steps_total) splits = pl->steps_total;
    if (splits < 1) splits = 1;
    pl->steps_per_split = (pl->steps_total + splits - 1) / splits;
    pl->splits = (pl->steps_total + pl->steps_per_split - 1) / pl->steps_per_split;
    return true;
}

void fast_kernel_name(int pass, const GemmPlan &pl, char *name, size_t name_bytes)
{
    const FastVariant &fv = kFast[pl.variant];
    if (pass == PASS_WGRAD) snprintf(name, name_bytes, "k_wgrad_fast<%d, %d, %d, %d, %d>", fv.TA, fv.TB, pl.BK, fv.WA, fv.WB);
    else snprintf(name, name_bytes, "k_conv_fast<%d, %d, %d, %d, %d, %d>", pass, fv.TA, fv.TB, pl.BK, fv.WA, fv.WB);
}

hipError_t fast_launch(const ConvArgs &a, hipStream_t st)
{
    KArgs p;
    p.g = a.g;
    extents(a.g, a.pass, &p.rowsA, &p.rowsB, &p.red);
    p.tilesA = a.plan.tilesA; p.tilesB = a.plan.tilesB;
    p.steps_total = a.plan.steps_total; p.steps_per_split = a.plan.steps_per_split; p.splits = a.plan.splits;
    p.flags = a.flags;
    p.x = a.x; p.w = a.w; p.dy = a.dy; p.ymask = nullptr; p.bias = a.bias; p.out = a.out; p.partial = a.partial;
    const FastVariant &fv = kFast[a.plan.variant];
    dim3 grid((unsigned)(p.tilesA * p.tilesB), (unsigned)p.splits, 1), block(64 * fv.WA * fv.WB, 1, 1);
    hipLaunchKernelGGL(pick_fast(a.pass, a.plan.variant, a.plan.BK), grid, block,
                       fast_lds_bytes(a.pass, fv.TA, fv.TB, a.plan.BK), st, p);
    dp_trace_main_kernel_done(st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.splits <= 1) return e;
    return launch_split_reduce(a, p.rowsA, p.rowsB, st);
}
