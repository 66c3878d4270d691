// Forward / backward-data kernels for stride-1 layers whose reduction has exactly 64 channels per
// tap (VGG conv1_2, conv2_1): the tiled kernels re-fetch every input pixel once per filter tap, and
// with only R*S reduction steps per tile that traffic through the per-CU global->LDS path is what
// bounds them.  Here a block owns a TH x TW patch of output pixels of one image (TH*TW = 256) and
// copies the input patch with its halo ((TH+R-1) x (TW+S-1) pixels x 64 channels, zero outside the
// image) into LDS ONCE; the R*S taps then read their pixel rows from that patch at shifted positions.
// Only the weight tile of each tap still streams through the NS-stage pipeline.
//
// Patch layout: pixel pp = pr*(TW+S-1) + pc occupies 128 bytes; its 16-byte channel chunk c sits at
// chunk position c ^ ((pp >> 1) & 7) (two 128-byte rows span the 64 banks), which makes the fragment reads of 32 consecutive pixels conflict-free.
// A direct-to-LDS instruction fills 8 consecutive patch pixels.
#include "dma_common.h"
#include <utility>
#include <cstdio>

namespace {

constexpr int HALO_TB = 256;        // output pixels per tile
constexpr int HALO_PP = 352;        // patch pixels the LDS slot holds (44 KiB): 10x34 and 18x18 fit

// PASS_FWD : A = weights [c_out][tap][64 c_in] (rows K-major in LDS), patch from x.
// PASS_DGRAD: A = weights [64 c_out][tap][c_in] kept reduction-major in LDS and read with the LDS
//             transpose read, patch from dy; tap (r, s) of the filter meets patch offset (R-1-r, S-1-s).
template <int PASS, int TA, int WA, int WB, int NS>
__global__ __launch_bounds__(64 * WA * WB) void k_halo(const KArgs p, int tws, int tiles_x, int tiles_y)
{
    constexpr int NT = 64 * WA * WB, NW = WA * WB, TB = HALO_TB;
    constexpr int KS = 4;                                     // 16-wide slices per 64-channel step
    constexpr int FA = TA / WA / 32, FB = TB / WB / 32;
    constexpr int A_BYTES = TA * 128;                         // one tap's weight tile (either orientation)
    constexpr int IA = A_BYTES / 1024 / NW;                   // weight copies per wave and step
    constexpr int IP = (HALO_PP * 128 / 1024 + NW - 1) / NW;  // patch copies per wave
    constexpr int PATCH_BYTES = IP * NW * 1024;
    static_assert(IA * NW * 1024 == A_BYTES, "weight tile must divide over the waves");
    constexpr int STAGES_END = PATCH_BYTES + NS * A_BYTES, EPI = TB * (TA + 8) * 2;
    constexpr int TILE_BYTES = STAGES_END > EPI ? STAGES_END : EPI;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    float *bias_lds = reinterpret_cast<float *>(smem + TILE_BYTES);   // [TA]

    const ConvGeom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int R = g.R, S = g.S, TW = 1 << tws, TH = TB >> tws, PW = TW + S - 1, PP = (TH + R - 1) * PW;
    const int tile = logical_block(blockIdx.x, gridDim.x);
    const int a0 = (tile % p.tilesA) * TA, bt = tile / p.tilesA;
    const int n = bt / (tiles_x * tiles_y), trem = bt - n * (tiles_x * tiles_y), ty = trem / tiles_x, tx = trem - ty * tiles_x;
    const int p0 = ty * TH, q0 = tx * TW;
    // image the patch is cut from, its extent, and the patch origin
    const int IH = PASS == PASS_FWD ? g.H : g.Ho, IW = PASS == PASS_FWD ? g.W : g.Wo;
    const int h0 = PASS == PASS_FWD ? p0 - g.ph : p0 + g.ph - (R - 1), w0 = PASS == PASS_FWD ? q0 - g.pw : q0 + g.pw - (S - 1);
    const int OH = PASS == PASS_FWD ? g.Ho : g.H, OW = PASS == PASS_FWD ? g.Wo : g.W;   // output image
    const int RSC = R * S * g.C;
    __amdgpu_buffer_rsrc_t rw = make_rsrc(p.w, (size_t)g.K * RSC * 2);
    __amdgpu_buffer_rsrc_t rsrc_in = PASS == PASS_FWD ? make_rsrc(p.x, (size_t)g.N * g.H * g.W * g.C * 2)
                                                      : make_rsrc(p.dy, (size_t)g.N * g.Ho * g.Wo * g.K * 2);
    const unsigned smem_base = lds_offset(smem);

    if ((p.flags & KF_BIAS) && PASS == PASS_FWD)
        for (int i = tid; i < TA; i += NT) bias_lds[i] = a0 + i < p.rowsA ? p.bias[a0 + i] : 0.f;

    // ---- patch: all copies issued up front -------------------------------------------------
#pragma unroll
    for (int q = 0; q < IP; ++q) {
        const int id = (wave * IP + q) * 64 + lane, pp = id >> 3, c = (id & 7) ^ ((pp >> 1) & 7);
        const int pr = pp / PW, pc = pp - pr * PW, ih = h0 + pr, iw = w0 + pc;
        const bool ok = pp < PP && (unsigned)ih < (unsigned)IH && (unsigned)iw < (unsigned)IW;
        const unsigned voff = ok ? (unsigned)(((n * IH + ih) * IW + iw) * 64 + c * 8) * 2u : OOR;
        dma16(rsrc_in, smem_base + (wave * IP + q) * 1024, voff);
    }

    // ---- weight tile of one tap ----------------------------------------------------------------
    unsigned voffA[IA];
#pragma unroll
    for (int q = 0; q < IA; ++q) {
        if (PASS == PASS_FWD) {   // row = c_out, 8 rows per copy, chunk swizzle by row pair
            const int row = (wave * IA + q) * 8 + lane / 8;
            const int c = (lane % 8) ^ ((row / 2) % 8);
            voffA[q] = ((unsigned)(a0 + row) * RSC + c * 8) * 2u;
        } else {                  // row = c_out (reduction), TA c_in per row, 512/TA rows per copy, segment swizzle
            const int t = (wave * IA + q) * (512 / TA) + lane / (TA / 8);
            const int c = (lane % (TA / 8)) ^ (seg_swz<TA>(t) << 2);
            voffA[q] = ((unsigned)t * RSC + a0 + c * 8) * 2u;
        }
    }
    const unsigned ldsA_w = smem_base + PATCH_BYTES + wave * IA * 1024;
    auto issueA = [&](int stage, int step) {   // filter tap of reduction step `step`
        const int tap = PASS == PASS_FWD ? step : (R * S - 1 - step);
        const unsigned ua = (unsigned)tap * g.C * 2u;
#pragma unroll
        for (int q = 0; q < IA; ++q) dma16(rw, ldsA_w + stage * A_BYTES + q * 1024, voffA[q] + ua);
    };

    f32x16 acc[FA][FB];
#pragma unroll
    for (int i = 0; i < FA; ++i)
#pragma unroll
        for (int j = 0; j < FB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    const int arow = (wave % WA) * FA * 32, brow = (wave / WA) * FB * 32;

    // fragment addresses of the weight tile
    unsigned fa[KS][PASS == PASS_FWD ? 1 : FA];
    if (PASS == PASS_FWD) {
        const int rA = arow + (lane & 31);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            fa[ks][0] = smem_base + PATCH_BYTES + rA * 128 + (((2 * ks + (lane >> 5)) ^ ((rA / 2) % 8)) << 4);
    } else {
        const int i16 = lane & 15, tl = (lane >> 5) * 8 + (i16 >> 2), cl = ((lane >> 4) & 1) * 16 + (i16 & 3) * 4;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int t = ks * 16 + tl;
#pragma unroll
            for (int i = 0; i < (PASS == PASS_FWD ? 1 : FA); ++i) {
                const int col = arow + i * 32 + cl;
                fa[ks][i] = smem_base + PATCH_BYTES + t * (TA * 2) + ((((col >> 5) ^ seg_swz<TA>(t)) << 6) | ((col & 31) << 1));
            }
        }
    }
    // patch pixel of this lane's row in each of its B fragments, at patch offset (0, 0)
    int pp0[FB];
#pragma unroll
    for (int j = 0; j < FB; ++j) {
        const int jj = brow + j * 32 + (lane & 31);
        pp0[j] = (jj >> tws) * PW + (jj & (TW - 1));
    }
    const unsigned hsel = lane >> 5;

    const int nsteps = R * S;
    constexpr int LPS = IA;
#pragma unroll
    for (int s = 0; s < NS; ++s)
        if (s < nsteps) issueA(s, s);

    u32x4 fr_a[2][FA], fr_b[2][FB];
    u32x2 tr_lo[2][FA], tr_hi[2][FA];
    unsigned brow_addr[FB], bsw[FB];
    auto set_tap = [&](int step) {   // patch rows of reduction step `step` (patch offset r*PW + s)
        const int r = step / S, s = step - r * S;
        const int off = r * PW + s;
#pragma unroll
        for (int j = 0; j < FB; ++j) {
            const int pp = pp0[j] + off;
            brow_addr[j] = smem_base + pp * 128;
            bsw[j] = (pp >> 1) & 7;
        }
    };
    auto read_slice = [&](int ks, int buf, unsigned sb) {
        if constexpr (PASS == PASS_FWD) {
            if constexpr (FA >= 1) fr_a[buf][0] = lds_read16<0>(fa[ks][0] + sb);
            if constexpr (FA >= 2) fr_a[buf][1] = lds_read16<32 * 128>(fa[ks][0] + sb);
            if constexpr (FA >= 3) fr_a[buf][2] = lds_read16<64 * 128>(fa[ks][0] + sb);
            if constexpr (FA >= 4) fr_a[buf][3] = lds_read16<96 * 128>(fa[ks][0] + sb);
        } else {
#pragma unroll
            for (int i = 0; i < FA; ++i) {
                tr_lo[buf][i] = lds_read_tr<0>(fa[ks][i] + sb);
                tr_hi[buf][i] = lds_read_tr<4 * TA * 2>(fa[ks][i] + sb);
            }
        }
#pragma unroll
        for (int j = 0; j < FB; ++j) fr_b[buf][j] = lds_read16<0>(brow_addr[j] + (((2 * ks + hsel) ^ bsw[j]) << 4));
    };
    constexpr int RPS_ = (PASS == PASS_FWD ? FA : 2 * FA) + FB;   // LDS reads per slice
    static_assert(RPS_ < 16, "lgkmcnt is a 4-bit counter");
    auto wait_slice = [&](int buf, bool newer_in_flight) {
        if (newer_in_flight) asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(RPS_));
        else asm volatile("s_waitcnt lgkmcnt(0)");
#pragma unroll
        for (int i = 0; i < FA; ++i) {
            if constexpr (PASS == PASS_FWD) asm volatile("" : "+v"(fr_a[buf][i]));
            else { asm volatile("" : "+v"(tr_lo[buf][i])); asm volatile("" : "+v"(tr_hi[buf][i])); }
        }
#pragma unroll
        for (int j = 0; j < FB; ++j) asm volatile("" : "+v"(fr_b[buf][j]));
    };

    // patch and the first weight tile have landed; later weight tiles may be in flight
    {
        const int younger = min(NS - 1, nsteps - 1);
        if (NS >= 2 && younger == NS - 1) wait_vmcnt<(NS - 1) * LPS>();
        else if (NS >= 3 && younger == NS - 2) wait_vmcnt<(NS >= 3 ? NS - 2 : 0) * LPS>();
        else if (NS >= 4 && younger == NS - 3) wait_vmcnt<(NS >= 4 ? NS - 3 : 0) * LPS>();
        else wait_vmcnt<0>();
    }
    __syncthreads();   // also publishes bias_lds
    set_tap(0);
    read_slice(0, 0, 0);
    for (int i = 0; i < nsteps; ++i) {
        const unsigned sb = (i % NS) * A_BYTES;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int cur = ks & 1;
            if (ks < KS - 1) {
                read_slice(ks + 1 < KS ? ks + 1 : 0, cur ^ 1, sb);
                wait_slice(cur, true);
            } else {
                wait_slice(cur, false);   // this wave has read all it needs of the weight stage
                if (i + 1 < nsteps) {
                    const int younger = min(i + NS - 1, nsteps - 1) - (i + 1);
                    if (NS >= 3 && younger == NS - 2) wait_vmcnt<(NS - 2) * LPS>();
                    else if (NS >= 4 && younger == NS - 3) wait_vmcnt<(NS >= 4 ? NS - 3 : 0) * LPS>();
                    else wait_vmcnt<0>();
                    __builtin_amdgcn_s_barrier();
                    if (i + NS < nsteps) issueA(i % NS, i + NS);
                    set_tap(i + 1);
                    read_slice(0, 0, ((i + 1) % NS) * A_BYTES);
                }
            }
#pragma unroll
            for (int ii = 0; ii < FA; ++ii)
#pragma unroll
                for (int jj = 0; jj < FB; ++jj) {
                    u32x4 av;
                    if constexpr (PASS == PASS_FWD) av = fr_a[cur][ii];
                    else av = u32x4{tr_lo[cur][ii].x, tr_lo[cur][ii].y, tr_hi[cur][ii].x, tr_hi[cur][ii].y};
                    acc[ii][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av),
                                                                         __builtin_bit_cast(bf16x8, fr_b[cur][jj]), acc[ii][jj], 0, 0, 0);
                }
        }
    }
    __syncthreads();   // every wave is done reading patch and stages before they are reused for staging

    // ---- epilogue: bias / ReLU / bf16 through LDS, 16-byte rows to the NHWC output ------------
    constexpr int LSO = TA + 8;
    bf16_t *stage = reinterpret_cast<bf16_t *>(smem);
#pragma unroll
    for (int i = 0; i < FA; ++i)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const int ch = arow + i * 32 + 8 * gq + 4 * (lane >> 5);
            f32x4 bv = {0.f, 0.f, 0.f, 0.f};
            if ((p.flags & KF_BIAS) && PASS == PASS_FWD) bv = *reinterpret_cast<const f32x4 *>(bias_lds + ch);
#pragma unroll
            for (int j = 0; j < FB; ++j) {
                float v0 = acc[i][j][4 * gq] + bv.x, v1 = acc[i][j][4 * gq + 1] + bv.y;
                float v2 = acc[i][j][4 * gq + 2] + bv.z, v3 = acc[i][j][4 * gq + 3] + bv.w;
                if ((p.flags & KF_RELU) && PASS == PASS_FWD) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f); }
                const int pix = brow + j * 32 + (lane & 31);
                *reinterpret_cast<u32x2 *>(stage + pix * LSO + ch) = u32x2{pack_bf16(v0, v1), pack_bf16(v2, v3)};
            }
        }
    constexpr int CPR = TA / 8;
    bf16_t *out = reinterpret_cast<bf16_t *>(p.out);
    if (PASS == PASS_DGRAD && (p.flags & KF_MASK_IN)) {
        // fused backward of the input ReLU: all saved-input vectors of this thread are requested before the
        // staging barrier, so that their latency overlaps
        constexpr int ITERS = TB * CPR / NT;
        static_assert(TB * CPR % NT == 0 && ITERS <= 16, "copy-out iterations");
        u32x4 xm[ITERS];
#pragma unroll
        for (int u = 0; u < ITERS; ++u) {
            const int id = tid + u * NT, pix = id / CPR, cc = id % CPR;
            const int pr = p0 + (pix >> tws), qc = q0 + (pix & (TW - 1)), gc = a0 + cc * 8;
            xm[u] = (pr < OH && qc < OW && gc < p.rowsA) ? ldg16(p.x + ((size_t)(n * OH + pr) * OW + qc) * p.rowsA + gc) : u32x4{0, 0, 0, 0};
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < ITERS; ++u) {
            const int id = tid + u * NT, pix = id / CPR, cc = id % CPR;
            const int pr = p0 + (pix >> tws), qc = q0 + (pix & (TW - 1)), gc = a0 + cc * 8;
            if (pr < OH && qc < OW && gc < p.rowsA)
                *reinterpret_cast<u32x4 *>(out + ((size_t)(n * OH + pr) * OW + qc) * p.rowsA + gc) =
                    apply_mask(*reinterpret_cast<const u32x4 *>(stage + pix * LSO + cc * 8), xm[u]);
        }
        return;
    }
    __syncthreads();
#pragma unroll
    for (int id = tid; id < TB * CPR; id += NT) {
        const int pix = id / CPR, cc = id % CPR;
        const int pr = p0 + (pix >> tws), qc = q0 + (pix & (TW - 1)), gc = a0 + cc * 8;
        if (pr < OH && qc < OW && gc < p.rowsA)
            *reinterpret_cast<u32x4 *>(out + ((size_t)(n * OH + pr) * OW + qc) * p.rowsA + gc) =
                *reinterpret_cast<const u32x4 *>(stage + pix * LSO + cc * 8);
    }
}

// Tiles of a persistent block.  Consecutive block ids go round-robin to the 8 XCDs, each with an L2 of its own: XCD x (blocks x,
// x + 8, ...) walks one contiguous eighth of the tile list, its blocks side by side, so that tiles that share halo pixels (left /
// right neighbours, and the row of tiles above / below) run on one XCD at about the same time and the second reader of a halo pixel
// finds it in that L2.  (Dealing the tiles out block by block over the whole chip, every halo pixel was fetched from memory again: L2
// hit rate 0.09 on conv1_2, and the copies of a CU are bound by its ~64 outstanding misses.)
struct TileWalk { int first, end, stride; };
DEVFN TileWalk tile_walk(int tiles)
{
    const int nb = gridDim.x;
    if ((nb & 7) != 0) return {(int)blockIdx.x, tiles, nb};
    const int x = blockIdx.x & 7;
    return {(int)((long long)tiles * x / 8) + (int)(blockIdx.x >> 3), (int)((long long)tiles * (x + 1) / 8), nb >> 3};
}

// ---------------------------------------------------------------------------------------
// Backward-filter with the input patch in LDS (stride 1, 64 input channels, up to 16 taps).
// The tiled kernel copies, for every 64 pixels of reduction, the x rows of each tap again; here a
// block copies the x patch of a 256-pixel tile once, next to the tile's 256 x 64 slice of dy, and
// wave t accumulates tap t: dW[k][t][c] += sum over the tile's pixels of dy[pixel][k] * x[pixel + tap t][c]
// (64 c_out x 64 c_in per wave = 4 matrix tiles).  Both operands are pixel-major in LDS (rows of 128
// bytes, 64-byte segment swizzle by (row/2)&1) and read with the LDS transpose read.  Blocks are
// persistent: they walk tiles blockIdx.x, +gridDim.x, ... with the next tile's copies in flight
// (two LDS buffers), keep their sums in registers, and write ONE fp32 partial per block, which the
// split-reduce kernel adds in block order.  grid = (blocks, 64-row tiles of c_out).
// ---------------------------------------------------------------------------------------
constexpr int WH_BUF = HALO_PP * 128 + HALO_TB * 128;   // patch + dy slice of one tile: 76 KiB

__global__ __launch_bounds__(1024) void k_wgrad_halo(const KArgs p, int tws, int tiles_x, int tiles_y, int tiles)
{
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const ConvGeom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;   // wave = tap
    const int R = g.R, S = g.S, TW = 1 << tws, TH = HALO_TB >> tws, PW = TW + S - 1, PP = (TH + R - 1) * PW;
    const int a0 = blockIdx.y * 64;
    const unsigned smem_base = lds_offset(smem);
    __amdgpu_buffer_rsrc_t rdy = make_rsrc(p.dy, (size_t)g.N * g.Ho * g.Wo * g.K * 2);
    __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, (size_t)g.N * g.H * g.W * g.C * 2);
    constexpr int NPI = HALO_PP / 8, NDI = HALO_TB / 8;   // copies (8 rows each) of the patch / of the dy slice

    auto issue_tile = [&](int tile, int buf) {
        const int n = tile / (tiles_x * tiles_y), trem = tile - n * (tiles_x * tiles_y), ty = trem / tiles_x, tx = trem - ty * tiles_x;
        const int p0 = ty * TH, q0 = tx * TW;
        const unsigned base = smem_base + buf * WH_BUF;
        for (int ii = wave; ii < NPI + NDI; ii += nwaves) {
            unsigned voff = OOR;
            if (ii < NPI) {   // patch rows 8*ii .. +7
                const int pp = ii * 8 + (lane >> 3), c = (lane & 7) ^ (seg_swz<64>(pp) << 2);
                const int pr = pp / PW, pc = pp - pr * PW, ih = p0 - g.ph + pr, iw = q0 - g.pw + pc;
                if (pp < PP && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W)
                    voff = (unsigned)(((n * g.H + ih) * g.W + iw) * 64 + c * 8) * 2u;
                dma16(rx, base + ii * 1024, voff);
            } else {          // dy rows (tile pixels) 8*d .. +7, c_out a0 .. a0+63
                const int d = ii - NPI, j = d * 8 + (lane >> 3), c = (lane & 7) ^ (seg_swz<64>(j) << 2);
                const int pr = p0 + (j >> tws), qc = q0 + (j & (TW - 1));
                if (pr < g.Ho && qc < g.Wo && a0 + c * 8 + 8 <= g.K)
                    voff = (unsigned)(((n * g.Ho + pr) * g.Wo + qc) * g.K + a0 + c * 8) * 2u;
                dma16(rdy, base + HALO_PP * 128 + d * 1024, voff);
            }
        }
    };

    f32x16 acc[2][2];   // [c_out half][c_in half]
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // transpose-read lane roles: reduction row tl (+4 for the second read), operand columns cl .. cl+3
    const int i16 = lane & 15, tl = (lane >> 5) * 8 + (i16 >> 2), cl = ((lane >> 4) & 1) * 16 + (i16 & 3) * 4;
    // A block launched with one wave more than taps sums the bias gradient in that wave: it multiplies the dy^T fragments with
    // an all-ones operand (column 0 of the product = sum over the tile's pixels) and reads no x.  The waves sit 3-3-2-2 on the
    // four SIMDs instead of 3-2-2-2, and this wave issues half the matrix instructions of a tap wave: the block is no slower.
    const bool dbw = wave == R * S;
    const int tr = dbw ? 0 : wave / S, ts = dbw ? 0 : wave - tr * S;        // this wave's tap
    const int tapoff = tr * PW + ts;
    unsigned a_lane[2];   // dy: row tl of slice 0, column half i; later slices add 16 rows = 2048 bytes
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int col = i * 32 + cl;
        a_lane[i] = HALO_PP * 128 + tl * 128 + ((((col >> 5) ^ seg_swz<64>(tl)) << 6) | ((col & 31) << 1));
    }

    const TileWalk tw = tile_walk(tiles);
    int tile = tw.first;
    if (tile < tw.end) issue_tile(tile, 0);
    for (int it = 0; tile < tw.end; tile += tw.stride, ++it) {
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();   // tile `it` has landed everywhere; the other buffer is no longer read
        if (tile + tw.stride < tw.end) issue_tile(tile + tw.stride, (it + 1) & 1);
        const unsigned base = smem_base + (it & 1) * WH_BUF;
        // fragments are double-buffered in registers: the transpose reads of slice sl+1 are issued before the
        // matrix instructions of slice sl
        u32x2 alo[2][2], ahi[2][2], blo[2][2], bhi[2][2];
        auto read_slice = [&](int sl, int buf) {
            const int j = sl * 16 + tl;
            const int pp = (j >> tws) * PW + (j & (TW - 1)) + tapoff;
            const unsigned brow = base + pp * 128, bsw = seg_swz<64>(pp);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                alo[buf][i] = lds_read_tr<0>(base + a_lane[i] + sl * 2048);
                ahi[buf][i] = lds_read_tr<4 * 128>(base + a_lane[i] + sl * 2048);
            }
            if (dbw) return;   // wave-uniform
#pragma unroll
            for (int jf = 0; jf < 2; ++jf) {
                const int col = jf * 32 + cl;
                const unsigned addr = brow + ((((col >> 5) ^ bsw) << 6) | ((col & 31) << 1));
                blo[buf][jf] = lds_read_tr<0>(addr);
                bhi[buf][jf] = lds_read_tr<4 * 128>(addr);
            }
        };
        auto multiply = [&](int buf, bool newer_in_flight) {
            // reads of the next slice issued after this slice's: 8 for a tap wave, 4 for the bias-gradient wave
            if (!newer_in_flight) asm volatile("s_waitcnt lgkmcnt(0)");
            else if (dbw) asm volatile("s_waitcnt lgkmcnt(4)");
            else asm volatile("s_waitcnt lgkmcnt(8)");
            if (dbw) {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    asm volatile("" : "+v"(alo[buf][i])); asm volatile("" : "+v"(ahi[buf][i]));
                }
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const u32x4 av = {alo[buf][i].x, alo[buf][i].y, ahi[buf][i].x, ahi[buf][i].y};
                    acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), ones_bf16(), acc[i][0], 0, 0, 0);
                }
                return;
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                asm volatile("" : "+v"(alo[buf][i])); asm volatile("" : "+v"(ahi[buf][i]));
                asm volatile("" : "+v"(blo[buf][i])); asm volatile("" : "+v"(bhi[buf][i]));
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int jf = 0; jf < 2; ++jf) {
                    const u32x4 av = {alo[buf][i].x, alo[buf][i].y, ahi[buf][i].x, ahi[buf][i].y};
                    const u32x4 bv = {blo[buf][jf].x, blo[buf][jf].y, bhi[buf][jf].x, bhi[buf][jf].y};
                    acc[i][jf] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, bv), acc[i][jf], 0, 0, 0);
                }
        };
        read_slice(0, 0);
        for (int sl = 0; sl < HALO_TB / 16; sl += 2) {
            read_slice(sl + 1, 1);
            multiply(0, true);
            if (sl + 2 < HALO_TB / 16) read_slice(sl + 2, 0);
            multiply(1, sl + 2 < HALO_TB / 16);
        }
    }
    if (dbw) {   // column 0 of the ones-product: this block's bias-gradient sums, one row of [blocks][c_out]
        if (p.dbp != nullptr)
#pragma unroll
            for (int i = 0; i < 2; ++i) store_db_fragment(acc[i][0], p.dbp + (size_t)blockIdx.x * p.rowsA, a0 + i * 32, p.rowsA, lane);
        return;
    }
    // partial[block][c_out][tap][c_in]; accumulator element v of lane l: row 8*(v/4) + 4*(l/32) + v%4, column l%32
    float *out = p.partial + (size_t)blockIdx.x * p.rowsA * p.rowsB;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jf = 0; jf < 2; ++jf)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = a0 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (k < p.rowsA) out[(size_t)k * p.rowsB + wave * 64 + jf * 32 + (lane & 31)] = acc[i][jf][v];
            }
}

// ---------------------------------------------------------------------------------------
// The 3x3 form of the kernel above with all nine taps in ONE wave.  With a wave per tap every wave reads
// the same dy fragments and one x fragment per matrix instruction: 1 KB of LDS reads per matrix
// instruction, which is the LDS port's whole bandwidth at the matrix cores' full rate, and ten waves sit
// 3-3-2-2 on the SIMDs.  Here a block has four waves, one per SIMD: wave (pg, ch) takes every second
// 16-pixel slice of the tile (pixel group pg) and c_in half ch for all 64 output channels and all nine
// taps (18 accumulator tiles, 288 registers): per slice it reads the two dy fragments once and one x
// fragment per tap, 11 fragments for 18 matrix instructions (0.61 KB each), and the four SIMDs carry
// the same load.  The (slice, tap) pairs form one stream of items; the transpose reads of item i+4 are
// issued before the matrix instructions of item i (ring of six x fragments, two dy fragment pairs; at
// most 14 reads in flight, the counter holds 15).  The two pixel groups' sums meet in LDS once, at the
// end of the kernel.  The bias gradient (dy x ones) rides in the ch = 0 waves, two more matrix
// instructions per slice.  Tile walk, LDS layout, copies and the per-block partial are the kernel's above.
// ---------------------------------------------------------------------------------------
// The matrix instructions are pinned (mfma_in_regs) to the accumulation registers or to the vector registers: 18 + 2 accumulator
// tiles are 320 registers, more than the 256 accumulation registers, and the compiler, left to itself, keeps them all there and
// copies tiles back and forth around every instruction (six copies per matrix instruction).
template <int OFF, bool AG> DEVFN void lds_write_f32(unsigned addr, float v)   // AG: the value sits in an accumulation register
{
    if constexpr (AG) asm volatile("ds_write_b32 %0, %1 offset:%2" : : "v"(addr), "a"(v), "n"(OFF) : "memory");
    else asm volatile("ds_write_b32 %0, %1 offset:%2" : : "v"(addr), "v"(v), "n"(OFF) : "memory");
}
template <int OFF> DEVFN float lds_read_f32(unsigned addr)
{
    float v;
    asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}

template <bool DB>
__global__ __launch_bounds__(256) void k_wgrad_halo9(const KArgs p, int tws, int tiles_x, int tiles_y, int tiles)
{
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const ConvGeom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int pg = wave >> 1, ch = wave & 1;
    const int TW = 1 << tws, TH = HALO_TB >> tws, PW = TW + 2, PP = (TH + 2) * PW;
    const int a0 = blockIdx.y * 64;
    const unsigned smem_base = lds_offset(smem);
    __amdgpu_buffer_rsrc_t rdy = make_rsrc(p.dy, (size_t)g.N * g.Ho * g.Wo * g.K * 2);
    __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, (size_t)g.N * g.H * g.W * g.C * 2);
    // Copies of a tile (8 LDS rows each): 44 of the patch, 32 of the dy slice; wave w issues patch copies w, w+4, ... and dy copies
    // w, w+4, ...  One wave per SIMD has nobody to hide the address arithmetic behind, so everything that does not depend on the
    // tile is computed once: the byte offset of the lane's 16 bytes relative to the tile's first patch / dy pixel and the pixel's
    // row and column in the patch / tile (packed; 0xffff rows mark lanes that never copy).  Per tile and copy that leaves two range
    // checks and an addition, and the copies of the next tile are dealt out over the items of this one.
    constexpr int NCP = HALO_PP / 8 / 4, NCD = HALO_TB / 8 / 4;
    static_assert(NCP * 32 == HALO_PP && NCD * 32 == HALO_TB, "the copies divide evenly over the four waves");
    unsigned xrel[NCP], xrc[NCP], drel[NCD], drc[NCD];
#pragma unroll
    for (int c = 0; c < NCP; ++c) {
        const int pp = (wave + 4 * c) * 8 + (lane >> 3), chunk = (lane & 7) ^ (seg_swz<64>(pp) << 2);
        const int pr = pp / PW, pc = pp - pr * PW;
        xrel[c] = (unsigned)((pr * g.W + pc) * 64 + chunk * 8) * 2u;
        xrc[c] = pp < PP ? (unsigned)(pr << 16 | pc) : 0xffff0000u;
    }
#pragma unroll
    for (int c = 0; c < NCD; ++c) {
        const int j = (wave + 4 * c) * 8 + (lane >> 3), chunk = (lane & 7) ^ (seg_swz<64>(j) << 2);
        const int jr = j >> tws, jc = j & (TW - 1);
        drel[c] = (unsigned)((jr * g.Wo + jc) * g.K + a0 + chunk * 8) * 2u;
        drc[c] = a0 + chunk * 8 + 8 <= g.K ? (unsigned)(jr << 16 | jc) : 0xffff0000u;
    }
    // tile-dependent part, wave-uniform: first patch / dy pixel of the tile as byte offsets (the patch origin may lie outside the
    // image: the sum wraps, and wraps back for every pixel that passes the range checks), and the tile's position
    int nt_p0 = 0, nt_q0 = 0;
    unsigned nt_xbase = 0, nt_dbase = 0, nt_lds = 0;
    auto set_tile = [&](int tile, int buf) {
        const int n = tile / (tiles_x * tiles_y), trem = tile - n * (tiles_x * tiles_y), ty = trem / tiles_x, tx = trem - ty * tiles_x;
        nt_p0 = ty * TH; nt_q0 = tx * TW;
        nt_xbase = (unsigned)(((n * g.H + nt_p0 - g.ph) * g.W + nt_q0 - g.pw) * 64) * 2u;
        nt_dbase = (unsigned)(((n * g.Ho + nt_p0) * g.Wo + nt_q0) * g.K) * 2u;
        nt_lds = smem_base + buf * WH_BUF;
    };
    auto issue_copy = [&](int c) {   // c: 0 .. NCP-1 patch copies, then NCD dy copies (compile-time)
        if (c < NCP) {
            const int ih = nt_p0 - g.ph + (int)(xrc[c] >> 16), iw = nt_q0 - g.pw + (int)(xrc[c] & 0xffffu);
            const bool ok = (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
            dma16(rx, nt_lds + (wave + 4 * c) * 1024, ok ? nt_xbase + xrel[c] : OOR);
        } else {
            const int d = c - NCP;
            const bool ok = nt_p0 + (int)(drc[d] >> 16) < g.Ho && nt_q0 + (int)(drc[d] & 0xffffu) < g.Wo;
            dma16(rdy, nt_lds + HALO_PP * 128 + (wave + 4 * d) * 1024, ok ? nt_dbase + drel[d] : OOR);
        }
    };

    f32x16 acc[9][2];   // [tap][c_out half]
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][i][v] = 0.f;
    f32x16 accdb[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) accdb[i][v] = 0.f;
    const bool do_db = DB && ch == 0;   // wave-uniform
    const u32x4 ones = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};   // bf16 1.0 in every element

    // transpose-read lane roles: reduction row tl (+4 for the second read), operand columns cl .. cl+3
    const int i16 = lane & 15, tl = (lane >> 5) * 8 + (i16 >> 2), cl = ((lane >> 4) & 1) * 16 + (i16 & 3) * 4;
    unsigned a_lane[2];   // dy: row tl of slice 0, column half i; later slices add 16 rows = 2048 bytes
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int col = i * 32 + cl;
        a_lane[i] = HALO_PP * 128 + tl * 128 + ((((col >> 5) ^ seg_swz<64>(tl)) << 6) | ((col & 31) << 1));
    }
    const unsigned x_lane = (unsigned)(ch << 6) | (unsigned)(cl << 1);   // segment ch, columns cl .. cl+3 (the segment bit is swizzled per row)
    int toff[9];   // patch pixels between tap (0,0) and tap t: wave-uniform
#pragma unroll
    for (int t = 0; t < 9; ++t) toff[t] = (t / 3) * PW + (t % 3);

    u32x2 xlo[6], xhi[6], dlo[2][2], dhi[2][2];
    // q: index of this wave's slice (slice pg + 2q of the tile); reads of one item: the x fragment of tap t of that slice
    auto read_dy = [&](unsigned base, int q, int buf) {
        const unsigned off = base + (unsigned)(pg + 2 * q) * 2048u;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            dlo[buf][i] = lds_read_tr<0>(off + a_lane[i]);
            dhi[buf][i] = lds_read_tr<4 * 128>(off + a_lane[i]);
        }
    };
    int tlv = tl;   // the lane's reduction row, made opaque once per slice: the fragment addresses are a few vector instructions per item,
                    // and computed per item they cost no registers, whereas the compiler would hoist all 72 of a tile (and spill)
    auto read_x = [&](unsigned base, int q, int t, int slot) {
        const int j = (pg + 2 * q) * 16 + tlv;
        const unsigned pp = (unsigned)((j >> tws) * PW + (j & (TW - 1)) + toff[t]);
        const unsigned addr = base + (pp << 7) + (x_lane ^ ((pp & 2u) << 5));
        xlo[slot] = lds_read_tr<0>(addr);
        xhi[slot] = lds_read_tr<4 * 128>(addr);
    };

    const TileWalk tw = tile_walk(tiles);
    int tile = tw.first;
    if (tile < tw.end) {
        set_tile(tile, 0);
#pragma unroll
        for (int c = 0; c < NCP + NCD; ++c) issue_copy(c);
    }
    for (int it = 0; tile < tw.end; tile += tw.stride, ++it) {
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();   // tile `it` has landed everywhere; the other buffer is no longer read
        const bool more = tile + tw.stride < tw.end;   // wave-uniform
        if (more) set_tile(tile + tw.stride, (it + 1) & 1);
        const unsigned base = smem_base + (it & 1) * WH_BUF;
        read_dy(base, 0, 0);
#pragma unroll
        for (int t = 0; t < 4; ++t) read_x(base, 0, t, t);
        for_constant<72>([&](auto ic) {   // every index below is a compile-time constant: registers, not indexed arrays
            constexpr int i = decltype(ic)::value;
            // reads of item i+4; past the tile's end the stream re-reads the last slice (never multiplied)
            constexpr int j = i + 4, jq = j < 72 ? j / 9 : 7, jt = j % 9;
            if constexpr (jt == 0) {
                asm volatile("" : "+v"(tlv));
                read_dy(base, jq, (j / 9) & 1);
            }
            read_x(base, jq, jt, j % 6);
            // reads issued after item i's own: items i+1 .. i+4, two each, four more where a slice begins
            constexpr int ti = i % 9;
            if constexpr (ti >= 5) asm volatile("s_waitcnt lgkmcnt(12)");
            else asm volatile("s_waitcnt lgkmcnt(8)");
            constexpr int s6 = i % 6, db = (i / 9) & 1;
            asm volatile("" : "+v"(xlo[s6])); asm volatile("" : "+v"(xhi[s6]));
#pragma unroll
            for (int k = 0; k < 2; ++k) { asm volatile("" : "+v"(dlo[db][k])); asm volatile("" : "+v"(dhi[db][k])); }
            const u32x4 bv = {xlo[s6].x, xlo[s6].y, xhi[s6].x, xhi[s6].y};
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const u32x4 av = {dlo[db][k].x, dlo[db][k].y, dhi[db][k].x, dhi[db][k].y};
                if constexpr (ti < 8) mfma_in_regs<true>(acc[ti][k], av, bv);    // taps 0-7: the 256 accumulation registers
                else mfma_in_regs<false>(acc[ti][k], av, bv);                    // tap 8 and the bias gradient: vector registers
            }
            if constexpr (ti == 0) {
                if (do_db) {
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        const u32x4 av = {dlo[db][k].x, dlo[db][k].y, dhi[db][k].x, dhi[db][k].y};
                        mfma_in_regs<false>(accdb[k], av, ones);
                    }
                }
            }
            // one copy of the next tile after each of the first 19 items: memory latency under load is a good part of a tile's time
            // (issued after every second item: 170 us instead of 162 for conv1_2 at batch 32; two per item: no faster)
            if constexpr (i < NCP + NCD) { if (more) issue_copy(i); }
        });
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the stream's reads past the end have returned
    }
    // the last matrix instructions have written their results before anything reads them (16 passes of 4 clocks)
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");

    // Epilogue, one round per half of the 64 output channels (nine accumulator tiles and one bias-gradient tile per wave): pixel
    // group 1 puts its tiles into an exchange area (lane-major: no bank conflicts), pixel group 0 adds its own and writes the sums in
    // the partial's layout [32 c_out][9 taps x 64 c_in] into the result area, and all four waves copy that out, 16 bytes per lane and
    // whole rows at a time.  The sums never go back into the accumulators (with all 320 of them live, adding in place made the
    // compiler spill accumulators; LDS float atomics instead of the exchange measured 30 us slower per block; storing from registers,
    // 4 bytes per lane with an address pair per store, spilled too).  The two areas (80 KB + 72 KB) are the 152 KB the tile buffers
    // held; they swap ends between the rounds.  Accumulator element v of lane l: row 8*(v/4) + 4*(l/32) + v%4, column l%32.
    constexpr int kXchBytes = 2 * 10 * 16 * 64 * 4, kResBytes = 32 * 576 * 4;
    static_assert(kXchBytes + kResBytes <= 2 * WH_BUF, "exchange and result areas fit in the two tile buffers");
    // The LDS traffic of the exchange is inline assembly: volatile statements keep their order, so at most one tile's values are in
    // flight and the register allocator has nothing to spill.
    for_constant<2>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        const unsigned xaddr = smem_base + (i == 0 ? kResBytes : 0) + ch * (10 * 16 * 256) + lane * 4;   // this lane's column of the exchange area
        float *res = reinterpret_cast<float *>(smem + (i == 0 ? 0 : kXchBytes));
        const unsigned raddr = smem_base + (i == 0 ? 0 : kXchBytes) + (unsigned)((4 * (lane >> 5)) * 576 + ch * 32 + (lane & 31)) * 4u;
        __syncthreads();   // round 0: every wave is past its last tile; round 1: the first half has been copied out
        if (pg == 1) {
            for_constant<10>([&](auto fc) {
                constexpr int f = decltype(fc)::value;
                const f32x16 &src = f < 9 ? acc[f < 9 ? f : 0][i] : accdb[i];
                for_constant<16>([&](auto vc) {
                    constexpr int v = decltype(vc)::value;
                    lds_write_f32<(f * 16 + v) * 256, (f < 8)>(xaddr, src[v]);   // taps 0-7 straight from the accumulation registers
                });
            });
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        __syncthreads();
        if (pg == 0) {
            for_constant<10>([&](auto fc) {
                constexpr int f = decltype(fc)::value;
                if (f == 9 && !(do_db && p.dbp != nullptr)) return;
                const f32x16 &mine = f < 9 ? acc[f < 9 ? f : 0][i] : accdb[i];
                f32x16 sum;
                for_constant<2>([&](auto hc) {   // eight values at a time (the counter of LDS operations in flight holds 15)
                    constexpr int h = decltype(hc)::value;
                    float tv[8];
                    for_constant<8>([&](auto vc) {
                        constexpr int w = decltype(vc)::value;
                        tv[w] = lds_read_f32<(f * 16 + h * 8 + w) * 256>(xaddr);
                    });
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    for_constant<8>([&](auto vc) {
                        constexpr int w = decltype(vc)::value, v = h * 8 + w;
                        asm volatile("" : "+v"(tv[w]));
                        float mv = mine[v];
                        if (f < 8) asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(mv) : "a"(mine[v]));   // in order: read early, these get spilled
                        sum[v] = mv + tv[w];
                        if (f < 9) lds_write_f32<((8 * (v >> 2) + (v & 3)) * 576 + (f < 9 ? f : 0) * 64) * 4, false>(raddr, sum[v]);
                    });
                });
                if (f == 9) store_db_fragment(sum, p.dbp + (size_t)blockIdx.x * p.rowsA, a0 + i * 32, p.rowsA, lane);
            });
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        __syncthreads();
        // partial[block][c_out][tap][c_in]: rows a0 + 32 i .. + 31 of it, 144 chunks of 16 bytes per row
        float *out = p.partial + ((size_t)blockIdx.x * p.rowsA + a0 + 32 * i) * 576;
        const int rows = min(32, p.rowsA - a0 - 32 * i);
        for (int c = tid; c < rows * 144; c += 256)
            *reinterpret_cast<f32x4 *>(out + (size_t)c * 4) = *reinterpret_cast<const f32x4 *>(res + c * 4);
    });
}

// ---------------------------------------------------------------------------------------
// 3x3 (nine-tap) forward / backward-data with 64 reduction channels per tap, weights stationary in
// REGISTERS.  A block has four waves, one per SIMD, so each may use the whole register file: a wave
// keeps the fragments of all 64 output channels for all nine taps (72 fragments, 288 registers) and
// multiplies them with 64 pixels of the tile; nothing but the input patch goes through LDS (512 bytes
// read per matrix instruction, half of what a 32-channel wave would need) and no barrier separates
// the taps.  Blocks are persistent (one per CU and 64-channel tile) and keep three patch buffers:
// while tile i is multiplied, the patches of tiles i+1 and i+2 are on their way.  The accumulators go
// straight to the NHWC output: a lane pair exchanges halves so that each lane stores 16 bytes.  One
// barrier per tile.
// ---------------------------------------------------------------------------------------
constexpr int WS_PATCH = HALO_PP * 128;   // 44 KiB per patch buffer
constexpr int WS_LDS = 3 * WS_PATCH + 64 * 4;
constexpr int WS_DEPTH = 3;               // fragment reads run this many 16-channel slices ahead of the matrix cores
constexpr int WS_CPW = HALO_PP / 8 / 4;   // patch copies per wave
static_assert(WS_CPW * 4 * 8 == HALO_PP, "patch copies divide evenly over the four waves");
static_assert(WS_PATCH + 9 * 8192 <= 3 * WS_PATCH, "the weights are staged behind the first patch buffer");

template <int PASS, bool MASK = false>   // MASK (backward-data): fused backward of the ReLU in front of the layer
__global__ __launch_bounds__(256) void k_halo_ws(const KArgs p, int tws, int tiles_x, int tiles_y, int tiles_all)
{
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const ConvGeom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int TW = 1 << tws, TH = HALO_TB >> tws, PW = TW + 2, PP = (TH + 2) * PW;
    const int a0 = blockIdx.y * 64;
    const int IH = PASS == PASS_FWD ? g.H : g.Ho, IW = PASS == PASS_FWD ? g.W : g.Wo;
    const int OH = PASS == PASS_FWD ? g.Ho : g.H, OW = PASS == PASS_FWD ? g.Wo : g.W;
    const int RSC = 9 * g.C;
    const unsigned smem_base = lds_offset(smem);
    float *bias_lds = reinterpret_cast<float *>(smem + 3 * WS_PATCH);
    __amdgpu_buffer_rsrc_t rin = PASS == PASS_FWD ? make_rsrc(p.x, (size_t)g.N * g.H * g.W * g.C * 2)
                                                  : make_rsrc(p.dy, (size_t)g.N * g.Ho * g.Wo * g.K * 2);
    __amdgpu_buffer_rsrc_t rw = make_rsrc(p.w, (size_t)g.K * RSC * 2);
    if (tid < 64) bias_lds[tid] = (PASS == PASS_FWD && (p.flags & KF_BIAS) && a0 + tid < p.rowsA) ? p.bias[a0 + tid] : 0.f;

    // patch copies of this lane: copy q of a wave fills patch pixels (wave*WS_CPW + q)*8 .. +7; the lane's
    // pixel (row, column) and channel chunk are fixed, only the tile origin changes
    unsigned pk[WS_CPW];
#pragma unroll
    for (int q = 0; q < WS_CPW; ++q) {
        const int pp = (wave * WS_CPW + q) * 8 + (lane >> 3), c = (lane & 7) ^ ((pp >> 1) & 7);
        const int pr = pp / PW, pc = pp - pr * PW;
        pk[q] = (unsigned)pr | ((unsigned)pc << 8) | ((unsigned)c << 16) | (pp < PP ? 1u << 24 : 0u);
    }
    auto issue_patch = [&](int tile, int buf) {
        const int n = tile / (tiles_x * tiles_y), trem = tile - n * (tiles_x * tiles_y), ty = trem / tiles_x, tx = trem - ty * tiles_x;
        const int h0 = PASS == PASS_FWD ? ty * TH - g.ph : ty * TH + g.ph - 2, w0 = PASS == PASS_FWD ? tx * TW - g.pw : tx * TW + g.pw - 2;
        const int nbase = n * IH;
#pragma unroll
        for (int q = 0; q < WS_CPW; ++q) {
            const int ih = h0 + (int)(pk[q] & 255u), iw = w0 + (int)((pk[q] >> 8) & 255u), c = (pk[q] >> 16) & 7;
            const bool ok = (pk[q] >> 24) != 0 && (unsigned)ih < (unsigned)IH && (unsigned)iw < (unsigned)IW;
            dma16(rin, smem_base + buf * WS_PATCH + (wave * WS_CPW + q) * 1024, ok ? (unsigned)(((nbase + ih) * IW + iw) * 64 + c * 8) * 2u : OOR);
        }
    };
    const TileWalk tw = tile_walk(tiles_all);
    int tile = tw.first;
    const int stride = tw.stride, tiles = tw.end;   // this block's tiles: tile, tile + stride, ... below `tiles`
    if (tile < tiles) issue_patch(tile, 0);

    // ---- weights: through LDS (behind the first patch buffer) into registers ------------------------
    // forward: the tile of step st is [64 c_out][64 c_in], chunk swizzle by row pair; backward-data: the tile
    // of step st (filter tap 8 - st) is [64 c_out][64 c_in] with c_out the reduction, read transposed
    const unsigned wst = smem_base + WS_PATCH;
#pragma unroll
    for (int q = 0; q < 18; ++q) {
        const int id = wave * 18 + q, st = id >> 3, row = (id & 7) * 8 + (lane >> 3);
        unsigned voff;
        if (PASS == PASS_FWD) {
            const int c = (lane & 7) ^ ((row >> 1) & 7);
            voff = a0 + row < p.rowsA ? ((unsigned)(a0 + row) * RSC + st * 64 + c * 8) * 2u : OOR;
        } else {
            const int c = (lane & 7) ^ (seg_swz<64>(row) << 2);
            voff = a0 + c * 8 < p.rowsA ? ((unsigned)row * RSC + (8 - st) * g.C + a0 + c * 8) * 2u : OOR;
        }
        dma16(rw, wst + id * 1024, voff);
    }
    wait_vmcnt<0>();
    __syncthreads();
    // (plain LDS loads here: the compiler places their waits; the hand-counted reads start with the tile loop)
    u32x4 afr[9][4][2];   // [step][slice][32-row half]
    {
        const char *wl = smem + WS_PATCH;
        typedef short v4s __attribute__((ext_vector_type(4)));
        typedef __attribute__((address_space(3))) v4s *lds_v4s;
        const int i16 = lane & 15, tl = (lane >> 5) * 8 + (i16 >> 2), cl = ((lane >> 4) & 1) * 16 + (i16 & 3) * 4;
#pragma unroll
        for (int st = 0; st < 9; ++st)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    if (PASS == PASS_FWD) {
                        const int row = i * 32 + (lane & 31);
                        afr[st][ks][i] = *reinterpret_cast<const u32x4 *>(wl + st * 8192 + row * 128 + (((2 * ks + (lane >> 5)) ^ ((row >> 1) & 7)) << 4));
                    } else {
                        const int t = ks * 16 + tl, col = i * 32 + cl;
                        const char *a = wl + st * 8192 + t * 128 + ((((col >> 5) ^ seg_swz<64>(t)) << 6) | ((col & 31) << 1));
                        const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(a));
                        const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(a + 4 * 128));
                        const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
                        afr[st][ks][i] = u32x4{l2.x, l2.y, h2.x, h2.y};
                    }
                }
    }
    __syncthreads();   // the staging area is free for patches; the first patch has landed (waited above)
    if (tile + stride < tiles) issue_patch(tile + stride, 1);

    int pp0[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int jj = wave * 64 + j * 32 + (lane & 31);
        pp0[j] = (jj >> tws) * PW + (jj & (TW - 1));
    }
    const unsigned hsel = lane >> 5;
    bf16_t *out = reinterpret_cast<bf16_t *>(p.out);

    // A wave that issues a memory instruction into a full queue stalls, matrix instructions included, so the
    // copies of the patch two tiles ahead and the stores of the previous tile's output (held packed in
    // registers meanwhile) are spread over the 36 slices of the running tile instead of issued in a burst.
    u32x4 ost[MASK ? 1 : 8];           // previous tile: [pixel fragment j][channel half i][group pair gp], 8 channels of one pixel each
    bf16_t *optr[2] = {out, out};   // this lane's output row of fragment j (previous tile), at channel a0
    bool ook[2] = {false, false};
    bool have_prev = false;
    // backward of the ReLU in front of the layer (KF_MASK_IN): the eight saved-input vectors that match this lane's eight output vectors of
    // the running tile are requested before its first matrix instruction and used in its epilogue, behind the wait that every tile ends with
    // (the masked form has no registers left to hold the previous tile's output as well: it stores each tile in its own epilogue)
    constexpr bool mask_in = MASK;
    u32x4 mk[MASK ? 8 : 1];
    auto store_one = [&](int k) {
        const int j = k >> 2, i = (k >> 1) & 1, gp = k & 1;
        const int ch = i * 32 + 8 * (2 * gp + (int)hsel);
        if (ook[j] && a0 + ch < p.rowsA) asm volatile("global_store_dwordx4 %0, %1, off" ::"v"(optr[j] + ch), "v"(ost[k]) : "memory");
    };

    for (int it = 0; tile < tiles; tile += stride, ++it) {
        // buffer (it + 2) % 3 held tile it - 1, which every wave had finished before the last barrier
        const bool more1 = tile + stride < tiles, more2 = tile + 2 * stride < tiles;
        int nh0 = 0, nw0 = 0, nnb = 0;   // origin of the patch two tiles ahead
        if (more2) {
            const int t2 = tile + 2 * stride;
            const int n = t2 / (tiles_x * tiles_y), trem = t2 - n * (tiles_x * tiles_y), ty = trem / tiles_x, tx = trem - ty * tiles_x;
            nh0 = PASS == PASS_FWD ? ty * TH - g.ph : ty * TH + g.ph - 2;
            nw0 = PASS == PASS_FWD ? tx * TW - g.pw : tx * TW + g.pw - 2;
            nnb = n * IH;
        }
        const unsigned nbuf = smem_base + ((it + 2) % 3) * WS_PATCH + wave * WS_CPW * 1024;
        auto copy_one = [&](int q) {
            const int ih = nh0 + (int)(pk[q] & 255u), iw = nw0 + (int)((pk[q] >> 8) & 255u), c = (pk[q] >> 16) & 7;
            const bool ok = (pk[q] >> 24) != 0 && (unsigned)ih < (unsigned)IH && (unsigned)iw < (unsigned)IW;
            dma16(rin, nbuf + q * 1024, ok ? (unsigned)(((nnb + ih) * IW + iw) * 64 + c * 8) * 2u : OOR);
        };
        const unsigned base = smem_base + (it % 3) * WS_PATCH;
        if (mask_in) {
            const int n = tile / (tiles_x * tiles_y), trem = tile - n * (tiles_x * tiles_y), ty = trem / tiles_x, tx = trem - ty * tiles_x;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int pix = wave * 64 + j * 32 + (lane & 31);
                const int pr = ty * TH + (pix >> tws), qc = tx * TW + (pix & (TW - 1));
                const bool ok = pr < OH && qc < OW;
                // a lane without an output pixel reads the first pixel instead: the load is issued by every lane, so the wait below counts right
                const bf16_t *xrow = p.x + (ok ? ((size_t)(n * OH + pr) * OW + qc) * p.rowsA + a0 : (size_t)0);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int gp = 0; gp < 2; ++gp) {
                        const int ch = i * 32 + 8 * (2 * gp + (int)hsel);
                        const bf16_t *src = xrow + (ok && a0 + ch < p.rowsA ? ch : 0);
                        asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(mk[j * 4 + i * 2 + gp]) : "v"(src) : "memory");
                    }
            }
        }
        asm volatile("" : "+v"(pp0[0]), "+v"(pp0[1]));   // keeps the 72 read addresses from being computed ahead of the loop
        f32x16 acc[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        u32x4 fb[WS_DEPTH + 1][2];   // [buffer][pixel fragment]
        // chunk (2*ks + hsel) ^ swz = ((hsel ^ swz) ^ 2*ks): the address of slice ks is the address of slice 0 with bits 5-6 flipped by ks,
        // so a tap costs one address computation per pixel fragment and three exclusive-ors
        unsigned b0[2] = {0, 0};
        auto read_b = [&](int sl) {
            const int st = sl >> 2, ks = sl & 3;
            if (ks == 0) {
                const int off = (st / 3) * PW + (st % 3);
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int pp = pp0[j] + off;
                    b0[j] = base + pp * 128 + (((int)hsel ^ ((pp >> 1) & 7)) << 4);
                }
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) fb[sl % (WS_DEPTH + 1)][j] = lds_read16<0>(b0[j] ^ (unsigned)(ks << 5));
        };
#pragma unroll
        for (int sl = 0; sl < WS_DEPTH; ++sl) read_b(sl);
#pragma unroll
        for (int sl = 0; sl < 36; ++sl) {
            if (sl + WS_DEPTH < 36) read_b(sl + WS_DEPTH);
            constexpr int kFull = 2 * WS_DEPTH;
            const int newer = 2 * (35 - sl < WS_DEPTH ? 35 - sl : WS_DEPTH);   // reads issued after this slice's
            if (newer == kFull) asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(kFull));
            else if (newer == 4) asm volatile("s_waitcnt lgkmcnt(4)");
            else if (newer == 2) asm volatile("s_waitcnt lgkmcnt(2)");
            else asm volatile("s_waitcnt lgkmcnt(0)");
            const int cur = sl % (WS_DEPTH + 1);
            asm volatile("" : "+v"(fb[cur][0]));
            asm volatile("" : "+v"(fb[cur][1]));
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, afr[sl >> 2][sl & 3][i]),
                                                                       __builtin_bit_cast(bf16x8, fb[cur][j]), acc[i][j], 0, 0, 0);
            if (sl % 3 == 1 && sl / 3 < WS_CPW) {
                if (more2) copy_one(sl / 3);
            }
            if (!MASK && sl % 4 == 2 && sl / 4 < 8) {
                if (have_prev) store_one(sl / 4);
            }
        }
        // this wave's share of the next patch has landed: of the loads issued after it (the copies above) none can
        // still be outstanding once at most that many operations are
        if (more1) {
            if (more2) wait_vmcnt<WS_CPW>();
            else wait_vmcnt<0>();
        } else if (mask_in) {
            wait_vmcnt<0>();
        }
        // the saved-input vectors were requested before everything this tile issued, so they have landed as well
        if (mask_in) {
#pragma unroll
            for (int k = 0; k < 8; ++k) asm volatile("" : "+v"(mk[k]));
        }
        // accumulator element v of lane l is channel i*32 + 8*(v/4) + 4*(l/32) + v%4 of pixel l%32 of fragment j; the lanes
        // l and l+32 swap halves of two channel groups, after which each holds 8 consecutive channels of one group
        {
            const int n = tile / (tiles_x * tiles_y), trem = tile - n * (tiles_x * tiles_y), ty = trem / tiles_x, tx = trem - ty * tiles_x;
            // the eight bias vectors of this lane's channels, read together (one wait instead of eight round trips to LDS)
            f32x4 bvv[2][4];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq)
                    bvv[i][gq] = PASS == PASS_FWD ? *reinterpret_cast<const f32x4 *>(bias_lds + i * 32 + 8 * gq + 4 * hsel) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) asm volatile("" : "+v"(bvv[i][gq]));   // all eight are in registers before the first is used
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int pix = wave * 64 + j * 32 + (lane & 31);
                const int pr = ty * TH + (pix >> tws), qc = tx * TW + (pix & (TW - 1));
                ook[j] = pr < OH && qc < OW;
                optr[j] = out + ((size_t)(n * OH + pr) * OW + qc) * p.rowsA + a0;
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int gp = 0; gp < 2; ++gp) {
                        unsigned pkd[2][2];   // [group 2gp, 2gp+1][channel pair]
#pragma unroll
                        for (int e = 0; e < 2; ++e) {
                            const int gq = 2 * gp + e;
                            const f32x4 bv = bvv[i][gq];
                            float v0 = acc[i][j][4 * gq] + bv.x, v1 = acc[i][j][4 * gq + 1] + bv.y, v2 = acc[i][j][4 * gq + 2] + bv.z,
                                  v3 = acc[i][j][4 * gq + 3] + bv.w;
                            if (PASS == PASS_FWD && (p.flags & KF_RELU)) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f); }
                            pkd[e][0] = pack_bf16(v0, v1);
                            pkd[e][1] = pack_bf16(v2, v3);
                        }
                        const auto s0 = __builtin_amdgcn_permlane32_swap(pkd[0][0], pkd[1][0], false, false);
                        const auto s1 = __builtin_amdgcn_permlane32_swap(pkd[0][1], pkd[1][1], false, false);
                        const u32x4 packed = u32x4{s0[0], s1[0], s0[1], s1[1]};
                        if constexpr (MASK) {
                            ost[0] = apply_mask(packed, mk[j * 4 + i * 2 + gp]);
                            const int ch = i * 32 + 8 * (2 * gp + (int)hsel);
                            if (ook[j] && a0 + ch < p.rowsA) asm volatile("global_store_dwordx4 %0, %1, off" ::"v"(optr[j] + ch), "v"(ost[0]) : "memory");
                        } else {
                            ost[j * 4 + i * 2 + gp] = packed;
                        }
                    }
            }
            have_prev = !MASK;
        }
        __builtin_amdgcn_s_barrier();   // all shares of the next patch have landed; this tile's buffer is free (no fence: copies and stores stay in flight)
    }
    if (have_prev) {
#pragma unroll
        for (int k = 0; k < 8; ++k) store_one(k);
    }
}

struct HaloVariant { int TA, WA, WB, NS; };
const HaloVariant kHalo[] = {{64, 1, 4, 2}, {128, 2, 2, 2}, {64, 1, 4, 3}, {64, 1, 4, 4}};
constexpr int kNumHalo = 4;
typedef void (*HaloFn)(const KArgs, int, int, int);
HaloFn pick_halo(int pass, int v)
{
    if (pass == PASS_FWD) {
        switch (v) {
        case 1: return k_halo<PASS_FWD, 128, 2, 2, 2>;
        case 2: return k_halo<PASS_FWD, 64, 1, 4, 3>;
        case 3: return k_halo<PASS_FWD, 64, 1, 4, 4>;
        default: return k_halo<PASS_FWD, 64, 1, 4, 2>;
        }
    }
    switch (v) {
    case 1: return k_halo<PASS_DGRAD, 128, 2, 2, 2>;
    case 2: return k_halo<PASS_DGRAD, 64, 1, 4, 3>;
    case 3: return k_halo<PASS_DGRAD, 64, 1, 4, 4>;
    default: return k_halo<PASS_DGRAD, 64, 1, 4, 2>;
    }
}
size_t halo_lds_bytes(const HaloVariant &h)
{
    const int nw = h.WA * h.WB;
    const size_t ip = (HALO_PP * 128 / 1024 + nw - 1) / nw;
    const size_t stages = ip * nw * 1024 + (size_t)h.NS * h.TA * 128, epi = (size_t)HALO_TB * (h.TA + 8) * 2;
    return (stages > epi ? stages : epi) + (size_t)h.TA * 4;
}
// tile shape with the least padded area: 8 x 32 (tws 5) or 16 x 16 (tws 4) output pixels
int halo_tws(int oh, int ow)
{
    const long long a5 = (long long)((oh + 7) / 8 * 8) * ((ow + 31) / 32 * 32), a4 = (long long)((oh + 15) / 16 * 16) * ((ow + 15) / 16 * 16);
    return a4 < a5 ? 4 : 5;
}

}  // namespace

hipError_t halo_init()
{
    {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_wgrad_halo), hipFuncAttributeMaxDynamicSharedMemorySize, 2 * WH_BUF);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_wgrad_halo9<true>), hipFuncAttributeMaxDynamicSharedMemorySize, 2 * WH_BUF);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_wgrad_halo9<false>), hipFuncAttributeMaxDynamicSharedMemorySize, 2 * WH_BUF);
        if (e != hipSuccess) return e;
    }
    {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_halo_ws<PASS_FWD>), hipFuncAttributeMaxDynamicSharedMemorySize, WS_LDS);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_halo_ws<PASS_DGRAD>), hipFuncAttributeMaxDynamicSharedMemorySize, WS_LDS);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_halo_ws<PASS_DGRAD, true>), hipFuncAttributeMaxDynamicSharedMemorySize, WS_LDS);
        if (e != hipSuccess) return e;
    }
    for (int pass = 0; pass < 2; ++pass)
        for (int v = 0; v < kNumHalo; ++v) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pick_halo(pass, v)), hipFuncAttributeMaxDynamicSharedMemorySize,
                                               (int)halo_lds_bytes(kHalo[v]));
            if (e != hipSuccess) return e;
        }
    return hipSuccess;
}

// variant override 400 + v; forward needs c_in == 64, backward-data c_out == 64; stride 1; no reduction split
bool halo_plan(const ConvGeom &g, int pass, int force_variant, int force_splits, GemmPlan *pl)
{
    if (pass == PASS_WGRAD) {   // 410: input-patch filter gradient, a wave per tap; 411: 3x3, all taps per wave; force_splits = number of persistent blocks
        if ((force_variant != 410 && force_variant != 411) || g.sh != 1 || g.sw != 1 || g.C != 64 || (g.K % 8) != 0 || g.R * g.S > 16) return false;
        if (force_variant == 411 && (g.R != 3 || g.S != 3)) return false;
        const int tws = halo_tws(g.Ho, g.Wo), tw = 1 << tws, th = HALO_TB >> tws;
        if ((th + g.R - 1) * (tw + g.S - 1) > HALO_PP) return false;
        const long long tiles = (long long)g.N * ((g.Ho + th - 1) / th) * ((g.Wo + tw - 1) / tw);
        const int ktiles = (g.K + 63) / 64;
        int blocks = force_splits > 1 ? force_splits : 256 / ktiles;   // default: one persistent block per CU
        if (blocks > tiles) blocks = (int)tiles;
        if (blocks < 2) return false;   // the split-reduce kernel writes the result
        pl->variant = force_variant - 400;
        pl->db_wave = force_variant == 411 || g.R * g.S <= 15;   // 16 waves per block at most; the nine-tap kernel sums it in its own waves
        pl->fast = true; pl->dma = true; pl->halo = true;
        pl->TA = 64; pl->TB = 64 * g.R * g.S; pl->BK = 16; pl->vecA = pl->vecB = true;
        pl->tilesA = ktiles; pl->tilesB = 1;
        pl->steps_total = (int)tiles * (HALO_TB / 16);
        pl->steps_per_split = (int)((tiles + blocks - 1) / blocks) * (HALO_TB / 16);
        pl->splits = blocks;
        return true;
    }
    if (pass != PASS_FWD && pass != PASS_DGRAD) return false;
    pl->blocks = 0;
    if (force_variant == 404) {   // weights in registers, persistent blocks; force_splits = blocks per 64-row tile
        const int red_c = pass == PASS_FWD ? g.C : g.K, rowsA = pass == PASS_FWD ? g.K : g.C;
        if (g.sh != 1 || g.sw != 1 || g.R != 3 || g.S != 3 || red_c != 64 || (rowsA % 8) != 0) return false;
        if (pass == PASS_DGRAD && (g.ph > 2 || g.pw > 2)) return false;
        const int oh = pass == PASS_FWD ? g.Ho : g.H, ow = pass == PASS_FWD ? g.Wo : g.W;
        const int tws = halo_tws(oh, ow), tw = 1 << tws, th = HALO_TB >> tws;
        const long long tiles = (long long)g.N * ((oh + th - 1) / th) * ((ow + tw - 1) / tw);
        if (tiles > 0x7fffff) return false;
        pl->variant = 4;
        pl->fast = true; pl->dma = true; pl->halo = true;
        pl->TA = 64; pl->TB = HALO_TB; pl->BK = 64; pl->vecA = pl->vecB = true;
        pl->tilesA = (rowsA + 63) / 64;
        pl->tilesB = (int)tiles;
        pl->steps_total = pl->steps_per_split = 9;
        pl->splits = 1;
        pl->blocks = force_splits > 1 ? force_splits : 0;
        return true;
    }
    if (force_variant < 400 || force_variant >= 400 + kNumHalo || force_splits > 1) return false;
    if (g.sh != 1 || g.sw != 1 || g.R * g.S > 32) return false;
    const int red_c = pass == PASS_FWD ? g.C : g.K, rowsA = pass == PASS_FWD ? g.K : g.C;
    if (red_c != 64 || (rowsA % 8) != 0) return false;
    if (pass == PASS_DGRAD && (g.ph > g.R - 1 || g.pw > g.S - 1)) return false;
    const int oh = pass == PASS_FWD ? g.Ho : g.H, ow = pass == PASS_FWD ? g.Wo : g.W;
    const int tws = halo_tws(oh, ow), tw = 1 << tws, th = HALO_TB >> tws;
    if ((th + g.R - 1) * (tw + g.S - 1) > HALO_PP) return false;
    const HaloVariant &h = kHalo[force_variant - 400];
    pl->variant = force_variant - 400;
    pl->fast = true; pl->dma = true; pl->halo = true;
    pl->TA = h.TA; pl->TB = HALO_TB; pl->BK = 64; pl->vecA = pl->vecB = true;
    pl->tilesA = (rowsA + h.TA - 1) / h.TA;
    pl->tilesB = g.N * ((oh + th - 1) / th) * ((ow + tw - 1) / tw);
    pl->steps_total = pl->steps_per_split = g.R * g.S;
    pl->splits = 1;
    return true;
}

void halo_kernel_name(int pass, const GemmPlan &pl, bool masked, char *name, size_t name_bytes)
{
    if (pass == PASS_WGRAD) { snprintf(name, name_bytes, pl.variant == 11 ? "k_wgrad_halo9<true>" : "k_wgrad_halo"); return; }
    if (pl.variant == 4) { snprintf(name, name_bytes, "k_halo_ws<%d, %s>", pass, pass == PASS_DGRAD && masked ? "true" : "false"); return; }
    const HaloVariant &h = kHalo[pl.variant];
    snprintf(name, name_bytes, "k_halo<%d, %d, %d, %d, %d>", pass, h.TA, h.WA, h.WB, h.NS);
}

hipError_t halo_launch(const ConvArgs &a, hipStream_t st)
{
    KArgs p;
    p.g = a.g;
    if (a.pass == PASS_WGRAD) {
        const ConvGeom &g = a.g;
        p.rowsA = g.K; p.rowsB = g.R * g.S * g.C; p.red = g.N * g.Ho * g.Wo;
        p.tilesA = a.plan.tilesA; p.tilesB = 1; p.steps_total = a.plan.steps_total; p.steps_per_split = a.plan.steps_per_split;
        p.splits = a.plan.splits; p.flags = a.flags;
        p.x = a.x; p.w = nullptr; p.dy = a.dy; p.ymask = nullptr; p.bias = nullptr; p.out = a.out; p.partial = a.partial;
        // the bias gradient, when asked for, is summed by one extra wave per block; its [blocks][c_out] rows are added up by the split-reduce
        const bool db = (a.flags & KF_DB) && a.plan.db_wave && a.db_partial != nullptr && a.db_out != nullptr;
        p.dbp = db ? a.db_partial : nullptr;
        if (!db) p.flags &= ~KF_DB;
        const int tws = halo_tws(g.Ho, g.Wo), tw = 1 << tws, th = HALO_TB >> tws;
        const int tiles_x = (g.Wo + tw - 1) / tw, tiles_y = (g.Ho + th - 1) / th;
        if (a.plan.variant == 11) {
            void (*kern)(const KArgs, int, int, int, int) = k_wgrad_halo9<false>;
            if (db) kern = k_wgrad_halo9<true>;
            hipLaunchKernelGGL(kern, dim3((unsigned)a.plan.splits, (unsigned)a.plan.tilesA), dim3(256), 2 * WH_BUF, st, p, tws, tiles_x, tiles_y,
                               g.N * tiles_x * tiles_y);
        } else
            hipLaunchKernelGGL(k_wgrad_halo, dim3((unsigned)a.plan.splits, (unsigned)a.plan.tilesA), dim3(64 * (g.R * g.S + (db ? 1 : 0))), 2 * WH_BUF, st, p, tws,
                               tiles_x, tiles_y, g.N * tiles_x * tiles_y);
        dp_trace_main_kernel_done(st);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        return launch_split_reduce(a, p.rowsA, p.rowsB, st, db);
    }
    const bool fwd = a.pass == PASS_FWD;
    p.rowsA = fwd ? a.g.K : a.g.C;
    p.rowsB = fwd ? a.g.N * a.g.Ho * a.g.Wo : a.g.N * a.g.H * a.g.W;
    p.red = a.g.R * a.g.S * 64;
    p.tilesA = a.plan.tilesA; p.tilesB = a.plan.tilesB;
    p.steps_total = a.plan.steps_total; p.steps_per_split = a.plan.steps_per_split; p.splits = 1;
    p.flags = a.flags;
    p.x = a.x; p.w = a.w; p.dy = a.dy; p.ymask = nullptr; p.bias = a.bias; p.out = a.out; p.partial = a.partial;
    const int oh = fwd ? a.g.Ho : a.g.H, ow = fwd ? a.g.Wo : a.g.W;
    const int tws = halo_tws(oh, ow), tw = 1 << tws, th = HALO_TB >> tws;
    const int tiles_x = (ow + tw - 1) / tw, tiles_y = (oh + th - 1) / th;
    if (a.plan.variant == 4) {
        int blocks = a.plan.blocks > 0 ? a.plan.blocks : 256 / p.tilesA;   // default: one persistent block per CU
        if (blocks < 1) blocks = 1;
        if (blocks > p.tilesB) blocks = p.tilesB;
        void (*kern)(const KArgs, int, int, int, int) = k_halo_ws<PASS_FWD>;
        if (!fwd) {
            if (p.flags & KF_MASK_IN) kern = k_halo_ws<PASS_DGRAD, true>;
            else kern = k_halo_ws<PASS_DGRAD>;
        }
        hipLaunchKernelGGL(kern, dim3((unsigned)blocks, (unsigned)p.tilesA), dim3(256), WS_LDS, st, p,
                           tws, tiles_x, tiles_y, p.tilesB);
        dp_trace_main_kernel_done(st);
        return hipGetLastError();
    }
    const HaloVariant &h = kHalo[a.plan.variant];
    dim3 grid((unsigned)(p.tilesA * p.tilesB), 1, 1), block(64 * h.WA * h.WB, 1, 1);
    hipLaunchKernelGGL(pick_halo(a.pass, a.plan.variant), grid, block, halo_lds_bytes(h), st, p, tws, tiles_x, tiles_y);
    dp_trace_main_kernel_done(st);
    return hipGetLastError();
}
