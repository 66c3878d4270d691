// bf16 implicit-GEMM convolution kernels for gfx950 matrix cores (fp32 accumulation).
//
// One tiled kernel per pass (forward, backward-data, backward-filter).  Every pass is
// a GEMM  D[i][j] = sum_t A[i][t] * B[j][t]  whose operands are gathered from the NHWC /
// KRSC tensors on the fly (no im2col buffer in HBM):
//
//   pass    A rows (i)   B rows (j)            reduction t        D goes to
//   fwd     c_out        output pixel (n,p,q)  (r,s,c)            y [pixel][c_out]
//   dgrad   c_in         input pixel (n,h,w)   (r,s,k)            dx[pixel][c_in]
//   wgrad   c_out        filter tap (r,s,c)    output pixel       dw[c_out][tap]
//
// Both operands of v_mfma_f32_32x32x16_bf16 want 8 consecutive reduction elements per
// lane.  Where the reduction index is contiguous in memory (fwd: both; dgrad: dy) a
// 16-byte global load feeds LDS directly.  Where it is the slow index (dgrad: w; wgrad:
// both) a thread loads an 8x8 block (8 reduction rows x 16 bytes), transposes it in
// registers (only 16-bit pair swaps cost instructions) and writes 8 reduction-contiguous
// rows to LDS.  LDS tiles are [row][BK + 8] bf16: the 16-byte pad makes the 16-byte
// fragment reads of 8 consecutive rows hit distinct banks.
//
// Pipeline per reduction step: global loads of step t+1 are issued into registers, the
// matrix cores run step t out of LDS buffer t&1, registers are stored to buffer (t+1)&1,
// one barrier.  A reduction can be split across blockIdx.y; splits write fp32 partial
// tiles and a second kernel sums them in split order (deterministic) and applies the
// epilogue (bias, ReLU, bf16 rounding).
#include "dp_kernels.h"
#include <cstdio>

#include "tile_common.h"

namespace {

// ---------------------------------------------------------------------------------------
// Operand loaders.  Each owns the registers of one in-flight tile slice:
//   init(...)  once; load(step) issues global loads; store(lds) writes them to an LDS tile.
// T = tile rows, BK = reduction elements per step, NT = threads, LS = LDS row stride.
// ---------------------------------------------------------------------------------------

// Rows of a row-major [rows][red] matrix (forward weights).
template <int T, int BK, int NT, bool VEC>
struct LoadRows {
    static constexpr int LS = BK + 8;
    static constexpr int CH = BK / 8, TOT = T * CH, PER = (TOT + NT - 1) / NT;
    static constexpr int EL = (T * BK + NT - 1) / NT;
    const bf16_t *src; int red, tid, row0, rows;
    u32x4 rv[VEC ? PER : 1]; unsigned off[VEC ? PER : 1]; bool ok[VEC ? PER : 1];
    bf16_t rs[VEC ? 1 : EL];

    DEVFN void init(const bf16_t *s, int row0_, int rows_, int red_, int tid_)
    {
        src = s; red = red_; tid = tid_; row0 = row0_; rows = rows_;
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                int id = tid + i * NT, row = id / CH, ch = id % CH;
                ok[i] = id < TOT && row0 + row < rows;
                off[i] = (unsigned)(row0 + row) * (unsigned)red + ch * 8;
            }
        }
    }
    DEVFN void load(int step)
    {
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                int ch = (tid + i * NT) % CH;
                bool v = ok[i] && step * BK + ch * 8 < red;
                rv[i] = v ? ldg16(src + off[i] + step * BK) : u32x4{0, 0, 0, 0};
            }
        } else {
#pragma unroll
            for (int i = 0; i < EL; ++i) {
                int id = tid + i * NT, row = id / BK, kk = step * BK + id % BK;
                bool v = id < T * BK && row0 + row < rows && kk < red;
                rs[i] = v ? src[(size_t)(row0 + row) * red + kk] : (bf16_t)0;
            }
        }
    }
    DEVFN void store(bf16_t *lds) const
    {
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                int id = tid + i * NT, row = id / CH, ch = id % CH;
                if (id < TOT) *reinterpret_cast<u32x4 *>(lds + row * LS + ch * 8) = rv[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < EL; ++i) {
                int id = tid + i * NT;
                if (id < T * BK) lds[(id / BK) * LS + id % BK] = rs[i];
            }
        }
    }
};

// Forward im2col rows: row = output pixel, reduction = (r,s,c) with c contiguous in x.
template <int T, int BK, int NT, bool VEC>
struct LoadFwdPixels {
    static constexpr int LS = BK + 8;
    static constexpr int CH = BK / 8, TOT = T * CH, PER = (TOT + NT - 1) / NT;
    static constexpr int EL = (T * BK + NT - 1) / NT;
    const bf16_t *x; ConvGeom g; int tid, row0, M;
    u32x4 rv[VEC ? PER : 1];
    int hb[VEC ? PER : 1], wb[VEC ? PER : 1], r[VEC ? PER : 1], s[VEC ? PER : 1], c[VEC ? PER : 1];
    unsigned base[VEC ? PER : 1]; bool ok[VEC ? PER : 1];
    bf16_t rs[VEC ? 1 : EL];

    DEVFN void init(const bf16_t *x_, const ConvGeom &g_, int row0_, int M_, int kbeg, int tid_)
    {
        x = x_; g = g_; tid = tid_; row0 = row0_; M = M_;
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                int id = tid + i * NT, row = id / CH, ch = id % CH;
                int m = row0 + row;
                ok[i] = id < TOT && m < M;
                int n = m / (g.Ho * g.Wo), rem = m - n * (g.Ho * g.Wo);
                int p = rem / g.Wo, q = rem - p * g.Wo;
                hb[i] = p * g.sh - g.ph; wb[i] = q * g.sw - g.pw;
                base[i] = (unsigned)n * (unsigned)(g.H * g.W * g.C);
                int kk = kbeg * BK + ch * 8, rsi = kk / g.C;
                c[i] = kk - rsi * g.C; r[i] = rsi / g.S; s[i] = rsi - r[i] * g.S;
            }
        }
    }
    DEVFN void load(int step)
    {
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                int ih = hb[i] + r[i], iw = wb[i] + s[i];
                bool v = ok[i] && r[i] < g.R && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
                rv[i] = v ? ldg16(x + base[i] + (unsigned)((ih * g.W + iw) * g.C + c[i])) : u32x4{0, 0, 0, 0};
                c[i] += BK;
                while (c[i] >= g.C) { c[i] -= g.C; if (++s[i] == g.S) { s[i] = 0; ++r[i]; } }
            }
        } else {
#pragma unroll
            for (int i = 0; i < EL; ++i) {
                int id = tid + i * NT, row = id / BK, kk = step * BK + id % BK;
                int m = row0 + row;
                int n = m / (g.Ho * g.Wo), rem = m - n * (g.Ho * g.Wo);
                int p = rem / g.Wo, q = rem - p * g.Wo;
                int rsi = kk / g.C, cc = kk - rsi * g.C, rr = rsi / g.S, ss = rsi - rr * g.S;
                int ih = p * g.sh - g.ph + rr, iw = q * g.sw - g.pw + ss;
                bool v = id < T * BK && m < M && rr < g.R && (unsigned)ih < (unsigned)g.H &&
                         (unsigned)iw < (unsigned)g.W;
                rs[i] = v ? x[((size_t)(n * g.H + ih) * g.W + iw) * g.C + cc] : (bf16_t)0;
            }
        }
    }
    DEVFN void store(bf16_t *lds) const
    {
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                int id = tid + i * NT, row = id / CH, ch = id % CH;
                if (id < TOT) *reinterpret_cast<u32x4 *>(lds + row * LS + ch * 8) = rv[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < EL; ++i) {
                int id = tid + i * NT;
                if (id < T * BK) lds[(id / BK) * LS + id % BK] = rs[i];
            }
        }
    }
};

// Backward-data rows: row = input pixel (n,h,w), reduction = (r,s,k) with k contiguous in dy.
// dy[n,p,q,k] contributes iff p*sh - ph + r == h and q*sw - pw + s == w.
template <int T, int BK, int NT, bool VEC>
struct LoadDgradPixels {
    static constexpr int LS = BK + 8;
    static constexpr int CH = BK / 8, TOT = T * CH, PER = (TOT + NT - 1) / NT;
    static constexpr int EL = (T * BK + NT - 1) / NT;
    const bf16_t *dy, *ym; ConvGeom g; int tid, row0, M;
    u32x4 rv[VEC ? PER : 1];
    int hb[VEC ? PER : 1], wb[VEC ? PER : 1], r[VEC ? PER : 1], s[VEC ? PER : 1], k[VEC ? PER : 1];
    unsigned base[VEC ? PER : 1]; bool ok[VEC ? PER : 1];
    bf16_t rs[VEC ? 1 : EL];

    DEVFN void init(const bf16_t *dy_, const bf16_t *ym_, const ConvGeom &g_, int row0_, int M_, int kbeg, int tid_)
    {
        dy = dy_; ym = ym_; g = g_; tid = tid_; row0 = row0_; M = M_;
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                int id = tid + i * NT, row = id / CH, ch = id % CH;
                int m = row0 + row;
                ok[i] = id < TOT && m < M;
                int n = m / (g.H * g.W), rem = m - n * (g.H * g.W);
                int h = rem / g.W, w = rem - h * g.W;
                hb[i] = h + g.ph; wb[i] = w + g.pw;
                base[i] = (unsigned)n * (unsigned)(g.Ho * g.Wo * g.K);
                int kk = kbeg * BK + ch * 8, rsi = kk / g.K;
                k[i] = kk - rsi * g.K; r[i] = rsi / g.S; s[i] = rsi - r[i] * g.S;
            }
        }
    }
    DEVFN bool locate(int hbv, int wbv, int rr, int ss, int &p, int &q) const
    {
        int hp = hbv - rr, wq = wbv - ss;
        if (rr >= g.R || hp < 0 || wq < 0) return false;
        if (g.sh == 1) p = hp; else { p = hp / g.sh; if (p * g.sh != hp) return false; }
        if (g.sw == 1) q = wq; else { q = wq / g.sw; if (q * g.sw != wq) return false; }
        return p < g.Ho && q < g.Wo;
    }
    DEVFN void load(int step)
    {
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                int p = 0, q = 0;
                bool v = ok[i] && locate(hb[i], wb[i], r[i], s[i], p, q);
                unsigned a = base[i] + (unsigned)((p * g.Wo + q) * g.K + k[i]);
                u32x4 val = v ? ldg16(dy + a) : u32x4{0, 0, 0, 0};
                if (ym != nullptr && v) val = apply_mask(val, ldg16(ym + a));
                rv[i] = val;
                k[i] += BK;
                while (k[i] >= g.K) { k[i] -= g.K; if (++s[i] == g.S) { s[i] = 0; ++r[i]; } }
            }
        } else {
#pragma unroll
            for (int i = 0; i < EL; ++i) {
                int id = tid + i * NT, row = id / BK, kk = step * BK + id % BK;
                int m = row0 + row;
                int n = m / (g.H * g.W), rem = m - n * (g.H * g.W);
                int h = rem / g.W, w = rem - h * g.W;
                int rsi = kk / g.K, kc = kk - rsi * g.K, rr = rsi / g.S, ss = rsi - rr * g.S;
                int p = 0, q = 0;
                bool v = id < T * BK && m < M && locate(h + g.ph, w + g.pw, rr, ss, p, q);
                size_t a = ((size_t)(n * g.Ho + p) * g.Wo + q) * g.K + kc;
                bf16_t val = v ? dy[a] : (bf16_t)0;
                if (ym != nullptr && v) val = mask1(val, ym[a]);
                rs[i] = val;
            }
        }
    }
    DEVFN void store(bf16_t *lds) const
    {
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                int id = tid + i * NT, row = id / CH, ch = id % CH;
                if (id < TOT) *reinterpret_cast<u32x4 *>(lds + row * LS + ch * 8) = rv[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < EL; ++i) {
                int id = tid + i * NT;
                if (id < T * BK) lds[(id / BK) * LS + id % BK] = rs[i];
            }
        }
    }
};

// 8x8 register transpose: in[t] holds 8 bf16 (columns 0..7) of reduction row t; out[c]
// holds reduction rows 0..7 of column c.  Only 16-bit pair swaps are instructions.
DEVFN void transpose8x8(const u32x4 (&in)[8], u32x4 (&out)[8])
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        unsigned e[4], o[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            unsigned a = in[2 * t][j], b = in[2 * t + 1][j];
            e[t] = (a & 0xffffu) | (b << 16);
            o[t] = (a >> 16) | (b & 0xffff0000u);
        }
        out[2 * j] = u32x4{e[0], e[1], e[2], e[3]};
        out[2 * j + 1] = u32x4{o[0], o[1], o[2], o[3]};
    }
}

// Transposing loader.  Unit = 8 operand rows (contiguous in memory, "columns") x 8 reduction
// rows.  KIND selects how a (reduction index, operand row) pair maps to memory:
//   0  backward-data weights : operand row c, reduction (r,s,k)   -> w[k][r][s][c]
//   1  backward-filter dy    : operand row k, reduction pixel m   -> dy[m][k] (masked by ymask)
//   2  backward-filter x     : operand row (r,s,c), reduction pixel m=(n,p,q)
//                                                         -> x[n][p*sh-ph+r][q*sw-pw+s][c]
// Lane bits 0..2 pick the reduction chunk, higher bits the operand-row chunk, so one load
// instruction of a wavefront touches 8 memory rows x 128 contiguous bytes and the eight
// lanes of a group write one contiguous 128-byte LDS row segment.
template <int T, int BK, int NT, bool VEC, int KIND>
struct LoadTransposed {
    static constexpr int LS = BK + 8;
    static constexpr int TCH = BK / 8, UNITS = (T / 8) * TCH, PER = (UNITS + NT - 1) / NT;
    static constexpr int EL = (T * BK + NT - 1) / NT;
    const bf16_t *src, *ym; ConvGeom g; int tid, row0, rows, red_end;
    u32x4 rv[VEC ? PER : 1][8];
    bf16_t rs[VEC ? 1 : EL];
    // per-unit state
    int a0[VEC ? PER : 1], a1[VEC ? PER : 1], a2[VEC ? PER : 1];  // KIND 0: r,s,k   KIND 2: n,p,q of first row
    int tr[VEC ? PER : 1], ts[VEC ? PER : 1];                        // KIND 2: tap r,s of the column chunk
    unsigned cofs[VEC ? PER : 1];                                    // column offset inside a memory row
    int t0[VEC ? PER : 1];                                           // KIND 1/2: first reduction index
    bool ok[VEC ? PER : 1];

    DEVFN void init(const bf16_t *src_, const bf16_t *ym_, const ConvGeom &g_, int row0_, int rows_,
                    int kbeg, int red_end_, int tid_)
    {
        src = src_; ym = ym_; g = g_; tid = tid_; row0 = row0_; rows = rows_; red_end = red_end_;
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                int u = tid + i * NT, tch = u % TCH, cch = u / TCH;
                int col = row0 + cch * 8;
                ok[i] = u < UNITS && col < rows;
                int t = kbeg * BK + tch * 8;
                t0[i] = t;
                if constexpr (KIND == 0) {
                    int rsi = t / g.K;
                    a2[i] = t - rsi * g.K; a0[i] = rsi / g.S; a1[i] = rsi - a0[i] * g.S;
                    cofs[i] = col;
                } else if constexpr (KIND == 1) {
                    cofs[i] = col;
                } else {
                    int rsi = col / g.C;
                    cofs[i] = col - rsi * g.C; tr[i] = rsi / g.S; ts[i] = rsi - tr[i] * g.S;
                    int n = t / (g.Ho * g.Wo), rem = t - n * (g.Ho * g.Wo);
                    a0[i] = n; a1[i] = rem / g.Wo; a2[i] = rem - a1[i] * g.Wo;
                }
            }
        }
    }
    DEVFN void load(int step)
    {
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                if constexpr (KIND == 0) {
                    bool v = ok[i] && a0[i] < g.R;
                    unsigned a = (unsigned)(((a2[i] * g.R + a0[i]) * g.S + a1[i]) * g.C) + cofs[i];
                    unsigned pitch = (unsigned)(g.R * g.S * g.C);
#pragma unroll
                    for (int t = 0; t < 8; ++t) rv[i][t] = v ? ldg16(src + a + t * pitch) : u32x4{0, 0, 0, 0};
                    a2[i] += BK;
                    while (a2[i] >= g.K) { a2[i] -= g.K; if (++a1[i] == g.S) { a1[i] = 0; ++a0[i]; } }
                } else if constexpr (KIND == 1) {
                    const int m = t0[i];
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        bool v = ok[i] && m + t < red_end;
                        unsigned a = (unsigned)(m + t) * (unsigned)g.K + cofs[i];
                        u32x4 val = v ? ldg16(src + a) : u32x4{0, 0, 0, 0};
                        if (ym != nullptr && v) val = apply_mask(val, ldg16(ym + a));
                        rv[i][t] = val;
                    }
                    t0[i] += BK;
                } else {
                    int n = a0[i], p = a1[i], q = a2[i], m = t0[i];
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        int ih = p * g.sh - g.ph + tr[i], iw = q * g.sw - g.pw + ts[i];
                        bool v = ok[i] && m + t < red_end && (unsigned)ih < (unsigned)g.H &&
                                 (unsigned)iw < (unsigned)g.W;
                        unsigned a = (unsigned)(((n * g.H + ih) * g.W + iw) * g.C) + cofs[i];
                        rv[i][t] = v ? ldg16(src + a) : u32x4{0, 0, 0, 0};
                        if (++q == g.Wo) { q = 0; if (++p == g.Ho) { p = 0; ++n; } }
                    }
                    t0[i] += BK;
                    a2[i] += BK;
                    while (a2[i] >= g.Wo) { a2[i] -= g.Wo; if (++a1[i] == g.Ho) { a1[i] = 0; ++a0[i]; } }
                }
            }
        } else {
            // element-wise fallback: operand row fastest across threads
#pragma unroll
            for (int i = 0; i < EL; ++i) {
                int id = tid + i * NT, colr = id % T, tt = id / T;
                int col = row0 + colr, t = step * BK + tt;
                bool v = id < T * BK && col < rows;
                bf16_t val = 0;
                if constexpr (KIND == 0) {
                    int rsi = t / g.K, kc = t - rsi * g.K, rr = rsi / g.S, ss = rsi - rr * g.S;
                    if (v && rr < g.R) val = src[((size_t)(kc * g.R + rr) * g.S + ss) * g.C + col];
                } else if constexpr (KIND == 1) {
                    if (v && t < red_end) {
                        size_t a = (size_t)t * g.K + col;
                        val = src[a];
                        if (ym != nullptr) val = mask1(val, ym[a]);
                    }
                } else {
                    if (v && t < red_end) {
                        int rsi = col / g.C, cc = col - rsi * g.C, rr = rsi / g.S, ss = rsi - rr * g.S;
                        int n = t / (g.Ho * g.Wo), rem = t - n * (g.Ho * g.Wo);
                        int p = rem / g.Wo, q = rem - p * g.Wo;
                        int ih = p * g.sh - g.ph + rr, iw = q * g.sw - g.pw + ss;
                        if ((unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W)
                            val = src[((size_t)(n * g.H + ih) * g.W + iw) * g.C + cc];
                    }
                }
                rs[i] = val;
            }
        }
    }
    DEVFN void store(bf16_t *lds) const
    {
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                int u = tid + i * NT, tch = u % TCH, cch = u / TCH;
                if (u < UNITS) {
                    u32x4 o[8];
                    transpose8x8(rv[i], o);
#pragma unroll
                    for (int cidx = 0; cidx < 8; ++cidx)
                        *reinterpret_cast<u32x4 *>(lds + (cch * 8 + cidx) * LS + tch * 8) = o[cidx];
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < EL; ++i) {
                int id = tid + i * NT;
                if (id < T * BK) lds[(id % T) * LS + id / T] = rs[i];
            }
        }
    }
};

// ---------------------------------------------------------------------------------------
// The tiled kernel.  PASS picks loaders and epilogue.
// ---------------------------------------------------------------------------------------
template <int PASS, int TA, int TB, int BK, int WA, int WB, bool VA, bool VB>
__global__ __launch_bounds__(64 * WA * WB) void k_conv_gemm(const KArgs p)
{
    constexpr int NT = 64 * WA * WB, LS = BK + 8;
    constexpr int FA = TA / WA / 32, FB = TB / WB / 32;
    static_assert(FA >= 1 && FB >= 1, "wave tile must hold at least one 32x32 block");
    extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
    bf16_t *As = lds;                   // [2][TA][LS]
    bf16_t *Bs = lds + 2 * TA * LS;     // [2][TB][LS]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tile = logical_block(blockIdx.x, gridDim.x);
    const int ta = tile % p.tilesA, tb = tile / p.tilesA;
    const int split = blockIdx.y;
    const int a0 = ta * TA, b0 = tb * TB;
    const int kbeg = split * p.steps_per_split;
    const int kend = min(kbeg + p.steps_per_split, p.steps_total);

    f32x16 acc[FA][FB];
#pragma unroll
    for (int i = 0; i < FA; ++i)
#pragma unroll
        for (int j = 0; j < FB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int arow = (wave % WA) * FA * 32, brow = (wave / WA) * FB * 32;

    auto run = [&](auto &la, auto &lb) {
        if (kbeg < kend) {
            la.load(kbeg); lb.load(kbeg);
            la.store(As); lb.store(Bs);
            __syncthreads();
            for (int step = kbeg; step < kend; ++step) {
                const int buf = (step - kbeg) & 1;
                const bool more = step + 1 < kend;
                if (more) { la.load(step + 1); lb.load(step + 1); }
                mma_step<FA, FB, BK>(As + buf * TA * LS, Bs + buf * TB * LS, arow, brow, lane, acc);
                if (more) { la.store(As + (buf ^ 1) * TA * LS); lb.store(Bs + (buf ^ 1) * TB * LS); }
                __syncthreads();
            }
        }
    };

    if constexpr (PASS == PASS_FWD) {
        LoadRows<TA, BK, NT, VA> la;
        LoadFwdPixels<TB, BK, NT, VB> lb;
        la.init(p.w, a0, p.rowsA, p.red, tid);
        lb.init(p.x, p.g, b0, p.rowsB, kbeg, tid);
        run(la, lb);
        store_pixel_major<FA, FB>(p, acc, a0 + arow, b0 + brow, lane, split);
    } else if constexpr (PASS == PASS_DGRAD) {
        LoadTransposed<TA, BK, NT, VA, 0> la;
        LoadDgradPixels<TB, BK, NT, VB> lb;
        la.init(p.w, nullptr, p.g, a0, p.rowsA, kbeg, p.red, tid);
        lb.init(p.dy, p.ymask, p.g, b0, p.rowsB, kbeg, tid);
        run(la, lb);
        store_pixel_major<FA, FB>(p, acc, a0 + arow, b0 + brow, lane, split);
    } else {
        LoadTransposed<TA, BK, NT, VA, 1> la;
        LoadTransposed<TB, BK, NT, VB, 2> lb;
        la.init(p.dy, p.ymask, p.g, a0, p.rowsA, kbeg, p.red, tid);
        // when each operand needs at most half of the threads, give the other half to B
        constexpr bool kSplitThreads = VA && VB && decltype(la)::UNITS <= NT / 2 && decltype(lb)::UNITS <= NT / 2;
        lb.init(p.x, nullptr, p.g, b0, p.rowsB, kbeg, p.red, kSplitThreads ? (tid + NT / 2) % NT : tid);
        run(la, lb);
        store_row_major<FA, FB>(p, acc, a0 + arow, b0 + brow, lane, split);
    }
}

// Sum split partials in split order and apply the epilogue.
// pixel-major ([rowsB][rowsA], bias per A row) for fwd / dgrad.
__global__ __launch_bounds__(256) void k_reduce_pixel_major(const KArgs p)
{
    const size_t total = (size_t)p.rowsB * p.rowsA;
    const size_t gstride = (size_t)gridDim.x * blockDim.x;
    if ((p.rowsA & 3) == 0) {
        for (size_t e = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4; e < total; e += gstride * 4) {
            f32x4 s = *reinterpret_cast<const f32x4 *>(p.partial + e);
            for (int sp = 1; sp < p.splits; ++sp) s += *reinterpret_cast<const f32x4 *>(p.partial + sp * total + e);
            float v[4] = {s.x, s.y, s.z, s.w};
            const int ch = (int)(e % p.rowsA);
            if (p.flags & KF_BIAS) for (int i = 0; i < 4; ++i) v[i] += p.bias[ch + i];
            if (p.flags & KF_RELU) for (int i = 0; i < 4; ++i) v[i] = v[i] > 0.f ? v[i] : 0.f;
            if (p.flags & KF_MASK_IN) for (int i = 0; i < 4; ++i) v[i] = mask1f(v[i], p.x[e + i]);
            if (p.flags & KF_OUT_F32)
                *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(p.out) + e) = f32x4{v[0], v[1], v[2], v[3]};
            else
                *reinterpret_cast<u32x2 *>(reinterpret_cast<bf16_t *>(p.out) + e) =
                    u32x2{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        }
    } else {
        for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += gstride) {
            float v = p.partial[e];
            for (int sp = 1; sp < p.splits; ++sp) v += p.partial[sp * total + e];
            if (p.flags & KF_BIAS) v += p.bias[e % p.rowsA];
            if (p.flags & KF_RELU) v = v > 0.f ? v : 0.f;
            if (p.flags & KF_MASK_IN) v = mask1f(v, p.x[e]);
            if (p.flags & KF_OUT_F32) reinterpret_cast<float *>(p.out)[e] = v;
            else reinterpret_cast<bf16_t *>(p.out)[e] = (bf16_t)f32_to_bf16(v);
        }
    }
}

// Blocks nb1 .. gridDim.x-1 of the two backward-filter reductions sum a second, small array in a fixed order (the
// bias gradient: partial2 [rows][total2] -> out2 [total2]; up to 512 rows).  A block takes 32 columns: 8 threads per
// column each add every 8th row with four independent sums in flight, the 8 part sums meet in LDS in order.
DEVFN void reduce_second(int blk, const float *partial2, float *out2, int total2, int rows)
{
    __shared__ float sm2[8][32];
    const int cl = threadIdx.x & 31, part = threadIdx.x >> 5;
    const int col = blk * 32 + cl;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (col < total2) {
        int b = part;
        for (; b + 24 < rows; b += 32) {
            s0 += partial2[(size_t)b * total2 + col];
            s1 += partial2[(size_t)(b + 8) * total2 + col];
            s2 += partial2[(size_t)(b + 16) * total2 + col];
            s3 += partial2[(size_t)(b + 24) * total2 + col];
        }
        for (; b < rows; b += 8) s0 += partial2[(size_t)b * total2 + col];
    }
    sm2[part][cl] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (part == 0 && col < total2) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) s += sm2[i][cl];
        out2[col] = s;
    }
}

__global__ __launch_bounds__(256) void k_reduce_flat(const float *partial, float *out, size_t total, int splits, int nb1,
                                                      const float *partial2, float *out2, int total2, int rows2)
{
    if ((int)blockIdx.x >= nb1) { reduce_second(blockIdx.x - nb1, partial2, out2, total2, rows2); return; }
    const size_t gstride = (size_t)nb1 * blockDim.x;
    if ((total & 3) == 0) {
        for (size_t e = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4; e < total; e += gstride * 4) {
            // four independent loads in flight; the sum order is fixed by the code, not by timing
            f32x4 s0 = *reinterpret_cast<const f32x4 *>(partial + e), s1 = {0, 0, 0, 0}, s2 = {0, 0, 0, 0}, s3 = {0, 0, 0, 0};
            int sp = 1;
            for (; sp + 3 < splits; sp += 4) {
                s1 += *reinterpret_cast<const f32x4 *>(partial + (size_t)sp * total + e);
                s2 += *reinterpret_cast<const f32x4 *>(partial + (size_t)(sp + 1) * total + e);
                s3 += *reinterpret_cast<const f32x4 *>(partial + (size_t)(sp + 2) * total + e);
                s0 += *reinterpret_cast<const f32x4 *>(partial + (size_t)(sp + 3) * total + e);
            }
            for (; sp < splits; ++sp) s1 += *reinterpret_cast<const f32x4 *>(partial + (size_t)sp * total + e);
            *reinterpret_cast<f32x4 *>(out + e) = (s0 + s1) + (s2 + s3);
        }
    } else {
        for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += gstride) {
            float v = partial[e];
            for (int sp = 1; sp < splits; ++sp) v += partial[sp * total + e];
            out[e] = v;
        }
    }
}

// Many splits over a small output (long reductions into a small filter): 8 threads share one group
// of four outputs, each sums every 8th partial, the 8 part sums are combined through LDS in order.
__global__ __launch_bounds__(256) void k_reduce_flat_wide(const float *partial, float *out, size_t total, int splits, int nb1,
                                                           const float *partial2, float *out2, int total2, int rows2)
{
    if ((int)blockIdx.x >= nb1) { reduce_second(blockIdx.x - nb1, partial2, out2, total2, rows2); return; }
    __shared__ f32x4 sm[8][32];
    const int g = threadIdx.x & 31, part = threadIdx.x >> 5;
    const size_t e = ((size_t)blockIdx.x * 32 + g) * 4;
    f32x4 s0 = {0, 0, 0, 0}, s1 = {0, 0, 0, 0};
    if (e < total) {
        int sp = part;
        for (; sp + 8 < splits; sp += 16) {
            s0 += *reinterpret_cast<const f32x4 *>(partial + (size_t)sp * total + e);
            s1 += *reinterpret_cast<const f32x4 *>(partial + (size_t)(sp + 8) * total + e);
        }
        for (; sp < splits; sp += 8) s0 += *reinterpret_cast<const f32x4 *>(partial + (size_t)sp * total + e);
    }
    sm[part][g] = s0 + s1;
    __syncthreads();
    if (part == 0 && e < total) {
        f32x4 s = sm[0][g];
#pragma unroll
        for (int i = 1; i < 8; ++i) s += sm[i][g];
        *reinterpret_cast<f32x4 *>(out + e) = s;
    }
}

// ---------------------------------------------------------------------------------------
// Tile variants and dispatch
// ---------------------------------------------------------------------------------------
struct Variant { int TA, TB, WA, WB; };
// index:                 0               1              2              3              4
const Variant kVariants[] = {{128, 128, 2, 2}, {64, 64, 2, 2}, {128, 32, 4, 1}, {64, 128, 2, 2}, {32, 128, 1, 4}};
constexpr int kNumVariants = 5;
constexpr int BK_FWD = 32, BK_WGRAD = 64;

int bk_of(int pass) { return pass == PASS_WGRAD ? BK_WGRAD : BK_FWD; }
size_t lds_bytes(int TA, int TB, int BK) { return (size_t)2 * (TA + TB) * (BK + 8) * sizeof(bf16_t); }

typedef void (*KernelFn)(const KArgs);

template <int PASS, int BK, bool VA, bool VB>
KernelFn pick_variant(int v)
{
    switch (v) {
    case 0: return k_conv_gemm<PASS, 128, 128, BK, 2, 2, VA, VB>;
    case 1: return k_conv_gemm<PASS, 64, 64, BK, 2, 2, VA, VB>;
    case 2: return k_conv_gemm<PASS, 128, 32, BK, 4, 1, VA, VB>;
    case 3: return k_conv_gemm<PASS, 64, 128, BK, 2, 2, VA, VB>;
    default: return k_conv_gemm<PASS, 32, 128, BK, 1, 4, VA, VB>;
    }
}

KernelFn pick_kernel(int pass, int v, bool va, bool vb)
{
    if (pass == PASS_FWD) {
        return (va && vb) ? pick_variant<PASS_FWD, BK_FWD, true, true>(v) : pick_variant<PASS_FWD, BK_FWD, false, false>(v);
    } else if (pass == PASS_DGRAD) {
        return (va && vb) ? pick_variant<PASS_DGRAD, BK_FWD, true, true>(v) : pick_variant<PASS_DGRAD, BK_FWD, false, false>(v);
    } else {
        if (va && vb) return pick_variant<PASS_WGRAD, BK_WGRAD, true, true>(v);
        if (va) return pick_variant<PASS_WGRAD, BK_WGRAD, true, false>(v);
        return pick_variant<PASS_WGRAD, BK_WGRAD, false, false>(v);
    }
}

void gemm_extents(const ConvGeom &g, int pass, int *rowsA, int *rowsB, int *red)
{
    if (pass == PASS_FWD) { *rowsA = g.K; *rowsB = g.N * g.Ho * g.Wo; *red = g.R * g.S * g.C; }
    else if (pass == PASS_DGRAD) { *rowsA = g.C; *rowsB = g.N * g.H * g.W; *red = g.R * g.S * g.K; }
    else { *rowsA = g.K; *rowsB = g.R * g.S * g.C; *red = g.N * g.Ho * g.Wo; }
}

}  // namespace

hipError_t mfma_init()
{
    for (int pass = 0; pass < 3; ++pass)
        for (int v = 0; v < kNumVariants; ++v)
            for (int va = 0; va < 2; ++va)
                for (int vb = 0; vb < 2; ++vb) {
                    KernelFn fn = pick_kernel(pass, v, va, vb);
                    size_t bytes = lds_bytes(kVariants[v].TA, kVariants[v].TB, bk_of(pass));
                    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
                    if (e != hipSuccess) return e;
                }
    return hipSuccess;
}

void mfma_plan(const ConvGeom &g, int pass, int force_variant, int force_splits, GemmPlan *pl)
{
    int rowsA, rowsB, red;
    gemm_extents(g, pass, &rowsA, &rowsB, &red);
    // operand vectorisation: 16-byte chunks must not straddle rows / taps and must be aligned
    bool c8 = (g.C % 8) == 0, k8 = (g.K % 8) == 0;
    if (pass == PASS_FWD) { pl->vecA = pl->vecB = c8; }
    else if (pass == PASS_DGRAD) { pl->vecA = pl->vecB = c8 && k8; }
    else { pl->vecA = k8; pl->vecB = k8 && c8; }

    int v;
    if (force_variant >= 0 && force_variant < kNumVariants) v = force_variant;
    else {
        // built-in choice: widest tile that still gives the chip enough blocks
        if (rowsA <= 32) v = 4;
        else if (rowsA <= 64) v = 3;
        else if (rowsB <= 32) v = 2;
        else {
            long long big = (long long)((rowsA + 127) / 128) * ((rowsB + 127) / 128);
            v = big >= 192 ? 0 : 1;
        }
    }
    const Variant &tv = kVariants[v];
    pl->fast = false; pl->dma = false;
    pl->variant = v; pl->TA = tv.TA; pl->TB = tv.TB; pl->BK = bk_of(pass);
    pl->tilesA = (rowsA + tv.TA - 1) / tv.TA;
    pl->tilesB = (rowsB + tv.TB - 1) / tv.TB;
    pl->steps_total = (red + pl->BK - 1) / pl->BK;
    long long tiles = (long long)pl->tilesA * pl->tilesB;
    int splits;
    if (force_splits > 0) splits = force_splits;
    else {
        const long long target = 512;  // two blocks per CU
        splits = tiles >= target ? 1 : (int)((target + tiles - 1) / tiles);
        int min_steps = pass == PASS_WGRAD ? 4 : 8;
        int max_splits = pl->steps_total / min_steps;
        if (max_splits < 1) max_splits = 1;
        if (splits > max_splits) splits = max_splits;
    }
    if (splits > pl->steps_total) splits = pl->steps_total;
    if (splits < 1) splits = 1;
    pl->steps_per_split = (pl->steps_total + splits - 1) / splits;
    pl->splits = (pl->steps_total + pl->steps_per_split - 1) / pl->steps_per_split;
}

size_t mfma_partial_bytes(const ConvGeom &g, int pass, const GemmPlan &pl)
{
    if (pl.splits <= 1) return 0;
    int rowsA, rowsB, red;
    gemm_extents(g, pass, &rowsA, &rowsB, &red);
    return (size_t)pl.splits * rowsA * rowsB * sizeof(float);
}

void mfma_kernel_name(int pass, const GemmPlan &pl, char *name, size_t name_bytes)
{
    const Variant &tv = kVariants[pl.variant];
    bool va = pl.vecA, vb = pl.vecB;
    if (pass != PASS_WGRAD) va = vb = (pl.vecA && pl.vecB);
    else if (!va) vb = false;
    snprintf(name, name_bytes, "k_conv_gemm<%d, %d, %d, %d, %d, %d, %s, %s>", pass, tv.TA, tv.TB, pl.BK, tv.WA, tv.WB,
             va ? "true" : "false", vb ? "true" : "false");
}

hipError_t mfma_launch(const ConvArgs &a, hipStream_t st)
{
    KArgs p;
    p.g = a.g;
    gemm_extents(a.g, a.pass, &p.rowsA, &p.rowsB, &p.red);
    p.tilesA = a.plan.tilesA; p.tilesB = a.plan.tilesB;
    p.steps_total = a.plan.steps_total; p.steps_per_split = a.plan.steps_per_split; p.splits = a.plan.splits;
    p.flags = a.flags;
    p.x = a.x; p.w = a.w; p.dy = a.dy; p.ymask = a.ymask; p.bias = a.bias; p.out = a.out; p.partial = a.partial;

    const Variant &tv = kVariants[a.plan.variant];
    KernelFn fn = pick_kernel(a.pass, a.plan.variant, a.plan.vecA, a.plan.vecB);
    dim3 grid((unsigned)(p.tilesA * p.tilesB), (unsigned)p.splits, 1), block(64 * tv.WA * tv.WB, 1, 1);
    size_t shmem = lds_bytes(tv.TA, tv.TB, a.plan.BK);
    hipLaunchKernelGGL(fn, grid, block, shmem, st, p);
    dp_trace_main_kernel_done(st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.splits > 1) e = launch_split_reduce(a, p.rowsA, p.rowsB, st);
    return e;
}

hipError_t launch_split_reduce(const ConvArgs &a, int rowsA, int rowsB, hipStream_t st, bool with_db)
{
    KArgs p{};
    p.rowsA = rowsA; p.rowsB = rowsB; p.splits = a.plan.splits; p.flags = a.flags;
    p.bias = a.bias; p.out = a.out; p.partial = a.partial; p.x = a.x;
    size_t total = (size_t)rowsA * rowsB;
    size_t work = (total + 3) / 4;
    unsigned nb = (unsigned)((work + 255) / 256);
    if (nb > 4096) nb = 4096;
    if (nb < 1) nb = 1;
    if (a.pass == PASS_WGRAD) {
        // the second array: bias-gradient sums of the main kernel's splits (with_db), or the row-block sums a pointwise
        // pass left there before the main kernel (db_rows)
        const bool db = (with_db || a.db_rows > 0) && a.db_partial != nullptr && a.db_out != nullptr;
        const unsigned nb2 = db ? (unsigned)((rowsA + 31) / 32) : 0u;
        const int rows2 = a.db_rows > 0 ? a.db_rows : p.splits;
        if ((total & 3) == 0 && p.splits >= 16 && work <= 65536) {
            const unsigned nbw = (unsigned)((work + 31) / 32);
            hipLaunchKernelGGL(k_reduce_flat_wide, dim3(nbw + nb2), dim3(256), 0, st, p.partial, reinterpret_cast<float *>(p.out), total, p.splits,
                               (int)nbw, a.db_partial, a.db_out, rowsA, rows2);
        } else
            hipLaunchKernelGGL(k_reduce_flat, dim3(nb + nb2), dim3(256), 0, st, p.partial, reinterpret_cast<float *>(p.out), total, p.splits, (int)nb,
                               a.db_partial, a.db_out, rowsA, rows2);
    } else
        hipLaunchKernelGGL(k_reduce_pixel_major, dim3(nb), dim3(256), 0, st, p);
    return hipGetLastError();
}
