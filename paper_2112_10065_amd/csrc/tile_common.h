// Shared device helpers of the tiled convolution kernels: vector types, bf16 rounding,
// XCD-aware block order, the matrix-core step on LDS tiles and the two epilogues.
#pragma once
#include "dp_kernels.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;

#define DEVFN __device__ __forceinline__

namespace {

struct KArgs {
    ConvGeom g;
    int rowsA, rowsB, red;  // GEMM extents
    int tilesA, tilesB, steps_total, steps_per_split, splits;
    unsigned flags;
    const bf16_t *x, *w, *dy, *ymask;
    const float *bias;
    void *out;
    float *partial;
    float *dbp;   // KF_DB: bias-gradient sums of split s go to dbp[s * rowsA + row]
    unsigned *tickets;   // KF_FUSED_REDUCE: one arrival counter per tile, zero before and after the launch
    // strided backward-data by phase: the B rows (input pixels) are enumerated phase by phase, phase (a, b) = (h % sh,
    // w % sw), each padded to whole tiles; B tiles ph_tile0[c] .. ph_tile0[c+1]-1 belong to phase c = a*sw + b
    int ph_on;
    int ph_tile0[5];
};

DEVFN u32x4 ldg16(const bf16_t *p) { return *reinterpret_cast<const u32x4 *>(p); }

// bits of a 32-bit word (two bf16) to keep where the matching saved output is > 0
DEVFN unsigned keep_bits(unsigned yw)
{
    unsigned lo = (((yw & 0xffffu) - 1u) < 0x7f80u) ? 0xffffu : 0u;   // +finite or +inf, nonzero
    unsigned hi = (((yw >> 16) - 1u) < 0x7f80u) ? 0xffff0000u : 0u;
    return lo | hi;
}
DEVFN u32x4 apply_mask(u32x4 v, u32x4 y)
{
    v.x &= keep_bits(y.x); v.y &= keep_bits(y.y); v.z &= keep_bits(y.z); v.w &= keep_bits(y.w);
    return v;
}
// Bias gradient through the matrix cores: multiplying a dy^T fragment (32 c_out x 16 pixels) with an all-ones
// operand sums its pixels; every column of the result holds the same 32 sums.
DEVFN bf16x8 ones_bf16() { return __builtin_bit_cast(bf16x8, u32x4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u}); }
// lanes 0 and 32 hold column 0: element v is row 8*(v/4) + 4*(lane/32) + v%4 of the fragment
DEVFN void store_db_fragment(const f32x16 &acc, float *dst, int row0, int rows, int lane)
{
    if ((lane & 31) != 0) return;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = row0 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (row < rows) dst[row] = acc[v];
    }
}
// The same sums at half the cost: a 32 x 16 fragment as it sits in a lane's registers (row l%32, reduction elements
// 8*(l/32) .. +7) IS a valid first operand of the 16x16x32 instruction, which reads lane l as row l%16, reduction group l/16:
// groups 0 and 2 then hold rows 0-15 of the fragment, groups 1 and 3 rows 16-31.  Against a second operand whose column 0
// is one in groups 0 and 2 and whose column 1 is one in groups 1 and 3 (zero elsewhere), column 0 of the result holds the sums
// of rows 0-15 and column 1 those of rows 16-31.  Four accumulator registers, four passes.
DEVFN bf16x8 colsum_selector(int lane)
{
    const int n = lane & 15, grp = lane >> 4;
    const unsigned one = ((n == 0 && (grp & 1) == 0) || (n == 1 && (grp & 1) == 1)) ? 0x3f803f80u : 0u;
    return __builtin_bit_cast(bf16x8, u32x4{one, one, one, one});
}
// result register v of lane l is row 4*(l/16) + v, column l%16: the lanes of columns 0 and 1 store
DEVFN void store_colsum_fragment(const f32x4 &acc, float *dst, int row0, int rows, int lane)
{
    if ((lane & 15) > 1) return;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int row = row0 + 16 * (lane & 15) + 4 * (lane >> 4) + v;
        if (row < rows) dst[row] = acc[v];
    }
}
DEVFN float mask1f(float v, bf16_t y) { return ((unsigned)(y - 1u) & 0xffffu) < 0x7f80u ? v : 0.f; }
DEVFN bf16_t mask1(bf16_t v, bf16_t y) { return ((unsigned)(y - 1u) & 0xffffu) < 0x7f80u ? v : (bf16_t)0; }

// fp32 -> bf16, round to nearest even, NaN stays NaN: the gfx950 conversion instruction
// (v_cvt_pk_bf16_f32), which the compiler emits for these casts
DEVFN unsigned f32_to_bf16(float f) { return __builtin_bit_cast(unsigned short, (__bf16)f); }
DEVFN unsigned pack_bf16(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}

// XCD-aware block order: hardware deals consecutive block ids round-robin to the 8 XCDs
// (each with its own L2); give every XCD one contiguous range of logical tiles.
DEVFN int logical_block(int bid, int nb)
{
    const int xcd = bid & 7, idx = bid >> 3;
    const int per = (nb + 7) >> 3, rem = nb & 7;
    if (rem == 0) return xcd * per + idx;
    return (xcd < rem ? xcd * per : rem * per + (xcd - rem) * (per - 1)) + idx;
}

// ---------------------------------------------------------------------------------------
// Matrix-core step on one pair of LDS tiles.  Lane l supplies row (l & 31) and the 8
// reduction elements starting at 8*(l >> 5) of each 16-wide slice, for both operands.
// ---------------------------------------------------------------------------------------
template <int FA, int FB, int BK>
DEVFN void mma_step(const bf16_t *As, const bf16_t *Bs, int arow, int brow, int lane, f32x16 (&acc)[FA][FB])
{
    constexpr int LS = BK + 8;
    const int lr = lane & 31, lk = (lane >> 5) * 8;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
        bf16x8 a[FA], b[FB];
#pragma unroll
        for (int i = 0; i < FA; ++i)
            a[i] = *reinterpret_cast<const bf16x8 *>(As + (arow + i * 32 + lr) * LS + ks * 16 + lk);
#pragma unroll
        for (int j = 0; j < FB; ++j)
            b[j] = *reinterpret_cast<const bf16x8 *>(Bs + (brow + j * 32 + lr) * LS + ks * 16 + lk);
#pragma unroll
        for (int i = 0; i < FA; ++i)
#pragma unroll
            for (int j = 0; j < FB; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
}

// Accumulator element v of lane l belongs to D row 8*(v/4) + 4*(l>>5) + v%4, column l&31.

// A 16-byte store written through to memory at device scope: blocks on other compute dies (each die has an L2 of its
// own) read it with device-scope loads, and neither side has to write back or invalidate a whole cache.
DEVFN void store_f32x4_device_scope(float *dst, f32x4 v) { asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(dst), "v"(v) : "memory"); }

// Epilogue for fwd / dgrad: out[j][i] (pixel-major, channel contiguous).
template <int FA, int FB>
DEVFN void store_pixel_major(const KArgs &p, const f32x16 (&acc)[FA][FB], int arow0, int brow0, int lane, int split)
{
    const bool to_partial = p.splits > 1;
    const bool vec4 = (p.rowsA & 3) == 0;
#pragma unroll
    for (int i = 0; i < FA; ++i)
#pragma unroll
        for (int j = 0; j < FB; ++j) {
            const int pix = brow0 + j * 32 + (lane & 31);
            if (pix >= p.rowsB) continue;
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int ch = arow0 + i * 32 + 8 * gq + 4 * (lane >> 5);
                if (ch >= p.rowsA) continue;
                float v[4] = {acc[i][j][4 * gq], acc[i][j][4 * gq + 1], acc[i][j][4 * gq + 2], acc[i][j][4 * gq + 3]};
                const size_t o = (size_t)pix * p.rowsA + ch;
                if (to_partial) {
                    float *dst = p.partial + (size_t)split * p.rowsB * p.rowsA + o;
                    if (p.flags & KF_FUSED_REDUCE) store_f32x4_device_scope(dst, f32x4{v[0], v[1], v[2], v[3]});   // rowsA % 4 == 0
                    else if (vec4) *reinterpret_cast<f32x4 *>(dst) = f32x4{v[0], v[1], v[2], v[3]};
                    else
                        for (int e = 0; e < 4; ++e) if (ch + e < p.rowsA) dst[e] = v[e];
                    continue;
                }
                if (p.flags & KF_BIAS)
                    for (int e = 0; e < 4; ++e) if (ch + e < p.rowsA) v[e] += p.bias[ch + e];
                if (p.flags & KF_RELU)
                    for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
                if (p.flags & KF_MASK_IN)
                    for (int e = 0; e < 4; ++e) if (ch + e < p.rowsA) v[e] = mask1f(v[e], p.x[o + e]);
                if (p.flags & KF_OUT_F32) {
                    float *dst = reinterpret_cast<float *>(p.out) + o;
                    if (vec4) *reinterpret_cast<f32x4 *>(dst) = f32x4{v[0], v[1], v[2], v[3]};
                    else
                        for (int e = 0; e < 4; ++e) if (ch + e < p.rowsA) dst[e] = v[e];
                } else {
                    bf16_t *dst = reinterpret_cast<bf16_t *>(p.out) + o;
                    if (vec4) {
                        u32x2 pk{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
                        *reinterpret_cast<u32x2 *>(dst) = pk;
                    } else
                        for (int e = 0; e < 4; ++e) if (ch + e < p.rowsA) dst[e] = (bf16_t)f32_to_bf16(v[e]);
                }
            }
        }
}

// Epilogue for wgrad: out[i][j] (c_out-major, tap contiguous), always fp32.
template <int FA, int FB>
DEVFN void store_row_major(const KArgs &p, const f32x16 (&acc)[FA][FB], int arow0, int brow0, int lane, int split)
{
    float *base = p.splits > 1 ? p.partial + (size_t)split * p.rowsA * p.rowsB : reinterpret_cast<float *>(p.out);
#pragma unroll
    for (int i = 0; i < FA; ++i)
#pragma unroll
        for (int j = 0; j < FB; ++j) {
            const int col = brow0 + j * 32 + (lane & 31);
            if (col >= p.rowsB) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = arow0 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row >= p.rowsA) continue;
                if (p.flags & KF_NT_OUT) __builtin_nontemporal_store(acc[i][j][v], base + (size_t)row * p.rowsB + col);
                else base[(size_t)row * p.rowsB + col] = acc[i][j][v];
            }
        }
}


}  // namespace
