// Dense (fully connected) forward at per-GPU batch <= 32, bound by reading the weights once (paper section 3.1: the
// small-batch regime leaves these layers with a few hundred flops per weight byte at most).
//
// y[n][o] = sum_i x[n][i] * W[o][i]: every weight is used N <= 32 times, so the kernel is a stream over W.  What the
// memory system rewards (measured): a wave-wide load that touches at most 8 rows with 128 contiguous bytes each, several
// such loads in flight per wave, eight or more waves per compute unit, and no block barrier in the stream.  So:
//   * a block owns 16 output rows (one 16x16x32 matrix-instruction tile of W rows x samples) and its 8 waves split the
//     input features among them; the waves' partial sums meet in LDS at the end (added in wave order), so there is no
//     second kernel and no partial sum in memory;
//   * every wave runs its own NS-stage pipeline of direct-to-LDS loads (two loads of 8 rows x 128 bytes per 64-feature
//     step) into its own LDS stages and reads the fragments back 16-byte chunk-swizzled (chunk c of row r sits at
//     position c ^ (r % 8)), waiting on its own load counter only;
//   * the activations (N rows, shared by all blocks, resident in L2) come straight from memory into registers, issued
//     together with the weight loads of the same step so that the in-order load counter never waits for a young load.
// Bias and ReLU are applied after the waves' sums are added.
#include "dma_common.h"
#include <type_traits>

namespace {

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4v;

// the weights are read once per pass: non-temporal, so that the stream does not push the step's activations out of the caches
DEVFN void dma16_soff(__amdgpu_buffer_rsrc_t r, unsigned lds_base, unsigned voff, unsigned soff)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_void)(size_t)lds_base, 16, voff, soff, 0, 2);
}
// 16 bytes per lane into registers, invisible to the compiler's wait placement (it would drain the whole pipeline once per
// trip of the unrolled loop): the caller waits on the load counter and then ties the registers to that wait
template <int OFF> DEVFN u32x4 load16_async(u32x4 rsrc, unsigned voff, unsigned soff)
{
    u32x4 v;
    asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen offset:%4" : "=v"(v) : "v"(voff), "s"(rsrc), "s"(soff), "n"(OFF) : "memory");
    return v;
}
DEVFN u32x4 raw_rsrc(const void *p, size_t bytes)   // the words of make_rsrc's descriptor
{
    const unsigned long long a = (unsigned long long)p;
    return u32x4{(unsigned)a, (unsigned)(a >> 32) & 0xffffu, (unsigned)bytes, 0x00020000u};
}

constexpr int DF_NS = 5, DF_WAVES = 8, DF_STAGE = 2048;

template <int NB>   // groups of 16 samples: 1 (N <= 16) or 2 (N <= 32)
__global__ __launch_bounds__(64 * DF_WAVES) void k_dense_fwd(int N, int C, int K, unsigned flags, const bf16_t *x, const bf16_t *w, const float *bias,
                                                             bf16_t *y)
{
    constexpr int D = DF_NS - 1, P = 2 + 2 * NB;   // prefetch distance in steps; memory instructions per step
    static_assert((D - 1) * P < 64, "the load counter has six bits");
    __shared__ __attribute__((aligned(1024))) char lds[DF_WAVES * DF_NS * DF_STAGE];
    static_assert(sizeof(lds) >= DF_WAVES * NB * 64 * sizeof(f32x4v), "the waves' sums fit the stages");
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g0 = blockIdx.x * 16;
    const int steps = C / 64, spw = (steps + DF_WAVES - 1) / DF_WAVES;
    const int sbeg = min(wave * spw, steps), nst = min(sbeg + spw, steps) - sbeg;
    __amdgpu_buffer_rsrc_t rw = make_rsrc(w, (size_t)K * C * 2);
    const u32x4 rx = raw_rsrc(x, (size_t)N * C * 2);
    const unsigned base = lds_offset(lds) + wave * (DF_NS * DF_STAGE);

    unsigned voffW[2], voffX[NB];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int row = 8 * j + (lane >> 3), c = (lane & 7) ^ (row & 7);
        voffW[j] = g0 + row < K ? ((unsigned)(g0 + row) * C + c * 8) * 2u : OOR;
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int n = 16 * b + (lane & 15);
        voffX[b] = n < N ? ((unsigned)n * C + (lane >> 4) * 8) * 2u : OOR;
    }
    // fragment of W for matrix instruction s of a step: row l%16, features 32*s + 8*(l/16) .. +7, i.e. chunk 4*s + l/16
    unsigned fa[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) fa[s] = base + (lane & 15) * 128 + (((4 * s + (lane >> 4)) ^ (lane & 7)) << 4);

    u32x4 xr[DF_NS][NB][2];
    auto issue = [&](int i, int stage) {   // loads of step i (relative to sbeg) into `stage`
        const unsigned soff = (unsigned)(sbeg + i) * 128u;
#pragma unroll
        for (int j = 0; j < 2; ++j) dma16_soff(rw, base + stage * DF_STAGE + j * 1024, voffW[j], soff);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            xr[stage][b][0] = load16_async<0>(rx, voffX[b], soff);
            xr[stage][b][1] = load16_async<64>(rx, voffX[b], soff);
        }
    };
    f32x4v acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) acc[b] = f32x4v{0.f, 0.f, 0.f, 0.f};

#pragma unroll
    for (int u = 0; u < D; ++u)
        if (u < nst) issue(u, u);
    for (int i0 = 0; i0 < nst; i0 += DF_NS) {
#pragma unroll
        for (int u = 0; u < DF_NS; ++u) {
            const int i = i0 + u;
            if (i < nst) {
                const int younger = min(D - 1, nst - 1 - i);
                if (younger == D - 1) wait_vmcnt<(D - 1) * P>();
                else if (D >= 3 && younger == D - 2) wait_vmcnt<(D >= 3 ? D - 2 : 0) * P>();
                else if (D >= 4 && younger == D - 3) wait_vmcnt<(D >= 4 ? D - 3 : 0) * P>();
                else wait_vmcnt<0>();
                if (i + D < nst) issue(i + D, (u + D) % DF_NS);   // the stage of step i - 1, whose reads have returned
                u32x4 a[2];
                a[0] = lds_read16<0>(fa[0] + u * DF_STAGE);
                a[1] = lds_read16<0>(fa[1] + u * DF_STAGE);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                asm volatile("" : "+v"(a[0]), "+v"(a[1]));
#pragma unroll
                for (int b = 0; b < NB; ++b) asm volatile("" : "+v"(xr[u][b][0]), "+v"(xr[u][b][1]));   // landed with the step's weight loads
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int b = 0; b < NB; ++b)
                        acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[s]), __builtin_bit_cast(bf16x8, xr[u][b][s]), acc[b], 0, 0, 0);
            }
        }
    }
    wait_vmcnt<0>();
    __syncthreads();   // every wave is done with its stages: they give way to the sums
    f32x4v *red = reinterpret_cast<f32x4v *>(lds);   // [wave][group][lane]
#pragma unroll
    for (int b = 0; b < NB; ++b) red[(wave * NB + b) * 64 + lane] = acc[b];
    __syncthreads();
    if (tid < 64 * NB) {
        const int b = tid >> 6;
        f32x4v s = red[b * 64 + lane];
#pragma unroll
        for (int wv = 1; wv < DF_WAVES; ++wv) s += red[(wv * NB + b) * 64 + lane];
        // element v of lane l: output row g0 + 4*(l/16) + v, sample 16*b + l%16
        const int n = 16 * b + (lane & 15), o = g0 + 4 * (lane >> 4);
        if (n < N) {
            float v[4] = {s[0], s[1], s[2], s[3]};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if ((flags & KF_BIAS) && o + e < K) v[e] += bias[o + e];
                if (flags & KF_RELU) v[e] = fmaxf(v[e], 0.f);
            }
            bf16_t *dst = y + (size_t)n * K + o;
            if (o + 4 <= K && (K & 3) == 0) *reinterpret_cast<u32x2 *>(dst) = u32x2{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
            else
                for (int e = 0; e < 4; ++e) if (o + e < K) dst[e] = (bf16_t)f32_to_bf16(v[e]);
        }
    }
}

// ---------------------------------------------------------------------------------------
// Backward-data of the same layers: dx[n][i] = sum_o dy[n][o] * W[o][i], again one pass over W.  A block owns 64 input
// features (128 contiguous bytes of every weight row) and its 8 waves split the output rows, the reduction, among
// them.  A step is 16 weight rows: two direct-to-LDS loads of 8 rows x 128 bytes into the wave's own stage, rows as they
// come from memory (the two 64-byte halves of a row swapped on odd row pairs); the matrix instruction wants the
// reduction contiguous per lane, which the LDS transpose read delivers.  The gradient operand (sample l%32, output rows
// 8*(l/32) .. +7 of the step) is 16 contiguous bytes of dy and goes from memory straight into registers, issued with the
// step's weight loads.  The waves' sums meet in LDS; the backward of the ReLU in front of the layer (mask by the saved
// input) and the conversion ride in that last pass.
// ---------------------------------------------------------------------------------------
constexpr int DG_NS = 4, DG_STAGE = 2048;
template <int OFF> DEVFN u32x2 lds_read_tr_off(unsigned addr)
{
    u32x2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
__global__ __launch_bounds__(64 * DF_WAVES) void k_dense_dgrad(int N, int C, int K, unsigned flags, const bf16_t *dy, const bf16_t *w, const bf16_t *xin,
                                                               void *dx)
{
    constexpr int D = DG_NS - 1, P = 3;   // prefetch distance in steps; memory instructions per step
    __shared__ __attribute__((aligned(1024))) char lds[DF_WAVES * DG_NS * DG_STAGE];   // 64 KiB: the stages, then the waves' sums
    static_assert(sizeof(lds) >= DF_WAVES * 2 * 64 * sizeof(f32x16), "the waves' sums fit the stages");
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i0 = blockIdx.x * 64;
    const int steps = (K + 15) / 16, spw = (steps + DF_WAVES - 1) / DF_WAVES;
    const int sbeg = min(wave * spw, steps), nst = min(sbeg + spw, steps) - sbeg;
    __amdgpu_buffer_rsrc_t rw = make_rsrc(w, (size_t)K * C * 2);
    const u32x4 rdy = raw_rsrc(dy, (size_t)N * K * 2);
    const unsigned base = lds_offset(lds) + wave * (DG_NS * DG_STAGE);

    // weight loads: lane l of load j fills 16-byte position l%8 of stage row 8*j + l/8 with global chunk (l%8) ^ 4*swz(row); rows
    // past the last output and chunks past the last input feature fetch zeros (the range check of the buffer covers the end only)
    unsigned voffW[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int t = 8 * j + (lane >> 3), c = (lane & 7) ^ (seg_swz<64>(t) << 2);
        voffW[j] = i0 + c * 8 < C ? ((unsigned)t * C + i0 + c * 8) * 2u : OOR;
    }
    const unsigned voffY = (lane & 31) < N ? ((unsigned)(lane & 31) * K + (lane >> 5) * 8) * 2u : OOR;
    // transpose-read addresses of the two 32-feature fragments: lane l of a 16-lane group points at stage row 8*(l>>5) + (l&15)/4
    // (+4 for the second half), features 16*((l>>4)&1) + 4*(l&3) .. +3 of the fragment
    const int i16 = lane & 15, tl = (lane >> 5) * 8 + (i16 >> 2), cl = ((lane >> 4) & 1) * 16 + (i16 & 3) * 4;
    unsigned fa[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) fa[i] = base + tl * 128 + (((i ^ seg_swz<64>(tl)) << 6) | (cl << 1));

    u32x4 yr[DG_NS];
    auto issue = [&](int i, int stage) {
        const int o0 = (sbeg + i) * 16;
        // rows of the step past K: the buffer's range check sees offsets past the end of W only for the very last rows, so mask here
        const unsigned soff = (unsigned)o0 * (unsigned)C * 2u;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const bool live = o0 + 8 * j + (lane >> 3) < K;
            dma16_soff(rw, base + stage * DG_STAGE + j * 1024, live ? voffW[j] : OOR, soff);
        }
        // eight output rows per lane: a chunk that straddles K is cut by the buffer's range check only at the very end of dy, so mask
        const bool ylive = o0 + (lane >> 5) * 8 + 8 <= K;
        yr[stage] = load16_async<0>(rdy, ylive ? voffY : OOR, (unsigned)o0 * 2u);
    };
    f32x16 acc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

#pragma unroll
    for (int u = 0; u < D; ++u)
        if (u < nst) issue(u, u);
    for (int it0 = 0; it0 < nst; it0 += DG_NS) {
#pragma unroll
        for (int u = 0; u < DG_NS; ++u) {
            const int it = it0 + u;
            if (it < nst) {
                const int younger = min(D - 1, nst - 1 - it);
                if (younger == D - 1) wait_vmcnt<(D - 1) * P>();
                else if (D >= 3 && younger == D - 2) wait_vmcnt<(D >= 3 ? D - 2 : 0) * P>();
                else wait_vmcnt<0>();
                if (it + D < nst) issue(it + D, (u + D) % DG_NS);   // the stage of step it - 1, whose reads have returned
                u32x2 lo[2], hi[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    lo[i] = lds_read_tr_off<0>(fa[i] + u * DG_STAGE);
                    hi[i] = lds_read_tr_off<512>(fa[i] + u * DG_STAGE);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                asm volatile("" : "+v"(lo[0]), "+v"(hi[0]), "+v"(lo[1]), "+v"(hi[1]), "+v"(yr[u]));
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, u32x4{lo[i].x, lo[i].y, hi[i].x, hi[i].y}),
                                                                     __builtin_bit_cast(bf16x8, yr[u]), acc[i], 0, 0, 0);
            }
        }
    }
    wait_vmcnt<0>();
    __syncthreads();   // every wave is done with its stages: they give way to the sums
    f32x4v *red = reinterpret_cast<f32x4v *>(lds);   // [wave][fragment][group of four registers][lane]
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq)
            red[((wave * 2 + i) * 4 + gq) * 64 + lane] = f32x4v{acc[i][4 * gq], acc[i][4 * gq + 1], acc[i][4 * gq + 2], acc[i][4 * gq + 3]};
    __syncthreads();
    {
        // wave w adds group w%4 of fragment w/4 over the eight waves, in wave order: registers 4*gq .. +3 of lane l are
        // features 32*i + 8*gq + 4*(l/32) .. +3 of sample l%32
        const int i = wave >> 2, gq = wave & 3;
        f32x4v s = red[((0 * 2 + i) * 4 + gq) * 64 + lane];
#pragma unroll
        for (int wv = 1; wv < DF_WAVES; ++wv) s += red[((wv * 2 + i) * 4 + gq) * 64 + lane];
        const int n = lane & 31, f = i0 + 32 * i + 8 * gq + 4 * (lane >> 5);
        if (n < N && f < C) {
            float v[4] = {s[0], s[1], s[2], s[3]};
            const size_t o = (size_t)n * C + f;
            if (flags & KF_MASK_IN)
                for (int e = 0; e < 4; ++e) if (f + e < C) v[e] = mask1f(v[e], xin[o + e]);
            if (flags & KF_OUT_F32) {
                float *dst = reinterpret_cast<float *>(dx) + o;
                if (f + 4 <= C && (C & 3) == 0) *reinterpret_cast<f32x4 *>(dst) = f32x4{v[0], v[1], v[2], v[3]};
                else
                    for (int e = 0; e < 4; ++e) if (f + e < C) dst[e] = v[e];
            } else {
                bf16_t *dst = reinterpret_cast<bf16_t *>(dx) + o;
                if (f + 4 <= C && (C & 3) == 0) *reinterpret_cast<u32x2 *>(dst) = u32x2{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
                else
                    for (int e = 0; e < 4; ++e) if (f + e < C) dst[e] = (bf16_t)f32_to_bf16(v[e]);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Filter gradient of the same layers: dW[o][i] = sum_n dy[n][o] * x[n][i] with N <= 32 is an outer product that writes
// K*C fp32 once and reads next to nothing, so it is a store stream.  A wave owns one 64 x 64 tile of dW: it copies its
// dy tile [32 samples][64 outputs] and its x tile [32 samples][64 inputs] into its own LDS (direct-to-LDS loads, rows of
// samples the batch does not have fetch zeros), reads both through the LDS transpose read (samples are the reduction),
// multiplies (one 16-sample slice, two beyond 16 samples) and stores its sums, non-temporally when the gradient is large.
// No barrier, no row tables, no partial sums.  The bias gradient (dy fragments times ones) is added by the waves of the
// first input tile.
// ---------------------------------------------------------------------------------------
template <bool NT>
__global__ __launch_bounds__(64 * DF_WAVES) void k_dense_wgrad(int N, int C, int K, const bf16_t *x, const bf16_t *dy, float *dw, float *db)
{
    __shared__ __attribute__((aligned(1024))) char lds[DF_WAVES * 8192];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int o0 = blockIdx.x * 64, i0 = (blockIdx.y * DF_WAVES + wave) * 64;
    if (i0 >= C) return;   // no barrier follows
    __amdgpu_buffer_rsrc_t rdy = make_rsrc(dy, (size_t)N * K * 2);
    __amdgpu_buffer_rsrc_t rx = make_rsrc(x, (size_t)N * C * 2);
    const unsigned base = lds_offset(lds) + wave * 8192;
    // lane l of load j fills 16-byte position l%8 of tile row (sample) 8*j + l/8 with global chunk (l%8) ^ 4*swz(row)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int t = 8 * j + (lane >> 3), c = (lane & 7) ^ (seg_swz<64>(t) << 2);
        const bool row = t < N;
        dma16(rdy, base + j * 1024, row && o0 + c * 8 < K ? ((unsigned)t * K + o0 + c * 8) * 2u : OOR);
        dma16(rx, base + 4096 + j * 1024, row && i0 + c * 8 < C ? ((unsigned)t * C + i0 + c * 8) * 2u : OOR);
    }
    const int i16 = lane & 15, tl = (lane >> 5) * 8 + (i16 >> 2), cl = ((lane >> 4) & 1) * 16 + (i16 & 3) * 4;
    unsigned fa[2];   // fragment f of either tile: sample rows tl (+4), columns 32*f + cl .. +3
#pragma unroll
    for (int f = 0; f < 2; ++f) fa[f] = base + tl * 128 + (((f ^ seg_swz<64>(tl)) << 6) | (cl << 1));
    f32x16 acc[2][2], accdb[2];
#pragma unroll
    for (int a = 0; a < 2; ++a) {
#pragma unroll
        for (int v = 0; v < 16; ++v) accdb[a][v] = 0.f;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    }
    const bool do_db = db != nullptr && i0 == 0;
    wait_vmcnt<0>();
    auto slice = [&](auto ks_tag) {
        constexpr int KS = decltype(ks_tag)::value;
        u32x2 alo[2], ahi[2], blo[2], bhi[2];
#pragma unroll
        for (int f = 0; f < 2; ++f) {
            alo[f] = lds_read_tr_off<KS * 2048>(fa[f]);
            ahi[f] = lds_read_tr_off<KS * 2048 + 512>(fa[f]);
            blo[f] = lds_read_tr_off<4096 + KS * 2048>(fa[f]);
            bhi[f] = lds_read_tr_off<4096 + KS * 2048 + 512>(fa[f]);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        asm volatile("" : "+v"(alo[0]), "+v"(ahi[0]), "+v"(alo[1]), "+v"(ahi[1]), "+v"(blo[0]), "+v"(bhi[0]), "+v"(blo[1]), "+v"(bhi[1]));
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            const bf16x8 av = __builtin_bit_cast(bf16x8, u32x4{alo[a].x, alo[a].y, ahi[a].x, ahi[a].y});
#pragma unroll
            for (int b = 0; b < 2; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8, u32x4{blo[b].x, blo[b].y, bhi[b].x, bhi[b].y}), acc[a][b], 0, 0, 0);
            if (do_db) accdb[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, ones_bf16(), accdb[a], 0, 0, 0);
        }
    };
    slice(std::integral_constant<int, 0>{});
    if (N > 16) slice(std::integral_constant<int, 1>{});
    // element v of lane l: output row 8*(v/4) + 4*(l/32) + v%4 of its fragment, input column l%32
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int o = o0 + 32 * a + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (o >= K) continue;
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int i = i0 + 32 * b + (lane & 31);
                if (i >= C) continue;
                if (NT) __builtin_nontemporal_store(acc[a][b][v], dw + (size_t)o * C + i);
                else dw[(size_t)o * C + i] = acc[a][b][v];
            }
        }
    if (do_db) {
#pragma unroll
        for (int a = 0; a < 2; ++a) store_db_fragment(accdb[a], db, o0 + 32 * a, K, lane);
    }
}

}  // namespace

// shapes the streaming dense forward takes: a 1x1 layer over at most 16 pixel rows (beyond that the activation operand, which
// every block re-reads, outweighs the weights), input features in whole 64-feature steps
bool dense_fwd_stream_shape(const ConvGeom &g)
{
    const long long rows = (long long)g.N * g.Ho * g.Wo;
    return g.R == 1 && g.S == 1 && g.sh == 1 && g.sw == 1 && g.ph == 0 && g.pw == 0 && rows <= 16 && g.C % 64 == 0 && g.C >= 64 * DF_WAVES &&
           (unsigned long long)g.K * g.C * 2 < (1ull << 32);
}

hipError_t dense_fwd_stream(const ConvGeom &g, unsigned flags, const bf16_t *x, const bf16_t *w, const float *bias, bf16_t *y, hipStream_t st)
{
    const int rows = g.N * g.Ho * g.Wo, blocks = (g.K + 15) / 16;
    if (rows <= 16) hipLaunchKernelGGL(k_dense_fwd<1>, dim3((unsigned)blocks), dim3(64 * DF_WAVES), 0, st, rows, g.C, g.K, flags, x, w, bias, y);
    else hipLaunchKernelGGL(k_dense_fwd<2>, dim3((unsigned)blocks), dim3(64 * DF_WAVES), 0, st, rows, g.C, g.K, flags, x, w, bias, y);
    return hipGetLastError();
}

// shapes the streaming dense backward-data takes: a 1x1 layer over at most 32 pixel rows whose output features do not come in whole
// 64-row reduction steps, which keeps the pipelined tile kernels away (the classifier layer with its 1000 outputs); input and output
// features in whole 8-element chunks (16-byte loads), enough output rows to give every wave of a block a few steps.  Where the
// pipelined kernels do run they are as fast (measured on 25088 x 4096 and 4096 x 4096: both forms read the 128-byte column strips
// of W at about 4 TB/s), so they keep those shapes.
bool dense_dgrad_stream_shape(const ConvGeom &g)
{
    const long long rows = (long long)g.N * g.H * g.W;
    return g.R == 1 && g.S == 1 && g.sh == 1 && g.sw == 1 && g.ph == 0 && g.pw == 0 && rows <= 32 && g.C % 8 == 0 && g.K % 8 == 0 &&
           g.K % 64 != 0 && g.K >= 16 * DF_WAVES && (unsigned long long)g.K * g.C * 2 < (1ull << 32);
}

hipError_t dense_dgrad_stream(const ConvGeom &g, unsigned flags, const bf16_t *dy, const bf16_t *w, const bf16_t *xin, void *dx, hipStream_t st)
{
    const int rows = g.N * g.H * g.W, blocks = (g.C + 63) / 64;
    hipLaunchKernelGGL(k_dense_dgrad, dim3((unsigned)blocks), dim3(64 * DF_WAVES), 0, st, rows, g.C, g.K, flags, dy, w, xin, dx);
    return hipGetLastError();
}

// shapes the streaming dense filter gradient takes: a 1x1 layer over at most 32 pixel rows, features in whole 8-element chunks,
// a gradient of 4 to 128 MB (measured: 4096 x 4096 28 -> 21 us and 4096 x 1000 19 -> 14 us against the pipelined tile kernel,
// which in turn writes the 411 MB of the 25088 x 4096 layer 15 us faster with its 128 x 128 tiles)
bool dense_wgrad_stream_shape(const ConvGeom &g)
{
    const long long rows = (long long)g.N * g.Ho * g.Wo, elems = (long long)g.K * g.C;
    return g.R == 1 && g.S == 1 && g.sh == 1 && g.sw == 1 && g.ph == 0 && g.pw == 0 && rows <= 32 && g.C % 8 == 0 && g.K % 8 == 0 &&
           elems >= (1 << 20) && elems <= (32 << 20);
}

hipError_t dense_wgrad_stream(const ConvGeom &g, const bf16_t *x, const bf16_t *dy, float *dw, float *db, hipStream_t st)
{
    const int rows = g.N * g.Ho * g.Wo;
    const dim3 grid((unsigned)((g.K + 63) / 64), (unsigned)((g.C + 64 * DF_WAVES - 1) / (64 * DF_WAVES)));
    if ((size_t)g.K * g.C * 4 >= ((size_t)32 << 20)) hipLaunchKernelGGL(k_dense_wgrad<true>, grid, dim3(64 * DF_WAVES), 0, st, rows, g.C, g.K, x, dy, dw, db);
    else hipLaunchKernelGGL(k_dense_wgrad<false>, grid, dim3(64 * DF_WAVES), 0, st, rows, g.C, g.K, x, dy, dw, db);
    return hipGetLastError();
}

const char *dense_fwd_stream_name(const ConvGeom &g) { return g.N * g.Ho * g.Wo <= 16 ? "k_dense_fwd<1>" : "k_dense_fwd<2>"; }
const char *dense_wgrad_stream_name(const ConvGeom &g) { return (size_t)g.K * g.C * 4 >= ((size_t)32 << 20) ? "k_dense_wgrad<true>" : "k_dense_wgrad<false>"; }
