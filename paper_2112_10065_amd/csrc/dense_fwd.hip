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
