// Filter gradient of 3x3 / stride 1 / pad 1 layers with the x operand shared by the three taps of a filter row.
//
// dW[k][r][s][c] = sum over pixels m of dy[m][k] * x[m + (r-1)*W + (s-1)][c] (pairs outside the image contribute
// nothing).  A block owns 256 output channels k, one filter row r, 64 input channels c and all three filter columns
// s: a 256 x 192 tile.  The reduction runs over pixel SLOTS, 64 per step: every image row gets a segment of SEG slots
// (the power of two >= W + 2; a step holds 64 / SEG image rows), the slots past W hold zeros.  With that padding the
// x pixels of the three taps are three windows, one slot apart, of ONE strip of 66 slots (slot u of a segment holds
// pixel w = u - 1, zero for w = -1 and w >= W), so the row-end wrap that a flat pixel order would need masks for
// cannot happen, and a step fetches 32 KB of dy and 8 KB of x instead of 32 + 24.  The price is SEG / W more matrix
// work (64/56 for the VGG widths 56, 28 and 14).
// Both operands are reduction-major in LDS ([slot][256 k] and [slot][64 c]) and go through the LDS transpose read.
// One wave per SIMD (4 waves of 128 x 96, 192 accumulators); the loop body holds matrix instructions, LDS reads and
// direct-to-LDS copies in fixed slots (see k_conv_strip in conv_dma.hip for why), three stages of both operands, the
// step's base address rides in the buffer resource (rebuilt per step with scalar instructions, so rows past the end of
// the tensors are out of range by construction).  Vertical validity (filter row 0 has no partner for image row 0,
// filter row 2 none for the last image row) is per strip row and step: one compare and select per copy.
// Output: fp32 dW directly, or fp32 partials [split][k][r][s][c] for the split-reduce kernel.
#include "dma_common.h"
#include <type_traits>

namespace {

DEVFN void mfma_pinned(f32x16 &c, const u32x4 &a, const u32x4 &b)
{
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);   // nothing moves across: the instruction stays in its slot
}

constexpr int kWsLds = 3 * 64 * 512 + 3 * 96 * 128;

__global__ __launch_bounds__(256) void k_wgrad_strip(const KArgs p)
{
#if __HIP_DEVICE_COMPILE__   // the host pass only needs the launch stub
    constexpr int TA = 256, FA = 4, FB = 3, NM = FA * FB, NRD = 2 * FA + 2 * FB;
    constexpr int ROWA = TA * 2, A_BYTES = 64 * ROWA, SROWS = 96, SROW = 128, S_BYTES = SROWS * SROW, IA = 8, IS = 3, LPS = IA + IS;
    static_assert(A_BYTES + 4 * ROWA < 65536 && 2 * S_BYTES + 4 * SROW < 65536, "stage offsets fit the 16-bit immediate");
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const ConvGeom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const unsigned wave_s = __builtin_amdgcn_readfirstlane(wave);
    const int SEG = p.ph_tile0[0], RS = 64 / SEG;   // slots per image row, image rows per step
    const int tile = blockIdx.y, split = blockIdx.x;
    const int a0 = (tile % p.tilesA) * TA, tb = tile / p.tilesA, CBT = g.C / 64;
    const int r = tb / CBT, c0 = (tb - r * CBT) * 64;
    const int nsteps = p.steps_per_split, NR = g.N * g.H;   // a multiple of 3 steps; image rows past NR are out of range
    const int row_first = split * p.steps_per_split * RS;
    const unsigned lds0 = lds_offset(smem), ldsS0 = lds0 + 3 * A_BYTES;

    // copies of dy: one fills two slots t of 512 bytes; lane l takes the 16-byte chunk (l % 32) ^ swizzle(t)
    unsigned voffA[IA], voffS[IS];
    int hbad[IS];
#pragma unroll
    for (int q = 0; q < IA; ++q) {
        const int t = (wave * IA + q) * 2 + lane / 32, seg = t / SEG, j = t - seg * SEG;
        const int col = a0 + ((lane % 32) ^ ((t & 3) << 2)) * 8;
        voffA[q] = j < g.W && col < g.K ? ((unsigned)(seg * g.W + j) * g.K + col) * 2u : OOR;
    }
    // copies of x: one fills eight strip rows U of 128 bytes; strip row U = slot + filter column; slot u of a segment holds pixel w = u - 1
#pragma unroll
    for (int q = 0; q < IS; ++q) {
        const int U = (wave * IS + q) * 8 + lane / 8, seg = U / SEG, u = U - seg * SEG;
        const int chunk = (lane % 8) ^ (((U >> 1) & 1) << 2);
        voffS[q] = U < 64 && u >= 1 && u <= g.W ? ((unsigned)(seg * g.W + u - 1) * g.C + c0 + chunk * 8) * 2u : OOR;
        // the strip row pairs image row h = (first row of the step + seg) mod H with x row h + r - 1: none for h = 0 (r = 0) and
        // h = H - 1 (r = 2); hbad is the value of (first row of the step) mod H at which this lane's row is that one
        const int hb = r == 0 ? 0 : g.H - 1;
        hbad[q] = r == 1 ? -1 : ((hb - seg) % g.H + g.H) % g.H;
    }
    // the next step to issue: first image row mod H, the windows of dy and x that start at its first row (x: r - 1 rows
    // earlier, one pixel is subtracted in the strip offsets) and the bytes left in the tensors from there (a step past the end
    // gets a zero-length window); all advance by one step's rows with a few scalar additions
    int hbase = row_first % g.H;
    const long long stride_a = (long long)RS * g.W * g.K * 2, stride_b = (long long)RS * g.W * g.C * 2;
    const char *pa = reinterpret_cast<const char *>(p.dy) + (long long)row_first * g.W * g.K * 2;
    const char *pb = reinterpret_cast<const char *>(p.x) + (long long)(row_first + r - 1) * g.W * g.C * 2;
    long long left_a = (long long)(NR - row_first) * g.W * g.K * 2, left_b = (long long)(NR - (row_first + r - 1)) * g.W * g.C * 2;
    auto window = [&](const char *base, long long left, bool on) {
        const long long n = !on || left < 0 ? 0 : left > 0x7fffffffLL ? 0x7fffffffLL : left;
        return make_rsrc(base, (size_t)n);
    };
    auto advance = [&]() {
        pa += stride_a; pb += stride_b; left_a -= stride_a; left_b -= stride_b;
        hbase += RS;
        if (hbase >= g.H) hbase -= g.H;
    };
    auto issue = [&](int stage, bool on) {   // copies of the next step into `stage`
        __amdgpu_buffer_rsrc_t ra_ = window(pa, left_a, on), rb_ = window(pb, left_a > 0 ? left_b : 0, on);
#pragma unroll
        for (int q = 0; q < IA; ++q) dma16(ra_, lds0 + stage * A_BYTES + (wave_s * IA + q) * 1024, voffA[q]);
#pragma unroll
        for (int q = 0; q < IS; ++q) dma16(rb_, ldsS0 + stage * S_BYTES + (wave_s * IS + q) * 1024, hbase != hbad[q] ? voffS[q] : OOR);
        advance();
    };

    f32x16 acc[FA][FB];
#pragma unroll
    for (int i = 0; i < FA; ++i)
#pragma unroll
        for (int j = 0; j < FB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    const int arow = (wave & 1) * 128, wb = wave >> 1;
    // transpose-read addresses: lane l points at slot ks*16 + 8*(l>>5) + (l&15)/4 (and 4 slots further for the second half),
    // operand rows row0 + 16*((l>>4)&1) + 4*(l&3) .. +3.  fa_hi: the third dy stage, out of reach of a 16-bit immediate.
    unsigned fa[4][FA], fa_hi[4][FA], fb[4][FB];
    {
        const int i16 = lane & 15, tl = (lane >> 5) * 8 + (i16 >> 2), cl = ((lane >> 4) & 1) * 16 + (i16 & 3) * 4;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int t = ks * 16 + tl;
#pragma unroll
            for (int i = 0; i < FA; ++i) {
                const int col = arow + i * 32 + cl;
                fa[ks][i] = lds0 + t * ROWA + ((((col >> 5) ^ (t & 3)) << 6) | ((col & 31) << 1));
                fa_hi[ks][i] = fa[ks][i] + 2 * A_BYTES;
            }
#pragma unroll
            for (int j = 0; j < FB; ++j) {
                const int gcol = wb * 96 + j * 32, s = gcol / 64, half = (gcol % 64) / 32, U = t + s;
                fb[ks][j] = ldsS0 + U * SROW + (((half ^ ((U >> 1) & 1)) << 6) | (cl << 1));
            }
        }
    }
    u32x2 alo[2][FA], ahi[2][FA], blo[2][FB], bhi[2][FB];
    // read j of slice ks from stage ST: a0lo a0hi b0lo b0hi a1lo ... (the dy fragments first where x has run out)
    auto read_slot = [&](int buf, int j, int ST, int ks) {
        const int f = j < 4 * FB ? j / 4 : FB + (j - 4 * FB) / 2, part = j < 4 * FB ? j % 4 : (j - 4 * FB) % 2;
        if (part < 2) {
            const unsigned ad = ST == 2 ? fa_hi[ks][f] : fa[ks][f];
            if (part == 0) alo[buf][f] = ST == 1 ? lds_read_tr<A_BYTES>(ad) : lds_read_tr<0>(ad);
            else ahi[buf][f] = ST == 1 ? lds_read_tr<A_BYTES + 4 * ROWA>(ad) : lds_read_tr<4 * ROWA>(ad);
        } else {
            const unsigned ad = fb[ks][f];
            if (part == 2) blo[buf][f] = ST == 0 ? lds_read_tr<0>(ad) : ST == 1 ? lds_read_tr<S_BYTES>(ad) : lds_read_tr<2 * S_BYTES>(ad);
            else bhi[buf][f] = ST == 0 ? lds_read_tr<4 * SROW>(ad) : ST == 1 ? lds_read_tr<S_BYTES + 4 * SROW>(ad) : lds_read_tr<2 * S_BYTES + 4 * SROW>(ad);
        }
    };
    auto read_slots = [&](int m, int buf, int ST, int ks) {   // 14 reads over 12 slots: two in each of the first two
#pragma unroll
        for (int j = 0; j < NRD; ++j) {
            const int slot = j < 2 * (NRD - NM) ? j / 2 : j - (NRD - NM);
            if (slot == m) read_slot(buf, j, ST, ks);
        }
    };
    auto landed = [&](int buf) {
        asm volatile("s_waitcnt lgkmcnt(0)");
#pragma unroll
        for (int f = 0; f < FA; ++f) { asm volatile("" : "+v"(alo[buf][f])); asm volatile("" : "+v"(ahi[buf][f])); }
#pragma unroll
        for (int f = 0; f < FB; ++f) { asm volatile("" : "+v"(blo[buf][f])); asm volatile("" : "+v"(bhi[buf][f])); }
    };
    auto multiply = [&](int buf, int m) {
        const u32x4 av = {alo[buf][m / FB].x, alo[buf][m / FB].y, ahi[buf][m / FB].x, ahi[buf][m / FB].y};
        const u32x4 bv = {blo[buf][m % FB].x, blo[buf][m % FB].y, bhi[buf][m % FB].x, bhi[buf][m % FB].y};
        mfma_pinned(acc[m / FB][m % FB], av, bv);
    };

    // prologue: three steps in flight (copies past the split's range are switched off: zero-length resources)
    issue(0, 0 < nsteps);
    issue(1, 1 < nsteps);
    issue(2, 2 < nsteps);
    wait_vmcnt<2 * LPS>();
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int m = 0; m < NM; ++m) read_slots(m, 0, 0, 0);

    auto step = [&](int i, auto stc) {
        constexpr int ST = decltype(stc)::value, STN = (ST + 1) % 3;
#pragma unroll
        for (int ks = 0; ks < 3; ++ks) {
            landed(ks & 1);
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                read_slots(m, (ks + 1) & 1, ST, ks + 1);
                multiply(ks & 1, m);
            }
        }
        landed(1);                 // the last slice is in registers: this wave is done with the stage
        wait_vmcnt<LPS>();         // the copies of step i+1 have landed; those of step i+2 may be in flight
        __builtin_amdgcn_s_barrier();
        // the freed stage takes step i+3: the copies' addresses first (a few scalar and vector instructions), then one copy per slot
        const bool on = i + 3 < nsteps;
        __amdgpu_buffer_rsrc_t ra_ = window(pa, left_a, on), rb_ = window(pb, left_a > 0 ? left_b : 0, on);
        unsigned vs[IS];
#pragma unroll
        for (int q = 0; q < IS; ++q) vs[q] = hbase != hbad[q] ? voffS[q] : OOR;
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            read_slots(m, 0, STN, 0);
            if (m < IA) dma16(ra_, lds0 + ST * A_BYTES + (wave_s * IA + m) * 1024, voffA[m]);
            else if (m < LPS) dma16(rb_, ldsS0 + ST * S_BYTES + (wave_s * IS + m - IA) * 1024, vs[m - IA]);
            multiply(1, m);
        }
        advance();
    };
    for (int i = 0; i < nsteps; i += 3) {
        step(i, std::integral_constant<int, 0>());
        step(i + 1, std::integral_constant<int, 1>());
        step(i + 2, std::integral_constant<int, 2>());
    }
    wait_vmcnt<0>();

    // accumulator element v of lane l belongs to k row 8*(v/4) + 4*(l>>5) + v%4, column l&31 of its fragment
    float *dst = p.splits > 1 ? p.partial + (size_t)split * p.rowsA * p.rowsB : reinterpret_cast<float *>(p.out);
#pragma unroll
    for (int j = 0; j < FB; ++j) {
        const int gcol = wb * 96 + j * 32, s = gcol / 64, half = (gcol % 64) / 32;
        const size_t colo = (size_t)(r * 3 + s) * g.C + c0 + half * 32 + (lane & 31);
#pragma unroll
        for (int i = 0; i < FA; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = a0 + arow + i * 32 + 8 * (v / 4) + 4 * (lane >> 5) + v % 4;
                if (k < g.K) dst[(size_t)k * p.rowsB + colo] = acc[i][j][v];
            }
    }
#endif
}

int seg_slots(int W)
{
    int seg = 16;
    while (seg < W + 2) seg *= 2;
    return seg;
}

}  // namespace

hipError_t wstrip_init()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(k_wgrad_strip), hipFuncAttributeMaxDynamicSharedMemorySize, kWsLds);
}

// Plan: 3x3, stride 1, pad 1, c_in % 64 == 0, c_out % 8 == 0, image rows of at most 62 pixels that fill at least 3/4 of their slots.
bool wstrip_plan(const ConvGeom &g, int force_splits, GemmPlan *pl)
{
    if (g.R != 3 || g.S != 3 || g.sh != 1 || g.sw != 1 || g.ph != 1 || g.pw != 1 || g.Ho != g.H || g.Wo != g.W) return false;
    if (g.C % 64 != 0 || g.K % 8 != 0 || g.W + 2 > 64) return false;
    const int seg = seg_slots(g.W);
    if (4 * g.W < 3 * seg) return false;
    const long long rows = (long long)g.N * g.H;
    if (rows * g.W * (long long)(g.K > g.C ? g.K : g.C) * 2 >= 0x7fffffffLL) return false;   // 32-bit offsets inside a step's window
    const int rs = 64 / seg;
    pl->variant = 16; pl->TA = 256; pl->TB = 192; pl->BK = 64;
    pl->vecA = pl->vecB = true; pl->fast = true; pl->dma = true; pl->halo = false; pl->phase = false; pl->wstrip = true;
    pl->tilesA = (g.K + 255) / 256;
    pl->tilesB = 3 * (g.C / 64);
    pl->steps_total = (int)((rows + rs - 1) / rs);
    const long long tiles = (long long)pl->tilesA * pl->tilesB;
    int splits = force_splits > 0 ? force_splits : (int)(256 / tiles > 0 ? 256 / tiles : 1);
    if (splits > pl->steps_total / 6) splits = pl->steps_total / 6 > 0 ? pl->steps_total / 6 : 1;
    int sps = (pl->steps_total + splits - 1) / splits;
    sps = (sps + 2) / 3 * 3;   // the kernel unrolls three steps (one per stage)
    pl->steps_per_split = sps;
    pl->splits = (pl->steps_total + sps - 1) / sps;
    return true;
}

hipError_t wstrip_launch(const ConvArgs &a, hipStream_t st)
{
    KArgs p;
    p.g = a.g;
    p.rowsA = a.g.K; p.rowsB = 9 * a.g.C; p.red = a.g.N * a.g.H * a.g.W;
    p.tilesA = a.plan.tilesA; p.tilesB = a.plan.tilesB;
    p.steps_total = a.plan.steps_total; p.steps_per_split = a.plan.steps_per_split; p.splits = a.plan.splits;
    p.flags = a.flags & ~KF_DB;   // the bias gradient is the caller's separate pass
    p.x = a.x; p.w = nullptr; p.dy = a.dy; p.ymask = nullptr; p.bias = nullptr; p.out = a.out; p.partial = a.partial; p.dbp = nullptr;
    p.ph_on = 0;
    p.ph_tile0[0] = seg_slots(a.g.W);
    dim3 grid((unsigned)p.splits, (unsigned)(p.tilesA * p.tilesB), 1), block(256, 1, 1);
    hipLaunchKernelGGL(k_wgrad_strip, grid, block, kWsLds, st, p);
    dp_trace_main_kernel_done(st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.splits <= 1) return e;
    return launch_split_reduce(a, p.rowsA, p.rowsB, st, false);
}
