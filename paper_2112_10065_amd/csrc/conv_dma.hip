// Forward / backward-data kernels with a multi-stage global->LDS pipeline (gfx950 direct-to-LDS
// buffer loads): the tiles of the next NS-1 reduction steps are in flight while the matrix
// cores work on the current one, no registers or ds_write instructions are spent on staging.
//
// A direct-to-LDS load writes the 64 lanes' 16-byte pieces to 1 KiB of consecutive LDS, so the
// tiles are unpadded; bank conflicts are avoided by choosing WHICH global chunk each lane
// fetches: the 16-byte chunk c of tile row `row` lives at chunk position c ^ ((row >> 1) & 7)
// of that row (rows are 128 bytes: BK = 64 bf16), which makes the fragment reads of 16
// consecutive rows hit 16 distinct 16-byte bank groups.
//
// The compiler waits for every outstanding LDS-DMA before any LDS read it can see, which would
// serialise the pipeline; the fragment reads are therefore inline assembly with explicit
// s_waitcnt, and the per-step "stage has landed" wait is an explicit vmcnt.
//
// Step i:  wait(loads of step i) ; barrier ; issue loads of step i+NS-1 into the stage that
//          step i-1 used ; matrix cores on stage i % NS.
#include "dma_common.h"
#include <type_traits>
#include <cstdio>
#include <cstdlib>
#include <atomic>
#include <mutex>

namespace {

template <int FA, int FB, int TA, int TB, int NT>
DEVFN void store_staged(const KArgs &p, const f32x16 (&acc)[FA][FB], bf16_t *stage, const float *bias_lds, int a0, int b0,
                        int arow, int brow, int tid, bool writer = true, const int *rowpix = nullptr, bool all_zero = false)
{
    // all_zero: the tile's sums are known to be zero (no tap reaches it), so the input-ReLU mask need not be read
    // rowpix (LDS, backward-data): output row of each tile row, -1 for none; else tile row i is output row b0 + i
    auto out_row = [&](int pix) { const int gp = rowpix != nullptr ? rowpix[pix] : b0 + pix; return (rowpix != nullptr || gp < p.rowsB) ? gp : -1; };
    // `writer`: this wave holds finished sums (false for the extra reduction groups of a block, which only
    // help with the copy-out below)
    constexpr int LSO = TA + 8;
    const int lane = tid & 63;
    if (writer)
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
    if ((p.flags & KF_MASK_IN) && !all_zero) {
        // fused backward of the input ReLU.  All saved-input vectors of the thread are requested before the staging barrier
        // and consumed in order, so that the tile pays the memory latency once.  Loads and stores go through buffer
        // resources: an element outside the tensor gets an out-of-range offset and the hardware drops it, which keeps the
        // copy-out free of branches (one branch per element made the compiler hold the later loads back behind the
        // earlier stores).  Tensors of 4 GiB and more do not fit a resource and take the grouped form below.
        constexpr int ITERS = (TB * CPR + NT - 1) / NT;
        const size_t bytes = (size_t)p.rowsB * p.rowsA * 2;
        if (ITERS <= 32 && bytes < 0xffffffffull) {
            const __amdgpu_buffer_rsrc_t rin = make_rsrc(p.x, bytes), rout = make_rsrc(out, bytes);
            auto offset = [&](int u) {
                const int id = tid + u * NT, pix = id / CPR, cc = id % CPR;
                const int gp = id < TB * CPR ? out_row(pix) : -1, gc = a0 + cc * 8;
                return (gp >= 0 && gc < p.rowsA) ? ((unsigned)gp * (unsigned)p.rowsA + gc) * 2u : OOR;
            };
            u32x4 xm[ITERS < 32 ? ITERS : 32];
#pragma unroll
            for (int u = 0; u < ITERS; ++u) xm[u] = __builtin_amdgcn_raw_buffer_load_b128(rin, offset(u), 0, 0);
            __syncthreads();
#pragma unroll
            for (int u = 0; u < ITERS; ++u) {
                const int id = tid + u * NT, pix = id / CPR, cc = id % CPR;
                const u32x4 v = id < TB * CPR ? *reinterpret_cast<const u32x4 *>(stage + pix * LSO + cc * 8) : u32x4{0, 0, 0, 0};
                __builtin_amdgcn_raw_buffer_store_b128(apply_mask(v, xm[u]), rout, offset(u), 0, 0);
            }
            return;
        }
        constexpr int GRP = ITERS < 8 ? ITERS : ITERS % 8 == 0 ? 8 : 4;
        static_assert(ITERS % GRP == 0, "copy-out iterations come in whole groups");
        u32x4 xm[GRP];
        auto fetch = [&](int g0) {
#pragma unroll
            for (int u = 0; u < GRP; ++u) {
                const int id = tid + (g0 + u) * NT, pix = id / CPR, cc = id % CPR;
                const int gp = id < TB * CPR ? out_row(pix) : -1, gc = a0 + cc * 8;
                xm[u] = (gp >= 0 && gc < p.rowsA) ? ldg16(p.x + (size_t)gp * p.rowsA + gc) : u32x4{0, 0, 0, 0};
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
                const int gp = id < TB * CPR ? out_row(pix) : -1, gc = a0 + cc * 8;
                if (gp >= 0 && gc < p.rowsA)
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
        const int gp = out_row(pix), gc = a0 + cc * 8;
        if (gp >= 0 && gc < p.rowsA)
            *reinterpret_cast<u32x4 *>(out + (size_t)gp * p.rowsA + gc) = *reinterpret_cast<const u32x4 *>(stage + pix * LSO + cc * 8);
    }
}

// Reduction split without a second kernel.  Every block of a tile stores its fp32 partial with device-scope (written
// through) stores, waits for them and takes a ticket from the tile's counter; the block that draws the last ticket adds the
// partials of all splits IN SPLIT ORDER (so the result does not depend on which block came last), applies the epilogue and
// stores the tile.  The counters live in a static device array, zero when no launch is using them: the last block of a
// tile resets its counter, and concurrent launches (the data-gradient chain and the filter gradients on another stream)
// get disjoint ranges from a host-side ring.
constexpr int kTicketRing = 1 << 16;
__device__ unsigned g_tickets[kTicketRing];

template <int TA, int TB, int NT>
DEVFN void fused_split_reduce(const KArgs &p, int tile, int a0, int b0, int tid)
{
    __shared__ unsigned s_last;
    // the partial sums were stored at device scope (written through); once the stores have completed they are visible to every block
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) s_last = atomicAdd(p.tickets + tile, 1u) == (unsigned)(p.splits - 1) ? 1u : 0u;
    __syncthreads();
    if (s_last == 0) return;
    if (tid == 0) atomicExch(p.tickets + tile, 0u);   // the next launch that is handed this counter finds it at zero
    const unsigned total = (unsigned)p.rowsB * (unsigned)p.rowsA;   // the host keeps splits * total * 4 below 2^31
    const __amdgpu_buffer_rsrc_t part = make_rsrc(p.partial, (size_t)p.splits * total * 4);
    constexpr int CPR = TA / 4;
    constexpr int kDeviceScope = 16;   // cache-policy bit sc1: the load is served coherently at device scope
    auto ld = [&](unsigned e, int sp) {
        return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(part, e * 4u, (unsigned)sp * total * 4u, kDeviceScope));
    };
    for (int id = tid; id < TB * CPR; id += NT) {
        const int pix = b0 + id / CPR, ch = a0 + (id % CPR) * 4;
        if (pix >= p.rowsB || ch >= p.rowsA) continue;
        const unsigned e = (unsigned)pix * (unsigned)p.rowsA + (unsigned)ch;
        // split order, as the separate reduction kernel adds them; four loads in flight
        f32x4 sum = ld(e, 0);
        int sp = 1;
        for (; sp + 4 <= p.splits; sp += 4) {
            const f32x4 l0 = ld(e, sp), l1 = ld(e, sp + 1), l2 = ld(e, sp + 2), l3 = ld(e, sp + 3);
            sum += l0; sum += l1; sum += l2; sum += l3;
        }
        for (; sp < p.splits; ++sp) sum += ld(e, sp);
        float v[4] = {sum.x, sum.y, sum.z, sum.w};
        for (int i = 0; i < 4; ++i) {
            if (p.flags & KF_BIAS) v[i] += p.bias[ch + i];
            if (p.flags & KF_RELU) v[i] = v[i] > 0.f ? v[i] : 0.f;
            if (p.flags & KF_MASK_IN) v[i] = mask1f(v[i], p.x[e + i]);
        }
        if (p.flags & KF_OUT_F32) *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(p.out) + e) = f32x4{v[0], v[1], v[2], v[3]};
        else *reinterpret_cast<u32x2 *>(reinterpret_cast<bf16_t *>(p.out) + e) = u32x2{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
    }
}

// Tiles: A [TA][BK] (weights rows), B [TB][BK] (pixel rows), unpadded, chunk-swizzled:
// CH = BK/8 chunks per row; chunk c of row `row` sits at position c ^ ((row / RPS) % CH), RPS = rows
// per 256 bytes.  One direct-to-LDS instruction fills RPI = 64/CH consecutive rows.
// KG > 1: the block holds KG groups of WA*WB waves; group g runs the same pipeline on its own LDS stages
// over the g-th part of the block's reduction range, and the groups' sums are added through LDS in group
// order before the epilogue: a reduction split without partials in memory or a second kernel, for grids
// too small to fill the chip with one tile per block.
template <int TA, int TB, int BK, int WA, int WB, int NS, int KG = 1>
__global__ __launch_bounds__(64 * WA * WB * KG) void k_fwd_dma(const KArgs p)
{
    constexpr int NT = 64 * WA * WB * KG, NW = WA * WB;
    constexpr int CH = BK / 8, RPI = 64 / CH, RPS = 128 / BK, ROWB = BK * 2, KS = BK / 16;
    constexpr int FA = TA / WA / 32, FB = TB / WB / 32;
    constexpr int A_BYTES = TA * ROWB, B_BYTES = TB * ROWB, STAGE = A_BYTES + B_BYTES;
    constexpr int IA = TA / RPI / NW, IB = TB / RPI / NW;   // direct-to-LDS instructions per wave and step
    static_assert(IA * NW * RPI == TA && IB * NW * RPI == TB, "tile rows must divide over the waves");
    static_assert(TB <= NT, "one thread per pixel row fills the row table");
    constexpr int GSUM = (KG - 1) * NW * FA * FB * 16 * 64 * 4;   // accumulators of the extra groups on their way to group 0
    constexpr int STAGES_ALL = KG * NS * STAGE > GSUM ? KG * NS * STAGE : GSUM;
    constexpr int TILE_BYTES = STAGES_ALL > TB * (TA + 8) * 2 ? STAGES_ALL : TB * (TA + 8) * 2;  // stages / staged epilogue
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    unsigned *rowtab = reinterpret_cast<unsigned *>(smem + TILE_BYTES);   // [TB][2]
    float *bias_lds = reinterpret_cast<float *>(rowtab + 2 * TB);         // [TA]

    const ConvGeom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), grp = wv / NW, wave = wv % NW;   // wave-uniform: scalar registers
    const int tile = logical_block(blockIdx.x, gridDim.x);
    const int a0 = (tile % p.tilesA) * TA, b0 = (tile / p.tilesA) * TB;
    const int bbeg = blockIdx.y * p.steps_per_split, bend = min(bbeg + p.steps_per_split, p.steps_total);
    // every group runs nsteps pipeline steps (same barrier count); steps past its range copy zeros
    const int nsteps = (bend - bbeg + KG - 1) / KG;
    const int kbeg = bbeg + grp * nsteps, live = max(0, min(bend - kbeg, nsteps));
    const int RSC = g.R * g.S * g.C;
    __amdgpu_buffer_rsrc_t rw = make_rsrc(p.w, (size_t)g.K * RSC * 2);
    __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, (size_t)g.N * g.H * g.W * g.C * 2);

    if (tid < TB) {
        const int m = b0 + tid;
        const int n = m / (g.Ho * g.Wo), rem = m - n * (g.Ho * g.Wo), pp = rem / g.Wo, qq = rem - pp * g.Wo;
        const int hb = pp * g.sh - g.ph, wb = qq * g.sw - g.pw;
        rowtab[2 * tid] = (unsigned)(((n * g.H + hb) * g.W + wb) * g.C) * 2u;
        rowtab[2 * tid + 1] = m < p.rowsB ? tap_mask(hb, wb, 1, g.R, g.S, g.H, g.W) : 0u;
    }
    if (p.flags & KF_BIAS)
        for (int i = tid; i < TA; i += NT) bias_lds[i] = a0 + i < p.rowsA ? p.bias[a0 + i] : 0.f;
    __syncthreads();

    // lane l of instruction q of this wave fills chunk position (l % CH) of tile row
    // rq = (wave*I + q)*RPI + l / CH; that position holds global chunk (l % CH) ^ swizzle(rq)
    unsigned voffA[IA], voffB[IB], maskB[IB];
#pragma unroll
    for (int q = 0; q < IA; ++q) {
        const int row = (wave * IA + q) * RPI + lane / CH;
        const int c = (lane % CH) ^ ((row / RPS) % CH);
        voffA[q] = ((unsigned)(a0 + row) * RSC + c * 8) * 2u;
    }
#pragma unroll
    for (int q = 0; q < IB; ++q) {
        const int row = (wave * IB + q) * RPI + lane / CH;
        const int c = (lane % CH) ^ ((row / RPS) % CH);
        const u32x2 e = *reinterpret_cast<const u32x2 *>(rowtab + 2 * row);
        voffB[q] = e.x + c * 16;
        maskB[q] = e.y;
    }
    const unsigned smem_base = lds_offset(smem) + grp * NS * STAGE;   // this group's stages
    const unsigned ldsA_w = smem_base + wave * IA * 1024, ldsB_w = smem_base + A_BYTES + wave * IB * 1024;

    int kk = kbeg * BK;
    int tap = kk / g.C, c0 = kk - tap * g.C;
    int tr = tap / g.S, ts = tap - tr * g.S;
    int issued = 0;
    auto issue = [&](unsigned sb) {   // loads of the next not-yet-issued step into the stage at byte offset sb
        const bool on = KG == 1 || issued < live;
        ++issued;
        const unsigned ua = (unsigned)(tap * g.C + c0) * 2u;
        const unsigned ub = (unsigned)((tr * g.W + ts) * g.C + c0) * 2u;
        const unsigned bit = on ? 1u << (tap & 31) : 0u;
        if (p.flags & KF_NT_A) {
#pragma unroll
            for (int q = 0; q < IA; ++q) dma16_nt(rw, ldsA_w + sb + q * 1024, on ? voffA[q] + ua : OOR);
        } else {
#pragma unroll
            for (int q = 0; q < IA; ++q) dma16(rw, ldsA_w + sb + q * 1024, on ? voffA[q] + ua : OOR);
        }
#pragma unroll
        for (int q = 0; q < IB; ++q) dma16(rx, ldsB_w + sb + q * 1024, (maskB[q] & bit) ? voffB[q] + ub : OOR);
        c0 += BK;
        if (c0 >= g.C) { c0 = 0; ++tap; if (++ts == g.S) { ts = 0; ++tr; } }
    };

    f32x16 acc[FA][FB];
#pragma unroll
    for (int i = 0; i < FA; ++i)
#pragma unroll
        for (int j = 0; j < FB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    const int arow = (wave % WA) * FA * 32, brow = (wave / WA) * FB * 32;

    // fragment addresses: row (lane & 31) of a 32-row block, chunk (2*ks + (lane >> 5)) ^ swizzle(row);
    // the swizzle term is the same for every 32-row block of the wave tile
    const int rA = arow + (lane & 31), rB = brow + (lane & 31);
    unsigned fa[KS], fb[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        fa[ks] = smem_base + rA * ROWB + (((2 * ks + (lane >> 5)) ^ ((rA / RPS) % CH)) << 4);
        fb[ks] = smem_base + A_BYTES + rB * ROWB + (((2 * ks + (lane >> 5)) ^ ((rB / RPS) % CH)) << 4);
    }

    constexpr int LPS = IA + IB;   // loads per thread and step
    static_assert(KS % 2 == 0, "fragment double buffer assumes an even number of slices per step");
    // All NS stages are filled up front.  The hand-over to the next step happens before the LAST
    // slice of a step is multiplied: by then every fragment of the step is in registers, so after
    // the barrier the stage is free (the loads of step i+NS go into it) and the first fragments of
    // step i+1 are fetched while the matrix cores still work on step i.
#pragma unroll
    for (int s = 0; s < NS; ++s)
        if (s < nsteps) issue(s * STAGE);
    u32x4 fr_a[2][FA], fr_b[2][FB];
    auto wait_landed = [&](int step) {   // loads of `step` have landed; younger steps may be in flight
        const int younger = min(step + NS - 1, nsteps - 1) - step;
        if (NS >= 2 && younger == NS - 1) wait_vmcnt<(NS - 1) * LPS>();
        else if (NS >= 3 && younger == NS - 2) wait_vmcnt<(NS >= 3 ? NS - 2 : 0) * LPS>();
        else if (NS >= 4 && younger == NS - 3) wait_vmcnt<(NS >= 4 ? NS - 3 : 0) * LPS>();
        else wait_vmcnt<0>();
    };
    if (nsteps > 0) {
        wait_landed(0);
        __builtin_amdgcn_s_barrier();
        read_frags<FA, FB, 32 * ROWB>(fr_a[0], fr_b[0], fa[0], fb[0]);
    }
    unsigned sb = 0;   // byte offset of step i's stage: a running scalar, one addition per fragment address
    for (int i = 0; i < nsteps; ++i) {
        const unsigned sn = sb + STAGE == NS * STAGE ? 0u : sb + STAGE;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks < KS - 1) {
                read_frags<FA, FB, 32 * ROWB>(fr_a[(ks + 1) & 1], fr_b[(ks + 1) & 1], fa[ks + 1 < KS ? ks + 1 : 0] + sb, fb[ks + 1 < KS ? ks + 1 : 0] + sb);
                wait_frags<FA + FB, FA, FB>(fr_a[ks & 1], fr_b[ks & 1]);
            } else {
                wait_frags<0, FA, FB>(fr_a[ks & 1], fr_b[ks & 1]);   // this wave has read all it needs of the stage
                if (i + 1 < nsteps) {
                    // step i+1 was issued before step i+2 .. i+NS-1, which may still be in flight
                    const int younger = min(i + NS - 1, nsteps - 1) - (i + 1);
                    if (NS >= 3 && younger == NS - 2) wait_vmcnt<(NS - 2) * LPS>();
                    else if (NS >= 4 && younger == NS - 3) wait_vmcnt<(NS >= 4 ? NS - 3 : 0) * LPS>();
                    else wait_vmcnt<0>();
                    __builtin_amdgcn_s_barrier();
                    if (i + NS < nsteps) issue(sb);
                    read_frags<FA, FB, 32 * ROWB>(fr_a[0], fr_b[0], fa[0] + sn, fb[0] + sn);
                }
            }
#pragma unroll
            for (int ii = 0; ii < FA; ++ii)
#pragma unroll
                for (int jj = 0; jj < FB; ++jj)
                    acc[ii][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fr_a[ks & 1][ii]),
                                                                         __builtin_bit_cast(bf16x8, fr_b[ks & 1][jj]), acc[ii][jj], 0, 0, 0);
        }
        sb = sn;
    }
    __syncthreads();   // every wave is done reading the stages before they are reused for staging
    if constexpr (KG > 1) {
        // groups 1 .. KG-1 hand their sums to group 0 through LDS ([group][wave][register][lane]), added in group order
        float *gs = reinterpret_cast<float *>(smem);
        if (grp > 0) {
#pragma unroll
            for (int i = 0; i < FA; ++i)
#pragma unroll
                for (int j = 0; j < FB; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) gs[((((grp - 1) * NW + wave) * FA * FB + i * FB + j) * 16 + v) * 64 + lane] = acc[i][j][v];
        }
        __syncthreads();
        if (grp == 0) {
            for (int gq = 0; gq < KG - 1; ++gq)
#pragma unroll
                for (int i = 0; i < FA; ++i)
#pragma unroll
                    for (int j = 0; j < FB; ++j)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[i][j][v] += gs[(((gq * NW + wave) * FA * FB + i * FB + j) * 16 + v) * 64 + lane];
        }
        __syncthreads();   // the sums have been read before the staged epilogue overwrites them
    }
    if (p.splits == 1 && !(p.flags & KF_OUT_F32) && (p.rowsA & 7) == 0)
        store_staged<FA, FB, TA, TB, NT>(p, acc, reinterpret_cast<bf16_t *>(smem), bias_lds, a0, b0, arow, brow, tid, grp == 0);
    else if (grp == 0)
        store_pixel_major<FA, FB>(p, acc, a0 + arow, b0 + brow, lane, blockIdx.y);
    if (p.splits > 1 && (p.flags & KF_FUSED_REDUCE)) fused_split_reduce<TA, TB, NT>(p, tile, a0, b0, tid);
}

// A matrix instruction pinned to its place in the instruction stream (kernels with one wave per SIMD order their
// slots by hand: nothing else would hide a stall).
DEVFN void mfma_pinned(f32x16 &c, const u32x4 &a, const u32x4 &b)
{
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);   // nothing moves across: the instruction stays in its slot
}

// ---------------------------------------------------------------------------------------
// 3x3 / stride 1 / pad 1, forward and backward-data, with the pixel operand kept in LDS across the three taps
// of a filter row.  In flat pixel order (n, h, w) tap (r, s) of output pixel m reads input pixel
// m + (r-1)*W + (s-1), so the 256 pixel rows of a tile for the taps s = 0, 1, 2 of one filter row are three
// windows, one row apart, of ONE strip of 258 pixels: the strip is copied to LDS once per (filter row, channel
// block) and serves three reduction steps; only the weights are fetched every step.  Pairs (pixel, tap) that
// fall outside the image would read a neighbour's pixel from the strip; those lanes read rows of zeros instead
// (the strip buffers are 288 rows long and the rows past 258 are always filled with zeros).
// Backward-data is the same walk over dy with the filter mirrored (tap (r, s) of the walk multiplies the weights
// of tap (2-r, 2-s)); its weights are reduction-major in LDS, [64 c_out][256 c_in], and go through the LDS
// transpose read as in k_dgrad_dma; the backward of an input ReLU rides in the staged epilogue.
// One wave per SIMD (4 waves, 128x128 each: 256 accumulators leave no room for a second wave), so nothing
// hides a stall and, measured, nothing overlaps the wave's own vector instructions with its matrix
// instructions.  The loop body therefore holds matrix instructions, LDS reads and direct-to-LDS copies only:
// every per-lane address is precomputed (48 registers of pixel addresses per filter row), stage and buffer
// offsets are instruction immediates (two strips = six steps are unrolled), step offsets of the copies ride in
// the scalar offset and a copy is switched off by a zero-length buffer resource.  Reads and copies sit in
// slots between matrix instructions; a scheduling barrier after each keeps the compiler from regrouping them.
// Reduction order: filter row, channel block, filter column.  Needs reduction channels % 128 == 0.
// ---------------------------------------------------------------------------------------
template <int OFF0, int BS> DEVFN u32x4 lds_read16_at(unsigned addr, int blk)   // offset OFF0 + blk * BS as an immediate
{
    switch (blk) {
    case 0: return lds_read16<OFF0>(addr);
    case 1: return lds_read16<OFF0 + BS>(addr);
    case 2: return lds_read16<OFF0 + 2 * BS>(addr);
    case 3: return lds_read16<OFF0 + 3 * BS>(addr);
    case 4: return lds_read16<OFF0 + 4 * BS>(addr);
    case 5: return lds_read16<OFF0 + 5 * BS>(addr);
    default: return lds_read16<OFF0 + 6 * BS>(addr);
    }
}

// which fragment read j of a slice fetches: fragment index * 4 + kind (0 weights / weights low half, 1 weights high half, 2 pixels);
// order: weights of fragment f (two transposed reads on backward-data), then pixels of fragment f while there are any
constexpr int strip_read_kind(int j, bool dg, int fa, int fb)
{
    int n = 0;
    for (int f = 0; f < 8; ++f) {
        if (f < fa && n++ == j) return f * 4;
        if (f < fa && dg && n++ == j) return f * 4 + 1;
        if (f < fb && n++ == j) return f * 4 + 2;
    }
    return -1;
}

// DG: backward-data; TB: pixel rows of a tile (256; 128 for grids that would leave most CUs idle; 224 where 256 leaves the
// last round of blocks mostly empty: 7 fragments do not split over a 2 x 2 wave grid, so the four waves then each take 64
// output channels and all 224 pixel rows); TA: output channels of a tile (256, or 128 for layers with 128 of them)
template <bool DG, int TB, int TA>
__global__ __launch_bounds__(256) void k_conv_strip(const KArgs p)
{
#if __HIP_DEVICE_COMPILE__   // the host pass only needs the launch stub (and silently drops it when it sees this body)
    constexpr int WA = TB % 64 ? 4 : 2, WB = 4 / WA;   // wave grid: channels x pixels
    constexpr int BK = 64, NT = 256, FA = TA / (32 * WA), FB = TB / (32 * WB), ROWB = 128, BS = 32 * ROWB;
    constexpr int NSA = TA == 256 && TB >= 224 ? 2 : 3;   // weight stages: what fits beside the two strip buffers
    constexpr int A_BYTES = TA * ROWB, SROWS = TB > 128 ? 288 : 192, S_BYTES = SROWS * ROWB, IA = TA / 32, ISB = SROWS / 32, ZROW = TB + 16;
    constexpr int ROWA = TA * 2;   // backward-data: a weight row in LDS holds the TA c_in of one c_out
    constexpr int LDS_TILES = NSA * A_BYTES + 2 * S_BYTES;
    constexpr int NM = FA * FB;                     // matrix instructions (= slots) per slice
    constexpr int NRD = (DG ? 2 * FA : FA) + FB;   // LDS reads per slice (a transposed weight fragment takes two)
    constexpr int SPS = ISB / 3, SM0 = NM - SPS - (NM == 16 ? 5 : 0);   // strip copies per slice and their first slot
    static_assert(TA * TB <= 256 * 256 && TA * TB >= 128 * 256, "tile shapes: 256x256, 224x256, 256x128, 128x256");
    static_assert(LDS_TILES >= TB * (TA + 8) * 2, "the staged epilogue reuses the tiles");
    static_assert(A_BYTES + 4 * ROWA + 3 * BS < 65536 && S_BYTES + (FB - 1) * BS < 65536 && FA <= 4 && FB <= 7, "stage offsets fit the 16-bit immediate");
    static_assert(ISB % 3 == 0 && SM0 >= 0 && SM0 + SPS <= NM && ZROW + 2 <= SROWS && (NSA == 2 || NM % IA == 0), "slot plan");
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    unsigned *rowtab = reinterpret_cast<unsigned *>(smem + LDS_TILES);   // [TB] tap masks
    float *bias_lds = reinterpret_cast<float *>(rowtab + TB);           // [TA]

    const ConvGeom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: scalar registers
    const int tile = logical_block(blockIdx.x, gridDim.x);
    const int a0 = (tile % p.tilesA) * TA, b0 = (tile / p.tilesA) * TB;
    const int CR = DG ? g.K : g.C;   // reduction channels = channels of the pixel operand
    // a reduction split (blockIdx.y) takes CB of the CR / 64 channel blocks, all nine taps of them
    const int RSC = 9 * g.C, NHW = g.N * g.H * g.W, CB = CR / BK / p.splits, cc0 = blockIdx.y * CB, nstrips = 3 * CB, nsteps = 3 * nstrips;
    const bf16_t *pix = DG ? p.dy : p.x;
    __amdgpu_buffer_rsrc_t rw = make_rsrc(p.w, (size_t)g.K * RSC * 2), rx = make_rsrc(pix, (size_t)NHW * CR * 2);
    __amdgpu_buffer_rsrc_t rw_off = make_rsrc(p.w, 0), rx_off = make_rsrc(pix, 0);   // every lane out of range: a switched-off copy
    // Fused input-ReLU mask: the epilogue reads the tile of the saved input, which no block has touched before, while the
    // matrix cores have nothing left to do.  The strip copies of the last strip have no strip to fetch; they fetch 16 bytes
    // of every 64 bytes of that tile instead (into the idle strip buffer, never read), so that the lines are in this
    // die's L2 when the epilogue asks for them.
    const size_t mask_bytes = (size_t)p.rowsB * p.rowsA * 2;
    const bool mask_ahead = DG && (p.flags & KF_MASK_IN) && p.splits == 1 && mask_bytes < 0xffffffffull;
    __amdgpu_buffer_rsrc_t rx_last = mask_ahead ? make_rsrc(p.x, mask_bytes) : rx_off;
    if (tid < TB) {
        const int m = b0 + tid;
        const int n = m / (g.H * g.W), rem = m - n * (g.H * g.W), hh = rem / g.W, ww = rem - hh * g.W;
        rowtab[tid] = m < p.rowsB ? tap_mask(hh - 1, ww - 1, 1, 3, 3, g.H, g.W) : 0u;
    }
    if (!DG && (p.flags & KF_BIAS) && tid < TA) bias_lds[tid] = a0 + tid < p.rowsA ? p.bias[a0 + tid] : 0.f;
    __syncthreads();

    const unsigned wave_s = __builtin_amdgcn_readfirstlane(wave);
    const unsigned lds0 = lds_offset(smem), ldsS0 = lds0 + NSA * A_BYTES;
    unsigned voffA[IA], voffS[ISB], voffS_r[ISB];
    int pixS[ISB];
#pragma unroll
    for (int q = 0; q < IA; ++q) {
        if constexpr (DG) {
            // one copy fills 512 / TA reduction rows t (c_out) of 2 * TA bytes: lane l takes the 16-byte chunk (l % CPRA) ^ swizzle(t)
            constexpr int CPRA = TA / 8;
            const int t = (wave * IA + q) * (64 / CPRA) + lane / CPRA, col = a0 + ((lane % CPRA) ^ ((t & 3) << 2)) * 8;
            voffA[q] = col < g.C ? ((unsigned)t * RSC + col) * 2u : OOR;   // columns past c_in stay zero
        } else {
            // lane l of copy q fills chunk position l % 8 of tile row rq = q*8 + l/8 with global chunk (l % 8) ^ swizzle(rq)
            const int row = (wave * IA + q) * 8 + lane / 8, c = (lane % 8) ^ ((row >> 1) & 7);
            voffA[q] = ((unsigned)(a0 + row) * RSC + c * 8) * 2u;
        }
    }
#pragma unroll
    for (int q = 0; q < ISB; ++q) {
        const int row = (wave * ISB + q) * 8 + lane / 8, c = (lane % 8) ^ ((row >> 1) & 7);
        pixS[q] = row < TB + 2 ? b0 - 1 + row : -0x40000000;   // strip row j holds pixel b0 - 1 + j + (r-1)*W
        voffS[q] = ((unsigned)(b0 - 1 + row) * CR + c * 8) * 2u;
    }
    auto strip_row_offsets = [&](int rr) {   // per filter row: where each strip row comes from, OOR (zeros) outside the tensor
        const int shift = (rr - 1) * g.W;
#pragma unroll
        for (int q = 0; q < ISB; ++q)
            voffS_r[q] = (unsigned)(pixS[q] + shift) < (unsigned)NHW ? voffS[q] + (unsigned)(shift * CR) * 2u : OOR;
    };
    // the step's offset is uniform: it rides in the scalar offset, which the range check ignores (weight rows / columns past
    // the tensor are out of range by their own offset)
    auto issue_a = [&](int stage, int rr, int cc, int ss, int q, bool on) {   // weights of walk tap (rr, ss), channel block cc
        const int soff = DG ? ((cc0 + cc) * BK * RSC + ((2 - rr) * 3 + (2 - ss)) * g.C) * 2 : ((rr * 3 + ss) * g.C + (cc0 + cc) * BK) * 2;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(on ? rw : rw_off, (lds_void)(size_t)(lds0 + stage * A_BYTES + (wave_s * IA + q) * 1024), 16, voffA[q], soff, 0, 0);
    };
    auto issue_s = [&](int buf, int cc, int q, bool on) {   // strip (filter row of voffS_r, channel block cc) into strip buffer `buf`
        __builtin_amdgcn_raw_ptr_buffer_load_lds(on ? rx : rx_last, (lds_void)(size_t)(ldsS0 + buf * S_BYTES + (wave_s * ISB + q) * 1024), 16, voffS_r[q],
                                                 on ? (cc0 + cc) * BK * 2 : 0, 0, 0);
    };
    // voffS_r for the last strip's copies (`last`): one 64-byte piece of the saved-input tile per lane; a select, not a
    // branch, so that the offsets stay in registers
    auto mask_tile_offsets = [&](bool last) {
        constexpr int PPR = TA / 32;   // pieces per pixel row of the tile
        static_assert(TB * PPR <= ISB * 256, "the last strip's copies cover the tile");
#pragma unroll
        for (int q = 0; q < ISB; ++q) {
            const int piece = (wave * ISB + q) * 64 + lane, row = piece / PPR, col = a0 + (piece % PPR) * 32;
            const unsigned off = (row < TB && b0 + row < p.rowsB && col < p.rowsA) ? ((unsigned)(b0 + row) * (unsigned)p.rowsA + col) * 2u : OOR;
            voffS_r[q] = last ? off : voffS_r[q];
        }
    };

    f32x16 acc[FA][FB];
#pragma unroll
    for (int i = 0; i < FA; ++i)
#pragma unroll
        for (int j = 0; j < FB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    const int arow = (wave % WA) * (TA / WA), brow = (wave / WA) * (TB / WB);
    const int rA = arow + (lane & 31), rB = brow + (lane & 31);
    // forward: slice ks of a weight row sits at chunk (2*ks + half) ^ swizzle; backward-data: the transpose read of
    // fragment i, slice ks starts at reduction row t = 16*ks + tl, 64-byte segment (col / 32) ^ swizzle(t).
    // fa_hi: the same for the third weight stage, which a 16-bit immediate cannot reach from the first
    unsigned fa[4][DG ? FA : 1], fa_hi[4][DG ? FA : 1], fbs[3], fmask[FB], vsel[3][FB][4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        if constexpr (DG) {
            const int i16 = lane & 15, t = ks * 16 + (lane >> 5) * 8 + (i16 >> 2), cl = ((lane >> 4) & 1) * 16 + (i16 & 3) * 4;
#pragma unroll
            for (int i = 0; i < FA; ++i) {
                const int col = arow + i * 32 + cl;
                fa[ks][i] = lds0 + t * ROWA + ((((col >> 5) ^ (t & 3)) << 6) | ((col & 31) << 1));
                fa_hi[ks][i] = fa[ks][i] + 2 * A_BYTES;
            }
        } else {
            fa[ks][0] = lds0 + rA * ROWB + (((2 * ks + (lane >> 5)) ^ ((rA >> 1) & 7)) << 4);
            fa_hi[ks][0] = fa[ks][0] + 2 * A_BYTES;
        }
    }
    // pixel rows: slice ks is the slice-0 address with ks << 5 xor-ed in
#pragma unroll
    for (int ss = 0; ss < 3; ++ss) fbs[ss] = ldsS0 + (rB + ss) * ROWB + (((lane >> 5) ^ (((rB + ss) >> 1) & 7)) << 4);
#pragma unroll
    for (int j = 0; j < FB; ++j) fmask[j] = rowtab[rB + 32 * j];
    // pixel addresses of filter row rr (strip buffer 0; fragment j is read at immediate offset j * BS): the strip row, or for a
    // pair outside the image the zero rows, at the same position within 256 bytes (the same banks as the neighbours expect)
    auto select_rows = [&](int rr) {
#pragma unroll
        for (int ss = 0; ss < 3; ++ss)
#pragma unroll
            for (int j = 0; j < FB; ++j) {
                const unsigned zeros = ldsS0 + ZROW * ROWB - j * BS + (fbs[ss] & 0xF0u);
                const unsigned base = (fmask[j] >> (rr * 3 + ss)) & 1u ? fbs[ss] : zeros;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) vsel[ss][j][ks] = base ^ (ks << 5);
            }
    };

    u32x4 ra[2][4], rb[2][FB];
    u32x2 alo[2][DG ? 4 : 1], ahi[2][DG ? 4 : 1];
    // read j of slice ks of the step that uses weight stage ST, strip buffer SB and filter column ss
    auto read_slot = [&](int buf, int j, int ST, int SB, int ss, int ks) {
        const int kind = strip_read_kind(j, DG, FA, FB), f = kind >> 2;
        if ((kind & 3) == 2) {
            rb[buf][f] = SB ? lds_read16_at<S_BYTES, BS>(vsel[ss][f][ks], f) : lds_read16_at<0, BS>(vsel[ss][f][ks], f);
        } else if constexpr (DG) {
            const unsigned ad = ST == 2 ? fa_hi[ks][f] : fa[ks][f];
            if ((kind & 3) == 0) alo[buf][f] = ST == 1 ? lds_read_tr<A_BYTES>(ad) : lds_read_tr<0>(ad);
            else ahi[buf][f] = ST == 1 ? lds_read_tr<A_BYTES + 4 * ROWA>(ad) : lds_read_tr<4 * ROWA>(ad);   // 4 rows on: same swizzle class
        } else {
            const unsigned ad = ST == 2 ? fa_hi[ks][0] : fa[ks][0];
            ra[buf][f] = ST == 1 ? lds_read16_at<A_BYTES, BS>(ad, f) : lds_read16_at<0, BS>(ad, f);
        }
    };
    // the reads of a slice sit in the first slots, one per slot (two in the first slots if there are more reads than slots)
    auto read_slots = [&](int m, int buf, int ST, int SB, int ss, int ks) {
#pragma unroll
        for (int j = 0; j < NRD; ++j) {
            const int slot = NRD <= NM ? j : (j < 2 * (NRD - NM) ? j / 2 : j - (NRD - NM));
            if (slot == m) read_slot(buf, j, ST, SB, ss, ks);
        }
    };
    auto landed = [&](int buf) {   // the LDS reads so far have arrived; the fragments depend on the wait
        asm volatile("s_waitcnt lgkmcnt(0)");
#pragma unroll
        for (int f = 0; f < FA; ++f) {
            if constexpr (DG) { asm volatile("" : "+v"(alo[buf][f])); asm volatile("" : "+v"(ahi[buf][f])); }
            else asm volatile("" : "+v"(ra[buf][f]));
        }
#pragma unroll
        for (int f = 0; f < FB; ++f) asm volatile("" : "+v"(rb[buf][f]));
    };
    auto multiply = [&](int buf, int m) {
        if constexpr (DG) {
            const u32x4 av = {alo[buf][m / FB].x, alo[buf][m / FB].y, ahi[buf][m / FB].x, ahi[buf][m / FB].y};
            mfma_pinned(acc[m / FB][m % FB], av, rb[buf][m % FB]);
        } else {
            mfma_pinned(acc[m / FB][m % FB], ra[buf][m / FB], rb[buf][m % FB]);
        }
    };

    // prologue: strip 0 and the weights of the first steps (two stages: step 0 and half of step 1; three: steps 0, 1, 2)
    strip_row_offsets(0);
    int row_loaded = 0;   // filter row of voffS_r
#pragma unroll
    for (int q = 0; q < ISB; ++q) issue_s(0, 0, q, true);
#pragma unroll
    for (int q = 0; q < IA; ++q) issue_a(0, 0, 0, 0, q, true);
    if constexpr (NSA == 2) {
#pragma unroll
        for (int q = 0; q < IA / 2; ++q) issue_a(1, 0, 0, 1, q, true);   // the second half follows in the first slice of step 0
    } else {
#pragma unroll
        for (int q = 0; q < IA; ++q) issue_a(1, 0, 0, 1, q, true);
#pragma unroll
        for (int q = 0; q < IA; ++q) issue_a(2, 0, 0, 2, q, true);
    }
    select_rows(0);
    wait_vmcnt<NSA == 2 ? IA / 2 : 2 * IA>();
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int m = 0; m < NM; ++m) read_slots(m, 0, 0, 0, 0, 0);

    int rr = 0, cc = 0;   // filter row and channel block of strip gg
    // one strip = three steps; SB = gg & 1 is the strip's buffer, and with it the parity of its first step
    auto strip_steps = [&](int gg, auto sbc) {
        constexpr int SB = decltype(sbc)::value;
        const bool more_strips = gg + 1 < nstrips;
        const int ccn = cc + 1 == CB ? 0 : cc + 1, rrn = cc + 1 == CB ? rr + 1 : rr;   // strip gg + 1
        if (rrn != row_loaded && rrn < 3) { strip_row_offsets(rrn); row_loaded = rrn; }
        mask_tile_offsets(!more_strips && mask_ahead);   // voffS_r has no strip left to describe
#pragma unroll
        for (int ss = 0; ss < 3; ++ss) {
            const int i = 3 * gg + ss;
            const int ST = NSA == 2 ? (SB + ss) & 1 : ss, STN = NSA == 2 ? ST ^ 1 : (ss + 1) % 3;   // weight stages of steps i, i+1
#pragma unroll
            for (int ks = 0; ks < 3; ++ks) {
                landed(ks & 1);
#pragma unroll
                for (int m = 0; m < NM; ++m) {
                    read_slots(m, (ks + 1) & 1, ST, SB, ss, ks + 1);
                    // two stages: second half of the weights of step i+1 (the first half went out after the last barrier),
                    // two slots apart (the address unit takes 16 clocks per copy) and all of them BEFORE the strip copies
                    // below: the wait at the barrier counts on the strip copies being the youngest
                    if (NSA == 2 && ks == 0 && m < 8 && (m & 1))
                        issue_a(STN, ss < 2 ? rr : rrn, ss < 2 ? cc : ccn, (ss + 1) % 3, IA / 2 + (m >> 1), i + 1 < nsteps);
                    // the strip after this one goes into the buffer the previous strip has left: SPS copies per slice
                    if (ss == 0 && m >= SM0 && m < SM0 + SPS) issue_s(SB ^ 1, ccn, ks * SPS + m - SM0, more_strips);
                    multiply(ks & 1, m);
                }
            }
            landed(1);   // the last slice is in registers: this wave is done with the weight stage
            if (ss == 2 && rrn != rr && rrn < 3) select_rows(rrn);   // the reads below already belong to the next filter row
            // the weights of step i+1 have landed; younger copies may be in flight: with two stages the strip copies of this
            // step; with three the weights of step i+2 and the strip copies issued after those of step i+1 (this step's if
            // ss == 0, the previous step's if ss == 1)
            if constexpr (NSA == 2) { if (ss == 0) wait_vmcnt<ISB>(); else wait_vmcnt<0>(); }
            else { if (ss == 2) wait_vmcnt<IA>(); else wait_vmcnt<IA + ISB>(); }
            __builtin_amdgcn_s_barrier();
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                read_slots(m, 0, STN, ss < 2 ? SB : SB ^ 1, (ss + 1) % 3, 0);
                if constexpr (NSA == 2) {
                    // first half of the weights of step i+2 into the stage just freed: same strip while ss + 2 < 3, else the next
                    if ((m & 3) == 1) issue_a(ST, ss == 0 ? rr : rrn, ss == 0 ? cc : ccn, (ss + 2) % 3, m >> 2, i + 2 < nsteps);
                } else {
                    if (m % (NM / IA) == 0) issue_a(ST, rrn, ccn, ss, m / (NM / IA), i + 3 < nsteps);   // weights of step i+3 (same column of the next strip)
                }
                multiply(1, m);
            }
        }
        rr = rrn; cc = ccn;
    };
    for (int gg = 0; gg < nstrips; gg += 2) {   // reduction channels % 128 == 0: an even number of strips per filter row
        strip_steps(gg, std::integral_constant<int, 0>());
        strip_steps(gg + 1, std::integral_constant<int, 1>());
    }
    wait_vmcnt<0>();   // switched-off copies still write zeros: they are done before the tiles are reused
    if (p.splits > 1) {   // fp32 partial sums [split][pixel][channel]; the split-reduce kernel applies the epilogue
        float *part = p.partial + (size_t)blockIdx.y * p.rowsB * p.rowsA;
#pragma unroll
        for (int i = 0; i < FA; ++i)
#pragma unroll
            for (int j = 0; j < FB; ++j) {
                const int pixel = b0 + brow + j * 32 + (lane & 31);
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int ch = a0 + arow + i * 32 + 8 * gq + 4 * (lane >> 5);   // rowsA % 8 == 0: whole groups of four
                    if (pixel < p.rowsB && ch < p.rowsA)
                        *reinterpret_cast<f32x4 *>(part + (size_t)pixel * p.rowsA + ch) =
                            f32x4{acc[i][j][4 * gq], acc[i][j][4 * gq + 1], acc[i][j][4 * gq + 2], acc[i][j][4 * gq + 3]};
                }
            }
        return;
    }
    __syncthreads();
    store_staged<FA, FB, TA, TB, NT>(p, acc, reinterpret_cast<bf16_t *>(smem), bias_lds, a0, b0, arow, brow, tid);
#endif
}
constexpr int strip_lds_bytes(int ta, int tb) { return (ta == 256 && tb >= 224 ? 2 : 3) * ta * 128 + 2 * (tb > 128 ? 288 : 192) * 128 + tb * 4 + ta * 4; }

// ---------------------------------------------------------------------------------------
// backward-filter with the same pipeline.  Both operands are reduction-major in LDS:
// A [BK pixels][TA c_out], B [BK pixels][TB taps]; fragments come from the LDS transpose read.
// Rows are T*2 bytes; the 64-byte segment g of reduction row t sits at segment g ^ swz(t) so that
// the four rows one transpose read touches fall into distinct banks.  One direct-to-LDS
// instruction fills 512/T reduction rows.  The x offsets change every step: threads t < BK keep a
// table {pixel base, tap mask} for the steps in flight, written and read with inline assembly
// for the same reason as the fragment reads.
// ---------------------------------------------------------------------------------------
template <int TA, int TB, int BK, int WA, int WB, int NS>
__global__ __launch_bounds__(64 * WA * WB) void k_wgrad_dma(const KArgs p)
{
    constexpr int NT = 64 * WA * WB, NW = WA * WB, KS = BK / 16;
    constexpr int FA = TA / WA / 32, FB = TB / WB / 32;
    constexpr int ROWA = TA * 2, ROWB = TB * 2;                  // bytes per reduction row
    constexpr int A_BYTES = BK * ROWA, B_BYTES = BK * ROWB, STAGE = A_BYTES + B_BYTES;
    constexpr int RPIA = 512 / TA, RPIB = 512 / TB;              // reduction rows per direct-to-LDS instruction
    constexpr int IA = BK / RPIA / NW, IB = BK / RPIB / NW;
    static_assert(IA * NW * RPIA == BK && IB * NW * RPIB == BK, "reduction rows must divide over the waves");
    // pixel table: {byte offset of the pixel's top-left tap in x, valid-tap mask} for TABN consecutive
    // reduction rows, two such chunks (the one the loads in flight read and the next one)
    constexpr int TABN = NT, SPC = TABN / BK;   // table entries and steps per chunk
    static_assert(TABN % BK == 0 && SPC >= NS, "a chunk holds whole steps and at least one pipeline depth");
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const unsigned smem_base = lds_offset(smem);
    const unsigned tab_base = smem_base + NS * STAGE;            // [2][TABN] x {base, mask}

    const ConvGeom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: scalar registers
    // grid = (splits, tiles): consecutive workgroup ids go round-robin to the 8 XCDs, so with the
    // split as the fast index (and a split count that is a multiple of 8) every block that reads a
    // given pixel range of x and dy runs on the same XCD and shares that XCD's L2
    const int tile = blockIdx.y, split = blockIdx.x;
    const int a0 = (tile % p.tilesA) * TA, b0 = (tile / p.tilesA) * TB;
    const int kbeg = split * p.steps_per_split, kend = min(kbeg + p.steps_per_split, p.steps_total);
    const int nsteps = kend - kbeg;
    const int M = p.red;
    __amdgpu_buffer_rsrc_t rdy = make_rsrc(p.dy, (size_t)M * g.K * 2);
    __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, (size_t)g.N * g.H * g.W * g.C * 2);

    // lane l of instruction q fills chunk position l % (T/8) of reduction row tq = (wave*I + q)*RPI + l / (T/8)
    unsigned voffA[IA];
#pragma unroll
    for (int q = 0; q < IA; ++q) {
        const int t = (wave * IA + q) * RPIA + lane / (TA / 8);
        const int c = (lane % (TA / 8)) ^ (seg_swz<TA>(t) << 2);
        voffA[q] = ((unsigned)t * g.K + a0 + c * 8) * 2u;
    }
    unsigned coffB[IB], bitB[IB], tabB[IB];
#pragma unroll
    for (int q = 0; q < IB; ++q) {
        const int t = (wave * IB + q) * RPIB + lane / (TB / 8);
        const int c = (lane % (TB / 8)) ^ (seg_swz<TB>(t) << 2);
        const int col = b0 + c * 8;
        const int tapi = col / g.C, ch = col - tapi * g.C, r = tapi / g.S, s = tapi - r * g.S;
        coffB[q] = (unsigned)((r * g.W + s) * g.C + ch) * 2u;
        bitB[q] = col < p.rowsB ? 1u << tapi : 0u;
        tabB[q] = tab_base + t * 8;
    }
    const unsigned ldsA_w = smem_base + wave * IA * 1024, ldsB_w = smem_base + A_BYTES + wave * IB * 1024;

    // every thread fills one entry of chunk `chunk` (reduction rows kbeg*BK + chunk*TABN + tid)
    auto fill_table = [&](int chunk) {
        const int m = kbeg * BK + chunk * TABN + tid;
        const int n = m / (g.Ho * g.Wo), rem = m - n * (g.Ho * g.Wo), pp = rem / g.Wo, pq = rem - pp * g.Wo;
        const int hb = pp * g.sh - g.ph, wb = pq * g.sw - g.pw;
        u32x2 e;
        e.x = (unsigned)(((n * g.H + hb) * g.W + wb) * g.C) * 2u;
        e.y = m < M ? tap_mask(hb, wb, 1, g.R, g.S, g.H, g.W) : 0u;
        const unsigned addr = tab_base + ((chunk & 1) * TABN + tid) * 8;
        asm volatile("ds_write_b64 %0, %1" ::"v"(addr), "v"(e) : "memory");
    };
    auto issue = [&](unsigned sb, int ls) {   // sb: byte offset of the stage to fill; ls: step index relative to kbeg
        const unsigned ua = (unsigned)(kbeg + ls) * BK * g.K * 2u;
        const unsigned tb = (unsigned)(ls % (2 * SPC)) * BK * 8;
        u32x2 e[IB];
#pragma unroll
        for (int q = 0; q < IB; ++q)
            asm volatile("ds_read_b64 %0, %1" : "=v"(e[q]) : "v"(tabB[q] + tb));
#pragma unroll
        for (int q = 0; q < IA; ++q) dma16(rdy, ldsA_w + sb + q * 1024, voffA[q] + ua);
        asm volatile("s_waitcnt lgkmcnt(0)");
#pragma unroll
        for (int q = 0; q < IB; ++q) asm volatile("" : "+v"(e[q]));
#pragma unroll
        for (int q = 0; q < IB; ++q) dma16(rx, ldsB_w + sb + q * 1024, (e[q].y & bitB[q]) ? e[q].x + coffB[q] : OOR);
    };

    f32x16 acc[FA][FB];
#pragma unroll
    for (int i = 0; i < FA; ++i)
#pragma unroll
        for (int j = 0; j < FB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    const int arow = (wave % WA) * FA * 32, brow = (wave / WA) * FB * 32;
    // fused bias gradient: the column sums of the dy^T fragments, by a 16x16x32 matrix instruction against a 0/1 selector
    // (half the time of the 32x32x16 form against ones, a quarter of its accumulators).  All blocks of a (c_out tile, split)
    // hold the same dy; the tile's TA/32 fragments are dealt over these tilesB blocks and, within a block, over the WB waves
    // that share the fragment's rows, so that no wave carries more than its share: fragment f belongs to block f % tilesB,
    // wave column (f / tilesB) % WB.  One writer per row of the [split][c_out] partial.
    const int wb_ = wave / WA;
    unsigned db_mask = 0;   // bit ii: this wave sums its fragment ii
    if (p.flags & KF_DB) {
        const int tb = tile / p.tilesA;
#pragma unroll
        for (int ii = 0; ii < FA; ++ii) {
            const int f = (wave % WA) * FA + ii;
            if (f % p.tilesB == tb && (f / p.tilesB) % WB == wb_) db_mask |= 1u << ii;
        }
    }
    db_mask = __builtin_amdgcn_readfirstlane(db_mask);
    const bool do_db = db_mask != 0;
    const bf16x8 db_sel = colsum_selector(lane);
    f32x4 accdb[FA];
#pragma unroll
    for (int i = 0; i < FA; ++i) accdb[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    // transpose-read addresses: lane l of a 16-lane block points at reduction row ks*16 + 8*(l>>5) + (l&15)/4
    // (and 4 rows further for the second half), operand rows row0 + 16*((l>>4)&1) + 4*(l&3) .. +3
    unsigned fa[KS][FA], fb[KS][FB];
    {
        const int i16 = lane & 15, tl = (lane >> 5) * 8 + (i16 >> 2), cl = ((lane >> 4) & 1) * 16 + (i16 & 3) * 4;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int t = ks * 16 + tl;   // the second read of a fragment is row t + 4, which has the same swizzle term
#pragma unroll
            for (int i = 0; i < FA; ++i) {
                const int col = arow + i * 32 + cl;
                fa[ks][i] = smem_base + t * ROWA + ((((col >> 5) ^ seg_swz<TA>(t)) << 6) | ((col & 31) << 1));
            }
#pragma unroll
            for (int j = 0; j < FB; ++j) {
                const int col = brow + j * 32 + cl;
                fb[ks][j] = smem_base + A_BYTES + t * ROWB + ((((col >> 5) ^ seg_swz<TB>(t)) << 6) | ((col & 31) << 1));
            }
        }
    }

    constexpr int LPS = IA + IB;
    fill_table(0);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __syncthreads();
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < nsteps) issue(s * STAGE, s);
    unsigned sb = 0, sfill = (NS - 1) * STAGE;   // stage of step i and the stage step i-1 used (filled next): running scalars
    for (int i = 0; i < nsteps; sfill = sb, sb = sb + STAGE == NS * STAGE ? 0u : sb + STAGE, ++i) {
        const int younger = min(nsteps - 1 - i, NS - 2);
        if (NS >= 3 && younger == NS - 2) wait_vmcnt<(NS - 2) * LPS>();
        else if (NS >= 4 && younger == NS - 3) wait_vmcnt<(NS >= 4 ? NS - 3 : 0) * LPS>();
        else wait_vmcnt<0>();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave's table writes are done
        __builtin_amdgcn_s_barrier();
        // at the first step of chunk c the entries of chunk c-1 have all been read (the last load that
        // used them was issued NS-1 steps ago, before a barrier): its half of the table takes chunk c+1,
        // whose first reader is the issue NS-1 steps before that chunk starts, after at least one barrier
        if (i % SPC == 0 && (i / SPC + 1) * SPC < nsteps + NS) fill_table(i / SPC + 1);
        if (i + NS - 1 < nsteps) issue(sfill, i + NS - 1);
        // fragments are double-buffered in registers: the transpose reads of slice ks+1 are issued
        // before the matrix instructions of slice ks
        u32x2 alo[2][FA], ahi[2][FA], blo[2][FB], bhi[2][FB];
        auto read_slice = [&](int ks, int buf) {
#pragma unroll
            for (int ii = 0; ii < FA; ++ii) {
                alo[buf][ii] = lds_read_tr<0>(fa[ks][ii] + sb);
                ahi[buf][ii] = lds_read_tr<4 * ROWA>(fa[ks][ii] + sb);   // 4 reduction rows further: same swizzle class
            }
#pragma unroll
            for (int jj = 0; jj < FB; ++jj) {
                blo[buf][jj] = lds_read_tr<0>(fb[ks][jj] + sb);
                bhi[buf][jj] = lds_read_tr<4 * ROWB>(fb[ks][jj] + sb);
            }
        };
        read_slice(0, 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int cur = ks & 1;
            if (ks < KS - 1) {
                read_slice(ks + 1 < KS ? ks + 1 : 0, cur ^ 1);
                static_assert(2 * (FA + FB) < 16, "lgkmcnt is a 4-bit counter");
                asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(2 * (FA + FB)));
            } else {
                asm volatile("s_waitcnt lgkmcnt(0)");
            }
#pragma unroll
            for (int ii = 0; ii < FA; ++ii) { asm volatile("" : "+v"(alo[cur][ii])); asm volatile("" : "+v"(ahi[cur][ii])); }
#pragma unroll
            for (int jj = 0; jj < FB; ++jj) { asm volatile("" : "+v"(blo[cur][jj])); asm volatile("" : "+v"(bhi[cur][jj])); }
#pragma unroll
            for (int ii = 0; ii < FA; ++ii)
#pragma unroll
                for (int jj = 0; jj < FB; ++jj) {
                    const u32x4 av = {alo[cur][ii].x, alo[cur][ii].y, ahi[cur][ii].x, ahi[cur][ii].y};
                    const u32x4 bv = {blo[cur][jj].x, blo[cur][jj].y, bhi[cur][jj].x, bhi[cur][jj].y};
                    acc[ii][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, bv),
                                                                         acc[ii][jj], 0, 0, 0);
                }
            if (do_db) {
#pragma unroll
                for (int ii = 0; ii < FA; ++ii)
                    if ((db_mask >> ii) & 1u) {
                        const u32x4 av = {alo[cur][ii].x, alo[cur][ii].y, ahi[cur][ii].x, ahi[cur][ii].y};
                        accdb[ii] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av), db_sel, accdb[ii], 0, 0, 0);
                    }
            }
        }
    }
    store_row_major<FA, FB>(p, acc, a0 + arow, b0 + brow, lane, split);
    if (do_db) {
#pragma unroll
        for (int ii = 0; ii < FA; ++ii)
            if ((db_mask >> ii) & 1u) store_colsum_fragment(accdb[ii], p.dbp + (size_t)split * p.rowsA, a0 + arow + ii * 32, p.rowsA, lane);
    }
}

// ---------------------------------------------------------------------------------------
// backward-data (c_out % BK == 0; any stride) with the same pipeline: A = weights, reduction-major
// [BK c_out rows][TA c_in] read through the LDS transpose read; B = dy pixel rows, K-major.
// ---------------------------------------------------------------------------------------
template <int TA, int TB, int BK, int WA, int WB, int NS, int KG = 1>   // KG: reduction groups per block, as in k_fwd_dma
__global__ __launch_bounds__(64 * WA * WB * KG) void k_dgrad_dma(const KArgs p)
{
    constexpr int NT = 64 * WA * WB * KG, NW = WA * WB;
    constexpr int CH = BK / 8, RPI = 64 / CH, RPS = 128 / BK, ROWB = BK * 2, KS = BK / 16;
    constexpr int FA = TA / WA / 32, FB = TB / WB / 32;
    constexpr int ROWA = TA * 2, RPIA = 512 / TA;
    constexpr int A_BYTES = BK * ROWA, B_BYTES = TB * ROWB, STAGE = A_BYTES + B_BYTES;
    constexpr int IA = BK / RPIA / NW, IB = TB / RPI / NW;
    static_assert(IA * NW * RPIA == BK && IB * NW * RPI == TB, "tile rows must divide over the waves");
    static_assert(TB <= NT, "one thread per pixel row fills the row table");
    constexpr int GSUM = (KG - 1) * NW * FA * FB * 16 * 64 * 4;
    constexpr int STAGES_ALL = KG * NS * STAGE > GSUM ? KG * NS * STAGE : GSUM;
    constexpr int TILE_BYTES = STAGES_ALL > TB * (TA + 8) * 2 ? STAGES_ALL : TB * (TA + 8) * 2;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    unsigned *rowtab = reinterpret_cast<unsigned *>(smem + TILE_BYTES);   // [TB][2]
    float *bias_lds = reinterpret_cast<float *>(rowtab + 2 * TB);         // unused (no bias in this pass)

    const ConvGeom &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), grp = wv / NW, wave = wv % NW;   // wave-uniform: scalar registers
    const int tile = logical_block(blockIdx.x, gridDim.x);
    const int a0 = (tile % p.tilesA) * TA, tb = tile / p.tilesA, b0 = tb * TB;
    // Stride phases (p.ph_on): a tile holds input pixels of one phase (h % sh, w % sw) = (pa, pb) only.  Of the R*S taps
    // only those with r = (pa + ph) mod sh, s = (pb + pw) mod sw can hit the output grid for such a pixel, so the
    // reduction walks that sub-lattice of taps: 1/(sh*sw) of the steps the masked form multiplies.
    int pa = 0, pb = 0, Hc = g.H, Wc = g.W, ml0 = b0;           // phase, its pixel grid, first phase-local row of the tile
    int tap_r0 = 0, tap_s0 = 0, step_r = 1, step_s = 1, tap_ns = g.S, ntaps = g.R * g.S;
    if (p.ph_on) {
        int cls = 0;
        while (cls + 1 < g.sh * g.sw && tb >= p.ph_tile0[cls + 1]) ++cls;
        pa = cls / g.sw; pb = cls - pa * g.sw;
        Hc = (g.H - pa + g.sh - 1) / g.sh; Wc = (g.W - pb + g.sw - 1) / g.sw;
        ml0 = (tb - p.ph_tile0[cls]) * TB;
        tap_r0 = (pa + g.ph) % g.sh; tap_s0 = (pb + g.pw) % g.sw; step_r = g.sh; step_s = g.sw;
        const int tap_nr = tap_r0 < g.R ? (g.R - tap_r0 + g.sh - 1) / g.sh : 0;
        tap_ns = tap_s0 < g.S ? (g.S - tap_s0 + g.sw - 1) / g.sw : 0;
        ntaps = tap_nr * tap_ns;
    }
    const int steps_tile = p.ph_on ? ntaps * (g.K / BK) : p.steps_total;
    const int bbeg = blockIdx.y * p.steps_per_split, bend = min(bbeg + p.steps_per_split, steps_tile);
    const int nsteps = (max(bend - bbeg, 0) + KG - 1) / KG;
    const int kbeg = bbeg + grp * nsteps, live = max(0, min(bend - kbeg, nsteps));
    const int RSC = g.R * g.S * g.C;
    __amdgpu_buffer_rsrc_t rw = make_rsrc(p.w, (size_t)g.K * RSC * 2);
    __amdgpu_buffer_rsrc_t rdy = make_rsrc(p.dy, (size_t)g.N * g.Ho * g.Wo * g.K * 2);
    int *rowpix = reinterpret_cast<int *>(bias_lds + TA);   // [TB] linear index of each tile row's input pixel, -1: none

    if (tid < TB) {
        int n, hh, ww;
        bool valid;
        if (p.ph_on) {
            const int ml = ml0 + tid, per = Hc * Wc;
            valid = per > 0 && ml < g.N * per;
            n = valid ? ml / per : 0;
            const int rem = ml - n * per, i = Wc > 0 ? rem / Wc : 0;
            hh = i * g.sh + pa; ww = (rem - i * Wc) * g.sw + pb;
        } else {
            const int m = b0 + tid;
            valid = m < p.rowsB;
            n = m / (g.H * g.W);
            const int rem = m - n * (g.H * g.W);
            hh = rem / g.W; ww = rem - hh * g.W;
        }
        // the output pixel of tap (r, s) is ((hb - r) / sh, (wb - s) / sw) when both divisions are exact; for such a tap
        // (hb - r) / sh == hb / sh - r / sh, so the row base uses hb / sh and every tap adds a wave-uniform offset
        const int hb = hh + g.ph, wb = ww + g.pw;
        rowtab[2 * tid] = (unsigned)(((n * g.Ho + hb / g.sh) * g.Wo + wb / g.sw) * g.K) * 2u;
        unsigned mask = 0;
        if (valid) {
            unsigned smask = 0;
            for (int s = 0; s < g.S; ++s) {
                const int d = wb - s;
                if (d >= 0 && d % g.sw == 0 && d / g.sw < g.Wo) smask |= 1u << s;
            }
            for (int r = 0; r < g.R; ++r) {
                const int d = hb - r;
                if (d >= 0 && d % g.sh == 0 && d / g.sh < g.Ho) mask |= smask << (r * g.S);
            }
        }
        rowtab[2 * tid + 1] = mask;
        rowpix[tid] = valid ? (n * g.H + hh) * g.W + ww : -1;
    }
    __syncthreads();

    unsigned voffA[IA], voffB[IB], maskB[IB];
#pragma unroll
    for (int q = 0; q < IA; ++q) {
        const int t = (wave * IA + q) * RPIA + lane / (TA / 8);
        const int c = (lane % (TA / 8)) ^ (seg_swz<TA>(t) << 2);
        voffA[q] = ((unsigned)t * RSC + a0 + c * 8) * 2u;
    }
#pragma unroll
    for (int q = 0; q < IB; ++q) {
        const int row = (wave * IB + q) * RPI + lane / CH;
        const int c = (lane % CH) ^ ((row / RPS) % CH);
        const u32x2 e = *reinterpret_cast<const u32x2 *>(rowtab + 2 * row);
        voffB[q] = e.x + c * 16;
        maskB[q] = e.y;
    }
    const unsigned smem_base = lds_offset(smem) + grp * NS * STAGE;   // this group's stages
    const unsigned ldsA_w = smem_base + wave * IA * 1024, ldsB_w = smem_base + A_BYTES + wave * IB * 1024;

    // position in the tap sub-lattice: list index li -> (tap_r0 + (li / tap_ns) * step_r, tap_s0 + (li % tap_ns) * step_s)
    int kk = kbeg * BK;
    const int li0 = kk / g.K;
    int c0 = kk - li0 * g.K;
    int tr = tap_r0 + (tap_ns > 0 ? li0 / tap_ns : 0) * step_r, ts = tap_s0 + (tap_ns > 0 ? li0 % tap_ns : 0) * step_s;
    int tap = tr * g.S + ts;
    // output-pixel offset of the tap, in dy rows: recomputed only when the tap changes (the divisions stay out of the
    // steady-state step; stride 1 needs none)
    auto tap_rows = [&]() { return (g.sh == 1 ? tr : tr / g.sh) * g.Wo + (g.sw == 1 ? ts : ts / g.sw); };
    int trow = tap_rows();
    int issued = 0;
    auto issue = [&](unsigned sb) {   // sb: byte offset of the stage to fill
        const bool on = KG == 1 || issued < live;
        ++issued;
        const unsigned ua = ((unsigned)c0 * RSC + (unsigned)tap * g.C) * 2u;
        const unsigned ub = (unsigned)(c0 - trow * g.K) * 2u;
        const unsigned bit = on ? 1u << (tap & 31) : 0u;
        if (p.flags & KF_NT_A) {
#pragma unroll
            for (int q = 0; q < IA; ++q) dma16_nt(rw, ldsA_w + sb + q * 1024, on ? voffA[q] + ua : OOR);
        } else {
#pragma unroll
            for (int q = 0; q < IA; ++q) dma16(rw, ldsA_w + sb + q * 1024, on ? voffA[q] + ua : OOR);
        }
#pragma unroll
        for (int q = 0; q < IB; ++q) dma16(rdy, ldsB_w + sb + q * 1024, (maskB[q] & bit) ? voffB[q] + ub : OOR);
        c0 += BK;
        if (c0 >= g.K) {
            c0 = 0;
            ts += step_s;
            if (ts >= g.S) { ts = tap_s0; tr += step_r; }
            tap = tr * g.S + ts;
            trow = tap_rows();
        }
    };

    f32x16 acc[FA][FB];
#pragma unroll
    for (int i = 0; i < FA; ++i)
#pragma unroll
        for (int j = 0; j < FB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    const int arow = (wave % WA) * FA * 32, brow = (wave / WA) * FB * 32;

    unsigned fa[KS][FA], fb[KS];
    {
        const int i16 = lane & 15, tl = (lane >> 5) * 8 + (i16 >> 2), cl = ((lane >> 4) & 1) * 16 + (i16 & 3) * 4;
        const int rB = brow + (lane & 31);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int t = ks * 16 + tl;
#pragma unroll
            for (int i = 0; i < FA; ++i) {
                const int col = arow + i * 32 + cl;
                fa[ks][i] = smem_base + t * ROWA + ((((col >> 5) ^ seg_swz<TA>(t)) << 6) | ((col & 31) << 1));
            }
            fb[ks] = smem_base + A_BYTES + rB * ROWB + (((2 * ks + (lane >> 5)) ^ ((rB / RPS) % CH)) << 4);
        }
    }

    constexpr int LPS = IA + IB;
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < nsteps) issue(s * STAGE);
    unsigned sb = 0, sfill = (NS - 1) * STAGE;   // stage of step i and the stage step i-1 used (filled next): running scalars
    for (int i = 0; i < nsteps; sfill = sb, sb = sb + STAGE == NS * STAGE ? 0u : sb + STAGE, ++i) {
        const int younger = min(nsteps - 1 - i, NS - 2);
        if (NS >= 3 && younger == NS - 2) wait_vmcnt<(NS - 2) * LPS>();
        else if (NS >= 4 && younger == NS - 3) wait_vmcnt<(NS >= 4 ? NS - 3 : 0) * LPS>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (i + NS - 1 < nsteps) issue(sfill);
        // fragments are double-buffered in registers: the reads of slice ks+1 are issued before the
        // matrix instructions of slice ks
        u32x2 alo[2][FA], ahi[2][FA];
        u32x4 b[2][FB];
        auto read_slice = [&](int ks, int buf) {
#pragma unroll
            for (int ii = 0; ii < FA; ++ii) {
                alo[buf][ii] = lds_read_tr<0>(fa[ks][ii] + sb);
                ahi[buf][ii] = lds_read_tr<4 * ROWA>(fa[ks][ii] + sb);
            }
            if constexpr (FB >= 1) b[buf][0] = lds_read16<0>(fb[ks] + sb);
            if constexpr (FB >= 2) b[buf][1] = lds_read16<32 * ROWB>(fb[ks] + sb);
            if constexpr (FB >= 3) b[buf][2] = lds_read16<64 * ROWB>(fb[ks] + sb);
            if constexpr (FB >= 4) b[buf][3] = lds_read16<96 * ROWB>(fb[ks] + sb);
        };
        read_slice(0, 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int cur = ks & 1;
            if (ks < KS - 1) {
                read_slice(ks + 1 < KS ? ks + 1 : 0, cur ^ 1);
                static_assert(2 * FA + FB < 16, "lgkmcnt is a 4-bit counter");
                asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(2 * FA + FB));
            } else {
                asm volatile("s_waitcnt lgkmcnt(0)");
            }
#pragma unroll
            for (int ii = 0; ii < FA; ++ii) { asm volatile("" : "+v"(alo[cur][ii])); asm volatile("" : "+v"(ahi[cur][ii])); }
#pragma unroll
            for (int jj = 0; jj < FB; ++jj) asm volatile("" : "+v"(b[cur][jj]));
#pragma unroll
            for (int ii = 0; ii < FA; ++ii)
#pragma unroll
                for (int jj = 0; jj < FB; ++jj) {
                    const u32x4 av = {alo[cur][ii].x, alo[cur][ii].y, ahi[cur][ii].x, ahi[cur][ii].y};
                    acc[ii][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, b[cur][jj]),
                                                                         acc[ii][jj], 0, 0, 0);
                }
        }
    }
    __syncthreads();
    if constexpr (KG > 1) {
        float *gs = reinterpret_cast<float *>(smem);
        if (grp > 0) {
#pragma unroll
            for (int i = 0; i < FA; ++i)
#pragma unroll
                for (int j = 0; j < FB; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) gs[((((grp - 1) * NW + wave) * FA * FB + i * FB + j) * 16 + v) * 64 + lane] = acc[i][j][v];
        }
        __syncthreads();
        if (grp == 0) {
            for (int gq = 0; gq < KG - 1; ++gq)
#pragma unroll
                for (int i = 0; i < FA; ++i)
#pragma unroll
                    for (int j = 0; j < FB; ++j)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[i][j][v] += gs[(((gq * NW + wave) * FA * FB + i * FB + j) * 16 + v) * 64 + lane];
        }
        __syncthreads();
    }
    if (p.splits == 1 && !(p.flags & KF_OUT_F32) && (p.rowsA & 7) == 0)
        store_staged<FA, FB, TA, TB, NT>(p, acc, reinterpret_cast<bf16_t *>(smem), bias_lds, a0, b0, arow, brow, tid, grp == 0, rowpix, steps_tile == 0);
    else if (grp == 0)
        store_pixel_major<FA, FB>(p, acc, a0 + arow, b0 + brow, lane, blockIdx.y);
    if (p.splits > 1 && (p.flags & KF_FUSED_REDUCE)) fused_split_reduce<TA, TB, NT>(p, tile, a0, b0, tid);
}

struct DmaVariant { int TA, TB, BK, WA, WB, NS, KG = 1; };
const DmaVariant kDma[] = {{128, 128, 64, 2, 2, 2}, {128, 128, 32, 2, 2, 2}, {128, 128, 32, 2, 2, 3}, {128, 128, 32, 2, 2, 4},
                           {64, 128, 64, 2, 2, 2}, {64, 128, 32, 2, 2, 3}, {128, 64, 64, 2, 2, 2}, {64, 64, 64, 2, 2, 3},
                           {256, 256, 64, 2, 4, 2}, {256, 128, 64, 4, 2, 2}, {128, 256, 64, 2, 4, 2}, {256, 256, 64, 4, 2, 2},
                           {64, 256, 64, 1, 4, 2}, {64, 256, 32, 1, 4, 2}, {256, 256, 32, 2, 4, 4}, {256, 256, 32, 2, 4, 3},
                           {128, 32, 64, 4, 1, 6}, {256, 32, 64, 4, 1, 4}, {128, 32, 64, 4, 1, 4}, {256, 64, 32, 4, 1, 6}, {64, 32, 64, 2, 1, 8},
                           {64, 64, 128, 2, 2, 3}, {64, 128, 128, 2, 2, 2}, {128, 128, 128, 2, 2, 2}, {128, 64, 128, 2, 2, 2}, {64, 64, 128, 2, 2, 4},
                           {64, 64, 64, 2, 2, 2, 4}, {64, 64, 64, 2, 2, 2, 2}, {64, 128, 64, 2, 2, 2, 2}, {128, 64, 64, 2, 2, 2, 2},
                           {256, 256, 64, 2, 2, 2}, {256, 128, 64, 2, 2, 3}, {128, 256, 64, 2, 2, 3}, {256, 224, 64, 4, 1, 2}};
constexpr int kNumDma = 34, kStripVariant = 30, kStripEnd = 34;   // entries 30..33 are k_conv_strip (4 waves; its own LDS layout)
inline bool is_strip(int v) { return v >= kStripVariant && v < kStripEnd; }
typedef void (*KernelFn)(const KArgs);
KernelFn pick_dma_d(int v)
{
    switch (v) {
    case 0: return k_dgrad_dma<128, 128, 64, 2, 2, 2>;
    case 1: return k_dgrad_dma<128, 128, 32, 2, 2, 2>;
    case 2: return k_dgrad_dma<128, 128, 32, 2, 2, 3>;
    case 3: return k_dgrad_dma<128, 128, 32, 2, 2, 4>;
    case 4: return k_dgrad_dma<64, 128, 64, 2, 2, 2>;
    case 5: return k_dgrad_dma<64, 128, 32, 2, 2, 3>;
    case 6: return k_dgrad_dma<128, 64, 64, 2, 2, 2>;
    case 8: return k_dgrad_dma<256, 256, 64, 2, 4, 2>;
    case 9: return k_dgrad_dma<256, 128, 64, 4, 2, 2>;
    case 10: return k_dgrad_dma<128, 256, 64, 2, 4, 2>;
    case 11: return k_dgrad_dma<256, 256, 64, 4, 2, 2>;
    case 12: return k_dgrad_dma<64, 256, 64, 1, 4, 2>;
    case 13: return k_dgrad_dma<64, 256, 32, 1, 4, 2>;
    case 14: return k_dgrad_dma<256, 256, 32, 2, 4, 4>;
    case 15: return k_dgrad_dma<256, 256, 32, 2, 4, 3>;
    case 16: return k_dgrad_dma<128, 32, 64, 4, 1, 6>;
    case 17: return k_dgrad_dma<256, 32, 64, 4, 1, 4>;
    case 18: return k_dgrad_dma<128, 32, 64, 4, 1, 4>;
    case 19: return k_dgrad_dma<256, 64, 32, 4, 1, 6>;
    case 20: return k_dgrad_dma<64, 32, 64, 2, 1, 8>;
    case 21: return k_dgrad_dma<64, 64, 128, 2, 2, 3>;
    case 22: return k_dgrad_dma<64, 128, 128, 2, 2, 2>;
    case 23: return k_dgrad_dma<128, 128, 128, 2, 2, 2>;
    case 24: return k_dgrad_dma<128, 64, 128, 2, 2, 2>;
    case 25: return k_dgrad_dma<64, 64, 128, 2, 2, 4>;
    case 26: return k_dgrad_dma<64, 64, 64, 2, 2, 2, 4>;
    case 27: return k_dgrad_dma<64, 64, 64, 2, 2, 2, 2>;
    case 28: return k_dgrad_dma<64, 128, 64, 2, 2, 2, 2>;
    case 29: return k_dgrad_dma<128, 64, 64, 2, 2, 2, 2>;
    case 30: return k_conv_strip<true, 256, 256>;
    case 31: return k_conv_strip<true, 128, 256>;
    case 32: return k_conv_strip<true, 256, 128>;
    case 33: return k_conv_strip<true, 224, 256>;
    default: return k_dgrad_dma<64, 64, 64, 2, 2, 3>;
    }
}
KernelFn pick_dma(int v)
{
    switch (v) {
    case 0: return k_fwd_dma<128, 128, 64, 2, 2, 2>;
    case 1: return k_fwd_dma<128, 128, 32, 2, 2, 2>;
    case 2: return k_fwd_dma<128, 128, 32, 2, 2, 3>;
    case 3: return k_fwd_dma<128, 128, 32, 2, 2, 4>;
    case 4: return k_fwd_dma<64, 128, 64, 2, 2, 2>;
    case 5: return k_fwd_dma<64, 128, 32, 2, 2, 3>;
    case 6: return k_fwd_dma<128, 64, 64, 2, 2, 2>;
    case 8: return k_fwd_dma<256, 256, 64, 2, 4, 2>;
    case 9: return k_fwd_dma<256, 128, 64, 4, 2, 2>;
    case 10: return k_fwd_dma<128, 256, 64, 2, 4, 2>;
    case 11: return k_fwd_dma<256, 256, 64, 4, 2, 2>;
    case 12: return k_fwd_dma<64, 256, 64, 1, 4, 2>;
    case 13: return k_fwd_dma<64, 256, 32, 1, 4, 2>;
    case 14: return k_fwd_dma<256, 256, 32, 2, 4, 4>;
    case 15: return k_fwd_dma<256, 256, 32, 2, 4, 3>;
    case 16: return k_fwd_dma<128, 32, 64, 4, 1, 6>;
    case 17: return k_fwd_dma<256, 32, 64, 4, 1, 4>;
    case 18: return k_fwd_dma<128, 32, 64, 4, 1, 4>;
    case 19: return k_fwd_dma<256, 64, 32, 4, 1, 6>;
    case 20: return k_fwd_dma<64, 32, 64, 2, 1, 8>;
    case 21: return k_fwd_dma<64, 64, 128, 2, 2, 3>;
    case 22: return k_fwd_dma<64, 128, 128, 2, 2, 2>;
    case 23: return k_fwd_dma<128, 128, 128, 2, 2, 2>;
    case 24: return k_fwd_dma<128, 64, 128, 2, 2, 2>;
    case 25: return k_fwd_dma<64, 64, 128, 2, 2, 4>;
    case 26: return k_fwd_dma<64, 64, 64, 2, 2, 2, 4>;
    case 27: return k_fwd_dma<64, 64, 64, 2, 2, 2, 2>;
    case 28: return k_fwd_dma<64, 128, 64, 2, 2, 2, 2>;
    case 29: return k_fwd_dma<128, 64, 64, 2, 2, 2, 2>;
    case 30: return k_conv_strip<false, 256, 256>;
    case 31: return k_conv_strip<false, 128, 256>;
    case 32: return k_conv_strip<false, 256, 128>;
    case 33: return k_conv_strip<false, 224, 256>;
    default: return k_fwd_dma<64, 64, 64, 2, 2, 3>;
    }
}
const DmaVariant kDmaW[] = {{128, 128, 32, 2, 2, 2}, {128, 128, 64, 2, 2, 2}, {128, 128, 32, 2, 2, 3}, {64, 128, 32, 2, 2, 2},
                            {128, 64, 32, 2, 2, 2}, {64, 64, 32, 2, 2, 2}, {64, 128, 64, 2, 2, 2}, {256, 128, 32, 4, 2, 2},
                            {64, 256, 32, 1, 4, 2}, {64, 256, 64, 1, 4, 2}, {256, 256, 32, 2, 4, 2}, {256, 256, 32, 2, 4, 3},
                            {256, 256, 64, 2, 4, 2}, {256, 256, 32, 4, 2, 2}, {128, 256, 32, 2, 4, 2}, {128, 256, 32, 1, 4, 2}};
constexpr int kNumDmaW = 16;
KernelFn pick_dma_w(int v)
{
    switch (v) {
    case 0: return k_wgrad_dma<128, 128, 32, 2, 2, 2>;
    case 1: return k_wgrad_dma<128, 128, 64, 2, 2, 2>;
    case 2: return k_wgrad_dma<128, 128, 32, 2, 2, 3>;
    case 3: return k_wgrad_dma<64, 128, 32, 2, 2, 2>;
    case 4: return k_wgrad_dma<128, 64, 32, 2, 2, 2>;
    case 5: return k_wgrad_dma<64, 64, 32, 2, 2, 2>;
    case 6: return k_wgrad_dma<64, 128, 64, 2, 2, 2>;
    case 8: return k_wgrad_dma<64, 256, 32, 1, 4, 2>;
    case 9: return k_wgrad_dma<64, 256, 64, 1, 4, 2>;
    case 10: return k_wgrad_dma<256, 256, 32, 2, 4, 2>;
    case 11: return k_wgrad_dma<256, 256, 32, 2, 4, 3>;
    case 12: return k_wgrad_dma<256, 256, 64, 2, 4, 2>;
    case 13: return k_wgrad_dma<256, 256, 32, 4, 2, 2>;
    case 14: return k_wgrad_dma<128, 256, 32, 2, 4, 2>;
    case 15: return k_wgrad_dma<128, 256, 32, 1, 4, 2>;
    default: return k_wgrad_dma<256, 128, 32, 4, 2, 2>;
    }
}
size_t dma_w_lds_bytes(const DmaVariant &d) { return (size_t)d.NS * (d.TA + d.TB) * d.BK * 2 + (size_t)2 * 64 * d.WA * d.WB * 8; }

size_t dma_lds_bytes(const DmaVariant &d)
{
    if (&d >= &kDma[kStripVariant] && &d < &kDma[kStripEnd]) return strip_lds_bytes(d.TA, d.TB);
    size_t stages = (size_t)d.KG * d.NS * (d.TA + d.TB) * d.BK * 2, epi = (size_t)d.TB * (d.TA + 8) * 2;
    const size_t gsum = (size_t)(d.KG - 1) * d.TA * d.TB * 4;   // extra groups' accumulators
    if (gsum > stages) stages = gsum;
    return (stages > epi ? stages : epi) + (size_t)d.TB * 8 + (size_t)d.TA * 4 + (size_t)d.TB * 4;   // + row table, bias, row map
}

}  // namespace

hipError_t dma_init()
{
    for (int v = 0; v < kNumDma; ++v) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pick_dma(v)), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)dma_lds_bytes(kDma[v]));
        if (e != hipSuccess) return e;
    }
    for (int v = 0; v < kNumDma; ++v) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pick_dma_d(v)), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)dma_lds_bytes(kDma[v]));
        if (e != hipSuccess) return e;
    }
    for (int v = 0; v < kNumDmaW; ++v) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pick_dma_w(v)), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)dma_w_lds_bytes(kDmaW[v]));
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// variant override 200 + v selects pipelined variant v; the built-in choice does not use them yet
// Strided backward-data by phase: B tiles and reduction steps (of BK) per phase (a, b) = (h % sh, w % sw).
// Returns the number of phases (sh * sw <= 4).
static int phase_layout(const ConvGeom &g, int TB, int BK, int tile0[5], int *max_steps)
{
    const int nph = g.sh * g.sw;
    int t = 0, ms = 0;
    for (int c = 0; c < nph; ++c) {
        const int a = c / g.sw, b = c % g.sw;
        const long long hc = g.H > a ? (g.H - a + g.sh - 1) / g.sh : 0, wc = g.W > b ? (g.W - b + g.sw - 1) / g.sw : 0;
        const long long rows = (long long)g.N * hc * wc;
        tile0[c] = t;
        t += (int)((rows + TB - 1) / TB);
        const int r0 = (a + g.ph) % g.sh, s0 = (b + g.pw) % g.sw;
        const int nr = r0 < g.R ? (g.R - r0 + g.sh - 1) / g.sh : 0, ns = s0 < g.S ? (g.S - s0 + g.sw - 1) / g.sw : 0;
        if (rows > 0 && nr * ns * (g.K / BK) > ms) ms = nr * ns * (g.K / BK);
    }
    for (int c = nph; c < 5; ++c) tile0[c] = t;
    *max_steps = ms;
    return nph;
}

bool dma_plan(const ConvGeom &g, int pass, int force_variant, int force_splits, GemmPlan *pl)
{
    if (g.R * g.S > 32) return false;
    int rowsA, rowsB, red;
    const DmaVariant *d;
    if (pass == PASS_FWD) {
        if (force_variant < 200 || force_variant >= 200 + kNumDma) return false;
        d = &kDma[force_variant - 200];
        if (g.C % d->BK != 0) return false;
        if (is_strip(force_variant - 200) &&   // 3x3, stride 1, pad 1, c_in % 128, whole groups of 8 output channels, no reduction split
            (g.C % 128 != 0 || g.R != 3 || g.S != 3 || g.sh != 1 || g.sw != 1 || g.ph != 1 || g.pw != 1 || g.Ho != g.H || g.Wo != g.W || g.K % 8 != 0))
            return false;
        pl->variant = force_variant - 200;
        rowsA = g.K; rowsB = g.N * g.Ho * g.Wo; red = g.R * g.S * g.C;
    } else if (pass == PASS_DGRAD) {
        if (force_variant < 200 || force_variant >= 200 + kNumDma) return false;
        d = &kDma[force_variant - 200];
        if (g.K % d->BK != 0 || g.C % 8 != 0) return false;
        if (is_strip(force_variant - 200) &&   // as forward, with c_out as the reduction; bf16 gradients only (the caller checks)
            (g.K % 128 != 0 || g.R != 3 || g.S != 3 || g.sh != 1 || g.sw != 1 || g.ph != 1 || g.pw != 1 || g.Ho != g.H || g.Wo != g.W))
            return false;   // any stride: taps that miss the stride grid are masked out
        pl->variant = force_variant - 200;
        rowsA = g.C; rowsB = g.N * g.H * g.W; red = g.R * g.S * g.K;
    } else if (pass == PASS_WGRAD) {
        if (force_variant == 316) return wstrip_plan(g, force_splits, pl);
        if (force_variant < 300 || force_variant >= 300 + kNumDmaW) return false;
        d = &kDmaW[force_variant - 300];
        if (g.K % 8 || g.C % 8) return false;
        pl->variant = force_variant - 300;
        rowsA = g.K; rowsB = g.R * g.S * g.C; red = g.N * g.Ho * g.Wo;
    } else return false;
    pl->fast = true; pl->dma = true; pl->TA = d->TA; pl->TB = d->TB; pl->BK = d->BK;
    pl->vecA = pl->vecB = true;
    pl->phase = false;
    pl->tilesA = (rowsA + d->TA - 1) / d->TA;
    pl->tilesB = (rowsB + d->TB - 1) / d->TB;
    pl->steps_total = (red + d->BK - 1) / d->BK;
    if (pass == PASS_DGRAD && (g.sh > 1 || g.sw > 1) && g.sh <= 2 && g.sw <= 2 && g.R * g.S > 1 && force_splits <= 1) {
        // no reduction split asked for: walk the pixels phase by phase and multiply only the taps that can hit
        // (a 1x1 filter gains nothing: its backward-data is bound by writing dx, three quarters of it zeros)
        int tile0[5], max_steps;
        phase_layout(g, d->TB, d->BK, tile0, &max_steps);
        if (max_steps > 0 && tile0[4] > 0) {
            pl->phase = true;
            pl->tilesB = tile0[4];
            pl->steps_total = pl->steps_per_split = max_steps;
            pl->splits = 1;
            return true;
        }
    }
    int splits;
    if (pass != PASS_WGRAD && is_strip(pl->variant)) {
        // a split takes whole channel blocks, an even number of them (two strips are unrolled): the largest such count <= the request
        const int cb = (pass == PASS_FWD ? g.C : g.K) / 64;
        splits = force_splits > 0 ? force_splits : 1;
        while (splits > 1 && cb % (2 * splits) != 0) --splits;
    } else if (force_splits > 0) splits = force_splits;
    else {
        long long tiles = (long long)pl->tilesA * pl->tilesB;
        splits = tiles >= 512 ? 1 : (int)((512 + tiles - 1) / tiles);
        int max_splits = pl->steps_total / 8;
        if (max_splits < 1) max_splits = 1;
        if (splits > max_splits) splits = max_splits;
    }
    if (splits > pl->steps_total) splits = pl->steps_total;
    if (splits < 1) splits = 1;
    pl->steps_per_split = (pl->steps_total + splits - 1) / splits;
    pl->splits = (pl->steps_total + pl->steps_per_split - 1) / pl->steps_per_split;
    return true;
}

bool dma_plan_is_strip(const GemmPlan &plan) { return plan.dma && !plan.halo && !plan.wstrip && is_strip(plan.variant); }

// Whether this forward / backward-data plan sums its reduction splits inside the main kernel: asked for by the plan, tiles in
// natural pixel order, and few enough tiles that a range of the counter ring is not handed out again for at least 64 later launches.
// The fused reduction stores and loads whole groups of four channels and addresses the partial sums through one buffer descriptor.
bool dma_fused_reduce_fits(int rowsA, int rowsB, int splits) { return (rowsA & 3) == 0 && (size_t)rowsA * rowsB * splits * 4 < ((size_t)1 << 31); }

bool dma_plan_fuses_reduce(const GemmPlan &plan)
{
    return plan.fused_reduce && plan.dma && !plan.halo && !plan.wstrip && plan.splits > 1 && !is_strip(plan.variant) && !plan.phase &&
           plan.tilesA * plan.tilesB <= kTicketRing / 64;
}

void dma_kernel_name(int pass, const GemmPlan &pl, char *name, size_t name_bytes)
{
    if (pl.wstrip) { snprintf(name, name_bytes, "k_wgrad_strip"); return; }
    const DmaVariant &d = pass == PASS_WGRAD ? kDmaW[pl.variant] : kDma[pl.variant];
    // as the profiler prints the instantiation: the forward / backward-data kernels carry the group count
    if (pass != PASS_WGRAD && is_strip(pl.variant)) snprintf(name, name_bytes, "k_conv_strip<%s, %d, %d>", pass == PASS_FWD ? "false" : "true", d.TB, d.TA);
    else if (pass == PASS_WGRAD) snprintf(name, name_bytes, "k_wgrad_dma<%d, %d, %d, %d, %d, %d>", d.TA, d.TB, d.BK, d.WA, d.WB, d.NS);
    else snprintf(name, name_bytes, "%s<%d, %d, %d, %d, %d, %d, %d>", pass == PASS_DGRAD ? "k_dgrad_dma" : "k_fwd_dma", d.TA, d.TB, d.BK, d.WA,
                  d.WB, d.NS, d.KG);
}

hipError_t dma_launch(const ConvArgs &a, hipStream_t st)
{
    KArgs p;
    p.g = a.g;
    if (a.pass == PASS_FWD) { p.rowsA = a.g.K; p.rowsB = a.g.N * a.g.Ho * a.g.Wo; p.red = a.g.R * a.g.S * a.g.C; }
    else if (a.pass == PASS_DGRAD) { p.rowsA = a.g.C; p.rowsB = a.g.N * a.g.H * a.g.W; p.red = a.g.R * a.g.S * a.g.K; }
    else { p.rowsA = a.g.K; p.rowsB = a.g.R * a.g.S * a.g.C; p.red = a.g.N * a.g.Ho * a.g.Wo; }
    p.tilesA = a.plan.tilesA; p.tilesB = a.plan.tilesB;
    p.steps_total = a.plan.steps_total; p.steps_per_split = a.plan.steps_per_split; p.splits = a.plan.splits;
    p.flags = a.flags;
    p.x = a.x; p.w = a.w; p.dy = a.dy; p.ymask = nullptr; p.bias = a.bias; p.out = a.out; p.partial = a.partial;
    const bool wg = a.pass == PASS_WGRAD;
    p.ph_on = 0;
    if (a.pass == PASS_DGRAD && a.plan.phase) {
        if (!(a.flags & KF_OUT_F32) && (p.rowsA & 7) == 0) {   // the staged bf16 epilogue carries the row map
            int max_steps;
            phase_layout(a.g, a.plan.TB, a.plan.BK, p.ph_tile0, &max_steps);
            p.ph_on = 1;
        } else {   // fp32 gradients: the same tiles in natural pixel order, all taps (masked)
            p.tilesB = (p.rowsB + a.plan.TB - 1) / a.plan.TB;
            p.steps_total = p.steps_per_split = (p.red + a.plan.BK - 1) / a.plan.BK;
        }
    }
    // operands touched exactly once are streamed past the caches: the weights of a pass with a single pixel tile (dense layers at
    // small batch), and a large filter gradient stored straight to its destination
    if (!wg && p.tilesB == 1 && (size_t)p.rowsA * p.red * 2 >= ((size_t)8 << 20)) p.flags |= KF_NT_A;
    if (wg && p.splits == 1 && (size_t)p.rowsA * p.rowsB * 4 >= ((size_t)32 << 20)) p.flags |= KF_NT_OUT;
    p.dbp = p.splits > 1 ? a.db_partial : a.db_out;
    if (!wg || p.dbp == nullptr || !plan_sums_bias_gradient(a.plan)) p.flags &= ~KF_DB;
    const DmaVariant &d = wg ? kDmaW[a.plan.variant] : kDma[a.plan.variant];
    p.tickets = nullptr;
    const bool fused = !wg && dma_plan_fuses_reduce(a.plan) && dma_fused_reduce_fits(p.rowsA, p.rowsB, p.splits);
    if (fused) {
        // counters of this launch: a range of the ring that no launch in flight is using (ranges are handed out in order; a range is
        // reused only after kTicketRing counters have been handed out since, i.e. thousands of launches later)
        constexpr int kMaxDev = 16;
        static unsigned *ring_base[kMaxDev] = {};   // each device holds its own copy of the array
        static unsigned ring_pos[kMaxDev] = {};
        static std::mutex ring_mu;
        const unsigned tiles = (unsigned)(p.tilesA * p.tilesB);
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= kMaxDev) return hipErrorInvalidDevice;
        unsigned start;
        {
            std::lock_guard<std::mutex> lock(ring_mu);
            if (ring_base[dev] == nullptr) {
                e = hipGetSymbolAddress((void **)&ring_base[dev], HIP_SYMBOL(g_tickets));
                if (e != hipSuccess) return e;
            }
            if (ring_pos[dev] + tiles > (unsigned)kTicketRing) ring_pos[dev] = 0;
            start = ring_pos[dev];
            ring_pos[dev] += tiles;
        }
        p.tickets = ring_base[dev] + start;
        p.flags |= KF_FUSED_REDUCE;
    }
    dim3 grid((unsigned)(p.tilesA * p.tilesB), (unsigned)p.splits, 1), block(64 * d.WA * d.WB * d.KG, 1, 1);
    if (wg) grid = dim3((unsigned)p.splits, (unsigned)(p.tilesA * p.tilesB), 1);
    hipLaunchKernelGGL(wg ? pick_dma_w(a.plan.variant) : a.pass == PASS_DGRAD ? pick_dma_d(a.plan.variant) : pick_dma(a.plan.variant), grid, block, wg ? dma_w_lds_bytes(d) : dma_lds_bytes(d), st, p);
    dp_trace_main_kernel_done(st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.splits <= 1 || fused) return e;
    return launch_split_reduce(a, p.rowsA, p.rowsB, st, (p.flags & KF_DB) != 0);
}
