// Device helpers shared by the kernels that fill LDS with direct-to-LDS buffer loads: buffer
// resources, the 16-byte copy, explicit waits, and LDS fragment reads as inline assembly (the compiler
// would otherwise wait for every outstanding copy before any LDS read it can see).
#pragma once
#include "tile_common.h"
#include <utility>
#include <type_traits>

namespace {

constexpr unsigned OOR = 0xFFFFFFFFu;
typedef __attribute__((address_space(3))) void *lds_void;

DEVFN __amdgpu_buffer_rsrc_t make_rsrc(const void *p, size_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)(unsigned)bytes, 0x00020000);
}
// 16 bytes per lane from the buffer straight into LDS at lds_base + lane*16 (lds_base wave-uniform)
DEVFN void dma16(__amdgpu_buffer_rsrc_t r, unsigned lds_base, unsigned voff)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_void)(size_t)lds_base, 16, voff, 0, 0, 0);
}
// the same copy with the non-temporal hint: for operands that are read exactly once (allocating them in the caches
// would push out dirty lines that then have to be written back in the middle of the stream)
DEVFN void dma16_nt(__amdgpu_buffer_rsrc_t r, unsigned lds_base, unsigned voff)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_void)(size_t)lds_base, 16, voff, 0, 0, 2);
}
DEVFN unsigned lds_offset(const void *p) { return (unsigned)(size_t)(__attribute__((address_space(3))) const char *)p; }

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index is a constant expression in the body
template <typename F, int... I> DEVFN void for_constant_impl(F &&f, std::integer_sequence<int, I...>) { (f(std::integral_constant<int, I>{}), ...); }
template <int N, typename F> DEVFN void for_constant(F &&f) { for_constant_impl(f, std::make_integer_sequence<int, N>{}); }

// The matrix instruction as inline assembly, its accumulator pinned to the accumulation registers (AG) or to the vector
// registers: a kernel whose accumulators fill the accumulation registers exactly must not leave the choice to the compiler,
// which otherwise keeps some tiles elsewhere and copies them around every instruction.  The statement is volatile: it stays
// in its place among the other volatile statements (LDS reads, waits).  s_nop 1: a vector instruction the compiler placed
// just before (a copy or a rematerialised constant that feeds an operand) needs two wait states before a matrix instruction
// reads its result, and the compiler adds them only for instructions it knows.  For the same reason the caller spaces the
// first read of a result from the instruction that wrote it.
template <bool AG> DEVFN void mfma_in_regs(f32x16 &c, const u32x4 a, const u32x4 b)
{
    if constexpr (AG) asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
    else asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
}

template <int N> DEVFN void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int OFF> DEVFN u32x4 lds_read16(unsigned addr)
{
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}


// issue the fragment reads of one 16-wide reduction slice (blocks of 32 rows are BS bytes apart)
template <int FA, int FB, int BS>
DEVFN void read_frags(u32x4 (&a)[FA], u32x4 (&b)[FB], unsigned pa, unsigned pb)
{
    if constexpr (FA >= 1) a[0] = lds_read16<0>(pa);
    if constexpr (FA >= 2) a[1] = lds_read16<BS>(pa);
    if constexpr (FA >= 3) a[2] = lds_read16<2 * BS>(pa);
    if constexpr (FA >= 4) a[3] = lds_read16<3 * BS>(pa);
    if constexpr (FB >= 1) b[0] = lds_read16<0>(pb);
    if constexpr (FB >= 2) b[1] = lds_read16<BS>(pb);
    if constexpr (FB >= 3) b[2] = lds_read16<2 * BS>(pb);
    if constexpr (FB >= 4) b[3] = lds_read16<3 * BS>(pb);
}
// The reads are invisible to the compiler: wait until at most N newer LDS reads are outstanding,
// with the fragments as operands so that no matrix instruction using them is scheduled earlier.
template <int N, int FA, int FB>
DEVFN void wait_frags(u32x4 (&a)[FA], u32x4 (&b)[FB])
{
    static_assert(N >= 0 && N < 16, "lgkmcnt is a 4-bit counter");
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N));
    // volatile statements keep their order; the empty ones make the fragments depend on the wait
#pragma unroll
    for (int i = 0; i < FA; ++i) asm volatile("" : "+v"(a[i]));
#pragma unroll
    for (int j = 0; j < FB; ++j) asm volatile("" : "+v"(b[j]));
}

// Valid-tap mask of a pixel row: bit r*S+s is set iff 0 <= hb + sg*r < Hlim and 0 <= wb + sg*s < Wlim.
DEVFN unsigned tap_mask(int hb, int wb, int sg, int R, int S, int Hlim, int Wlim)
{
    unsigned smask = 0;
    for (int s = 0; s < S; ++s) smask |= ((unsigned)(wb + sg * s) < (unsigned)Wlim) ? 1u << s : 0u;
    unsigned mask = 0;
    for (int r = 0; r < R; ++r) mask |= ((unsigned)(hb + sg * r) < (unsigned)Hlim) ? smask << (r * S) : 0u;
    return mask;
}

template <int T> DEVFN int seg_swz(int t)
{
    constexpr int SPR = T / 32, RPS = T >= 128 ? 1 : 128 / T;   // segments per row, rows per 256 bytes
    return (t / RPS) & (SPR >= 4 ? 3 : SPR - 1);
}

template <int OFF> DEVFN u32x2 lds_read_tr(unsigned addr)
{
    u32x2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}


}  // namespace
