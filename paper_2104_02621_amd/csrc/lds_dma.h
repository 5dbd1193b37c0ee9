// Internal: direct global -> LDS copies through buffer descriptors, and a compile-time loop,
// shared by the kernels whose K loops are scheduled by hand.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>
#include <utility>

namespace capscaps {

typedef int rsrc_t __attribute__((ext_vector_type(4)));  // raw buffer descriptor (4 SGPRs)

// compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(<N-1>)
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

// Raw buffer descriptor: 48-bit base, stride 0, `bytes` addressable, dword data format.
// Offsets at or beyond `bytes` read as zero.
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, unsigned bytes)
{
    const unsigned long long a = reinterpret_cast<unsigned long long>(base);
    rsrc_t r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)(a & 0xffffffffu));
    r[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)((a >> 32) & 0xffffu));
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    r[3] = 0x00020000;
    return r;
}

// One wave-wide copy global -> LDS: lane i moves the 16 bytes at base + voff_i + soff_a + soff_b
// to LDS byte address lds_base + LDS_IMM + 16*i.  The sum of the offsets is range-checked
// against the descriptor: at or beyond its size the lane stores zeros.  Asynchronous;
// completion is counted in vmcnt.  Inline assembly on purpose: the waits are exactly the
// s_waitcnt vmcnt(n) placed by hand in the K loop (the compiler would drain all such copies
// before any later LDS read, which would undo the multi-stage prefetch).  The scalar add
// between the M0 write and the copy is the wait state that sequence needs.
template <int LDS_IMM>
__device__ __forceinline__ void copy_to_lds_16B(rsrc_t rs, unsigned lds_base, unsigned voff,
                                                int soff_a, int soff_b)
{
    int tmp;
    asm volatile(
        "s_add_u32 m0, %1, %5\n\ts_add_u32 %0, %3, %4\n\tbuffer_load_dwordx4 %2, %6, %0 offen lds"
        : "=&s"(tmp)
        : "s"(lds_base), "v"(voff), "s"(soff_a), "s"(soff_b), "i"(LDS_IMM), "s"(rs)
        : "memory", "scc");
}

// Same with a run-time LDS address and DW = 3 or 4 dwords per lane (a 12-byte copy still lands
// at a 16-byte lane stride in LDS and leaves the slot's fourth dword untouched).
template <int DW>
__device__ __forceinline__ void copy_to_lds_dwords(rsrc_t rs, unsigned lds_addr, unsigned voff,
                                                   int soff)
{
    static_assert(DW == 3 || DW == 4, "12- or 16-byte copies");
    const int lds_s = __builtin_amdgcn_readfirstlane((int)lds_addr);
    const int soff_s = __builtin_amdgcn_readfirstlane(soff);
    if (DW == 3)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx3 %1, %2, %3 offen lds"
                     :
                     : "s"(lds_s), "v"(voff), "s"(rs), "s"(soff_s)
                     : "memory");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                     :
                     : "s"(lds_s), "v"(voff), "s"(rs), "s"(soff_s)
                     : "memory");
}

}  // namespace capscaps
