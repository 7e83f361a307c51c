// The transposing LDS read of gfx950 (ds_read_b64_tr_b16), issued as inline assembly.
//
// In each block of 16 lanes, lane i receives as value j (of four 16-bit values) the element i&3 of the
// 8 bytes addressed by lane 4j + (i>>2): a 4 x 16 patch of 16-bit elements comes back transposed, which
// turns rows that lie in LDS as they lie in memory (contiguous along the outer index) into MFMA
// fragments (contiguous along the reduction index).
//
// Why not the compiler's builtin: it takes such a read for one that may touch LDS bytes which direct-to-LDS
// loads still in flight are going to write, and puts s_waitcnt vmcnt(0) in front of it -- every global load
// the wave has issued, the prefetch of the next tiles included, must then land first, and the prefetch
// overlaps nothing (seen in the ISA of both kernels that use these reads; plain LDS loads get no such wait).
// The kernels order their LDS reads against the arrival of those loads themselves, with s_waitcnt vmcnt(n)
// and a workgroup barrier.
//
// As assembly the read is invisible to the compiler's wait-count bookkeeping, so the CALLER waits:
// lds_tr_wait<N>() lets at most N of the wave's LDS operations (issued after the ones needed) be
// outstanding; LDS operations return in order.  The "memory" clobber keeps the reads in program order
// with respect to the loads, waits and barriers around them.
#pragma once

#include <type_traits>
#include <utility>

namespace xp {

// f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{}): a loop whose index is
// a constant expression inside the body (instruction offsets must be)
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

typedef unsigned int lds_tr_u32x2 __attribute__((ext_vector_type(2)));

// LDS byte address of a pointer into a __shared__ array
__device__ __forceinline__ unsigned lds_address(const void *p)
{
    return (unsigned)(unsigned long long)(__attribute__((address_space(3))) const void *)p;
}

template <int OFFSET>
__device__ __forceinline__ lds_tr_u32x2 lds_read_tr16_b64(unsigned address)
{
    static_assert(OFFSET >= 0 && OFFSET < 65536, "the instruction's offset field has 16 bits");
    lds_tr_u32x2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(address), "n"(OFFSET) : "memory");
    return v;
}

// A plain 16-byte LDS read issued the same way, for kernels that take ALL their fragment reads out of
// the compiler's bookkeeping: with only some of them hidden, the waits the compiler computes for the
// reads it does see count too few operations in flight and end up waiting for reads issued much later.
typedef unsigned int lds_tr_u32x4 __attribute__((ext_vector_type(4)));
template <int OFFSET>
__device__ __forceinline__ lds_tr_u32x4 lds_read_b128(unsigned address)
{
    static_assert(OFFSET >= 0 && OFFSET < 65536 && OFFSET % 16 == 0, "the instruction's offset field has 16 bits");
    lds_tr_u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(address), "n"(OFFSET) : "memory");
    return v;
}

// s_waitcnt lgkmcnt(N), the other counters left open
template <int N>
__device__ __forceinline__ void lds_wait()
{
    static_assert(N >= 0 && N <= 15, "lgkmcnt is a 4-bit counter");
    asm volatile("s_waitcnt lgkmcnt(%0)" : : "n"(N) : "memory");
}

// Ties a register to the preceding lds_wait: the value passes through an (empty) statement as an in/out
// operand, so that no instruction using it can be scheduled in front of the wait (volatile statements
// keep their order among themselves; a bare s_waitcnt orders nothing but memory operations).
template <class V>
__device__ __forceinline__ void lds_tie(V &value)
{
    asm volatile("" : "+v"(value));
}

// A 16-byte MFMA fragment gathered by two transposing reads.  The halves are separate values until the wait for
// them has passed: a fragment composed from the two read results right away could be given registers of its own,
// and the copies into them would execute before the data has arrived.
struct FragHalves {
    lds_tr_u32x2 lo, hi;
};
__device__ __forceinline__ void frag_tie(lds_tr_u32x4 &f) { lds_tie(f); }
__device__ __forceinline__ void frag_tie(FragHalves &f)
{
    lds_tie(f.lo);
    lds_tie(f.hi);
}
__device__ __forceinline__ lds_tr_u32x4 frag_value(const lds_tr_u32x4 &f) { return f; }
__device__ __forceinline__ lds_tr_u32x4 frag_value(const FragHalves &f) { return lds_tr_u32x4{f.lo[0], f.lo[1], f.hi[0], f.hi[1]}; }

// the two together
template <int N, class... V>
__device__ __forceinline__ void lds_tr_wait(V &...values)
{
    lds_wait<N>();
    (..., lds_tie(values));
}

}  // namespace xp
