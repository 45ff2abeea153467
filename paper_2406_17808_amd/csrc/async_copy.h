// Asynchronous copies from global memory straight into LDS (gfx950), and the waits on them.
//
// The instructions are written out as inline assembly so that the waits stay under the
// kernel's control: the compiler does not know these copies, so it inserts no wait for them,
// and the kernel waits with s_waitcnt vmcnt(N) for exactly the copies it is about to read.
// Vector memory operations of a wave retire in order, so the compiler's own vmcnt waits for its
// ordinary loads can only wait longer, never less.
#pragma once

#include <stdint.h>

#include "internal.h"

namespace ckv {

// One 1 KB copy: lane i moves the 16 bytes at base + voff(i) to LDS address lds + 16 i.
// base and lds are the same for all lanes of the wave.
__device__ inline void async_copy_1k(const void* base, uint32_t voff, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(voff), "s"(base), "s"(lds)
                 : "memory");
}

// The same for data that is read once: the nt modifier keeps it from displacing what the caches
// hold (measured on the decode step, whose two passes stream 4.3 GB each: -5 %).
__device__ inline void async_copy_1k_stream(const void* base, uint32_t voff, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                 :
                 : "v"(voff), "s"(base), "s"(lds)
                 : "memory");
}

// One 256-byte copy: lane i moves the 4 bytes at base + voff(i) to LDS address lds + 4 i.
__device__ inline void async_copy_256(const void* base, uint32_t voff, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :
                 : "v"(voff), "s"(base), "s"(lds)
                 : "memory");
}

__device__ inline void async_copy_256_stream(const void* base, uint32_t voff, uint32_t lds)   // read once, as above
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1 nt"
                 :
                 : "v"(voff), "s"(base), "s"(lds)
                 : "memory");
}

// A 4-byte store the compiler does not count either (it takes part in the same in-order
// sequence of vector memory operations as the copies): the active lanes write value to
// base + voff.
__device__ inline void counted_store_f32(void* base, uint32_t voff, float value)
{
    asm volatile("global_store_dword %0, %1, %2" : : "v"(voff), "v"(value), "s"(base) : "memory");
}

template <int N> __device__ inline void wait_vm()   // at most N vector memory operations outstanding
{
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// The same, and the compiler moves no memory access across it (for a wave that reads what its
// own copies brought, with no barrier in between).
template <int N> __device__ inline void wait_vm_fenced()
{
    asm volatile("" ::: "memory");
    wait_vm<N>();
    asm volatile("" ::: "memory");
}

// All LDS reads of this wave have returned (before a copy may overwrite what they read).
__device__ inline void wait_lds_reads()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0), the other counters left alone
    asm volatile("" ::: "memory");
}

// Workgroup barrier without the memory fence of __syncthreads (which would wait for the copies
// still in flight).  The callers wait for exactly the copies the barrier publishes; the empty asm
// statements keep the compiler from moving LDS accesses across it.
__device__ inline void wg_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
__device__ inline uint32_t lds_address(const void* p) { return (uint32_t)(uintptr_t)(lds_byte_t*)p; }

}  // namespace ckv
