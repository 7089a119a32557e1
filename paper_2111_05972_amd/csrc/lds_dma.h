// Buffer descriptors and buffer loads that write straight into LDS (gfx950), shared by the GEMM and the attention
// kernels.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace tpl {

typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((address_space(3))) void* lds_void_ptr;

// Raw buffer descriptor over `bytes` bytes at p (stride 0): loads at offsets >= bytes return zero
// instead of touching memory.
__device__ __forceinline__ i32x4 make_rsrc(const void* p, unsigned bytes) {
    const uint64_t a = (uint64_t)(uintptr_t)p;
    i32x4 r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)a);
    r[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)(a >> 32) & 0xffff);
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    r[3] = 0x00020000;
    return r;
}

// One 16-byte-per-lane buffer load straight into LDS (lane l lands at lds_addr + 16*l).  Issued as
// inline assembly on purpose: the compiler then keeps no record of an LDS write in flight, so it does
// not drain the whole prefetch ring (vmcnt(0)) in front of later LDS reads; the kernel waits on
// vmcnt itself, with the exact number of loads allowed to remain in flight.
__device__ __forceinline__ void buffer_load_lds_b128(i32x4 rsrc, unsigned lds_addr, unsigned voffset) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_addr), "v"(voffset), "s"(rsrc) : "memory", "m0");
}

// The same with a scalar byte offset added by the instruction (the k position of a stage), so that the
// per-lane offset stays loop invariant and no vector arithmetic is spent per load.
__device__ __forceinline__ void buffer_load_lds_b128_s(i32x4 rsrc, unsigned lds_addr, unsigned voffset, unsigned soffset) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset) : "memory", "m0");
}
}  // namespace tpl
