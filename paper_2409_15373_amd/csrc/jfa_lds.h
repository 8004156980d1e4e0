// Explicit LDS instructions shared by the direct-to-LDS kernels: global -> LDS copies, and LDS reads that stay in
// flight until the caller waits for them.  Not part of the C ABI.
#pragma once
#include <cstdint>
#include <hip/hip_runtime.h>
#include "jfa_mfma.h"

namespace jfa {

// Global -> LDS copies of 16 (or 4) bytes per lane: source = `base` (wave-uniform, scalar registers) +
// `byte_offset` (per lane, unsigned 32 bits), destination = lds_wave_base + 16 (or 4) * lane.  The scalar-base
// form needs no 64-bit vector address arithmetic and no vector registers for addresses.
// The instruction is written out instead of going through the compiler's builtin: the compiler follows every copy it
// knows of and protects LDS reads that it cannot tell apart from a copy's target with a wait for ALL copies in
// flight -- in the backward kernels before the reads of one stage in three, which cost a full memory latency each time.
// The kernels order copies and reads themselves (a partial vmcnt wait and a barrier at the end of every stage), so
// nothing is lost; copies the compiler does not count only make its own waits for other loads more conservative
// (loads return in order).  m0 holds the LDS address of lane 0's destination.
__device__ inline uint32_t lds_byte_address(const void *p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char *)p;
}
__device__ inline void bd_dma16(const void *base, uint32_t byte_offset, char *lds_wave_base) {
    const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_byte_address(lds_wave_base));
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 : : "s"(dst), "v"(byte_offset), "s"(base) : "memory", "m0");
}
__device__ inline void bd_dma4(const void *base, uint32_t byte_offset, char *lds_wave_base) {
    const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_byte_address(lds_wave_base));
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 : : "s"(dst), "v"(byte_offset), "s"(base) : "memory", "m0");
}

// LDS reads that stay in flight: the instruction is issued here and the caller waits for it later with lds_arrived.
// Left to the compiler, every operand read sits right in front of the matrix instruction that uses it, behind a wait
// for it, so that each matrix instruction (32 cycles) costs an LDS round trip (well over 100); issued a few matrix
// instructions ahead, the round trip is hidden.  The compiler does not know that the result registers are pending:
// nothing may touch them before lds_arrived has named them, which also keeps the wait in front of their first use.
// Counts passed to lds_arrived are the LDS instructions issued after the one waited for (LDS returns in order;
// instructions of the compiler's own in between only make the wait longer).
// `offset` is the instruction's own unsigned 16-bit byte offset, added to the address register.
template <int offset> __device__ inline bf16x8 lds_fetch_b128(uint32_t addr) {
    static_assert(offset >= 0 && offset < 65536, "ds offset field");
    bf16x8 r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(offset));
    return r;
}
template <int offset> __device__ inline bf16x4 lds_fetch_tr16(uint32_t addr) {   // see lds_read_tr16 for what a lane receives
    static_assert(offset >= 0 && offset < 65536, "ds offset field");
    bf16x4 r;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(offset));
    return r;
}
typedef __attribute__((ext_vector_type(4))) float f32x4;
template <int offset> __device__ inline void lds_fetch_4x_f32x4(uint32_t addr, f32x4 &x0, f32x4 &x1, f32x4 &x2, f32x4 &x3) {   // offset + 0, 32, 64, 96
    static_assert(offset >= 0 && offset + 96 < 65536, "ds offset field");
    asm volatile("ds_read_b128 %0, %4 offset:%5\n\tds_read_b128 %1, %4 offset:%6\n\tds_read_b128 %2, %4 offset:%7\n\t"
                 "ds_read_b128 %3, %4 offset:%8" : "=&v"(x0), "=&v"(x1), "=&v"(x2), "=&v"(x3)
                 : "v"(addr), "n"(offset), "n"(offset + 32), "n"(offset + 64), "n"(offset + 96));
}
// Wait until at most `later` LDS instructions are pending; the operands named are usable from here on, and the
// accumulator is named too so that the wait keeps its place between the matrix instructions before and after it.
template <int later> __device__ inline void lds_arrived(bf16x8 &x, f32x16 &acc) {
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(x), "+v"(acc) : "n"(later));
}
template <int later> __device__ inline void lds_arrived(bf16x4 &x0, bf16x4 &x1, f32x16 &acc) {
    asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(x0), "+v"(x1), "+v"(acc) : "n"(later));
}
template <int later> __device__ inline void lds_arrived(f32x4 &x0, f32x4 &x1, f32x4 &x2, f32x4 &x3) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3) : "n"(later));
}

}  // namespace jfa
