// Pieces shared by the direct-to-LDS backward kernels (jfa_bwd_bf16_dma.hip, jfa_bwd_dkv_dma.hip); not part of the C ABI.
#pragma once
#include "jfa_common.h"
#include "jfa_mfma.h"

namespace jfa {

constexpr int kBdThreads = 512;
constexpr int kBdBN = 64;             // streamed rows per LDS stage
constexpr int kBdD = 128;
constexpr int kBdTile = kBdBN * kBdD * 2;

enum BwdMode { kModeDQ = 0, kModeDK = 1, kModeDV = 2 };

template <int N> using IntB = std::integral_constant<int, N>;

// Row r, 16-byte chunk ch of a streamed tile sits at r * 256 + ((ch ^ swz(r)) << 4): conflict-free for the
// 16-byte row reads (16 consecutive rows hit 16 different chunk columns) and for the transposing reads
// (4 consecutive rows hit 4 different 64-byte groups) on the 64-bank LDS.
__device__ inline int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// Global -> LDS copies of 16 (or 4) bytes per lane: source = `base` (wave-uniform, scalar registers) +
// `byte_offset` (per lane, unsigned 32 bits), destination = lds_wave_base + 16 (or 4) * lane.  The scalar-base
// form needs no 64-bit vector address arithmetic and no vector registers for addresses.
__device__ inline void bd_dma16(const void *base, uint32_t byte_offset, char *lds_wave_base) {
    const char *src = reinterpret_cast<const char *>(base) + byte_offset;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                     (__attribute__((address_space(3))) void *)lds_wave_base, 16, 0, 0);
}
__device__ inline void bd_dma4(const void *base, uint32_t byte_offset, char *lds_wave_base) {
    const char *src = reinterpret_cast<const char *>(base) + byte_offset;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                     (__attribute__((address_space(3))) void *)lds_wave_base, 4, 0, 0);
}

}  // namespace jfa
