// Pieces shared by the direct-to-LDS backward kernels (jfa_bwd_dq_dma.hip, jfa_bwd_dkv_dma.hip); not part of the C ABI.
#pragma once
#include "jfa_common.h"
#include "jfa_mfma.h"
#include "jfa_lds.h"

namespace jfa {

constexpr int kBdThreads = 512;
constexpr int kBdBN = 64;             // streamed rows per LDS stage
constexpr int kBdD = 128;
constexpr int kBdTile = kBdBN * kBdD * 2;

template <int N> using IntB = std::integral_constant<int, N>;

// Row r, 16-byte chunk ch of a streamed tile sits at r * 256 + ((ch ^ swz(r)) << 4): conflict-free for the
// 16-byte row reads (16 consecutive rows hit 16 different chunk columns) and for the transposing reads
// (4 consecutive rows hit 4 different 64-byte groups) on the 64-bank LDS.
__device__ inline int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

}  // namespace jfa
