// Layout of an INT4 group-quantised expert block (MOE_LAYOUT_TILED_INT4).
//
// Values: each matrix of Eq. 3 is cut into groups of 32 consecutive elements
// along its contraction dimension (d_model for W_g and W_u, d_ff for W_d); a
// group holds 32 codes q in 0..15 and one bf16 scale s; weight = s * (q - 8).
//
// Gate/up section: one record per (row tile rt of 16 rows of d_ff, super-block
// sb of 128 columns), records ordered [rt][sb]:
//     [ 0,1024)  W_g: lane l of a wave owns 16 bytes; its 32-bit word j holds the
//                eight codes of row 16 rt + l%16, columns 128 sb + 32 j + 8 (l/16) + e,
//                e = 0..7, element e in nibble (e & 1) * 4 + (e >> 1)
//     [1024,2048) W_u, same arrangement
//     [2048,2304) scales: for row r = 0..15: bf16 s_g[j = 0..3], s_u[j = 0..3] of
//                the groups (row 16 rt + r, k-block 4 sb + j)
// Down section (after all gate/up records): one record per (chunk c of 32
// columns of W_d = 32 rows of d_ff, block dq of 64 rows of W_d), ordered [c][dq]:
//     [ 0,1024)  lane l, word j: codes of row 64 dq + 4 (l%16) + j, columns
//                32 c + 8 (l/16) + e, nibbles as above
//     [1024,1152) scales: for r = 0..15: bf16 s_d of rows 64 dq + 4 r + j, j = 0..3, group c
#pragma once
#include <stddef.h>

namespace moe {
namespace q4 {

constexpr size_t kGateUpRecord = 2304;
constexpr size_t kDownRecord = 1152;

__host__ __device__ inline size_t gate_up_bytes(int d, int f) { return (size_t)(f / 16) * (d / 128) * kGateUpRecord; }
__host__ __device__ inline size_t down_bytes(int d, int f) { return (size_t)(f / 32) * (d / 64) * kDownRecord; }
__host__ __device__ inline size_t block_bytes(int d, int f) { return gate_up_bytes(d, f) + down_bytes(d, f); }
__host__ __device__ inline int nibble_of(int e) { return (e & 1) * 4 + (e >> 1); }

}  // namespace q4
}  // namespace moe
