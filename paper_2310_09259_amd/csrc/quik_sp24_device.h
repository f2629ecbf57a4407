// Operand formats of the 2:4-sparse 4-bit path (signed 4-bit weights of which at most two in every
// group of four consecutive base columns are nonzero: the joint INT4 + 2:4 format of Section 4.3.2
// of arXiv 2310.09259, whose arithmetic is Algorithm 1 unchanged).
// Private to the shared library.
//
// gfx950 multiplies a 2:4-compressed int8 operand at twice its dense int8 rate
// (v_smfmac_i32_32x32x64_i8: 32 x 32 outputs, 64 columns per step, exact INT32 accumulation).  Measured
// operand layout of that instruction, lane l = (row or column l % 32, half g = l / 32):
//   dense operand:   32 bytes per lane; byte b of half g is column 32 g + b of the step, so dword d is
//                    the group of four columns kappa = 8 g + d;
//   sparse operand:  16 bytes per lane; bytes 2 q, 2 q + 1 (q = 0 .. 7) are the two kept values of group
//                    kappa = 8 (q / 4) + 4 g + q % 4;
//   index register:  bits [2 c, 2 c + 2) of the sparse operand's lane = position (0 .. 3) inside its group
//                    of the value in byte c;
//   accumulator:     lane = column of the dense operand, register r = row 8 (r / 4) + 4 g + r % 4 of the
//                    sparse operand.
//
// Both matrices are stored stage by stage (a stage = 64 columns = one step, columns padded with zeros to
// S = ceil(K_b / 64) stages), the rows of a stage one after the other, so the rows of an output tile are
// one contiguous run per stage.
//
// Activations (R = T rows): 32 bytes per row and stage, byte (s R + r) 32 + b.  Byte b = 4 m + p holds
// columns 8 m + p (high nibble) and 8 m + 4 + p (low nibble) of the stage as two's complement nibbles:
// (word & 0xF0F0F0F0) and ((word << 4) & 0xF0F0F0F0) are then sixteen times the int8 values of two
// whole groups of four, byte p = position p, which is what the dense operand wants.
//
// Weights (R = N rows): 32 bytes per row and stage, one 16-byte record per half: 8 bytes of values, the
// 4-byte index word, 4 bytes of zero padding (so that one 16-byte LDS read fetches all a lane needs; read
// instructions, not bytes, are what the K loop pays for).  Value c (0 .. 15) of a half sits in dword c / 8
// of its 8 bytes, byte c % 4, low nibble if (c / 4) % 2 == 0, else high: (dword << 4) & 0xF0F0F0F0 and
// dword & 0xF0F0F0F0 of the two dwords are the four registers of the sparse operand, sixteen times the
// int8 values.
// Kept positions of a group: its nonzero positions, filled up to two with the lowest unused positions
// (whose values are zero), in ascending order.
// Accumulators are exactly 256 times the integer dot products; |256 * 64 * K_b / 2| < 2^31 for
// K_b < 262144.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace quik {
namespace sp24 {

__host__ __device__ inline int stages(int K_b) { return (K_b + 63) >> 6; }
constexpr int kActBytes = 32;      // per row and stage
constexpr int kWgtBytes = 32;

// group kappa of a stage -> (half g, pair q) of the sparse operand
__host__ __device__ inline int half_of_group(int kappa) { return (kappa >> 2) & 1; }
__host__ __device__ inline int pair_of_group(int kappa) { return 4 * (kappa >> 3) + (kappa & 3); }

// Eight two's complement nibbles, column i in nibble i -> the activation byte order of this format:
// byte p = column p in the high nibble, column p + 4 in the low nibble.
__device__ __forceinline__ uint32_t act_word(uint32_t w) {
    // byte pairs (B0, B0, B1, B1) and (B2, B2, B3, B3) of w
    const uint32_t P = __builtin_amdgcn_perm(0u, w, 0x01010000u);
    const uint32_t Q = __builtin_amdgcn_perm(0u, w, 0x03030202u);
    const uint32_t hi = ((P << 4) & 0x00F000F0u) | (P & 0xF000F000u);          // columns 0 .. 3
    const uint32_t lo = (Q & 0x000F000Fu) | ((Q >> 4) & 0x0F000F00u);          // columns 4 .. 7
    return hi | lo;
}

}  // namespace sp24
}  // namespace quik
