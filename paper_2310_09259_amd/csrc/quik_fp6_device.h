// FP6 (E3M2) operand format of the higher-rate 4-bit path.
// Private to the shared library.
//
// The signed 4-bit codes of QUIK-4B (Algorithm 1 of arXiv 2310.09259: values -8 .. 7) are all exactly
// representable in the 6-bit float format E3M2 (1 sign, 3 exponent bits with bias 3, 2 mantissa bits),
// their products are integers of magnitude <= 64, and a dot product over K_b < 262144 columns stays
// below 2^24, so an fp32 accumulator holds the integer result exactly.  gfx950 multiplies FP6 operands
// at twice its int8 rate (v_mfma_f32_32x32x64_f8f6f4), and the operands need no widening in registers.
//
// Operand layout ("panels").  The columns of a matrix with R rows are padded with zero codes to S
// stages of 64 columns (one step of the matrix instruction), and the matrix is stored stage by stage:
// stage s of row r is the 48-byte block at byte (s * R + r) * 48, so the rows of an output tile are one
// contiguous run per stage (whole cache lines for the copy engine, and nothing to rearrange on the way
// into LDS).  A stage holds two groups of 32 columns, g = 0, 1: the half of the wave's lanes that
// consumes it.  A group is 32 x 6 bits = six dwords d0 .. d5, column j of the group in bits
// [6j, 6j + 6) of that 192-bit little-endian string: exactly the register image one lane hands to the
// matrix instruction.  d0 .. d3 of group g sit at byte 16 g of the block, d4, d5 at byte 32 + 8 g.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace quik {
namespace fp6 {

// stages of 64 columns that cover K_b columns
__host__ __device__ inline int stages(int K_b) { return (K_b + 63) >> 6; }
// bytes of one row summed over its stages (a matrix of R rows takes R times this)
__host__ __device__ inline int row_bytes(int K_b) { return 48 * stages(K_b); }
// index (in dwords, inside the 48-byte block of its stage) of dword d (0 .. 5) of group g (0, 1)
__host__ __device__ inline int block_dword(int g, int d) { return d < 4 ? 4 * g + d : 8 + 2 * g + (d - 4); }

// E3M2 patterns of u - 8 for the unsigned codes u = 0 .. 7 (values -8 .. -1) and u = 8 .. 15 (0 .. 7)
constexpr uint32_t kNeg0 = 0x35363738u, kNeg1 = 0x2C303234u;   // -8 -7 -6 -5 | -4 -3 -2 -1
constexpr uint32_t kPos0 = 0x12100C00u, kPos1 = 0x17161514u;   //  0  1  2  3 |  4  5  6  7

// four unsigned codes, one per byte -> their four E3M2 patterns, one per byte
__device__ __forceinline__ uint32_t convert4(uint32_t n) {
    const uint32_t sel = n & 0x07070707u;
    const uint32_t m = ((n >> 3) & 0x01010101u) * 255u;          // 0xFF where u >= 8
    const uint32_t neg = __builtin_amdgcn_perm(kNeg1, kNeg0, sel);
    const uint32_t pos = __builtin_amdgcn_perm(kPos1, kPos0, sel);
    return (pos & m) | (neg & ~m);
}
// bytes b0 .. b3 (6 significant bits each) -> b0 | b1 << 12 | b2 << 24 | b3 << 36
__device__ __forceinline__ uint64_t spread4(uint32_t c) {
    const uint32_t lo = (c & 0x3Fu) | ((c & 0x3F00u) << 4) | ((c & 0x3F0000u) << 8);
    const uint32_t hi = (c >> 24) << 4;
    return ((uint64_t)hi << 32) | lo;
}
// eight unsigned 4-bit codes (element i in nibble i) -> 48 bits, element i in bits [6i, 6i + 6)
__device__ __forceinline__ uint64_t pack8(uint32_t codes) {
    const uint32_t even = convert4(codes & 0x0F0F0F0Fu);
    const uint32_t odd = convert4((codes >> 4) & 0x0F0F0F0Fu);
    return spread4(even) | (spread4(odd) << 6);
}

}  // namespace fp6
}  // namespace quik
