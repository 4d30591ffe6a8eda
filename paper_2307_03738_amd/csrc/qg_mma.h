// Device helpers shared by the matrix-core kernels of libqg (GEMV and small-M GEMM): the cell /
// unit / step constants of each bit width and the unpacking of raw code words into bf16 operands
// of the matrix instructions.  Internal; every definition has internal linkage.
#pragma once

#include "qg_common.h"

namespace {

template <int BITS> struct Fmt;
template <> struct Fmt<4> { static constexpr int CELL = 8,  PLANES = 1, STEP_UNITS = 4, ZBITS = 4; };
template <> struct Fmt<2> { static constexpr int CELL = 16, PLANES = 1, STEP_UNITS = 4, ZBITS = 2; };
template <> struct Fmt<3> { static constexpr int CELL = 32, PLANES = 3, STEP_UNITS = 2, ZBITS = 4; };

template <int BITS> constexpr int loads_per_step() { return Fmt<BITS>::STEP_UNITS * Fmt<BITS>::PLANES; }
template <int BITS> constexpr int cells_per_step() { return Fmt<BITS>::STEP_UNITS * 4; }
template <int BITS> constexpr int codes_per_step() { return cells_per_step<BITS>() * Fmt<BITS>::CELL; }

__device__ inline uint32_t word_of(const uint4 &v, int j)
{
    return j == 0 ? v.x : j == 1 ? v.y : j == 2 ? v.z : v.w;
}

typedef __bf16 mma_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 mma_bf16x2 __attribute__((ext_vector_type(2)));
typedef float mma_floatx2 __attribute__((ext_vector_type(2)));
typedef float mma_floatx16 __attribute__((ext_vector_type(16)));

union MmaOperand {
    mma_bf16x8 v;
    uint32_t r[4];
    uint4 q;
};
// LDS holds the parts of x as 16-bit patterns written one by one and read eight at a time:
// both accesses go through types that may alias anything, so that they stay in program order
typedef uint16_t __attribute__((may_alias)) lds_u16;
typedef uint4 __attribute__((may_alias)) lds_u128;

#define QG_MMA_MAGIC 0x43004300u       // two bf16 128.0

// (v & mask) | magic.  Mask and magic reach this as register values the optimiser cannot see
// through (MmaConst), which is what makes it one v_and_or_b32 instead of an AND and an OR with
// literal operands.
__device__ inline uint32_t and_or(uint32_t v, uint32_t mask, uint32_t magic)
{
    return (v & mask) | magic;
}

struct MmaConst {
    uint32_t mask, magic;
    uint32_t mask_up;      // the mask of the fields one field further up (3 bits: three bits up; 2 bits: two)
    uint32_t mask_up2;     // 2 bits (gemv_mma4): the fields two fields further up
};

template <int BITS>
__device__ inline MmaConst mma_constants()
{
    MmaConst c;
    c.mask = BITS == 4 ? 0x000f000fu : BITS == 2 ? 0x00030003u : 0x00070007u;
    c.magic = QG_MMA_MAGIC;
    c.mask_up = BITS == 2 ? 0x000c000cu : 0x00380038u;
    c.mask_up2 = 0x00300030u;
    asm("" : "+s"(c.mask));
    asm("" : "+v"(c.magic));
    asm("" : "+s"(c.mask_up));
    asm("" : "+s"(c.mask_up2));
    return c;
}

// Codes per matrix-instruction operand: 8 per lane.  A cell unpacks into OPS operands.
template <int BITS> constexpr int mma_ops() { return Fmt<BITS>::CELL / 8; }

// Position (operand, element) of code i of a cell after unpacking; the x values are stored
// in the same order.
template <int BITS>
__device__ inline int mma_slot(int i)
{
    if constexpr (BITS == 4) {
        return i < 4 ? 2 * i : 2 * (i - 4) + 1;                 // register j = codes j, j + 4
    } else if constexpr (BITS == 2) {
        const int j = i & 7;                                     // register j = codes j, j + 8
        return (j >> 2) * 8 + 2 * (j & 3) + (i >> 3);
    } else {
        // word A, B, C or T holds codes 8 w + {0..7}: byte b has code b (low field) and
        // 4 + b (high field); registers take bytes (0, 2) low, (0, 2) high, (1, 3) low, (1, 3) high
        const int w = i >> 3, r = i & 7;
        const int b = r & 3, high = r >> 2;
        return w * 8 + ((b & 1) * 2 + high) * 2 + (b >> 1);
    }
}

// Unpacks the word(s) of one cell (already exchanged between the halves) into OPS operands.
template <int BITS>
__device__ inline void mma_unpack(const uint32_t *w, const MmaConst &c, MmaOperand *op)
{
    const uint32_t mask = c.mask, magic = c.magic;
    if constexpr (BITS == 4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) op[0].r[j] = and_or(w[0] >> (4 * j), mask, magic);
    } else if constexpr (BITS == 2) {
#pragma unroll
        for (int j = 0; j < 8; ++j) op[j >> 2].r[j & 3] = and_or(w[0] >> (2 * j), mask, magic);
    } else {
        // The high field of a byte is taken where it stands, three bits up in the mantissa:
        // those elements are 128 + 8 q instead of 128 + q (still exact in bf16), the x values
        // they meet are stored divided by 8, and the group's closing accounts for the offset
        // 16 instead of 128 (gemv_mma).  One shift per word instead of three.
        const uint32_t t = ((w[0] >> 6) & 0x03030303u) | ((w[1] >> 4) & 0x0c0c0c0cu) | ((w[2] >> 2) & 0x30303030u);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t src = k < 3 ? w[k] : t;
            const uint32_t up = src >> 8;
            op[k].r[0] = and_or(src, mask, magic);
            op[k].r[1] = and_or(src, c.mask_up, magic);
            op[k].r[2] = and_or(up, mask, magic);
            op[k].r[3] = and_or(up, c.mask_up, magic);
        }
    }
}

}  // namespace
