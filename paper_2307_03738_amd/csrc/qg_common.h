// Internal definitions shared by the HIP sources of libqg: the device blob layout and the
// argument checks.  Not part of the public interface (that is include/qg.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "qg.h"

#define QG_WAVE 64                 // gfx950 wavefront; one lane per output inside a tile
#define QG_SECTION_ALIGN 256       // byte alignment of the sections of a device blob
#define QG_MAX_CHUNKS 32           // upper bound of the K-split per tile (sizes the workspace)

// Device layout ("tile-major, one lane per output").
//
// Outputs are cut into tiles of 64 consecutive n; lane l of a wavefront owns output
// n = 64*tile + l, so x[k] is the same for every lane of the wavefront (it lives in scalar
// registers) and no cross-lane reduction is needed.  Along k the codes are cut into cells
// (8 codes = 1 word at 4 bits, 16 codes = 1 word at 2 bits, 32 codes = 3 words at 3 bits),
// four cells make a unit, and a unit is stored as `planes` 128-bit vectors per lane:
//
//   codes : uint4  [tile][unit][plane][lane]      one coalesced 1 KB load per wavefront
//   scales: float  [tile][group][lane]
//   zeros : uint32 [tile][zword][lane]            zbits per group, low bits first
//
// 2 and 4 bits: word j of the uint4 is cell j, fields in the paper's order (Algorithm 2:
// code i of the word in bits [b*i, b*i+b)).
// 3 bits: cell j is (plane0.w[j], plane1.w[j], plane2.w[j]) = (A, B, C).  Byte i of A holds
// code i in bits 0-2 and code 4+i in bits 3-5; B likewise codes 8+i, 12+i; C codes 16+i,
// 20+i.  The two spare bits of each of the three bytes i, concatenated A,B,C (low first),
// hold code 24+i (low three) and code 28+i (high three).  Every field is then reachable
// with one shift and one byte-lane mask, so no extraction has to cross a register.
//
// K is padded with zero codes to a whole number of steps (a step is what one wavefront
// loads per loop iteration: 4 units at 2 and 4 bits, 2 units at 3 bits); N is padded to
// whole tiles with zero codes, zero scales and zero zero-points.
struct QgLayout {
    int bits, group;
    int64_t N, K;
    int cell;        // codes per cell
    int unit;        // codes per unit = 4 cells
    int planes;      // uint4 per unit per lane
    int step_units;  // units per step
    int zbits;       // bits per stored zero-point
    int64_t tiles, units, steps, ngroups, zwords;
    size_t codes_off, scales_off, zeros_off, total;
};

static inline __host__ __device__ int qg_cell_of(int bits)
{
    return bits == 4 ? 8 : bits == 2 ? 16 : bits == 3 ? 32 : 0;
}

static inline size_t qg_round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Fills L and returns QG_OK, or the status that rejects the shape.
static inline int qg_make_layout(int64_t N, int64_t K, int bits, int group, QgLayout *L)
{
    if (bits != 2 && bits != 3 && bits != 4) return QG_ERR_UNSUPPORTED;
    if (N <= 0 || K <= 0 || group <= 0) return QG_ERR_SHAPE;
    if (N > (int64_t)1 << 24 || K > (int64_t)1 << 24) return QG_ERR_SHAPE;
    if (K % group != 0) return QG_ERR_SHAPE;
    const int cell = qg_cell_of(bits);
    if (group % cell != 0) return QG_ERR_SHAPE;
    L->bits = bits;
    L->group = group;
    L->N = N;
    L->K = K;
    L->cell = cell;
    L->unit = 4 * cell;
    L->planes = bits == 3 ? 3 : 1;
    L->step_units = bits == 3 ? 2 : 4;
    L->zbits = bits == 2 ? 2 : 4;
    L->tiles = (N + QG_WAVE - 1) / QG_WAVE;
    const int64_t step_codes = (int64_t)L->unit * L->step_units;
    L->steps = (K + step_codes - 1) / step_codes;
    L->units = L->steps * L->step_units;
    L->ngroups = K / group;
    const int zper = 32 / L->zbits;
    L->zwords = (L->ngroups + zper - 1) / zper;
    L->codes_off = 0;
    const size_t codes_bytes = (size_t)L->tiles * L->units * L->planes * QG_WAVE * 16;
    L->scales_off = qg_round_up(L->codes_off + codes_bytes, QG_SECTION_ALIGN);
    const size_t scales_bytes = (size_t)L->tiles * L->ngroups * QG_WAVE * 4;
    L->zeros_off = qg_round_up(L->scales_off + scales_bytes, QG_SECTION_ALIGN);
    const size_t zeros_bytes = (size_t)L->tiles * L->zwords * QG_WAVE * 4;
    L->total = qg_round_up(L->zeros_off + zeros_bytes, QG_SECTION_ALIGN);
    return QG_OK;
}

// Canonical blob: codes | scales | zeros, all uint32/float arrays with n contiguous.
struct QgCanonical {
    int64_t code_words, ngroups, zero_words;
    size_t codes_off, scales_off, zeros_off, total;
};

static inline int qg_make_canonical(int64_t N, int64_t K, int bits, int group, QgCanonical *C)
{
    if (bits != 2 && bits != 3 && bits != 4) return QG_ERR_UNSUPPORTED;
    if (N <= 0 || K <= 0 || group <= 0) return QG_ERR_SHAPE;
    if (N > (int64_t)1 << 24 || K > (int64_t)1 << 24) return QG_ERR_SHAPE;
    if (K % group != 0 || (K * bits) % 32 != 0) return QG_ERR_SHAPE;
    C->code_words = K * bits / 32;
    C->ngroups = K / group;
    C->zero_words = (C->ngroups * bits + 31) / 32;
    C->codes_off = 0;
    C->scales_off = (size_t)C->code_words * N * 4;
    C->zeros_off = C->scales_off + (size_t)C->ngroups * N * 4;
    C->total = C->zeros_off + (size_t)C->zero_words * N * 4;
    return QG_OK;
}

// Compute units of the current device (launch planning: wavefronts per CU).  Asked once per
// device; 256 (MI355X) if the runtime cannot say.
static inline int qg_compute_units()
{
    static int cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

static inline bool qg_aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

// Launch check: hipGetLastError after a launch, mapped to the library's status.
static inline int qg_launch_status()
{
    return hipGetLastError() == hipSuccess ? QG_OK : QG_ERR_DEVICE;
}
