// libqg: the GEMV on the "narrow" device layout.
//
// y[n] = sum_g s[n][g] ( sum_{k in g} q[n][k] x[k]  -  z[n][g] sum_{k in g} x[k] )       (eq. (2))
//
// Same arithmetic as gemv_mma4i (qg_gemv.hip): codes enter v_mfma_i32_4x4x4_16B_i8 as int8 after
// masks, x as 32-bit fixed point cut into four signed base-256 digits, groups closed in fp32.
// What differs is which outputs and which k a wavefront's 1 KB load holds.
//
// The wide device layout gives a wavefront 64 outputs x one step of K per loop iteration, so a
// matrix with K = 4096 is 32 steps deep and a launch of short jobs (a few KB per wavefront, handed
// out by the hardware as others end -- what streams fastest on this machine) has to add partial
// results of several workgroups per output.  The narrow layout holds the same bytes in rows of
// 16 outputs x 4 steps: lane = 16 * slice + output, slice j of wave-step w being step 4 w + j.
// Eight wavefronts with one wave-step each then cover K = 4096 (4 bits) of their 16 outputs, a
// workgroup owns its outputs, and nothing is added across workgroups: no workspace, no atomics.
//
// What a wavefront needs for one wave-step is one contiguous record (with scales and zero-points
// in sections of their own -- three distant pieces per wave-step -- a 3-bit layer set of 140 MB ran
// 1 us longer; at 4 bits the two forms measured alike):
//
//   record [tile16][wave-step]:
//     codes : uint4  [load][lane]                       lane = 16 * slice + output
//     scales: float  [group of the step][lane]
//     zeros : uint32 [64 * zb / 32]                     zb = groups of a step x bits of a zero-point: lane l's
//                                                       zero-points are bits (l % (32 / zb)) * zb ... of word
//                                                       l / (32 / zb), its first group lowest; padded to 16 bytes
//
// Steps past the end of K and outputs past N hold zero codes, zero scales and zero zero-points.
//
// 4 bits: bit 7 of every code byte is stored inverted, which makes the byte's high code q read
// h = q - 8 as a two's-complement nibble, and the whole byte, read as int8, lo + 16 h.  The
// kernel multiplies x_lo with the whole byte and (x_hi / 16 - x_lo) with the byte under the mask
// 0xf0 (16 h):  x_lo (lo + 16 h) + (x_hi / 16 - x_lo) 16 h = x_lo lo + x_hi h, exactly, the
// subtraction being made on the fixed-point integers.  That is one mask per eight codes instead
// of two masks and a shift; 8 times the sum of the x that meet high codes puts the 8 back.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <stdint.h>

#include "qg_common.h"
#include "qg_mma.h"

namespace {

constexpr int NW_OUT = 16;             // outputs per wavefront
constexpr int NW_SLICES = 4;           // steps per wave-step
constexpr int NW_MAX_TEAM = 8;         // wavefronts per workgroup
constexpr int NW_MAX_SPW = 8;          // wave-steps one wavefront takes at most

struct NarrowLayout {
    int bits, group, gps, loads;       // gps: groups per step; loads: 128-bit vectors per lane and step
    int zb;                            // bits of zero-points per lane and wave-step
    int code_bytes, meta_zeros, meta_bytes;    // a record: codes, then scales, then (at meta_zeros behind the codes) zero-points
    int rec_bytes;
    int64_t N, K, tiles16, steps, wsteps;
    size_t total;
    QgLayout wide;
};

// (the same numbers at compile time, for the kernel)
template <int BITS, int GPS>
struct NarrowRecord {
    static constexpr int ZB = GPS * Fmt<BITS>::ZBITS;
    static constexpr int ZEROS = GPS * QG_WAVE * 4;
    static constexpr int META = ZEROS + (QG_WAVE * ZB / 8 + 15) / 16 * 16;
    static constexpr int CODES = loads_per_step<BITS>() * QG_WAVE * 16;
    static constexpr int BYTES = CODES + META;
};

// The formats the narrow layout takes: K a whole number of steps, groups of 16 weights (32 at 3
// bits) up to one step that divide a step, K within what one workgroup covers.
int make_narrow_layout(int64_t N, int64_t K, int bits, int group, NarrowLayout *L)
{
    const int rc = qg_make_layout(N, K, bits, group, &L->wide);
    if (rc != QG_OK) return rc;
    const int S = L->wide.unit * L->wide.step_units;
    if (K % S != 0 || group > S || S % group != 0 || group < (bits == 3 ? 32 : 16)) return QG_ERR_UNSUPPORTED;
    L->bits = bits;
    L->group = group;
    L->gps = S / group;
    L->loads = L->wide.step_units * L->wide.planes;
    L->N = N;
    L->K = K;
    L->tiles16 = (N + NW_OUT - 1) / NW_OUT;
    L->steps = L->wide.steps;
    L->wsteps = (L->steps + NW_SLICES - 1) / NW_SLICES;
    if (L->wsteps > NW_MAX_TEAM * NW_MAX_SPW) return QG_ERR_UNSUPPORTED;
    L->zb = L->gps * L->wide.zbits;
    if (L->zb > 32) return QG_ERR_UNSUPPORTED;
    L->meta_zeros = L->gps * QG_WAVE * 4;
    L->meta_bytes = L->meta_zeros + (QG_WAVE * L->zb / 8 + 15) / 16 * 16;
    L->code_bytes = L->loads * QG_WAVE * 16;
    L->rec_bytes = L->code_bytes + L->meta_bytes;
    L->total = qg_round_up((size_t)L->tiles16 * L->wsteps * L->rec_bytes, QG_SECTION_ALIGN);
    return QG_OK;
}

// ---- wide <-> narrow: 16-byte pieces and scales move, zero-points are re-packed ---------------
struct RepackArgs {
    const char *src;
    char *dst;
    size_t w_codes, w_scales, w_zeros;      // section offsets of the wide blob
    long tiles64, tiles16, steps, wsteps, ngroups, zwords;
    int loads, gps, zbits, zb;
    int meta_zeros, code_bytes, rec_bytes;
    uint32_t flip;                          // what every code word is XORed with on its way (either way)
};

// One thread per 16-byte piece of codes, per scale and per zero word of the blob that is written
// (the narrow records' zero words, or the wide blob's).
template <bool TO_NARROW>
__global__ void repack_narrow(const RepackArgs A)
{
    const size_t recs = (size_t)A.tiles16 * A.wsteps;
    const size_t per_rec = (size_t)(A.loads + A.gps) * QG_WAVE;
    const int zper = 32 / A.zbits, lpd = 32 / A.zb;         // zero-points per wide word; lanes per narrow word
    const uint32_t zmask = (1u << A.zbits) - 1u;
    size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < recs * per_rec) {
        const size_t r = e / per_rec;
        const int i = (int)(e % per_rec);
        const long w = (long)(r % A.wsteps), T = (long)(r / A.wsteps);
        const int lane = i % QG_WAVE;
        const long t = NW_SLICES * w + (lane >> 4), tile = T / 4;
        const int lane64 = (int)(T % 4) * NW_OUT + (lane & 15);
        const bool real = t < A.steps;
        const size_t codes_at = r * A.rec_bytes, meta_at = codes_at + A.code_bytes;
        if (i < A.loads * QG_WAVE) {
            const int ld = i / QG_WAVE;
            const size_t wide = ((size_t)(tile * A.steps + (real ? t : 0)) * A.loads + ld) * QG_WAVE + lane64;
            if (TO_NARROW) {
                uint4 v = make_uint4(0u, 0u, 0u, 0u);       // (a padded step meets zero scales: what its codes read as is immaterial)
                if (real) {
                    v = ((const uint4 *)(A.src + A.w_codes))[wide];
                    v.x ^= A.flip; v.y ^= A.flip; v.z ^= A.flip; v.w ^= A.flip;
                }
                ((uint4 *)(A.dst + codes_at))[ld * QG_WAVE + lane] = v;
            } else if (real) {
                uint4 v = ((const uint4 *)(A.src + codes_at))[ld * QG_WAVE + lane];
                v.x ^= A.flip; v.y ^= A.flip; v.z ^= A.flip; v.w ^= A.flip;
                ((uint4 *)(A.dst + A.w_codes))[wide] = v;
            }
        } else {
            const int gs = i / QG_WAVE - A.loads;
            const size_t wide = (size_t)(tile * A.ngroups + (real ? t * A.gps + gs : 0)) * QG_WAVE + lane64;
            if (TO_NARROW) ((float *)(A.dst + meta_at))[gs * QG_WAVE + lane] = real ? ((const float *)(A.src + A.w_scales))[wide] : 0.0f;
            else if (real) ((float *)(A.dst + A.w_scales))[wide] = ((const float *)(A.src + meta_at))[gs * QG_WAVE + lane];
        }
        return;
    }
    e -= recs * per_rec;
    if (TO_NARROW) {
        const int words = 2 * A.zb;                                 // zero words of a record
        if (e >= recs * words) return;
        const size_t r = e / words;
        const int d = (int)(e % words);
        const long w = (long)(r % A.wsteps), T = (long)(r / A.wsteps);
        uint32_t val = 0;
        for (int li = 0; li < lpd; ++li) {
            const int lane = d * lpd + li;
            const long t = NW_SLICES * w + (lane >> 4);
            if (t >= A.steps) continue;
            const int lane64 = (int)(T % 4) * NW_OUT + (lane & 15);
            for (int gs = 0; gs < A.gps; ++gs) {
                const long g = t * A.gps + gs;
                const uint32_t zw = ((const uint32_t *)(A.src + A.w_zeros))[(size_t)((T / 4) * A.zwords + g / zper) * QG_WAVE + lane64];
                val |= ((zw >> (A.zbits * (int)(g % zper))) & zmask) << (li * A.zb + gs * A.zbits);
            }
        }
        ((uint32_t *)(A.dst + r * A.rec_bytes + A.code_bytes + A.meta_zeros))[d] = val;
    } else {
        if (e >= (size_t)A.tiles64 * A.zwords * QG_WAVE) return;
        const int lane64 = (int)(e % QG_WAVE);
        const long zw = (long)((e / QG_WAVE) % A.zwords), tile = (long)(e / QG_WAVE / A.zwords);
        const long T = tile * 4 + lane64 / NW_OUT;
        uint32_t val = 0;
        if (T < A.tiles16)
            for (int f = 0; f < zper; ++f) {
                const long g = zw * zper + f;
                if (g >= A.ngroups) break;
                const long t = g / A.gps;
                const int gs = (int)(g % A.gps), lane = (int)(t % NW_SLICES) * NW_OUT + lane64 % NW_OUT;
                const size_t meta_at = ((size_t)T * A.wsteps + t / NW_SLICES) * A.rec_bytes + A.code_bytes;
                const uint32_t word = ((const uint32_t *)(A.src + meta_at + A.meta_zeros))[lane / lpd];
                val |= ((word >> ((lane % lpd) * A.zb + gs * A.zbits)) & zmask) << (A.zbits * f);
            }
        ((uint32_t *)(A.dst + A.w_zeros))[e] = val;
    }
}

__global__ void zero_bytes16(uint4 *p, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

// ---- the kernel --------------------------------------------------------------------------------
struct NarrowProblem {
    const char *blob;       // records [tile16][wave-step]
    const float *x;
    float *y;
    int N, steps, wsteps;
    int tiles16;
    int spw;                // wave-steps per wavefront
    int team;               // wavefronts with work
    int block_begin;        // first workgroup of this problem
};
struct NarrowArgs {
    NarrowProblem p[QG_MAX_GROUPED];
    int more_first[4];      // first workgroups of problems 13, 14, 15 (0x7fffffff past the last)
};
// The first workgroups of problems 1 ... 12 (0x7fffffff past the last) travel as twelve leading
// scalar kernel arguments: those reach a wavefront in registers when it starts (kernel-argument
// preload), so the search for its problem begins without a load, and the load of the problem's
// entry is the only one in front of the first loads of weights (launches of more than 13
// problems read the rest of the table from the argument buffer first).
typedef int nw_v4i __attribute__((ext_vector_type(4)));
#define NW_FIRST_BLOCKS const nw_v4i fb_a, const nw_v4i fb_b, const nw_v4i fb_c

typedef int nw_acc __attribute__((ext_vector_type(4)));
typedef uint8_t __attribute__((may_alias)) nw_lds_u8;
typedef uint32_t __attribute__((may_alias)) nw_lds_u32;

// v op (v moved across lanes by the DPP control CTRL), inside rows of 16 lanes
// (for bit patterns of non-negative floats: they order like unsigned integers, and a NaN is the largest)
template <int CTRL>
__device__ inline uint32_t nw_dpp_max(uint32_t v)
{
    const uint32_t moved = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, false);
    return v > moved ? v : moved;
}
template <int CTRL>
__device__ inline float nw_dpp_add(float v)
{
    const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false);
    return v + __int_as_float(moved);
}
constexpr int NW_QUAD_XOR1 = 0xB1, NW_QUAD_XOR2 = 0x4E, NW_HALF_MIRROR = 0x141, NW_ROW_MIRROR = 0x140;
constexpr int NW_ROW_BCAST0 = 0x150;          // lane n of every row to all lanes of the row: 0x150 + n

// Where value e of a lane's XPL consecutive x values goes among the lane's XPL operand bytes (the
// order the masked code fields have inside the B operands), and what its field counts.
template <int BITS>
__device__ constexpr int nw_byte_of(int e)
{
    return BITS == 4 ? (e % 2) * 4 + e / 2 : BITS == 2 ? (e % 4) * 4 + e / 4 : e;
}
template <int BITS>
__device__ constexpr int nw_value_at(int byte)      // inverse of nw_byte_of
{
    return BITS == 4 ? 2 * (byte % 4) + byte / 4 : BITS == 2 ? 4 * (byte % 4) + byte / 4 : byte;
}
template <int BITS>
__device__ constexpr float nw_xdiv(int e)           // 1 / (what the field of the code that meets value e counts)
{
    return BITS == 3 ? ((e & 7) >= 4 ? 0.125f : 1.0f)
         : BITS == 2 ? ((e & 3) == 1 ? 0.25f : (e & 3) == 2 ? 0.0625f : 1.0f)
                     : ((e & 1) ? 0.0625f : 1.0f);
}

// lane G * LPG of every row of 16 lanes to all lanes of the row, for G = 0 .. GPS - 1
template <int GPS, int LPG, int G = 0>
__device__ inline void nw_spread(float part, float *xhat)
{
    if constexpr (G < GPS) {
        xhat[G] = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(part), NW_ROW_BCAST0 + G * LPG, 0xf, 0xf, false));
        nw_spread<GPS, LPG, G + 1>(part, xhat);
    }
}

// TPW: tiles of 16 outputs a wavefront takes through its wave-steps, one after the other against
// the same digits of x (the staging of x is the larger part of a wave-step's vector work).
template <int BITS, int GPS, int TPW>
__global__ __launch_bounds__(NW_MAX_TEAM * QG_WAVE) void gemv_narrow(NW_FIRST_BLOCKS, const NarrowArgs A)
{
    using F = Fmt<BITS>;
    constexpr int L = loads_per_step<BITS>();
    constexpr int S = codes_per_step<BITS>();
    constexpr int XPL = S / NW_OUT;                 // x values per lane and wave-step: 8 or 16
    constexpr int READS = S / 16;                   // 128-bit reads of A per step, four matrix instructions each
    constexpr int RPG = READS / GPS;
    constexpr int LPG = NW_OUT / GPS;               // lanes whose x values make up one group
    using R = NarrowRecord<BITS, GPS>;
    constexpr int LPW = 32 / R::ZB;                 // lanes whose zero-points share a word
    constexpr int PITCH = S + 16;                   // bytes per digit row: the four rows on different banks
    static_assert(GPS >= 1 && GPS <= NW_OUT && READS % GPS == 0 && R::ZB <= 32 && 32 % R::ZB == 0, "groups of a step");
    __shared__ float red[NW_MAX_TEAM][TPW * NW_OUT];
    // per wavefront and slice: the four digit rows of the slice's x in operand order
    __shared__ __attribute__((aligned(16))) nw_lds_u8 xs[NW_MAX_TEAM][NW_SLICES][4][PITCH];

    // which problem: the last one whose first workgroup is <= this one
    const int first[12] = {fb_a.x, fb_a.y, fb_a.z, fb_a.w, fb_b.x, fb_b.y, fb_b.z, fb_b.w, fb_c.x, fb_c.y, fb_c.z, fb_c.w};
    const int bid = (int)blockIdx.x;
    int pi = 0;
#pragma unroll
    for (int i = 0; i < 12; ++i)
        if (bid >= first[i]) pi = i + 1;
    if (first[11] != 0x7fffffff) {
#pragma unroll
        for (int i = 0; i < 3; ++i)
            if (bid >= A.more_first[i]) pi = 13 + i;
    }
    const NarrowProblem P = A.p[pi];
    // every field now, so that the loads of the entry are issued together
    asm volatile("" ::"s"(P.blob), "s"(P.x), "s"(P.y));
    asm volatile("" ::"s"(P.N), "s"(P.steps), "s"(P.wsteps), "s"(P.tiles16), "s"(P.spw), "s"(P.team),
                 "s"(P.block_begin));
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int T0 = (bid - P.block_begin) * TPW;
    const int j = lane >> 4, o = lane & 15;
    const int w0 = wave * P.spw;
    if (w0 >= P.wsteps) return;                     // no work: leave before the barrier
    const int w1 = w0 + P.spw < P.wsteps ? w0 + P.spw : P.wsteps;

    // uniform bases; what a lane adds to them fits 32 bits.  A tile past the last one reads the
    // last one again and stores nothing.
    const char *records[TPW];                       // the tile's record of wave-step 0
#pragma unroll
    for (int u = 0; u < TPW; ++u) {
        const int T = T0 + u < P.tiles16 ? T0 + u : P.tiles16 - 1;
        records[u] = P.blob + (size_t)T * P.wsteps * R::BYTES;
    }
    nw_lds_u8 *mine = &xs[wave][j][0][0] + o * XPL;              // this lane's bytes of digit row 0
    const nw_lds_u8 *abase = &xs[wave][j][lane & 3][0];         // the digit row this lane supplies to its block

    float yacc[TPW];
#pragma unroll
    for (int u = 0; u < TPW; ++u) yacc[u] = 0.0f;
    for (int w = w0; w < w1; ++w) {
        // A slice past the end of K has zero codes and zero scales and adds nothing whatever x it
        // meets; it takes the last step's x (its output meets that x in a real slice as well).
        const int t = NW_SLICES * w + j;
        const uint32_t tc = (uint32_t)(t < P.steps ? t : P.steps - 1);
        // x goes first: loads return in order, and its digits are made while the codes are on their way
        float xv[XPL];
        {
            const float4 *src = (const float4 *)P.x;
#pragma unroll
            for (int q = 0; q < XPL / 4; ++q) {
                const float4 f = src[tc * (S / 4) + (uint32_t)o * (XPL / 4) + q];
                xv[4 * q + 0] = f.x;
                xv[4 * q + 1] = f.y;
                xv[4 * q + 2] = f.z;
                xv[4 * q + 3] = f.w;
            }
        }
        uint4 v[TPW][L];
        float s[TPW][GPS];
        uint32_t zword[TPW];
#pragma unroll
        for (int u = 0; u < TPW; ++u) {
#pragma unroll
            for (int i = 0; i < L; ++i)
                v[u][i] = *(const uint4 *)(records[u] + ((uint32_t)w * R::BYTES + (uint32_t)(i * QG_WAVE + lane) * 16u));
#pragma unroll
            for (int g = 0; g < GPS; ++g)
                s[u][g] = *(const float *)(records[u] + ((uint32_t)w * R::BYTES + R::CODES + (uint32_t)(g * QG_WAVE + lane) * 4u));
            zword[u] = *(const uint32_t *)(records[u] + ((uint32_t)w * R::BYTES + R::CODES + R::ZEROS + (uint32_t)(lane / LPW) * 4u));
        }
        __builtin_amdgcn_sched_barrier(0);                        // every load is requested before the arithmetic starts
#pragma unroll
        for (int u = 0; u < TPW; ++u) zword[u] >>= (lane % LPW) * R::ZB;     // this lane's zero-points, first group lowest

        // fixed point of the slice: |x| scale < 2^30 for its largest |x|
        float mf = 0.0f;
#pragma unroll
        for (int e = 0; e < XPL; ++e) mf = fmaxf(mf, fabsf(xv[e]));
        uint32_t m = __float_as_uint(mf);
        m = nw_dpp_max<NW_QUAD_XOR1>(m);
        m = nw_dpp_max<NW_QUAD_XOR2>(m);
        m = nw_dpp_max<NW_HALF_MIRROR>(m);
        m = nw_dpp_max<NW_ROW_MIRROR>(m);                         // every lane of the row holds the row's maximum
        uint32_t eb = m >> 23;                                    // biased exponent (m >= 0)
        eb = eb < 30u ? 30u : eb > 254u ? 254u : eb;
        const float scale = __uint_as_float((283u - eb) << 23);   // 2^(156 - eb)
        const float inv = __uint_as_float((eb - 29u) << 23);      // 2^(eb - 156)
        uint32_t pat[XPL];
#pragma unroll
        for (int e = 0; e < XPL; ++e) {
            // the four bytes of (fixed + 0x808080) ^ 0x808080, read as signed, are digits base 256 of
            // `fixed`; the 0x808080 is added in fp32 (where that rounds, it rounds below the last bit of x)
            int lifted = (int)fmaf(xv[e], scale * nw_xdiv<BITS>(e), (BITS == 4 && (e & 1)) ? 2.0f * 8421504.0f : 8421504.0f);
            // 4 bits: the value that meets a byte's high code is x_hi / 16 - x_lo in fixed point (the
            // low code's operand is the whole byte, lo + 16 hi': what x_lo gathers from hi' comes off here)
            if constexpr (BITS == 4)
                if (e & 1) lifted -= (int)(pat[e - 1] ^ 0x00808080u);
            pat[e] = (uint32_t)lifted ^ 0x00808080u;
        }
        // digit row r of this lane: byte b holds digit r of the value that belongs at byte b
        // (a 4 x 4 byte transpose per four values)
#pragma unroll
        for (int d = 0; d < XPL / 4; ++d) {
            const uint32_t p0 = pat[nw_value_at<BITS>(4 * d + 0)], p1 = pat[nw_value_at<BITS>(4 * d + 1)];
            const uint32_t p2 = pat[nw_value_at<BITS>(4 * d + 2)], p3 = pat[nw_value_at<BITS>(4 * d + 3)];
            const uint32_t lo01 = __builtin_amdgcn_perm(p1, p0, 0x05010400u), hi01 = __builtin_amdgcn_perm(p1, p0, 0x07030602u);
            const uint32_t lo23 = __builtin_amdgcn_perm(p3, p2, 0x05010400u), hi23 = __builtin_amdgcn_perm(p3, p2, 0x07030602u);
            *(nw_lds_u32 *)(mine + 0 * PITCH + 4 * d) = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);
            *(nw_lds_u32 *)(mine + 1 * PITCH + 4 * d) = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
            *(nw_lds_u32 *)(mine + 2 * PITCH + 4 * d) = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
            *(nw_lds_u32 *)(mine + 3 * PITCH + 4 * d) = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
        }

        // x-hat of the slice's groups: the lanes of a group add up, every lane of the row gets every sum
        // (4 bits: the high codes read 8 too low, which 8 times the sum of the x they meet makes up for)
        float part = 0.0f, part_high = 0.0f;
#pragma unroll
        for (int e = 0; e < XPL; ++e) {
            if (BITS == 4 && (e & 1)) part_high += xv[e];
            else part += xv[e];
        }
        if constexpr (BITS == 4) part += part_high;
        if constexpr (LPG >= 2) part = nw_dpp_add<NW_QUAD_XOR1>(part);
        if constexpr (LPG >= 4) part = nw_dpp_add<NW_QUAD_XOR2>(part);
        if constexpr (LPG >= 8) part = nw_dpp_add<NW_HALF_MIRROR>(part);
        if constexpr (LPG >= 16) part = nw_dpp_add<NW_ROW_MIRROR>(part);
        float xhat[GPS], lift[GPS];
        if constexpr (GPS == 1) {
            xhat[0] = part;
        } else {
            nw_spread<GPS, LPG>(part, xhat);
        }
        if constexpr (BITS == 4) {
            part_high *= 8.0f;
            if constexpr (LPG >= 2) part_high = nw_dpp_add<NW_QUAD_XOR1>(part_high);
            if constexpr (LPG >= 4) part_high = nw_dpp_add<NW_QUAD_XOR2>(part_high);
            if constexpr (LPG >= 8) part_high = nw_dpp_add<NW_HALF_MIRROR>(part_high);
            if constexpr (LPG >= 16) part_high = nw_dpp_add<NW_ROW_MIRROR>(part_high);
            if constexpr (GPS == 1) {
                lift[0] = part_high;
            } else {
                nw_spread<GPS, LPG>(part_high, lift);
            }
        } else {
#pragma unroll
            for (int g = 0; g < GPS; ++g) lift[g] = 0.0f;
        }

        // the matrix instructions: per 128-bit read of A (16 k) two 4-bit cells, one 2-bit cell or
        // half a 3-bit cell; lane l receives the sums of its own output.  The B operands are the
        // code fields where they sit in their bytes (the x that meets a field counts it by its
        // place: nw_xdiv), 4 bits: the whole byte and its high nibble.
        nw_acc acc0[TPW], acc1[TPW];
        uint32_t spare[TPW];
#pragma unroll
        for (int u = 0; u < TPW; ++u) {
            acc0[u] = nw_acc{0, 0, 0, 0};
            acc1[u] = nw_acc{0, 0, 0, 0};
            spare[u] = 0;
        }
#pragma unroll
        for (int rd = 0; rd < READS; ++rd) {
            MmaOperand a;
            a.q = *(const lds_u128 *)(abase + rd * 16);
#pragma unroll
            for (int u = 0; u < TPW; ++u) {
                uint32_t b[4];
                if constexpr (BITS == 4) {
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        const int cell = 2 * rd + c;
                        const uint32_t wd = word_of(v[u][cell >> 2], cell & 3);
                        b[2 * c] = wd;                      // int8: lo + 16 (hi - 8)
                        b[2 * c + 1] = wd & 0xf0f0f0f0u;    // int8: 16 (hi - 8), against x_hi / 16 - x_lo
                    }
                } else if constexpr (BITS == 2) {
                    const uint32_t wd = word_of(v[u][rd >> 2], rd & 3);
                    b[0] = wd & 0x03030303u;
                    b[1] = wd & 0x0c0c0c0cu;
                    b[2] = wd & 0x30303030u;
                    b[3] = (wd >> 6) & 0x03030303u;
                } else {
                    const int cell = rd >> 1, un = cell >> 2, c = cell & 3;
                    if ((rd & 1) == 0) {
                        const uint32_t wa = word_of(v[u][un * 3], c), wb = word_of(v[u][un * 3 + 1], c),
                                       wc = word_of(v[u][un * 3 + 2], c);
                        spare[u] = ((wa >> 6) & 0x03030303u) | ((wb >> 4) & 0x0c0c0c0cu) | ((wc >> 2) & 0x30303030u);
                        b[0] = wa & 0x07070707u;
                        b[1] = wa & 0x38383838u;
                        b[2] = wb & 0x07070707u;
                        b[3] = wb & 0x38383838u;
                    } else {
                        const uint32_t wc = word_of(v[u][un * 3 + 2], c);
                        b[0] = wc & 0x07070707u;
                        b[1] = wc & 0x38383838u;
                        b[2] = spare[u] & 0x07070707u;
                        b[3] = spare[u] & 0x38383838u;
                    }
                }
                acc0[u] = __builtin_amdgcn_mfma_i32_4x4x4i8((int)a.r[0], (int)b[0], acc0[u], 0, 0, 0);
                acc1[u] = __builtin_amdgcn_mfma_i32_4x4x4i8((int)a.r[1], (int)b[1], acc1[u], 0, 0, 0);
                acc0[u] = __builtin_amdgcn_mfma_i32_4x4x4i8((int)a.r[2], (int)b[2], acc0[u], 0, 0, 0);
                acc1[u] = __builtin_amdgcn_mfma_i32_4x4x4i8((int)a.r[3], (int)b[3], acc1[u], 0, 0, 0);
                if ((rd + 1) % RPG == 0) {
                    const int gs = (rd + 1) / RPG - 1;
                    // sum_i 256^i D_i of the group, in units of 1 / scale (|D_i| stays below 2^21)
                    const int lo = (acc0[u][1] + acc1[u][1]) * 256 + (acc0[u][0] + acc1[u][0]);
                    const int hi = (acc0[u][3] + acc1[u][3]) * 256 + (acc0[u][2] + acc1[u][2]);
                    acc0[u] = nw_acc{0, 0, 0, 0};
                    acc1[u] = nw_acc{0, 0, 0, 0};
                    const float tsum = fmaf((float)hi, 65536.0f, (float)lo) * inv;
                    const uint32_t zq = (zword[u] >> (F::ZBITS * gs)) & ((1u << F::ZBITS) - 1u);
                    yacc[u] = fmaf(s[u][gs], fmaf(-(float)zq, xhat[gs], BITS == 4 ? tsum + lift[gs] : tsum), yacc[u]);
                }
            }
        }
    }

    // the four slices of an output, then the wavefronts of the workgroup in order
    // (lanes 16 u + o of wavefront 0 finish tile u)
    float mine_y = 0.0f;
#pragma unroll
    for (int u = 0; u < TPW; ++u) {
        yacc[u] += __shfl_xor(yacc[u], 16, QG_WAVE);
        yacc[u] += __shfl_xor(yacc[u], 32, QG_WAVE);
        if (j == u) mine_y = yacc[u];
    }
    if (lane < TPW * NW_OUT) red[wave][lane] = mine_y;
    __syncthreads();
    if (wave != 0 || lane >= TPW * NW_OUT) return;
    float sum = red[0][lane];
    for (int k = 1; k < P.team; ++k) sum += red[k][lane];
    const int n = (T0 + j) * NW_OUT + o;
    if (T0 + j < P.tiles16 && n < P.N) P.y[n] = sum;
}

typedef void (*NarrowKernel)(nw_v4i, nw_v4i, nw_v4i, const NarrowArgs);

template <int BITS, int TPW>
NarrowKernel pick_narrow(int gps)
{
    switch (gps) {
    case 1: return gemv_narrow<BITS, 1, TPW>;
    case 2: return gemv_narrow<BITS, 2, TPW>;
    case 4: return gemv_narrow<BITS, 4, TPW>;
    case 8: return gemv_narrow<BITS, 8, TPW>;
    case 16:
        if constexpr (BITS == 2) return gemv_narrow<2, 16, TPW>;
        return nullptr;
    default: return nullptr;
    }
}

int g_narrow_tpw = 0;       // measurement knob: tiles per wavefront, 0 = built-in choice

char g_narrow_kernel[48] = "";

int repack(const void *src, void *dst, int64_t N, int64_t K, int bits, int group, bool to_narrow, hipStream_t st)
{
    NarrowLayout L;
    const int rc = make_narrow_layout(N, K, bits, group, &L);
    if (rc != QG_OK) return rc;
    if (!src || !dst) return QG_ERR_NULL;
    if (!qg_aligned16(src) || !qg_aligned16(dst)) return QG_ERR_ALIGN;
    RepackArgs A;
    A.src = (const char *)src;
    A.dst = (char *)dst;
    A.w_codes = L.wide.codes_off; A.w_scales = L.wide.scales_off; A.w_zeros = L.wide.zeros_off;
    A.tiles64 = (long)L.wide.tiles; A.tiles16 = (long)L.tiles16; A.steps = (long)L.steps; A.wsteps = (long)L.wsteps;
    A.ngroups = (long)L.wide.ngroups; A.zwords = (long)L.wide.zwords;
    A.zbits = L.wide.zbits; A.zb = L.zb;
    A.meta_zeros = L.meta_zeros; A.code_bytes = L.code_bytes; A.rec_bytes = L.rec_bytes;
    A.loads = L.loads; A.gps = L.gps;
    A.flip = bits == 4 ? 0x80808080u : 0u;
    const size_t elements = (size_t)L.tiles16 * L.wsteps * (L.loads + L.gps) * QG_WAVE +
                            (to_narrow ? (size_t)L.tiles16 * L.wsteps * 2 * L.zb : (size_t)L.wide.tiles * L.wide.zwords * QG_WAVE);
    if ((elements + 255) / 256 > 0x7fffffffu) return QG_ERR_SHAPE;
    const unsigned blocks = (unsigned)((elements + 255) / 256);
    // the destination is cleared first: the padding of its records or sections, and (wide) the
    // outputs past the last tile of 16, are written by nothing else
    const size_t n16 = (to_narrow ? L.total : L.wide.total) / 16;
    hipLaunchKernelGGL(zero_bytes16, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, st, (uint4 *)dst, n16);
    if (qg_launch_status() != QG_OK) return QG_ERR_DEVICE;
    if (to_narrow) hipLaunchKernelGGL(repack_narrow<true>, dim3(blocks), dim3(256), 0, st, A);
    else hipLaunchKernelGGL(repack_narrow<false>, dim3(blocks), dim3(256), 0, st, A);
    return qg_launch_status();
}
}  // namespace

size_t qg_narrow_bytes(int64_t N, int64_t K, int bits, int group)
{
    NarrowLayout L;
    return make_narrow_layout(N, K, bits, group, &L) == QG_OK ? L.total : 0;
}

extern "C" int qg_to_narrow(const void *packed, int64_t N, int64_t K, int bits, int group, void *narrow, void *stream)
{
    return repack(packed, narrow, N, K, bits, group, true, (hipStream_t)stream);
}

extern "C" int qg_from_narrow(const void *narrow, int64_t N, int64_t K, int bits, int group, void *packed, void *stream)
{
    return repack(narrow, packed, N, K, bits, group, false, (hipStream_t)stream);
}

extern "C" const char *qg_last_narrow_kernel(void) { return g_narrow_kernel; }

extern "C" int qg_set_narrow_tuning(int tiles_per_wave)
{
    if (tiles_per_wave < 0 || tiles_per_wave > 2) return QG_ERR_SHAPE;
    g_narrow_tpw = tiles_per_wave;
    return QG_OK;
}

extern "C" int qg_gemv_grouped_narrow(const qg_gemv_desc *descs, int count, void *stream)
{
    if (!descs) return QG_ERR_NULL;
    if (count <= 0) return QG_ERR_SHAPE;
    if (count > QG_MAX_GROUPED) return QG_ERR_UNSUPPORTED;
    NarrowLayout L[QG_MAX_GROUPED];
    for (int i = 0; i < count; ++i) {
        const int rc = make_narrow_layout(descs[i].N, descs[i].K, descs[i].bits, descs[i].group, &L[i]);
        if (rc != QG_OK) return rc;
        if (!descs[i].packed || !descs[i].x || !descs[i].y) return QG_ERR_NULL;
        if (!qg_aligned16(descs[i].packed) || ((uintptr_t)descs[i].x & 63u)) return QG_ERR_ALIGN;
        if (L[i].tiles16 > (1 << 24)) return QG_ERR_SHAPE;
    }
    // one launch per (bits, groups per step); inside a launch the longest K first, so that the
    // wavefronts that run longest start first.  Two passes: every launch is planned before the
    // first one is enqueued.
    for (int pass = 0; pass < 2; ++pass) {
        bool done[QG_MAX_GROUPED] = {false};
        for (int i = 0; i < count; ++i) {
            if (done[i]) continue;
            int idx[QG_MAX_GROUPED], n = 0;
            for (int k = i; k < count; ++k)
                if (!done[k] && L[k].bits == L[i].bits && L[k].gps == L[i].gps) {
                    idx[n++] = k;
                    done[k] = true;
                }
            for (int a = 1; a < n; ++a)
                for (int b = a; b > 0 && L[idx[b]].K > L[idx[b - 1]].K; --b) {
                    const int t = idx[b]; idx[b] = idx[b - 1]; idx[b - 1] = t;
                }
            // (measured on the three layer sets: two tiles per wavefront pay at 2 bits, where a wave-step's
            // codes are half as many bytes per x value staged; one tile is ahead at 3 and 4 bits)
            const int tpw = g_narrow_tpw ? g_narrow_tpw : L[i].bits == 2 ? 2 : 1;
            const NarrowKernel fn = tpw == 2 ? (L[i].bits == 4 ? pick_narrow<4, 2>(L[i].gps) : L[i].bits == 2 ? pick_narrow<2, 2>(L[i].gps) : pick_narrow<3, 2>(L[i].gps))
                                             : (L[i].bits == 4 ? pick_narrow<4, 1>(L[i].gps) : L[i].bits == 2 ? pick_narrow<2, 1>(L[i].gps) : pick_narrow<3, 1>(L[i].gps));
            if (!fn) return QG_ERR_UNSUPPORTED;
            NarrowArgs A;
            int first[QG_MAX_GROUPED];
            for (int k = 0; k < QG_MAX_GROUPED; ++k) first[k] = 0x7fffffff;
            long blocks = 0;
            int team_max = 1;
            for (int k = 0; k < n; ++k) {
                const NarrowLayout &Lk = L[idx[k]];
                const qg_gemv_desc &d = descs[idx[k]];
                NarrowProblem &P = A.p[k];
                P.blob = (const char *)d.packed;
                P.x = d.x;
                P.y = d.y;
                P.N = (int)Lk.N;
                P.steps = (int)Lk.steps;
                P.wsteps = (int)Lk.wsteps;
                P.tiles16 = (int)Lk.tiles16;
                P.spw = (int)((Lk.wsteps + NW_MAX_TEAM - 1) / NW_MAX_TEAM);
                P.team = (int)((Lk.wsteps + P.spw - 1) / P.spw);
                P.block_begin = (int)blocks;
                first[k] = (int)blocks;
                blocks += (long)((Lk.tiles16 + tpw - 1) / tpw);
                if (P.team > team_max) team_max = P.team;
            }
            for (int k = n; k < QG_MAX_GROUPED; ++k) A.p[k] = A.p[0];
            if (blocks > 0x7fffffffL) return QG_ERR_SHAPE;
            if (pass == 0) continue;
            const nw_v4i fa = {first[1], first[2], first[3], first[4]}, fb = {first[5], first[6], first[7], first[8]};
            const nw_v4i fc = {first[9], first[10], first[11], first[12]};
            A.more_first[0] = first[13]; A.more_first[1] = first[14]; A.more_first[2] = first[15]; A.more_first[3] = 0x7fffffff;
            hipLaunchKernelGGL(fn, dim3((unsigned)blocks), dim3((unsigned)team_max * QG_WAVE), 0, (hipStream_t)stream, fa, fb, fc, A);
            if (qg_launch_status() != QG_OK) return QG_ERR_DEVICE;
            snprintf(g_narrow_kernel, sizeof g_narrow_kernel, "gemv_narrow<%d, %d, %d>", L[i].bits, L[i].gps, tpw);
        }
    }
    return QG_OK;
}

extern "C" int qg_gemv_narrow(const void *narrow, int64_t N, int64_t K, int bits, int group,
                              const float *x, float *y, void *stream)
{
    qg_gemv_desc d;
    d.packed = narrow;
    d.N = N;
    d.K = K;
    d.bits = bits;
    d.group = group;
    d.x = x;
    d.y = y;
    return qg_gemv_grouped_narrow(&d, 1, stream);
}
