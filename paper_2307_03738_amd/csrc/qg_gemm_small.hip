// qg_gemm_small: Y = X What^T for a few prompt tokens (M <= 128) on the matrix cores.
//
// The paper treats only the vector input; this is the same What = s (q - z) (Section 2,
// eq. (1)) applied to M activation rows at once.  X and the dequantized weights are rounded
// to bf16, products are accumulated in fp32 by v_mfma_f32_32x32x16_bf16.
//
// Mapping (4-bit codes, groups of 32, 64, 128 or a multiple of 128).  A wavefront owns one
// tile of 64 outputs -- the same device layout the GEMV reads, lane l holding 32 consecutive
// k of output 64*tile + l in one 128-bit vector -- and all M rows.  The matrix instruction
// wants, for a block of 32 outputs, lanes l and l+32 to hold the SAME output with two
// different k-octets; the layout has them hold two different outputs with the same k.  One
// v_permlane32_swap of the raw code words (w0 with w2, w1 with w3) turns one into the other
// for both 32-output blocks at once, so weights go from HBM to the MFMA operand through
// registers only: mask, convert, one FMA with the group's (s, -z s), pack to bf16.  Every
// weight is dequantized exactly once.
//
// A wavefront holds at most 64 activation rows (64 accumulator registers); more rows run as
// two row blocks on the grid's z axis.  A workgroup is four wavefronts laid out as TN tiles x
// KW k-slices (TN * KW = 4): four neighbouring tiles over the same k (KW = 1) when the launch
// has enough workgroups anyway, otherwise two or four consecutive k-steps of fewer tiles
// (KW = 2, 4), whose accumulators are added through LDS at the end -- more wavefronts for
// small problems without more partial results.  The activation rows are converted to bf16
// on their way into LDS, KW * 128 k at a time, double-buffered, shared by the workgroup; the
// loads of the next chunk are issued a quarter at a time between the units of the running
// step, because the path from L2 into a compute unit is what the activations load most.
// Codes, scales and zero-points of the next step are in flight while the current one is
// computed.  K may also be cut into `splits` ranges handled by different workgroups; their
// fp32 partial results are added by a second small kernel in a fixed order.
//
// Other bit widths and group sizes take the fp32 GEMV kernel once per activation row, up to
// 16 rows per launch.
#include <mutex>
#include <type_traits>

#include "qg_common.h"
#include "qg_mma.h"

size_t qg_gemm_workspace_bytes(const QgLayout &L, int M);
int qg_gemm_rows16(const void *packed, int64_t N, int64_t K, int bits, int group, const float *X,
                   int M, float *Y, void *workspace, void *stream, bool dry);   // qg_gemv.hip
int qg_gemv_grouped_check(const qg_gemv_desc *descs, int count, void *workspace, size_t workspace_bytes);

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int KC = 128;            // k per step of the 4-bit layout

struct GemmArgs {
    const uint4 *codes;
    const float *scales;
    const uint32_t *zeros;
    const float *X;            // activations [M][K] fp32
    float *out;                // Y, or partial results [split][M][N]
    int M, N, K, tiles, steps, ngroups, zwords;
    int group_shift;           // log2(G) for G <= 128
    int steps_per_group;       // G / 128 for G > 128, else 1
    int steps_per_split;       // a multiple of KW and of steps_per_group
};

__device__ inline uint32_t opaque(uint32_t v)
{
    asm("" : "+v"(v));
    return v;
}

union Operand {
    bf16x8 v;
    bf16x2 p[4];
};

// Eight 4-bit codes of one word -> eight bf16 values s*(q - z), in code order.  The odd codes
// are taken with one mask, sixteen times too large, and multiplied by s / 16 (exact).
__device__ inline bf16x8 dequant_word(uint32_t w, float s, float nzs)
{
    const uint32_t lo = opaque(w & 0x0f0f0f0fu);          // codes 0, 2, 4, 6
    const uint32_t hi = opaque(w & 0xf0f0f0f0u);          // codes 1, 3, 5, 7, times 16
    const float sh = s * 0.0625f;
    Operand o;
    floatx2 t;
    t[0] = fmaf((float)(lo & 0xffu), s, nzs);          t[1] = fmaf((float)(hi & 0xffu), sh, nzs);
    o.p[0] = __builtin_convertvector(t, bf16x2);
    t[0] = fmaf((float)((lo >> 8) & 0xffu), s, nzs);   t[1] = fmaf((float)((hi >> 8) & 0xffu), sh, nzs);
    o.p[1] = __builtin_convertvector(t, bf16x2);
    t[0] = fmaf((float)((lo >> 16) & 0xffu), s, nzs);  t[1] = fmaf((float)((hi >> 16) & 0xffu), sh, nzs);
    o.p[2] = __builtin_convertvector(t, bf16x2);
    t[0] = fmaf((float)(lo >> 24), s, nzs);            t[1] = fmaf((float)(hi >> 24), sh, nzs);
    o.p[3] = __builtin_convertvector(t, bf16x2);
    return o.v;
}

// v_permlane32_swap(a, b) returns {[a.low half | b.low half], [a.high half | b.high half]}
// (halves of 32 lanes): `low` is a in lanes 0-31 and b's lanes 0-31 in lanes 32-63; `high` is
// a's lanes 32-63 in lanes 0-31 and b in lanes 32-63.
__device__ inline void swap_halves(uint32_t a, uint32_t b, uint32_t &low, uint32_t &high)
{
    const auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
    low = r[0];
    high = r[1];
}

// What one wavefront needs for one step (128 k of its tile): four code vectors, the scale of
// each 32-k unit and the word holding the zero-points of the step's groups.
struct StepRegs {
    uint4 v[4];
    float s[4];
    uint32_t zw;
};

template <int MB, int TN, int KW, bool G128>
__global__ __launch_bounds__(TN * KW * 64) void gemm_small_b4(const GemmArgs A)
{
    constexpr int GEMM_THREADS = TN * KW * 64; // TN tiles x KW k-slices, one wavefront each
    constexpr int ROWS = MB * 32;              // activation rows held (rows past M are zero)
    constexpr int XK = KW * KC;                // k per workgroup iteration
    constexpr int XPITCH = XK + 8;             // bf16 per LDS row: conflict-free 128-bit reads
    constexpr int XLOADS = ROWS * (XK / 4) / GEMM_THREADS;   // float4 loads per thread and chunk
    constexpr int ACC = MB * 2 * 16;           // accumulator registers per lane
    // two activation buffers: the chunk of the next iteration is written while this one is
    // read; reused at the end for the accumulators of the k-slices 1 .. KW-1
    constexpr int XBYTES = 2 * ROWS * XPITCH * 2;
    constexpr int RBYTES = (KW - 1) * TN * ACC * 64 * 4;
    __shared__ __attribute__((aligned(16))) char smem[XBYTES > RBYTES ? XBYTES : RBYTES];
    __bf16 *Xs = (__bf16 *)smem;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tn = wave % TN, kw = wave / TN;
    const int tile = blockIdx.x * TN + tn;
    const bool have_tile = tile < A.tiles;
    const int m0 = blockIdx.z * ROWS;                       // first activation row of this workgroup
    const int rows = A.M - m0 < ROWS ? A.M - m0 : ROWS;      // real rows among the ROWS held
    const int st0 = blockIdx.y * A.steps_per_split;
    int st1 = st0 + A.steps_per_split;
    if (st1 > A.steps) st1 = A.steps;
    const int iters = (st1 - st0 + KW - 1) / KW;

    const int tclamp = have_tile ? tile : A.tiles - 1;
    const uint4 *codes = A.codes + (size_t)tclamp * A.steps * 4 * QG_WAVE + lane;
    const float *sc = A.scales + (size_t)tclamp * A.ngroups * QG_WAVE + lane;
    const uint32_t *zr = A.zeros + (size_t)tclamp * A.zwords * QG_WAVE + lane;

    floatx16 acc[MB][2];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mb][nb][i] = 0.0f;

    const int half = lane >> 5;           // which k-octet pair this lane feeds
    const int row = lane & 31;

    // group of unit u (32 k) of a step: G <= 128 has 128/G groups per step, G > 128 has
    // G/128 steps per group (then group_shift is 7 and the unit term vanishes)
    const int step_shift = 7 - A.group_shift;
    auto first_group = [&](int step) { return (step / A.steps_per_group) << step_shift; };
    auto unit_group = [&](int g0, int u) { return g0 + ((u * 32) >> A.group_shift); };
    auto fetch = [&](int step, StepRegs &r) {
#pragma unroll
        for (int u = 0; u < 4; ++u) r.v[u] = codes[((size_t)step * 4 + u) * QG_WAVE];
        const int g0 = first_group(step);
#pragma unroll
        for (int u = 0; u < 4; ++u) r.s[u] = sc[(size_t)unit_group(g0, u) * QG_WAVE];
        r.zw = zr[(size_t)(g0 >> 3) * QG_WAVE];      // a step's groups share one zero word
    };

    // this thread's share of an activation chunk: XLOADS pieces of 4 consecutive k, RPP rows
    // apart, converted to bf16 (round to nearest even) on the way into LDS.  Pieces with no
    // real row are skipped (their LDS rows keep whatever they held), other rows past M repeat
    // the last real row, and k past K repeats the last piece: a row of the A operand only
    // reaches the same row of the result, and rows past M are never stored; k past K belongs
    // to steps no wavefront runs.  Offsets are rebuilt at every use (two operations per piece) rather
    // than kept in registers across the loop.
    constexpr int RPP = GEMM_THREADS / (XK / 4);
    constexpr int XPART = XLOADS / 4;          // pieces issued per 32-k unit of the running step
    const int xrow = threadIdx.x / (XK / 4), xcol = (threadIdx.x % (XK / 4)) * 4;
    float4 xr[XLOADS];
    auto load_x_part = [&](int k0, int part) {
        const float *base = A.X + (size_t)m0 * A.K + k0;     // uniform
        const uint32_t r = opaque((uint32_t)xrow);
        const uint32_t last = (uint32_t)(A.K - 4 - k0);
        const uint32_t col = (uint32_t)xcol < last ? (uint32_t)xcol : last;
#pragma unroll
        for (int j = part * XPART; j < (part + 1) * XPART; ++j) {
            if (j * RPP >= rows) continue;                   // uniform: no real row in this piece
            uint32_t m = r + j * RPP;
            m = m < (uint32_t)rows ? m : (uint32_t)(rows - 1);
            xr[j] = *(const float4 *)(base + (m * (uint32_t)A.K + col));
        }
    };
    auto store_x = [&](int buf) {
        __bf16 *dst = Xs + (size_t)(buf * ROWS + xrow) * XPITCH + xcol;
#pragma unroll
        for (int j = 0; j < XLOADS; ++j) {
            if (j * RPP >= rows) continue;
            floatx2 a = {xr[j].x, xr[j].y}, b = {xr[j].z, xr[j].w};
            bf16x2 pa = __builtin_convertvector(a, bf16x2), pb = __builtin_convertvector(b, bf16x2);
            uint2 packed;
            packed.x = *(uint32_t *)&pa;
            packed.y = *(uint32_t *)&pb;
            *(uint2 *)(dst + j * RPP * XPITCH) = packed;
        }
    };

    // One step of this wavefront: dequantize 64 outputs x 128 k, multiply with all rows.  The
    // A operands of unit u + 1 are read from LDS while unit u is multiplied; with `xk0` >= 0 a
    // quarter of the next activation chunk is requested at the start of every unit, so the
    // memory pipeline works alongside the arithmetic instead of ahead of it.
    auto compute = [&](const StepRegs &r, int step, int buf, int xk0) {
        const int g0 = first_group(step);
        const __bf16 *xs = Xs + (size_t)buf * ROWS * XPITCH + kw * KC + row * XPITCH + half * 16;
        bf16x8 a0[MB], a1[MB], n0[MB], n1[MB];
        uint32_t sP = 0, sQ = 0, nP = 0, nQ = 0;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            a0[mb] = *(const bf16x8 *)(xs + mb * 32 * XPITCH);          // octet 0 or 2
            a1[mb] = *(const bf16x8 *)(xs + mb * 32 * XPITCH + 8);      // octet 1 or 3
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (xk0 >= 0) load_x_part(xk0, u);
            if (u < 3) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    n0[mb] = *(const bf16x8 *)(xs + mb * 32 * XPITCH + (u + 1) * 32);
                    n1[mb] = *(const bf16x8 *)(xs + mb * 32 * XPITCH + (u + 1) * 32 + 8);
                }
            }
            // outputs 0-31 of the tile in both halves (P), outputs 32-63 in both halves (Q);
            // G128: the units of a step share one group, whose scale and zero term are
            // exchanged once per step (the lane exchange costs about five issue slots)
            uint32_t P0, Q0, P1, Q1;
            if (!G128 || u == 0) {
                const float s = r.s[u];
                const int g = unit_group(g0, u);
                const float nzs = -(float)((r.zw >> (4 * (g & 7))) & 15u) * s;
                swap_halves(__float_as_uint(s), __float_as_uint(s), sP, sQ);
                swap_halves(__float_as_uint(nzs), __float_as_uint(nzs), nP, nQ);
            }
            swap_halves(r.v[u].x, r.v[u].z, P0, Q0);   // k-octets 0 (low lanes) and 2 (high lanes)
            swap_halves(r.v[u].y, r.v[u].w, P1, Q1);   // k-octets 1 and 3
            const bf16x8 bP0 = dequant_word(P0, __uint_as_float(sP), __uint_as_float(nP));
            const bf16x8 bQ0 = dequant_word(Q0, __uint_as_float(sQ), __uint_as_float(nQ));
            const bf16x8 bP1 = dequant_word(P1, __uint_as_float(sP), __uint_as_float(nP));
            const bf16x8 bQ1 = dequant_word(Q1, __uint_as_float(sQ), __uint_as_float(nQ));
            // consecutive matrix instructions write different accumulators
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                acc[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[mb], bP0, acc[mb][0], 0, 0, 0);
                acc[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[mb], bQ0, acc[mb][1], 0, 0, 0);
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                acc[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[mb], bP1, acc[mb][0], 0, 0, 0);
                acc[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[mb], bQ1, acc[mb][1], 0, 0, 0);
            }
            if (u < 3) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    a0[mb] = n0[mb];
                    a1[mb] = n1[mb];
                }
            }
            __builtin_amdgcn_sched_barrier(0);     // units stay in order
        }
    };
    // Every iteration but the last has all KW steps inside the split, so the loop body is
    // straight-line code: issue the loads of iteration it + 1, compute iteration it from
    // registers and LDS filled one iteration earlier, then move the new data into place.
    StepRegs cur, nxt;
    if (iters > 0) {
        const int step = st0 + kw;
        fetch(step < st1 ? step : st1 - 1, cur);
#pragma unroll
        for (int part = 0; part < 4; ++part) load_x_part(st0 * KC, part);
        store_x(0);
    }
    __syncthreads();
    int buf = 0;
    for (int it = 0; it + 1 < iters; ++it) {
        const int step = st0 + it * KW + kw;
        const int ns = step + KW;
        fetch(ns < st1 ? ns : st1 - 1, nxt);
        __builtin_amdgcn_sched_barrier(0);     // weight loads first ...
        compute(cur, step, buf, (st0 + (it + 1) * KW) * KC);
        __builtin_amdgcn_sched_barrier(0);     // ... and nothing that waits for them before the arithmetic is done
        store_x(buf ^ 1);
        cur = nxt;
        __syncthreads();      // next chunk written, this chunk's readers done
        buf ^= 1;
    }
    if (iters > 0) {
        const int step = st0 + (iters - 1) * KW + kw;
        if (step < st1) compute(cur, step, buf, -1);
    }

    if constexpr (KW > 1) {
        // k-slices 1 .. KW-1 hand their accumulators to slice 0 of the same tile, which adds
        // them in slice order; the buffers of X are reused once every reader is done
        float *red = (float *)smem;
        __syncthreads();
        if (kw > 0) {
            float *dst = red + ((size_t)((kw - 1) * TN + tn) * ACC) * 64 + lane;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) dst[((mb * 2 + nb) * 16 + i) * 64] = acc[mb][nb][i];
        }
        __syncthreads();
        if (kw > 0) return;
#pragma unroll
        for (int k = 1; k < KW; ++k) {
            const float *src = red + ((size_t)((k - 1) * TN + tn) * ACC) * 64 + lane;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[mb][nb][i] += src[((mb * 2 + nb) * 16 + i) * 64];
        }
    }

    if (!have_tile) return;
    float *out = A.out + (size_t)blockIdx.y * A.M * A.N;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            const int n = tile * QG_WAVE + nb * 32 + row;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int m = m0 + mb * 32 + 8 * (i / 4) + 4 * half + (i % 4);
                if (m < A.M && n < A.N) out[(size_t)m * A.N + n] = acc[mb][nb][i];
            }
        }
}

// ---------------------------------------------------------------------------------------
// The same product for 33 ... 128 rows with every activation row in one wavefront, so each
// weight is dequantized once however many rows there are, and with the dequantization of unit
// u + 1 issued between the matrix instructions of unit u: a wavefront alone keeps the vector
// ALU and the matrix core busy at the same time (the kernel above clumps them, and two
// wavefronts per SIMD that leave a barrier together clump in step).
//
// A workgroup is TN wavefronts = TN neighbouring tiles over the same k range (no k-slices);
// an iteration is a pair of steps (256 k).  The activations of the next pair go through
// registers into the second LDS buffer an eighth at a time, each eighth stored DELAY units
// after it was requested; codes, scales and zero words are requested one iteration (two
// steps) ahead.
// ---------------------------------------------------------------------------------------
template <int MB, int TN, bool G128>
__global__ __launch_bounds__(TN * 64, MB == 2 ? 2 : 1) void gemm_wide_b4(const GemmArgs A)
{
    constexpr int THREADS = TN * 64;
    constexpr int ROWS = MB * 32;
    constexpr int XK = 2 * KC;                              // k per iteration
    constexpr int XPITCH = XK + 8;                          // bf16 per LDS row
    constexpr int XLOADS = ROWS * (XK / 4) / THREADS;       // float4 per thread and chunk
    constexpr int XPART = XLOADS / 8;                       // ... and unit
    constexpr int RPP = THREADS / (XK / 4);                 // rows between a thread's pieces
    constexpr int DELAY = 2;                                // units between a request for activations and its use
    constexpr int NM = MB * 4;                              // matrix instructions per unit
    constexpr int PPM = 16 / NM;                            // pieces of dequantization per matrix instruction
    static_assert(XPART >= 1 && XLOADS % 8 == 0, "a chunk is moved in eight parts");
    static_assert(MB == 2 || MB == 4, "16 pieces are dealt over 8 or 16 matrix instructions");
    __shared__ __attribute__((aligned(16))) char smem[2 * ROWS * XPITCH * 2];
    __bf16 *Xs = (__bf16 *)smem;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tile = blockIdx.x * TN + wave;
    const bool have_tile = tile < A.tiles;
    const int rows = A.M < ROWS ? A.M : ROWS;
    const int st0 = blockIdx.y * A.steps_per_split;
    int st1 = st0 + A.steps_per_split;
    if (st1 > A.steps) st1 = A.steps;
    const int npairs = (st1 - st0 + 1) / 2;

    const int tclamp = have_tile ? tile : A.tiles - 1;
    const uint4 *codes = A.codes + (size_t)tclamp * A.steps * 4 * QG_WAVE + lane;
    const float *sc = A.scales + (size_t)tclamp * A.ngroups * QG_WAVE + lane;
    const uint32_t *zr = A.zeros + (size_t)tclamp * A.zwords * QG_WAVE + lane;

    floatx16 acc[MB][2];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mb][nb][i] = 0.0f;

    const int half = lane >> 5;
    const int row = lane & 31;
    const int step_shift = 7 - A.group_shift;
    auto first_group = [&](int step) { return (step / A.steps_per_group) << step_shift; };
    auto unit_group = [&](int g0, int u) { return g0 + ((u * 32) >> A.group_shift); };
    auto fetch = [&](int step, StepRegs &r) {
        step = step < st1 ? step : st1 - 1;            // past the range: loaded again, not used
#pragma unroll
        for (int u = 0; u < 4; ++u) r.v[u] = codes[((size_t)step * 4 + u) * QG_WAVE];
        const int g0 = first_group(step);
#pragma unroll
        for (int u = 0; u < 4; ++u) r.s[u] = sc[(size_t)unit_group(g0, u) * QG_WAVE];
        r.zw = zr[(size_t)(g0 >> 3) * QG_WAVE];
    };

    // Activations: piece j of a thread is 4 consecutive k of row j * RPP + wave, so a wavefront
    // reads 1 KB of one row.  Rows past M repeat the last real row (a row of the A operand only
    // reaches the same row of the result, and those are not stored); k past K repeats the last
    // piece of the row (it belongs to a step that is not run).  No branches: the loads of a
    // part must stay countable for the waits that follow.
    const int xcol = lane * 4;
    auto load_x = [&](int k0, int j, float4 &dst) {
        const float *base = A.X + k0;                          // uniform
        const uint32_t last = (uint32_t)(A.K - 4 - k0);
        const uint32_t col = (uint32_t)xcol < last ? (uint32_t)xcol : last;
        int m = j * RPP + wave;                                // uniform
        m = m < rows ? m : rows - 1;
        dst = *(const float4 *)(base + ((size_t)m * (uint32_t)A.K + col));
    };
    auto store_x = [&](int buf, int j, const float4 &src) {
        floatx2 a = {src.x, src.y}, b = {src.z, src.w};
        bf16x2 pa = __builtin_convertvector(a, bf16x2), pb = __builtin_convertvector(b, bf16x2);
        uint2 packed;
        packed.x = *(uint32_t *)&pa;
        packed.y = *(uint32_t *)&pb;
        *(uint2 *)(Xs + (size_t)(buf * ROWS + j * RPP + wave) * XPITCH + xcol) = packed;
    };

    // Dequantization of one unit in 16 pieces (4 words x 4 byte positions, two codes each).
    struct UnitPrep {
        uint32_t lo[4], hi[4];     // words P0, Q0, P1, Q1: even codes, odd codes (times 16)
        float s[2], sh[2], nz[2];  // of outputs 0-31 (P) and 32-63 (Q)
    };
    // G128: the four units of a step share one group (G >= 128), so the scale and zero term
    // are exchanged between the halves once per step (the lane exchange is the most expensive
    // vector instruction of the loop: about five issue slots)
    auto prepare = [&](const StepRegs &r, int g0, int u, UnitPrep &pr) {
        uint32_t w[4];
        if (!G128 || u == 0) {
            const float s = r.s[u];
            const int g = unit_group(g0, u);
            const float nzs = -(float)((r.zw >> (4 * (g & 7))) & 15u) * s;
            uint32_t sP, sQ, nP, nQ;
            swap_halves(__float_as_uint(s), __float_as_uint(s), sP, sQ);
            swap_halves(__float_as_uint(nzs), __float_as_uint(nzs), nP, nQ);
            pr.s[0] = __uint_as_float(sP);  pr.s[1] = __uint_as_float(sQ);
            pr.sh[0] = pr.s[0] * 0.0625f;   pr.sh[1] = pr.s[1] * 0.0625f;
            pr.nz[0] = __uint_as_float(nP); pr.nz[1] = __uint_as_float(nQ);
        }
        swap_halves(r.v[u].x, r.v[u].z, w[0], w[1]);       // k-octets 0 | 2
        swap_halves(r.v[u].y, r.v[u].w, w[2], w[3]);       // k-octets 1 | 3
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            pr.lo[i] = opaque(w[i] & 0x0f0f0f0fu);
            pr.hi[i] = opaque(w[i] & 0xf0f0f0f0u);
        }
    };
    UnitPrep pr;               // lives across units and iterations: with G128 its scale part is per step
    auto piece = [&](const UnitPrep &pr, int i, Operand (&o)[4]) {
        const int wd = i >> 2, j = i & 3, pq = wd & 1;
        floatx2 t;
        t[0] = fmaf((float)((pr.lo[wd] >> (8 * j)) & 0xffu), pr.s[pq], pr.nz[pq]);
        t[1] = fmaf((float)((pr.hi[wd] >> (8 * j)) & 0xffu), pr.sh[pq], pr.nz[pq]);
        bf16x2 pair = __builtin_convertvector(t, bf16x2);
        // an empty volatile statement: keeps this piece in the slot it is written in
        uint32_t bits = *(uint32_t *)&pair;
        asm volatile("" : "+v"(bits));
        o[wd].p[j] = *(bf16x2 *)&bits;
    };

    // The units of one iteration.  Matrix instruction k of unit uu is followed by pieces of
    // the dequantization of unit uu + 1 (of the next pair's first step after the last unit,
    // if NEXT), by the LDS reads of that unit's A operands and by the traffic of the next
    // activation chunk; every such slot is fenced, so the order written here is the order
    // issued.  bq: B operands P0, Q0, P1, Q1 of the unit about to be multiplied.
    auto compute = [&](auto nu_tag, auto next_tag, const StepRegs &r0, const StepRegs &r1, const StepRegs &rn,
                       int step0, int buf, Operand (&bq)[4]) {
        constexpr int NU = decltype(nu_tag)::value;
        constexpr bool NEXT = decltype(next_tag)::value;
        const int g00 = first_group(step0), g01 = first_group(step0 + 1), g02 = first_group(step0 + 2);
        const int xk0 = (step0 + 2) * KC;
        const __bf16 *xs = Xs + (size_t)buf * ROWS * XPITCH + row * XPITCH + half * 16;
        bf16x8 a0[MB], a1[MB], n0[MB], n1[MB];
        float4 xr[DELAY + 1][XPART];
        Operand bn[4];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            a0[mb] = *(const bf16x8 *)(xs + mb * 32 * XPITCH);
            a1[mb] = *(const bf16x8 *)(xs + mb * 32 * XPITCH + 8);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int uu = 0; uu < NU; ++uu) {
            const bool more = uu + 1 < NU;                  // next unit in this pair
            const bool dq = more || NEXT;                   // something to dequantize
#pragma unroll
            for (int k = 0; k < NM; ++k) {
                const int mb = (k % (MB * 2)) / 2, nb = k % 2;
                if (k < MB * 2)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[mb], bq[nb].v, acc[mb][nb], 0, 0, 0);
                else
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[mb], bq[2 + nb].v, acc[mb][nb], 0, 0, 0);
                if (k == 0) {
                    if (NEXT) {
#pragma unroll
                        for (int i = 0; i < XPART; ++i) load_x(xk0, uu * XPART + i, xr[uu % (DELAY + 1)][i]);
                    }
                    if (more) {
#pragma unroll
                        for (int m2 = 0; m2 < MB; ++m2) {
                            n0[m2] = *(const bf16x8 *)(xs + m2 * 32 * XPITCH + (uu + 1) * 32);
                            n1[m2] = *(const bf16x8 *)(xs + m2 * 32 * XPITCH + (uu + 1) * 32 + 8);
                        }
                    }
                    if (dq) {
                        if (more) prepare(uu + 1 < 4 ? r0 : r1, uu + 1 < 4 ? g00 : g01, (uu + 1) & 3, pr);
                        else prepare(rn, g02, 0, pr);
                    }
                }
                if (dq) {
#pragma unroll
                    for (int q = 0; q < PPM; ++q) piece(pr, k * PPM + q, bn);
                }
                if (NEXT && k == NM / 2 && uu >= DELAY) {
#pragma unroll
                    for (int i = 0; i < XPART; ++i)
                        store_x(buf ^ 1, (uu - DELAY) * XPART + i, xr[(uu - DELAY) % (DELAY + 1)][i]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (more) {
#pragma unroll
                for (int m2 = 0; m2 < MB; ++m2) {
                    a0[m2] = n0[m2];
                    a1[m2] = n1[m2];
                }
            }
            if (dq) {
#pragma unroll
                for (int i = 0; i < 4; ++i) bq[i].v = bn[i].v;
            }
        }
        if (NEXT) {
#pragma unroll
            for (int uu = NU - DELAY; uu < NU; ++uu)
#pragma unroll
                for (int i = 0; i < XPART; ++i) store_x(buf ^ 1, uu * XPART + i, xr[uu % (DELAY + 1)][i]);
        }
    };

    using std::integral_constant;
    StepRegs c0, c1, n0, n1;
    Operand bq[4];
    if (npairs > 0) {
        fetch(st0, c0);
        fetch(st0 + 1, c1);
        float4 xall[XLOADS];
#pragma unroll
        for (int j = 0; j < XLOADS; ++j) load_x(st0 * KC, j, xall[j]);
#pragma unroll
        for (int j = 0; j < XLOADS; ++j) store_x(0, j, xall[j]);
        prepare(c0, first_group(st0), 0, pr);
#pragma unroll
        for (int i = 0; i < 16; ++i) piece(pr, i, bq);
    }
    __syncthreads();
    int buf = 0;
    for (int p = 0; p + 1 < npairs; ++p) {
        const int s = st0 + 2 * p;
        fetch(s + 2, n0);
        fetch(s + 3, n1);
        __builtin_amdgcn_sched_barrier(0);
        compute(integral_constant<int, 8>(), integral_constant<bool, true>(), c0, c1, n0, s, buf, bq);
        __builtin_amdgcn_sched_barrier(0);
        c0 = n0;
        c1 = n1;
        __syncthreads();      // next chunk written, this chunk's readers done
        buf ^= 1;
    }
    if (npairs > 0) {
        const int s = st0 + 2 * (npairs - 1);
        if (s + 1 < st1) compute(integral_constant<int, 8>(), integral_constant<bool, false>(), c0, c1, c1, s, buf, bq);
        else compute(integral_constant<int, 4>(), integral_constant<bool, false>(), c0, c1, c1, s, buf, bq);
    }

    if (!have_tile) return;
    float *out = A.out + (size_t)blockIdx.y * A.M * A.N;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            const int n = tile * QG_WAVE + nb * 32 + row;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int m = mb * 32 + 8 * (i / 4) + 4 * half + (i % 4);
                if (m < A.M && n < A.N) out[(size_t)m * A.N + n] = acc[mb][nb][i];
            }
        }
}


// ---------------------------------------------------------------------------------------
// gemm_codes: the same product with the weights entering the matrix instruction as RAW CODES.
//
// Nothing is dequantized per weight.  A code q becomes the exact bf16 integer 128 + q with a mask
// and an OR (mma_unpack, as in the matrix-core GEMV), the matrix instruction accumulates
//     T[m][n] = sum_{k in group} xb[m][k] (128 + q[n][k]),      xb = X rounded to bf16,
// in fp32 (the products are exact), and scale and zero-point are applied once per group and
// accumulator element, which is eq. (2) per element of Y:
//     Y[m][n] += s[n][g] * ( T[m][n] - (128 + z[n][g]) * xhat[m][g] ),   xhat[m][g] = sum_k xb[m][k].
// The subtraction rides on the matrix cores as well: xhat, cut into three bf16 parts (exact), is one
// more A operand per group and -(128 + z) one more B operand, so a group costs one fused
// multiply-add per accumulator element and nothing else on the vector ALU.
// (3 bits: the high field of a byte stays where it is, so half of the codes enter as 128 + 8 q
// against activations stored divided by 8; those have an xhat of their own and the offset 16.)
//
// Two kernels.  prepare_x converts X once per call: bf16 in the order the unpacked codes have
// inside an operand, rows padded with zeros to whole blocks of 32, K to whole steps, plus the
// xhat operands -- so that the product kernel moves activations into LDS with plain copies and
// spends its vector instructions on the weights alone.  gemm_codes: a wavefront owns a tile of
// 64 outputs (device layout, lane = output); one v_permlane32_swap per pair of code words turns
// "lane = output" into the operand layout (lanes l and l + 32 hold two neighbouring cells of the
// same output).  A workgroup is 8 wavefronts = TN tiles x KW k-slices that share the activation
// chunk of an iteration (KW steps) in LDS, double buffered; the k-slices add their results
// through LDS at the end.  A wavefront holds MB blocks of 32 activation rows; more rows run as
// further workgroups (grid z), and K may be cut into ranges handled by different workgroups
// whose partial results add_splits sums.
// CPG: cells per group (groups inside a step), or 0 for groups of whole steps (any number; a
// group cut by a k-slice or a K range is closed piecewise, the sums being linear).
// ---------------------------------------------------------------------------------------
struct CodesArgs {
    const uint4 *codes;
    const float *scales;
    const uint32_t *zeros;
    const uint16_t *Xop;       // [rows_padded][steps * S] bf16, operand order (prepare_x)
    const uint16_t *Corr;      // [xhat entries][rows_padded][16] bf16 (prepare_x)
    float *out;                // Y, or partial results [split][M][N]
    int M, N, tiles, steps, ngroups, zwords;
    int rows_padded;           // M rounded up to whole row blocks of the launch
    int steps_padded;          // steps rounded up to a multiple of 4: what prepare_x has written (zeros past K)
    int steps_per_group;       // CPG == 0: steps one group spans
    int steps_per_split;       // a multiple of KW
};

struct PrepArgs {
    const float *X;            // [M][K] fp32
    uint16_t *Xop, *Corr;
    int M, K, rows_padded, kpad;   // kpad = padded steps * S: every element of it is written
    int groupk;                // k one xhat covers: the group, or a step for groups of whole steps
};

// One item = OCT consecutive k of one row (a cell at 2 bits, a word of a cell otherwise).
// Consecutive threads take consecutive items of a row, so the items of one xhat sit in
// neighbouring lanes.
template <int BITS>
__global__ __launch_bounds__(256) void prepare_x(const PrepArgs A)
{
    using F = Fmt<BITS>;
    constexpr int S = codes_per_step<BITS>();
    constexpr int OPS = mma_ops<BITS>();
    constexpr int OCT = BITS == 2 ? 16 : 8;
    const int m = blockIdx.y;
    const int item = blockIdx.x * 256 + threadIdx.x;
    const int items = A.kpad / OCT;
    const bool live = item < items;                         // the last block of a row may overhang
    const int k0 = (live ? item : items - 1) * OCT;
    const bool real = live && m < A.M && k0 < A.K;
    float val[OCT];
    if (real) {
        const float4 *src = (const float4 *)(A.X + (size_t)m * A.K + k0);
#pragma unroll
        for (int q = 0; q < OCT / 4; ++q) {
            const float4 v = src[q];
            val[4 * q + 0] = v.x; val[4 * q + 1] = v.y; val[4 * q + 2] = v.z; val[4 * q + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < OCT; ++e) val[e] = 0.0f;
    }
    const int in_step = k0 % S, step = k0 / S;
    const int cell = in_step / F::CELL;
    const int op0 = BITS == 3 ? (in_step % F::CELL) / 8 : 0;          // 3 bits: an item is one word of a cell
    uint16_t h[OCT];                    // bf16 patterns in operand order: [operand][element]
    float sum0 = 0.0f, sum1 = 0.0f;
#pragma unroll
    for (int e = 0; e < OCT; e += 2) {
        // (3 bits) codes 4 ... 7 of a word are taken three bits up and enter as 128 + 8 q
        const bool up = BITS == 3 && (e & 7) >= 4;
        mma_floatx2 t2 = {val[e] * (up ? 0.125f : 1.0f), val[e + 1] * (up ? 0.125f : 1.0f)};
        const mma_bf16x2 hb = __builtin_convertvector(t2, mma_bf16x2);            // round to nearest even
        const uint32_t bits = *(const uint32_t *)&hb;
        h[mma_slot<BITS>(e)] = (uint16_t)bits;
        h[mma_slot<BITS>(e + 1)] = (uint16_t)(bits >> 16);
        const float back = __uint_as_float(bits << 16) + __uint_as_float(bits & 0xffff0000u);
        if (up) sum1 += back * 8.0f; else sum0 += back;
    }
    if (live) {
        uint16_t *row = A.Xop + (size_t)m * A.kpad + (size_t)step * S;
#pragma unroll
        for (int o = 0; o < OCT / 8; ++o) {
            uint4 piece;
            piece.x = h[8 * o + 0] | ((uint32_t)h[8 * o + 1] << 16);
            piece.y = h[8 * o + 2] | ((uint32_t)h[8 * o + 3] << 16);
            piece.z = h[8 * o + 4] | ((uint32_t)h[8 * o + 5] << 16);
            piece.w = h[8 * o + 6] | ((uint32_t)h[8 * o + 7] << 16);
            *(uint4 *)(row + ((cell >> 1) * OPS + op0 + o) * 16 + (cell & 1) * 8) = piece;
        }
    }
    // xhat: the groupk / OCT neighbouring lanes hold its items (every lane takes part)
    const int wr = A.groupk / OCT;
    for (int off = 1; off < wr; off *= 2) {
        sum0 += __shfl_xor(sum0, off, 64);
        sum1 += __shfl_xor(sum1, off, 64);
    }
    if (live && item % wr == 0) {
        uint32_t part[2][3];            // three bf16 parts that add up to the sum exactly
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            float rest = c == 0 ? sum0 : sum1;
#pragma unroll
            for (int p3 = 0; p3 < 3; ++p3) {
                mma_floatx2 t2 = {rest, 0.0f};
                const mma_bf16x2 hb = __builtin_convertvector(t2, mma_bf16x2);
                part[c][p3] = *(const uint32_t *)&hb & 0xffffu;
                rest -= __uint_as_float(part[c][p3] << 16);
            }
        }
        uint16_t *ce = A.Corr + ((size_t)(k0 / A.groupk) * A.rows_padded + m) * 16;
        *(uint4 *)ce = make_uint4(part[0][0] | (part[0][1] << 16), part[0][2], 0u, 0u);
        *(uint4 *)(ce + 8) = make_uint4(part[1][0] | (part[1][1] << 16), part[1][2], 0u, 0u);
    }
}

template <int BITS, int CPG, int MB, int KW>
__global__ __launch_bounds__(512) void gemm_codes(const CodesArgs A)
{
    using F = Fmt<BITS>;
    constexpr int THREADS = 512;
    constexpr int TN = 8 / KW;
    constexpr int L = loads_per_step<BITS>();
    constexpr int S = codes_per_step<BITS>();
    constexpr int CELLS = cells_per_step<BITS>();
    constexpr int GPS = CPG > 0 ? CELLS / CPG : 1;       // xhat entries per step (CPG == 0: one, the step's)
    constexpr int OPS = mma_ops<BITS>();                  // B operands per cell
    constexpr int ROWS = 32 * MB;
    constexpr int CK = KW * S;                            // k per workgroup iteration
    constexpr int PITCH = CK + 8;                         // bf16 per LDS row: conflict-free 128-bit reads
    constexpr int CG = KW * GPS;                          // xhat entries per iteration
    constexpr int XP = ROWS * CK / 8 / THREADS;           // 16-byte pieces of activations per thread and iteration
    constexpr int CP = (ROWS * CG * 2 + THREADS - 1) / THREADS;   // ... of xhat operands
    constexpr int ZPER = 32 / F::ZBITS;
    constexpr int ACC = MB * 2 * 16;
    static_assert(CPG == 0 || (CPG % 2 == 0 && CELLS % CPG == 0), "a group holds whole pairs of cells");
    static_assert(ROWS * CK / 8 % THREADS == 0, "copy layout");
    constexpr int XBYTES = 2 * ROWS * PITCH * 2;
    extern __shared__ __attribute__((aligned(16))) char smem[];       // max(activations + xhat operands, reduction)
    lds_u16 *Xs = (lds_u16 *)smem;                                    // [2][ROWS][PITCH]
    lds_u16 *Cs = (lds_u16 *)(smem + XBYTES);                         // [2][CG][ROWS][16]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tn = wave % TN, kw = wave / TN;
    const int tile = blockIdx.x * TN + tn;
    const bool have_tile = tile < A.tiles;
    const int m0 = blockIdx.z * ROWS;
    const int st0 = blockIdx.y * A.steps_per_split;
    int st1 = st0 + A.steps_per_split;
    if (st1 > A.steps) st1 = A.steps;
    const int iters = (st1 - st0 + KW - 1) / KW;
    const int kpad = A.steps_padded * S;

    const int tclamp = have_tile ? tile : A.tiles - 1;
    const uint4 *codes = A.codes + (size_t)tclamp * A.steps * L * QG_WAVE + lane;
    const float *sc = A.scales + (size_t)tclamp * A.ngroups * QG_WAVE + lane;
    const uint32_t *zr = A.zeros + (size_t)tclamp * A.zwords * QG_WAVE + lane;

    struct StepRegs {
        uint4 v[L];
        float s[GPS];
        uint32_t zw;
    };
    // group of xhat entry `gs` of a step, clamped to the groups that exist (K is padded to whole
    // steps with zero codes; what the padding adds up to is zero whatever scale it meets)
    auto group_of = [&](int step, int gs) {
        int g = CPG > 0 ? step * GPS + gs : step / A.steps_per_group;
        return g < A.ngroups ? g : A.ngroups - 1;
    };
    auto fetch = [&](int step, StepRegs &r) {
        step = step < st1 ? step : st1 - 1;            // past the range: loaded again, not used
#pragma unroll
        for (int i = 0; i < L; ++i) r.v[i] = codes[((size_t)step * L + i) * QG_WAVE];
#pragma unroll
        for (int g = 0; g < GPS; ++g) r.s[g] = sc[(size_t)group_of(step, g) * QG_WAVE];
        r.zw = zr[(size_t)(group_of(step, 0) / ZPER) * QG_WAVE];       // a step's groups share one zero word
    };

    // ---- activations and xhat operands of one iteration: plain 16-byte copies into LDS ----
    // (a chunk that begins past the last step is read from the last chunk again and never used)
    typedef uint32_t copy128 __attribute__((ext_vector_type(4)));       // a plain vector: stays in registers
    typedef copy128 __attribute__((may_alias)) copy128_lds;
    copy128 xq[XP], cq[CP];
    auto load_x = [&](int first_step) {
        const int fs = first_step + KW <= A.steps_padded ? first_step : A.steps_padded - KW;
#pragma unroll
        for (int j = 0; j < XP; ++j) {
            const int p = j * THREADS + threadIdx.x;          // piece: row p / (CK / 8), 8 k at p % (CK / 8)
            const int r = p / (CK / 8), c = p % (CK / 8);
            xq[j] = *(const copy128 *)(A.Xop + (size_t)(m0 + r) * kpad + (size_t)fs * S + c * 8);
        }
#pragma unroll
        for (int j = 0; j < CP; ++j) {
            int p = j * THREADS + threadIdx.x;                // piece: entry p / (ROWS * 2), 16 bytes of row (p / 2) % ROWS
            p = p < ROWS * CG * 2 ? p : ROWS * CG * 2 - 1;
            const int e = p / (ROWS * 2), rr = p % (ROWS * 2);
            cq[j] = *(const copy128 *)(A.Corr + ((size_t)(fs * GPS + e) * A.rows_padded + m0) * 16 + rr * 8);
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int j = 0; j < XP; ++j) {
            const int p = j * THREADS + threadIdx.x;
            const int r = p / (CK / 8), c = p % (CK / 8);
            *(copy128_lds *)(Xs + ((size_t)buf * ROWS + r) * PITCH + c * 8) = xq[j];
        }
#pragma unroll
        for (int j = 0; j < CP; ++j) {
            const int p = j * THREADS + threadIdx.x;
            if (p < ROWS * CG * 2) *(copy128_lds *)(Cs + (size_t)buf * CG * ROWS * 16 + (size_t)p * 8) = cq[j];
        }
    };

    // ---- accumulators ----
    mma_floatx16 accP[MB], accQ[MB];          // T of the running group: outputs 0-31 (P) and 32-63 (Q) of the tile
    float yP[MB][16], yQ[MB][16];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) { accP[mb][i] = 0.0f; accQ[mb][i] = 0.0f; yP[mb][i] = 0.0f; yQ[mb][i] = 0.0f; }
    const int half = lane >> 5, row = lane & 31;
    const MmaConst mc = mma_constants<BITS>();
    // Y += s * T, with the scales of outputs lane % 32 (P) and 32 + lane % 32 (Q)
    auto fold = [&](float sP, float sQ) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                yP[mb][i] = fmaf(sP, accP[mb][i], yP[mb][i]);
                yQ[mb][i] = fmaf(sQ, accQ[mb][i], yQ[mb][i]);
            }
    };
    // the B operand of the zero-point term: -(128 + z) against the parts of xhat in lanes 0-31,
    // -(16 + z) against the parts of the other xhat in lanes 32-63 (3 bits only; else zeros there)
    auto corr_operand = [&](uint32_t zq) {
        const float c = half == 0 ? -(float)(zq + 128u) : BITS == 3 ? -(float)(zq + 16u) : 0.0f;
        const uint32_t cb = __float_as_uint(c) >> 16;                  // small integers are exact in bf16
        MmaOperand b;
        b.r[0] = cb | (cb << 16);
        b.r[1] = cb;
        b.r[2] = 0u;
        b.r[3] = 0u;
        return b;
    };
    float heldP = 0.0f, heldQ = 0.0f;         // CPG == 0: scale of the group the accumulators belong to
    int held_g = -1;
    bool fresh = true;                        // CPG == 0: no step has been computed yet

    auto compute = [&](const StepRegs &r, int step, int buf) {
        const lds_u16 *xs = Xs + ((size_t)buf * ROWS + row) * PITCH + kw * S + half * 8;
        const lds_u16 *cs = Cs + ((size_t)buf * CG + kw * GPS) * ROWS * 16 + row * 16 + half * 8;
        const auto zsw = __builtin_amdgcn_permlane32_swap(r.zw, r.zw, false, false);
        const uint32_t zwP = zsw[0], zwQ = zsw[1];
        const mma_floatx16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        if constexpr (CPG == 0) {
            const int g = group_of(step, 0);
            if (g != held_g) {                       // uniform: the running group ended before this step
                if (!fresh) fold(heldP, heldQ);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    accP[mb] = zero16;
                    accQ[mb] = zero16;
                }
                const auto ssw = __builtin_amdgcn_permlane32_swap(__float_as_uint(r.s[0]), __float_as_uint(r.s[0]), false, false);
                heldP = __uint_as_float(ssw[0]);
                heldQ = __uint_as_float(ssw[1]);
                held_g = g;
            }
        }
        // what closes a group after pair cp: the zero-point term on the matrix cores, then Y += s T
        auto close_group = [&](int cp) {
            const bool group_ends = CPG > 0 ? (2 * cp + 2) % CPG == 0 : cp == CELLS / 2 - 1;
            if (group_ends) {
                const int gs = CPG > 0 ? (2 * cp + 2) / CPG - 1 : 0;
                const int gabs = group_of(step, gs);
                const uint32_t zP = (zwP >> (F::ZBITS * (gabs % ZPER))) & ((1u << F::ZBITS) - 1u);
                const uint32_t zQ = (zwQ >> (F::ZBITS * (gabs % ZPER))) & ((1u << F::ZBITS) - 1u);
                const MmaOperand cP = corr_operand(zP), cQ = corr_operand(zQ);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    MmaOperand a;
                    a.q = *(const lds_u128 *)(cs + ((size_t)gs * ROWS + mb * 32) * 16);
                    accP[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, cP.v, accP[mb], 0, 0, 0);
                    accQ[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, cQ.v, accQ[mb], 0, 0, 0);
                }
                if constexpr (CPG > 0) {
                    const auto ssw = __builtin_amdgcn_permlane32_swap(__float_as_uint(r.s[gs]), __float_as_uint(r.s[gs]), false, false);
                    fold(__uint_as_float(ssw[0]), __uint_as_float(ssw[1]));
                }
            }
        };
        if constexpr (BITS == 4) {
            // 4 bits: a software pipeline.  The matrix instructions of pair cp alternate with the
            // pieces of the unpacking of pair cp + 1 (and with its lane exchange and LDS reads), every
            // slot fenced, so that a wavefront keeps the matrix core and the vector ALU busy at the
            // same time instead of in turns (two wavefronts of a SIMD that leave a barrier together
            // would otherwise take those turns in step).
            constexpr int NP = CELLS / 2;
            MmaOperand bP, bQ, nP, nQ, aC[MB], aN[MB];
            uint32_t wP = 0, wQ = 0;
            auto swap_words = [&](int cp) {
                const int c0 = 2 * cp, u = c0 >> 2, j = c0 & 3;
                const auto sw = __builtin_amdgcn_permlane32_swap(word_of(r.v[u], j), word_of(r.v[u], j + 1), false, false);
                wP = sw[0];           // outputs 0-31: cell 2 cp in lanes 0-31, cell 2 cp + 1 in lanes 32-63
                wQ = sw[1];           // outputs 32-63
            };
            auto piece = [&](int i) {       // quarter i of the unpacking of (wP, wQ) into (nP, nQ)
                const uint32_t w = i < 2 ? wP : wQ;
                MmaOperand &b = i < 2 ? nP : nQ;
                const int j0 = 2 * (i & 1);
                b.r[j0] = and_or(w >> (4 * j0), mc.mask, mc.magic);
                b.r[j0 + 1] = and_or(w >> (4 * (j0 + 1)), mc.mask, mc.magic);
                asm volatile("" : "+v"(b.r[j0]), "+v"(b.r[j0 + 1]));      // keeps the piece in its slot
            };
            auto read_a = [&](int cp, MmaOperand *a) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) a[mb].q = *(const lds_u128 *)(xs + (size_t)mb * 32 * PITCH + cp * 16);
            };
            swap_words(0);
#pragma unroll
            for (int i = 0; i < 4; ++i) piece(i);
            bP = nP;
            bQ = nQ;
            read_a(0, aC);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int cp = 0; cp < NP; ++cp) {
                const bool more = cp + 1 < NP;
                const bool starts = CPG > 0 && (2 * cp) % CPG == 0;       // a group starts from zero
#pragma unroll
                for (int k = 0; k < 2 * MB; ++k) {
                    const int mb = k >> 1;
                    if ((k & 1) == 0)
                        accP[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aC[mb].v, bP.v, starts ? zero16 : accP[mb], 0, 0, 0);
                    else
                        accQ[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aC[mb].v, bQ.v, starts ? zero16 : accQ[mb], 0, 0, 0);
                    if (more) {
                        if (k == 0) {
                            swap_words(cp + 1);
                            read_a(cp + 1, aN);
                        }
                        if constexpr (MB == 1) {
                            piece(2 * k);
                            piece(2 * k + 1);
                        } else {
                            piece(k);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                close_group(cp);
                if (more) {
                    bP = nP;
                    bQ = nQ;
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) aC[mb] = aN[mb];
                }
            }
        } else {
#pragma unroll
        for (int cp = 0; cp < CELLS / 2; ++cp) {
            uint32_t wp[F::PLANES], wq[F::PLANES];
            const int c0 = 2 * cp, u = c0 >> 2, j = c0 & 3;
#pragma unroll
            for (int pl = 0; pl < F::PLANES; ++pl) {
                const auto sw = __builtin_amdgcn_permlane32_swap(word_of(r.v[u * F::PLANES + pl], j),
                                                                 word_of(r.v[u * F::PLANES + pl], j + 1), false, false);
                wp[pl] = sw[0];       // outputs 0-31: cell 2 cp in lanes 0-31, cell 2 cp + 1 in lanes 32-63
                wq[pl] = sw[1];       // outputs 32-63
            }
            MmaOperand bp[OPS], bq[OPS];
            mma_unpack<BITS>(wp, mc, bp);
            mma_unpack<BITS>(wq, mc, bq);
            // the first matrix instruction of a group starts from zero instead of the old sums
            const bool starts = CPG > 0 ? (2 * cp) % CPG == 0 : false;
#pragma unroll
            for (int op = 0; op < OPS; ++op) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    MmaOperand a;
                    a.q = *(const lds_u128 *)(xs + (size_t)mb * 32 * PITCH + (cp * OPS + op) * 16);
                    if (CPG > 0 && starts && op == 0) {
                        accP[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, bp[op].v, zero16, 0, 0, 0);
                        accQ[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, bq[op].v, zero16, 0, 0, 0);
                    } else {
                        accP[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, bp[op].v, accP[mb], 0, 0, 0);
                        accQ[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, bq[op].v, accQ[mb], 0, 0, 0);
                    }
                }
            }
            close_group(cp);
        }
        }
        fresh = false;
    };

    // Every iteration is straight-line code: request the activations of iteration it + 1 and then
    // its weights (clamped past the end), compute iteration it from registers and LDS, then move
    // the new activations into place.  The activation copies are requested BEFORE the weights:
    // loads return in order, and the copies are waited for at the end of the same iteration,
    // while the weights are not needed before the next one.  Two register sets take turns, so
    // that no iteration moves (and so waits for) the weights it has just requested.
    StepRegs ra, rb;
    if (iters > 0) {
        load_x(st0);
        fetch(st0 + kw, ra);
        store_x(0);
    }
    __syncthreads();
    int buf = 0;
    auto iteration = [&](int it, const StepRegs &use, StepRegs &request) {
        const int step = st0 + it * KW + kw;
        load_x(st0 + (it + 1) * KW);
        fetch(step + KW, request);
        __builtin_amdgcn_sched_barrier(0);
        if (step < st1) compute(use, step, buf);
        __builtin_amdgcn_sched_barrier(0);
        store_x(buf ^ 1);
        __syncthreads();          // next chunk written, this chunk's readers done
        buf ^= 1;
    };
    for (int it = 0; it < iters; it += 2) {
        iteration(it, ra, rb);
        if (it + 1 >= iters) break;
        iteration(it + 1, rb, ra);
    }
    if constexpr (CPG == 0) {
        if (!fresh) fold(heldP, heldQ);
    }

    if constexpr (KW > 1) {
        // k-slices 1 .. KW-1 hand their results to slice 0 of the same tile, which adds them in
        // slice order; the activation buffers are reused (every reader is past the last barrier)
        float *red = (float *)smem;
        if (kw > 0) {
            float *dst = red + ((size_t)((kw - 1) * TN + tn) * ACC) * 64 + lane;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    dst[((mb * 2 + 0) * 16 + i) * 64] = yP[mb][i];
                    dst[((mb * 2 + 1) * 16 + i) * 64] = yQ[mb][i];
                }
        }
        __syncthreads();
        if (kw > 0) return;
#pragma unroll
        for (int k = 1; k < KW; ++k) {
            const float *src = red + ((size_t)((k - 1) * TN + tn) * ACC) * 64 + lane;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    yP[mb][i] += src[((mb * 2 + 0) * 16 + i) * 64];
                    yQ[mb][i] += src[((mb * 2 + 1) * 16 + i) * 64];
                }
        }
    }

    if (!have_tile) return;
    // Register i of an accumulator is row 8 (i / 4) + 4 half + i % 4 of its block: bands of eight
    // rows, four registers each.  A band that lies inside M in a tile that lies inside N is
    // stored without a test per lane (both conditions are the same for the whole wavefront).
    const int nP = tile * QG_WAVE + row, nQ = nP + 32;
    float *out = A.out + (size_t)blockIdx.y * A.M * A.N + (size_t)(m0 + 4 * half) * A.N + nP;
    const int rows_left = A.M - m0;
    const bool whole_tile = (tile + 1) * QG_WAVE <= A.N;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int band = 0; band < 4; ++band) {
            const int r0 = mb * 32 + 8 * band;
            if (r0 >= rows_left) break;
            if (whole_tile && r0 + 8 <= rows_left) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float *o = out + (size_t)(r0 + j) * A.N;
                    o[0] = yP[mb][4 * band + j];
                    o[32] = yQ[mb][4 * band + j];
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool in_m = r0 + 4 * half + j < rows_left;
                    float *o = out + (size_t)(r0 + j) * A.N;
                    if (in_m && nP < A.N) o[0] = yP[mb][4 * band + j];
                    if (in_m && nQ < A.N) o[32] = yQ[mb][4 * band + j];
                }
            }
        }
}

template <int BITS, int CPG, int MB, int KW>
constexpr size_t gemm_codes_lds()
{
    constexpr int S = codes_per_step<BITS>();
    constexpr int GPS = CPG > 0 ? cells_per_step<BITS>() / CPG : 1;
    constexpr size_t x = 2 * (32 * MB) * (KW * S + 8) * 2, c = 2 * (32 * MB) * (KW * GPS) * 16 * 2;
    constexpr size_t r = (size_t)(KW - 1) * (8 / KW) * (MB * 2 * 16) * 64 * 4;
    return x + c > r ? x + c : r;
}

// Y = sum of the K-split partial results, in split order.  All (up to 8) loads of a thread
// are issued before the first addition; a loop over a run-time split count would wait for
// each load in turn.
__global__ void add_splits(const float *__restrict__ partial, int splits, size_t count,
                           float *__restrict__ Y)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    float v[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) v[s] = s < splits ? partial[(size_t)s * count + i] : 0.0f;
    float t = v[0];
#pragma unroll
    for (int s = 1; s < 8; ++s) t += v[s];       // the missing ones add +0.0
    Y[i] = t;
}

bool fast_path(const QgLayout &L)
{
    return L.bits == 4 && L.group % 32 == 0 && L.K % KC == 0 && L.K <= (1 << 20) &&
           (L.group <= KC ? KC % L.group == 0 : L.group % KC == 0);
}

constexpr int MAX_SPLITS = 8;
int g_tune_splits = 0;      // measurement knobs: 0 = built-in choice
int g_tune_shape = 0;       // 1 + index into SHAPES, NSHAPES + 1: the raw-code kernel, -1: gemm_rows16

// Choices recorded per problem (qg_gemm_autotune): used where both knobs are 0.
struct GemmTuneEntry {
    int64_t N, K;
    int bits, group, M, splits, shape;
};
constexpr int GEMM_TUNE_ENTRIES = 64;
GemmTuneEntry g_gemm_table[GEMM_TUNE_ENTRIES];
int g_gemm_count = 0, g_gemm_next = 0;
std::mutex g_gemm_mutex;

bool gemm_tuning_for(int64_t N, int64_t K, int bits, int group, int M, int *splits, int *shape)
{
    std::lock_guard<std::mutex> lock(g_gemm_mutex);
    for (int i = 0; i < g_gemm_count; ++i) {
        const GemmTuneEntry &e = g_gemm_table[i];
        if (e.N == N && e.K == K && e.bits == bits && e.group == group && e.M == M) {
            *splits = e.splits;
            *shape = e.shape;
            return true;
        }
    }
    return false;
}

void gemm_record_tuning(int64_t N, int64_t K, int bits, int group, int M, int splits, int shape)
{
    std::lock_guard<std::mutex> lock(g_gemm_mutex);
    int at = -1;
    for (int i = 0; i < g_gemm_count; ++i) {
        const GemmTuneEntry &e = g_gemm_table[i];
        if (e.N == N && e.K == K && e.bits == bits && e.group == group && e.M == M) at = i;
    }
    if (at < 0) {
        if (g_gemm_count < GEMM_TUNE_ENTRIES) at = g_gemm_count++;
        else { at = g_gemm_next; g_gemm_next = (g_gemm_next + 1) % GEMM_TUNE_ENTRIES; }
    }
    g_gemm_table[at] = {N, K, bits, group, M, splits, shape};
}

int gcd(int a, int b) { return b == 0 ? a : gcd(b, a % b); }

// What a launch would run, for the search that prices candidates before it times them
// (qg_gemm_autotune): filled instead of launching when a launcher is handed one.
struct KernelInfo {
    const void *kernel;
    int threads;
    size_t lds_dynamic;
};

template <int MB, int TN, int KW>
void launch(const GemmArgs &A, dim3 grid, hipStream_t st, KernelInfo *query)
{
    if (query) {
        *query = {A.group_shift == 7 ? (const void *)gemm_small_b4<MB, TN, KW, true>
                                     : (const void *)gemm_small_b4<MB, TN, KW, false>, TN * KW * 64, 0};
        return;
    }
    if (A.group_shift == 7)
        hipLaunchKernelGGL((gemm_small_b4<MB, TN, KW, true>), grid, dim3(TN * KW * 64), 0, st, A);
    else
        hipLaunchKernelGGL((gemm_small_b4<MB, TN, KW, false>), grid, dim3(TN * KW * 64), 0, st, A);
}

template <int MB, int TN>
void launch_wide(const GemmArgs &A, dim3 grid, hipStream_t st, KernelInfo *query)
{
    if (query) {
        *query = {A.group_shift == 7 ? (const void *)gemm_wide_b4<MB, TN, true> : (const void *)gemm_wide_b4<MB, TN, false>,
                  TN * 64, 0};
        return;
    }
    if (A.group_shift == 7) hipLaunchKernelGGL((gemm_wide_b4<MB, TN, true>), grid, dim3(TN * 64), 0, st, A);
    else hipLaunchKernelGGL((gemm_wide_b4<MB, TN, false>), grid, dim3(TN * 64), 0, st, A);
}

// Workgroup shapes: {rows / 32, tiles, k-slices, gemm_wide_b4 (all rows in one wavefront)}
struct Shape {
    int mb, tn, kw;
    bool wide;
};
constexpr Shape SHAPES[] = {
    {1, 1, 4, false}, {1, 2, 4, false}, {1, 4, 2, false},                       // up to 32 rows
    {2, 2, 2, false}, {2, 4, 1, false}, {2, 4, 2, false}, {2, 8, 1, false},     // blocks of 64 rows
    {2, 4, 1, true},  {2, 2, 1, true},                                          // up to 64 rows
    {4, 4, 1, true},  {4, 2, 1, true},                                          // up to 128 rows
    {2, 8, 1, true},                                                            // up to 64 rows
};
constexpr int NSHAPES = sizeof(SHAPES) / sizeof(SHAPES[0]);

void launch_shape(int i, const GemmArgs &A, dim3 grid, hipStream_t st, KernelInfo *query = nullptr)
{
    switch (i) {
    case 0: launch<1, 1, 4>(A, grid, st, query); break;
    case 1: launch<1, 2, 4>(A, grid, st, query); break;
    case 2: launch<1, 4, 2>(A, grid, st, query); break;
    case 3: launch<2, 2, 2>(A, grid, st, query); break;
    case 4: launch<2, 4, 1>(A, grid, st, query); break;
    case 5: launch<2, 4, 2>(A, grid, st, query); break;
    case 6: launch<2, 8, 1>(A, grid, st, query); break;
    case 7: launch_wide<2, 4>(A, grid, st, query); break;
    case 8: launch_wide<2, 2>(A, grid, st, query); break;
    case 9: launch_wide<4, 4>(A, grid, st, query); break;
    case 10: launch_wide<4, 2>(A, grid, st, query); break;
    default: launch_wide<2, 8>(A, grid, st, query); break;
    }
}


// ---- gemm_codes: which layouts it takes, and its launch ----
int codes_cpg(const QgLayout &L)       // cells per group, 0 for groups of whole steps, -1: not taken
{
    const int S = L.unit * L.step_units, cells = 4 * L.step_units;
    if (L.K % 16 != 0 || L.K > (1 << 22)) return -1;
    if (L.group % S == 0 && L.group > S) return 0;
    const int cpg = L.group / L.cell;        // (a group of exactly one step closes at a compile-time position)
    if (L.group > S || cpg < 2 || cpg % 2 != 0 || cells % cpg != 0) return -1;
    return cpg;
}

// Workspace of the raw-code path: converted activations, xhat operands, K-split partial results.
struct CodesSpace {
    size_t xop_off, corr_off, partial_off, total;
    int rows_padded, steps_padded, groupk;
};
CodesSpace codes_space(const QgLayout &L, int M)
{
    CodesSpace W;
    const int S = L.unit * L.step_units;
    const int rows_per_block = M <= 32 ? 32 : 64;
    W.rows_padded = (M + rows_per_block - 1) / rows_per_block * rows_per_block;
    W.steps_padded = (int)((L.steps + 3) / 4 * 4);
    W.groupk = L.group % S == 0 ? S : L.group;
    const size_t kpad = (size_t)W.steps_padded * S;
    W.xop_off = 0;
    W.corr_off = qg_round_up(W.xop_off + (size_t)W.rows_padded * kpad * 2, QG_SECTION_ALIGN);
    W.partial_off = qg_round_up(W.corr_off + kpad / W.groupk * W.rows_padded * 32, QG_SECTION_ALIGN);
    W.total = qg_round_up(W.partial_off + (size_t)MAX_SPLITS * M * L.N * sizeof(float), QG_SECTION_ALIGN);
    return W;
}

template <int BITS, int CPG, int MB>
int launch_codes(const CodesArgs &A, dim3 grid, hipStream_t st, KernelInfo *query)
{
    constexpr int KW = BITS == 4 ? (MB == 1 ? 4 : 2) : (MB == 1 ? 2 : 1);
    constexpr size_t lds = gemm_codes_lds<BITS, CPG, MB, KW>();
    if (query) {
        *query = {(const void *)gemm_codes<BITS, CPG, MB, KW>, 512, lds};
        return QG_OK;
    }
    static bool prepared = false;              // dynamic LDS above 64 KB has to be asked for once
    if (!prepared) {
        if (hipFuncSetAttribute((const void *)gemm_codes<BITS, CPG, MB, KW>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            return QG_ERR_DEVICE;
        }
        prepared = true;
    }
    hipLaunchKernelGGL((gemm_codes<BITS, CPG, MB, KW>), grid, dim3(512), lds, st, A);
    return QG_OK;
}

template <int BITS, int MB>
int launch_codes_cpg(int cpg, const CodesArgs &A, dim3 grid, hipStream_t st, KernelInfo *query)
{
    switch (cpg) {
    case 0: return launch_codes<BITS, 0, MB>(A, grid, st, query);
    case 2: return launch_codes<BITS, 2, MB>(A, grid, st, query);
    case 4: return launch_codes<BITS, 4, MB>(A, grid, st, query);
    case 8: return launch_codes<BITS, 8, MB>(A, grid, st, query);
    case 16:
        if constexpr (BITS != 3) return launch_codes<BITS, 16, MB>(A, grid, st, query);
        return QG_ERR_UNSUPPORTED;
    default: return QG_ERR_UNSUPPORTED;
    }
}

constexpr int codes_kw(int bits, int mb) { return bits == 4 ? (mb == 1 ? 4 : 2) : (mb == 1 ? 2 : 1); }
}  // namespace

size_t qg_gemm_workspace_bytes(const QgLayout &L, int M)
{
    // partial results of the K split, or the GEMV workspaces of the rows of one grouped launch
    const size_t partial = (size_t)MAX_SPLITS * M * L.N * sizeof(float);
    const size_t gemv = qg_round_up((size_t)L.tiles * (QG_MAX_CHUNKS + 1) * QG_WAVE * sizeof(uint32_t),
                                    QG_SECTION_ALIGN);                                    // as qg_gemv asks
    const int rows = M < QG_MAX_GROUPED ? M : QG_MAX_GROUPED;
    size_t need = fast_path(L) && partial > gemv * rows ? partial : gemv * rows;
    if (M > 1 && codes_cpg(L) >= 0 && codes_space(L, M).total > need) need = codes_space(L, M).total;
    return qg_round_up(need, QG_SECTION_ALIGN);
}

extern "C" int qg_set_gemm_tuning(int splits, int shape)
{
    if (splits < 0 || splits > MAX_SPLITS || shape < -1 || shape > NSHAPES + 1) return QG_ERR_SHAPE;
    g_tune_splits = splits;
    g_tune_shape = shape;
    return QG_OK;
}

namespace {
// What one candidate of the launch-shape search costs, by the machine's budget (filled by a
// planning pass of gemm_small, which then enqueues nothing).
struct GemmPrice {
    int family;                // 0 raw codes, 1 gemm_rows16, 2 one GEMV per row, 3 dequantizing kernels
    int shape, splits;         // what the planner settled on (shape: index into SHAPES for family 3)
    long workgroups;           // of the main launch
    long iterations;           // barrier-to-barrier iterations one workgroup runs one after the other
    int launches;              // kernels the call enqueues
    KernelInfo kernel;
};

// Checks, plans and (price == NULL) enqueues one product; knob_*: as qg_set_gemm_tuning.
int gemm_small(const void *packed, int64_t N, int64_t K, int bits, int group, const float *X, int M,
               float *Y, void *workspace, size_t workspace_bytes, void *stream, int knob_splits,
               int knob_shape, GemmPrice *price)
{
    QgLayout L;
    const int rc = qg_make_layout(N, K, bits, group, &L);
    if (rc != QG_OK) return rc;
    if (M <= 0 || M > 128) return QG_ERR_SHAPE;
    if (!packed || !X || !Y) return QG_ERR_NULL;
    if (!qg_aligned16(packed) || ((uintptr_t)X & 63u) || !qg_aligned16(Y)) return QG_ERR_ALIGN;
    if (!workspace || workspace_bytes < qg_gemm_workspace_bytes(L, M)) return QG_ERR_WORKSPACE;
    if (!qg_aligned16(workspace)) return QG_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;

    // The raw-code kernel: every layout it takes that the 4-bit kernels below do not (2 and 3
    // bits, 4-bit groups of 16), and whatever shape 13 sends it.  (Measured on the 7B shapes at 4
    // bits, group 128: within 0-20 % of the dequantizing kernels, behind mostly by the launch of
    // prepare_x; at 2 and 3 bits 2-15 times ahead of one GEMV per row.)
    const int cpg = codes_cpg(L);
    // (... and, measured, 3-6 % ahead of them beyond 64 rows on the larger 7B shapes)
    const bool large = M > 64 && L.tiles * L.steps >= 4096;
    if (cpg >= 0 && M > 1 && (knob_shape == NSHAPES + 1 || (knob_shape == 0 && (!fast_path(L) || large)))) {
        const int mb = M <= 32 ? 1 : 2;
        const int kw = codes_kw(bits, mb), tn = 8 / kw;
        const int rows_per_block = 32 * mb;
        const int zblocks = (M + rows_per_block - 1) / rows_per_block;
        const int blocks_x = (int)((L.tiles + tn - 1) / tn);
        const int quanta = (int)((L.steps + kw - 1) / kw);
        const int cus = qg_compute_units();
        // as many K ranges as keep the launch within one workgroup per compute unit (a workgroup
        // takes half of a unit's registers or more, so one more would wait for a second round)
        int splits = knob_splits ? knob_splits : cus / (blocks_x * zblocks);
        if (splits < 1) splits = 1;
        if (splits > MAX_SPLITS) splits = MAX_SPLITS;
        if (splits > quanta) splits = quanta;
        const int sps = (quanta + splits - 1) / splits * kw;
        splits = (int)((L.steps + sps - 1) / sps);
        const CodesSpace W = codes_space(L, M);
        char *ws = (char *)workspace;
        PrepArgs P;
        P.X = X;
        P.Xop = (uint16_t *)(ws + W.xop_off);
        P.Corr = (uint16_t *)(ws + W.corr_off);
        P.M = M;
        P.K = (int)K;
        P.rows_padded = W.rows_padded;
        P.kpad = W.steps_padded * L.unit * L.step_units;
        P.groupk = W.groupk;
        CodesArgs A;
        const char *base = (const char *)packed;
        A.codes = (const uint4 *)(base + L.codes_off);
        A.scales = (const float *)(base + L.scales_off);
        A.zeros = (const uint32_t *)(base + L.zeros_off);
        A.Xop = P.Xop;
        A.Corr = P.Corr;
        A.out = splits > 1 ? (float *)(ws + W.partial_off) : Y;
        A.M = M;
        A.N = (int)N;
        A.tiles = (int)L.tiles;
        A.steps = (int)L.steps;
        A.ngroups = (int)L.ngroups;
        A.zwords = (int)L.zwords;
        A.rows_padded = W.rows_padded;
        A.steps_padded = W.steps_padded;
        A.steps_per_group = cpg == 0 ? group / (L.unit * L.step_units) : 1;
        A.steps_per_split = sps;
        const dim3 grid((unsigned)blocks_x, (unsigned)splits, (unsigned)zblocks);
        KernelInfo info = {nullptr, 0, 0};
        auto main_kernel = [&](KernelInfo *query) {
            if (bits == 4) return mb == 1 ? launch_codes_cpg<4, 1>(cpg, A, grid, st, query) : launch_codes_cpg<4, 2>(cpg, A, grid, st, query);
            if (bits == 2) return mb == 1 ? launch_codes_cpg<2, 1>(cpg, A, grid, st, query) : launch_codes_cpg<2, 2>(cpg, A, grid, st, query);
            return mb == 1 ? launch_codes_cpg<3, 1>(cpg, A, grid, st, query) : launch_codes_cpg<3, 2>(cpg, A, grid, st, query);
        };
        // (the instance is looked up before anything is enqueued: a layout without one is an error
        // that leaves nothing behind)
        const int have = main_kernel(&info);
        if (have != QG_OK) return have;
        if (price) {
            *price = {0, NSHAPES, splits, (long)blocks_x * splits * zblocks, sps / kw, splits > 1 ? 3 : 2, info};
            return QG_OK;
        }
        const dim3 pgrid((unsigned)((P.kpad / (bits == 2 ? 16 : 8) + 255) / 256), (unsigned)W.rows_padded);
        if (bits == 4) hipLaunchKernelGGL(prepare_x<4>, pgrid, dim3(256), 0, st, P);
        else if (bits == 2) hipLaunchKernelGGL(prepare_x<2>, pgrid, dim3(256), 0, st, P);
        else hipLaunchKernelGGL(prepare_x<3>, pgrid, dim3(256), 0, st, P);
        if (qg_launch_status() != QG_OK) return QG_ERR_DEVICE;
        const int r = main_kernel(nullptr);
        if (r != QG_OK) return r;
        if (qg_launch_status() != QG_OK) return QG_ERR_DEVICE;
        if (splits > 1) {
            const size_t count = (size_t)M * N;
            hipLaunchKernelGGL(add_splits, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st,
                               (const float *)(ws + W.partial_off), splits, count, Y);
        }
        return qg_launch_status();
    }

    // Up to 16 rows: the barrier-free kernel on the GEMV's launch structure, where it applies.
    // It has one workgroup per tile and no split of K over workgroups, so it needs enough tiles
    // to cover the chip (measured: ahead from about 128 tiles; shape -1 forces it).
    if (M <= 16 && (knob_shape == 0 ? L.tiles >= 128 : knob_shape < 0)) {
        const int r = qg_gemm_rows16(packed, N, K, bits, group, X, M, Y, workspace, stream, price != nullptr);
        if (r == QG_OK && price) *price = {1, -1, 1, (long)L.tiles, 0, 1, {nullptr, 0, 0}};
        if (r != QG_ERR_UNSUPPORTED) return r;
    }

    if (!fast_path(L)) {
        // the fp32 GEMV once per activation row, up to 16 rows per launch (rows of X stay
        // 64-byte aligned only if K % 16 == 0)
        if (K % 16 != 0 && M > 1) return QG_ERR_UNSUPPORTED;
        // two passes over the launches of 16 rows: the first only checks and plans, so that an
        // error leaves nothing enqueued
        for (int pass = 0; pass < (price ? 1 : 2); ++pass)
            for (int m0 = 0; m0 < M; m0 += QG_MAX_GROUPED) {
                qg_gemv_desc d[QG_MAX_GROUPED];
                const int rows = M - m0 < QG_MAX_GROUPED ? M - m0 : QG_MAX_GROUPED;
                for (int i = 0; i < rows; ++i) {
                    d[i].packed = packed;
                    d[i].N = N;
                    d[i].K = K;
                    d[i].bits = bits;
                    d[i].group = group;
                    d[i].x = X + (size_t)(m0 + i) * K;
                    d[i].y = Y + (size_t)(m0 + i) * N;
                }
                const int r = pass == 0 ? qg_gemv_grouped_check(d, rows, workspace, workspace_bytes)
                                        : qg_gemv_grouped(d, rows, workspace, workspace_bytes, stream);
                if (r != QG_OK) return r;
            }
        if (price) *price = {2, -1, 1, 0, 0, (M + QG_MAX_GROUPED - 1) / QG_MAX_GROUPED, {nullptr, 0, 0}};
        return QG_OK;
    }

    // Workgroup shape (measured choices).  Up to 32 rows: one block of rows, two tiles x four
    // k-slices.  Up to 64 rows: gemm_wide_b4 with four tiles per workgroup.  More: all rows
    // in one wavefront (gemm_wide_b4, every weight dequantized once) when the launch has
    // enough tiles for it, otherwise blocks of 64 rows on the grid's z axis, four tiles x two
    // k-slices (two blocks double the wavefronts of a launch at the price of dequantizing
    // twice, which pays as long as the launch cannot fill the chip).
    int shape = M <= 32 ? 1 : M <= 64 ? 7 : L.tiles >= 128 ? 9 : 5;
    if (knob_shape > 0 && knob_shape <= NSHAPES) {
        const Shape &sh = SHAPES[knob_shape - 1];
        if (sh.wide ? (M > 32 && M <= sh.mb * 32) : ((sh.mb == 1) == (M <= 32))) shape = knob_shape - 1;
    }
    const int rows_per_block = SHAPES[shape].mb * 32;
    const int zblocks = (M + rows_per_block - 1) / rows_per_block;
    const int kw = SHAPES[shape].kw, tn = SHAPES[shape].tn;
    const int blocks_x = (int)((L.tiles + tn - 1) / tn);
    const int steps_per_group = group > KC ? group / KC : 1;
    // a split is a whole number of workgroup iterations and of groups
    const int quantum = kw / gcd(kw, steps_per_group) * steps_per_group;
    const int quanta = (int)((L.steps + quantum - 1) / quantum);
    // about one workgroup per compute unit, each with at least one quantum of work
    const int cus = qg_compute_units();
    int splits = knob_splits ? knob_splits : (cus + blocks_x * zblocks - 1) / (blocks_x * zblocks);
    if (splits > MAX_SPLITS) splits = MAX_SPLITS;
    if (splits > quanta) splits = quanta;
    const int sps = (quanta + splits - 1) / splits * quantum;
    splits = (int)((L.steps + sps - 1) / sps);

    GemmArgs A;
    const char *base = (const char *)packed;
    A.codes = (const uint4 *)(base + L.codes_off);
    A.scales = (const float *)(base + L.scales_off);
    A.zeros = (const uint32_t *)(base + L.zeros_off);
    float *partial = (float *)workspace;
    A.X = X;
    A.out = splits > 1 ? partial : Y;
    A.M = M;
    A.N = (int)N;
    A.K = (int)K;
    A.tiles = (int)L.tiles;
    A.steps = (int)L.steps;
    A.ngroups = (int)L.ngroups;
    A.zwords = (int)L.zwords;
    A.group_shift = group == 32 ? 5 : group == 64 ? 6 : 7;
    A.steps_per_group = steps_per_group;
    A.steps_per_split = sps;
    const dim3 grid((unsigned)blocks_x, (unsigned)splits, (unsigned)zblocks);
    if (price) {
        KernelInfo info = {nullptr, 0, 0};
        launch_shape(shape, A, grid, st, &info);
        // (gemm_wide_b4 runs two steps per iteration)
        *price = {3, shape, splits, (long)blocks_x * splits * zblocks, sps / (SHAPES[shape].wide ? 2 : kw) + 1,
                  splits > 1 ? 2 : 1, info};
        return QG_OK;
    }
    launch_shape(shape, A, grid, st);
    if (qg_launch_status() != QG_OK) return QG_ERR_DEVICE;
    if (splits > 1) {
        const size_t count = (size_t)M * N;
        hipLaunchKernelGGL(add_splits, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st,
                           (const float *)partial, splits, count, Y);
    }
    return qg_launch_status();
}
}  // namespace

void qg_gemm_clear_tuning()
{
    std::lock_guard<std::mutex> lock(g_gemm_mutex);
    g_gemm_count = 0;
    g_gemm_next = 0;
}

extern "C" int qg_gemm_small(const void *packed, int64_t N, int64_t K, int bits, int group,
                             const float *X, int M, float *Y, void *workspace,
                             size_t workspace_bytes, void *stream)
{
    int splits = g_tune_splits, shape = g_tune_shape;
    if (splits == 0 && shape == 0 && g_gemm_count > 0) (void)gemm_tuning_for(N, K, bits, group, M, &splits, &shape);
    return gemm_small(packed, N, K, bits, group, X, M, Y, workspace, workspace_bytes, stream, splits, shape, nullptr);
}

// The launch-shape search of the small-M product: the counterpart of the paper's parameter search
// (Section 3, Algorithm 4, with the resource model of eqs. (3)-(5)) for this call.  Candidates
// are (kernel family / workgroup shape) x (number of K ranges).  Each is planned without being
// launched (a shape that does not fit the problem falls back to the built-in one, and a plan
// seen before is not tried again) and priced: the registers per lane and the LDS per workgroup of its kernel instance
// give the workgroups the chip holds at once, hence the rounds the launch needs; a round costs
// a workgroup's fixed time plus its iterations, and every further kernel of the call a launch.
// Candidates priced above 1.5 times the cheapest are dropped, the others timed.
namespace {
constexpr int GT_SHAPES = NSHAPES + 3;           // 0 (built-in choice), -1 (gemm_rows16), 1 ... NSHAPES, NSHAPES + 1 (raw codes)
constexpr int GT_CANDIDATES = GT_SHAPES * MAX_SPLITS;
constexpr int gt_shape(int c) { return c / MAX_SPLITS == 0 ? 0 : c / MAX_SPLITS == 1 ? -1 : c / MAX_SPLITS - 1; }
float g_gt_us[GT_CANDIDATES];                    // -1: dropped by the price, -2: same plan as an earlier candidate
int g_gt_timed = 0, g_gt_dropped = 0;
// measured on this machine: a workgroup's time outside its loop (first loads, reduction across
// k-slices, output), one barrier-to-barrier iteration (a memory round trip), one more kernel in a call
constexpr double GT_FIXED_US = 3.3, GT_ITERATION_US = 2.0, GT_LAUNCH_US = 3.0;

double gemm_price_us(const GemmPrice &p)
{
    if (p.family == 1 || p.family == 2) return 0.0;          // no model: always timed
    int resident = 1;
    hipFuncAttributes attr;
    if (p.kernel.kernel && hipFuncGetAttributes(&attr, p.kernel.kernel) == hipSuccess) {
        const int waves = p.kernel.threads / QG_WAVE;
        const int regs = ((attr.numRegs > 0 ? attr.numRegs : 128) + 7) / 8 * 8;
        int per_simd = 512 / regs;
        if (per_simd > 8) per_simd = 8;
        if (per_simd < 1) per_simd = 1;
        resident = per_simd * 4 / waves;
        const size_t lds = attr.sharedSizeBytes + p.kernel.lds_dynamic;
        if (lds > 0 && (int)((160u << 10) / lds) < resident) resident = (int)((160u << 10) / lds);
        if (resident < 1) resident = 1;
    } else {
        (void)hipGetLastError();
    }
    const long capacity = (long)resident * qg_compute_units();
    const long rounds = (p.workgroups + capacity - 1) / capacity;
    return (double)rounds * (GT_FIXED_US + (double)p.iterations * GT_ITERATION_US) + (double)(p.launches - 1) * GT_LAUNCH_US;
}
}  // namespace

extern "C" int qg_gemm_autotune(const void *const *packed_sets, int sets, int64_t N, int64_t K, int bits,
                                int group, const float *X, int M, float *Y, void *workspace,
                                size_t workspace_bytes, void *stream, int repeats, int *splits,
                                int *shape, float *best_us)
{
    if (repeats <= 0 || sets <= 0) return QG_ERR_SHAPE;
    if (!packed_sets) return QG_ERR_NULL;
    for (int s = 0; s < sets; ++s)
        if (!packed_sets[s]) return QG_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    // 1. plan and price every candidate
    GemmPrice plan[GT_CANDIDATES];
    double price[GT_CANDIDATES], cheapest = -1.0;
    bool valid[GT_CANDIDATES];
    for (int c = 0; c < GT_CANDIDATES; ++c) {
        const int sh = gt_shape(c), sp = 1 + c % MAX_SPLITS;
        const int rc = gemm_small(packed_sets[0], N, K, bits, group, X, M, Y, workspace, workspace_bytes, stream, sp, sh, &plan[c]);
        if (rc == QG_ERR_UNSUPPORTED) { valid[c] = false; continue; }
        if (rc != QG_OK) return rc;
        valid[c] = true;
        for (int e = 0; e < c && valid[c]; ++e)          // a knob the planner did not follow: seen already
            if (valid[e] && plan[e].family == plan[c].family && plan[e].shape == plan[c].shape && plan[e].splits == plan[c].splits)
                valid[c] = false;
        if (!valid[c]) continue;
        price[c] = gemm_price_us(plan[c]);
        if (price[c] > 0.0 && (cheapest < 0.0 || price[c] < cheapest)) cheapest = price[c];
    }
    // 2. time the survivors
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return QG_ERR_DEVICE;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return QG_ERR_DEVICE; }
    int best = -1, rc = QG_OK, turn = 0;
    float best_ms = -1.0f;
    g_gt_timed = 0;
    g_gt_dropped = 0;
    for (int c = 0; c < GT_CANDIDATES && rc == QG_OK; ++c) {
        g_gt_us[c] = -2.0f;
        if (!valid[c]) continue;
        if (price[c] > 1.5 * cheapest && cheapest > 0.0) {
            g_gt_us[c] = -1.0f;
            ++g_gt_dropped;
            continue;
        }
        const int sh = gt_shape(c), sp = 1 + c % MAX_SPLITS;
        auto run = [&]() {
            return gemm_small(packed_sets[turn++ % sets], N, K, bits, group, X, M, Y, workspace, workspace_bytes, stream, sp, sh, nullptr);
        };
        for (int i = 0; i < 2 && rc == QG_OK; ++i) rc = run();
        if (rc != QG_OK) break;
        if (hipEventRecord(e0, st) != hipSuccess) { rc = QG_ERR_DEVICE; break; }
        for (int i = 0; i < repeats && rc == QG_OK; ++i) rc = run();
        if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) rc = QG_ERR_DEVICE;
        float ms = 0.0f;
        if (rc == QG_OK && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = QG_ERR_DEVICE;
        if (rc != QG_OK) break;
        g_gt_us[c] = ms * 1e3f / (float)repeats;
        ++g_gt_timed;
        if (best < 0 || ms < best_ms) {
            best_ms = ms;
            best = c;
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != QG_OK || best < 0) return rc != QG_OK ? rc : QG_ERR_DEVICE;
    const int won_shape = gt_shape(best), won_splits = 1 + best % MAX_SPLITS;
    gemm_record_tuning(N, K, bits, group, M, won_splits, won_shape);
    if (splits) *splits = won_splits;
    if (shape) *shape = won_shape;
    if (best_us) *best_us = best_ms * 1e3f / (float)repeats;
    return QG_OK;
}

extern "C" int qg_gemm_autotune_report(float *us, int capacity, int *timed, int *dropped)
{
    if (us) {
        if (capacity < GT_CANDIDATES) return QG_ERR_SHAPE;
        for (int c = 0; c < GT_CANDIDATES; ++c) us[c] = g_gt_us[c];
    }
    if (timed) *timed = g_gt_timed;
    if (dropped) *dropped = g_gt_dropped;
    return QG_OK;
}
