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
#include <type_traits>

#include "qg_common.h"

size_t qg_gemm_workspace_bytes(const QgLayout &L, int M);
int qg_gemm_rows16(const void *packed, int64_t N, int64_t K, int bits, int group, const float *X,
                   int M, float *Y, void *workspace, void *stream);   // qg_gemv.hip

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
int g_tune_shape = 0;       // 1 + index into SHAPES

int gcd(int a, int b) { return b == 0 ? a : gcd(b, a % b); }

template <int MB, int TN, int KW>
void launch(const GemmArgs &A, dim3 grid, hipStream_t st)
{
    if (A.group_shift == 7)
        hipLaunchKernelGGL((gemm_small_b4<MB, TN, KW, true>), grid, dim3(TN * KW * 64), 0, st, A);
    else
        hipLaunchKernelGGL((gemm_small_b4<MB, TN, KW, false>), grid, dim3(TN * KW * 64), 0, st, A);
}

template <int MB, int TN>
void launch_wide(const GemmArgs &A, dim3 grid, hipStream_t st)
{
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

void launch_shape(int i, const GemmArgs &A, dim3 grid, hipStream_t st)
{
    switch (i) {
    case 0: launch<1, 1, 4>(A, grid, st); break;
    case 1: launch<1, 2, 4>(A, grid, st); break;
    case 2: launch<1, 4, 2>(A, grid, st); break;
    case 3: launch<2, 2, 2>(A, grid, st); break;
    case 4: launch<2, 4, 1>(A, grid, st); break;
    case 5: launch<2, 4, 2>(A, grid, st); break;
    case 6: launch<2, 8, 1>(A, grid, st); break;
    case 7: launch_wide<2, 4>(A, grid, st); break;
    case 8: launch_wide<2, 2>(A, grid, st); break;
    case 9: launch_wide<4, 4>(A, grid, st); break;
    case 10: launch_wide<4, 2>(A, grid, st); break;
    default: launch_wide<2, 8>(A, grid, st); break;
    }
}

}  // namespace

size_t qg_gemm_workspace_bytes(const QgLayout &L, int M)
{
    // partial results of the K split, or the GEMV workspaces of the rows of one grouped launch
    const size_t partial = (size_t)MAX_SPLITS * M * L.N * sizeof(float);
    const size_t gemv = qg_round_up((size_t)L.tiles * (QG_MAX_CHUNKS + 1) * QG_WAVE * sizeof(uint32_t),
                                    QG_SECTION_ALIGN);                                    // as qg_gemv asks
    const int rows = M < QG_MAX_GROUPED ? M : QG_MAX_GROUPED;
    return qg_round_up(fast_path(L) ? partial : gemv * rows, QG_SECTION_ALIGN);
}

extern "C" int qg_set_gemm_tuning(int splits, int shape)
{
    if (splits < 0 || splits > MAX_SPLITS || shape < -1 || shape > NSHAPES) return QG_ERR_SHAPE;
    g_tune_splits = splits;
    g_tune_shape = shape;
    return QG_OK;
}

extern "C" int qg_gemm_small(const void *packed, int64_t N, int64_t K, int bits, int group,
                             const float *X, int M, float *Y, void *workspace,
                             size_t workspace_bytes, void *stream)
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

    // Up to 16 rows: the barrier-free kernel on the GEMV's launch structure, where it applies.
    // It has one workgroup per tile and no split of K over workgroups, so it needs enough tiles
    // to cover the chip (measured: ahead from about 128 tiles; shape -1 forces it).
    if (M <= 16 && (g_tune_shape == 0 ? L.tiles >= 128 : g_tune_shape < 0)) {
        const int r = qg_gemm_rows16(packed, N, K, bits, group, X, M, Y, workspace, stream);
        if (r != QG_ERR_UNSUPPORTED) return r;
    }

    if (!fast_path(L)) {
        // the fp32 GEMV once per activation row, up to 16 rows per launch (rows of X stay
        // 64-byte aligned only if K % 16 == 0)
        if (K % 16 != 0 && M > 1) return QG_ERR_UNSUPPORTED;
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
            const int r = qg_gemv_grouped(d, rows, workspace, workspace_bytes, stream);
            if (r != QG_OK) return r;
        }
        return QG_OK;
    }

    // Workgroup shape (measured choices).  Up to 32 rows: one block of rows, two tiles x four
    // k-slices.  Up to 64 rows: gemm_wide_b4 with four tiles per workgroup.  More: all rows
    // in one wavefront (gemm_wide_b4, every weight dequantized once) when the launch has
    // enough tiles for it, otherwise blocks of 64 rows on the grid's z axis, four tiles x two
    // k-slices (two blocks double the wavefronts of a launch at the price of dequantizing
    // twice, which pays as long as the launch cannot fill the chip).
    int shape = M <= 32 ? 1 : M <= 64 ? 7 : L.tiles >= 128 ? 9 : 5;
    if (g_tune_shape > 0) {
        const Shape &s = SHAPES[g_tune_shape - 1];
        if (s.wide ? (M > 32 && M <= s.mb * 32) : ((s.mb == 1) == (M <= 32))) shape = g_tune_shape - 1;
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
    int splits = g_tune_splits ? g_tune_splits : (cus + blocks_x * zblocks - 1) / (blocks_x * zblocks);
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
    launch_shape(shape, A, grid, st);
    if (qg_launch_status() != QG_OK) return QG_ERR_DEVICE;
    if (splits > 1) {
        const size_t count = (size_t)M * N;
        hipLaunchKernelGGL(add_splits, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st,
                           (const float *)partial, splits, count, Y);
    }
    return qg_launch_status();
}
