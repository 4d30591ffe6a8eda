// qg_gemm_small: Y = X What^T for a few prompt tokens (M <= 128) on the matrix cores.
//
// The paper treats only the vector input; this is the same What = s (q - z) (Section 2,
// eq. (1)) applied to M activation rows at once.  X and the dequantized weights are rounded
// to bf16, products are accumulated in fp32 by v_mfma_f32_32x32x16_bf16.
//
// Mapping (4-bit codes, groups of a multiple of 32).  A wavefront owns one tile of 64
// outputs -- the same device layout the GEMV reads, lane l holding 32 consecutive k of output
// 64*tile + l in one 128-bit vector -- and all M rows.  The matrix instruction wants, for a
// block of 32 outputs, lanes l and l+32 to hold the SAME output with two different k-octets;
// the layout has them hold two different outputs with the same k.  One v_permlane32_swap of
// the raw code words (w0 with w2, w1 with w3) turns one into the other for both 32-output
// blocks at once, so weights go from HBM to the MFMA operand through registers only:
// mask, convert, one FMA with the group's (s, -z s), pack to bf16.  Every weight is
// dequantized exactly once.  The activation rows are converted to bf16 on their way into
// LDS, chunk by chunk (128 k), double-buffered, shared by the four wavefronts
// of a workgroup, which work on four neighbouring tiles over the same k range.  K may be
// cut into `splits` ranges handled by different workgroups; their fp32 partial results are
// added by a second small kernel in a fixed order.
//
// Other bit widths and group sizes take the fp32 GEMV kernel once per activation row.
#include "qg_common.h"

size_t qg_gemm_workspace_bytes(const QgLayout &L, int M);

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int KC = 128;            // k per chunk = one step of the 4-bit layout
constexpr int XPITCH = KC + 8;     // bf16 per LDS row: 272 bytes, conflict-free 128-bit reads
constexpr int GEMM_WAVES = 4;

struct GemmArgs {
    const uint4 *codes;
    const float *scales;
    const uint32_t *zeros;
    const float *X;            // activations [M][K] fp32
    float *out;                // Y, or partial results [split][M][N]
    int M, N, K, tiles, steps, ngroups, zwords, group;
    int steps_per_split;
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

// Eight 4-bit codes of one word -> eight bf16 values s*(q - z), in code order.
__device__ inline bf16x8 dequant_word(uint32_t w, float s, float nzs)
{
    const uint32_t lo = opaque(w & 0x0f0f0f0fu);          // codes 0, 2, 4, 6
    const uint32_t hi = opaque((w >> 4) & 0x0f0f0f0fu);   // codes 1, 3, 5, 7
    Operand o;
    floatx2 t;
    t[0] = fmaf((float)(lo & 0xffu), s, nzs);          t[1] = fmaf((float)(hi & 0xffu), s, nzs);
    o.p[0] = __builtin_convertvector(t, bf16x2);
    t[0] = fmaf((float)((lo >> 8) & 0xffu), s, nzs);   t[1] = fmaf((float)((hi >> 8) & 0xffu), s, nzs);
    o.p[1] = __builtin_convertvector(t, bf16x2);
    t[0] = fmaf((float)((lo >> 16) & 0xffu), s, nzs);  t[1] = fmaf((float)((hi >> 16) & 0xffu), s, nzs);
    o.p[2] = __builtin_convertvector(t, bf16x2);
    t[0] = fmaf((float)(lo >> 24), s, nzs);            t[1] = fmaf((float)(hi >> 24), s, nzs);
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

template <int MB>
__global__ __launch_bounds__(GEMM_WAVES * 64) void gemm_small_b4(const GemmArgs A)
{
    // two activation buffers: the chunk of the next step is written while this one is read
    __shared__ __attribute__((aligned(16))) __bf16 Xs[2][MB * 32 * XPITCH];
    constexpr int XLOADS = MB * 32 * (KC / 4) / (GEMM_WAVES * 64);   // float4 loads per thread and chunk

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tile = blockIdx.x * GEMM_WAVES + wave;
    const bool have_tile = tile < A.tiles;
    const int st0 = blockIdx.y * A.steps_per_split;
    int st1 = st0 + A.steps_per_split;
    if (st1 > A.steps) st1 = A.steps;

    const int tclamp = have_tile ? tile : A.tiles - 1;
    const uint4 *codes = A.codes + (size_t)tclamp * A.steps * 4 * QG_WAVE + lane;
    const float *sc = A.scales + (size_t)tclamp * A.ngroups * QG_WAVE + lane;
    const uint32_t *zr = A.zeros + (size_t)tclamp * A.zwords * QG_WAVE + lane;
    const int groups_per_step = KC / A.group > 0 ? KC / A.group : 1;   // G = 32, 64, 128 -> 4, 2, 1
    const int steps_per_group = A.group / KC > 0 ? A.group / KC : 1;    // G = 256, ... -> 2, ...

    floatx16 acc[MB][2];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mb][nb][i] = 0.0f;

    const int half = lane >> 5;           // which k-octet pair this lane feeds
    const int row = lane & 31;

    // this thread's share of an activation chunk: XLOADS pieces of 4 consecutive k, converted
    // to bf16 (round to nearest even) on the way into LDS; rows past M are zero
    float4 xr[XLOADS];
    auto load_x = [&](int step) {
#pragma unroll
        for (int j = 0; j < XLOADS; ++j) {
            const int i = j * GEMM_WAVES * 64 + threadIdx.x;
            const int m = i / (KC / 4), c4 = i % (KC / 4);
            xr[j] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (m < A.M) xr[j] = *(const float4 *)(A.X + (size_t)m * A.K + (size_t)step * KC + c4 * 4);
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int j = 0; j < XLOADS; ++j) {
            const int i = j * GEMM_WAVES * 64 + threadIdx.x;
            const int m = i / (KC / 4), c4 = i % (KC / 4);
            floatx2 a = {xr[j].x, xr[j].y}, b = {xr[j].z, xr[j].w};
            bf16x2 pa = __builtin_convertvector(a, bf16x2), pb = __builtin_convertvector(b, bf16x2);
            uint2 packed;
            packed.x = *(uint32_t *)&pa;
            packed.y = *(uint32_t *)&pb;
            *(uint2 *)(&Xs[buf][m * XPITCH + c4 * 4]) = packed;
        }
    };

    uint4 v[4], vn[4];
    if (st0 < st1) {
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = codes[((size_t)st0 * 4 + u) * QG_WAVE];
        load_x(st0);
        store_x(0);
    }
    __syncthreads();

    int buf = 0;
    for (int step = st0; step < st1; ++step) {
        const bool more = step + 1 < st1;
        if (more) {
#pragma unroll
            for (int u = 0; u < 4; ++u) vn[u] = codes[((size_t)(step + 1) * 4 + u) * QG_WAVE];
            load_x(step + 1);
        }
        // scale and zero of the step's groups (G is a multiple of 32)
        float s_u[4], nzs_u[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int g = steps_per_group > 1 ? step / steps_per_group
                                              : step * groups_per_step + (u * 32) / A.group;
            s_u[u] = sc[(size_t)g * QG_WAVE];
            const uint32_t zword = zr[(size_t)(g / 8) * QG_WAVE];
            nzs_u[u] = -(float)((zword >> (4 * (g % 8))) & 15u) * s_u[u];
        }
        const __bf16 *xs = Xs[buf];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            // outputs 0-31 of the tile in both halves (P), outputs 32-63 in both halves (Q)
            uint32_t sP, sQ, nP, nQ, P0, Q0, P1, Q1;
            swap_halves(__float_as_uint(s_u[u]), __float_as_uint(s_u[u]), sP, sQ);
            swap_halves(__float_as_uint(nzs_u[u]), __float_as_uint(nzs_u[u]), nP, nQ);
            swap_halves(v[u].x, v[u].z, P0, Q0);       // k-octets 0 (low lanes) and 2 (high lanes)
            swap_halves(v[u].y, v[u].w, P1, Q1);       // k-octets 1 and 3
            const bf16x8 bP0 = dequant_word(P0, __uint_as_float(sP), __uint_as_float(nP));
            const bf16x8 bP1 = dequant_word(P1, __uint_as_float(sP), __uint_as_float(nP));
            const bf16x8 bQ0 = dequant_word(Q0, __uint_as_float(sQ), __uint_as_float(nQ));
            const bf16x8 bQ1 = dequant_word(Q1, __uint_as_float(sQ), __uint_as_float(nQ));
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const __bf16 *xp = xs + (mb * 32 + row) * XPITCH + u * 32 + half * 16;
                const bf16x8 a0 = *(const bf16x8 *)(xp);          // octet 0 or 2
                const bf16x8 a1 = *(const bf16x8 *)(xp + 8);      // octet 1 or 3
                acc[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bP0, acc[mb][0], 0, 0, 0);
                acc[mb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bP1, acc[mb][0], 0, 0, 0);
                acc[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bQ0, acc[mb][1], 0, 0, 0);
                acc[mb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bQ1, acc[mb][1], 0, 0, 0);
            }
        }
        if (more) {
            store_x(buf ^ 1);
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = vn[u];
        }
        __syncthreads();      // next chunk written, this chunk's readers done
        buf ^= 1;
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

__global__ void add_splits(const float *__restrict__ partial, int splits, size_t count,
                           float *__restrict__ Y)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    float t = partial[i];
    for (int s = 1; s < splits; ++s) t += partial[(size_t)s * count + i];
    Y[i] = t;
}

bool fast_path(const QgLayout &L)
{
    return L.bits == 4 && L.group % 32 == 0 && L.K % KC == 0 &&
           (L.group <= KC ? KC % L.group == 0 : L.group % KC == 0);
}

int max_splits(int M) { return M <= 32 ? 8 : 4; }

}  // namespace

size_t qg_gemm_workspace_bytes(const QgLayout &L, int M)
{
    // partial results of the K split, or the GEMV workspace for the row-by-row path
    const size_t partial = (size_t)max_splits(M) * M * L.N * sizeof(float);
    const size_t gemv = (size_t)L.tiles * QG_MAX_CHUNKS * QG_WAVE * sizeof(uint32_t);
    return qg_round_up(fast_path(L) ? partial : gemv, QG_SECTION_ALIGN);
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

    if (!fast_path(L)) {
        // fp32 GEMV per activation row (rows of X stay 64-byte aligned only if K % 16 == 0)
        if (K % 16 != 0 && M > 1) return QG_ERR_UNSUPPORTED;
        for (int m = 0; m < M; ++m) {
            const int r = qg_gemv(packed, N, K, bits, group, X + (size_t)m * K, Y + (size_t)m * N,
                                  workspace, workspace_bytes, stream);
            if (r != QG_OK) return r;
        }
        return QG_OK;
    }

    // enough wavefronts for about one per SIMD, within the workspace's split budget
    int splits = (int)((1024 + L.tiles - 1) / L.tiles);
    if (splits > max_splits(M)) splits = max_splits(M);
    if (splits > L.steps) splits = (int)L.steps;
    int sps = (int)((L.steps + splits - 1) / splits);
    if (L.group > KC) {                                   // keep whole groups inside a split
        const int q = L.group / KC;
        sps = (sps + q - 1) / q * q;
    }
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
    A.group = group;
    A.steps_per_split = sps;
    const dim3 grid((unsigned)((L.tiles + GEMM_WAVES - 1) / GEMM_WAVES), (unsigned)splits);
    const dim3 block(GEMM_WAVES * 64);
    if (M <= 32) hipLaunchKernelGGL(gemm_small_b4<1>, grid, block, 0, st, A);
    else if (M <= 64) hipLaunchKernelGGL(gemm_small_b4<2>, grid, block, 0, st, A);
    else hipLaunchKernelGGL(gemm_small_b4<4>, grid, block, 0, st, A);
    if (qg_launch_status() != QG_OK) return QG_ERR_DEVICE;
    if (splits > 1) {
        const size_t count = (size_t)M * N;
        hipLaunchKernelGGL(add_splits, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st,
                           (const float *)partial, splits, count, Y);
    }
    return qg_launch_status();
}
