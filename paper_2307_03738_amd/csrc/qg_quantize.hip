// qg_quantize: per-group min-max round-to-nearest quantization (Section 2, quantization
// function Q in its integer-zero form).  One team of TEAM lanes per group; every fp32 step is
// a single correctly rounded operation so the codes are reproducible bit for bit.
#include "qg_common.h"

namespace {

template <int TEAM>
__global__ __launch_bounds__(256) void quantize_kernel(const float4 *__restrict__ W,
                                                       int64_t total_groups, int f4_per_group,
                                                       int qmax, uint32_t *__restrict__ q4,
                                                       float *__restrict__ s,
                                                       uint8_t *__restrict__ z)
{
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t team = tid / TEAM;
    const int lane = (int)(tid % TEAM);
    if (team >= total_groups) return;   // whole teams leave together (TEAM divides 64)

    const float4 *g = W + team * f4_per_group;
    float lo = 0.0f, hi = 0.0f;         // the range always contains 0
    for (int i = lane; i < f4_per_group; i += TEAM) {
        const float4 v = g[i];
        lo = v.x < lo ? v.x : lo;  hi = v.x > hi ? v.x : hi;
        lo = v.y < lo ? v.y : lo;  hi = v.y > hi ? v.y : hi;
        lo = v.z < lo ? v.z : lo;  hi = v.z > hi ? v.z : hi;
        lo = v.w < lo ? v.w : lo;  hi = v.w > hi ? v.w : hi;
    }
#pragma unroll
    for (int off = TEAM / 2; off >= 1; off >>= 1) {
        const float ol = __shfl_xor(lo, off);
        const float oh = __shfl_xor(hi, off);
        lo = ol < lo ? ol : lo;
        hi = oh > hi ? oh : hi;
    }

    const float range = hi - lo;
    float scale = 1.0f;
    int zero = 0;
    if (range != 0.0f) {
        scale = range / (float)qmax;               // s = (hi - lo) / (2^b - 1)
        zero = (int)rintf(-lo / scale);            // z = rint(-lo / s), clamped
        zero = zero < 0 ? 0 : (zero > qmax ? qmax : zero);
    }
    if (lane == 0) {
        s[team] = scale;
        z[team] = (uint8_t)zero;
    }

    uint32_t *qo = q4 + team * f4_per_group;
    for (int i = lane; i < f4_per_group; i += TEAM) {
        const float4 v = g[i];
        const float w[4] = {v.x, v.y, v.z, v.w};
        uint32_t packed = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int c = (int)rintf(w[j] / scale) + zero;   // ties to even, integer add of z
            c = c < 0 ? 0 : (c > qmax ? qmax : c);
            packed |= (uint32_t)c << (8 * j);
        }
        qo[i] = packed;
    }
}

// The same for groups of 4 * R * TEAM weights (TEAM a power of two <= 64): every lane keeps its
// R float4 in registers, so W is read once, and handles U groups whose loads are all issued
// before the first is reduced.  Teams of one wavefront work on neighbouring groups, so each
// load instruction reads 1 KB of consecutive weights.
template <int TEAM, int R, int U>
__global__ __launch_bounds__(256) void quantize_regs(const float4 *__restrict__ W, int64_t total_groups,
                                                     int qmax, uint32_t *__restrict__ q4,
                                                     float *__restrict__ s, uint8_t *__restrict__ z)
{
    constexpr int F4 = TEAM * R;                   // float4 per group
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t teams = (int64_t)gridDim.x * blockDim.x / TEAM;
    const int64_t team = tid / TEAM;
    const int lane = (int)(tid % TEAM);

    float4 v[U][R];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        int64_t g = team + u * teams;
        g = g < total_groups ? g : total_groups - 1;          // past the end: reloaded, not stored
#pragma unroll
        for (int r = 0; r < R; ++r) v[u][r] = W[g * F4 + r * TEAM + lane];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t g = team + u * teams;
        float lo = 0.0f, hi = 0.0f;                // the range always contains 0
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float4 a = v[u][r];
            lo = a.x < lo ? a.x : lo;  hi = a.x > hi ? a.x : hi;
            lo = a.y < lo ? a.y : lo;  hi = a.y > hi ? a.y : hi;
            lo = a.z < lo ? a.z : lo;  hi = a.z > hi ? a.z : hi;
            lo = a.w < lo ? a.w : lo;  hi = a.w > hi ? a.w : hi;
        }
#pragma unroll
        for (int off = TEAM / 2; off >= 1; off >>= 1) {
            const float ol = __shfl_xor(lo, off);
            const float oh = __shfl_xor(hi, off);
            lo = ol < lo ? ol : lo;
            hi = oh > hi ? oh : hi;
        }
        const float range = hi - lo;
        float scale = 1.0f;
        int zero = 0;
        if (range != 0.0f) {
            scale = range / (float)qmax;
            zero = (int)rintf(-lo / scale);
            zero = zero < 0 ? 0 : (zero > qmax ? qmax : zero);
        }
        if (g >= total_groups) continue;
        if (lane == 0) {
            s[g] = scale;
            z[g] = (uint8_t)zero;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float w[4] = {v[u][r].x, v[u][r].y, v[u][r].z, v[u][r].w};
            uint32_t packed = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int c = (int)rintf(w[j] / scale) + zero;
                c = c < 0 ? 0 : (c > qmax ? qmax : c);
                packed |= (uint32_t)c << (8 * j);
            }
            q4[g * F4 + r * TEAM + lane] = packed;
        }
    }
}

template <int TEAM, int R>
int launch_regs(const float *W, int64_t groups, int qmax, uint8_t *q, float *s, uint8_t *z,
                hipStream_t stream)
{
    constexpr int U = R >= 8 ? 1 : R >= 4 ? 2 : 4;
    const int64_t threads = (groups + U - 1) / U * TEAM;
    const int64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffff) return QG_ERR_SHAPE;
    hipLaunchKernelGGL((quantize_regs<TEAM, R, U>), dim3((unsigned)blocks), dim3(256), 0, stream,
                       (const float4 *)W, groups, qmax, (uint32_t *)q, s, z);
    return qg_launch_status();
}

template <int TEAM>
int launch(const float *W, int64_t groups, int f4, int qmax, uint8_t *q, float *s, uint8_t *z,
           hipStream_t stream)
{
    const int64_t threads = groups * TEAM;
    const int64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffff) return QG_ERR_SHAPE;
    hipLaunchKernelGGL(quantize_kernel<TEAM>, dim3((unsigned)blocks), dim3(256), 0, stream,
                       (const float4 *)W, groups, f4, qmax, (uint32_t *)q, s, z);
    return qg_launch_status();
}

}  // namespace

extern "C" int qg_quantize(const float *W, int64_t N, int64_t K, int bits, int group,
                           uint8_t *q, float *s, uint8_t *z, void *stream)
{
    if (bits != 2 && bits != 3 && bits != 4) return QG_ERR_UNSUPPORTED;
    if (N <= 0 || K <= 0 || group <= 0 || K % group != 0 || group % 4 != 0) return QG_ERR_SHAPE;
    if (N > (int64_t)1 << 24 || K > (int64_t)1 << 24) return QG_ERR_SHAPE;
    if (!W || !q || !s || !z) return QG_ERR_NULL;
    if (!qg_aligned16(W) || !qg_aligned16(q)) return QG_ERR_ALIGN;
    const int64_t groups = N * (K / group);
    const int f4 = group / 4;
    const int qmax = (1 << bits) - 1;
    hipStream_t st = (hipStream_t)stream;
    switch (f4) {                                  // groups of 16 ... 4096 weights: W read once
    case 4: return launch_regs<4, 1>(W, groups, qmax, q, s, z, st);
    case 8: return launch_regs<8, 1>(W, groups, qmax, q, s, z, st);
    case 16: return launch_regs<16, 1>(W, groups, qmax, q, s, z, st);
    case 32: return launch_regs<32, 1>(W, groups, qmax, q, s, z, st);
    case 64: return launch_regs<64, 1>(W, groups, qmax, q, s, z, st);
    case 128: return launch_regs<64, 2>(W, groups, qmax, q, s, z, st);
    case 256: return launch_regs<64, 4>(W, groups, qmax, q, s, z, st);
    case 512: return launch_regs<64, 8>(W, groups, qmax, q, s, z, st);
    case 1024: return launch_regs<64, 16>(W, groups, qmax, q, s, z, st);
    default: break;
    }
    if (f4 >= 64) return launch<64>(W, groups, f4, qmax, q, s, z, st);
    if (f4 >= 32) return launch<32>(W, groups, f4, qmax, q, s, z, st);
    if (f4 >= 16) return launch<16>(W, groups, f4, qmax, q, s, z, st);
    if (f4 >= 8) return launch<8>(W, groups, f4, qmax, q, s, z, st);
    if (f4 >= 4) return launch<4>(W, groups, f4, qmax, q, s, z, st);
    if (f4 >= 2) return launch<2>(W, groups, f4, qmax, q, s, z, st);
    return launch<1>(W, groups, f4, qmax, q, s, z, st);
}
