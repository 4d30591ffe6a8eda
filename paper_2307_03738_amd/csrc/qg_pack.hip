// qg_pack / qg_unpack: codes, scales and zero-points <-> packed blob, for the paper's
// canonical word format (Section 3 "Data format", Algorithm 2) and for the device layout
// described in qg_common.h.  Pure integer work; results are exact.
#include "qg_common.h"

namespace {

// ------------------------------------------------------------------ canonical layout

// Word w of the bit stream of output n: bits [32w, 32w+32) of sum_k v[n][k] << (b k).
__global__ void canon_pack_stream(const uint8_t *__restrict__ v, int64_t N, int64_t count,
                                  int bits, int64_t words, uint32_t *__restrict__ P)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= words * N) return;
    const int64_t w = idx / N, n = idx % N;
    const int64_t first = (32 * w) / bits;
    const int64_t last = (32 * w + 31) / bits;
    uint32_t word = 0;
    for (int64_t k = first; k <= last && k < count; ++k) {
        const uint32_t c = v[n * count + k];
        const int pos = (int)(bits * k - 32 * w);
        word |= pos >= 0 ? c << pos : c >> (-pos);
    }
    P[idx] = word;
}

__global__ void canon_unpack_stream(const uint32_t *__restrict__ P, int64_t N, int64_t count,
                                    int bits, uint8_t *__restrict__ v)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= N * count) return;
    const int64_t n = idx / count, k = idx % count;
    const int64_t bit = bits * k;
    const int64_t w = bit / 32;
    const int off = (int)(bit % 32);
    uint32_t c = P[w * N + n] >> off;
    if (off + bits > 32) c |= P[(w + 1) * N + n] << (32 - off);   // field straddles two words
    v[idx] = (uint8_t)(c & ((1u << bits) - 1u));
}

// s [N][G] <-> St [G][N]
__global__ void transpose_f32(const float *__restrict__ in, int64_t rows, int64_t cols,
                              float *__restrict__ out)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * cols) return;
    const int64_t c = idx / rows, r = idx % rows;   // out [cols][rows], r contiguous
    out[idx] = in[r * cols + c];
}

// ------------------------------------------------------------------ device layout

__device__ inline uint32_t byte_of(uint32_t w, int i) { return (w >> (8 * i)) & 0xffu; }

// One thread builds the `planes` uint4 of one (tile, unit, lane).
template <int BITS>
__global__ __launch_bounds__(256) void device_pack_codes(const uint8_t *__restrict__ q,
                                                         int64_t N, int64_t K, int64_t tiles,
                                                         int64_t units, uint4 *__restrict__ out)
{
    constexpr int CELL = BITS == 4 ? 8 : BITS == 2 ? 16 : 32;
    constexpr int PLANES = BITS == 3 ? 3 : 1;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= tiles * units * QG_WAVE) return;
    const int lane = (int)(idx % QG_WAVE);
    const int64_t unit = (idx / QG_WAVE) % units;
    const int64_t tile = idx / QG_WAVE / units;
    const int64_t n = tile * QG_WAVE + lane;

    uint32_t words[PLANES][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t k0 = (unit * 4 + j) * CELL;
        uint8_t c[CELL];
#pragma unroll
        for (int i = 0; i < CELL; ++i)
            c[i] = (n < N && k0 + i < K) ? q[n * K + k0 + i] : (uint8_t)0;
        if constexpr (BITS == 4 || BITS == 2) {
            uint32_t w = 0;
#pragma unroll
            for (int i = 0; i < CELL; ++i) w |= (uint32_t)c[i] << (BITS * i);
            words[0][j] = w;
        } else {
            uint32_t a = 0, b = 0, cc = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t t = (uint32_t)c[24 + i] | ((uint32_t)c[28 + i] << 3);  // 6 spare bits
                a |= ((uint32_t)c[i] | ((uint32_t)c[4 + i] << 3) | ((t & 3u) << 6)) << (8 * i);
                b |= ((uint32_t)c[8 + i] | ((uint32_t)c[12 + i] << 3) | (((t >> 2) & 3u) << 6)) << (8 * i);
                cc |= ((uint32_t)c[16 + i] | ((uint32_t)c[20 + i] << 3) | (((t >> 4) & 3u) << 6)) << (8 * i);
            }
            words[0][j] = a;
            words[1 % PLANES][j] = b;
            words[2 % PLANES][j] = cc;
        }
    }
#pragma unroll
    for (int p = 0; p < PLANES; ++p)
        out[((tile * units + unit) * PLANES + p) * QG_WAVE + lane] =
            make_uint4(words[p][0], words[p][1], words[p][2], words[p][3]);
}

template <int BITS>
__global__ __launch_bounds__(256) void device_unpack_codes(const uint4 *__restrict__ in,
                                                           int64_t N, int64_t K, int64_t tiles,
                                                           int64_t units, uint8_t *__restrict__ q)
{
    constexpr int CELL = BITS == 4 ? 8 : BITS == 2 ? 16 : 32;
    constexpr int PLANES = BITS == 3 ? 3 : 1;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= tiles * units * QG_WAVE) return;
    const int lane = (int)(idx % QG_WAVE);
    const int64_t unit = (idx / QG_WAVE) % units;
    const int64_t tile = idx / QG_WAVE / units;
    const int64_t n = tile * QG_WAVE + lane;
    if (n >= N) return;

    uint32_t words[PLANES][4];
#pragma unroll
    for (int p = 0; p < PLANES; ++p) {
        const uint4 v = in[((tile * units + unit) * PLANES + p) * QG_WAVE + lane];
        words[p][0] = v.x; words[p][1] = v.y; words[p][2] = v.z; words[p][3] = v.w;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t k0 = (unit * 4 + j) * CELL;
        uint8_t c[CELL];
        if constexpr (BITS == 4 || BITS == 2) {
#pragma unroll
            for (int i = 0; i < CELL; ++i)
                c[i] = (uint8_t)((words[0][j] >> (BITS * i)) & ((1u << BITS) - 1u));
        } else {
            const uint32_t a = words[0][j], b = words[1 % PLANES][j], cc = words[2 % PLANES][j];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t ba = byte_of(a, i), bb = byte_of(b, i), bc = byte_of(cc, i);
                const uint32_t t = (ba >> 6) | ((bb >> 6) << 2) | ((bc >> 6) << 4);
                c[i] = ba & 7u;        c[4 + i] = (ba >> 3) & 7u;
                c[8 + i] = bb & 7u;    c[12 + i] = (bb >> 3) & 7u;
                c[16 + i] = bc & 7u;   c[20 + i] = (bc >> 3) & 7u;
                c[24 + i] = t & 7u;    c[28 + i] = (t >> 3) & 7u;
            }
        }
#pragma unroll
        for (int i = 0; i < CELL; ++i)
            if (k0 + i < K) q[n * K + k0 + i] = c[i];
    }
}

// scales [tile][group][lane] and zero words [tile][zword][lane]
__global__ void device_pack_meta(const float *__restrict__ s, const uint8_t *__restrict__ z,
                                 int64_t N, int64_t ngroups, int64_t tiles, int64_t zwords,
                                 int zbits, float *__restrict__ sd, uint32_t *__restrict__ zd)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t ns = tiles * ngroups * QG_WAVE;
    const int64_t nz = tiles * zwords * QG_WAVE;
    if (idx < ns) {
        const int lane = (int)(idx % QG_WAVE);
        const int64_t g = (idx / QG_WAVE) % ngroups;
        const int64_t n = idx / QG_WAVE / ngroups * QG_WAVE + lane;
        sd[idx] = n < N ? s[n * ngroups + g] : 0.0f;
    } else if (idx < ns + nz) {
        const int64_t i = idx - ns;
        const int lane = (int)(i % QG_WAVE);
        const int64_t w = (i / QG_WAVE) % zwords;
        const int64_t n = i / QG_WAVE / zwords * QG_WAVE + lane;
        const int per = 32 / zbits;
        uint32_t word = 0;
        for (int j = 0; j < per; ++j) {
            const int64_t g = w * per + j;
            if (n < N && g < ngroups) word |= (uint32_t)z[n * ngroups + g] << (zbits * j);
        }
        zd[i] = word;
    }
}

__global__ void device_unpack_meta(const float *__restrict__ sd, const uint32_t *__restrict__ zd,
                                   int64_t N, int64_t ngroups, int64_t zwords, int zbits,
                                   float *__restrict__ s, uint8_t *__restrict__ z)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= N * ngroups) return;
    const int64_t n = idx / ngroups, g = idx % ngroups;
    const int64_t tile = n / QG_WAVE;
    const int lane = (int)(n % QG_WAVE);
    const int per = 32 / zbits;
    s[idx] = sd[(tile * ngroups + g) * QG_WAVE + lane];
    const uint32_t word = zd[(tile * zwords + g / per) * QG_WAVE + lane];
    z[idx] = (uint8_t)((word >> (zbits * (int)(g % per))) & ((1u << zbits) - 1u));
}

inline unsigned blocks_for(int64_t threads) { return (unsigned)((threads + 255) / 256); }

}  // namespace

extern "C" int qg_cell(int bits) { return qg_cell_of(bits); }

extern "C" const char *qg_status_string(int status)
{
    switch (status) {
    case QG_OK: return "ok";
    case QG_ERR_NULL: return "a required pointer is NULL";
    case QG_ERR_SHAPE: return "shape not accepted (sizes, K % group, group % cell)";
    case QG_ERR_UNSUPPORTED: return "unsupported bits, layout or problem count";
    case QG_ERR_ALIGN: return "pointer not 16-byte aligned";
    case QG_ERR_WORKSPACE: return "workspace missing or too small";
    case QG_ERR_DEVICE: return "HIP launch failed";
    default: return "unknown status";
    }
}

extern "C" size_t qg_packed_bytes(int64_t N, int64_t K, int bits, int group, int layout)
{
    if (layout == QG_LAYOUT_CANONICAL) {
        QgCanonical C;
        if (qg_make_canonical(N, K, bits, group, &C) != QG_OK) return 0;
        if (group % qg_cell_of(bits) != 0) return 0;
        return C.total;
    }
    if (layout == QG_LAYOUT_DEVICE) {
        QgLayout L;
        return qg_make_layout(N, K, bits, group, &L) == QG_OK ? L.total : 0;
    }
    return 0;
}

extern "C" int qg_pack(const uint8_t *q, const float *s, const uint8_t *z, int64_t N, int64_t K,
                       int bits, int group, int layout, void *packed, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (layout != QG_LAYOUT_CANONICAL && layout != QG_LAYOUT_DEVICE) return QG_ERR_UNSUPPORTED;
    QgLayout L;
    int rc = qg_make_layout(N, K, bits, group, &L);
    if (rc != QG_OK) return rc;
    if (!q || !s || !z || !packed) return QG_ERR_NULL;
    if (!qg_aligned16(packed)) return QG_ERR_ALIGN;
    char *base = (char *)packed;

    if (layout == QG_LAYOUT_CANONICAL) {
        QgCanonical C;
        rc = qg_make_canonical(N, K, bits, group, &C);
        if (rc != QG_OK) return rc;
        hipLaunchKernelGGL(canon_pack_stream, dim3(blocks_for(C.code_words * N)), dim3(256), 0, st,
                           q, N, K, bits, C.code_words, (uint32_t *)(base + C.codes_off));
        hipLaunchKernelGGL(transpose_f32, dim3(blocks_for(N * C.ngroups)), dim3(256), 0, st,
                           s, N, C.ngroups, (float *)(base + C.scales_off));
        hipLaunchKernelGGL(canon_pack_stream, dim3(blocks_for(C.zero_words * N)), dim3(256), 0, st,
                           z, N, C.ngroups, bits, C.zero_words, (uint32_t *)(base + C.zeros_off));
        return qg_launch_status();
    }

    const int64_t threads = L.tiles * L.units * QG_WAVE;
    uint4 *codes = (uint4 *)(base + L.codes_off);
    if (bits == 4)
        hipLaunchKernelGGL(device_pack_codes<4>, dim3(blocks_for(threads)), dim3(256), 0, st,
                           q, N, K, L.tiles, L.units, codes);
    else if (bits == 2)
        hipLaunchKernelGGL(device_pack_codes<2>, dim3(blocks_for(threads)), dim3(256), 0, st,
                           q, N, K, L.tiles, L.units, codes);
    else
        hipLaunchKernelGGL(device_pack_codes<3>, dim3(blocks_for(threads)), dim3(256), 0, st,
                           q, N, K, L.tiles, L.units, codes);
    const int64_t meta = L.tiles * (L.ngroups + L.zwords) * QG_WAVE;
    hipLaunchKernelGGL(device_pack_meta, dim3(blocks_for(meta)), dim3(256), 0, st,
                       s, z, N, L.ngroups, L.tiles, L.zwords, L.zbits,
                       (float *)(base + L.scales_off), (uint32_t *)(base + L.zeros_off));
    return qg_launch_status();
}

extern "C" int qg_unpack(const void *packed, int64_t N, int64_t K, int bits, int group,
                         int layout, uint8_t *q, float *s, uint8_t *z, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (layout != QG_LAYOUT_CANONICAL && layout != QG_LAYOUT_DEVICE) return QG_ERR_UNSUPPORTED;
    QgLayout L;
    int rc = qg_make_layout(N, K, bits, group, &L);
    if (rc != QG_OK) return rc;
    if (!q || !s || !z || !packed) return QG_ERR_NULL;
    if (!qg_aligned16(packed)) return QG_ERR_ALIGN;
    const char *base = (const char *)packed;

    if (layout == QG_LAYOUT_CANONICAL) {
        QgCanonical C;
        rc = qg_make_canonical(N, K, bits, group, &C);
        if (rc != QG_OK) return rc;
        hipLaunchKernelGGL(canon_unpack_stream, dim3(blocks_for(N * K)), dim3(256), 0, st,
                           (const uint32_t *)(base + C.codes_off), N, K, bits, q);
        hipLaunchKernelGGL(transpose_f32, dim3(blocks_for(N * C.ngroups)), dim3(256), 0, st,
                           (const float *)(base + C.scales_off), C.ngroups, N, s);
        hipLaunchKernelGGL(canon_unpack_stream, dim3(blocks_for(N * C.ngroups)), dim3(256), 0, st,
                           (const uint32_t *)(base + C.zeros_off), N, C.ngroups, bits, z);
        return qg_launch_status();
    }

    const int64_t threads = L.tiles * L.units * QG_WAVE;
    const uint4 *codes = (const uint4 *)(base + L.codes_off);
    if (bits == 4)
        hipLaunchKernelGGL(device_unpack_codes<4>, dim3(blocks_for(threads)), dim3(256), 0, st,
                           codes, N, K, L.tiles, L.units, q);
    else if (bits == 2)
        hipLaunchKernelGGL(device_unpack_codes<2>, dim3(blocks_for(threads)), dim3(256), 0, st,
                           codes, N, K, L.tiles, L.units, q);
    else
        hipLaunchKernelGGL(device_unpack_codes<3>, dim3(blocks_for(threads)), dim3(256), 0, st,
                           codes, N, K, L.tiles, L.units, q);
    hipLaunchKernelGGL(device_unpack_meta, dim3(blocks_for(N * L.ngroups)), dim3(256), 0, st,
                       (const float *)(base + L.scales_off), (const uint32_t *)(base + L.zeros_off),
                       N, L.ngroups, L.zwords, L.zbits, s, z);
    return qg_launch_status();
}
