// qg_pack / qg_unpack: codes, scales and zero-points <-> packed blob, for the paper's
// canonical word format (Section 3 "Data format", Algorithm 2) and for the device layout
// described in qg_common.h.  Pure integer work; results are exact.
#include "qg_common.h"

namespace {

// Every kernel here moves a block of 64 rows (outputs) x SPAN columns of a row-major matrix
// through LDS, so that the row-major side is read or written in 16-byte pieces, 16 or more
// consecutive lanes on one row, and the packed side with lane = output, 64 lanes on
// consecutive words.  A workgroup is 256 threads = 4 wavefronts.  Rows of the LDS image are
// PITCH = SPAN + 16 bytes apart: with lane = row, 128-bit LDS accesses then fall on distinct
// banks.
constexpr int PK_THREADS = 256;

// rows [r0, r0+64) x columns [c0, c0+SPAN) of v [rows][cols] -> lds; zeros outside the matrix.
// `wide`: cols % 16 == 0 and v 16-byte aligned, so the block is moved in 16-byte pieces.
template <int SPAN>
__device__ inline void rows_to_lds(const uint8_t *__restrict__ v, int64_t rows, int64_t cols,
                                   int64_t r0, int64_t c0, bool wide, uint8_t *lds)
{
    constexpr int PITCH = SPAN + 16;
    if (wide) {
        // all loads of the thread are issued before the first is stored
        constexpr int PIECES = SPAN / 16;
        constexpr int PER = QG_WAVE * PIECES / PK_THREADS;
        uint4 val[PER];
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int i = threadIdx.x + j * PK_THREADS;
            const int r = i / PIECES, p = i % PIECES;
            const int64_t n = r0 + r, c = c0 + 16 * p;
            val[j] = make_uint4(0u, 0u, 0u, 0u);
            if (n < rows && c < cols) val[j] = *(const uint4 *)(v + n * cols + c);
        }
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int i = threadIdx.x + j * PK_THREADS;
            *(uint4 *)(lds + (i / PIECES) * PITCH + 16 * (i % PIECES)) = val[j];
        }
    } else {
        for (int i = threadIdx.x; i < QG_WAVE * SPAN; i += PK_THREADS) {
            const int r = i / SPAN, b = i % SPAN;
            const int64_t n = r0 + r, c = c0 + b;
            lds[r * PITCH + b] = (n < rows && c < cols) ? v[n * cols + c] : (uint8_t)0;
        }
    }
}

// the inverse: the part of the block that lies inside the matrix is written
template <int SPAN>
__device__ inline void lds_to_rows(uint8_t *__restrict__ v, int64_t rows, int64_t cols,
                                   int64_t r0, int64_t c0, bool wide, const uint8_t *lds)
{
    constexpr int PITCH = SPAN + 16;
    if (wide) {
        constexpr int PIECES = SPAN / 16;
        for (int i = threadIdx.x; i < QG_WAVE * PIECES; i += PK_THREADS) {
            const int r = i / PIECES, p = i % PIECES;
            const int64_t n = r0 + r, c = c0 + 16 * p;
            if (n < rows && c < cols) *(uint4 *)(v + n * cols + c) = *(const uint4 *)(lds + r * PITCH + 16 * p);
        }
    } else {
        for (int i = threadIdx.x; i < QG_WAVE * SPAN; i += PK_THREADS) {
            const int r = i / SPAN, b = i % SPAN;
            const int64_t n = r0 + r, c = c0 + b;
            if (n < rows && c < cols) v[n * cols + c] = lds[r * PITCH + b];
        }
    }
}

// Four codes, one per byte of d, <-> their fields side by side in the low bits.
__device__ inline uint32_t squeeze4(uint32_t d)          // -> 16 bits
{
    const uint32_t t = (d | (d >> 4)) & 0x00ff00ffu;
    return (t | (t >> 8)) & 0xffffu;
}
__device__ inline uint32_t squeeze2(uint32_t d)          // -> 8 bits
{
    const uint32_t t = (d | (d >> 6)) & 0x000f000fu;
    return (t | (t >> 12)) & 0xffu;
}
__device__ inline uint32_t squeeze3(uint32_t d)          // -> 12 bits
{
    const uint32_t t = (d | (d >> 5)) & 0x003f003fu;
    return (t | (t >> 10)) & 0xfffu;
}
__device__ inline uint32_t spread4(uint32_t u)
{
    const uint32_t t = (u | (u << 8)) & 0x00ff00ffu;
    return (t | (t << 4)) & 0x0f0f0f0fu;
}
__device__ inline uint32_t spread2(uint32_t u)
{
    const uint32_t t = (u | (u << 12)) & 0x000f000fu;
    return (t | (t << 6)) & 0x03030303u;
}
__device__ inline uint32_t spread3(uint32_t u)
{
    const uint32_t t = (u | (u << 10)) & 0x003f003fu;
    return (t | (t << 5)) & 0x07070707u;
}

// Words of the little-endian bit stream of FB-bit fields (Section 3 "Data format";
// Algorithm 2 for 4 bits) built from / cut back into codes held one per byte, four to a
// dword.  A "run" is the shortest piece of the stream that ends on a word boundary:
// 8 codes = 1 word at 4 bits, 16 codes = 1 word at 2 bits, 32 codes = 3 words at 3 bits.
template <int FB> struct Run;
template <> struct Run<4> {
    static constexpr int CODES = 8, WORDS = 1;
    static __device__ inline void pack(const uint32_t *d, uint32_t *w) { w[0] = squeeze4(d[0]) | (squeeze4(d[1]) << 16); }
    static __device__ inline void unpack(const uint32_t *w, uint32_t *d)
    {
        d[0] = spread4(w[0] & 0xffffu);
        d[1] = spread4(w[0] >> 16);
    }
};
template <> struct Run<2> {
    static constexpr int CODES = 16, WORDS = 1;
    static __device__ inline void pack(const uint32_t *d, uint32_t *w)
    {
        w[0] = squeeze2(d[0]) | (squeeze2(d[1]) << 8) | (squeeze2(d[2]) << 16) | (squeeze2(d[3]) << 24);
    }
    static __device__ inline void unpack(const uint32_t *w, uint32_t *d)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) d[i] = spread2((w[0] >> (8 * i)) & 0xffu);
    }
};
template <> struct Run<3> {
    static constexpr int CODES = 32, WORDS = 3;
    static __device__ inline void pack(const uint32_t *d, uint32_t *w)
    {
        uint32_t p[8];                                   // 12 bits each
#pragma unroll
        for (int i = 0; i < 8; ++i) p[i] = squeeze3(d[i]);
        w[0] = p[0] | (p[1] << 12) | (p[2] << 24);
        w[1] = (p[2] >> 8) | (p[3] << 4) | (p[4] << 16) | (p[5] << 28);
        w[2] = (p[5] >> 4) | (p[6] << 8) | (p[7] << 20);
    }
    static __device__ inline void unpack(const uint32_t *w, uint32_t *d)
    {
        d[0] = spread3(w[0] & 0xfffu);
        d[1] = spread3((w[0] >> 12) & 0xfffu);
        d[2] = spread3(((w[0] >> 24) | (w[1] << 8)) & 0xfffu);
        d[3] = spread3((w[1] >> 4) & 0xfffu);
        d[4] = spread3((w[1] >> 16) & 0xfffu);
        d[5] = spread3(((w[1] >> 28) | (w[2] << 4)) & 0xfffu);
        d[6] = spread3((w[2] >> 8) & 0xfffu);
        d[7] = spread3(w[2] >> 20);
    }
};

// columns of the row-major side that one workgroup handles
template <int FB> constexpr int span_of() { return FB == 3 ? 512 : 256; }

// ------------------------------------------------------------------ bit-stream words
//
// v [N][cols], one FB-bit value per byte  <->  words of the bit stream of each row, stored
//   canonical:  P [word][n]                  (TILED = false)
//   per tile:   P [tile][word][lane]         (TILED = true; lanes past N hold zero words)
// `words` = words per row.  Each wavefront of the workgroup takes a quarter of the block's runs.
template <int FB, bool TILED>
__global__ __launch_bounds__(PK_THREADS) void stream_pack(const uint8_t *__restrict__ v, int64_t N,
                                                          int64_t cols, int64_t words, int spans,
                                                          bool wide, uint32_t *__restrict__ P)
{
    using R = Run<FB>;
    constexpr int SPAN = span_of<FB>(), PITCH = SPAN + 16;
    constexpr int RUNS = SPAN / R::CODES / 4;            // per wavefront
    __shared__ __align__(16) uint8_t lds[QG_WAVE * PITCH];
    const int64_t tile = blockIdx.x / spans;
    const int span = blockIdx.x % spans;
    rows_to_lds<SPAN>(v, N, cols, tile * QG_WAVE, (int64_t)span * SPAN, wide, lds);
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t n = tile * QG_WAVE + lane;
    if (!TILED && n >= N) return;
#pragma unroll
    for (int r = 0; r < RUNS; ++r) {
        const int run = wave * RUNS + r;                 // within the block
        uint32_t d[R::CODES / 4], w[R::WORDS];
        const uint4 *src = (const uint4 *)(lds + lane * PITCH + run * R::CODES);
        if constexpr (R::CODES == 8) {
            const uint2 a = *(const uint2 *)src;
            d[0] = a.x; d[1] = a.y;
        } else {
#pragma unroll
            for (int i = 0; i < R::CODES / 16; ++i) {
                const uint4 a = src[i];
                d[4 * i] = a.x; d[4 * i + 1] = a.y; d[4 * i + 2] = a.z; d[4 * i + 3] = a.w;
            }
        }
        R::pack(d, w);
#pragma unroll
        for (int j = 0; j < R::WORDS; ++j) {
            const int64_t word = ((int64_t)span * (SPAN / R::CODES) + run) * R::WORDS + j;
            if (word < words) P[TILED ? (tile * words + word) * QG_WAVE + lane : word * N + n] = w[j];
        }
    }
}

template <int FB, bool TILED>
__global__ __launch_bounds__(PK_THREADS) void stream_unpack(const uint32_t *__restrict__ P, int64_t N,
                                                            int64_t cols, int64_t words, int spans,
                                                            bool wide, uint8_t *__restrict__ v)
{
    using R = Run<FB>;
    constexpr int SPAN = span_of<FB>(), PITCH = SPAN + 16;
    constexpr int RUNS = SPAN / R::CODES / 4;
    __shared__ __align__(16) uint8_t lds[QG_WAVE * PITCH];
    const int64_t tile = blockIdx.x / spans;
    const int span = blockIdx.x % spans;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t n = tile * QG_WAVE + lane;
    if (TILED || n < N) {
#pragma unroll
        for (int r = 0; r < RUNS; ++r) {
            const int run = wave * RUNS + r;
            uint32_t d[R::CODES / 4], w[R::WORDS];
#pragma unroll
            for (int j = 0; j < R::WORDS; ++j) {
                const int64_t word = ((int64_t)span * (SPAN / R::CODES) + run) * R::WORDS + j;
                w[j] = word < words ? P[TILED ? (tile * words + word) * QG_WAVE + lane : word * N + n] : 0u;
            }
            R::unpack(w, d);
            uint4 *dst = (uint4 *)(lds + lane * PITCH + run * R::CODES);
            if constexpr (R::CODES == 8) {
                *(uint2 *)dst = make_uint2(d[0], d[1]);
            } else {
#pragma unroll
                for (int i = 0; i < R::CODES / 16; ++i)
                    dst[i] = make_uint4(d[4 * i], d[4 * i + 1], d[4 * i + 2], d[4 * i + 3]);
            }
        }
    }
    __syncthreads();
    lds_to_rows<SPAN>(v, N, cols, tile * QG_WAVE, (int64_t)span * SPAN, wide, lds);
}

// ------------------------------------------------------------------ device layout: codes

// One cell (CELL codes, one per byte in d) -> its word (2, 4 bits) or its three plane words.
template <int BITS>
__device__ inline void cell_pack(const uint32_t *d, uint32_t *w)
{
    if constexpr (BITS != 3) {
        Run<BITS>::pack(d, w);
    } else {
        const uint32_t t = d[6] | (d[7] << 3);           // codes 24+i, 28+i: the 6 spare bits of byte i
        w[0] = d[0] | (d[1] << 3) | ((t & 0x03030303u) << 6);
        w[1] = d[2] | (d[3] << 3) | (((t >> 2) & 0x03030303u) << 6);
        w[2] = d[4] | (d[5] << 3) | (((t >> 4) & 0x03030303u) << 6);
    }
}

template <int BITS>
__device__ inline void cell_unpack(const uint32_t *w, uint32_t *d)
{
    if constexpr (BITS != 3) {
        Run<BITS>::unpack(w, d);
    } else {
        constexpr uint32_t M3 = 0x07070707u, M2 = 0x03030303u;
        d[0] = w[0] & M3;  d[1] = (w[0] >> 3) & M3;
        d[2] = w[1] & M3;  d[3] = (w[1] >> 3) & M3;
        d[4] = w[2] & M3;  d[5] = (w[2] >> 3) & M3;
        const uint32_t t = ((w[0] >> 6) & M2) | (((w[1] >> 6) & M2) << 2) | (((w[2] >> 6) & M2) << 4);
        d[6] = t & M3;     d[7] = (t >> 3) & M3;
    }
}

// q [N][K] -> codes uint4 [tile][unit][plane][lane].  A workgroup takes one tile and
// 4 * UPW consecutive units; a wavefront UPW of them, lane = output.
template <int BITS>
__global__ __launch_bounds__(PK_THREADS) void device_pack_codes(const uint8_t *__restrict__ q, int64_t N,
                                                                int64_t K, int64_t units, int spans,
                                                                bool wide, uint4 *__restrict__ out)
{
    constexpr int CELL = BITS == 4 ? 8 : BITS == 2 ? 16 : 32;
    constexpr int PLANES = BITS == 3 ? 3 : 1;
    constexpr int UNIT = 4 * CELL;
    constexpr int SPAN = span_of<BITS>(), PITCH = SPAN + 16;
    constexpr int UPW = SPAN / UNIT / 4;
    __shared__ __align__(16) uint8_t lds[QG_WAVE * PITCH];
    const int64_t tile = blockIdx.x / spans;
    const int span = blockIdx.x % spans;
    rows_to_lds<SPAN>(q, N, K, tile * QG_WAVE, (int64_t)span * SPAN, wide, lds);
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int u = 0; u < UPW; ++u) {
        const int64_t unit = (int64_t)span * (4 * UPW) + wave * UPW + u;
        if (unit >= units) break;
        uint32_t words[PLANES][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t d[CELL / 4], w[PLANES];
            const uint8_t *src = lds + lane * PITCH + ((wave * UPW + u) * 4 + j) * CELL;
            if constexpr (CELL == 8) {
                const uint2 a = *(const uint2 *)src;
                d[0] = a.x; d[1] = a.y;
            } else {
#pragma unroll
                for (int i = 0; i < CELL / 16; ++i) {
                    const uint4 a = ((const uint4 *)src)[i];
                    d[4 * i] = a.x; d[4 * i + 1] = a.y; d[4 * i + 2] = a.z; d[4 * i + 3] = a.w;
                }
            }
            cell_pack<BITS>(d, w);
#pragma unroll
            for (int p = 0; p < PLANES; ++p) words[p][j] = w[p];
        }
#pragma unroll
        for (int p = 0; p < PLANES; ++p)
            out[((tile * units + unit) * PLANES + p) * QG_WAVE + lane] =
                make_uint4(words[p][0], words[p][1], words[p][2], words[p][3]);
    }
}

template <int BITS>
__global__ __launch_bounds__(PK_THREADS) void device_unpack_codes(const uint4 *__restrict__ in, int64_t N,
                                                                  int64_t K, int64_t units, int spans,
                                                                  bool wide, uint8_t *__restrict__ q)
{
    constexpr int CELL = BITS == 4 ? 8 : BITS == 2 ? 16 : 32;
    constexpr int PLANES = BITS == 3 ? 3 : 1;
    constexpr int UNIT = 4 * CELL;
    constexpr int SPAN = span_of<BITS>(), PITCH = SPAN + 16;
    constexpr int UPW = SPAN / UNIT / 4;
    __shared__ __align__(16) uint8_t lds[QG_WAVE * PITCH];
    const int64_t tile = blockIdx.x / spans;
    const int span = blockIdx.x % spans;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int u = 0; u < UPW; ++u) {
        const int64_t unit = (int64_t)span * (4 * UPW) + wave * UPW + u;
        if (unit >= units) break;                        // that part of the block lies past K
        uint32_t words[PLANES][4];
#pragma unroll
        for (int p = 0; p < PLANES; ++p) {
            const uint4 a = in[((tile * units + unit) * PLANES + p) * QG_WAVE + lane];
            words[p][0] = a.x; words[p][1] = a.y; words[p][2] = a.z; words[p][3] = a.w;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t d[CELL / 4], w[PLANES];
#pragma unroll
            for (int p = 0; p < PLANES; ++p) w[p] = words[p][j];
            cell_unpack<BITS>(w, d);
            uint8_t *dst = lds + lane * PITCH + ((wave * UPW + u) * 4 + j) * CELL;
            if constexpr (CELL == 8) {
                *(uint2 *)dst = make_uint2(d[0], d[1]);
            } else {
#pragma unroll
                for (int i = 0; i < CELL / 16; ++i)
                    ((uint4 *)dst)[i] = make_uint4(d[4 * i], d[4 * i + 1], d[4 * i + 2], d[4 * i + 3]);
            }
        }
    }
    __syncthreads();
    lds_to_rows<SPAN>(q, N, K, tile * QG_WAVE, (int64_t)span * SPAN, wide, lds);
}

// ------------------------------------------------------------------ scales
//
// s [N][G] (row-major)  <->  canonical St [G][N]  or  per tile sd [tile][G][lane] (lanes past
// N hold 0).  A workgroup moves 64 outputs x 64 groups through LDS.
template <bool TILED>
__global__ __launch_bounds__(PK_THREADS) void scales_pack(const float *__restrict__ s, int64_t N, int64_t G,
                                                          int spans, float *__restrict__ out)
{
    __shared__ float lds[QG_WAVE][QG_WAVE + 1];
    const int64_t tile = blockIdx.x / spans;
    const int64_t g0 = (int64_t)(blockIdx.x % spans) * QG_WAVE;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float val[QG_WAVE / 4];                    // all loads of the thread before the first store
#pragma unroll
    for (int j = 0; j < QG_WAVE / 4; ++j) {
        const int64_t n = tile * QG_WAVE + wave + 4 * j, g = g0 + lane;
        val[j] = (n < N && g < G) ? s[n * G + g] : 0.0f;
    }
#pragma unroll
    for (int j = 0; j < QG_WAVE / 4; ++j) lds[wave + 4 * j][lane] = val[j];
    __syncthreads();
    const int64_t n = tile * QG_WAVE + lane;
#pragma unroll
    for (int j = 0; j < QG_WAVE / 4; ++j) {
        const int c = wave + 4 * j;
        const int64_t g = g0 + c;
        if (g >= G) break;
        if (TILED) out[(tile * G + g) * QG_WAVE + lane] = lds[lane][c];
        else if (n < N) out[g * N + n] = lds[lane][c];
    }
}

template <bool TILED>
__global__ __launch_bounds__(PK_THREADS) void scales_unpack(const float *__restrict__ in, int64_t N, int64_t G,
                                                            int spans, float *__restrict__ s)
{
    __shared__ float lds[QG_WAVE][QG_WAVE + 1];
    const int64_t tile = blockIdx.x / spans;
    const int64_t g0 = (int64_t)(blockIdx.x % spans) * QG_WAVE;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t nl = tile * QG_WAVE + lane;
    float val[QG_WAVE / 4];
#pragma unroll
    for (int j = 0; j < QG_WAVE / 4; ++j) {
        const int64_t g = g0 + wave + 4 * j;
        val[j] = 0.0f;
        if (g < G && (TILED || nl < N)) val[j] = in[TILED ? (tile * G + g) * QG_WAVE + lane : g * N + nl];
    }
#pragma unroll
    for (int j = 0; j < QG_WAVE / 4; ++j) lds[lane][wave + 4 * j] = val[j];
    __syncthreads();
    for (int r = wave; r < QG_WAVE; r += 4) {
        const int64_t n = tile * QG_WAVE + r, g = g0 + lane;
        if (n < N && g < G) s[n * G + g] = lds[r][lane];
    }
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// workgroups of a launch over `tiles` x `spans` blocks, or 0 if HIP's grid cannot hold them
inline unsigned grid_for(int64_t tiles, int64_t spans)
{
    return tiles * spans > 0x7fffffff ? 0u : (unsigned)(tiles * spans);
}

// stream_pack / stream_unpack for a [N][cols] byte matrix with `fb`-bit fields
template <bool TILED>
int launch_stream(bool pack, int fb, const void *bytes, int64_t N, int64_t cols, int64_t words,
                  const void *packed, hipStream_t st)
{
    const int64_t tiles = ceil_div(N, QG_WAVE);
    const int spans = (int)ceil_div(cols, fb == 3 ? span_of<3>() : span_of<4>());
    const unsigned grid = grid_for(tiles, spans);
    if (!grid) return QG_ERR_SHAPE;
    const bool wide = cols % 16 == 0 && qg_aligned16(bytes);
    const uint8_t *vin = (const uint8_t *)bytes;
    uint8_t *vout = (uint8_t *)bytes;
    const uint32_t *pin = (const uint32_t *)packed;
    uint32_t *pout = (uint32_t *)packed;
#define QG_STREAM(FB)                                                                                   \
    if (pack) hipLaunchKernelGGL((stream_pack<FB, TILED>), dim3(grid), dim3(PK_THREADS), 0, st, vin, N, \
                                 cols, words, spans, wide, pout);                                       \
    else hipLaunchKernelGGL((stream_unpack<FB, TILED>), dim3(grid), dim3(PK_THREADS), 0, st, pin, N,    \
                            cols, words, spans, wide, vout)
    if (fb == 4) { QG_STREAM(4); }
    else if (fb == 2) { QG_STREAM(2); }
    else { QG_STREAM(3); }
#undef QG_STREAM
    return QG_OK;
}

template <bool TILED>
int launch_scales(bool pack, const float *s, int64_t N, int64_t G, const float *packed, hipStream_t st)
{
    const int spans = (int)ceil_div(G, QG_WAVE);
    const unsigned grid = grid_for(ceil_div(N, QG_WAVE), spans);
    if (!grid) return QG_ERR_SHAPE;
    if (pack) hipLaunchKernelGGL(scales_pack<TILED>, dim3(grid), dim3(PK_THREADS), 0, st, s, N, G, spans,
                                 (float *)packed);
    else hipLaunchKernelGGL(scales_unpack<TILED>, dim3(grid), dim3(PK_THREADS), 0, st, packed, N, G, spans,
                            (float *)s);
    return QG_OK;
}

int launch_device_codes(bool pack, const QgLayout &L, const void *q, const void *codes, hipStream_t st)
{
    const int span_units = (L.bits == 3 ? span_of<3>() : span_of<4>()) / L.unit;
    const int spans = (int)ceil_div(L.units, span_units);
    const unsigned grid = grid_for(L.tiles, spans);
    if (!grid) return QG_ERR_SHAPE;
    const bool wide = L.K % 16 == 0 && qg_aligned16(q);
#define QG_CODES(B)                                                                                      \
    if (pack) hipLaunchKernelGGL(device_pack_codes<B>, dim3(grid), dim3(PK_THREADS), 0, st,              \
                                 (const uint8_t *)q, L.N, L.K, L.units, spans, wide, (uint4 *)codes);    \
    else hipLaunchKernelGGL(device_unpack_codes<B>, dim3(grid), dim3(PK_THREADS), 0, st,                 \
                            (const uint4 *)codes, L.N, L.K, L.units, spans, wide, (uint8_t *)q)
    if (L.bits == 4) { QG_CODES(4); }
    else if (L.bits == 2) { QG_CODES(2); }
    else { QG_CODES(3); }
#undef QG_CODES
    return QG_OK;
}

// both directions of qg_pack / qg_unpack: the same three sections either way
int convert(bool pack, const void *q, const void *s, const void *z, int64_t N, int64_t K, int bits,
            int group, int layout, const void *packed, hipStream_t st)
{
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
        rc = launch_stream<false>(pack, bits, q, N, K, C.code_words, base + C.codes_off, st);
        if (rc == QG_OK) rc = launch_scales<false>(pack, (const float *)s, N, C.ngroups,
                                                   (const float *)(base + C.scales_off), st);
        if (rc == QG_OK) rc = launch_stream<false>(pack, bits, z, N, C.ngroups, C.zero_words,
                                                   base + C.zeros_off, st);
    } else {
        rc = launch_device_codes(pack, L, q, base + L.codes_off, st);
        if (rc == QG_OK) rc = launch_scales<true>(pack, (const float *)s, N, L.ngroups,
                                                  (const float *)(base + L.scales_off), st);
        if (rc == QG_OK) rc = launch_stream<true>(pack, L.zbits, z, N, L.ngroups, L.zwords,
                                                  base + L.zeros_off, st);
    }
    return rc == QG_OK ? qg_launch_status() : rc;
}

}  // namespace

extern "C" int qg_cell(int bits) { return qg_cell_of(bits); }

#ifndef QG_BUILD_ID
#define QG_BUILD_ID "unknown"
#endif
extern "C" const char *qg_build_id(void) { return QG_BUILD_ID; }

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

size_t qg_narrow_bytes(int64_t N, int64_t K, int bits, int group);   // qg_gemv_narrow.hip

extern "C" size_t qg_packed_bytes(int64_t N, int64_t K, int bits, int group, int layout)
{
    if (layout == QG_LAYOUT_DEVICE_NARROW) return qg_narrow_bytes(N, K, bits, group);
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
    return convert(true, q, s, z, N, K, bits, group, layout, packed, (hipStream_t)stream);
}

extern "C" int qg_unpack(const void *packed, int64_t N, int64_t K, int bits, int group,
                         int layout, uint8_t *q, float *s, uint8_t *z, void *stream)
{
    return convert(false, q, s, z, N, K, bits, group, layout, packed, (hipStream_t)stream);
}
