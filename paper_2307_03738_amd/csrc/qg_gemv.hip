// qg_gemv / qg_gemv_grouped: y = What x straight from the packed codes (eq. (2), Algorithm 1).
//
// Mapping.  One lane per output: lane l of a wavefront owns output n = 64*tile + l and reads
// its own 128-bit vectors of codes, so each wavefront load is one contiguous 1 KB piece of
// the blob.  x[k] is the same for all 64 lanes; it is read through the scalar path and used
// as a scalar operand of the fused multiply-add, so the activation costs no vector
// register, no LDS bandwidth and no cross-lane traffic.  This is the register picture of the
// paper's micro-kernel (Algorithm 3: vector accumulators over outputs, x broadcast) at
// wavefront width.
//
// Arithmetic per group g (eq. (2) with the scale kept on the zero term):
//     y_n += s_{n,g} * ( sum_{k in g} q_{n,k} x_k  -  z_{n,g} * sum_{k in g} x_k )
// The inner sum runs on raw codes: mask four byte lanes of a word at once, convert a byte
// lane to float in one instruction, one fused multiply-add per weight.  sum_k x_k per group
// is the paper's x-hat (Algorithm 1 input), computed once per wavefront with a cross-lane
// reduction and kept one group per lane.
//
// K is split over the wavefronts of a workgroup (LDS reduction in a fixed order) and, for
// tiles whose K is too long for one workgroup, over 2, 4, ... workgroups whose partial
// vectors are combined pairwise up a fixed binary tree: the two partners of a pair meet in
// one 32-bit slot by atomic exchange -- whoever arrives second finds the other's value,
// adds it (a + b = b + a, so the bits do not depend on who was second) and carries the sum
// to the next level.  The value travels inside the atomic itself, so no fence and no cache
// maintenance is needed, and results do not depend on timing.
//
// Kernels: gemv_static (groups up to one step, the arithmetic above on the vector ALU),
// gemv_runtime (groups of whole steps up to one group per output, eq. (1)), gemv_generic
// (anything else), and three forms with the multiply-adds on the matrix cores, still one lane
// per output: gemv_mma4i (4 x 4 x 4 instruction on int8, x in fixed point; the built-in choice
// wherever it applies), gemv_mma4 (the same instruction on bf16, x in three bf16 parts) and
// gemv_mma (32 x 32 x 16 on bf16).  All share the work distribution and the reductions.
#include <cstdio>
#include <mutex>

#include "qg_common.h"
#include "qg_mma.h"

namespace {

struct alignas(128) GemvProblem {
    const uint4 *codes;
    const float *scales;
    const uint32_t *zeros;
    const float *x;
    float *y;
    uint32_t *slots;       // [tile][QG_MAX_CHUNKS][64] meeting slots of the reduction tree
    int N, K, tiles, steps, ngroups, zwords;
    int group;             // G
    int chunks;            // K-split over workgroups, a power of two (1: a workgroup covers all of K)
    int chunk_shift;       // log2(chunks)
    int waves_per_tile;    // wavefronts of a workgroup that share one tile
    int inv_waves_per_tile;   // ceil(65536 / waves_per_tile): wave / wpt = (wave * inv) >> 16 for wave < 16
    int team_full;         // wavefronts of a team that have work when a workgroup covers all of K
    int tiles_per_block;   // tiles one workgroup handles (1 if chunks > 1)
    int steps_per_wave;
    int steps_per_group;   // runtime-group kernel only
    int block_begin;       // first block of this problem in the grid
    int pair_tiles;        // > 0: outputs [0, 64 pair_tiles) gate outputs [64 pair_tiles, ...), see emit_output
    float *h;              // gated result (pair_tiles > 0)
    int rows;              // gemm_rows16 only: activation rows M (x is X [M][K], y is Y [M][N])
};

// Every field of a problem entry in scalar registers at one point: the loads that fetch the
// entry from the argument buffer are then issued together and waited for once, instead of
// one miss after the other as the fields come into use.
__device__ inline void pin_problem(const GemvProblem &P)
{
    asm volatile("" ::"s"(P.codes), "s"(P.scales), "s"(P.zeros), "s"(P.x), "s"(P.y), "s"(P.slots), "s"(P.h));
    asm volatile("" ::"s"(P.N), "s"(P.K), "s"(P.tiles), "s"(P.steps), "s"(P.ngroups), "s"(P.zwords), "s"(P.group),
                 "s"(P.chunks), "s"(P.chunk_shift), "s"(P.waves_per_tile), "s"(P.inv_waves_per_tile),
                 "s"(P.team_full), "s"(P.tiles_per_block), "s"(P.steps_per_wave), "s"(P.steps_per_group),
                 "s"(P.block_begin), "s"(P.pair_tiles), "s"(P.rows));
}

#define QG_SLOT_EMPTY 0xffffffffu

// The bit pattern of a partial result as it enters a meeting slot.  The "empty" marker is itself
// a NaN pattern, and arithmetic passes a NaN operand's payload through, so an x holding exactly
// that pattern could hand it to a sum; such a sum is entered as the default quiet NaN instead
// (still a NaN, so it reaches y as one).
__device__ inline uint32_t slot_bits(float v)
{
    const uint32_t b = __float_as_uint(v);
    return b == QG_SLOT_EMPTY ? 0x7fc00000u : b;
}

struct GemvArgs {
    int count;
    int block_begin[QG_MAX_GROUPED];   // first block of problem i; INT_MAX beyond `count`
    GemvProblem p[QG_MAX_GROUPED];
};

// Keeps a masked word opaque to the optimiser so that the byte-lane conversions below stay
// "convert byte i of this register" instead of being rewritten as shift-and-mask per code.
__device__ inline uint32_t opaque(uint32_t v)
{
    asm("" : "+v"(v));
    return v;
}

// Four byte lanes of m times four x values.  Byte i of m is one code.
#define QG_B0(m) ((float)((m) & 0xffu))
#define QG_B1(m) ((float)(((m) >> 8) & 0xffu))
#define QG_B2(m) ((float)(((m) >> 16) & 0xffu))
#define QG_B3(m) ((float)((m) >> 24))

// 32 consecutive x values held in scalar registers (x is uniform across the wavefront).
typedef float xvec16 __attribute__((ext_vector_type(16)));
struct XBatch {
    xvec16 lo, hi;
    __device__ inline float operator[](int i) const { return i < 16 ? lo[i] : hi[i - 16]; }
};
// x is read-only for the whole launch, so it is read through the constant address space: that
// keeps these loads on the scalar path whatever else the kernel does.
typedef __attribute__((address_space(4))) const xvec16 *ConstX16;
__device__ inline XBatch load_x32(const float *__restrict__ p)
{
    const ConstX16 cp = (ConstX16)(unsigned long long)p;
    XBatch b;
    b.lo = cp[0];
    b.hi = cp[1];
    return b;
}

// Scalar loads return out of order, so the only wait the hardware offers is "all of them".
// To overlap the load of the next batch with the arithmetic on the current one, the first
// use of the current batch has to come BEFORE the next load is issued.  The loops below
// therefore run one octet of the batch, then issue the next load, then run the other three,
// with scheduling fences so that this order survives instruction scheduling.
#define QG_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// Octet `o` (0..3) of batch `bt` of a step: eight codes times eight of the 32 x values in xb.
// 4 bits: an octet is a cell (one word; code i in bits [4i, 4i+4), Algorithm 2).
// 2 bits: a cell (one word, code i in bits [2i, 2i+2)) is two octets; field set f holds
//         codes f, 4+f, 8+f, 12+f, and an octet takes two field sets.
// 3 bits: a cell (words A, B, C, layout in qg_common.h) is four octets, one per source word
//         A, B, C and the word T gathered from the spare bits.
// Two independent accumulation chains per wavefront: a single dependent chain of FMAs can only
// issue every ~5 cycles, two chains keep the SIMD busy with fewer resident wavefronts.  The
// two halves are added once per group.  The second chain takes the upper field of every byte
// WITHOUT shifting it down (one mask instead of shift and mask): its codes count 2^BITS times
// too much, which acc_total undoes -- powers of two, so every bit of the result is the same.
struct Acc2 {
    float a, b;
};

template <int BITS>
__device__ inline float acc_total(const Acc2 &acc)
{
    return fmaf(acc.b, 1.0f / (float)(1 << BITS), acc.a);
}

template <int BITS>
__device__ inline void octet_dot(const uint4 *v, int bt, int o, const XBatch &xb, Acc2 &acc)
{
    if constexpr (BITS == 4) {
        const int cell = bt * 4 + o;
        const uint32_t w = word_of(v[cell >> 2], cell & 3);
        const uint32_t lo = opaque(w & 0x0f0f0f0fu);          // even codes
        const uint32_t hi = opaque(w & 0xf0f0f0f0u);          // odd codes, times 16
        const int x0 = 8 * o;
        acc.a = fmaf(QG_B0(lo), xb[x0 + 0], acc.a);  acc.b = fmaf(QG_B0(hi), xb[x0 + 1], acc.b);
        acc.a = fmaf(QG_B1(lo), xb[x0 + 2], acc.a);  acc.b = fmaf(QG_B1(hi), xb[x0 + 3], acc.b);
        acc.a = fmaf(QG_B2(lo), xb[x0 + 4], acc.a);  acc.b = fmaf(QG_B2(hi), xb[x0 + 5], acc.b);
        acc.a = fmaf(QG_B3(lo), xb[x0 + 6], acc.a);  acc.b = fmaf(QG_B3(hi), xb[x0 + 7], acc.b);
    } else if constexpr (BITS == 2) {
        const int cell = bt * 2 + (o >> 1);
        const uint32_t w = word_of(v[cell >> 2], cell & 3);
        const int x0 = 16 * (o >> 1);
        const int f = 2 * (o & 1);
        const uint32_t m0 = opaque((w >> (2 * f)) & 0x03030303u);
        const uint32_t m1 = opaque((w >> (2 * f)) & 0x0c0c0c0cu);      // the next field set, times 4
        acc.a = fmaf(QG_B0(m0), xb[x0 + f], acc.a);       acc.b = fmaf(QG_B0(m1), xb[x0 + f + 1], acc.b);
        acc.a = fmaf(QG_B1(m0), xb[x0 + 4 + f], acc.a);   acc.b = fmaf(QG_B1(m1), xb[x0 + 4 + f + 1], acc.b);
        acc.a = fmaf(QG_B2(m0), xb[x0 + 8 + f], acc.a);   acc.b = fmaf(QG_B2(m1), xb[x0 + 8 + f + 1], acc.b);
        acc.a = fmaf(QG_B3(m0), xb[x0 + 12 + f], acc.a);  acc.b = fmaf(QG_B3(m1), xb[x0 + 12 + f + 1], acc.b);
    } else {
        const int cell = bt;
        const int u = cell >> 2, j = cell & 3;
        uint32_t src;
        if (o < 3) {
            src = word_of(v[u * 3 + o], j);
        } else {
            const uint32_t a = word_of(v[u * 3 + 0], j);
            const uint32_t b = word_of(v[u * 3 + 1], j);
            const uint32_t c = word_of(v[u * 3 + 2], j);
            src = ((a >> 6) & 0x03030303u) | ((b >> 4) & 0x0c0c0c0cu) | ((c >> 2) & 0x30303030u);
        }
        const uint32_t m0 = opaque(src & 0x07070707u);
        const uint32_t m1 = opaque(src & 0x38383838u);                 // the upper codes, times 8
        const int x0 = 8 * o;
        acc.a = fmaf(QG_B0(m0), xb[x0 + 0], acc.a);  acc.b = fmaf(QG_B0(m1), xb[x0 + 4], acc.b);
        acc.a = fmaf(QG_B1(m0), xb[x0 + 1], acc.a);  acc.b = fmaf(QG_B1(m1), xb[x0 + 5], acc.b);
        acc.a = fmaf(QG_B2(m0), xb[x0 + 2], acc.a);  acc.b = fmaf(QG_B2(m1), xb[x0 + 6], acc.b);
        acc.a = fmaf(QG_B3(m0), xb[x0 + 3], acc.a);  acc.b = fmaf(QG_B3(m1), xb[x0 + 7], acc.b);
    }
}

// ---- cross-lane sums on the DPP path (no LDS, no memory) ------------------------------
// v + (v moved across lanes by the DPP control CTRL); rows that ROW_MASK disables add 0.
template <int CTRL, int ROW_MASK = 0xf>
__device__ inline float dpp_add(float v)
{
    const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false);
    return v + __int_as_float(moved);
}
#define QG_DPP_QUAD_XOR1 0xB1      // quad_perm [1,0,3,2]
#define QG_DPP_QUAD_XOR2 0x4E      // quad_perm [2,3,0,1]
#define QG_DPP_HALF_MIRROR 0x141   // lane i <-> 7-i inside each 8 lanes
#define QG_DPP_ROW_MIRROR 0x140    // lane i <-> 15-i inside each row of 16 lanes
#define QG_DPP_BCAST15 0x142       // lane 15 of each row to the next row
#define QG_DPP_BCAST31 0x143       // lane 31 to rows 2 and 3

__device__ inline float uniform_lane(float v, int lane)     // lane is a compile-time constant
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// Sums of consecutive segments of SEG lanes (SEG = 4, 8, 16, 32 or 64) of v, returned as
// wavefront-uniform values out[0 .. 64/SEG).  This is x-hat of Algorithm 1 for one group
// when lane l holds x[k0 + l].
template <int SEG>
__device__ inline void segment_sums(float v, float *out)
{
    v = dpp_add<QG_DPP_QUAD_XOR1>(v);
    v = dpp_add<QG_DPP_QUAD_XOR2>(v);                        // every 4 lanes hold their sum
    if constexpr (SEG == 4) {
#pragma unroll
        for (int i = 0; i < 16; ++i) out[i] = uniform_lane(v, 4 * i);
        return;
    }
    v = dpp_add<QG_DPP_HALF_MIRROR>(v);                      // every 8 lanes hold their sum
    if constexpr (SEG == 8) {
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = uniform_lane(v, 8 * i);
        return;
    }
    v = dpp_add<QG_DPP_ROW_MIRROR>(v);                       // every row of 16 holds its sum
    if constexpr (SEG == 16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) out[i] = uniform_lane(v, 16 * i + 15);
        return;
    }
    v = dpp_add<QG_DPP_BCAST15, 0xa>(v);                     // rows 1 and 3 += previous row
    if constexpr (SEG == 32) {
        out[0] = uniform_lane(v, 31);
        out[1] = uniform_lane(v, 63);
        return;
    }
    v = dpp_add<QG_DPP_BCAST31, 0xc>(v);                     // row 3 += rows 0 and 1
    out[0] = uniform_lane(v, 63);
}

// What one wavefront does.  A workgroup is a pool of wavefronts; `waves_per_tile` of them
// share one tile of 64 outputs, each taking `steps_per_wave` consecutive items along K, and
// a workgroup holds `tiles_per_block` such teams (tiles with a short K pack several teams
// into a workgroup, tiles with a long K use all of it, so every wavefront of a launch has
// about the same amount of work).  With chunks > 1 a tile's K is also cut over workgroups.
struct WaveJob {
    int tile, chunk;
    int item0, item1;   // range along K (steps, or groups in the generic kernel)
    int lead;           // wavefront of the block that leads this tile's team
    int team;           // wavefronts of the team that have work
    bool work;
};

__device__ inline WaveJob locate(const GemvProblem &P, int local_block, int items, int wave)
{
    WaveJob j;
    const int wpt = P.waves_per_tile, spw = P.steps_per_wave;
    const int slot = (wave * P.inv_waves_per_tile) >> 16;     // wave / wpt without a division
    const int sub = wave - slot * wpt;
    int first = 0;
    if (P.chunks > 1) {                                       // K also split over workgroups
        j.tile = local_block >> P.chunk_shift;
        j.chunk = local_block - (j.tile << P.chunk_shift);
        first = j.chunk * wpt * spw;
        const int left = (items - first + spw - 1) / spw;
        j.team = left < wpt ? left : wpt;
    } else {
        j.tile = local_block * P.tiles_per_block + slot;
        j.chunk = 0;
        j.team = P.team_full;
    }
    j.item0 = first + sub * spw;
    j.item1 = j.item0 + spw < items ? j.item0 + spw : items;
    j.lead = slot * wpt;
    j.work = slot < P.tiles_per_block && j.tile < P.tiles && j.item0 < j.item1;
    return j;
}

// Where a finished output goes.  Plain product: y[n].  Gated pair (the MLP of a LLaMA block:
// the packed matrix holds the "gate" projection in its first 64 * pair_tiles outputs and the
// "up" projection in the rest, same x): tile t and tile t + pair_tiles meet in one slot per
// lane exactly like two partners of the reduction tree, and the second to arrive writes
// h = silu(gate) * up -- the elementwise step that follows the two products, without a launch.
__device__ inline void emit_output(const GemvProblem &P, int tile, int lane, float v)
{
    if (P.pair_tiles == 0) {
        const int n = tile * QG_WAVE + lane;
        if (n < P.N) P.y[n] = v;
        return;
    }
    const bool is_up = tile >= P.pair_tiles;
    const int t = is_up ? tile - P.pair_tiles : tile;
    // the pair slots follow the tree slots of all tiles
    uint32_t *slot = P.slots + (size_t)P.tiles * QG_MAX_CHUNKS * QG_WAVE + (size_t)t * QG_WAVE + lane;
    const uint32_t other = __hip_atomic_exchange(slot, slot_bits(v), __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
    if (other == QG_SLOT_EMPTY) return;
    __hip_atomic_store(slot, QG_SLOT_EMPTY, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const float g = is_up ? __uint_as_float(other) : v;
    const float u = is_up ? v : __uint_as_float(other);
    P.h[t * QG_WAVE + lane] = g / (1.0f + expf(-g)) * u;
}

// K-split epilogue.  The wavefronts of a team pass their 64 partial outputs through LDS
// (wavefronts without work have already ended; a barrier only waits for wavefronts that are
// still alive); the team's lead adds them in wavefront order and either stores y or enters
// the tile's reduction tree.  An empty slot holds a NaN pattern no partial sum enters it with (slot_bits).
__device__ inline void finish_tile(const GemvProblem &P, const WaveJob &j, float yacc,
                                   float (*red)[QG_WAVE])
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    red[wave][lane] = yacc;
    __syncthreads();
    if (wave != j.lead) return;
    float t = red[j.lead][lane];
    for (int w = 1; w < j.team; ++w) t += red[j.lead + w][lane];
    const int tile = j.tile, chunk = j.chunk;
    if (P.chunks == 1) {
        emit_output(P, tile, lane, t);
        return;
    }
    // pairwise reduction tree over the chunks of this tile, one independent tree per lane
    uint32_t *slots = P.slots + (size_t)tile * QG_MAX_CHUNKS * QG_WAVE + lane;
    int node = chunk, width = P.chunks, base = 0;
    float v = t;
    while (width > 1) {
        uint32_t *slot = slots + (size_t)(base + (node >> 1)) * QG_WAVE;
        const uint32_t other = __hip_atomic_exchange(slot, slot_bits(v), __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT);
        if (other == QG_SLOT_EMPTY) return;               // first of the pair: the partner carries on
        v += __uint_as_float(other);
        __hip_atomic_store(slot, QG_SLOT_EMPTY, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        base += width >> 1;
        width >>= 1;
        node >>= 1;
    }
    emit_output(P, tile, lane, v);
}

// The first blocks of problems 1 ... 12 once more, as twelve leading scalar kernel arguments:
// those are handed to a wavefront in registers when it starts (kernel-argument preload), so
// the search below does not begin with a load from the argument buffer, and the load of the
// problem's own entry is the only one in front of the first loads of weights.
typedef int qg_v4i __attribute__((ext_vector_type(4)));
struct FirstBlocks {
    qg_v4i a, b, c;        // block_begin[1 .. 12]
};
#define QG_FIRST_BLOCKS const qg_v4i fb_a, const qg_v4i fb_b, const qg_v4i fb_c

// Index of the problem a block belongs to: the last one whose first block is <= bid.
__device__ inline int find_problem(const qg_v4i fa, const qg_v4i fb, const qg_v4i fc, const GemvArgs &A, int bid)
{
    const int first[12] = {fa.x, fa.y, fa.z, fa.w, fb.x, fb.y, fb.z, fb.w, fc.x, fc.y, fc.z, fc.w};
    int p = 0;
#pragma unroll
    for (int i = 0; i < 12; ++i)
        if (bid >= first[i]) p = i + 1;
    if (first[11] != 0x7fffffff) {              // more than 12 problems: the rest from the buffer
#pragma unroll
        for (int i = 13; i < QG_MAX_GROUPED; ++i)
            if (bid >= A.block_begin[i]) p = i;
    }
    return p;
}

// What one wavefront fetches for one step: the codes, the scale and zero word(s) of the
// step's groups (GPS = 0: groups span steps, metadata is fetched per group instead) and the
// step's x values once more, one per lane, for the group sums.
template <int BITS, int GPS>
struct StepData {
    static constexpr int L = loads_per_step<BITS>();
    static constexpr int NXV = codes_per_step<BITS>() / 128;   // lane l holds x[128 i + 2l], x[128 i + 2l + 1]
    static constexpr int ZPER = 32 / Fmt<BITS>::ZBITS;
    static constexpr int ZW = GPS > ZPER ? GPS / ZPER : 1;
    uint4 v[L];
    float2 xv[NXV];
    float s[GPS > 0 ? GPS : 1];
    uint32_t zw[ZW];
};

struct TileView {            // per-lane base pointers of one tile of one problem
    const uint4 *codes;
    const float *scales;
    const uint32_t *zeros;
    const float *x;
};

template <int BITS, int GPS>
__device__ inline void fetch_step(StepData<BITS, GPS> &d, const TileView &T, int step, int lane)
{
    using D = StepData<BITS, GPS>;
    // Loads complete in order.  At 2 and 3 bits x (needed first, for the group sums) and the
    // small metadata go ahead of the codes, so that the arithmetic can start on the first code
    // vector while the others are still on their way; at 4 bits, where memory is the limit, the
    // codes go first (measured: 3 % either way).
    constexpr bool CODES_FIRST = BITS == 4;
    if constexpr (CODES_FIRST) {
#pragma unroll
        for (int i = 0; i < D::L; ++i) d.v[i] = T.codes[((size_t)step * D::L + i) * QG_WAVE];
    }
#pragma unroll
    for (int i = 0; i < D::NXV; ++i)
        d.xv[i] = *(const float2 *)(T.x + (size_t)step * codes_per_step<BITS>() + i * 128 + 2 * lane);
    if constexpr (GPS > 0) {
#pragma unroll
        for (int g = 0; g < GPS; ++g) d.s[g] = T.scales[(size_t)(step * GPS + g) * QG_WAVE];
#pragma unroll
        for (int w = 0; w < D::ZW; ++w) d.zw[w] = T.zeros[(size_t)((step * GPS) / D::ZPER + w) * QG_WAVE];
    }
    if constexpr (!CODES_FIRST) {
#pragma unroll
        for (int i = 0; i < D::L; ++i) d.v[i] = T.codes[((size_t)step * D::L + i) * QG_WAVE];
    }
}

// The arithmetic of one step on data that has arrived.  xb holds the first 32 x values of
// the step on entry and the 32 values at `xs_next` on exit (the start of the next step; for
// the last step of a wavefront the caller passes an address that is valid to read again).
// GPS > 0: the step's groups are closed here (yacc updated).  GPS == 0: acc and xacc carry
// the running group across steps.
template <int BITS, int GPS>
__device__ inline void compute_step(const StepData<BITS, GPS> &d, const float *__restrict__ xs,
                                    const float *__restrict__ xs_next, XBatch &xb, int step,
                                    bool valid, Acc2 &acc, float &xacc, float &yacc)
{
    using F = Fmt<BITS>;
    using D = StepData<BITS, GPS>;
    constexpr int S = codes_per_step<BITS>();
    constexpr int NB = S / 32;

    // x-hat of the step's groups (Algorithm 1's sum of x, per group)
    float xhat[GPS > 0 ? GPS : 1];
    if constexpr (GPS == 0) {
#pragma unroll
        for (int i = 0; i < D::NXV; ++i) xacc += d.xv[i].x + d.xv[i].y;
    } else {
        constexpr int G = S / GPS;
        if constexpr (G >= 128) {
#pragma unroll
            for (int g = 0; g < GPS; ++g) {
                float v = 0.0f;
#pragma unroll
                for (int i = 0; i < G / 128; ++i) v += d.xv[g * (G / 128) + i].x + d.xv[g * (G / 128) + i].y;
                segment_sums<64>(v, &xhat[g]);
            }
        } else {
            // a group of G codes sits in G/2 neighbouring lanes
#pragma unroll
            for (int i = 0; i < D::NXV; ++i) segment_sums<G / 2>(d.xv[i].x + d.xv[i].y, &xhat[i * (128 / G)]);
        }
    }

#pragma unroll
    for (int bt = 0; bt < NB; ++bt) {
        XBatch xn = xb;
#pragma unroll
        for (int o = 0; o < 4; ++o) {
            if (o == 0) QG_SCHED_FENCE();
            octet_dot<BITS>(d.v, bt, o, xb, acc);
            if (o == 0) {
                QG_SCHED_FENCE();
                // next batch in flight (it may belong to the next step)
                xn = load_x32(bt + 1 < NB ? xs + 32 * (bt + 1) : xs_next);
                QG_SCHED_FENCE();
            }
            if constexpr (GPS > 0) {
                constexpr int G = S / GPS;
                const int done = (bt * 4 + o + 1) * 8;            // codes of the step done so far
                if (done % G == 0) {
                    const int gs = done / G - 1;                  // group within the step
                    const int gabs = step * GPS + gs;
                    const uint32_t zword = d.zw[D::ZW > 1 ? gs / D::ZPER : 0];
                    const float zf = (float)((zword >> (F::ZBITS * (gabs % D::ZPER))) & ((1u << F::ZBITS) - 1u));
                    // a step past the end of the wavefront's range counts with scale 0
                    yacc = fmaf(valid ? d.s[gs] : 0.0f, fmaf(-zf, xhat[gs], acc_total<BITS>(acc)), yacc);
                    acc.a = 0.0f;
                    acc.b = 0.0f;
                }
            }
        }
        xb = xn;
    }
}

// ---------------------------------------------------------------------------------------
// Groups no larger than a step: CPG cells per group, GPS = groups per step, all static.
// ---------------------------------------------------------------------------------------
template <int BITS, int CPG>
__global__ __launch_bounds__(1024) void gemv_static(QG_FIRST_BLOCKS, const GemvArgs A)
{
    constexpr int L = loads_per_step<BITS>();
    constexpr int S = codes_per_step<BITS>();
    constexpr int GPS = cells_per_step<BITS>() / CPG;
    __shared__ float red[16][QG_WAVE];

    const int pi = find_problem(fb_a, fb_b, fb_c, A, blockIdx.x);
    const GemvProblem P = A.p[pi];                 // one copy: all fields fetched at once
    pin_problem(P);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const WaveJob job = locate(P, blockIdx.x - P.block_begin, P.steps, wave);
    if (!job.work) return;                      // no work: leave before the barrier
    const int tile = job.tile, s0 = job.item0, s1 = job.item1;

    TileView T;
    T.codes = P.codes + (size_t)tile * P.steps * L * QG_WAVE + lane;
    T.scales = P.scales + (size_t)tile * P.ngroups * QG_WAVE + lane;
    T.zeros = P.zeros + (size_t)tile * P.zwords * QG_WAVE + lane;
    T.x = P.x;
    const float *__restrict__ x = P.x;

    // Two buffers used alternately: the next step is in flight while this one is computed.
    // A fetch past the wavefront's range repeats its last step (no branch around the loads).
    const int last = s1 - 1;
    StepData<BITS, GPS> da, db;
    fetch_step(da, T, s0, lane);
    XBatch xb = load_x32(x + (size_t)s0 * S);
    float yacc = 0.0f, xacc = 0.0f;
    Acc2 acc = {0.0f, 0.0f};
    for (int s = s0; s < s1; s += 2) {
        const int sb = s + 1 < last ? s + 1 : last;
        const int sc = s + 2 < last ? s + 2 : last;
        fetch_step(db, T, sb, lane);
        compute_step(da, x + (size_t)s * S, x + (size_t)sb * S, xb, s, true, acc, xacc, yacc);
        if (s + 1 >= s1) break;                       // odd number of steps
        fetch_step(da, T, sc, lane);
        compute_step(db, x + (size_t)sb * S, x + (size_t)sc * S, xb, sb, true, acc, xacc, yacc);
    }
    finish_tile(P, job, yacc, red);
}

// ---------------------------------------------------------------------------------------
// The same product with the multiply-adds on the matrix cores.
//
// The 2- and 3-bit kernels above are bound by vector-ALU issue (mask, convert and multiply-add
// are three instructions per code), not by memory.  Here a code costs about one vector
// instruction: two codes are masked into the mantissas of two bf16 numbers 128 + q with one
// shift and one and-or (0x4300 is 128.0 in bf16, and 128 + q needs 8 significant bits), and
// v_mfma_f32_32x32x16_bf16 multiplies 32 outputs x 16 k of them with x and accumulates in fp32.
// x stays exact: every fp32 value is the sum of three bf16 numbers (8 + 8 + 8 significant bits),
// which occupy three rows of the instruction's A operand; the other 29 rows are zero.  The
// products are exact in fp32, the sums are fp32, and per group
//     y_n += s (T - (128 + z) xhat),   T = sum_k x_k (128 + q_k)
// which is eq. (2) again with the offset of the code folded into the zero-point.
//
// Data movement.  A wavefront still owns 64 outputs, one per lane.  The matrix instruction
// wants lanes l and l + 32 to hold two different k-octets of the SAME output, so two
// neighbouring cells of a lane (c, c + 1) are exchanged between the wavefront's halves with
// v_permlane32_swap: afterwards lanes 0-31 hold cell c and lanes 32-63 cell c + 1 of outputs
// 0-31 (P), and likewise for outputs 32-63 (Q).  The wavefront keeps its x values of the step
// in LDS, split into the three parts and stored in the order the unpacked codes have inside
// an operand; each wavefront has its own region (no barriers), double-buffered over steps.
// ---------------------------------------------------------------------------------------
// x-hat of the groups of a step from the per-lane x values (Algorithm 1's sum of x)
template <int BITS, int GPS>
__device__ inline void step_group_sums(const StepData<BITS, GPS> &d, float *xhat, float w0 = 1.0f, float w1 = 1.0f)
{
    using D = StepData<BITS, GPS>;
    constexpr int G = codes_per_step<BITS>() / GPS;
    if constexpr (G >= 128) {
#pragma unroll
        for (int g = 0; g < GPS; ++g) {
            float v = 0.0f;
#pragma unroll
            for (int i = 0; i < G / 128; ++i) v += d.xv[g * (G / 128) + i].x * w0 + d.xv[g * (G / 128) + i].y * w1;
            segment_sums<64>(v, &xhat[g]);
        }
    } else {
#pragma unroll
        for (int i = 0; i < D::NXV; ++i)
            segment_sums<G / 2>(d.xv[i].x * w0 + d.xv[i].y * w1, &xhat[i * (128 / G)]);
    }
}

template <int BITS, int CPG>
__global__ __launch_bounds__(512) void gemv_mma(QG_FIRST_BLOCKS, const GemvArgs A)
{
    using F = Fmt<BITS>;
    constexpr int L = loads_per_step<BITS>();
    constexpr int S = codes_per_step<BITS>();
    constexpr int CELLS = cells_per_step<BITS>();
    constexpr int GPS = CELLS / CPG;
    constexpr int OPS = mma_ops<BITS>();
    constexpr int NXV = S / 128;
    using D = StepData<BITS, GPS>;
    static_assert(CPG >= 2 && CPG % 2 == 0, "a group must hold whole pairs of cells");
    __shared__ float red[16][QG_WAVE];
    // one block of zeros for the unused rows of the A operand, shared by everybody; per
    // wavefront and buffer three parts of x in operand order (dynamic: sized by the launch for
    // the wavefronts a workgroup really has, so that more workgroups fit a compute unit)
    __shared__ __attribute__((aligned(16))) lds_u16 zeros[S];
    extern __shared__ __attribute__((aligned(16))) lds_u16 xs_raw[];
    lds_u16(*xs)[2][3][S] = (lds_u16(*)[2][3][S])xs_raw;

    const int pi = find_problem(fb_a, fb_b, fb_c, A, blockIdx.x);
    const GemvProblem P = A.p[pi];
    pin_problem(P);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const WaveJob job = locate(P, blockIdx.x - P.block_begin, P.steps, wave);
    if (!job.work) return;                      // no work: leave before the barrier
    const int tile = job.tile, s0 = job.item0, s1 = job.item1;

    TileView T;
    T.codes = P.codes + (size_t)tile * P.steps * L * QG_WAVE + lane;
    T.scales = P.scales + (size_t)tile * P.ngroups * QG_WAVE + lane;
    T.zeros = P.zeros + (size_t)tile * P.zwords * QG_WAVE + lane;
    T.x = P.x;

    // every wavefront clears the zero block itself before it reads it (same values from all)
#pragma unroll
    for (int i = lane; i < S; i += QG_WAVE) zeros[i] = 0;

    // where this lane's x values go: x[128 i + 2 lane + e] of the step is code (k % CELL) of
    // cell k / CELL; cells pair up as (2 cp, 2 cp + 1) = the two halves of an operand
    int xpos[NXV][2];
#pragma unroll
    for (int i = 0; i < NXV; ++i)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int k = 128 * i + 2 * lane + e;
            const int cell = k / F::CELL, slot = mma_slot<BITS>(k % F::CELL);
            xpos[i][e] = (((cell >> 1) * OPS + (slot >> 3)) * 2 + (cell & 1)) * 8 + (slot & 7);
        }
    // A operand: row = lane % 32 (rows 0-2 = the parts of x, the others zero), half = lane / 32
    const int row = lane & 31, half = lane >> 5;
    const lds_u16 *abase[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) abase[b] = row < 3 ? &xs[wave][b][row][half * 8] : &zeros[half * 8];

    // 3 bits: this lane's two x values meet codes taken three bits up (8 q) if k % 8 >= 4,
    // i.e. lane % 4 >= 2; they are stored divided by 8 (exact) and summed apart for x-hat
    const bool up_class = BITS == 3 && (lane & 2);
    const float xscale = up_class ? 0.125f : 1.0f;
    // splits the step's x values into three bf16 parts and stores them for the A operands
    auto stage_x = [&](const D &d, int buf) {
#pragma unroll
        for (int i = 0; i < NXV; ++i) {
            mma_floatx2 r = {d.xv[i].x * xscale, d.xv[i].y * xscale};
#pragma unroll
            for (int part = 0; part < 3; ++part) {
                const mma_bf16x2 h = __builtin_convertvector(r, mma_bf16x2);     // round to nearest even
                const uint32_t bits = *(const uint32_t *)&h;
                xs[wave][buf][part][xpos[i][0]] = (uint16_t)bits;
                xs[wave][buf][part][xpos[i][1]] = (uint16_t)(bits >> 16);
                r[0] -= __uint_as_float(bits << 16);                             // exact
                r[1] -= __uint_as_float(bits & 0xffff0000u);
            }
        }
    };

    const MmaConst mc = mma_constants<BITS>();
    float yacc = 0.0f;

    auto compute = [&](const D &d, int step, int buf) {
        // x-hat of the step's groups; at 3 bits apart for the codes read as 128 + q (xhat) and
        // as 128 + 8 q (xhat_up)
        float xhat[GPS], xhat_up[GPS];
        if constexpr (BITS == 3) {
            step_group_sums<BITS, GPS>(d, xhat, up_class ? 0.0f : 1.0f, up_class ? 0.0f : 1.0f);
            step_group_sums<BITS, GPS>(d, xhat_up, up_class ? 1.0f : 0.0f, up_class ? 1.0f : 0.0f);
        } else {
            step_group_sums<BITS, GPS>(d, xhat);
        }
        mma_floatx16 accP, accQ;
#pragma unroll
        for (int i = 0; i < 16; ++i) { accP[i] = 0.0f; accQ[i] = 0.0f; }
#pragma unroll
        for (int cp = 0; cp < CELLS / 2; ++cp) {
            // words of cells 2 cp and 2 cp + 1, exchanged between the halves
            uint32_t wp[F::PLANES], wq[F::PLANES];
            const int c0 = 2 * cp, u = c0 >> 2, j = c0 & 3;
#pragma unroll
            for (int pl = 0; pl < F::PLANES; ++pl) {
                const auto sw = __builtin_amdgcn_permlane32_swap(word_of(d.v[u * F::PLANES + pl], j),
                                                                 word_of(d.v[u * F::PLANES + pl], j + 1), false, false);
                wp[pl] = sw[0];       // outputs 0-31: cell 2 cp in lanes 0-31, cell 2 cp + 1 in lanes 32-63
                wq[pl] = sw[1];       // outputs 32-63
            }
            MmaOperand bp[OPS], bq[OPS];
            mma_unpack<BITS>(wp, mc, bp);
            mma_unpack<BITS>(wq, mc, bq);
#pragma unroll
            for (int op = 0; op < OPS; ++op) {
                MmaOperand a;
                a.q = *(const lds_u128 *)(abase[buf] + (cp * OPS + op) * 16);
                accP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, bp[op].v, accP, 0, 0, 0);
                accQ = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, bq[op].v, accQ, 0, 0, 0);
            }
            if ((2 * cp + 2) % CPG == 0) {
                // a group is complete: rows 0-2 of the result (lanes 0-31) are the three parts
                const int gs = (2 * cp + 2) / CPG - 1;
                const int gabs = step * GPS + gs;
                const float tp = accP[0] + accP[1] + accP[2], tq = accQ[0] + accQ[1] + accQ[2];
                const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(tp), __float_as_uint(tq), false, false);
                const float tsum = __uint_as_float(sw[0]);           // lane l: output l of the tile
                const uint32_t zword = d.zw[D::ZW > 1 ? gs / D::ZPER : 0];
                const uint32_t zq = (zword >> (F::ZBITS * (gabs % D::ZPER))) & ((1u << F::ZBITS) - 1u);
                float tz = fmaf(-(float)(zq + 128u), xhat[gs], tsum);
                if constexpr (BITS == 3) tz = fmaf(-(float)(zq + 16u), xhat_up[gs], tz);
                yacc = fmaf(d.s[gs], tz, yacc);
#pragma unroll
                for (int i = 0; i < 16; ++i) { accP[i] = 0.0f; accQ[i] = 0.0f; }
            }
        }
    };

    // two register buffers and two LDS buffers used alternately, as in gemv_static
    const int last = s1 - 1;
    D da, db;
    fetch_step(da, T, s0, lane);
    stage_x(da, 0);
    for (int s = s0; s < s1; s += 2) {
        const int sb = s + 1 < last ? s + 1 : last;
        const int sc = s + 2 < last ? s + 2 : last;
        fetch_step(db, T, sb, lane);
        compute(da, s, 0);
        if (s + 1 >= s1) break;                       // odd number of steps
        stage_x(db, 1);
        fetch_step(da, T, sc, lane);
        compute(db, sb, 1);
        stage_x(da, 0);
    }
    finish_tile(P, job, yacc, red);
}

// ---------------------------------------------------------------------------------------
// The matrix-core GEMV on v_mfma_f32_4x4x4_16B_bf16: 16 independent 4 x 4 x 4 products per
// instruction, one per group of four lanes.  Lane l supplies the B column of ITS OWN output
// (four consecutive operand elements = four codes 128 + q), the A rows of a block are the
// three bf16 parts of the four x values those codes meet (row 3 is zero; lane l supplies row
// l % 4, the same in every block), and lane l receives its output's three partial sums in
// registers 0-2 of the result.  Compared with gemv_mma (32 x 32 x 16): nothing is exchanged
// between lanes, the accumulator is 4 registers instead of 32, and 64 outputs x 256 k take
// 64 instructions of 8 cycles instead of 32 of 32 cycles.  The unpacking (mma_unpack) and
// the exactness argument are the same; so is the 3-bit in-place high field.
//
// CPG > 0: groups of CPG cells inside a step (closed at compile-time positions).
// CPG == 0: groups of whole steps (G = 256 ... K).  The accumulators run across steps, and a
// group -- or the piece of it inside this wavefront's range, since s (sum q x - z sum x) is
// linear in the two sums -- is closed when it ends; no per-step group work is left.
// ---------------------------------------------------------------------------------------
typedef short mma4_ab __attribute__((ext_vector_type(4)));
typedef float mma4_acc __attribute__((ext_vector_type(4)));
typedef uint2 __attribute__((may_alias)) lds_u64;

// Position (operand of the cell, element) of code c of a cell: operand o of a cell is the
// register pair (2 o, 2 o + 1) of mma_unpack's output; returns 4 * operand + element.
template <int BITS>
__device__ inline int mma4_slot(int c)
{
    if constexpr (BITS == 3) {
        const int w = c >> 3, r = c & 7;            // word (A, B, C, T), code within it
        return (2 * w + (r & 1)) * 4 + (r >> 1);
    } else {
        constexpr int HALF = BITS == 2 ? 8 : 4;     // register j holds codes j and j + HALF
        const int j = c % HALF, hi = c / HALF;
        return (j >> 1) * 4 + (j & 1) * 2 + hi;
    }
}

// Fields taken where they stand.  A field that sits f bits up in the mantissa makes the
// element 128 + 2^f q instead of 128 + q, still exact in bf16 as long as it stays below 256;
// the x values such an element meets are stored divided by 2^f (exact), so the product is
// (128 / 2^f) x + q x, and the closing of a group subtracts (128 / 2^f + z) times the sum of
// those x values.  Codes therefore fall into classes by their f:
//   4 bits: one class (every field is shifted down to f = 0);
//   3 bits: f = 0 for the low field of a byte, f = 3 for the high field (as in gemv_mma);
//   2 bits: register j of a word (codes j and j + 8, field at bit 2 j) is read from the word
//           shifted by 6 (j / 3) with f = 2 (j % 3): two shifts per word instead of seven.
template <int BITS> struct Mma4Classes;
template <> struct Mma4Classes<4> { static constexpr int N = 1; };
template <> struct Mma4Classes<3> { static constexpr int N = 2; };
template <> struct Mma4Classes<2> { static constexpr int N = 3; };

// class (0 .. N-1, f = BITS * class) of code c of a cell
template <int BITS>
__device__ inline int mma4_class(int c)
{
    if constexpr (BITS == 4) return 0;
    else if constexpr (BITS == 3) return (c & 7) >> 2;      // code within its word: 4 .. 7 are high fields
    else return (c & 7) % 3;
}

template <int BITS>
__device__ inline void mma4_unpack(const uint32_t *w, const MmaConst &c, MmaOperand *op)
{
    if constexpr (BITS == 2) {
        const uint32_t w6 = w[0] >> 6, w12 = w[0] >> 12;
        op[0].r[0] = and_or(w[0], c.mask, c.magic);
        op[0].r[1] = and_or(w[0], c.mask_up, c.magic);
        op[0].r[2] = and_or(w[0], c.mask_up2, c.magic);
        op[0].r[3] = and_or(w6, c.mask, c.magic);
        op[1].r[0] = and_or(w6, c.mask_up, c.magic);
        op[1].r[1] = and_or(w6, c.mask_up2, c.magic);
        op[1].r[2] = and_or(w12, c.mask, c.magic);
        op[1].r[3] = and_or(w12, c.mask_up, c.magic);
    } else {
        mma_unpack<BITS>(w, c, op);
    }
}

template <int BITS, int CPG>
__global__ __launch_bounds__(512) void gemv_mma4(QG_FIRST_BLOCKS, const GemvArgs A)
{
    using F = Fmt<BITS>;
    constexpr int L = loads_per_step<BITS>();
    constexpr int S = codes_per_step<BITS>();
    constexpr int CELLS = cells_per_step<BITS>();
    constexpr int GPS = CPG > 0 ? CELLS / CPG : 0;
    constexpr int OPC = F::CELL / 4;                // matrix instructions (operands) per cell
    constexpr int NXV = S / 128;
    constexpr int ZPER = 32 / F::ZBITS;
    constexpr int PITCH = S + 8;                    // u16 per part: the four parts on different banks
    constexpr int NCL = Mma4Classes<BITS>::N;
    using D = StepData<BITS, GPS>;
    __shared__ float red[16][QG_WAVE];
    // per wavefront and buffer: the three parts of the step's x in operand order, and a part of zeros
    extern __shared__ __attribute__((aligned(16))) lds_u16 xs_raw[];
    lds_u16(*xs)[2][4][PITCH] = (lds_u16(*)[2][4][PITCH])xs_raw;

    const int pi = find_problem(fb_a, fb_b, fb_c, A, blockIdx.x);
    const GemvProblem P = A.p[pi];
    pin_problem(P);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const WaveJob job = locate(P, blockIdx.x - P.block_begin, P.steps, wave);
    if (!job.work) return;                      // no work: leave before the barrier
    const int tile = job.tile, s0 = job.item0, s1 = job.item1;

    TileView T;
    T.codes = P.codes + (size_t)tile * P.steps * L * QG_WAVE + lane;
    T.scales = P.scales + (size_t)tile * P.ngroups * QG_WAVE + lane;
    T.zeros = P.zeros + (size_t)tile * P.zwords * QG_WAVE + lane;
    T.x = P.x;

#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int i = lane; i < PITCH; i += QG_WAVE) xs[wave][b][3][i] = 0;

    // where this lane's x values go: x[128 i + 2 lane + e] of the step; and the class of the
    // codes they meet (the same for every i: 128 is a multiple of the cell size), as a scale
    // for the stored value and as 0 / 1 weights for the x-hat of each class
    int xpos[NXV][2];
    float xscale[2], cw[NCL][2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int cls = mma4_class<BITS>((2 * lane + e) % F::CELL);
        xscale[e] = cls == 0 ? 1.0f : cls == 1 ? (BITS == 3 ? 0.125f : 0.25f) : 0.0625f;
#pragma unroll
        for (int c = 0; c < NCL; ++c) cw[c][e] = cls == c ? 1.0f : 0.0f;
    }
#pragma unroll
    for (int i = 0; i < NXV; ++i)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int k = 128 * i + 2 * lane + e;
            xpos[i][e] = (k / F::CELL) * (OPC * 4) + mma4_slot<BITS>(k % F::CELL);
        }
    const lds_u16 *abase[2] = {&xs[wave][0][lane & 3][0], &xs[wave][1][lane & 3][0]};

    auto stage_x = [&](const D &d, int buf) {
#pragma unroll
        for (int i = 0; i < NXV; ++i) {
            mma_floatx2 r = {d.xv[i].x * xscale[0], d.xv[i].y * xscale[1]};
#pragma unroll
            for (int part = 0; part < 3; ++part) {
                const mma_bf16x2 h = __builtin_convertvector(r, mma_bf16x2);
                const uint32_t bits = *(const uint32_t *)&h;
                xs[wave][buf][part][xpos[i][0]] = (uint16_t)bits;
                xs[wave][buf][part][xpos[i][1]] = (uint16_t)(bits >> 16);
                r[0] -= __uint_as_float(bits << 16);
                r[1] -= __uint_as_float(bits & 0xffff0000u);
            }
        }
    };

    const MmaConst mc = mma_constants<BITS>();
    float yacc = 0.0f;
    mma4_acc acc0 = {0.0f, 0.0f, 0.0f, 0.0f}, acc1 = {0.0f, 0.0f, 0.0f, 0.0f};
    float xacc[NCL];                                // CPG == 0: x of the running piece, per class
#pragma unroll
    for (int c = 0; c < NCL; ++c) xacc[c] = 0.0f;
    // (128 / 2^f + z) of class c
    auto offset_of = [](int c, uint32_t zq) { return (float)(zq + (c == 0 ? 128u : c == 1 ? (BITS == 3 ? 16u : 32u) : 8u)); };

    // the matrix instructions of one cell: OPC operands, two per 128-bit read of A
    auto cell_mfma = [&](const D &d, int cell, int buf) {
        uint32_t w[F::PLANES];
        const int u = cell >> 2, j = cell & 3;
#pragma unroll
        for (int pl = 0; pl < F::PLANES; ++pl) w[pl] = word_of(d.v[u * F::PLANES + pl], j);
        MmaOperand op[mma_ops<BITS>()];
        mma4_unpack<BITS>(w, mc, op);
#pragma unroll
        for (int o = 0; o < OPC; o += 2) {
            MmaOperand a;
            a.q = *(const lds_u128 *)(abase[buf] + (cell * OPC + o) * 4);
            const uint2 a0 = make_uint2(a.r[0], a.r[1]), a1 = make_uint2(a.r[2], a.r[3]);
            const uint2 b0 = make_uint2(op[o >> 1].r[0], op[o >> 1].r[1]);
            const uint2 b1 = make_uint2(op[o >> 1].r[2], op[o >> 1].r[3]);
            acc0 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(*(const mma4_ab *)&a0, *(const mma4_ab *)&b0, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(*(const mma4_ab *)&a1, *(const mma4_ab *)&b1, acc1, 0, 0, 0);
        }
    };
    // T of the finished group for this lane's output; clears the accumulators
    auto take_sum = [&]() {
        const float t = (acc0[0] + acc1[0]) + (acc0[1] + acc1[1]) + (acc0[2] + acc1[2]);
        acc0 = mma4_acc{0.0f, 0.0f, 0.0f, 0.0f};
        acc1 = mma4_acc{0.0f, 0.0f, 0.0f, 0.0f};
        return t;
    };

    auto compute = [&](const D &d, int step, int buf) {
        if constexpr (CPG > 0) {
            float xhat[NCL][GPS];
#pragma unroll
            for (int c = 0; c < NCL; ++c) step_group_sums<BITS, GPS>(d, xhat[c], cw[c][0], cw[c][1]);
#pragma unroll
            for (int cell = 0; cell < CELLS; ++cell) {
                cell_mfma(d, cell, buf);
                if ((cell + 1) % CPG == 0) {
                    const int gs = (cell + 1) / CPG - 1;
                    const int gabs = step * GPS + gs;
                    const float tsum = take_sum();
                    const uint32_t zword = d.zw[D::ZW > 1 ? gs / D::ZPER : 0];
                    const uint32_t zq = (zword >> (F::ZBITS * (gabs % D::ZPER))) & ((1u << F::ZBITS) - 1u);
                    float tz = tsum;
#pragma unroll
                    for (int c = 0; c < NCL; ++c) tz = fmaf(-offset_of(c, zq), xhat[c][gs], tz);
                    yacc = fmaf(d.s[gs], tz, yacc);
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < NXV; ++i)
#pragma unroll
                for (int c = 0; c < NCL; ++c) xacc[c] += d.xv[i].x * cw[c][0] + d.xv[i].y * cw[c][1];
#pragma unroll
            for (int cell = 0; cell < CELLS; ++cell) cell_mfma(d, cell, buf);
        }
    };

    // CPG == 0: closes the piece of group g this wavefront has seen, if step s ends the group or the range
    const int spg = P.steps_per_group;
    int g = CPG == 0 ? s0 / spg : 0;
    int left = CPG == 0 ? (g + 1) * spg - s0 : 0;
    auto close_group = [&](int s) {
        if constexpr (CPG == 0) {
            if (--left != 0 && s + 1 != s1) return;
            float xhat[NCL];
#pragma unroll
            for (int c = 0; c < NCL; ++c) segment_sums<64>(xacc[c], &xhat[c]);
            const float tsum = take_sum();
            const float scale = T.scales[(size_t)g * QG_WAVE];
            const uint32_t zword = T.zeros[(size_t)(g / ZPER) * QG_WAVE];
            const uint32_t zq = (zword >> (F::ZBITS * (g % ZPER))) & ((1u << F::ZBITS) - 1u);
            float tz = tsum;
#pragma unroll
            for (int c = 0; c < NCL; ++c) {
                tz = fmaf(-offset_of(c, zq), xhat[c], tz);
                xacc[c] = 0.0f;
            }
            yacc = fmaf(scale, tz, yacc);
            ++g;
            left = spg;
        }
    };

    // two register buffers and two LDS buffers used alternately, as in gemv_static
    const int last = s1 - 1;
    D da, db;
    fetch_step(da, T, s0, lane);
    stage_x(da, 0);
    for (int s = s0; s < s1; s += 2) {
        const int sb = s + 1 < last ? s + 1 : last;
        const int sc = s + 2 < last ? s + 2 : last;
        fetch_step(db, T, sb, lane);
        compute(da, s, 0);
        close_group(s);
        if (s + 1 >= s1) break;                       // odd number of steps
        stage_x(db, 1);
        fetch_step(da, T, sc, lane);
        compute(db, sb, 1);
        close_group(sb);
        stage_x(da, 0);
    }
    finish_tile(P, job, yacc, red);
}

// ---------------------------------------------------------------------------------------
// gemv_mma4i: the 4 x 4 x 4 matrix instruction on 8-bit integers.  A code needs no exponent
// around it to be an int8, so a word of 4-bit codes becomes two operands with two ANDs and one
// shift (w & 0x0f0f0f0f holds codes 0, 2, 4, 6 as bytes, (w >> 4) & 0x0f0f0f0f codes 1, 3, 5,
// 7), a word of 2-bit codes four operands with four ANDs and one shift (the fields at bits 2
// and 4 of a byte stay where they are and count 4 q and 16 q; the x values they meet are
// stored divided by 4 and 16), and a word of the 3-bit cell -- every byte holds one code in
// bits 0-2 and one in bits 3-5 -- two operands with two ANDs (q and 8 q; the fourth word of
// the cell is put together from the spare bits 6-7 first).  x goes in as 32-bit fixed
// point relative to the largest |x| of the step (a power of two, so scaling is exact),
// cut into four signed bytes that fill the four rows of the A operand: lane l receives
// D_i = sum_k q_k digit_i(x_k) for its own output, and sum_i 256^i D_i / scale = sum_k q_k x_k
// to 2^-30 of the step's largest |x| per term.  There is no 128 to take out again: the
// closing of a group is eq. (2) as it stands, y += s (T - z xhat), with one xhat per group.
template <int BITS>
__device__ inline int mma4i_slot(int c)              // 4 * operand of the cell + byte, of code c of a cell
{
    if constexpr (BITS == 3) {
        const int w = c >> 3, r = c & 7;             // word (A, B, C, T); byte r & 3, low or high field
        return (2 * w + (r >> 2)) * 4 + (r & 3);
    } else {
        constexpr int OPC = Fmt<BITS>::CELL / 4;
        return (c % OPC) * 4 + c / OPC;
    }
}

// what the field of code c of a cell counts, as the divisor applied to the x it meets
template <int BITS>
__device__ inline float mma4i_xdiv(int c)
{
    if constexpr (BITS == 3) return (c & 7) >= 4 ? 0.125f : 1.0f;
    else if constexpr (BITS == 2) return (c & 3) == 1 ? 0.25f : (c & 3) == 2 ? 0.0625f : 1.0f;
    else return 1.0f;
}

typedef int mma4i_acc __attribute__((ext_vector_type(4)));
typedef uint8_t __attribute__((may_alias)) lds_u8;

template <int CTRL, int ROW_MASK = 0xf>
__device__ inline float dpp_max(float v)             // for v >= 0: disabled rows see 0
{
    const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false);
    return fmaxf(v, __int_as_float(moved));
}

template <int BITS, int CPG>
__global__ __launch_bounds__(512) void gemv_mma4i(QG_FIRST_BLOCKS, const GemvArgs A)
{
    static_assert(CPG == 0 || BITS != 4 || CPG % 2 == 0, "a 128-bit read of A covers two 4-bit cells");
    using F = Fmt<BITS>;
    constexpr int L = loads_per_step<BITS>();
    constexpr int S = codes_per_step<BITS>();
    constexpr int CELLS = cells_per_step<BITS>();
    constexpr int GPS = CPG > 0 ? CELLS / CPG : 0;
    constexpr int READS = S / 16;                   // 128-bit reads of A per step: 16 k, four matrix instructions each
    constexpr int NXV = S / 128;
    constexpr int ZPER = 32 / F::ZBITS;
    constexpr int PITCH = S + 16;                   // bytes per digit row: the four rows on different banks
    using D = StepData<BITS, GPS>;
    __shared__ float red[16][QG_WAVE];
    // per wavefront and buffer: the four digit rows of the step's x in operand order
    extern __shared__ __attribute__((aligned(16))) lds_u8 xs8_raw[];
    lds_u8(*xs)[2][4][PITCH] = (lds_u8(*)[2][4][PITCH])xs8_raw;

    const int pi = find_problem(fb_a, fb_b, fb_c, A, blockIdx.x);
    const GemvProblem P = A.p[pi];
    pin_problem(P);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const WaveJob job = locate(P, blockIdx.x - P.block_begin, P.steps, wave);
    if (!job.work) return;                      // no work: leave before the barrier
    const int tile = job.tile, s0 = job.item0, s1 = job.item1;

    TileView T;
    T.codes = P.codes + (size_t)tile * P.steps * L * QG_WAVE + lane;
    T.scales = P.scales + (size_t)tile * P.ngroups * QG_WAVE + lane;
    T.zeros = P.zeros + (size_t)tile * P.zwords * QG_WAVE + lane;
    T.x = P.x;

    // where this lane's x values go: x[128 i + 2 lane + e] of the step; and what the field of
    // the code they meet counts (the same for every i: 128 is a multiple of the cell size)
    int xpos[NXV][2];
    float xdiv[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) xdiv[e] = mma4i_xdiv<BITS>((2 * lane + e) % F::CELL);
#pragma unroll
    for (int i = 0; i < NXV; ++i)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int k = 128 * i + 2 * lane + e;
            xpos[i][e] = (k / F::CELL) * F::CELL + mma4i_slot<BITS>(k % F::CELL);
        }
    const lds_u8 *abase[2] = {&xs[wave][0][lane & 3][0], &xs[wave][1][lane & 3][0]};

    // Fixed point of the step: |x| scale < 2^30 for the largest |x| of the step.  Returns 1 / scale.
    auto stage_x = [&](const D &d, int buf) -> float {
        float m = 0.0f;
#pragma unroll
        for (int i = 0; i < NXV; ++i) m = fmaxf(m, fmaxf(fabsf(d.xv[i].x), fabsf(d.xv[i].y)));
        m = dpp_max<QG_DPP_QUAD_XOR1>(m);
        m = dpp_max<QG_DPP_QUAD_XOR2>(m);
        m = dpp_max<QG_DPP_HALF_MIRROR>(m);
        m = dpp_max<QG_DPP_ROW_MIRROR>(m);
        m = dpp_max<QG_DPP_BCAST15, 0xa>(m);
        m = dpp_max<QG_DPP_BCAST31, 0xc>(m);
        uint32_t eb = (uint32_t)__builtin_amdgcn_readlane(__float_as_int(m), 63) >> 23;   // biased exponent
        eb = eb < 30u ? 30u : eb > 254u ? 254u : eb;
        const float scale = __uint_as_float((283u - eb) << 23);                             // 2^(156 - eb)
#pragma unroll
        for (int i = 0; i < NXV; ++i) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const float xv = e == 0 ? d.xv[i].x : d.xv[i].y;
                const int fixed = (int)(xv * (scale * xdiv[e]));
                // the four bytes of (fixed + 0x808080) ^ 0x808080, read as signed, are digits
                // base 256 of `fixed`
                const uint32_t pat = ((uint32_t)fixed + 0x00808080u) ^ 0x00808080u;
                xs[wave][buf][0][xpos[i][e]] = (uint8_t)pat;
                xs[wave][buf][1][xpos[i][e]] = (uint8_t)(pat >> 8);
                xs[wave][buf][2][xpos[i][e]] = (uint8_t)(pat >> 16);
                xs[wave][buf][3][xpos[i][e]] = (uint8_t)(pat >> 24);
            }
        }
        return __uint_as_float((eb - 29u) << 23);                                           // 2^(eb - 156)
    };

    float yacc = 0.0f;
    mma4i_acc acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
    float tacc = 0.0f, xacc = 0.0f;                 // CPG == 0: T and x of the running piece of a group

    // the four matrix instructions of one 128-bit read of A (16 k): two 4-bit cells, one 2-bit
    // cell or half a 3-bit cell
    uint32_t spare = 0;                             // 3 bits: the fourth word of the cell in hand
    auto read_mfma = [&](const D &d, int rd, int buf) {
        MmaOperand a;
        a.q = *(const lds_u128 *)(abase[buf] + rd * 16);
        uint32_t b[4];
        if constexpr (BITS == 4) {
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const int cell = 2 * rd + c;
                const uint32_t w = word_of(d.v[cell >> 2], cell & 3);
                b[2 * c] = w & 0x0f0f0f0fu;
                b[2 * c + 1] = (w >> 4) & 0x0f0f0f0fu;
            }
        } else if constexpr (BITS == 2) {
            const uint32_t w = word_of(d.v[rd >> 2], rd & 3);
            b[0] = w & 0x03030303u;
            b[1] = w & 0x0c0c0c0cu;
            b[2] = w & 0x30303030u;
            b[3] = (w >> 6) & 0x03030303u;
        } else {
            const int cell = rd >> 1, u = cell >> 2, j = cell & 3;
            if ((rd & 1) == 0) {
                const uint32_t wa = word_of(d.v[u * 3], j), wb = word_of(d.v[u * 3 + 1], j), wc = word_of(d.v[u * 3 + 2], j);
                spare = ((wa >> 6) & 0x03030303u) | ((wb >> 4) & 0x0c0c0c0cu) | ((wc >> 2) & 0x30303030u);
                b[0] = wa & 0x07070707u;
                b[1] = wa & 0x38383838u;
                b[2] = wb & 0x07070707u;
                b[3] = wb & 0x38383838u;
            } else {
                const uint32_t wc = word_of(d.v[u * 3 + 2], j);
                b[0] = wc & 0x07070707u;
                b[1] = wc & 0x38383838u;
                b[2] = spare & 0x07070707u;
                b[3] = spare & 0x38383838u;
            }
        }
        acc0 = __builtin_amdgcn_mfma_i32_4x4x4i8((int)a.r[0], (int)b[0], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_i32_4x4x4i8((int)a.r[1], (int)b[1], acc1, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_i32_4x4x4i8((int)a.r[2], (int)b[2], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_i32_4x4x4i8((int)a.r[3], (int)b[3], acc1, 0, 0, 0);
    };
    // sum_i 256^i D_i of the finished cells for this lane's output, in units of 1 / scale;
    // clears the accumulators
    auto take_sum = [&]() {
        // (|D_i| of a step stays below 2^21, so the sums fit 32 bits)
        const int lo = (acc0[1] + acc1[1]) * 256 + (acc0[0] + acc1[0]);
        const int hi = (acc0[3] + acc1[3]) * 256 + (acc0[2] + acc1[2]);
        acc0 = mma4i_acc{0, 0, 0, 0};
        acc1 = mma4i_acc{0, 0, 0, 0};
        return fmaf((float)hi, 65536.0f, (float)lo);
    };

    auto compute = [&](const D &d, int step, int buf, float inv) {
        if constexpr (CPG > 0) {
            float xhat[GPS];
            step_group_sums<BITS, GPS>(d, xhat);
            constexpr int RPG = CPG * F::CELL / 16;           // reads per group
#pragma unroll
            for (int rd = 0; rd < READS; ++rd) {
                read_mfma(d, rd, buf);
                if ((rd + 1) % RPG == 0) {
                    const int gs = (rd + 1) / RPG - 1;
                    const int gabs = step * GPS + gs;
                    const float tsum = take_sum() * inv;
                    const uint32_t zword = d.zw[D::ZW > 1 ? gs / D::ZPER : 0];
                    const uint32_t zq = (zword >> (F::ZBITS * (gabs % D::ZPER))) & ((1u << F::ZBITS) - 1u);
                    yacc = fmaf(d.s[gs], fmaf(-(float)zq, xhat[gs], tsum), yacc);
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < NXV; ++i) xacc += d.xv[i].x + d.xv[i].y;
#pragma unroll
            for (int rd = 0; rd < READS; ++rd) read_mfma(d, rd, buf);
            tacc = fmaf(take_sum(), inv, tacc);     // every step has a scale of its own
        }
    };

    // CPG == 0: closes the piece of group g this wavefront has seen, if step s ends the group or the range
    const int spg = P.steps_per_group;
    int g = CPG == 0 ? s0 / spg : 0;
    int left = CPG == 0 ? (g + 1) * spg - s0 : 0;
    auto close_group = [&](int s) {
        if constexpr (CPG == 0) {
            if (--left != 0 && s + 1 != s1) return;
            float xhat;
            segment_sums<64>(xacc, &xhat);
            const float scale = T.scales[(size_t)g * QG_WAVE];
            const uint32_t zword = T.zeros[(size_t)(g / ZPER) * QG_WAVE];
            const uint32_t zq = (zword >> (F::ZBITS * (g % ZPER))) & ((1u << F::ZBITS) - 1u);
            yacc = fmaf(scale, fmaf(-(float)zq, xhat, tacc), yacc);
            tacc = 0.0f;
            xacc = 0.0f;
            ++g;
            left = spg;
        }
    };

    // two register buffers and two LDS buffers used alternately, as in gemv_static
    const int last = s1 - 1;
    D da, db;
    fetch_step(da, T, s0, lane);
    float inv_a = stage_x(da, 0), inv_b = 0.0f;
    for (int s = s0; s < s1; s += 2) {
        const int sb = s + 1 < last ? s + 1 : last;
        const int sc = s + 2 < last ? s + 2 : last;
        fetch_step(db, T, sb, lane);
        compute(da, s, 0, inv_a);
        close_group(s);
        if (s + 1 >= s1) break;                       // odd number of steps
        inv_b = stage_x(db, 1);
        fetch_step(da, T, sc, lane);
        compute(db, sb, 1, inv_b);
        close_group(sb);
        inv_a = stage_x(da, 0);
    }
    finish_tile(P, job, yacc, red);
}

// ---------------------------------------------------------------------------------------
// Up to 16 activation rows at once (a few prompt tokens): Y = X What^T with the launch
// structure of the GEMV -- one wavefront per 64 outputs and K range, no workgroup barrier in
// the loop, K split over the wavefronts of a team -- and the arithmetic of gemv_mma: 4-bit
// codes become exact bf16 integers 128 + q, the matrix instruction multiplies them with the
// rows of X (rounded to bf16; rows 16-31 of the A operand are zero), and per group
//     Y[m][n] += s_n (T[m][n] - (128 + z_n) xhat[m]),   xhat[m] = sum_k bf16(X[m][k]),
// where xhat comes out of one more matrix instruction per operand (X times a column of ones),
// so it sits in the same registers as T.  Each wavefront converts the X rows of its own step
// and keeps them in its own LDS region, one 16-byte operand piece per (row, cell).
// ---------------------------------------------------------------------------------------
template <int CPG>
__global__ __launch_bounds__(512) void gemm_rows16(QG_FIRST_BLOCKS, const GemvArgs A)
{
    using F = Fmt<4>;
    constexpr int L = loads_per_step<4>();          // 4 code vectors per step
    constexpr int S = codes_per_step<4>();          // 128 k per step
    constexpr int CELLS = cells_per_step<4>();      // 16 cells of 8 codes
    constexpr int GPS = CELLS / CPG;
    constexpr int ZPER = 32 / F::ZBITS;
    constexpr int ZW = GPS > ZPER ? GPS / ZPER : 1;
    constexpr int PITCH = S + 8;                    // bf16 per LDS row: conflict-free 128-bit reads
    constexpr int XL = 16 * CELLS / QG_WAVE;        // (row, cell) pieces per lane and step: 4
    static_assert(CPG >= 2 && CPG % 2 == 0, "a group must hold whole pairs of cells");
    // per wavefront: 16 rows of X for one step (reused at the end for the team's partial
    // results); one row of zeros for rows 16-31 of the A operand
    extern __shared__ __attribute__((aligned(16))) lds_u16 rows_raw[];
    __shared__ __attribute__((aligned(16))) lds_u16 zero_row[PITCH];

    const int pi = find_problem(fb_a, fb_b, fb_c, A, blockIdx.x);
    const GemvProblem P = A.p[pi];
    pin_problem(P);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const WaveJob job = locate(P, blockIdx.x - P.block_begin, P.steps, wave);
    if (!job.work) return;                      // no work: leave before the barrier
    const int tile = job.tile, s0 = job.item0, s1 = job.item1;
    const int M = P.rows;

    const uint4 *codes = P.codes + (size_t)tile * P.steps * L * QG_WAVE + lane;
    const float *scales = P.scales + (size_t)tile * P.ngroups * QG_WAVE + lane;
    const uint32_t *zeros = P.zeros + (size_t)tile * P.zwords * QG_WAVE + lane;
    lds_u16 *xs = rows_raw + (size_t)wave * 16 * PITCH;

#pragma unroll
    for (int i = lane; i < PITCH; i += QG_WAVE) zero_row[i] = 0;

    struct Regs {
        uint4 v[L];
        float s[GPS];
        uint32_t zw[ZW];
        float4 x[XL][2];       // pieces (row, cell) = (4 j + lane / 16, lane % 16): 8 consecutive k of X
    };
    // groups of four rows with no real row are not loaded; other rows past M read row M - 1
    // again; both are cleared on their way into LDS
    const int xrow0 = lane >> 4, xcell = lane & 15;
    auto fetch = [&](int step, Regs &r) {
#pragma unroll
        for (int i = 0; i < L; ++i) r.v[i] = codes[((size_t)step * L + i) * QG_WAVE];
#pragma unroll
        for (int g = 0; g < GPS; ++g) r.s[g] = scales[(size_t)(step * GPS + g) * QG_WAVE];
#pragma unroll
        for (int w = 0; w < ZW; ++w) r.zw[w] = zeros[(size_t)((step * GPS) / ZPER + w) * QG_WAVE];
#pragma unroll
        for (int j = 0; j < XL; ++j) {
            if (4 * j >= M) continue;                    // uniform
            int m = 4 * j + xrow0;
            m = m < M ? m : M - 1;
            const float4 *src = (const float4 *)(P.x + (size_t)m * P.K + (size_t)step * S + xcell * 8);
            r.x[j][0] = src[0];
            r.x[j][1] = src[1];
        }
    };
    // X of one step into LDS: per piece the eight values in the order the unpacked codes have
    // inside an operand (register j = codes j and j + 4)
    auto stage = [&](const Regs &r) {
#pragma unroll
        for (int j = 0; j < XL; ++j) {
            const int m = 4 * j + xrow0;
            MmaOperand o;
            if (4 * j >= M) {                            // uniform: nothing was loaded
                o.q = make_uint4(0u, 0u, 0u, 0u);
                *(lds_u128 *)(xs + m * PITCH + xcell * 8) = o.q;
                continue;
            }
            const float4 a = r.x[j][0], b = r.x[j][1];
            const float keep = m < M ? 1.0f : 0.0f;
            mma_floatx2 t2;
            t2[0] = a.x * keep; t2[1] = b.x * keep;
            { const mma_bf16x2 h = __builtin_convertvector(t2, mma_bf16x2); o.r[0] = *(const uint32_t *)&h; }
            t2[0] = a.y * keep; t2[1] = b.y * keep;
            { const mma_bf16x2 h = __builtin_convertvector(t2, mma_bf16x2); o.r[1] = *(const uint32_t *)&h; }
            t2[0] = a.z * keep; t2[1] = b.z * keep;
            { const mma_bf16x2 h = __builtin_convertvector(t2, mma_bf16x2); o.r[2] = *(const uint32_t *)&h; }
            t2[0] = a.w * keep; t2[1] = b.w * keep;
            { const mma_bf16x2 h = __builtin_convertvector(t2, mma_bf16x2); o.r[3] = *(const uint32_t *)&h; }
            *(lds_u128 *)(xs + m * PITCH + xcell * 8) = o.q;
        }
    };

    // A operand: row = lane % 32 (rows 16-31 are zero), half = lane / 32 = which cell of the pair
    const int row = lane & 31, half = lane >> 5;
    const lds_u16 *abase = row < 16 ? xs + row * PITCH + half * 8 : zero_row + half * 8;
    const MmaConst mc = mma_constants<4>();
    MmaOperand ones;
#pragma unroll
    for (int j = 0; j < 4; ++j) ones.r[j] = 0x3f803f80u;     // two bf16 1.0

    // results of this wavefront: rows 8 (i / 4) + 4 half + i % 4 (i < 8) of outputs lane % 32 (P)
    // and 32 + lane % 32 (Q) of the tile
    float yp[8], yq[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) { yp[i] = 0.0f; yq[i] = 0.0f; }

    auto compute = [&](const Regs &r, int step) {
        mma_floatx16 accP, accQ, accX;
#pragma unroll
        for (int i = 0; i < 16; ++i) { accP[i] = 0.0f; accQ[i] = 0.0f; accX[i] = 0.0f; }
#pragma unroll
        for (int cp = 0; cp < CELLS / 2; ++cp) {
            const int c0 = 2 * cp, u = c0 >> 2, j = c0 & 3;
            const auto sw = __builtin_amdgcn_permlane32_swap(word_of(r.v[u], j), word_of(r.v[u], j + 1), false, false);
            uint32_t wp[1] = {sw[0]}, wq[1] = {sw[1]};
            MmaOperand bp[1], bq[1], a;
            mma_unpack<4>(wp, mc, bp);
            mma_unpack<4>(wq, mc, bq);
            a.q = *(const lds_u128 *)(abase + cp * 16);
            accP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, bp[0].v, accP, 0, 0, 0);
            accQ = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, bq[0].v, accQ, 0, 0, 0);
            accX = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, ones.v, accX, 0, 0, 0);
            if ((2 * cp + 2) % CPG == 0) {
                const int gs = (2 * cp + 2) / CPG - 1;
                const int gabs = step * GPS + gs;
                const uint32_t zword = r.zw[ZW > 1 ? gs / ZPER : 0];
                const float s = r.s[gs];
                const float nzs = -(float)(((zword >> (F::ZBITS * (gabs % ZPER))) & ((1u << F::ZBITS) - 1u)) + 128u) * s;
                // scale and zero term of the outputs this lane's accumulators belong to
                const auto ss = __builtin_amdgcn_permlane32_swap(__float_as_uint(s), __float_as_uint(s), false, false);
                const auto zz = __builtin_amdgcn_permlane32_swap(__float_as_uint(nzs), __float_as_uint(nzs), false, false);
                const float sP = __uint_as_float(ss[0]), sQ = __uint_as_float(ss[1]);
                const float zP = __uint_as_float(zz[0]), zQ = __uint_as_float(zz[1]);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    yp[i] += fmaf(sP, accP[i], zP * accX[i]);
                    yq[i] += fmaf(sQ, accQ[i], zQ * accX[i]);
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) { accP[i] = 0.0f; accQ[i] = 0.0f; accX[i] = 0.0f; }
            }
        }
    };

    // two register buffers used alternately; the rows of X of a step are converted into the
    // wavefront's LDS region right before the step is computed
    const int last = s1 - 1;
    Regs ra, rb;
    fetch(s0, ra);
    for (int s = s0; s < s1; s += 2) {
        const int sb = s + 1 < last ? s + 1 : last;
        const int sc = s + 2 < last ? s + 2 : last;
        fetch(sb, rb);
        stage(ra);
        compute(ra, s);
        if (s + 1 >= s1) break;                       // odd number of steps
        fetch(sc, ra);
        stage(rb);
        compute(rb, sb);
    }

    // team reduction through LDS (each wavefront writes its own region first), then the lead
    // adds the partial results in wavefront order and stores Y
    float *mine = (float *)(rows_raw + (size_t)wave * 16 * PITCH);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        mine[i * QG_WAVE + lane] = yp[i];
        mine[(8 + i) * QG_WAVE + lane] = yq[i];
    }
    __syncthreads();
    if (wave != job.lead) return;
    for (int w = 1; w < job.team; ++w) {
        const float *other = (const float *)(rows_raw + (size_t)(job.lead + w) * 16 * PITCH);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            yp[i] += other[i * QG_WAVE + lane];
            yq[i] += other[(8 + i) * QG_WAVE + lane];
        }
    }
    const int col = lane & 31;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int m = 8 * (i / 4) + 4 * half + (i % 4);
        const int np = tile * QG_WAVE + col, nq = np + 32;
        if (m < M && np < P.N) P.y[(size_t)m * P.N + np] = yp[i];
        if (m < M && nq < P.N) P.y[(size_t)m * P.N + nq] = yq[i];
    }
}

// ---------------------------------------------------------------------------------------
// Groups that are a whole number of steps (G = 256, ..., up to one group per output: the
// full-column case of eq. (1)).  A wavefront's range of steps need not begin or end at a group
// boundary: s (sum q x - z sum x) is linear in the two sums, so the pieces of a group that
// different wavefronts hold are closed separately, each with the group's s and z, and add up
// in the team's reduction.
// ---------------------------------------------------------------------------------------
template <int BITS>
__global__ __launch_bounds__(1024) void gemv_runtime(QG_FIRST_BLOCKS, const GemvArgs A)
{
    using F = Fmt<BITS>;
    constexpr int L = loads_per_step<BITS>();
    constexpr int S = codes_per_step<BITS>();
    constexpr int ZPER = 32 / F::ZBITS;
    __shared__ float red[16][QG_WAVE];

    const int pi = find_problem(fb_a, fb_b, fb_c, A, blockIdx.x);
    const GemvProblem P = A.p[pi];                 // one copy: all fields fetched at once
    pin_problem(P);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int spg = P.steps_per_group;
    const WaveJob job = locate(P, blockIdx.x - P.block_begin, P.steps, wave);
    if (!job.work) return;                      // no work: leave before the barrier
    const int tile = job.tile, s0 = job.item0, s1 = job.item1;

    TileView T;
    T.codes = P.codes + (size_t)tile * P.steps * L * QG_WAVE + lane;
    T.scales = P.scales + (size_t)tile * P.ngroups * QG_WAVE + lane;
    T.zeros = P.zeros + (size_t)tile * P.zwords * QG_WAVE + lane;
    T.x = P.x;
    const float *__restrict__ x = P.x;

    float yacc = 0.0f, xacc = 0.0f;
    Acc2 acc = {0.0f, 0.0f};
    int g = s0 / spg;                                   // running group
    int left = (g + 1) * spg - s0;                      // its steps still to come
    // closes the piece of group g this wavefront has seen, if step s ends the group or the range
    auto close_group = [&](int s) {
        if (--left != 0 && s + 1 != s1) return;
        float xhat;
        segment_sums<64>(xacc, &xhat);
        const float scale = T.scales[(size_t)g * QG_WAVE];
        const uint32_t zword = T.zeros[(size_t)(g / ZPER) * QG_WAVE];
        const float zf = (float)((zword >> (F::ZBITS * (g % ZPER))) & ((1u << F::ZBITS) - 1u));
        yacc = fmaf(scale, fmaf(-zf, xhat, acc_total<BITS>(acc)), yacc);
        acc.a = 0.0f;
        acc.b = 0.0f;
        xacc = 0.0f;
        ++g;
        left = spg;
    };

    // two buffers used alternately, as in gemv_static
    const int last = s1 - 1;
    StepData<BITS, 0> da, db;
    fetch_step(da, T, s0, lane);
    XBatch xb = load_x32(x + (size_t)s0 * S);
    for (int s = s0; s < s1; s += 2) {
        const int sb = s + 1 < last ? s + 1 : last;
        const int sc = s + 2 < last ? s + 2 : last;
        fetch_step(db, T, sb, lane);
        compute_step(da, x + (size_t)s * S, x + (size_t)sb * S, xb, s, true, acc, xacc, yacc);
        close_group(s);
        if (s + 1 >= s1) break;                       // odd number of steps
        fetch_step(da, T, sc, lane);
        compute_step(db, x + (size_t)sb * S, x + (size_t)sc * S, xb, sb, true, acc, xacc, yacc);
        close_group(sb);
    }
    finish_tile(P, job, yacc, red);
}

// ---------------------------------------------------------------------------------------
// Any other group size (a whole number of cells): one cell at a time, group sums added up
// serially.  Slow and simple; covers shapes the two kernels above do not.
// ---------------------------------------------------------------------------------------
template <int BITS>
__global__ __launch_bounds__(1024) void gemv_generic(QG_FIRST_BLOCKS, const GemvArgs A)
{
    using F = Fmt<BITS>;
    constexpr int L = loads_per_step<BITS>();
    constexpr int ZPER = 32 / F::ZBITS;
    __shared__ float red[16][QG_WAVE];

    const int pi = find_problem(fb_a, fb_b, fb_c, A, blockIdx.x);
    const GemvProblem P = A.p[pi];                 // one copy: all fields fetched at once
    pin_problem(P);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int cpg = P.group / F::CELL;
    // here the items along K are groups
    const WaveJob job = locate(P, blockIdx.x - P.block_begin, P.ngroups, wave);
    if (!job.work) return;                      // no work: leave before the barrier
    const int tile = job.tile, g0 = job.item0, g1 = job.item1;

    float yacc = 0.0f;
    const uint4 *codes = P.codes + (size_t)tile * P.steps * L * QG_WAVE + lane;
    const float *sc = P.scales + (size_t)tile * P.ngroups * QG_WAVE + lane;
    const uint32_t *zr = P.zeros + (size_t)tile * P.zwords * QG_WAVE + lane;
    const float *__restrict__ x = P.x;
    for (int g = g0; g < g1; ++g) {
        Acc2 acc = {0.0f, 0.0f};
        float sx = 0.0f;
        for (int c = g * cpg; c < (g + 1) * cpg; ++c) {
            const int unit = c >> 2;
            uint4 v[3];
#pragma unroll
            for (int p = 0; p < F::PLANES; ++p) v[p] = codes[((size_t)unit * F::PLANES + p) * QG_WAVE];
            const float *xs = x + (size_t)c * F::CELL;
            // the cell sits at position (c & 3) of its unit; place its x values where
            // octet_dot expects them inside a batch of 32
            constexpr int CPB = 32 / F::CELL;                 // cells per batch
            const int bt = (c & 3) / CPB, pos = (c & 3) % CPB;
            XBatch xb;
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                const int rel = i - pos * F::CELL;
                const float val = (rel >= 0 && rel < F::CELL) ? xs[rel] : 0.0f;
                if (i < 16) xb.lo[i] = val; else xb.hi[i - 16] = val;
            }
#pragma unroll
            for (int o = 0; o < 4; ++o)
                if (o / (4 / CPB) == pos) octet_dot<BITS>(v, bt, o, xb, acc);
#pragma unroll
            for (int i = 0; i < F::CELL; ++i) sx += xs[i];
        }
        const uint32_t zword = zr[(size_t)(g / ZPER) * QG_WAVE];
        const float zf = (float)((zword >> (F::ZBITS * (g % ZPER))) & ((1u << F::ZBITS) - 1u));
        yacc = fmaf(sc[(size_t)g * QG_WAVE], fmaf(-zf, sx, acc_total<BITS>(acc)), yacc);
    }
    finish_tile(P, job, yacc, red);
}

__global__ void fill_u32(uint32_t *p, size_t n, uint32_t value)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

// ------------------------------------------------------------------ host side

// Launch-shape knobs: 0 = built-in choice.  The process-wide ones (qg_set_gemv_tuning) win; where
// they are all 0, a launch takes what the tuning table holds for its list of shapes
// (qg_gemv_autotune, qg_gemv_record_tuning); t_cur is what the launch being planned uses.
struct Tuning {
    int wpb, bytes_per_wave, kernel;      // kernel: 1 = vector ALU, 2-4 = the matrix-core kernels
};
int g_tune_wpb = 0;
int g_tune_bytes_per_wave = 0;
int g_tune_kernel = 0;
thread_local Tuning t_cur = {0, 0, 0};

struct TuneEntry {
    uint64_t key;
    Tuning t;
};
constexpr int TUNE_ENTRIES = 64;
TuneEntry g_tune_table[TUNE_ENTRIES];
int g_tune_count = 0, g_tune_next = 0;          // entries in use; the one replaced when the table is full
std::mutex g_tune_mutex;

// FNV-1a over the shapes of a launch, in the caller's order
uint64_t launch_signature(const qg_gemv_desc *descs, int count)
{
    uint64_t h = 0xcbf29ce484222325ull;
    auto mix = [&](uint64_t v) {
        for (int b = 0; b < 8; ++b) {
            h ^= (v >> (8 * b)) & 0xffu;
            h *= 0x100000001b3ull;
        }
    };
    mix((uint64_t)count);
    for (int i = 0; i < count; ++i) {
        mix((uint64_t)descs[i].N);
        mix((uint64_t)descs[i].K);
        mix(((uint64_t)(uint32_t)descs[i].bits << 32) | (uint32_t)descs[i].group);
    }
    return h;
}

Tuning tuning_for(const qg_gemv_desc *descs, int count)
{
    if (g_tune_wpb || g_tune_bytes_per_wave || g_tune_kernel) return {g_tune_wpb, g_tune_bytes_per_wave, g_tune_kernel};
    std::lock_guard<std::mutex> lock(g_tune_mutex);
    if (g_tune_count == 0) return {0, 0, 0};
    const uint64_t key = launch_signature(descs, count);
    for (int i = 0; i < g_tune_count; ++i)
        if (g_tune_table[i].key == key) return g_tune_table[i].t;
    return {0, 0, 0};
}

void record_tuning(const qg_gemv_desc *descs, int count, Tuning t)
{
    std::lock_guard<std::mutex> lock(g_tune_mutex);
    const uint64_t key = launch_signature(descs, count);
    int at = -1;
    for (int i = 0; i < g_tune_count; ++i)
        if (g_tune_table[i].key == key) at = i;
    if (at < 0) {
        if (g_tune_count < TUNE_ENTRIES) at = g_tune_count++;
        else { at = g_tune_next; g_tune_next = (g_tune_next + 1) % TUNE_ENTRIES; }
    }
    g_tune_table[at].key = key;
    g_tune_table[at].t = t;
}

enum Kind { KIND_STATIC, KIND_RUNTIME, KIND_GENERIC };

// What the last launch of this thread's process ran (for bench reports): kernel family and
// template arguments.
char g_last_kernel[64] = "";

// The K-split of one problem: work items along K are steps for the two fast kernels and
// groups for the generic one; a wavefront takes `spw` consecutive items.
struct Plan {
    Kind kind;
    int64_t items;
    int64_t steps_per_group;   // runtime kernel: steps one group spans
    int64_t max_spw;   // x-hat is kept one group per lane: at most 64 groups per wavefront
    size_t item_bytes; // packed code bytes one wavefront reads per item
};

Plan make_plan(const QgLayout &L)
{
    Plan pl;
    const int cpg = L.group / L.cell;
    const int cps = 4 * L.step_units;
    const int64_t step_codes = (int64_t)L.unit * L.step_units;
    const size_t step_bytes = (size_t)L.step_units * L.planes * QG_WAVE * 16;
    pl.kind = KIND_GENERIC;
    if (L.K % step_codes == 0) {
        if (cpg <= cps && (cpg & (cpg - 1)) == 0) pl.kind = KIND_STATIC;
        else if (L.group % step_codes == 0) pl.kind = KIND_RUNTIME;
    }
    if (pl.kind == KIND_STATIC) {
        pl.items = L.steps;
        pl.steps_per_group = 1;
        pl.max_spw = 64 / (cps / cpg);
        pl.item_bytes = step_bytes;
    } else if (pl.kind == KIND_RUNTIME) {
        pl.items = L.steps;
        pl.steps_per_group = L.group / step_codes;
        pl.max_spw = (int64_t)1 << 30;               // the running group is one scalar
        pl.item_bytes = step_bytes;
    }
    // a fast kernel that cannot cover K with 16 wavefronts x QG_MAX_CHUNKS blocks: generic
    if (pl.kind != KIND_GENERIC &&
        (pl.items + pl.max_spw - 1) / pl.max_spw > (int64_t)16 * QG_MAX_CHUNKS)
        pl.kind = KIND_GENERIC;
    if (pl.kind == KIND_GENERIC) {
        pl.items = L.ngroups;
        pl.steps_per_group = 1;
        pl.max_spw = (int64_t)1 << 30;
        pl.item_bytes = (size_t)L.group * L.bits / 8 * QG_WAVE;
    }
    return pl;
}

size_t workspace_for(const QgLayout &L)
{
    // meeting slots of the reduction tree, then one more row of slots for gated pairs
    return (size_t)L.tiles * (QG_MAX_CHUNKS + 1) * QG_WAVE * sizeof(uint32_t);
}

FirstBlocks first_blocks(const GemvArgs &A)
{
    FirstBlocks f;
    for (int i = 0; i < 4; ++i) {
        f.a[i] = A.block_begin[1 + i];
        f.b[i] = A.block_begin[5 + i];
        f.c[i] = A.block_begin[9 + i];
    }
    return f;
}

// Every GEMV kernel has the same signature; the host picks an instance and launches it through
// a pointer, so that the planner can also ask the runtime what the instance needs (registers,
// LDS) without launching it.
typedef void (*GemvKernel)(qg_v4i, qg_v4i, qg_v4i, GemvArgs);

void launch_kernel(GemvKernel fn, unsigned blocks, unsigned threads, size_t lds, hipStream_t st, const GemvArgs &A)
{
    const FirstBlocks f = first_blocks(A);
    hipLaunchKernelGGL(fn, dim3(blocks), dim3(threads), lds, st, f.a, f.b, f.c, A);
}

template <int BITS>
GemvKernel pick_static(int cpg)
{
    switch (cpg) {
    case 1: return gemv_static<BITS, 1>;
    case 2: return gemv_static<BITS, 2>;
    case 4: return gemv_static<BITS, 4>;
    case 8: return gemv_static<BITS, 8>;
    case 16:
        if constexpr (BITS != 3) return gemv_static<BITS, 16>;
        return nullptr;
    default: return nullptr;
    }
}

template <int BITS>
GemvKernel pick_mma(int cpg)
{
    switch (cpg) {
    case 2: return gemv_mma<BITS, 2>;
    case 4: return gemv_mma<BITS, 4>;
    case 8: return gemv_mma<BITS, 8>;
    case 16:
        if constexpr (BITS != 3) return gemv_mma<BITS, 16>;
        return nullptr;
    default: return nullptr;
    }
}

// gemv_mma4 / gemv_mma4i: cpg = cells per group, 0 for groups of whole steps
template <int BITS>
GemvKernel pick_mma4(int cpg)
{
    switch (cpg) {
    case 0: return gemv_mma4<BITS, 0>;
    case 1: return gemv_mma4<BITS, 1>;
    case 2: return gemv_mma4<BITS, 2>;
    case 4: return gemv_mma4<BITS, 4>;
    case 8: return gemv_mma4<BITS, 8>;
    case 16:
        if constexpr (BITS != 3) return gemv_mma4<BITS, 16>;
        return nullptr;
    default: return nullptr;
    }
}

template <int BITS>
GemvKernel pick_mma4i(int cpg)
{
    switch (cpg) {
    case 0: return gemv_mma4i<BITS, 0>;
    case 1:
        if constexpr (BITS != 4) return gemv_mma4i<BITS, 1>;
        return nullptr;
    case 2: return gemv_mma4i<BITS, 2>;
    case 4: return gemv_mma4i<BITS, 4>;
    case 8: return gemv_mma4i<BITS, 8>;
    case 16:
        if constexpr (BITS != 3) return gemv_mma4i<BITS, 16>;
        return nullptr;
    default: return nullptr;
    }
}

template <int CPG> GemvKernel pick_rows16() { return gemm_rows16<CPG>; }

// dynamic LDS of the matrix-core kernels: the x of a step per wavefront and buffer
size_t lds_mma(int bits, unsigned threads)      // three bf16 parts
{
    const size_t S = bits == 4 ? 128 : 256;
    return (size_t)(threads / QG_WAVE) * 2 * 3 * S * sizeof(uint16_t);
}
size_t lds_mma4(int bits, unsigned threads)     // three bf16 parts and a part of zeros
{
    const size_t S = bits == 4 ? 128 : 256;
    return (size_t)(threads / QG_WAVE) * 2 * 4 * (S + 8) * sizeof(uint16_t);
}
size_t lds_mma4i(int bits, unsigned threads)    // four rows of int8 digits
{
    const size_t S = bits == 4 ? 128 : 256;
    return (size_t)(threads / QG_WAVE) * 2 * 4 * (S + 16);
}
size_t lds_rows16(unsigned threads) { return (size_t)(threads / QG_WAVE) * 16 * (128 + 8) * sizeof(uint16_t); }

// What a planned launch looks like to the machine: filled by launch_class for the search over
// launch shapes, which prices candidates before it times them.
struct LaunchShape {
    const void *kernel;
    unsigned threads, blocks;
    size_t lds_dynamic;
    long waves;                 // wavefronts with work
    size_t bytes_in_flight;     // packed bytes one wavefront has requested while it computes
};

// Which kernel multiplies: the vector ALU (gemv_static / gemv_runtime), the 32 x 32 x 16 matrix
// instruction (gemv_mma, groups of at least two cells inside a step), or the 4 x 4 x 4 one on
// bf16 (gemv_mma4) or int8 (gemv_mma4i), both for groups of whole cells inside a step and for
// groups of whole steps (gemv_mma4 not at 4 bits there; gemv_mma4i not for 4-bit groups of a
// single cell).  Measured on the three layer sets over G = 16 ... K: gemv_mma4i is ahead of
// the others nearly everywhere (2-13 % over gemv_mma4, which was 5-13 % ahead of the vector ALU
// at 2 and 3 bits).  At 4 bits with groups inside a step the vector-ALU kernel is bound by
// memory on the largest launches and level with the others or ahead, depending on the machine;
// it stays there.
enum Mul { MUL_VALU, MUL_MMA32, MUL_MMA4, MUL_MMA4I };
constexpr size_t QG_VALU4_FROM = (size_t)256 << 20;      // code bytes of a launch
Mul multiplier(int bits, int cpg, Kind kind, size_t code_bytes)
{
    if (kind != KIND_STATIC && kind != KIND_RUNTIME) return MUL_VALU;
    const int want = t_cur.kernel ? t_cur.kernel
                   : bits == 4 && kind == KIND_STATIC && code_bytes >= QG_VALU4_FROM ? 1 : 4;
    if (want == 4 && !(bits == 4 && kind == KIND_STATIC && cpg < 2)) return MUL_MMA4I;
    if (want >= 3 && (kind == KIND_STATIC || bits != 4)) return MUL_MMA4;
    if (want == 2 && kind == KIND_STATIC && cpg >= 2) return MUL_MMA32;
    return MUL_VALU;
}

// One launch for problems that share (bits, group, kernel kind).
// rows > 0: the problems are products with `rows` <= 16 activation rows (x = X [rows][K],
// y = Y [rows][N]) for gemm_rows16; the caller has checked that the kernel applies.
// dry: plan and check only -- returns the status the launch would have up to the point where
// the kernel is enqueued, and enqueues nothing.
int launch_class(const qg_gemv_desc *descs, const int *idx, int count, const size_t *ws_off,
                 char *workspace, hipStream_t st, const int64_t *gate_rows, float *const *gated,
                 int rows = 0, bool dry = false, LaunchShape *report = nullptr)
{
    GemvArgs A;
    A.count = count;
    for (int i = 0; i < QG_MAX_GROUPED; ++i) A.block_begin[i] = 0x7fffffff;
    QgLayout L[QG_MAX_GROUPED];
    Plan pl[QG_MAX_GROUPED];
    for (int i = 0; i < count; ++i) {
        const qg_gemv_desc &d = descs[idx[i]];
        qg_make_layout(d.N, d.K, d.bits, d.group, &L[i]);
        pl[i] = make_plan(L[i]);
    }
    const Kind kind = pl[0].kind;

    // Launch shape.  Every wavefront of the launch gets about the same amount of work
    // (`target` bytes of codes), so that all of them are resident at once and finish together.
    // A tile of 64 outputs is covered by a team of up to `cap` wavefronts inside one
    // workgroup (they meet in LDS); a tile whose K needs more wavefronts than that is cut
    // into 2, 4, ... workgroups that meet in the reduction tree.  Short teams are packed
    // several to a workgroup.  Launches with little work per wavefront slot use less than
    // `target` per wavefront so that the chip is still covered.
    size_t code_bytes = 0;
    for (int i = 0; i < count; ++i) code_bytes += (size_t)L[i].tiles * pl[i].items * pl[i].item_bytes;
    const int bits_all = L[0].bits;
    Mul mul = rows == 0 ? multiplier(bits_all, L[0].group / L[0].cell, kind, code_bytes) : MUL_VALU;
    const bool mma = mul != MUL_VALU;
    // wavefronts per team, at most (measured: 12 is best for the 4-bit vector-ALU kernel with
    // groups inside a step, 8 for the 2- and 3-bit ones, which hold more registers per wavefront)
    int cap = t_cur.wpb > 0 ? t_cur.wpb : (bits_all == 4 ? 12 : 8);
    if (rows > 0 && cap > 8) cap = 8;          // gemm_rows16 is built for at most 8 wavefronts
    if (mma) {                                 // the matrix-core kernels are built for at most 8 wavefronts;
        if (cap > 8) cap = 8;                  // measured: teams of 4 are best for them ...
        if (t_cur.wpb == 0) cap = 4;
    }
    size_t target = (size_t)t_cur.bytes_per_wave;               // code bytes per wavefront
    // ... except for 2- and 3-bit groups inside a step on gemv_mma4i below 192 MB of codes: there
    // teams of up to 8 with a single step per wavefront are 4-13 % ahead (7B- and 13B-shaped
    // sets; on the 65B-shaped one that shape is 0-6 % behind).  The same on gemv_mma4 for 3-bit
    // groups of up to 64 weights (8-12 % ahead on the smaller sets, level on the large one).
    const bool one_step = rows == 0 && kind == KIND_STATIC &&
                          ((mul == MUL_MMA4I && bits_all != 4 && code_bytes < ((size_t)192 << 20)) ||
                           (mul == MUL_MMA4 && bits_all == 3 && L[0].group <= 64));
    if (one_step) {
        if (t_cur.wpb == 0) cap = 8;
        if (target == 0) target = pl[0].item_bytes;
    }
    // Few, long wavefronts (teams of up to 4, about 10 wavefronts per CU, up to 48-64 KB of codes
    // each) for groups of whole steps at any width and for gemv_mma4 at 4 bits: measured 5-15 %
    // ahead of many short ones there (at 2 and 3 bits with groups inside a step the short ones
    // win, and so they do at 4 bits on the largest launches).
    const bool few_long = rows == 0 && (bits_all == 4 ? code_bytes < QG_VALU4_FROM && (mul == MUL_MMA4 || mul == MUL_MMA4I || kind == KIND_RUNTIME)
                                                      : kind == KIND_RUNTIME);
    if (few_long) {
        const size_t share = code_bytes / ((size_t)qg_compute_units() * 10);
        // (the vector-ALU kernel keeps its wider teams while a wavefront has a single step)
        if (t_cur.wpb == 0 && (mma || share > 4096)) cap = 4;
        if (target == 0) {
            size_t most = bits_all == 4 ? 65536 : 49152;
            // (groups of one or two cells: a wavefront holds at most 64 groups, and half of that
            // measured faster than all of it)
            if (kind == KIND_STATIC && pl[0].max_spw <= 8) most = (size_t)pl[0].max_spw * pl[0].item_bytes / 2;
            target = share < 4096 ? 4096 : share > most ? most : share;
        }
    }
    if (target == 0) {
        target = code_bytes / ((size_t)qg_compute_units() * 24);    // about 24 wavefronts per CU
        if (target < 4096) target = 4096;
        if (target > 16384) target = 16384;
    }

    // The limit of 64 groups per wavefront belongs to the vector-ALU kernel (it keeps x-hat one
    // group per lane); the 4 x 4 x 4 kernels form x-hat step by step and take any number of steps.
    int64_t valu_max_spw[QG_MAX_GROUPED];
    for (int i = 0; i < count; ++i) {
        valu_max_spw[i] = pl[i].max_spw;
        if (mul == MUL_MMA4 || mul == MUL_MMA4I) pl[i].max_spw = (int64_t)1 << 30;
    }

    int wpb = 1;
    int64_t spw_of[QG_MAX_GROUPED], team_of[QG_MAX_GROUPED], chunks_of[QG_MAX_GROUPED];
    auto plan_all = [&](int limit) -> bool {
        wpb = 1;
        for (int i = 0; i < count; ++i) {
            const Plan &q = pl[i];
            int64_t want = (int64_t)((target + q.item_bytes / 2) / q.item_bytes);   // items per wavefront
            if (want < 1) want = 1;
            if (want > q.max_spw) want = q.max_spw;
            // Among the ways to cover K with `chunks` (a power of two) non-empty workgroups of `team`
            // <= cap wavefronts, take the one whose items per wavefront come closest to `want`;
            // on a tie the fewest workgroups, then the smallest team.
            bool found = false;
            int64_t best_miss = 0;
            // (the many-row kernel has no reduction across workgroups)
            for (int64_t chunks = 1; chunks <= (rows > 0 ? 1 : QG_MAX_CHUNKS); chunks *= 2) {
                for (int64_t team = 1; team <= limit; ++team) {
                    const int64_t spw = (q.items + chunks * team - 1) / (chunks * team);
                    if (spw > q.max_spw) continue;
                    if ((chunks - 1) * team * spw >= q.items) continue;       // an empty workgroup
                    const int64_t miss = spw > want ? spw - want : want - spw;
                    if (!found || miss < best_miss) {
                        spw_of[i] = spw;
                        team_of[i] = team;
                        chunks_of[i] = chunks;
                        best_miss = miss;
                        found = true;
                    }
                }
            }
            if (!found) return false;
            if (team_of[i] > wpb) wpb = (int)team_of[i];
        }
        return true;
    };
    // A long K with few items per wavefront allowed (small groups) may not fit the preferred
    // team size: then the widest team the kernel is built for, then the vector-ALU kernel,
    // whose teams go up to 16 wavefronts (make_plan has checked that those cover K).
    if (!plan_all(cap)) {
        const int widest = (mma || rows > 0) ? 8 : 16;
        bool ok = cap < widest && plan_all(widest);
        if (!ok && mma) {
            mul = MUL_VALU;
            for (int i = 0; i < count; ++i) pl[i].max_spw = valu_max_spw[i];
            ok = plan_all(16);
        }
        if (!ok) return QG_ERR_UNSUPPORTED;
    }

    int blocks = 0;
    for (int i = 0; i < count; ++i) {
        const qg_gemv_desc &d = descs[idx[i]];
        GemvProblem &P = A.p[i];
        const char *base = (const char *)d.packed;
        P.codes = (const uint4 *)(base + L[i].codes_off);
        P.scales = (const float *)(base + L[i].scales_off);
        P.zeros = (const uint32_t *)(base + L[i].zeros_off);
        P.x = d.x;
        P.y = d.y;
        P.slots = (uint32_t *)(workspace + ws_off[idx[i]]);
        P.N = (int)L[i].N;
        P.K = (int)L[i].K;
        P.tiles = (int)L[i].tiles;
        P.steps = (int)L[i].steps;
        P.ngroups = (int)L[i].ngroups;
        P.zwords = (int)L[i].zwords;
        P.group = L[i].group;
        P.steps_per_group = (int)pl[i].steps_per_group;
        P.steps_per_wave = (int)spw_of[i];
        P.chunks = (int)chunks_of[i];
        P.chunk_shift = 0;
        while ((1 << P.chunk_shift) < P.chunks) ++P.chunk_shift;
        P.waves_per_tile = (int)team_of[i];
        P.inv_waves_per_tile = (65536 + P.waves_per_tile - 1) / P.waves_per_tile;
        P.team_full = (int)((pl[i].items + spw_of[i] - 1) / spw_of[i]);
        if (P.team_full > P.waves_per_tile) P.team_full = P.waves_per_tile;
        P.tiles_per_block = P.chunks > 1 ? 1 : wpb / P.waves_per_tile;
        P.pair_tiles = gate_rows ? (int)(gate_rows[idx[i]] / QG_WAVE) : 0;
        P.h = gated ? gated[idx[i]] : nullptr;
        P.rows = rows;
        P.block_begin = blocks;
        A.block_begin[i] = blocks;
        const int64_t nb = P.chunks > 1 ? (int64_t)P.tiles * P.chunks
                                        : (P.tiles + P.tiles_per_block - 1) / P.tiles_per_block;
        if (blocks + nb > 0x3fffffff) return QG_ERR_SHAPE;
        blocks += (int)nb;
    }

    const unsigned threads = (unsigned)wpb * QG_WAVE;
    const int bits = L[0].bits;
    const int cpg = L[0].group / L[0].cell;
    GemvKernel fn = nullptr;
    size_t lds = 0;
    const char *family;
    int shown_cpg = cpg;
    if (rows > 0) {
        family = "gemm_rows16";
        fn = cpg == 2 ? pick_rows16<2>() : cpg == 4 ? pick_rows16<4>() : cpg == 8 ? pick_rows16<8>() : pick_rows16<16>();
        lds = lds_rows16(threads);
    } else if (kind == KIND_STATIC) {
        if (mul == MUL_MMA4I) {
            family = "gemv_mma4i";
            fn = bits == 4 ? pick_mma4i<4>(cpg) : bits == 2 ? pick_mma4i<2>(cpg) : pick_mma4i<3>(cpg);
            lds = lds_mma4i(bits, threads);
        } else if (mul == MUL_MMA4) {
            family = "gemv_mma4";
            fn = bits == 4 ? pick_mma4<4>(cpg) : bits == 2 ? pick_mma4<2>(cpg) : pick_mma4<3>(cpg);
            lds = lds_mma4(bits, threads);
        } else if (mul == MUL_MMA32) {
            family = "gemv_mma";
            fn = bits == 4 ? pick_mma<4>(cpg) : bits == 2 ? pick_mma<2>(cpg) : pick_mma<3>(cpg);
            lds = lds_mma(bits, threads);
        } else {
            family = "gemv_static";
            fn = bits == 4 ? pick_static<4>(cpg) : bits == 2 ? pick_static<2>(cpg) : pick_static<3>(cpg);
        }
        if (!fn) return QG_ERR_UNSUPPORTED;            // no kernel was built for this group size
    } else if (kind == KIND_RUNTIME && mul == MUL_MMA4I) {
        family = "gemv_mma4i";
        shown_cpg = 0;
        fn = bits == 2 ? pick_mma4i<2>(0) : bits == 3 ? pick_mma4i<3>(0) : pick_mma4i<4>(0);
        lds = lds_mma4i(bits, threads);
    } else if (kind == KIND_RUNTIME && mul == MUL_MMA4) {
        family = "gemv_mma4";
        shown_cpg = 0;
        fn = bits == 2 ? pick_mma4<2>(0) : pick_mma4<3>(0);
        lds = lds_mma4(bits, threads);
    } else if (kind == KIND_RUNTIME) {
        family = "gemv_runtime";
        shown_cpg = -1;
        fn = bits == 4 ? gemv_runtime<4> : bits == 2 ? gemv_runtime<2> : gemv_runtime<3>;
    } else {
        family = "gemv_generic";
        shown_cpg = -1;
        fn = bits == 4 ? gemv_generic<4> : bits == 2 ? gemv_generic<2> : gemv_generic<3>;
    }
    if (report) {
        report->kernel = (const void *)fn;
        report->threads = threads;
        report->blocks = (unsigned)blocks;
        report->lds_dynamic = lds;
        long waves = 0;
        size_t in_flight = 0;
        for (int i = 0; i < count; ++i) {
            const int64_t per_tile = (pl[i].items + spw_of[i] - 1) / spw_of[i];
            waves += (long)(L[i].tiles * per_tile);
            // two register buffers: the step being computed has arrived, the next one is in flight
            const size_t mine = (size_t)(spw_of[i] > 1 ? 2 : 1) * pl[i].item_bytes;
            if (mine > in_flight) in_flight = mine;
        }
        report->waves = waves;
        report->bytes_in_flight = in_flight;
    }
    if (dry) return QG_OK;
    if (shown_cpg >= 0) snprintf(g_last_kernel, sizeof g_last_kernel, "%s<%d, %d>", family, bits, shown_cpg);
    else snprintf(g_last_kernel, sizeof g_last_kernel, "%s<%d>", family, bits);
    launch_kernel(fn, (unsigned)blocks, threads, lds, st, A);
    return qg_launch_status();
}

}  // namespace

extern "C" const char *qg_last_gemv_kernel(void) { return g_last_kernel; }

extern "C" int qg_set_gemv_tuning(int waves_per_block, int bytes_per_wave, int kernel)
{
    if (waves_per_block < 0 || waves_per_block > 16 || bytes_per_wave < 0 || kernel < 0 || kernel > 4)
        return QG_ERR_SHAPE;
    g_tune_wpb = waves_per_block;
    g_tune_bytes_per_wave = bytes_per_wave;
    g_tune_kernel = kernel;
    return QG_OK;
}

extern "C" int qg_gemv_record_tuning(const qg_gemv_desc *descs, int count, int waves_per_block,
                                     int bytes_per_wave, int kernel)
{
    if (!descs) return QG_ERR_NULL;
    if (count <= 0 || waves_per_block < 0 || waves_per_block > 16 || bytes_per_wave < 0 || kernel < 0 || kernel > 4)
        return QG_ERR_SHAPE;
    if (count > QG_MAX_GROUPED) return QG_ERR_UNSUPPORTED;
    record_tuning(descs, count, {waves_per_block, bytes_per_wave, kernel});
    return QG_OK;
}

void qg_gemm_clear_tuning();     // qg_gemm_small.hip

extern "C" void qg_clear_tuning(void)
{
    {
        std::lock_guard<std::mutex> lock(g_tune_mutex);
        g_tune_count = 0;
        g_tune_next = 0;
    }
    qg_gemm_clear_tuning();
}

size_t qg_gemm_workspace_bytes(const QgLayout &L, int M);   // qg_gemm_small.hip

extern "C" size_t qg_workspace_bytes(int64_t N, int64_t K, int bits, int group, int M)
{
    QgLayout L;
    if (M <= 0 || qg_make_layout(N, K, bits, group, &L) != QG_OK) return 0;
    return M == 1 ? workspace_for(L) : qg_gemm_workspace_bytes(L, M);
}

extern "C" int qg_workspace_init(void *workspace, size_t bytes, void *stream)
{
    if (!workspace) return QG_ERR_NULL;
    if (((uintptr_t)workspace & 3u) || (bytes & 3u)) return QG_ERR_ALIGN;
    const size_t n = bytes / 4;
    if (n == 0) return QG_OK;
    hipLaunchKernelGGL(fill_u32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                       (hipStream_t)stream, (uint32_t *)workspace, n, QG_SLOT_EMPTY);
    return qg_launch_status();
}

// gate_rows / gated: per problem, the number of gate outputs and the result vector of a gated
// pair (0 / unused for a plain product); both NULL for plain launches.
// check_only: argument checks and planning, nothing enqueued.
static int gemv_grouped(const qg_gemv_desc *descs, int count, void *workspace, size_t workspace_bytes,
                        void *stream, const int64_t *gate_rows, float *const *gated, bool check_only = false,
                        LaunchShape *report = nullptr)       // report: the shape of the call's largest launch
{
    if (!descs) return QG_ERR_NULL;
    if (count <= 0) return QG_ERR_SHAPE;
    if (count > QG_MAX_GROUPED) return QG_ERR_UNSUPPORTED;
    size_t ws_off[QG_MAX_GROUPED];
    size_t need = 0;
    for (int i = 0; i < count; ++i) {
        QgLayout L;
        const int rc = qg_make_layout(descs[i].N, descs[i].K, descs[i].bits, descs[i].group, &L);
        if (rc != QG_OK) return rc;
        const bool pair = gate_rows && gate_rows[i] > 0;
        if (!descs[i].packed || !descs[i].x || !(pair ? (const void *)gated[i] : (const void *)descs[i].y))
            return QG_ERR_NULL;
        // x is read with 64-byte scalar loads
        if (!qg_aligned16(descs[i].packed) || ((uintptr_t)descs[i].x & 63u)) return QG_ERR_ALIGN;
        ws_off[i] = need;
        need += workspace_for(L);
    }
    if (!workspace || workspace_bytes < need) return QG_ERR_WORKSPACE;
    if (!qg_aligned16(workspace)) return QG_ERR_ALIGN;
    t_cur = tuning_for(descs, count);

    // one launch per distinct (bits, kernel kind), and per group size where the kernel has it
    // as a compile-time constant.  Two passes: the first plans every class and launches
    // nothing, so that an error leaves nothing enqueued; the second launches.
    for (int pass = 0; pass < (check_only ? 1 : 2); ++pass) {
        bool done[QG_MAX_GROUPED] = {false};
        for (int i = 0; i < count; ++i) {
            if (done[i]) continue;
            QgLayout Li;
            qg_make_layout(descs[i].N, descs[i].K, descs[i].bits, descs[i].group, &Li);
            int idx[QG_MAX_GROUPED], n = 0;
            for (int j = i; j < count; ++j) {
                if (done[j]) continue;
                QgLayout Lj;
                qg_make_layout(descs[j].N, descs[j].K, descs[j].bits, descs[j].group, &Lj);
                const Kind ki = make_plan(Li).kind;
                if (Lj.bits == Li.bits && make_plan(Lj).kind == ki && (ki != KIND_STATIC || Lj.group == Li.group)) {
                    idx[n++] = j;
                    done[j] = true;
                }
            }
            // longest K first: its wavefronts run longest, so they should start first
            for (int a = 1; a < n; ++a)
                for (int b = a; b > 0 && descs[idx[b]].K > descs[idx[b - 1]].K; --b) {
                    const int t = idx[b]; idx[b] = idx[b - 1]; idx[b - 1] = t;
                }
            LaunchShape shape;
            const int rc = launch_class(descs, idx, n, ws_off, (char *)workspace, (hipStream_t)stream,
                                        gate_rows, gated, 0, pass == 0, report ? &shape : nullptr);
            if (rc != QG_OK) return rc;
            if (report && pass == 0 && (i == 0 || shape.waves > report->waves)) *report = shape;
        }
    }
    return QG_OK;
}

extern "C" int qg_gemv_grouped(const qg_gemv_desc *descs, int count, void *workspace,
                               size_t workspace_bytes, void *stream)
{
    return gemv_grouped(descs, count, workspace, workspace_bytes, stream, nullptr, nullptr);
}

// Argument checks and planning of a grouped launch without enqueuing anything (for callers in
// this library that make several launches and must not fail between them).
int qg_gemv_grouped_check(const qg_gemv_desc *descs, int count, void *workspace, size_t workspace_bytes)
{
    return gemv_grouped(descs, count, workspace, workspace_bytes, nullptr, nullptr, nullptr, true);
}

// Y = X What^T for M <= 16 rows on the GEMV's launch structure (used by qg_gemm_small).
// Returns QG_ERR_UNSUPPORTED if the shape is not one gemm_rows16 takes; the arguments have
// been checked by the caller.  dry: plan only, nothing enqueued.
int qg_gemm_rows16(const void *packed, int64_t N, int64_t K, int bits, int group, const float *X,
                   int M, float *Y, void *workspace, void *stream, bool dry)
{
    QgLayout L;
    if (qg_make_layout(N, K, bits, group, &L) != QG_OK) return QG_ERR_UNSUPPORTED;
    const Plan pl = make_plan(L);
    const int cpg = group / L.cell;
    if (bits != 4 || M < 1 || M > 16 || pl.kind != KIND_STATIC || cpg < 2) return QG_ERR_UNSUPPORTED;
    if ((int64_t)M * K >= ((int64_t)1 << 31)) return QG_ERR_UNSUPPORTED;
    qg_gemv_desc d;
    d.packed = packed;
    d.N = N;
    d.K = K;
    d.bits = bits;
    d.group = group;
    d.x = X;
    d.y = Y;
    const int idx = 0;
    const size_t ws_off = 0;
    t_cur = {g_tune_wpb, g_tune_bytes_per_wave, g_tune_kernel};
    return launch_class(&d, &idx, 1, &ws_off, (char *)workspace, (hipStream_t)stream, nullptr, nullptr, M, dry);
}

extern "C" int qg_gemv_swiglu(const void *packed, int64_t I, int64_t K, int bits, int group,
                              const float *x, float *h, void *workspace, size_t workspace_bytes,
                              void *stream)
{
    if (I <= 0 || I % QG_WAVE != 0) return QG_ERR_SHAPE;
    qg_gemv_desc d;
    d.packed = packed;
    d.N = 2 * I;
    d.K = K;
    d.bits = bits;
    d.group = group;
    d.x = x;
    d.y = nullptr;
    const int64_t gate_rows = I;
    float *const gated = h;
    return gemv_grouped(&d, 1, workspace, workspace_bytes, stream, &gate_rows, &gated);
}

// ---- qg_gemv for callers that cannot allocate -------------------------------------------
// The meeting slots of the K-split live in a file-scope device array instead of a caller's
// workspace.  Each GPU holds its own copy of the array at its own address: the address is
// asked from the runtime once per device, with that device current, and only that pointer is
// ever handed to kernels (the array's name is a host-side stand-in, not a device address).
static __device__ __align__(256) uint32_t scratch[QG_NOALLOC_SCRATCH_BYTES / sizeof(uint32_t)];

namespace {
std::mutex g_scratch_lock;
uint32_t *g_scratch_ptr[64];          // per device; nullptr until asked

// Device address of `scratch` on the current device, or nullptr with *status set.
uint32_t *scratch_of_current_device(int *status)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) { *status = QG_ERR_DEVICE; return nullptr; }
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        uint32_t *ptr = nullptr;
        if (hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            *status = QG_ERR_DEVICE;
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" int qg_gemv_noalloc(const void *packed, int64_t N, int64_t K, int bits, int group,
                               const float *x, float *y, void *stream)
{
    QgLayout L;
    const int rc = qg_make_layout(N, K, bits, group, &L);
    if (rc != QG_OK) return rc;
    const size_t need = workspace_for(L);
    if (need > QG_NOALLOC_SCRATCH_BYTES) return QG_ERR_WORKSPACE;      // more outputs than the scratch has slots for
    qg_gemv_desc d;
    d.packed = packed;
    d.N = N;
    d.K = K;
    d.bits = bits;
    d.group = group;
    d.x = x;
    d.y = y;
    int status = QG_OK;
    uint32_t *ptr = scratch_of_current_device(&status);
    if (!ptr) return status;
    // argument checks and planning first, so that an error leaves nothing enqueued
    const int checked = gemv_grouped(&d, 1, ptr, need, stream, nullptr, nullptr, true);
    if (checked != QG_OK) return checked;
    // The array keeps whatever the last call on this GPU left: the slots this call may use are
    // put into the "empty" state by a fill kernel (not a memset node, so a caller may capture it).
    const size_t words = need / sizeof(uint32_t);
    hipLaunchKernelGGL(fill_u32, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       ptr, words, QG_SLOT_EMPTY);
    if (qg_launch_status() != QG_OK) return QG_ERR_DEVICE;
    return gemv_grouped(&d, 1, ptr, need, stream, nullptr, nullptr);
}

extern "C" int qg_gemv(const void *packed, int64_t N, int64_t K, int bits, int group,
                       const float *x, float *y, void *workspace, size_t workspace_bytes,
                       void *stream)
{
    qg_gemv_desc d;
    d.packed = packed;
    d.N = N;
    d.K = K;
    d.bits = bits;
    d.group = group;
    d.x = x;
    d.y = y;
    return qg_gemv_grouped(&d, 1, workspace, workspace_bytes, stream);
}

// Choice of the launch shape for one grouped launch: the counterpart of the paper's parameter
// search (Section 3, Algorithm 4 with the model of eqs. (3)-(5)).  The paper bounds its block
// sizes by what the cache and the register file hold; here a candidate (team size, bytes per
// wavefront, kernel) is first priced against this machine's budget -- the registers per lane
// and the LDS per workgroup of the kernel instance give the wavefronts a compute unit can hold,
// those times the bytes a wavefront keeps requested give the bytes in flight per unit, and a
// candidate that cannot keep the memory system's round trip covered is dropped -- and only the
// survivors are timed; the fastest is recorded for launches with this list of shapes (as the
// paper's search result is kept per matrix size).  Unlike every other call this one waits for
// the GPU.
namespace {
constexpr int AT_TEAMS[] = {0, 2, 4, 8, 12, 16};
constexpr int AT_SIZES[] = {0, 4096, 8192, 16384, 32768, 49152, 65536};
constexpr int AT_NT = sizeof(AT_TEAMS) / sizeof(AT_TEAMS[0]), AT_NS = sizeof(AT_SIZES) / sizeof(AT_SIZES[0]);
constexpr int AT_CANDIDATES = 4 * AT_NT * AT_NS;
float g_at_us[AT_CANDIDATES];        // microseconds per launch; -1: dropped by the budget
int g_at_timed = 0, g_at_dropped = 0;

constexpr double AT_HBM_BYTES_PER_S = 8e12;      // MI355X peak
constexpr double AT_ROUND_TRIP_S = 1.5e-6;       // a request's way to HBM and back under load (measured)
constexpr size_t AT_LDS_PER_CU = 160 * 1024;
constexpr int AT_VGPRS_PER_SIMD = 512, AT_MAX_WAVES_PER_SIMD = 8;

// Wavefronts of this kernel instance one compute unit can hold.
int resident_waves_per_cu(const LaunchShape &sh)
{
    hipFuncAttributes attr;
    if (hipFuncGetAttributes(&attr, sh.kernel) != hipSuccess) {
        (void)hipGetLastError();
        return 4 * AT_MAX_WAVES_PER_SIMD;
    }
    const int waves_per_wg = (int)(sh.threads / QG_WAVE);
    const int regs = ((attr.numRegs > 0 ? attr.numRegs : 64) + 7) / 8 * 8;       // allocated in blocks of 8
    int per_simd = AT_VGPRS_PER_SIMD / regs;
    if (per_simd > AT_MAX_WAVES_PER_SIMD) per_simd = AT_MAX_WAVES_PER_SIMD;
    if (per_simd < 1) per_simd = 1;
    int wgs = per_simd * 4 / waves_per_wg;                    // a workgroup's wavefronts are dealt over the four SIMDs
    const size_t lds = attr.sharedSizeBytes + sh.lds_dynamic;
    if (lds > 0 && (int)(AT_LDS_PER_CU / lds) < wgs) wgs = (int)(AT_LDS_PER_CU / lds);
    if (wgs < 1) wgs = 1;
    return wgs * waves_per_wg;
}

// Packed bytes the launch keeps requested per compute unit while it streams.
double bytes_in_flight_per_cu(const LaunchShape &sh)
{
    const int cus = qg_compute_units();
    const long share = (sh.waves + cus - 1) / cus;            // wavefronts the launch has per unit
    const int resident = resident_waves_per_cu(sh);
    return (double)(share < resident ? share : resident) * (double)sh.bytes_in_flight;
}
}  // namespace

extern "C" int qg_gemv_autotune(const qg_gemv_desc *descs, int count, int sets, void *workspace,
                                size_t workspace_bytes, void *stream, int repeats,
                                int *waves_per_block, int *bytes_per_wave, int *kernel,
                                float *best_us)
{
    if (repeats <= 0 || sets <= 0) return QG_ERR_SHAPE;
    if (!descs) return QG_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    const int saved[3] = {g_tune_wpb, g_tune_bytes_per_wave, g_tune_kernel};
    auto restore = [&]() { g_tune_wpb = saved[0]; g_tune_bytes_per_wave = saved[1]; g_tune_kernel = saved[2]; };
    int rc = QG_OK;
    for (int s = 0; s < sets && rc == QG_OK; ++s)                                  // argument checks
        rc = gemv_grouped(descs + (size_t)s * count, count, workspace, workspace_bytes, stream, nullptr, nullptr, true);
    if (rc != QG_OK) return rc;

    // 1. price every candidate: plan it (nothing is launched) and ask what its kernel instance needs
    double in_flight[AT_CANDIDATES], most = 0.0;
    for (int c = 0; c < AT_CANDIDATES && rc == QG_OK; ++c) {
        g_tune_kernel = 1 + c / (AT_NT * AT_NS);
        g_tune_wpb = AT_TEAMS[(c / AT_NS) % AT_NT];
        g_tune_bytes_per_wave = AT_SIZES[c % AT_NS];
        LaunchShape sh;
        rc = gemv_grouped(descs, count, workspace, workspace_bytes, stream, nullptr, nullptr, true, &sh);
        if (rc != QG_OK) break;
        in_flight[c] = bytes_in_flight_per_cu(sh);
        if (in_flight[c] > most) most = in_flight[c];
    }
    if (rc != QG_OK) { restore(); return rc; }
    // what a unit has to keep requested to cover the round trip at the peak rate; a launch too
    // small to get there anyway is held to half of what its best candidate reaches
    double need = AT_HBM_BYTES_PER_S * AT_ROUND_TRIP_S / qg_compute_units();
    if (need > 0.5 * most) need = 0.5 * most;

    // 2. time the survivors
    int turn = 0;
    auto run = [&]() {
        const qg_gemv_desc *d = descs + (size_t)(turn++ % sets) * count;
        return qg_gemv_grouped(d, count, workspace, workspace_bytes, stream);
    };
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) { restore(); return QG_ERR_DEVICE; }
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); restore(); return QG_ERR_DEVICE; }
    int best = -1;
    float best_ms = -1.0f;
    g_at_timed = 0;
    g_at_dropped = 0;
    for (int c = 0; c < AT_CANDIDATES && rc == QG_OK; ++c) {
        if (in_flight[c] < need) {
            g_at_us[c] = -1.0f;
            ++g_at_dropped;
            continue;
        }
        g_tune_kernel = 1 + c / (AT_NT * AT_NS);
        g_tune_wpb = AT_TEAMS[(c / AT_NS) % AT_NT];
        g_tune_bytes_per_wave = AT_SIZES[c % AT_NS];
        for (int i = 0; i < 2 && rc == QG_OK; ++i) rc = run();
        if (rc != QG_OK) break;
        if (hipEventRecord(e0, st) != hipSuccess) { rc = QG_ERR_DEVICE; break; }
        for (int i = 0; i < repeats && rc == QG_OK; ++i) rc = run();
        if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) rc = QG_ERR_DEVICE;
        float ms = 0.0f;
        if (rc == QG_OK && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = QG_ERR_DEVICE;
        if (rc != QG_OK) break;
        g_at_us[c] = ms * 1e3f / (float)repeats;
        ++g_at_timed;
        if (best < 0 || ms < best_ms) {
            best_ms = ms;
            best = c;
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != QG_OK || best < 0) {
        restore();
        return rc != QG_OK ? rc : QG_ERR_DEVICE;
    }
    const Tuning won = {AT_TEAMS[(best / AT_NS) % AT_NT], AT_SIZES[best % AT_NS], 1 + best / (AT_NT * AT_NS)};
    restore();
    record_tuning(descs, count, won);
    if (waves_per_block) *waves_per_block = won.wpb;
    if (bytes_per_wave) *bytes_per_wave = won.bytes_per_wave;
    if (kernel) *kernel = won.kernel;
    if (best_us) *best_us = best_ms * 1e3f / (float)repeats;
    return QG_OK;
}

extern "C" int qg_gemv_autotune_report(float *us, int capacity, int *timed, int *dropped)
{
    if (us) {
        if (capacity < AT_CANDIDATES) return QG_ERR_SHAPE;
        for (int c = 0; c < AT_CANDIDATES; ++c) us[c] = g_at_us[c];
    }
    if (timed) *timed = g_at_timed;
    if (dropped) *dropped = g_at_dropped;
    return QG_OK;
}
