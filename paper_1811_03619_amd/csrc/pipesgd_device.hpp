// Device-side building blocks of libpipesgd's kernels (gfx950 / CDNA4): tile and
// workgroup geometry, cache-policy helpers, the kernel argument structures, the
// block-to-tile addressing, the block-wide maximum, the codecs of Sec. 3.2 of the
// paper (arXiv 1811.03619) and the vectorised unit loads and stores.  Private to
// pipesgd_kernels.hip, which includes it once; everything sits in that
// translation unit's anonymous namespace.
#pragma once

#include <hip/hip_runtime.h>

#include <cfloat>
#include <cstdint>

#include "pipesgd.h"

#pragma clang fp contract(off)

namespace {

constexpr int kTile = PIPESGD_QBLOCK;        // elements per tile
constexpr int kTileQuads = kTile / 4;
constexpr int kMaxW = PIPESGD_MAX_WORKERS;
constexpr int kMaxB = PIPESGD_MAX_BUCKETS;

// Which quads of a unit a thread owns.  Strided (the default): quad i of thread t
// is quad i*THREADS + t, so every load instruction of a wave covers one contiguous
// run.  Lane-contiguous (build with -DPIPESGD_LANE_CONTIGUOUS=1): quad i of thread t
// is quad t*QUADS + i, so a thread's 16-bit (QUADS = 2) or 8-bit (QUADS = 4) payload
// is ONE 128-bit load, at the price of fp32 loads whose lanes sit 32 or 64 bytes
// apart.  Measured slower on MI355X (16-bit update at 61M elements: 5.8 TB/s with
// QUADS = 2 and 3.4 TB/s with QUADS = 4, against 6.5 TB/s strided; the hop kernels
// lose 4-11 %), so it is off; kept as a build option because results do not depend
// on it (the parity tests pass with either).
#ifndef PIPESGD_LANE_CONTIGUOUS
#define PIPESGD_LANE_CONTIGUOUS 0
#endif

// Workgroup geometry.  kUnit elements per workgroup; kSplit units per tile.
template <int THREADS, int QUADS> struct Geo {
    static constexpr int kThreads = THREADS;
    static constexpr int kQuads = QUADS;
    static constexpr int kPerThread = 4 * QUADS;
    static constexpr int kUnit = THREADS * QUADS * 4;
    static constexpr int kSplit = kTile / kUnit;
    static constexpr int kWaves = THREADS / 64;
    static constexpr bool kContig = PIPESGD_LANE_CONTIGUOUS != 0;
    static_assert(THREADS % 64 == 0 && kUnit <= kTile && kTile % kUnit == 0, "geometry");
    // index, within the unit, of the i-th quad this thread owns
    __device__ static __forceinline__ uint32_t quad(int i)
    {
        return kContig ? threadIdx.x * QUADS + i : i * THREADS + threadIdx.x;
    }
};

// ------------------------------------------------- streaming memory access --
// Native vector types (the nontemporal builtins take these, not HIP's structs).
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Cache policy per stream.  "Streamed" data is touched once per launch and not
// again soon: loading/storing it with the nontemporal hint keeps it from
// displacing the hop payloads, which ARE re-read by the next launch.
#ifndef PIPESGD_NT_GRAD
#define PIPESGD_NT_GRAD 1        // local gradients: read once per iteration
#endif
#ifndef PIPESGD_NT_PAYIN
#define PIPESGD_NT_PAYIN 1       // incoming hop payload: this is its last use
#endif
#ifndef PIPESGD_NT_PAYOUT
#define PIPESGD_NT_PAYOUT 0      // outgoing hop payload: the next round reads it
#endif
#ifndef PIPESGD_NT_UPDATE
#define PIPESGD_NT_UPDATE 1      // slot, w, v of the update: 2 GB streamed once
#endif
#ifndef PIPESGD_NT_CODEC_OUT
#define PIPESGD_NT_CODEC_OUT 0   // output of the stand-alone codec calls: the hint costs 5-10 % while the output
                                 // fits the memory-side cache (up to ~0.5 GB) and gains 5 % at 1.1 GB
#endif
constexpr bool kNtGrad = PIPESGD_NT_GRAD, kNtPayIn = PIPESGD_NT_PAYIN, kNtPayOut = PIPESGD_NT_PAYOUT,
               kNtUpdate = PIPESGD_NT_UPDATE, kNtCodecOut = PIPESGD_NT_CODEC_OUT;

template <bool NT, typename V> __device__ __forceinline__ V ld(const V *p)
{
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}
template <bool NT, typename V> __device__ __forceinline__ void st(V *p, V x)
{
    if (NT) __builtin_nontemporal_store(x, p); else *p = x;
}

// ------------------------------------------------------------ kernel args --

// Bucket geometry, passed by value (lives in the kernarg segment, read with
// scalar loads).  A "slot" is a tile position inside one ring block: bucket b
// contributes ce_tiles[b] slots; worker/chunk selection happens per launch.
struct BucketTable {
    uint32_t count;
    uint32_t slot_prefix[kMaxB + 1];
    uint32_t ce_tiles[kMaxB];
    uint64_t start[kMaxB];
    uint64_t n[kMaxB];
};

// One launch of a ring kernel.  Worker r (blockIdx.y) handles chunk
// (r - chunk_rot - blockIdx.z) mod p, tile slots [slot_base, slot_base + gridDim.x / split).
struct RingArgs {
    const float *g[kMaxW];      // local gradients
    const void *in[kMaxW];      // payload worker r receives: the sender's slot, or r's own receive staging
    const float *in_sc[kMaxW];
    void *out[kMaxW];           // payload worker r writes
    float *out_sc[kMaxW];
    int p;
    int chunk_rot;
    uint32_t slot_base;
    uint32_t units;             // copy kernel only: units to cover (gridDim.x may be smaller: a throttled link)
};

struct UpdateArgs {
    const void *pay[kMaxW];
    const float *sc[kMaxW];
    float *w[kMaxW];
    float *v[kMaxW];
    uint64_t n;
    float lr, momentum, grad_scale;
};

// The full/short decision and the short length are deliberately kept as two
// separate values (a flag and a plain truncation) instead of one clamped length:
// the kernels branch on `full` once and the short body reads `len` as is.
struct UnitRef {
    uint64_t elem0;     // first element, packed-buffer coordinates
    uint32_t len;       // elements to process; meaningful only when !full (then 1..kUnit-1)
    bool full;          // a whole unit of kUnit elements
    bool empty;         // nothing to do
};

__device__ __forceinline__ int mod_p(int a, int p)
{
    int m = a % p;
    return m < 0 ? m + p : m;
}

// blockIdx.x -> (bucket, tile of chunk `chunk`, unit of that tile).  All
// operands are wave-uniform.
template <class G>
__device__ __forceinline__ UnitRef locate(const BucketTable &bt, uint32_t block, int chunk)
{
    const uint32_t slot = block / G::kSplit;
    const uint32_t sub = block % G::kSplit;
    uint32_t lo = 0, hi = bt.count;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (bt.slot_prefix[mid] <= slot) lo = mid; else hi = mid;
    }
    const uint64_t ce = static_cast<uint64_t>(bt.ce_tiles[lo]) * kTile;
    const uint64_t t = slot - bt.slot_prefix[lo];
    const uint64_t nb = bt.n[lo];
    const uint64_t lo_e = static_cast<uint64_t>(chunk) * ce + t * kTile + static_cast<uint64_t>(sub) * G::kUnit;
    uint64_t hi_e = (static_cast<uint64_t>(chunk) + 1) * ce;
    if (hi_e > nb) hi_e = nb;
    UnitRef r;
    r.empty = lo_e >= hi_e;
    r.elem0 = bt.start[lo] + lo_e;
    const uint64_t rem = hi_e - lo_e;
    r.full = rem >= static_cast<uint64_t>(G::kUnit);
    r.len = static_cast<uint32_t>(rem);
    return r;
}

// Addressing-only geometry: UNIT elements per workgroup.
template <int UNIT> struct UnitOnly {
    static constexpr int kUnit = UNIT;
    static constexpr int kSplit = kTile / UNIT;
    static_assert(UNIT <= kTile && kTile % UNIT == 0, "unit");
};

// Unit of a flat vector.
template <class G>
__device__ __forceinline__ UnitRef locate_flat(uint64_t n, uint32_t block)
{
    UnitRef r;
    r.elem0 = static_cast<uint64_t>(block) * G::kUnit;
    const uint64_t rem = n - r.elem0;           // the grid has ceil(n / kUnit) blocks: rem >= 1
    r.empty = false;
    r.full = rem >= static_cast<uint64_t>(G::kUnit);
    r.len = static_cast<uint32_t>(rem);
    return r;
}

// ------------------------------------------------------- block-wide max --

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// red: one float of LDS per wavefront.  One barrier per call; callers that
// reduce repeatedly alternate between two such arrays.
template <class G>
__device__ __forceinline__ float block_max(float v, float *red)
{
    v = wave_max(v);
    if (G::kWaves == 1) return v;
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float m = red[0];
#pragma unroll
    for (int i = 1; i < G::kWaves; ++i) m = fmaxf(m, red[i]);
    return m;
}

// ----------------------------------------------------------------- codecs --
// Sec. 3.2 of the paper.  MODE is one of PIPESGD_NONE / TRUNC16 / QUANT8.

__device__ __forceinline__ uint32_t f2u(float x) { return __float_as_uint(x); }
__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }

// 127/scale with the saturation that keeps codes finite for scales below
// 127/FLT_MAX; 0 for an all-zero block (every code is then 0).
__device__ __forceinline__ float quant_inverse(float scale)
{
    if (scale == 0.0f) return 0.0f;
    const float inv = 127.0f / scale;
    return inv > FLT_MAX ? FLT_MAX : inv;
}
__device__ __forceinline__ int quant_code(float x, float inv)
{
    const int q = static_cast<int>(rintf(x * inv));      // ties to even
    return min(max(q, -127), 127);
}
__device__ __forceinline__ int sext8(uint32_t u, int byte)
{
    return static_cast<int>(u << (24 - 8 * byte)) >> 24;
}

template <int MODE> struct Codec;

template <> struct Codec<PIPESGD_NONE> {
    using Raw = f32x4;
    static constexpr int kBytes = 4;
    __device__ static void decode(const Raw &r, float, float *x) { x[0] = r.x; x[1] = r.y; x[2] = r.z; x[3] = r.w; }
    __device__ static Raw encode(const float *x, float) { return Raw{x[0], x[1], x[2], x[3]}; }
    __device__ static float decode1(const void *pay, uint64_t i, float) { return static_cast<const float *>(pay)[i]; }
    __device__ static void encode1(void *pay, uint64_t i, float x, float) { static_cast<float *>(pay)[i] = x; }
};

template <> struct Codec<PIPESGD_TRUNC16> {
    using Raw = u32x2;                                      // four uint16, little endian
    static constexpr int kBytes = 2;
    __device__ static void decode(const Raw &r, float, float *x)
    {
        x[0] = u2f(r.x << 16); x[1] = u2f(r.x & 0xffff0000u);
        x[2] = u2f(r.y << 16); x[3] = u2f(r.y & 0xffff0000u);
    }
    __device__ static Raw encode(const float *x, float)
    {
        return Raw{(f2u(x[0]) >> 16) | (f2u(x[1]) & 0xffff0000u),
                   (f2u(x[2]) >> 16) | (f2u(x[3]) & 0xffff0000u)};
    }
    __device__ static float decode1(const void *pay, uint64_t i, float)
    {
        return u2f(static_cast<uint32_t>(static_cast<const uint16_t *>(pay)[i]) << 16);
    }
    __device__ static void encode1(void *pay, uint64_t i, float x, float)
    {
        static_cast<uint16_t *>(pay)[i] = static_cast<uint16_t>(f2u(x) >> 16);
    }
};

template <> struct Codec<PIPESGD_QUANT8> {
    using Raw = uint32_t;                                   // four int8
    static constexpr int kBytes = 1;
    // `step` = scale/127 when decoding, `inv` = quant_inverse(scale) when encoding
    __device__ static void decode(const Raw &r, float step, float *x)
    {
        x[0] = static_cast<float>(sext8(r, 0)) * step; x[1] = static_cast<float>(sext8(r, 1)) * step;
        x[2] = static_cast<float>(sext8(r, 2)) * step; x[3] = static_cast<float>(sext8(r, 3)) * step;
    }
    __device__ static Raw encode(const float *x, float inv)
    {
        const uint32_t a = quant_code(x[0], inv) & 0xff, b = quant_code(x[1], inv) & 0xff;
        const uint32_t c = quant_code(x[2], inv) & 0xff, d = quant_code(x[3], inv) & 0xff;
        return a | (b << 8) | (c << 16) | (d << 24);
    }
    __device__ static float decode1(const void *pay, uint64_t i, float step)
    {
        return static_cast<float>(static_cast<const int8_t *>(pay)[i]) * step;
    }
    __device__ static void encode1(void *pay, uint64_t i, float x, float inv)
    {
        static_cast<int8_t *>(pay)[i] = static_cast<int8_t>(quant_code(x, inv));
    }
};

// Lane-contiguous layout: when a thread's QUADS consecutive quads of payload make
// up exactly 16 bytes they travel as one 128-bit vector.
template <class C, class G>
constexpr bool kWide128 = G::kContig && sizeof(typename C::Raw) * G::kQuads == 16 && sizeof(typename C::Raw) < 16;

template <class C> __device__ __forceinline__ void split128(const u32x4 &q, typename C::Raw *r)
{
    if constexpr (sizeof(typename C::Raw) == 8) { r[0] = typename C::Raw{q.x, q.y}; r[1] = typename C::Raw{q.z, q.w}; }
    else { r[0] = q.x; r[1] = q.y; r[2] = q.z; r[3] = q.w; }
}
template <class C> __device__ __forceinline__ u32x4 join128(const typename C::Raw *r)
{
    if constexpr (sizeof(typename C::Raw) == 8) return u32x4{r[0].x, r[0].y, r[1].x, r[1].y};
    else return u32x4{r[0], r[1], r[2], r[3]};
}

// ------------------------------------------------------- unit load / store --
// x[4*QUADS] of a thread: x[4*i + e] = element 4*G::quad(i) + e of the unit.  The *_full variants assume a whole, 16-byte aligned unit; the *_tail
// variants guard every element against `len` and fill the rest with zero.
// FULL is a template parameter everywhere: a kernel decides once per workgroup
// which body to run, so that in the full body nothing separates the loads and
// they are all in flight together.

template <class G, bool NT>
__device__ __forceinline__ void load_f32_full(const float *base, float *x)
{
    const f32x4 *v = reinterpret_cast<const f32x4 *>(base);
    f32x4 r[G::kQuads];
#pragma unroll
    for (int i = 0; i < G::kQuads; ++i) r[i] = ld<NT>(v + G::quad(i));
#pragma unroll
    for (int i = 0; i < G::kQuads; ++i) { x[4 * i] = r[i].x; x[4 * i + 1] = r[i].y; x[4 * i + 2] = r[i].z; x[4 * i + 3] = r[i].w; }
}
// Short units (1 <= len < kUnit): every lane loads from an index clamped into
// the unit and the out-of-range values are replaced afterwards, so the loads
// carry no branches and are all in flight together here too.
template <class G>
__device__ __forceinline__ void load_f32_tail(const float *base, uint32_t len, float *x)
{
    float r[G::kPerThread];
#pragma unroll
    for (int i = 0; i < G::kQuads; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t idx = 4 * G::quad(i) + e;
            r[4 * i + e] = base[min(idx, len - 1)];
        }
#pragma unroll
    for (int i = 0; i < G::kQuads; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t idx = 4 * G::quad(i) + e;
            x[4 * i + e] = idx < len ? r[4 * i + e] : 0.0f;
        }
}
template <class G, bool FULL, bool NT>
__device__ __forceinline__ void load_f32(const float *base, uint32_t len, float *x)
{
    if (FULL) load_f32_full<G, NT>(base, x); else load_f32_tail<G>(base, len, x);
}
template <class G, bool FULL, bool NT>
__device__ __forceinline__ void store_f32(float *base, uint32_t len, const float *x)
{
    if (FULL) {
        f32x4 *v = reinterpret_cast<f32x4 *>(base);
#pragma unroll
        for (int i = 0; i < G::kQuads; ++i)
            st<NT>(v + G::quad(i), f32x4{x[4 * i], x[4 * i + 1], x[4 * i + 2], x[4 * i + 3]});
    } else {
#pragma unroll
        for (int i = 0; i < G::kQuads; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t idx = 4 * G::quad(i) + e;
                if (idx < len) base[idx] = x[4 * i + e];
            }
    }
}

// Payload of a unit -> fp32.  `pay` points at the payload array's element 0,
// e0 is the unit's first element, `scale` the stored scale of its tile (QUANT8).
template <int MODE, class G, bool FULL, bool NT>
__device__ __forceinline__ void load_payload(const void *pay, uint64_t e0, uint32_t len, float scale, float *x)
{
    using C = Codec<MODE>;
    const float step = MODE == PIPESGD_QUANT8 ? scale / 127.0f : 0.0f;
    if (FULL) {
        const typename C::Raw *v =
            reinterpret_cast<const typename C::Raw *>(static_cast<const char *>(pay) + e0 * C::kBytes);
        typename C::Raw r[G::kQuads];
        if constexpr (kWide128<C, G>) {
            // the thread's QUADS consecutive quads of payload are 16 bytes: one 128-bit load
            const u32x4 q = ld<NT>(reinterpret_cast<const u32x4 *>(v) + threadIdx.x);
            split128<C>(q, r);
        } else {
#pragma unroll
            for (int i = 0; i < G::kQuads; ++i) r[i] = ld<NT>(v + G::quad(i));
        }
#pragma unroll
        for (int i = 0; i < G::kQuads; ++i) C::decode(r[i], step, x + 4 * i);
    } else {
        float r[G::kPerThread];
#pragma unroll
        for (int i = 0; i < G::kQuads; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t idx = 4 * G::quad(i) + e;
                r[4 * i + e] = C::decode1(pay, e0 + min(idx, len - 1), step);
            }
#pragma unroll
        for (int i = 0; i < G::kQuads; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t idx = 4 * G::quad(i) + e;
                x[4 * i + e] = idx < len ? r[4 * i + e] : 0.0f;
            }
    }
}

// Largest magnitude of a whole tile (QUANT8's range, Sec. 3.2); needs a
// geometry whose unit is the tile.  Elements past `len` were loaded as zero
// and do not disturb it.
template <class G>
__device__ __forceinline__ float tile_absmax(const float *x, float *red)
{
    static_assert(G::kUnit == kTile, "the quantisation range needs the whole block in one workgroup");
    float m = 0.0f;
#pragma unroll
    for (int k = 0; k < G::kPerThread; ++k) m = fmaxf(m, fabsf(x[k]));
    return block_max<G>(m, red);
}

// fp32 -> payload of a unit.  For QUANT8 `scale` is the tile's range
// (tile_absmax); it is stored by thread 0.
template <int MODE, class G, bool FULL, bool NT>
__device__ __forceinline__ void store_payload(void *pay, float *sc, uint64_t e0, uint32_t len, float scale, const float *x)
{
    using C = Codec<MODE>;
    const float inv = MODE == PIPESGD_QUANT8 ? quant_inverse(scale) : 0.0f;
    if (FULL) {
        typename C::Raw *v = reinterpret_cast<typename C::Raw *>(static_cast<char *>(pay) + e0 * C::kBytes);
        if constexpr (kWide128<C, G>) {
            typename C::Raw r[G::kQuads];
#pragma unroll
            for (int i = 0; i < G::kQuads; ++i) r[i] = C::encode(x + 4 * i, inv);
            st<NT>(reinterpret_cast<u32x4 *>(v) + threadIdx.x, join128<C>(r));
        } else {
#pragma unroll
            for (int i = 0; i < G::kQuads; ++i) st<NT>(v + G::quad(i), C::encode(x + 4 * i, inv));
        }
    } else {
#pragma unroll
        for (int i = 0; i < G::kQuads; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t idx = 4 * G::quad(i) + e;
                if (idx < len) C::encode1(pay, e0 + idx, x[4 * i + e], inv);
            }
    }
    if (MODE == PIPESGD_QUANT8 && threadIdx.x == 0) sc[e0 / kTile] = scale;
}

// What a receiver sees of a value it is sent: D(C(x)), without touching
// memory (used by the fused schedule).
template <int MODE, class G>
__device__ __forceinline__ void through_the_wire(float *x, float scale)
{
    if (MODE == PIPESGD_TRUNC16) {
#pragma unroll
        for (int k = 0; k < G::kPerThread; ++k) x[k] = u2f(f2u(x[k]) & 0xffff0000u);
    } else if (MODE == PIPESGD_QUANT8) {
        const float inv = quant_inverse(scale);
        const float step = scale / 127.0f;
#pragma unroll
        for (int k = 0; k < G::kPerThread; ++k) x[k] = static_cast<float>(quant_code(x[k], inv)) * step;
    }
}

// QUANT8 kernels that compute a range must see a whole tile per workgroup.
template <int MODE, class G> struct RangeOk {
    static constexpr bool value = MODE != PIPESGD_QUANT8 || G::kUnit == kTile;
};

}  // namespace
