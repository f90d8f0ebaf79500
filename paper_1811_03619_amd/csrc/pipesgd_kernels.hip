// HIP kernels and device entry points of libpipesgd (gfx950 / CDNA4).
//
// Everything here streams: each element is read, combined with one or two
// other streams and written, a handful of ALU operations per 6..20 bytes.  The
// bound is HBM bandwidth, so the kernels are organised around memory access:
//   * the unit of work is one TILE of 4096 consecutive elements (= one
//     quantisation block, = 16 KiB of fp32), handled by one 256-thread group;
//   * a thread owns 4 "quads" (4 consecutive elements each) spaced 256 quads
//     apart, so that every wave-level access is one contiguous run: 16 B per
//     lane on fp32 streams, 8 B per lane on 16-bit payloads, 4 B per lane on
//     8-bit payloads; all of a thread's loads are issued before any use;
//   * ring blocks, bucket starts and therefore tiles are 4096-aligned, which
//     makes every full tile vector-aligned; only the last tile of a ring block
//     can be short and takes a guarded scalar path;
//   * no matrix cores: nothing on this path is a contraction.
// Arithmetic is written so that each operation is exactly one IEEE binary32
// rounding (contraction is switched off for the file; the update's two fused
// multiply-adds are explicit).
#include <hip/hip_runtime.h>

#include <cfloat>
#include <cstdint>

#include "pipesgd.h"

#pragma clang fp contract(off)

namespace {

constexpr int kTile = PIPESGD_QBLOCK;        // elements per tile
constexpr int kThreads = 256;                // 4 wavefronts of 64
constexpr int kQuads = 4;                    // quads per thread per tile
constexpr int kPerThread = 4 * kQuads;       // 16 elements
static_assert(kThreads * kPerThread == kTile, "tile geometry");
constexpr int kMaxW = PIPESGD_MAX_WORKERS;
constexpr int kMaxB = PIPESGD_MAX_BUCKETS;

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
constexpr bool kNtGrad = PIPESGD_NT_GRAD, kNtPayIn = PIPESGD_NT_PAYIN, kNtPayOut = PIPESGD_NT_PAYOUT,
               kNtUpdate = PIPESGD_NT_UPDATE;

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

struct RingArgs {
    const float *g[kMaxW];
    void *pay[kMaxW];
    float *sc[kMaxW];
    int p;
    int step;
};

struct UpdateArgs {
    const void *pay[kMaxW];
    const float *sc[kMaxW];
    float *w[kMaxW];
    float *v[kMaxW];
    uint64_t n;
    float lr, momentum, grad_scale;
};

struct TileRef {
    uint64_t elem0;     // first element, packed-buffer coordinates
    uint32_t len;       // 1..4096, or 0 if the slot is empty for this chunk
};

__device__ __forceinline__ int mod_p(int a, int p)
{
    int m = a % p;
    return m < 0 ? m + p : m;
}

// Slot -> (bucket, tile of chunk `chunk`).  All operands are wave-uniform.
__device__ __forceinline__ TileRef locate(const BucketTable &bt, uint32_t slot, int chunk)
{
    uint32_t lo = 0, hi = bt.count;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (bt.slot_prefix[mid] <= slot) lo = mid; else hi = mid;
    }
    const uint64_t ce = static_cast<uint64_t>(bt.ce_tiles[lo]) * kTile;
    const uint64_t t = slot - bt.slot_prefix[lo];
    const uint64_t nb = bt.n[lo];
    const uint64_t lo_e = static_cast<uint64_t>(chunk) * ce + t * kTile;
    uint64_t hi_e = (static_cast<uint64_t>(chunk) + 1) * ce;
    if (hi_e > nb) hi_e = nb;
    TileRef r;
    if (lo_e >= hi_e) { r.elem0 = 0; r.len = 0; return r; }
    r.elem0 = bt.start[lo] + lo_e;
    const uint64_t rem = hi_e - lo_e;
    r.len = rem < static_cast<uint64_t>(kTile) ? static_cast<uint32_t>(rem) : static_cast<uint32_t>(kTile);
    return r;
}

// ------------------------------------------------------- block-wide max --

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// red: 4 floats of LDS, one per wavefront.  One barrier per call; callers that
// reduce repeatedly alternate between two such arrays.
__device__ __forceinline__ float block_max(float v, float *red)
{
    v = wave_max(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
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

// ------------------------------------------------------- tile load / store --
// x[16] of a thread: x[4*i + e] = element 4*(i*256 + tid) + e of the tile.
// The *_full variants assume a whole, 16-byte aligned tile; the *_tail
// variants guard every element against `len` and fill the rest with zero.

template <bool NT>
__device__ __forceinline__ void load_f32_full(const float *base, float *x)
{
    const f32x4 *v = reinterpret_cast<const f32x4 *>(base);
    f32x4 r[kQuads];
#pragma unroll
    for (int i = 0; i < kQuads; ++i) r[i] = ld<NT>(v + i * kThreads + threadIdx.x);
#pragma unroll
    for (int i = 0; i < kQuads; ++i) { x[4 * i] = r[i].x; x[4 * i + 1] = r[i].y; x[4 * i + 2] = r[i].z; x[4 * i + 3] = r[i].w; }
}
__device__ __forceinline__ void load_f32_tail(const float *base, uint32_t len, float *x)
{
#pragma unroll
    for (int i = 0; i < kQuads; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t idx = 4 * (i * kThreads + threadIdx.x) + e;
            x[4 * i + e] = idx < len ? base[idx] : 0.0f;
        }
}
template <bool NT>
__device__ __forceinline__ void store_f32_full(float *base, const float *x)
{
    f32x4 *v = reinterpret_cast<f32x4 *>(base);
#pragma unroll
    for (int i = 0; i < kQuads; ++i)
        st<NT>(v + i * kThreads + threadIdx.x, f32x4{x[4 * i], x[4 * i + 1], x[4 * i + 2], x[4 * i + 3]});
}
__device__ __forceinline__ void store_f32_tail(float *base, uint32_t len, const float *x)
{
#pragma unroll
    for (int i = 0; i < kQuads; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t idx = 4 * (i * kThreads + threadIdx.x) + e;
            if (idx < len) base[idx] = x[4 * i + e];
        }
}

// Payload of a tile -> fp32.  `pay` points at the payload array's element 0,
// e0 is the tile's first element, `scale` the tile's stored scale (QUANT8).
template <int MODE, bool FULL, bool NT>
__device__ __forceinline__ void load_payload(const void *pay, uint64_t e0, uint32_t len, float scale, float *x)
{
    using C = Codec<MODE>;
    const float step = MODE == PIPESGD_QUANT8 ? scale / 127.0f : 0.0f;
    if (FULL) {
        const typename C::Raw *v =
            reinterpret_cast<const typename C::Raw *>(static_cast<const char *>(pay) + e0 * C::kBytes);
        typename C::Raw r[kQuads];
#pragma unroll
        for (int i = 0; i < kQuads; ++i) r[i] = ld<NT>(v + i * kThreads + threadIdx.x);
#pragma unroll
        for (int i = 0; i < kQuads; ++i) C::decode(r[i], step, x + 4 * i);
    } else {
#pragma unroll
        for (int i = 0; i < kQuads; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t idx = 4 * (i * kThreads + threadIdx.x) + e;
                x[4 * i + e] = idx < len ? C::decode1(pay, e0 + idx, step) : 0.0f;
            }
    }
}

// Largest magnitude of the tile (QUANT8's range, Sec. 3.2).  Elements past
// `len` were loaded as zero and do not disturb it.
__device__ __forceinline__ float tile_absmax(const float *x, float *red)
{
    float m = 0.0f;
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) m = fmaxf(m, fabsf(x[k]));
    return block_max(m, red);
}

// fp32 -> payload of a tile.  For QUANT8 `scale` is the tile's range
// (tile_absmax); it is stored by thread 0.
template <int MODE, bool FULL, bool NT>
__device__ __forceinline__ void store_payload(void *pay, float *sc, uint64_t e0, uint32_t len, float scale, const float *x)
{
    using C = Codec<MODE>;
    const float inv = MODE == PIPESGD_QUANT8 ? quant_inverse(scale) : 0.0f;
    if (FULL) {
        typename C::Raw *v = reinterpret_cast<typename C::Raw *>(static_cast<char *>(pay) + e0 * C::kBytes);
#pragma unroll
        for (int i = 0; i < kQuads; ++i) st<NT>(v + i * kThreads + threadIdx.x, C::encode(x + 4 * i, inv));
    } else {
#pragma unroll
        for (int i = 0; i < kQuads; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t idx = 4 * (i * kThreads + threadIdx.x) + e;
                if (idx < len) C::encode1(pay, e0 + idx, x[4 * i + e], inv);
            }
    }
    if (MODE == PIPESGD_QUANT8 && threadIdx.x == 0) sc[e0 / kTile] = scale;
}

// What a receiver sees of a value it is sent: D(C(x)), without touching
// memory (used by the fused schedule).
template <int MODE>
__device__ __forceinline__ void through_the_wire(float *x, float scale)
{
    if (MODE == PIPESGD_TRUNC16) {
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) x[k] = u2f(f2u(x[k]) & 0xffff0000u);
    } else if (MODE == PIPESGD_QUANT8) {
        const float inv = quant_inverse(scale);
        const float step = scale / 127.0f;
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) x[k] = static_cast<float>(quant_code(x[k], inv)) * step;
    }
}

// ---------------------------------------------------------------- kernels --

// One ring hop for every worker (blockIdx.y = receiving worker r).
//   HAS_IN = false: the first send.  C(g_r[chunk r]) -> slot r.
//   HAS_IN = true : transmit-and-reduce round a.step.  D(slot r-1) + g_r -> C -> slot r.
//   in_is_grad    : uncompressed round 0 reads the sender's gradient itself.
template <int MODE, bool HAS_IN>
__global__ __launch_bounds__(kThreads) void ring_hop_kernel(RingArgs a, BucketTable bt, int in_is_grad)
{
    __shared__ float red[4];
    const int r = blockIdx.y;
    const int chunk = HAS_IN ? mod_p(r - a.step - 1, a.p) : r;
    const TileRef t = locate(bt, blockIdx.x, chunk);
    if (t.len == 0) return;
    const bool full = t.len == kTile;

    float P[kPerThread];
    if (full) load_f32_full<kNtGrad>(a.g[r] + t.elem0, P); else load_f32_tail(a.g[r] + t.elem0, t.len, P);

    if (HAS_IN) {
        const int src = mod_p(r - 1, a.p);
        float x[kPerThread];
        if (MODE == PIPESGD_NONE && in_is_grad) {
            if (full) load_f32_full<kNtGrad>(a.g[src] + t.elem0, x); else load_f32_tail(a.g[src] + t.elem0, t.len, x);
        } else {
            const float scale_in = MODE == PIPESGD_QUANT8 ? a.sc[src][t.elem0 / kTile] : 0.0f;
            if (full) load_payload<MODE, true, kNtPayIn>(a.pay[src], t.elem0, t.len, scale_in, x);
            else      load_payload<MODE, false, false>(a.pay[src], t.elem0, t.len, scale_in, x);
        }
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) P[k] = x[k] + P[k];
    }

    const float scale = MODE == PIPESGD_QUANT8 ? tile_absmax(P, red) : 0.0f;
    if (full) store_payload<MODE, true, kNtPayOut>(a.pay[r], a.sc[r], t.elem0, t.len, scale, P);
    else      store_payload<MODE, false, false>(a.pay[r], a.sc[r], t.elem0, t.len, scale, P);
}

// One send-back round for every worker: byte copy of a chunk's payload (and
// scales) from slot r-1 to slot r.
template <int MODE>
__global__ __launch_bounds__(kThreads) void ring_allgather_kernel(RingArgs a, BucketTable bt)
{
    using C = Codec<MODE>;
    const int r = blockIdx.y;
    const int src = mod_p(r - 1, a.p);
    const int chunk = mod_p(r - a.step, a.p);
    const TileRef t = locate(bt, blockIdx.x, chunk);
    if (t.len == 0) return;
    const char *in = static_cast<const char *>(a.pay[src]) + t.elem0 * C::kBytes;
    char *out = static_cast<char *>(a.pay[r]) + t.elem0 * C::kBytes;
    if (t.len == kTile) {
        constexpr int kVecs = kTile * C::kBytes / 16;          // 1024, 512 or 256 16-byte vectors
        const u32x4 *vi = reinterpret_cast<const u32x4 *>(in);
        u32x4 *vo = reinterpret_cast<u32x4 *>(out);
        constexpr int kIter = kVecs / kThreads;
        u32x4 tmp[kIter];
#pragma unroll
        for (int i = 0; i < kIter; ++i) tmp[i] = ld<kNtPayIn>(vi + i * kThreads + threadIdx.x);
#pragma unroll
        for (int i = 0; i < kIter; ++i) st<kNtPayOut>(vo + i * kThreads + threadIdx.x, tmp[i]);
    } else {
        const uint32_t bytes = t.len * C::kBytes;
        for (uint32_t i = threadIdx.x; i < bytes; i += kThreads) out[i] = in[i];
    }
    if (MODE == PIPESGD_QUANT8 && threadIdx.x == 0) a.sc[r][t.elem0 / kTile] = a.sc[src][t.elem0 / kTile];
}

// The whole chain of one tile in registers (blockIdx.y = chunk c):
// P = g_c; for j = 1..p-1: P = D(C(P)) + g_{c+j}; every slot <- C(P).
template <int MODE>
__global__ __launch_bounds__(kThreads) void ring_fused_kernel(RingArgs a, BucketTable bt)
{
    __shared__ float red[2][4];
    const int c = blockIdx.y;
    const TileRef t = locate(bt, blockIdx.x, c);
    if (t.len == 0) return;
    const bool full = t.len == kTile;
    const int p = a.p;

    float P[kPerThread], g[kPerThread];
    if (full) load_f32_full<kNtGrad>(a.g[c] + t.elem0, P); else load_f32_tail(a.g[c] + t.elem0, t.len, P);
    int flip = 0;
    for (int j = 1; j < p; ++j) {
        const int wkr = mod_p(c + j, p);
        if (full) load_f32_full<kNtGrad>(a.g[wkr] + t.elem0, g); else load_f32_tail(a.g[wkr] + t.elem0, t.len, g);
        float scale = 0.0f;
        if (MODE == PIPESGD_QUANT8) { scale = tile_absmax(P, red[flip]); flip ^= 1; }
        through_the_wire<MODE>(P, scale);
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) P[k] = P[k] + g[k];
    }
    float scale = 0.0f;
    if (MODE == PIPESGD_QUANT8) scale = tile_absmax(P, red[flip]);
    for (int r = 0; r < p; ++r) {
        if (full) store_payload<MODE, true, true>(a.pay[r], a.sc[r], t.elem0, t.len, scale, P);
        else      store_payload<MODE, false, false>(a.pay[r], a.sc[r], t.elem0, t.len, scale, P);
    }
}

// Stand-alone codec over a flat vector (blockIdx.x = tile).
template <int MODE>
__global__ __launch_bounds__(kThreads) void compress_kernel(const float *src, uint64_t n, void *pay, float *sc)
{
    __shared__ float red[4];
    const uint64_t e0 = static_cast<uint64_t>(blockIdx.x) * kTile;
    const uint64_t rem = n - e0;
    const uint32_t len = rem < static_cast<uint64_t>(kTile) ? static_cast<uint32_t>(rem) : kTile;
    float x[kPerThread];
    if (len == kTile) load_f32_full<true>(src + e0, x); else load_f32_tail(src + e0, len, x);
    const float scale = MODE == PIPESGD_QUANT8 ? tile_absmax(x, red) : 0.0f;
    if (len == kTile) store_payload<MODE, true, false>(pay, sc, e0, len, scale, x);
    else              store_payload<MODE, false, false>(pay, sc, e0, len, scale, x);
}

template <int MODE>
__global__ __launch_bounds__(kThreads) void decompress_kernel(const void *pay, const float *sc, uint64_t n, float *dst)
{
    const uint64_t e0 = static_cast<uint64_t>(blockIdx.x) * kTile;
    const uint64_t rem = n - e0;
    const uint32_t len = rem < static_cast<uint64_t>(kTile) ? static_cast<uint32_t>(rem) : kTile;
    const float scale = MODE == PIPESGD_QUANT8 ? sc[blockIdx.x] : 0.0f;
    float x[kPerThread];
    if (len == kTile) { load_payload<MODE, true, true>(pay, e0, len, scale, x); store_f32_full<false>(dst + e0, x); }
    else              { load_payload<MODE, false, false>(pay, e0, len, scale, x); store_f32_tail(dst + e0, len, x); }
}

// Decompress + momentum-SGD step (Alg. 1 compute thread lines 4-5) for every
// replica (blockIdx.y): reads the stale slot, v and w once, writes v and w once.
template <int MODE, bool MOMENTUM>
__global__ __launch_bounds__(kThreads) void update_kernel(UpdateArgs a)
{
    const int r = blockIdx.y;
    const uint64_t e0 = static_cast<uint64_t>(blockIdx.x) * kTile;
    const uint64_t rem = a.n - e0;
    const uint32_t len = rem < static_cast<uint64_t>(kTile) ? static_cast<uint32_t>(rem) : kTile;
    const bool full = len == kTile;
    const float scale = MODE == PIPESGD_QUANT8 ? a.sc[r][blockIdx.x] : 0.0f;
    float *w = a.w[r] + e0;
    float *v = MOMENTUM ? a.v[r] + e0 : nullptr;

    float g[kPerThread], wv[kPerThread], vv[kPerThread];
    if (full) {
        load_payload<MODE, true, kNtUpdate>(a.pay[r], e0, len, scale, g);
        load_f32_full<kNtUpdate>(w, wv);
        if (MOMENTUM) load_f32_full<kNtUpdate>(v, vv);
    } else {
        load_payload<MODE, false, false>(a.pay[r], e0, len, scale, g);
        load_f32_tail(w, len, wv);
        if (MOMENTUM) load_f32_tail(v, len, vv);
    }
    const float gs = a.grad_scale, m = a.momentum, neg_lr = -a.lr;
    if (gs != 1.0f) {
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) g[k] = g[k] * gs;
    }
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
        if (MOMENTUM) {
            vv[k] = fmaf(m, vv[k], g[k]);
            wv[k] = fmaf(neg_lr, vv[k], wv[k]);
        } else {
            wv[k] = fmaf(neg_lr, g[k], wv[k]);
        }
    }
    if (full) {
        if (MOMENTUM) store_f32_full<kNtUpdate>(v, vv);
        store_f32_full<kNtUpdate>(w, wv);
    } else {
        if (MOMENTUM) store_f32_tail(v, len, vv);
        store_f32_tail(w, len, wv);
    }
}

// Many tensor <-> packed-buffer copies in one launch.  The segment table is in
// device memory; a block finds its segment by binary search on first_tile.
template <bool TO_PACKED>
__global__ __launch_bounds__(kThreads) void segment_copy_kernel(const pipesgd_segment *seg, uint32_t num)
{
    const uint64_t tile = blockIdx.x;
    uint32_t lo = 0, hi = num;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (seg[mid].first_tile <= tile) lo = mid; else hi = mid;
    }
    const pipesgd_segment s = seg[lo];
    const uint64_t e0 = (tile - s.first_tile) * kTile;
    if (e0 >= s.numel) return;
    const uint64_t rem = s.numel - e0;
    const uint32_t len = rem < static_cast<uint64_t>(kTile) ? static_cast<uint32_t>(rem) : kTile;
    const float *in = (TO_PACKED ? s.tensor : s.packed) + e0;
    float *out = (TO_PACKED ? s.packed : s.tensor) + e0;
    const bool vec = len == kTile &&
        ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & 15) == 0;
    if (vec) {
        float x[kPerThread];
        load_f32_full<true>(in, x);
        store_f32_full<false>(out, x);
    } else {
        for (uint32_t i = threadIdx.x; i < len; i += kThreads) out[i] = in[i];
    }
}

// ------------------------------------------------------------ host helpers --

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline bool mode_ok(int mode) { return mode == PIPESGD_NONE || mode == PIPESGD_TRUNC16 || mode == PIPESGD_QUANT8; }
inline int launch_status() { return hipGetLastError() == hipSuccess ? PIPESGD_OK : PIPESGD_ERR_HIP; }

// Validates a ring and turns it into kernel arguments.  total_slots = grid.x.
int prepare_ring(const pipesgd_ring *ring, RingArgs &ra, BucketTable &bt, uint64_t &total_slots)
{
    if (!ring) return PIPESGD_ERR_ARG;
    if (!mode_ok(ring->mode)) return PIPESGD_ERR_MODE;
    if (ring->workers < 1 || ring->reserved != 0) return PIPESGD_ERR_ARG;
    if (ring->workers > kMaxW || ring->num_buckets > static_cast<uint32_t>(kMaxB)) return PIPESGD_ERR_CAPACITY;
    if (ring->num_buckets > 0 && !ring->buckets) return PIPESGD_ERR_ARG;
    const int p = ring->workers;
    for (int r = 0; r < kMaxW; ++r) {
        ra.g[r] = nullptr; ra.pay[r] = nullptr; ra.sc[r] = nullptr;
    }
    for (int r = 0; r < p; ++r) {
        if (ring->n > 0) {
            if (!ring->g_local[r] || !ring->g_sum_c[r]) return PIPESGD_ERR_ARG;
            if (ring->mode == PIPESGD_QUANT8 && !ring->scales[r]) return PIPESGD_ERR_ARG;
        }
        if (!aligned16(ring->g_local[r]) || !aligned16(ring->g_sum_c[r]) || !aligned16(ring->scales[r]))
            return PIPESGD_ERR_ALIGN;
        ra.g[r] = ring->g_local[r];
        ra.pay[r] = ring->g_sum_c[r];
        ra.sc[r] = ring->scales[r];
    }
    ra.p = p;
    ra.step = 0;

    const pipesgd_bucket whole = {0, ring->n};
    const pipesgd_bucket *b = ring->num_buckets ? ring->buckets : &whole;
    const uint32_t nb = ring->num_buckets ? ring->num_buckets : 1;
    uint64_t slots = 0, prev_end = 0;
    for (uint32_t i = 0; i < nb; ++i) {
        if (b[i].start % kTile) return PIPESGD_ERR_ALIGN;
        if (b[i].start < prev_end || b[i].n > ring->n || b[i].start > ring->n - b[i].n) return PIPESGD_ERR_ARG;
        prev_end = b[i].start + b[i].n;
        const uint64_t ce_tiles = pipesgd_chunk_elems(b[i].n, p) / kTile;
        if (ce_tiles > 0xffffffffull) return PIPESGD_ERR_CAPACITY;
        bt.slot_prefix[i] = static_cast<uint32_t>(slots);
        bt.ce_tiles[i] = static_cast<uint32_t>(ce_tiles);
        bt.start[i] = b[i].start;
        bt.n[i] = b[i].n;
        slots += ce_tiles;
        if (slots > 0x7fffffffull) return PIPESGD_ERR_CAPACITY;
    }
    for (uint32_t i = nb; i < static_cast<uint32_t>(kMaxB); ++i) {
        bt.slot_prefix[i] = static_cast<uint32_t>(slots);
        bt.ce_tiles[i] = 0; bt.start[i] = 0; bt.n[i] = 0;
    }
    bt.slot_prefix[kMaxB] = static_cast<uint32_t>(slots);
    bt.count = nb;
    total_slots = slots;
    return PIPESGD_OK;
}

template <int MODE>
int launch_first_send(const RingArgs &ra, const BucketTable &bt, uint64_t slots, hipStream_t s)
{
    hipLaunchKernelGGL((ring_hop_kernel<MODE, false>), dim3(static_cast<uint32_t>(slots), ra.p), dim3(kThreads), 0, s,
                       ra, bt, 0);
    return launch_status();
}
template <int MODE>
int launch_rs(const RingArgs &ra, const BucketTable &bt, uint64_t slots, hipStream_t s)
{
    hipLaunchKernelGGL((ring_hop_kernel<MODE, true>), dim3(static_cast<uint32_t>(slots), ra.p), dim3(kThreads), 0, s,
                       ra, bt, (MODE == PIPESGD_NONE && ra.step == 0) ? 1 : 0);
    return launch_status();
}
template <int MODE>
int launch_ag(const RingArgs &ra, const BucketTable &bt, uint64_t slots, hipStream_t s)
{
    hipLaunchKernelGGL((ring_allgather_kernel<MODE>), dim3(static_cast<uint32_t>(slots), ra.p), dim3(kThreads), 0, s,
                       ra, bt);
    return launch_status();
}
template <int MODE>
int launch_fused(const RingArgs &ra, const BucketTable &bt, uint64_t slots, hipStream_t s)
{
    hipLaunchKernelGGL((ring_fused_kernel<MODE>), dim3(static_cast<uint32_t>(slots), ra.p), dim3(kThreads), 0, s,
                       ra, bt);
    return launch_status();
}

#define PIPESGD_DISPATCH_MODE(mode, fn, ...)                                   \
    ((mode) == PIPESGD_NONE      ? fn<PIPESGD_NONE>(__VA_ARGS__)               \
     : (mode) == PIPESGD_TRUNC16 ? fn<PIPESGD_TRUNC16>(__VA_ARGS__)            \
                                 : fn<PIPESGD_QUANT8>(__VA_ARGS__))

int first_send_impl(int mode, const RingArgs &ra, const BucketTable &bt, uint64_t slots, hipStream_t s)
{
    // uncompressed, p > 1: the first round reads the sender's gradient in place
    if (slots == 0 || (mode == PIPESGD_NONE && ra.p > 1)) return PIPESGD_OK;
    return PIPESGD_DISPATCH_MODE(mode, launch_first_send, ra, bt, slots, s);
}

template <int MODE>
int launch_compress(const float *src, uint64_t n, void *pay, float *sc, uint64_t tiles, hipStream_t s)
{
    hipLaunchKernelGGL((compress_kernel<MODE>), dim3(static_cast<uint32_t>(tiles)), dim3(kThreads), 0, s, src, n, pay, sc);
    return launch_status();
}
template <int MODE>
int launch_decompress(const void *pay, const float *sc, uint64_t n, float *dst, uint64_t tiles, hipStream_t s)
{
    hipLaunchKernelGGL((decompress_kernel<MODE>), dim3(static_cast<uint32_t>(tiles)), dim3(kThreads), 0, s, pay, sc, n, dst);
    return launch_status();
}
template <int MODE>
int launch_update(const UpdateArgs &ua, int replicas, uint64_t tiles, bool momentum, hipStream_t s)
{
    const dim3 grid(static_cast<uint32_t>(tiles), replicas);
    if (momentum) hipLaunchKernelGGL((update_kernel<MODE, true>), grid, dim3(kThreads), 0, s, ua);
    else          hipLaunchKernelGGL((update_kernel<MODE, false>), grid, dim3(kThreads), 0, s, ua);
    return launch_status();
}

}  // namespace

// ------------------------------------------------------------ entry points --

extern "C" {

int pipesgd_compress(int mode, const float *src, uint64_t n, void *payload, float *scales, void *stream)
{
    if (!mode_ok(mode)) return PIPESGD_ERR_MODE;
    if (n == 0) return PIPESGD_OK;
    if (!src || !payload || (mode == PIPESGD_QUANT8 && !scales)) return PIPESGD_ERR_ARG;
    if (!aligned16(src) || !aligned16(payload) || (mode == PIPESGD_QUANT8 && !aligned16(scales))) return PIPESGD_ERR_ALIGN;
    const uint64_t tiles = (n + kTile - 1) / kTile;
    if (tiles > 0x7fffffffull) return PIPESGD_ERR_CAPACITY;
    return PIPESGD_DISPATCH_MODE(mode, launch_compress, src, n, payload, scales, tiles, static_cast<hipStream_t>(stream));
}

int pipesgd_decompress(int mode, const void *payload, const float *scales, uint64_t n, float *dst, void *stream)
{
    if (!mode_ok(mode)) return PIPESGD_ERR_MODE;
    if (n == 0) return PIPESGD_OK;
    if (!dst || !payload || (mode == PIPESGD_QUANT8 && !scales)) return PIPESGD_ERR_ARG;
    if (!aligned16(dst) || !aligned16(payload) || (mode == PIPESGD_QUANT8 && !aligned16(scales))) return PIPESGD_ERR_ALIGN;
    const uint64_t tiles = (n + kTile - 1) / kTile;
    if (tiles > 0x7fffffffull) return PIPESGD_ERR_CAPACITY;
    return PIPESGD_DISPATCH_MODE(mode, launch_decompress, payload, scales, n, dst, tiles, static_cast<hipStream_t>(stream));
}

int pipesgd_ring_first_send(const pipesgd_ring *ring, void *stream)
{
    RingArgs ra; BucketTable bt; uint64_t slots = 0;
    const int rc = prepare_ring(ring, ra, bt, slots);
    if (rc != PIPESGD_OK) return rc;
    return first_send_impl(ring->mode, ra, bt, slots, static_cast<hipStream_t>(stream));
}

int pipesgd_ring_reduce_scatter_step(const pipesgd_ring *ring, int step, void *stream)
{
    RingArgs ra; BucketTable bt; uint64_t slots = 0;
    const int rc = prepare_ring(ring, ra, bt, slots);
    if (rc != PIPESGD_OK) return rc;
    if (step < 0 || step > ring->workers - 2) return PIPESGD_ERR_ARG;
    if (slots == 0) return PIPESGD_OK;
    ra.step = step;
    return PIPESGD_DISPATCH_MODE(ring->mode, launch_rs, ra, bt, slots, static_cast<hipStream_t>(stream));
}

int pipesgd_ring_allgather_step(const pipesgd_ring *ring, int step, void *stream)
{
    RingArgs ra; BucketTable bt; uint64_t slots = 0;
    const int rc = prepare_ring(ring, ra, bt, slots);
    if (rc != PIPESGD_OK) return rc;
    if (step < 0 || step > ring->workers - 2) return PIPESGD_ERR_ARG;
    if (slots == 0) return PIPESGD_OK;
    ra.step = step;
    return PIPESGD_DISPATCH_MODE(ring->mode, launch_ag, ra, bt, slots, static_cast<hipStream_t>(stream));
}

int pipesgd_allreduce_sim(const pipesgd_ring *ring, int schedule, void *stream)
{
    RingArgs ra; BucketTable bt; uint64_t slots = 0;
    int rc = prepare_ring(ring, ra, bt, slots);
    if (rc != PIPESGD_OK) return rc;
    if (schedule != PIPESGD_STEPWISE && schedule != PIPESGD_FUSED) return PIPESGD_ERR_MODE;
    if (slots == 0) return PIPESGD_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int mode = ring->mode, p = ring->workers;
    if (schedule == PIPESGD_FUSED) return PIPESGD_DISPATCH_MODE(mode, launch_fused, ra, bt, slots, s);
    rc = first_send_impl(mode, ra, bt, slots, s);
    for (int step = 0; rc == PIPESGD_OK && step <= p - 2; ++step) {
        ra.step = step;
        rc = PIPESGD_DISPATCH_MODE(mode, launch_rs, ra, bt, slots, s);
    }
    for (int step = 0; rc == PIPESGD_OK && step <= p - 2; ++step) {
        ra.step = step;
        rc = PIPESGD_DISPATCH_MODE(mode, launch_ag, ra, bt, slots, s);
    }
    return rc;
}

int pipesgd_apply_update_multi(int mode, int replicas, const void *const *g_sum_c,
                               const float *const *scales, uint64_t n, float *const *w,
                               float *const *v, float lr, float momentum, float grad_scale,
                               void *stream)
{
    if (!mode_ok(mode)) return PIPESGD_ERR_MODE;
    if (replicas < 1) return PIPESGD_ERR_ARG;
    if (replicas > kMaxW) return PIPESGD_ERR_CAPACITY;
    if (!g_sum_c || !w) return PIPESGD_ERR_ARG;
    const bool mom = momentum != 0.0f;
    if (mom && !v) return PIPESGD_ERR_ARG;
    if (mode == PIPESGD_QUANT8 && !scales) return PIPESGD_ERR_ARG;
    if (n == 0) return PIPESGD_OK;
    UpdateArgs ua;
    for (int r = 0; r < kMaxW; ++r) { ua.pay[r] = nullptr; ua.sc[r] = nullptr; ua.w[r] = nullptr; ua.v[r] = nullptr; }
    for (int r = 0; r < replicas; ++r) {
        if (!g_sum_c[r] || !w[r] || (mom && !v[r]) || (mode == PIPESGD_QUANT8 && !scales[r])) return PIPESGD_ERR_ARG;
        if (!aligned16(g_sum_c[r]) || !aligned16(w[r]) || (mom && !aligned16(v[r])) ||
            (mode == PIPESGD_QUANT8 && !aligned16(scales[r])))
            return PIPESGD_ERR_ALIGN;
        ua.pay[r] = g_sum_c[r];
        ua.sc[r] = mode == PIPESGD_QUANT8 ? scales[r] : nullptr;
        ua.w[r] = w[r];
        ua.v[r] = mom ? v[r] : nullptr;
    }
    ua.n = n; ua.lr = lr; ua.momentum = momentum; ua.grad_scale = grad_scale;
    const uint64_t tiles = (n + kTile - 1) / kTile;
    if (tiles > 0x7fffffffull) return PIPESGD_ERR_CAPACITY;
    return PIPESGD_DISPATCH_MODE(mode, launch_update, ua, replicas, tiles, mom, static_cast<hipStream_t>(stream));
}

int pipesgd_apply_update(int mode, const void *g_sum_c, const float *scales, uint64_t n,
                         float *w, float *v, float lr, float momentum, float grad_scale,
                         void *stream)
{
    const void *pay[1] = {g_sum_c};
    const float *sc[1] = {scales};
    float *ww[1] = {w};
    float *vv[1] = {v};
    return pipesgd_apply_update_multi(mode, 1, pay, sc, n, ww, momentum != 0.0f ? vv : nullptr, lr, momentum,
                                      grad_scale, stream);
}

static int segment_copy(const pipesgd_segment *segments, uint64_t num, uint64_t total_tiles, void *stream, bool to_packed)
{
    if (num == 0 || total_tiles == 0) return PIPESGD_OK;
    if (!segments) return PIPESGD_ERR_ARG;
    if (!aligned16(segments)) return PIPESGD_ERR_ALIGN;
    if (num > 0x7fffffffull || total_tiles > 0x7fffffffull) return PIPESGD_ERR_CAPACITY;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid(static_cast<uint32_t>(total_tiles));
    if (to_packed) hipLaunchKernelGGL((segment_copy_kernel<true>), grid, dim3(kThreads), 0, s, segments, static_cast<uint32_t>(num));
    else           hipLaunchKernelGGL((segment_copy_kernel<false>), grid, dim3(kThreads), 0, s, segments, static_cast<uint32_t>(num));
    return launch_status();
}

int pipesgd_pack(const pipesgd_segment *segments, uint64_t num, uint64_t total_tiles, void *stream)
{
    return segment_copy(segments, num, total_tiles, stream, true);
}

int pipesgd_unpack(const pipesgd_segment *segments, uint64_t num, uint64_t total_tiles, void *stream)
{
    return segment_copy(segments, num, total_tiles, stream, false);
}

}  // extern "C"
