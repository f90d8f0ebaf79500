// HIP kernels and device entry points of libpipesgd (gfx950 / CDNA4).
//
// Everything here streams: each element is read, combined with one or two
// other streams and written, a handful of ALU operations per 6..20 bytes.  The
// bound is HBM bandwidth, so the kernels are organised around memory access:
//   * data is addressed in TILES of 4096 consecutive elements (= one
//     quantisation block = 16 KiB of fp32).  Ring blocks and bucket starts are
//     4096-aligned, so every whole tile is vector-aligned; only the last tile of
//     a ring block can be short and takes a guarded scalar path;
//   * a workgroup of THREADS threads handles one UNIT = THREADS*QUADS quads of
//     a tile (a quad = 4 consecutive elements); a thread owns QUADS quads spaced
//     THREADS quads apart, so every wave-level access is one contiguous run
//     (16 B per lane on fp32, 8 B on 16-bit payloads, 4 B on 8-bit payloads),
//     and all of a thread's loads are issued before the first use;
//   * the (THREADS, QUADS) geometry and an LDS reservation that caps the number
//     of resident workgroups per compute unit are launch parameters: measured
//     on MI355X, HBM delivers its best rate with roughly 20-30 KB of loads in
//     flight per compute unit -- far fewer than full occupancy would issue;
//   * streamed operands use nontemporal loads/stores, hop payloads that the
//     next launch re-reads use normal stores;
//   * no matrix cores: nothing on this path is a contraction.
// Arithmetic is written so that each operation is exactly one IEEE binary32
// rounding (contraction is switched off for the file; the update's two fused
// multiply-adds are explicit).
#include <hip/hip_runtime.h>

#include <atomic>
#include <cfloat>
#include <cstdint>
#include <new>
#include <vector>

#include "pipesgd.h"
#include "pipesgd_internal.hpp"

#pragma clang fp contract(off)

// Host-side resources of the two-stream schedules: HIP events only.
struct pipesgd_overlap {
    std::vector<hipEvent_t> events;
};

#include "pipesgd_device.hpp"

namespace {

// ---------------------------------------------------------------- kernels --

// One ring hop for every worker (blockIdx.y = receiving worker r).
//   HAS_IN = false: the first send.  C(g_r[chunk]) -> out_r.
//   HAS_IN = true : transmit-and-reduce.  D(in_r) + g_r -> C -> out_r.
template <int MODE, bool HAS_IN, class G, bool FULL>
__device__ __forceinline__ void ring_hop_body(const RingArgs &a, const UnitRef &t, int r, float *red)
{
    float P[G::kPerThread];
    float x[G::kPerThread];
    if (HAS_IN) {
        const float scale_in = MODE == PIPESGD_QUANT8 ? a.in_sc[r][t.elem0 / kTile] : 0.0f;
        load_payload<MODE, G, FULL, kNtPayIn>(a.in[r], t.elem0, t.len, scale_in, x);
    }
    load_f32<G, FULL, kNtGrad>(a.g[r] + t.elem0, t.len, P);
    if (HAS_IN) {
#pragma unroll
        for (int k = 0; k < G::kPerThread; ++k) P[k] = x[k] + P[k];
    }
    float scale = 0.0f;
    if constexpr (MODE == PIPESGD_QUANT8) scale = tile_absmax<G>(P, red);
    store_payload<MODE, G, FULL, kNtPayOut>(a.out[r], a.out_sc[r], t.elem0, t.len, scale, P);
}

template <int MODE, bool HAS_IN, class G>
__global__ __launch_bounds__(G::kThreads) void ring_hop_kernel(RingArgs a, BucketTable bt)
{
    if constexpr (RangeOk<MODE, G>::value) {
        __shared__ float red[G::kWaves];
        const int r = blockIdx.y;
        const UnitRef t = locate<G>(bt, blockIdx.x + a.slot_base * G::kSplit,
                                    mod_p(r - a.chunk_rot - static_cast<int>(blockIdx.z), a.p));
        if (t.empty) return;
        if (t.full) ring_hop_body<MODE, HAS_IN, G, true>(a, t, r, red);
        else        ring_hop_body<MODE, HAS_IN, G, false>(a, t, r, red);
    }
}

// Byte copy of one unit of payload (and, for a tile's first unit, its scale).
// Geometry counts 16-byte vectors here: a workgroup copies THREADS*QUADS of them.
template <int MODE, class G>
__device__ __forceinline__ void copy_unit(const void *in_pay, const float *in_sc, void *out_pay, float *out_sc, const UnitRef &t)
{
    using C = Codec<MODE>;
    const char *in = static_cast<const char *>(in_pay) + t.elem0 * C::kBytes;
    char *out = static_cast<char *>(out_pay) + t.elem0 * C::kBytes;
    if (t.full) {
        const u32x4 *vi = reinterpret_cast<const u32x4 *>(in);
        u32x4 *vo = reinterpret_cast<u32x4 *>(out);
        u32x4 tmp[G::kQuads];
#pragma unroll
        for (int i = 0; i < G::kQuads; ++i) tmp[i] = ld<kNtPayIn>(vi + i * G::kThreads + threadIdx.x);
#pragma unroll
        for (int i = 0; i < G::kQuads; ++i) st<kNtPayOut>(vo + i * G::kThreads + threadIdx.x, tmp[i]);
    } else {
        const uint32_t bytes = t.len * C::kBytes;
        for (uint32_t i = threadIdx.x; i < bytes; i += G::kThreads) out[i] = in[i];
    }
    if (MODE == PIPESGD_QUANT8 && threadIdx.x == 0 && t.elem0 % kTile == 0)
        out_sc[t.elem0 / kTile] = in_sc[t.elem0 / kTile];
}

// Payload transfer for every worker: byte copy of one chunk's payload (and
// scales) from in_r to out_r.  Used for the send-back rounds (in = the
// neighbour's slot, out = the worker's own slot) and as the "wire" stage of the
// pipelined schedule (out = the worker's receive staging).
template <int MODE, class G>
__global__ __launch_bounds__(G::kThreads) void ring_copy_kernel(RingArgs a, BucketTable bt)
{
    using C = Codec<MODE>;
    constexpr int kTileVecs = kTile * C::kBytes / 16;          // 1024, 512 or 256
    constexpr int kUnitVecs = G::kThreads * G::kQuads;
    if constexpr (kUnitVecs <= kTileVecs) {
        constexpr int kSplit = kTileVecs / kUnitVecs;
        constexpr int kUnitElems = kTile / kSplit;
        const int r = blockIdx.y;
        const int chunk = mod_p(r - a.chunk_rot, a.p);
        // one pass when the grid covers all units; fewer workgroups than units
        // make each of them walk the range (a link of limited bandwidth)
        for (uint32_t u = blockIdx.x; u < a.units; u += gridDim.x) {
            const UnitRef t = locate<UnitOnly<kUnitElems>>(bt, u + a.slot_base * kSplit, chunk);
            if (t.empty) continue;
            copy_unit<MODE, G>(a.in[r], a.in_sc[r], a.out[r], a.out_sc[r], t);
        }
    }
}

// The whole chain of one unit in registers (blockIdx.y = chunk c):
// P = g_c; for j = 1..p-1: P = D(C(P)) + g_{c+j}; every slot <- C(P).
template <int MODE, class G, bool FULL>
__device__ __forceinline__ void ring_fused_body(const RingArgs &a, const UnitRef &t, int c, float (*red)[G::kWaves])
{
    const int p = a.p;
    float P[G::kPerThread], g[G::kPerThread], gnext[G::kPerThread];
    load_f32<G, FULL, kNtGrad>(a.g[c] + t.elem0, t.len, P);
    if (p > 1) load_f32<G, FULL, kNtGrad>(a.g[mod_p(c + 1, p)] + t.elem0, t.len, gnext);
    int flip = 0;
    for (int j = 1; j < p; ++j) {
#pragma unroll
        for (int k = 0; k < G::kPerThread; ++k) g[k] = gnext[k];
        // the next worker's block is requested before this hop's arithmetic
        if (j + 1 < p) load_f32<G, FULL, kNtGrad>(a.g[mod_p(c + j + 1, p)] + t.elem0, t.len, gnext);
        float scale = 0.0f;
        if constexpr (MODE == PIPESGD_QUANT8) { scale = tile_absmax<G>(P, red[flip]); flip ^= 1; }
        through_the_wire<MODE, G>(P, scale);
#pragma unroll
        for (int k = 0; k < G::kPerThread; ++k) P[k] = P[k] + g[k];
    }
    float scale = 0.0f;
    if constexpr (MODE == PIPESGD_QUANT8) scale = tile_absmax<G>(P, red[flip]);
    for (int r = 0; r < p; ++r) store_payload<MODE, G, FULL, true>(a.out[r], a.out_sc[r], t.elem0, t.len, scale, P);
}

template <int MODE, class G>
__global__ __launch_bounds__(G::kThreads) void ring_fused_kernel(RingArgs a, BucketTable bt)
{
    if constexpr (RangeOk<MODE, G>::value) {
        __shared__ float red[2][G::kWaves];
        const int c = blockIdx.y;
        const UnitRef t = locate<G>(bt, blockIdx.x + a.slot_base * G::kSplit, c);
        if (t.empty) return;
        if (t.full) ring_fused_body<MODE, G, true>(a, t, c, red);
        else        ring_fused_body<MODE, G, false>(a, t, c, red);
    }
}

// Owner-side reduction of the one-exchange ("direct") schedule, blockIdx.y =
// owner j = chunk j: P = g_j; for d = 1..p-1: P = P + D(in_{(j+d) mod p}); every
// slot <- C(P).  in_k is what worker k sent: its own compressed copy of chunk j.
template <int MODE, class G, bool FULL>
__device__ __forceinline__ void direct_reduce_body(const RingArgs &a, const UnitRef &t, int j, float *red)
{
    const int p = a.p;
    float P[G::kPerThread], x[G::kPerThread];
    load_f32<G, FULL, kNtGrad>(a.g[j] + t.elem0, t.len, P);
    for (int d = 1; d < p; ++d) {
        const int k = mod_p(j + d, p);
        const float scale_in = MODE == PIPESGD_QUANT8 ? a.in_sc[k][t.elem0 / kTile] : 0.0f;
        load_payload<MODE, G, FULL, kNtPayIn>(a.in[k], t.elem0, t.len, scale_in, x);
#pragma unroll
        for (int i = 0; i < G::kPerThread; ++i) P[i] = P[i] + x[i];
    }
    float scale = 0.0f;
    if constexpr (MODE == PIPESGD_QUANT8) scale = tile_absmax<G>(P, red);
    for (int r = 0; r < p; ++r) store_payload<MODE, G, FULL, true>(a.out[r], a.out_sc[r], t.elem0, t.len, scale, P);
}

template <int MODE, class G>
__global__ __launch_bounds__(G::kThreads) void direct_reduce_kernel(RingArgs a, BucketTable bt)
{
    if constexpr (RangeOk<MODE, G>::value) {
        __shared__ float red[G::kWaves];
        const int j = blockIdx.y;
        const UnitRef t = locate<G>(bt, blockIdx.x + a.slot_base * G::kSplit, j);
        if (t.empty) return;
        if (t.full) direct_reduce_body<MODE, G, true>(a, t, j, red);
        else        direct_reduce_body<MODE, G, false>(a, t, j, red);
    }
}

// ---- recursive halving and doubling (Sec. 3.1 names it beside the ring) ----
// One launch for every worker (blockIdx.y = r).  The worker handles `half`
// consecutive chunks (blockIdx.z): those starting at r with the bits below
// `half` cleared (the chunks it keeps in this round), or that start XOR `flip`.
struct HdArgs {
    const float *src[kMaxW];    // fp32 operand: the local gradient, later the worker's partial sums
    const void *in[kMaxW];      // what the worker receives: the partner's send buffer (or slot, when doubling)
    const float *in_sc[kMaxW];
    void *pay[kMaxW];           // payload written: the worker's send buffer, or its result slot
    float *pay_sc[kMaxW];
    float *acc[kMaxW];          // partial sums the worker keeps in fp32
    int half;
    int flip;
    int next_half;              // kHdReduce: chunks that differ from r in this bit are sent next, so they leave as payload
};
enum { kHdSend = 0, kHdReduce = 1, kHdLast = 2 };

__device__ __forceinline__ int hd_chunk(const HdArgs &a, int r)
{
    return ((r & ~(a.half - 1)) ^ a.flip) + static_cast<int>(blockIdx.z);
}

//   kHdSend  : C(src_r)                -> pay_r            (first round's message)
//   kHdReduce: P = src_r + D(in_r);  P -> acc_r  for the chunks kept next round,
//                                  C(P) -> pay_r  for the chunks sent next round
//   kHdLast  : C(src_r + D(in_r))      -> pay_r            (the worker's own block, fully reduced)
template <int MODE, int STAGE, class G, bool FULL>
__device__ __forceinline__ void hd_body(const HdArgs &a, const UnitRef &t, int r, bool as_payload, float *red)
{
    float P[G::kPerThread];
    float x[G::kPerThread];
    if (STAGE != kHdSend) {
        const float scale_in = MODE == PIPESGD_QUANT8 ? a.in_sc[r][t.elem0 / kTile] : 0.0f;
        load_payload<MODE, G, FULL, kNtPayIn>(a.in[r], t.elem0, t.len, scale_in, x);
    }
    load_f32<G, FULL, kNtGrad>(a.src[r] + t.elem0, t.len, P);
    if (STAGE != kHdSend) {
#pragma unroll
        for (int k = 0; k < G::kPerThread; ++k) P[k] = P[k] + x[k];
    }
    if (as_payload) {                                   // uniform over the workgroup
        float scale = 0.0f;
        if constexpr (MODE == PIPESGD_QUANT8) scale = tile_absmax<G>(P, red);
        store_payload<MODE, G, FULL, kNtPayOut>(a.pay[r], a.pay_sc[r], t.elem0, t.len, scale, P);
    } else {
        store_f32<G, FULL, false>(a.acc[r] + t.elem0, t.len, P);
    }
}

template <int MODE, int STAGE, class G>
__global__ __launch_bounds__(G::kThreads) void hd_kernel(HdArgs a, BucketTable bt)
{
    if constexpr (RangeOk<MODE, G>::value) {
        __shared__ float red[G::kWaves];
        const int r = blockIdx.y;
        const int chunk = hd_chunk(a, r);
        const UnitRef t = locate<G>(bt, blockIdx.x, chunk);
        if (t.empty) return;
        const bool as_payload = STAGE != kHdReduce || ((chunk ^ r) & a.next_half) != 0;
        if (t.full) hd_body<MODE, STAGE, G, true>(a, t, r, as_payload, red);
        else        hd_body<MODE, STAGE, G, false>(a, t, r, as_payload, red);
    }
}

// Doubling round: worker r copies, byte for byte, the `half` chunks its partner holds.
template <int MODE, class G>
__global__ __launch_bounds__(G::kThreads) void hd_copy_kernel(HdArgs a, BucketTable bt)
{
    using C = Codec<MODE>;
    constexpr int kTileVecs = kTile * C::kBytes / 16;
    constexpr int kUnitVecs = G::kThreads * G::kQuads;
    if constexpr (kUnitVecs <= kTileVecs) {
        constexpr int kSplit = kTileVecs / kUnitVecs;
        constexpr int kUnitElems = kTile / kSplit;
        const int r = blockIdx.y;
        const UnitRef t = locate<UnitOnly<kUnitElems>>(bt, blockIdx.x, hd_chunk(a, r));
        if (t.empty) return;
        copy_unit<MODE, G>(a.in[r], a.in_sc[r], a.pay[r], a.pay_sc[r], t);
    }
}

// Stand-alone codec over a flat vector (blockIdx.x = unit).
template <int MODE, class G, bool FULL>
__device__ __forceinline__ void compress_body(const float *src, const UnitRef &t, void *pay, float *sc, float *red)
{
    float x[G::kPerThread];
    load_f32<G, FULL, true>(src + t.elem0, t.len, x);
    float scale = 0.0f;
    if constexpr (MODE == PIPESGD_QUANT8) scale = tile_absmax<G>(x, red);
    store_payload<MODE, G, FULL, kNtCodecOut>(pay, sc, t.elem0, t.len, scale, x);
}

template <int MODE, class G>
__global__ __launch_bounds__(G::kThreads) void compress_kernel(const float *src, uint64_t n, void *pay, float *sc)
{
    if constexpr (RangeOk<MODE, G>::value) {
        __shared__ float red[G::kWaves];
        const UnitRef t = locate_flat<G>(n, blockIdx.x);
        if (t.full) compress_body<MODE, G, true>(src, t, pay, sc, red);
        else        compress_body<MODE, G, false>(src, t, pay, sc, red);
    }
}

template <int MODE, class G, bool FULL>
__device__ __forceinline__ void decompress_body(const void *pay, float scale, const UnitRef &t, float *dst)
{
    float x[G::kPerThread];
    load_payload<MODE, G, FULL, true>(pay, t.elem0, t.len, scale, x);
    store_f32<G, FULL, kNtCodecOut>(dst + t.elem0, t.len, x);
}

template <int MODE, class G>
__global__ __launch_bounds__(G::kThreads) void decompress_kernel(const void *pay, const float *sc, uint64_t n, float *dst)
{
    const UnitRef t = locate_flat<G>(n, blockIdx.x);
    const float scale = MODE == PIPESGD_QUANT8 ? sc[t.elem0 / kTile] : 0.0f;
    if (t.full) decompress_body<MODE, G, true>(pay, scale, t, dst);
    else        decompress_body<MODE, G, false>(pay, scale, t, dst);
}

// Decompress + momentum-SGD step (Alg. 1 compute thread lines 4-5) for every
// replica (blockIdx.y): reads the stale slot, v and w once, writes v and w once.
template <int MODE, bool MOMENTUM, class G, bool FULL>
__device__ __forceinline__ void update_body(const UpdateArgs &a, const UnitRef &t, int r, float scale)
{
    float *w = a.w[r] + t.elem0;
    float *v = MOMENTUM ? a.v[r] + t.elem0 : nullptr;

    float g[G::kPerThread], wv[G::kPerThread], vv[G::kPerThread];
    load_payload<MODE, G, FULL, kNtUpdate>(a.pay[r], t.elem0, t.len, scale, g);
    load_f32<G, FULL, kNtUpdate>(w, t.len, wv);
    if (MOMENTUM) load_f32<G, FULL, kNtUpdate>(v, t.len, vv);

    const float gs = a.grad_scale, m = a.momentum, neg_lr = -a.lr;
    if (gs != 1.0f) {
#pragma unroll
        for (int k = 0; k < G::kPerThread; ++k) g[k] = g[k] * gs;
    }
#pragma unroll
    for (int k = 0; k < G::kPerThread; ++k) {
        if (MOMENTUM) {
            vv[k] = fmaf(m, vv[k], g[k]);
            wv[k] = fmaf(neg_lr, vv[k], wv[k]);
        } else {
            wv[k] = fmaf(neg_lr, g[k], wv[k]);
        }
    }
    if (MOMENTUM) store_f32<G, FULL, kNtUpdate>(v, t.len, vv);
    store_f32<G, FULL, kNtUpdate>(w, t.len, wv);
}

template <int MODE, bool MOMENTUM, class G>
__global__ __launch_bounds__(G::kThreads) void update_kernel(UpdateArgs a)
{
    const int r = blockIdx.y;
    const UnitRef t = locate_flat<G>(a.n, blockIdx.x);
    const float scale = MODE == PIPESGD_QUANT8 ? a.sc[r][t.elem0 / kTile] : 0.0f;
    if (t.full) update_body<MODE, MOMENTUM, G, true>(a, t, r, scale);
    else        update_body<MODE, MOMENTUM, G, false>(a, t, r, scale);
}

// Measurement aid, not part of the method: the update's memory streams with the
// arithmetic taken out, over the update's own buffers and grid.  Whole units only.
//   kProbeRead : loads slot, w, v of a unit; stores nothing (the loads feed a test that never holds)
//   kProbeWrite: stores a bit pattern derived from the index into w and v
//   kProbeMixed: loads slot, w, v; stores v's values into w and w's into v -- the
//                update's 10 bytes read : 8 written per element (TRUNC16), no FMAs
//   kProbeCopy : loads w, stores it into v (the classic 1 : 1 copy)
enum { kProbeRead = 0, kProbeWrite = 1, kProbeMixed = 2, kProbeCopy = 3 };

template <int MODE, int KIND, class G>
__global__ __launch_bounds__(G::kThreads) void stream_probe_kernel(UpdateArgs a, uint32_t salt)
{
    const int r = blockIdx.y;
    const uint64_t e0 = static_cast<uint64_t>(blockIdx.x) * G::kUnit;
    float *w = a.w[r] + e0;
    float *v = a.v[r] + e0;
    float g[G::kPerThread], wv[G::kPerThread], vv[G::kPerThread];
    if (KIND == kProbeRead || KIND == kProbeMixed) {
        load_payload<MODE, G, true, kNtUpdate>(a.pay[r], e0, G::kUnit, 1.0f, g);
        load_f32<G, true, kNtUpdate>(w, G::kUnit, wv);
        load_f32<G, true, kNtUpdate>(v, G::kUnit, vv);
    } else if (KIND == kProbeCopy) {
        load_f32<G, true, kNtUpdate>(w, G::kUnit, wv);
    }
    if (KIND == kProbeRead) {
        uint32_t acc = 0;
#pragma unroll
        for (int k = 0; k < G::kPerThread; ++k) acc |= f2u(g[k]) ^ f2u(wv[k]) ^ f2u(vv[k]);
        if (acc == salt) w[threadIdx.x] = u2f(salt);          // the compiler cannot rule it out, so every load stays;
                                                              // in practice it never holds (and the probes' data is scratch)
    } else if (KIND == kProbeWrite) {
#pragma unroll
        for (int k = 0; k < G::kPerThread; ++k) {
            const uint32_t h = (static_cast<uint32_t>(e0) + threadIdx.x * G::kPerThread + k) * 2654435761u + salt;
            wv[k] = u2f(0x3a000000u | (h >> 9));               // finite, varied mantissas, magnitudes near 5e-4
            vv[k] = u2f(0xba000000u | (h & 0x007fffffu));
        }
        store_f32<G, true, kNtUpdate>(v, G::kUnit, vv);
        store_f32<G, true, kNtUpdate>(w, G::kUnit, wv);
    } else if (KIND == kProbeMixed) {
        uint32_t acc = 0;
#pragma unroll
        for (int k = 0; k < G::kPerThread; ++k) acc |= f2u(g[k]);
        if (acc == salt) vv[0] = u2f(salt);                   // as above: keeps every payload load alive
        store_f32<G, true, kNtUpdate>(v, G::kUnit, wv);
        store_f32<G, true, kNtUpdate>(w, G::kUnit, vv);
    } else {
        store_f32<G, true, kNtUpdate>(v, G::kUnit, wv);
    }
}

// A whole width-2 iteration in ONE launch, for gradients so small that launch
// latency, not bandwidth, sets the pace: the AllReduce of this iteration's
// gradients (chain in registers, as in ring_fused_kernel) and the update from
// the previous iteration's slot touch disjoint buffers (that independence is
// the paper's pipeline), so they can share a grid.  Workgroups with
// blockIdx.x < ring_blocks walk a ring unit of chunk blockIdx.y, the others
// update a unit of replica blockIdx.y.
template <int MODE, bool MOMENTUM>
__global__ __launch_bounds__(256) void iteration_fused_kernel(RingArgs a, BucketTable bt, UpdateArgs u, uint32_t ring_blocks)
{
    using G = Geo<256, 4>;
    __shared__ float red[2][G::kWaves];
    if (blockIdx.x < ring_blocks) {
        const int c = blockIdx.y;
        if (c >= a.p) return;
        const UnitRef t = locate<G>(bt, blockIdx.x, c);
        if (t.empty) return;
        if (t.full) ring_fused_body<MODE, G, true>(a, t, c, red);
        else        ring_fused_body<MODE, G, false>(a, t, c, red);
    } else {
        const int r = blockIdx.y;
        const uint32_t unit = blockIdx.x - ring_blocks;
        if (static_cast<uint64_t>(unit) * G::kUnit >= u.n) return;
        const UnitRef t = locate_flat<G>(u.n, unit);
        const float scale = MODE == PIPESGD_QUANT8 ? u.sc[r][t.elem0 / kTile] : 0.0f;
        if (t.full) update_body<MODE, MOMENTUM, G, true>(u, t, r, scale);
        else        update_body<MODE, MOMENTUM, G, false>(u, t, r, scale);
    }
}

// Many tensor <-> packed-buffer copies in one launch.  The segment table is in
// device memory; a block finds its segment by binary search on first_tile.
template <bool TO_PACKED>
__global__ __launch_bounds__(256) void segment_copy_kernel(const pipesgd_segment *seg, uint32_t num)
{
    using G = Geo<256, 4>;
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
    const float *in = (TO_PACKED ? s.tensor : s.packed) + e0;
    float *out = (TO_PACKED ? s.packed : s.tensor) + e0;
    const bool whole = rem >= static_cast<uint64_t>(kTile);
    const bool aligned = ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & 15) == 0;
    if (whole && aligned) {
        float x[G::kPerThread];
        load_f32_full<G, true>(in, x);
        store_f32<G, true, false>(out, kTile, x);
    } else {
        // tensors sit at arbitrary 4-byte offsets inside a bucket: element-wise, still coalesced
        for (uint64_t i = threadIdx.x; i < rem && i < static_cast<uint64_t>(kTile); i += 256) out[i] = in[i];
    }
}

// --------------------------------------------------------- launch configs --

enum KernelKind { kFirstSend = 0, kReduceScatter, kAllGather, kFused, kUpdate, kCompress, kDecompress, kDirectReduce, kNumKinds };

struct LaunchConfig {
    int threads, quads;
    int lds_bytes;           // dynamic LDS reserved per workgroup: caps resident workgroups per CU
};

// Defaults from sweeps on MI355X (NONE at 25.6M elements per worker, TRUNC16 at
// 61M, QUANT8 at 138M; p = 4; buffers staggered within the 4 KiB channel
// interleave).  The update is fastest with about 24-30 KiB of loads in flight per
// compute unit: small workgroups and an LDS reservation that admits two or three
// of them per CU.  The hop kernels are nearly flat across geometries.  [kind][mode]
// Each entry is one atomic word, so a launch that reads it while another thread
// calls pipesgd_set_launch_config uses the old or the new geometry, never a
// mixture of the two.
constexpr uint64_t pack_cfg(int threads, int quads, int lds_bytes)
{
    return static_cast<uint64_t>(threads) | (static_cast<uint64_t>(quads) << 16) | (static_cast<uint64_t>(lds_bytes) << 32);
}
std::atomic<uint64_t> g_cfg[kNumKinds][3] = {
    /* first send     */ {pack_cfg(256, 4, 0), pack_cfg(128, 2, 0), pack_cfg(512, 2, 32768)},
    /* reduce-scatter */ {pack_cfg(128, 2, 0), pack_cfg(128, 2, 0), pack_cfg(256, 4, 32768)},
    /* all-gather     */ {pack_cfg(128, 2, 0), pack_cfg(256, 2, 0), pack_cfg(256, 1, 0)},
    /* fused          */ {pack_cfg(256, 1, 0), pack_cfg(512, 1, 49152), pack_cfg(256, 4, 61440)},
    /* update         */ {pack_cfg(256, 1, 65536), pack_cfg(64, 4, 53248), pack_cfg(64, 4, 53248)},
    /* compress       */ {pack_cfg(256, 4, 0), pack_cfg(128, 4, 16384), pack_cfg(512, 2, 0)},
    /* decompress     */ {pack_cfg(256, 4, 0), pack_cfg(256, 2, 0), pack_cfg(256, 4, 49152)},
    /* direct reduce  */ {pack_cfg(256, 1, 0), pack_cfg(512, 1, 0), pack_cfg(512, 2, 32768)},
};
inline LaunchConfig cfg_of(int kind, int mode)
{
    const uint64_t v = g_cfg[kind][mode].load(std::memory_order_relaxed);
    return LaunchConfig{static_cast<int>(v & 0xffff), static_cast<int>((v >> 16) & 0xffff), static_cast<int>(v >> 32)};
}

constexpr int kMaxLds = 159 * 1024;        // a CU has 160 KiB; leave room for the kernels' own few bytes

#define PIPESGD_FOR_EACH_GEO(X) X(64, 4) X(128, 2) X(128, 4) X(256, 1) X(256, 2) X(256, 4) X(512, 1) X(512, 2) X(1024, 1)

inline bool geo_known(int threads, int quads)
{
#define X(T, Q) if (threads == T && quads == Q) return true;
    PIPESGD_FOR_EACH_GEO(X)
#undef X
    return false;
}

// Does this geometry work for this kernel kind and mode?
bool config_ok(int kind, int mode, const LaunchConfig &c)
{
    if (!geo_known(c.threads, c.quads) || c.lds_bytes < 0 || c.lds_bytes > kMaxLds) return false;
    const int unit_quads = c.threads * c.quads;
    if (kind == kAllGather) {
        const int tile_vecs = kTile * (mode == PIPESGD_NONE ? 4 : mode == PIPESGD_TRUNC16 ? 2 : 1) / 16;
        return unit_quads <= tile_vecs;
    }
    const bool needs_range = mode == PIPESGD_QUANT8 && (kind == kFirstSend || kind == kReduceScatter || kind == kFused ||
                                                        kind == kCompress || kind == kDirectReduce);
    return !needs_range || unit_quads == kTileQuads;
}

// Kernels that reserve more than 64 KiB of dynamic LDS must say so once per device.
template <typename K>
int allow_lds(K kernel, int lds_bytes, std::atomic<uint32_t> &done_mask)
{
    if (lds_bytes <= 64 * 1024) return PIPESGD_OK;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return PIPESGD_ERR_HIP;
    const uint32_t bit = 1u << (dev & 31);
    if (done_mask.load(std::memory_order_acquire) & bit) return PIPESGD_OK;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds) != hipSuccess)
        return PIPESGD_ERR_HIP;
    done_mask.fetch_or(bit, std::memory_order_release);
    return PIPESGD_OK;
}

template <typename K, typename... Args>
int launch(K kernel, dim3 grid, int threads, int lds_bytes, hipStream_t s, std::atomic<uint32_t> &done_mask, Args... args)
{
    const int rc = allow_lds(kernel, lds_bytes, done_mask);
    if (rc != PIPESGD_OK) return rc;
    hipLaunchKernelGGL(kernel, grid, dim3(threads), lds_bytes, s, args...);
    return hipGetLastError() == hipSuccess ? PIPESGD_OK : PIPESGD_ERR_HIP;
}

// ------------------------------------------------------------ host helpers --

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline bool mode_ok(int mode) { return mode == PIPESGD_NONE || mode == PIPESGD_TRUNC16 || mode == PIPESGD_QUANT8; }

// Validates a ring and turns it into kernel arguments.  total_slots = tile
// slots of one ring block, summed over buckets.
int prepare_ring(const pipesgd_ring *ring, RingArgs &ra, BucketTable &bt, uint64_t &total_slots)
{
    if (!ring) return PIPESGD_ERR_ARG;
    if (!mode_ok(ring->mode)) return PIPESGD_ERR_MODE;
    if (ring->workers < 1 || ring->reserved != 0) return PIPESGD_ERR_ARG;
    if (ring->workers > kMaxW || ring->num_buckets > static_cast<uint32_t>(kMaxB)) return PIPESGD_ERR_CAPACITY;
    if (ring->num_buckets > 0 && !ring->buckets) return PIPESGD_ERR_ARG;
    const int p = ring->workers;
    for (int r = 0; r < kMaxW; ++r) {
        ra.g[r] = nullptr; ra.in[r] = nullptr; ra.in_sc[r] = nullptr; ra.out[r] = nullptr; ra.out_sc[r] = nullptr;
    }
    const bool q8 = ring->mode == PIPESGD_QUANT8;         // scales[] is read in this mode only
    for (int r = 0; r < p; ++r) {
        if (ring->n > 0) {
            if (!ring->g_local[r] || !ring->g_sum_c[r]) return PIPESGD_ERR_ARG;
            if (q8 && !ring->scales[r]) return PIPESGD_ERR_ARG;
        }
        if (!aligned16(ring->g_local[r]) || !aligned16(ring->g_sum_c[r]) || (q8 && !aligned16(ring->scales[r])))
            return PIPESGD_ERR_ALIGN;
        ra.g[r] = ring->g_local[r];
        ra.out[r] = ring->g_sum_c[r];
        ra.out_sc[r] = q8 ? ring->scales[r] : nullptr;
    }
    // default wiring: worker r receives what worker r-1 holds in its slot
    for (int r = 0; r < p; ++r) {
        const int src = (r + p - 1) % p;
        ra.in[r] = ring->g_sum_c[src];
        ra.in_sc[r] = q8 ? ring->scales[src] : nullptr;
    }
    ra.p = p;
    ra.chunk_rot = 0;
    ra.slot_base = 0;
    ra.units = 0;

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
        if (slots > 0x07ffffffull) return PIPESGD_ERR_CAPACITY;      // x 8 units per tile still fits gridDim.x
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

// Staging a schedule needs, checked against what the caller says it has
// allocated.  `kind` is a PIPESGD_WS_* schedule.  On success stage / stage_sc /
// partial hold the p buffers (nullptr where the schedule and mode need none).
struct Staging {
    void *stage[kMaxW];
    float *stage_sc[kMaxW];
    float *partial[kMaxW];
};
int check_workspace(const pipesgd_ring *ring, const pipesgd_workspace *ws, int kind, Staging &st)
{
    for (int r = 0; r < kMaxW; ++r) { st.stage[r] = nullptr; st.stage_sc[r] = nullptr; st.partial[r] = nullptr; }
    uint64_t need[3];
    const int rc = pipesgd_workspace_bytes(kind, ring->mode, ring->n, ring->workers, need);
    if (rc != PIPESGD_OK) return rc;
    if (need[0] == 0 && need[1] == 0 && need[2] == 0) return PIPESGD_OK;      // one worker or an empty vector
    if (!ws) return PIPESGD_ERR_ARG;
    const int p = ring->workers;
    if ((need[0] && !ws->stage) || (need[1] && !ws->stage_scales) || (need[2] && !ws->partial)) return PIPESGD_ERR_ARG;
    for (int r = 0; r < p; ++r) {
        if ((need[0] && !ws->stage[r]) || (need[1] && !ws->stage_scales[r]) || (need[2] && !ws->partial[r]))
            return PIPESGD_ERR_ARG;
        if ((need[0] && !aligned16(ws->stage[r])) || (need[1] && !aligned16(ws->stage_scales[r])) ||
            (need[2] && !aligned16(ws->partial[r])))
            return PIPESGD_ERR_ALIGN;
    }
    if (ws->stage_bytes < need[0] || (need[1] && ws->stage_scales_bytes < need[1]) ||
        (need[2] && ws->partial_bytes < need[2]))
        return PIPESGD_ERR_CAPACITY;
    for (int r = 0; r < p; ++r) {
        st.stage[r] = ws->stage[r];
        st.stage_sc[r] = need[1] ? ws->stage_scales[r] : nullptr;
        st.partial[r] = need[2] ? ws->partial[r] : nullptr;
    }
    return PIPESGD_OK;
}

// ---- per-kind dispatch over (mode, geometry) ----

#define PIPESGD_MODE_SWITCH(mode, CALL)                      \
    switch (mode) {                                          \
    case PIPESGD_NONE:    CALL(PIPESGD_NONE) break;          \
    case PIPESGD_TRUNC16: CALL(PIPESGD_TRUNC16) break;       \
    default:              CALL(PIPESGD_QUANT8) break;        \
    }

template <int MODE, bool HAS_IN>
int launch_hop(const LaunchConfig &c, const RingArgs &ra, const BucketTable &bt, uint64_t slots, int zdim, hipStream_t s)
{
#define X(T, Q)                                                                                                  \
    if (c.threads == T && c.quads == Q) {                                                                        \
        static std::atomic<uint32_t> done{0};                                                                    \
        using G = Geo<T, Q>;                                                                                     \
        return launch(ring_hop_kernel<MODE, HAS_IN, G>, dim3(static_cast<uint32_t>(slots * G::kSplit), ra.p, zdim), T, \
                      c.lds_bytes, s, done, ra, bt);                                                             \
    }
    PIPESGD_FOR_EACH_GEO(X)
#undef X
    return PIPESGD_ERR_ARG;
}

template <int MODE>
int launch_copy(const LaunchConfig &c, RingArgs ra, const BucketTable &bt, uint64_t slots, uint32_t max_groups, hipStream_t s)
{
    constexpr int kTileVecs = kTile * Codec<MODE>::kBytes / 16;
#define X(T, Q)                                                                                                  \
    if (c.threads == T && c.quads == Q) {                                                                        \
        if constexpr (T * Q <= kTileVecs) {                                                                      \
            static std::atomic<uint32_t> done{0};                                                                \
            constexpr int kSplit = kTileVecs / (T * Q);                                                          \
            ra.units = static_cast<uint32_t>(slots * kSplit);                                                    \
            const uint32_t gx = (max_groups && max_groups < ra.units) ? max_groups : ra.units;                   \
            return launch(ring_copy_kernel<MODE, Geo<T, Q>>, dim3(gx, ra.p), T, c.lds_bytes, s, done, ra, bt);   \
        }                                                                                                        \
    }
    PIPESGD_FOR_EACH_GEO(X)
#undef X
    return PIPESGD_ERR_ARG;
}

template <int MODE>
int launch_fused(const LaunchConfig &c, const RingArgs &ra, const BucketTable &bt, uint64_t slots, hipStream_t s)
{
#define X(T, Q)                                                                                                  \
    if (c.threads == T && c.quads == Q) {                                                                        \
        static std::atomic<uint32_t> done{0};                                                                    \
        using G = Geo<T, Q>;                                                                                     \
        return launch(ring_fused_kernel<MODE, G>, dim3(static_cast<uint32_t>(slots * G::kSplit), ra.p), T,       \
                      c.lds_bytes, s, done, ra, bt);                                                             \
    }
    PIPESGD_FOR_EACH_GEO(X)
#undef X
    return PIPESGD_ERR_ARG;
}

template <int MODE>
int launch_direct_reduce(const LaunchConfig &c, const RingArgs &ra, const BucketTable &bt, uint64_t slots, hipStream_t s)
{
#define X(T, Q)                                                                                                  \
    if (c.threads == T && c.quads == Q) {                                                                        \
        static std::atomic<uint32_t> done{0};                                                                    \
        using G = Geo<T, Q>;                                                                                     \
        return launch(direct_reduce_kernel<MODE, G>, dim3(static_cast<uint32_t>(slots * G::kSplit), ra.p), T,    \
                      c.lds_bytes, s, done, ra, bt);                                                             \
    }
    PIPESGD_FOR_EACH_GEO(X)
#undef X
    return PIPESGD_ERR_ARG;
}

template <int MODE>
int launch_compress(const LaunchConfig &c, const float *src, uint64_t n, void *pay, float *sc, hipStream_t s)
{
#define X(T, Q)                                                                                                  \
    if (c.threads == T && c.quads == Q) {                                                                        \
        static std::atomic<uint32_t> done{0};                                                                    \
        using G = Geo<T, Q>;                                                                                     \
        const uint64_t units = (n + G::kUnit - 1) / G::kUnit;                                                    \
        if (units > 0x7fffffffull) return PIPESGD_ERR_CAPACITY;                                                  \
        return launch(compress_kernel<MODE, G>, dim3(static_cast<uint32_t>(units)), T, c.lds_bytes, s, done,     \
                      src, n, pay, sc);                                                                          \
    }
    PIPESGD_FOR_EACH_GEO(X)
#undef X
    return PIPESGD_ERR_ARG;
}

template <int MODE>
int launch_decompress(const LaunchConfig &c, const void *pay, const float *sc, uint64_t n, float *dst, hipStream_t s)
{
#define X(T, Q)                                                                                                  \
    if (c.threads == T && c.quads == Q) {                                                                        \
        static std::atomic<uint32_t> done{0};                                                                    \
        using G = Geo<T, Q>;                                                                                     \
        const uint64_t units = (n + G::kUnit - 1) / G::kUnit;                                                    \
        if (units > 0x7fffffffull) return PIPESGD_ERR_CAPACITY;                                                  \
        return launch(decompress_kernel<MODE, G>, dim3(static_cast<uint32_t>(units)), T, c.lds_bytes, s, done,   \
                      pay, sc, n, dst);                                                                          \
    }
    PIPESGD_FOR_EACH_GEO(X)
#undef X
    return PIPESGD_ERR_ARG;
}

template <int MODE, bool MOMENTUM>
int launch_update(const LaunchConfig &c, const UpdateArgs &ua, int replicas, hipStream_t s)
{
#define X(T, Q)                                                                                                  \
    if (c.threads == T && c.quads == Q) {                                                                        \
        static std::atomic<uint32_t> done{0};                                                                    \
        using G = Geo<T, Q>;                                                                                     \
        const uint64_t units = (ua.n + G::kUnit - 1) / G::kUnit;                                                 \
        if (units > 0x7fffffffull) return PIPESGD_ERR_CAPACITY;                                                  \
        return launch(update_kernel<MODE, MOMENTUM, G>, dim3(static_cast<uint32_t>(units), replicas), T,         \
                      c.lds_bytes, s, done, ua);                                                                 \
    }
    PIPESGD_FOR_EACH_GEO(X)
#undef X
    return PIPESGD_ERR_ARG;
}

template <int MODE, int KIND>
int launch_probe(const LaunchConfig &c, const UpdateArgs &ua, int replicas, hipStream_t s)
{
#define X(T, Q)                                                                                                  \
    if (c.threads == T && c.quads == Q) {                                                                        \
        static std::atomic<uint32_t> done{0};                                                                    \
        using G = Geo<T, Q>;                                                                                     \
        const uint64_t units = ua.n / G::kUnit;                                                                  \
        if (units > 0x7fffffffull) return PIPESGD_ERR_CAPACITY;                                                  \
        if (units == 0) return PIPESGD_OK;                                                                       \
        return launch(stream_probe_kernel<MODE, KIND, G>, dim3(static_cast<uint32_t>(units), replicas), T,       \
                      c.lds_bytes, s, done, ua, 0x9e3779b9u);                                                    \
    }
    PIPESGD_FOR_EACH_GEO(X)
#undef X
    return PIPESGD_ERR_ARG;
}

template <int MODE, int STAGE>
int launch_hd(const LaunchConfig &c, const HdArgs &ha, const BucketTable &bt, uint64_t slots, int p, hipStream_t s)
{
#define X(T, Q)                                                                                                  \
    if (c.threads == T && c.quads == Q) {                                                                        \
        static std::atomic<uint32_t> done{0};                                                                    \
        using G = Geo<T, Q>;                                                                                     \
        return launch(hd_kernel<MODE, STAGE, G>, dim3(static_cast<uint32_t>(slots * G::kSplit), p, ha.half), T,  \
                      c.lds_bytes, s, done, ha, bt);                                                             \
    }
    PIPESGD_FOR_EACH_GEO(X)
#undef X
    return PIPESGD_ERR_ARG;
}

template <int MODE>
int launch_hd_copy(const LaunchConfig &c, const HdArgs &ha, const BucketTable &bt, uint64_t slots, int p, hipStream_t s)
{
    constexpr int kTileVecs = kTile * Codec<MODE>::kBytes / 16;
#define X(T, Q)                                                                                                  \
    if (c.threads == T && c.quads == Q) {                                                                        \
        if constexpr (T * Q <= kTileVecs) {                                                                      \
            static std::atomic<uint32_t> done{0};                                                                \
            constexpr int kSplit = kTileVecs / (T * Q);                                                          \
            return launch(hd_copy_kernel<MODE, Geo<T, Q>>, dim3(static_cast<uint32_t>(slots * kSplit), p, ha.half), T, \
                          c.lds_bytes, s, done, ha, bt);                                                         \
        }                                                                                                        \
    }
    PIPESGD_FOR_EACH_GEO(X)
#undef X
    return PIPESGD_ERR_ARG;
}

// The four launches below work on tile slots [ra.slot_base, ra.slot_base + slots)
// of every bucket-chunk; the plain entry points pass the whole range.

int first_send_impl(int mode, RingArgs ra, const BucketTable &bt, uint64_t slots, hipStream_t s)
{
    // uncompressed, p > 1: the first round reads the sender's gradient in place
    if (slots == 0 || (mode == PIPESGD_NONE && ra.p > 1)) return PIPESGD_OK;
    const LaunchConfig c = cfg_of(kFirstSend, mode);
    ra.chunk_rot = 0;
#define CALL(M) return launch_hop<M, false>(c, ra, bt, slots, 1, s);
    PIPESGD_MODE_SWITCH(mode, CALL)
#undef CALL
    return PIPESGD_ERR_MODE;
}

// `staged`: worker r's incoming payload has been put into ra.in[r] by the
// caller (receive staging); otherwise it is read from the sender's buffers.
int rs_impl(int mode, RingArgs ra, const BucketTable &bt, uint64_t slots, int step, bool staged, hipStream_t s)
{
    const LaunchConfig c = cfg_of(kReduceScatter, mode);
    ra.chunk_rot = step + 1;
    if (!staged && mode == PIPESGD_NONE && step == 0)
        for (int r = 0; r < ra.p; ++r) ra.in[r] = ra.g[(r + ra.p - 1) % ra.p];
#define CALL(M) return launch_hop<M, true>(c, ra, bt, slots, 1, s);
    PIPESGD_MODE_SWITCH(mode, CALL)
#undef CALL
    return PIPESGD_ERR_MODE;
}

// Copy chunk (r - rot) mod p from ra.in[r] to ra.out[r] for every worker.
int copy_impl(int mode, RingArgs ra, const BucketTable &bt, uint64_t slots, int rot, uint32_t max_groups, hipStream_t s)
{
    const LaunchConfig c = cfg_of(kAllGather, mode);
    ra.chunk_rot = rot;
#define CALL(M) return launch_copy<M>(c, ra, bt, slots, max_groups, s);
    PIPESGD_MODE_SWITCH(mode, CALL)
#undef CALL
    return PIPESGD_ERR_MODE;
}

int fused_impl(int mode, const RingArgs &ra, const BucketTable &bt, uint64_t slots, hipStream_t s)
{
    const LaunchConfig c = cfg_of(kFused, mode);
#define CALL(M) return launch_fused<M>(c, ra, bt, slots, s);
    PIPESGD_MODE_SWITCH(mode, CALL)
#undef CALL
    return PIPESGD_ERR_MODE;
}

}  // namespace

// -------------------------------------------------- static scratch array --
// Send buffers of pipesgd_allreduce_direct_static: part of the code object, so
// every GPU that loads the library holds its own copy at its own address.  In
// host code the name `scratch` is only a handle for hipGetSymbolAddress; the
// device address it yields (kept per device below) is what the kernels get.
static __device__ __align__(256) unsigned char scratch[PIPESGD_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<unsigned char *> g_scratch_ptr[kMaxDevices];

// Device address of the current device's copy of `scratch`; looked up once per device.
int scratch_base(unsigned char **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return PIPESGD_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return PIPESGD_ERR_CAPACITY;
    unsigned char *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        void *sym = nullptr;
        if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) return PIPESGD_ERR_HIP;
        ptr = static_cast<unsigned char *>(sym);
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return PIPESGD_OK;
}

inline uint64_t round_up_256(uint64_t x) { return (x + 255) / 256 * 256; }

}  // namespace

// ------------------------------------------------------------ entry points --

extern "C" {

int pipesgd_set_launch_config(int kernel, int mode, int threads, int quads, int lds_bytes)
{
    if (kernel < 0 || kernel >= kNumKinds) return PIPESGD_ERR_ARG;
    if (!mode_ok(mode)) return PIPESGD_ERR_MODE;
    const LaunchConfig c = {threads, quads, lds_bytes};
    if (!config_ok(kernel, mode, c)) return PIPESGD_ERR_ARG;
    g_cfg[kernel][mode].store(pack_cfg(threads, quads, lds_bytes), std::memory_order_relaxed);
    return PIPESGD_OK;
}

int pipesgd_get_launch_config(int kernel, int mode, int *threads, int *quads, int *lds_bytes)
{
    if (kernel < 0 || kernel >= kNumKinds || !threads || !quads || !lds_bytes) return PIPESGD_ERR_ARG;
    if (!mode_ok(mode)) return PIPESGD_ERR_MODE;
    const LaunchConfig c = cfg_of(kernel, mode);
    *threads = c.threads;
    *quads = c.quads;
    *lds_bytes = c.lds_bytes;
    return PIPESGD_OK;
}

int pipesgd_compress(int mode, const float *src, uint64_t n, void *payload, float *scales, void *stream)
{
    if (!mode_ok(mode)) return PIPESGD_ERR_MODE;
    if (n == 0) return PIPESGD_OK;
    if (!src || !payload || (mode == PIPESGD_QUANT8 && !scales)) return PIPESGD_ERR_ARG;
    if (!aligned16(src) || !aligned16(payload) || (mode == PIPESGD_QUANT8 && !aligned16(scales))) return PIPESGD_ERR_ALIGN;
    const LaunchConfig c = cfg_of(kCompress, mode);
    hipStream_t s = static_cast<hipStream_t>(stream);
#define CALL(M) return launch_compress<M>(c, src, n, payload, scales, s);
    PIPESGD_MODE_SWITCH(mode, CALL)
#undef CALL
    return PIPESGD_ERR_MODE;
}

int pipesgd_decompress(int mode, const void *payload, const float *scales, uint64_t n, float *dst, void *stream)
{
    if (!mode_ok(mode)) return PIPESGD_ERR_MODE;
    if (n == 0) return PIPESGD_OK;
    if (!dst || !payload || (mode == PIPESGD_QUANT8 && !scales)) return PIPESGD_ERR_ARG;
    if (!aligned16(dst) || !aligned16(payload) || (mode == PIPESGD_QUANT8 && !aligned16(scales))) return PIPESGD_ERR_ALIGN;
    const LaunchConfig c = cfg_of(kDecompress, mode);
    hipStream_t s = static_cast<hipStream_t>(stream);
#define CALL(M) return launch_decompress<M>(c, payload, scales, n, dst, s);
    PIPESGD_MODE_SWITCH(mode, CALL)
#undef CALL
    return PIPESGD_ERR_MODE;
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
    return rs_impl(ring->mode, ra, bt, slots, step, false, static_cast<hipStream_t>(stream));
}

int pipesgd_ring_allgather_step(const pipesgd_ring *ring, int step, void *stream)
{
    RingArgs ra; BucketTable bt; uint64_t slots = 0;
    const int rc = prepare_ring(ring, ra, bt, slots);
    if (rc != PIPESGD_OK) return rc;
    if (step < 0 || step > ring->workers - 2) return PIPESGD_ERR_ARG;
    if (slots == 0) return PIPESGD_OK;
    return copy_impl(ring->mode, ra, bt, slots, step, 0, static_cast<hipStream_t>(stream));
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
    if (schedule == PIPESGD_FUSED) return fused_impl(mode, ra, bt, slots, s);
    rc = first_send_impl(mode, ra, bt, slots, s);
    for (int step = 0; rc == PIPESGD_OK && step <= p - 2; ++step) rc = rs_impl(mode, ra, bt, slots, step, false, s);
    for (int step = 0; rc == PIPESGD_OK && step <= p - 2; ++step) rc = copy_impl(mode, ra, bt, slots, step, 0, s);
    return rc;
}


// ------------------------------------------------- the one-exchange schedule --

// Both exchanges of the one-exchange schedule on validated arguments.
static int direct_impl(int mode, const RingArgs &ra, const BucketTable &bt, uint64_t slots, const Staging &st, hipStream_t s)
{
    const int p = ra.p;
    int rc = PIPESGD_OK;
    if (p > 1) {
        // exchange 1: worker k compresses every chunk it does not own into its send buffer
        // (chunks k-1, k-2, ..., k-(p-1) along gridDim.z)
        RingArgs sc = ra;
        for (int r = 0; r < p; ++r) { sc.out[r] = st.stage[r]; sc.out_sc[r] = st.stage_sc[r]; }
        sc.chunk_rot = 1;
        const LaunchConfig c = cfg_of(kFirstSend, mode);
#define CALL(M) rc = launch_hop<M, false>(c, sc, bt, slots, p - 1, s);
        PIPESGD_MODE_SWITCH(mode, CALL)
#undef CALL
        if (rc != PIPESGD_OK) return rc;
    }
    // owner j sums its own block and what the others sent, compresses once, and
    // (exchange 2) writes the result into every worker's slot
    RingArgs rd = ra;
    for (int r = 0; r < p; ++r) {
        rd.in[r] = p > 1 ? st.stage[r] : nullptr;
        rd.in_sc[r] = p > 1 ? st.stage_sc[r] : nullptr;
    }
    const LaunchConfig c2 = cfg_of(kDirectReduce, mode);
#define CALL(M) return launch_direct_reduce<M>(c2, rd, bt, slots, s);
    PIPESGD_MODE_SWITCH(mode, CALL)
#undef CALL
    return PIPESGD_ERR_MODE;
}

int pipesgd_allreduce_direct(const pipesgd_ring *ring, const pipesgd_workspace *ws, void *stream)
{
    RingArgs ra; BucketTable bt; uint64_t slots = 0;
    int rc = prepare_ring(ring, ra, bt, slots);
    if (rc != PIPESGD_OK) return rc;
    Staging st;
    rc = check_workspace(ring, ws, PIPESGD_WS_DIRECT, st);
    if (rc != PIPESGD_OK) return rc;
    if (slots == 0) return PIPESGD_OK;
    return direct_impl(ring->mode, ra, bt, slots, st, static_cast<hipStream_t>(stream));
}

int pipesgd_allreduce_direct_static(const pipesgd_ring *ring, void *stream)
{
    RingArgs ra; BucketTable bt; uint64_t slots = 0;
    int rc = prepare_ring(ring, ra, bt, slots);
    if (rc != PIPESGD_OK) return rc;
    const int mode = ring->mode, p = ring->workers;
    // the p send buffers and their scales, each at a multiple of 256 bytes of the array
    const uint64_t pay_stride = round_up_256(pipesgd_payload_bytes(mode, ring->n));
    const uint64_t sc_stride = round_up_256(4 * pipesgd_num_scales(mode, ring->n));
    if (pay_stride > PIPESGD_STATIC_SCRATCH_BYTES || sc_stride > PIPESGD_STATIC_SCRATCH_BYTES ||
        static_cast<uint64_t>(p) * (pay_stride + sc_stride) > PIPESGD_STATIC_SCRATCH_BYTES)
        return PIPESGD_ERR_CAPACITY;
    if (slots == 0) return PIPESGD_OK;
    Staging st;
    for (int r = 0; r < kMaxW; ++r) { st.stage[r] = nullptr; st.stage_sc[r] = nullptr; st.partial[r] = nullptr; }
    if (p > 1) {
        unsigned char *base = nullptr;
        rc = scratch_base(&base);
        if (rc != PIPESGD_OK) return rc;
        for (int r = 0; r < p; ++r) {
            st.stage[r] = base + static_cast<uint64_t>(r) * pay_stride;
            if (mode == PIPESGD_QUANT8)
                st.stage_sc[r] = reinterpret_cast<float *>(base + static_cast<uint64_t>(p) * pay_stride +
                                                           static_cast<uint64_t>(r) * sc_stride);
        }
    }
    return direct_impl(mode, ra, bt, slots, st, static_cast<hipStream_t>(stream));
}

// ------------------------------------------ recursive halving and doubling --

int pipesgd_allreduce_halving_doubling(const pipesgd_ring *ring, const pipesgd_workspace *ws, void *stream)
{
    RingArgs ra; BucketTable bt; uint64_t slots = 0;
    int rc = prepare_ring(ring, ra, bt, slots);
    if (rc != PIPESGD_OK) return rc;
    const int mode = ring->mode, p = ring->workers;
    if ((p & (p - 1)) != 0) return PIPESGD_ERR_ARG;
    Staging st;
    rc = check_workspace(ring, ws, PIPESGD_WS_HALVING_DOUBLING, st);
    if (rc != PIPESGD_OK) return rc;
    if (slots == 0) return PIPESGD_OK;
    const bool q8 = mode == PIPESGD_QUANT8;
    void *const *stage = st.stage;
    float *const *stage_scales = st.stage_sc;
    float *const *partial = st.partial;
    hipStream_t s = static_cast<hipStream_t>(stream);
    HdArgs ha;
    for (int r = 0; r < kMaxW; ++r) {
        ha.src[r] = nullptr; ha.in[r] = nullptr; ha.in_sc[r] = nullptr; ha.pay[r] = nullptr; ha.pay_sc[r] = nullptr;
        ha.acc[r] = nullptr;
    }
    ha.half = 1; ha.flip = 0; ha.next_half = 0;
    const LaunchConfig c_send = cfg_of(kFirstSend, mode), c_red = cfg_of(kReduceScatter, mode), c_copy = cfg_of(kAllGather, mode);

    if (p == 1) {                                        // nothing to exchange: the slot is C(g)
        ha.src[0] = ra.g[0]; ha.pay[0] = ra.out[0]; ha.pay_sc[0] = ra.out_sc[0];
#define CALL(M) return launch_hd<M, kHdSend>(c_send, ha, bt, slots, p, s);
        PIPESGD_MODE_SWITCH(mode, CALL)
#undef CALL
    }

    // first message: every worker compresses the half it gives away (uncompressed
    // payloads are read from the partner's gradient in place instead)
    if (mode != PIPESGD_NONE) {
        for (int r = 0; r < p; ++r) { ha.src[r] = ra.g[r]; ha.pay[r] = stage[r]; ha.pay_sc[r] = q8 ? stage_scales[r] : nullptr; }
        ha.half = p / 2; ha.flip = p / 2;
#define CALL(M) rc = launch_hd<M, kHdSend>(c_send, ha, bt, slots, p, s);
        PIPESGD_MODE_SWITCH(mode, CALL)
#undef CALL
        if (rc != PIPESGD_OK) return rc;
    }
    // halving rounds: receive, sum, and in the same pass compress what goes out next
    for (int h = p / 2; h >= 1; h /= 2) {
        const bool first = h == p / 2, last = h == 1;
        for (int r = 0; r < p; ++r) {
            const int partner = r ^ h;
            ha.src[r] = first ? ra.g[r] : partial[r];
            ha.in[r] = (first && mode == PIPESGD_NONE) ? static_cast<const void *>(ra.g[partner]) : stage[partner];
            ha.in_sc[r] = q8 ? stage_scales[partner] : nullptr;
            ha.pay[r] = last ? ra.out[r] : stage[r];
            ha.pay_sc[r] = last ? ra.out_sc[r] : (q8 ? stage_scales[r] : nullptr);
            ha.acc[r] = last ? nullptr : partial[r];
        }
        ha.half = h; ha.flip = 0; ha.next_half = h / 2;
        if (last) {
#define CALL(M) rc = launch_hd<M, kHdLast>(c_red, ha, bt, slots, p, s);
            PIPESGD_MODE_SWITCH(mode, CALL)
#undef CALL
        } else {
#define CALL(M) rc = launch_hd<M, kHdReduce>(c_red, ha, bt, slots, p, s);
            PIPESGD_MODE_SWITCH(mode, CALL)
#undef CALL
        }
        if (rc != PIPESGD_OK) return rc;
    }
    // doubling rounds: swap everything held so far with the partner at distance d
    for (int d = 1; d < p; d *= 2) {
        for (int r = 0; r < p; ++r) {
            const int partner = r ^ d;
            ha.in[r] = ra.out[partner]; ha.in_sc[r] = ra.out_sc[partner];
            ha.pay[r] = ra.out[r]; ha.pay_sc[r] = ra.out_sc[r];
        }
        ha.half = d; ha.flip = d; ha.next_half = 0;
#define CALL(M) rc = launch_hd_copy<M>(c_copy, ha, bt, slots, p, s);
        PIPESGD_MODE_SWITCH(mode, CALL)
#undef CALL
        if (rc != PIPESGD_OK) return rc;
    }
    return PIPESGD_OK;
}

// ------------------------------------------ pipelining within the AllReduce --

int pipesgd_overlap_create(pipesgd_overlap **out)
{
    if (!out) return PIPESGD_ERR_ARG;
    pipesgd_overlap *ov = new (std::nothrow) pipesgd_overlap();
    if (!ov) return PIPESGD_ERR_CAPACITY;
    *out = ov;
    return PIPESGD_OK;
}

void pipesgd_overlap_destroy(pipesgd_overlap *ov)
{
    if (!ov) return;
    for (hipEvent_t e : ov->events) (void)hipEventDestroy(e);
    delete ov;
}

static bool overlap_event(pipesgd_overlap *ov, size_t i, hipEvent_t *e)
{
    while (ov->events.size() <= i) {
        hipEvent_t ne;
        if (hipEventCreateWithFlags(&ne, hipEventDisableTiming) != hipSuccess) return false;
        ov->events.push_back(ne);
    }
    *e = ov->events[i];
    return true;
}

int pipesgd_allreduce_pipelined(const pipesgd_ring *ring, const pipesgd_workspace *ws,
                                int segments, int wire_workgroups, float link_us_per_mib, pipesgd_overlap *ov,
                                void *compute_stream, void *wire_stream)
{
    RingArgs ra; BucketTable bt; uint64_t slots = 0;
    int rc = prepare_ring(ring, ra, bt, slots);
    if (rc != PIPESGD_OK) return rc;
    if (!ov || segments < 1 || wire_workgroups < 0 || !(link_us_per_mib >= 0.0f)) return PIPESGD_ERR_ARG;
    if (segments > PIPESGD_MAX_SEGMENTS) return PIPESGD_ERR_CAPACITY;
    const int mode = ring->mode, p = ring->workers;
    Staging stg;
    rc = check_workspace(ring, ws, PIPESGD_WS_PIPELINED, stg);
    if (rc != PIPESGD_OK) return rc;
    // time on the link for `tiles` tiles of one worker's payload (all workers' links run in parallel);
    // the longest single delay is that of a whole ring block and must be one the stand-in accepts
    const double tile_mib = static_cast<double>(pipesgd_payload_bytes(mode, kTile)) / (1024.0 * 1024.0);
    auto link_us = [&](uint64_t tiles) { return static_cast<double>(link_us_per_mib) * tile_mib * static_cast<double>(tiles); };
    if (link_us(slots) > 1.0e6) return PIPESGD_ERR_ARG;
    if (slots == 0) return PIPESGD_OK;
    void *const *recv = stg.stage;
    float *const *recv_scales = stg.stage_sc;
    hipStream_t cs = static_cast<hipStream_t>(compute_stream), ws_ = static_cast<hipStream_t>(wire_stream);
    const uint64_t S = static_cast<uint64_t>(segments) < slots ? static_cast<uint64_t>(segments) : slots;
    auto seg_lo = [&](uint64_t g) { return slots * g / S; };
    auto link_delay = [&](uint64_t tiles, hipStream_t st) -> int {
        if (link_us_per_mib <= 0.0f) return PIPESGD_OK;
        return pipesgd_synthetic_compute(static_cast<float>(link_us(tiles)), 1, st);
    };

    // events: entry, all reduced, done; per sub-block "sent"; per (round, sub-block) "copied" and "reduced".
    // All of them exist before the first launch, so that running out of them cannot leave half an AllReduce enqueued.
    const size_t events_needed = 3 + S + 2 * S * static_cast<size_t>(p > 1 ? p - 1 : 0);
    try {
        hipEvent_t unused;
        if (!overlap_event(ov, events_needed - 1, &unused)) return PIPESGD_ERR_HIP;
    } catch (const std::bad_alloc &) {
        return PIPESGD_ERR_CAPACITY;
    }
    size_t next_event = 0;
    auto record = [&](hipStream_t st, hipEvent_t *out_e) -> bool {
        hipEvent_t e = ov->events[next_event++];
        if (hipEventRecord(e, st) != hipSuccess) return false;
        *out_e = e;
        return true;
    };
    auto wait = [&](hipStream_t st, hipEvent_t e) -> bool { return hipStreamWaitEvent(st, e, 0) == hipSuccess; };

    hipEvent_t entry;
    if (!record(cs, &entry) || !wait(ws_, entry)) return PIPESGD_ERR_HIP;

    hipEvent_t ready[PIPESGD_MAX_SEGMENTS];           // per sub-block: what the next wire copy must wait for
    for (uint64_t g = 0; g < S; ++g) ready[g] = entry;
    for (uint64_t g = 0; g < S; ++g) {                // first send, sub-block by sub-block
        RingArgs a = ra;
        a.slot_base = static_cast<uint32_t>(seg_lo(g));
        rc = first_send_impl(mode, a, bt, seg_lo(g + 1) - seg_lo(g), cs);
        if (rc != PIPESGD_OK) return rc;
        if (!(mode == PIPESGD_NONE && p > 1) && !record(cs, &ready[g])) return PIPESGD_ERR_HIP;
    }
    for (int step = 0; step <= p - 2; ++step) {
        for (uint64_t g = 0; g < S; ++g) {
            const uint64_t count = seg_lo(g + 1) - seg_lo(g);
            // stage 1, the compressed communication: the sender's payload travels into the receiver's staging
            RingArgs w = ra;
            w.slot_base = static_cast<uint32_t>(seg_lo(g));
            for (int r = 0; r < p; ++r) {
                const int src = (r + p - 1) % p;
                w.in[r] = (mode == PIPESGD_NONE && step == 0) ? static_cast<const void *>(ra.g[src]) : ra.out[src];
                w.in_sc[r] = ra.out_sc[src];
                w.out[r] = recv[r];
                w.out_sc[r] = recv_scales[r];
            }
            if (!wait(ws_, ready[g])) return PIPESGD_ERR_HIP;
            rc = link_delay(count, ws_);              // the payload is under way for this long, then it lands
            if (rc == PIPESGD_OK) rc = copy_impl(mode, w, bt, count, step + 1, static_cast<uint32_t>(wire_workgroups), ws_);
            if (rc != PIPESGD_OK) return rc;
            hipEvent_t copied;
            if (!record(ws_, &copied) || !wait(cs, copied)) return PIPESGD_ERR_HIP;
            // stage 2, (decompress, sum, compress) on what has arrived
            RingArgs h = ra;
            h.slot_base = static_cast<uint32_t>(seg_lo(g));
            for (int r = 0; r < p; ++r) {
                h.in[r] = recv[r];
                h.in_sc[r] = recv_scales[r];
            }
            rc = rs_impl(mode, h, bt, count, step, true, cs);
            if (rc != PIPESGD_OK) return rc;
            if (!record(cs, &ready[g])) return PIPESGD_ERR_HIP;
        }
    }
    // send-back rounds: communication only, on the wire stream, after the last reductions
    hipEvent_t reduced_all;
    if (!record(cs, &reduced_all) || !wait(ws_, reduced_all)) return PIPESGD_ERR_HIP;
    for (int step = 0; step <= p - 2; ++step) {
        rc = link_delay(slots, ws_);
        if (rc == PIPESGD_OK) rc = copy_impl(mode, ra, bt, slots, step, static_cast<uint32_t>(wire_workgroups), ws_);
        if (rc != PIPESGD_OK) return rc;
    }
    hipEvent_t done;
    if (!record(ws_, &done) || !wait(cs, done)) return PIPESGD_ERR_HIP;
    return PIPESGD_OK;
}

static int prepare_update(int mode, int replicas, const void *const *g_sum_c, const float *const *scales, uint64_t n,
                          float *const *w, float *const *v, float lr, float momentum, float grad_scale, UpdateArgs &ua)
{
    if (!mode_ok(mode)) return PIPESGD_ERR_MODE;
    if (replicas < 1) return PIPESGD_ERR_ARG;
    if (replicas > kMaxW) return PIPESGD_ERR_CAPACITY;
    if (!g_sum_c || !w) return PIPESGD_ERR_ARG;
    const bool mom = momentum != 0.0f;
    if (mom && !v) return PIPESGD_ERR_ARG;
    if (mode == PIPESGD_QUANT8 && !scales) return PIPESGD_ERR_ARG;
    for (int r = 0; r < kMaxW; ++r) { ua.pay[r] = nullptr; ua.sc[r] = nullptr; ua.w[r] = nullptr; ua.v[r] = nullptr; }
    for (int r = 0; r < replicas && n > 0; ++r) {
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
    return PIPESGD_OK;
}

int pipesgd_apply_update_multi(int mode, int replicas, const void *const *g_sum_c,
                               const float *const *scales, uint64_t n, float *const *w,
                               float *const *v, float lr, float momentum, float grad_scale,
                               void *stream)
{
    UpdateArgs ua;
    const int rc = prepare_update(mode, replicas, g_sum_c, scales, n, w, v, lr, momentum, grad_scale, ua);
    if (rc != PIPESGD_OK) return rc;
    if (n == 0) return PIPESGD_OK;
    const bool mom = momentum != 0.0f;
    const LaunchConfig c = cfg_of(kUpdate, mode);
    hipStream_t s = static_cast<hipStream_t>(stream);
#define CALL(M) return mom ? launch_update<M, true>(c, ua, replicas, s) : launch_update<M, false>(c, ua, replicas, s);
    PIPESGD_MODE_SWITCH(mode, CALL)
#undef CALL
    return PIPESGD_ERR_MODE;
}

int pipesgd_probe_stream(int kind, int mode, int replicas, const void *const *g_sum_c, float *const *w, float *const *v,
                         uint64_t n, int threads, int quads, int lds_bytes, void *stream)
{
    if (kind < kProbeRead || kind > kProbeCopy) return PIPESGD_ERR_ARG;
    if (mode != PIPESGD_TRUNC16 && mode != PIPESGD_QUANT8 && mode != PIPESGD_NONE) return PIPESGD_ERR_MODE;
    const LaunchConfig c = {threads, quads, lds_bytes};
    if (!config_ok(kUpdate, mode, c)) return PIPESGD_ERR_ARG;
    UpdateArgs ua;
    // the same checks as the update's (momentum form: v is needed); the probes never read scales
    alignas(16) static const float no_scale[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    const float *sc[kMaxW];
    for (int r = 0; r < kMaxW; ++r) sc[r] = no_scale;
    const int rc = prepare_update(mode, replicas, g_sum_c, sc, n, w, v, 0.0f, 0.5f, 1.0f, ua);
    if (rc != PIPESGD_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
#define CALL(M)                                                                            \
    switch (kind) {                                                                        \
    case kProbeRead:  return launch_probe<M, kProbeRead>(c, ua, replicas, s);              \
    case kProbeWrite: return launch_probe<M, kProbeWrite>(c, ua, replicas, s);             \
    case kProbeMixed: return launch_probe<M, kProbeMixed>(c, ua, replicas, s);             \
    default:          return launch_probe<M, kProbeCopy>(c, ua, replicas, s);              \
    }
    PIPESGD_MODE_SWITCH(mode, CALL)
#undef CALL
    return PIPESGD_ERR_MODE;
}

int pipesgd_iteration_fused(const pipesgd_ring *ring, const void *const *stale_g_sum_c,
                            const float *const *stale_scales, float *const *w, float *const *v,
                            float lr, float momentum, float grad_scale, void *stream)
{
    RingArgs ra; BucketTable bt; uint64_t slots = 0;
    int rc = prepare_ring(ring, ra, bt, slots);
    if (rc != PIPESGD_OK) return rc;
    UpdateArgs ua;
    rc = prepare_update(ring->mode, ring->workers, stale_g_sum_c, stale_scales, ring->n, w, v, lr, momentum, grad_scale, ua);
    if (rc != PIPESGD_OK) return rc;
    if (ring->n == 0) return PIPESGD_OK;
    for (int r = 0; r < ring->workers; ++r)                 // the two halves must not touch the same slot set
        for (int q = 0; q < ring->workers; ++q)
            if (stale_g_sum_c[r] == ring->g_sum_c[q]) return PIPESGD_ERR_ARG;
    const uint64_t upd_units = (ring->n + kTile - 1) / kTile;
    if (slots + upd_units > 0x7fffffffull) return PIPESGD_ERR_CAPACITY;
    const dim3 grid(static_cast<uint32_t>(slots + upd_units), ring->workers);
    const uint32_t ring_blocks = static_cast<uint32_t>(slots);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool mom = momentum != 0.0f;
#define CALL(M)                                                                                                        \
    if (mom) hipLaunchKernelGGL((iteration_fused_kernel<M, true>), grid, dim3(256), 0, s, ra, bt, ua, ring_blocks);    \
    else     hipLaunchKernelGGL((iteration_fused_kernel<M, false>), grid, dim3(256), 0, s, ra, bt, ua, ring_blocks);
    PIPESGD_MODE_SWITCH(ring->mode, CALL)
#undef CALL
    return hipGetLastError() == hipSuccess ? PIPESGD_OK : PIPESGD_ERR_HIP;
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
    // 36 KiB of (unused) LDS per workgroup admits four workgroups of one 16 KiB tile each per compute unit:
    // as for the other streaming kernels, fewer requests in flight than full occupancy issues run faster
    // (gather of 161 tensors x 4 workers, 818 MB moved: 5.5 TB/s against 5.1 TB/s without the cap)
    constexpr int kPackLds = 36 * 1024;
    if (to_packed) hipLaunchKernelGGL((segment_copy_kernel<true>), grid, dim3(256), kPackLds, s, segments, static_cast<uint32_t>(num));
    else           hipLaunchKernelGGL((segment_copy_kernel<false>), grid, dim3(256), kPackLds, s, segments, static_cast<uint32_t>(num));
    return hipGetLastError() == hipSuccess ? PIPESGD_OK : PIPESGD_ERR_HIP;
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

int pipesgd_internal_check_allreduce(const pipesgd_ring *ring, int schedule)
{
    RingArgs ra; BucketTable bt; uint64_t slots = 0;
    const int rc = prepare_ring(ring, ra, bt, slots);
    if (rc != PIPESGD_OK) return rc;
    return (schedule == PIPESGD_STEPWISE || schedule == PIPESGD_FUSED) ? PIPESGD_OK : PIPESGD_ERR_MODE;
}

int pipesgd_internal_check_update(int mode, int replicas, const void *const *g_sum_c, const float *const *scales,
                                  uint64_t n, float *const *w, float *const *v, float momentum)
{
    UpdateArgs ua;
    int rc = prepare_update(mode, replicas, g_sum_c, scales, n, w, v, 0.0f, momentum, 1.0f, ua);
    if (rc == PIPESGD_OK && (n + 1023) / 1024 > 0x7fffffffull) rc = PIPESGD_ERR_CAPACITY;   // more units than a grid holds
    return rc;
}

