/*
 * libpipesgd -- the gradient aggregation + update path of Pipe-SGD
 * (arXiv 1811.03619) for one AMD MI355X (gfx950), behind a C ABI.
 *
 * The p workers of the paper's cluster are simulated as p gradient buffers in
 * one GPU's memory: this library runs every worker's share of the ring
 * AllReduce (Sec. 3.1), the light lossy compression on every ring hop
 * (Sec. 3.2) and the pipelined SGD update (Algorithm 1), as HIP kernels.
 *
 * Conventions common to every entry point
 *   - Return value: 0 on success, a negative PIPESGD_ERR_* otherwise.  Nothing
 *     throws, aborts or logs.  Arguments are checked before the first launch:
 *     on any error other than PIPESGD_ERR_HIP nothing has been enqueued.
 *   - "DEVICE" pointers are HIP device memory owned by the caller; the library
 *     allocates no device memory at run time.  The only device memory of its
 *     own is the fixed array of PIPESGD_STATIC_SCRATCH_BYTES inside its code
 *     object, used by pipesgd_allreduce_direct_static alone.  The state it
 *     keeps on the host: the launch-geometry table (see "tuning"), that array's
 *     address per device, and what the opaque pipesgd_overlap and
 *     pipesgd_runtime objects hold (HIP events, two streams).  "HOST" pointers
 *     are ordinary host memory read during the call only.
 *   - Every DEVICE pointer must be 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work on it and return without synchronising.  Calls on
 *     one stream execute in order; calls that touch the same buffers from
 *     different streams must be ordered by the caller.
 *   - Inputs declared const are never written; gradients are never modified.
 *   - Inputs must be finite.  NaN or Inf in a quantised block is a caller
 *     error and is not detected.
 *
 * Layout
 *   A gradient is a flat fp32 vector of n elements.  It is split into p ring
 *   blocks ("chunks") of pipesgd_chunk_elems(n, p) elements (the last ones
 *   may be short or empty).  A compressed vector ("payload") uses the same
 *   element index space: element i of the payload encodes element i of the
 *   vector, so chunk c of a payload starts at element c * chunk_elems.
 *     PIPESGD_NONE     payload = float[n]
 *     PIPESGD_TRUNC16  payload = uint16_t[n]  (upper half of the fp32 pattern)
 *     PIPESGD_QUANT8   payload = int8_t[n] plus scales = float[ceil(n/4096)],
 *                      scales[b] belonging to elements [4096 b, 4096 b + 4096)
 *   With bucketing, several vectors ("buckets") live in one packed buffer, each
 *   starting at a multiple of 4096 elements; each bucket is ring-reduced as a
 *   vector of its own with its own p chunks.  Padding between buckets must be
 *   zero in the gradients and is never written in payloads.
 */
#ifndef PIPESGD_H
#define PIPESGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PIPESGD_VERSION      100      /* major*10000 + minor*100 + patch */
#define PIPESGD_MAX_WORKERS  16
#define PIPESGD_MAX_BUCKETS  64
#define PIPESGD_QBLOCK       4096     /* elements per quantisation block and per tile */

/* compression modes (Sec. 3.2; widths from the results part of Sec. 4:
 * truncation to 16 bits, there called T, and quantisation to 8 bits, Q) */
#define PIPESGD_NONE     0
#define PIPESGD_TRUNC16  1
#define PIPESGD_QUANT8   2

/* schedules of pipesgd_allreduce_sim */
#define PIPESGD_STEPWISE 0   /* one launch per ring round; every hop's payload is written to memory */
#define PIPESGD_FUSED    1   /* one launch; hop payloads stay in registers; same result bits */

#define PIPESGD_OK             0
#define PIPESGD_ERR_ARG       -1   /* null pointer, count or index out of range */
#define PIPESGD_ERR_ALIGN     -2   /* a DEVICE pointer is not 16-byte aligned, or a bucket start is not a multiple of 4096 */
#define PIPESGD_ERR_MODE      -3   /* unknown compression mode or schedule */
#define PIPESGD_ERR_CAPACITY  -4   /* more workers, buckets or sub-blocks than the library supports; an output
                                      table or a workspace buffer too small */
#define PIPESGD_ERR_HIP       -5   /* the HIP runtime refused the launch */

const char *pipesgd_strerror(int err);
int pipesgd_version(void);

/* ------------------------------------------------------------------ sizes -- */

/* Length of one ring block: ceil(n/p) rounded up to a multiple of 4096, so that
 * no quantisation block straddles two ring blocks (Sec. 3.1 splits the gradient
 * vector into one block per worker; n/p in Eq. 5).  0 if p < 1. */
uint64_t pipesgd_chunk_elems(uint64_t n, int workers);
/* Bytes of a payload of n elements, scales not included; 0 for a bad mode. */
uint64_t pipesgd_payload_bytes(int mode, uint64_t n);
/* Number of fp32 scales that go with a payload of n elements (0 unless QUANT8). */
uint64_t pipesgd_num_scales(int mode, uint64_t n);

/* ----------------------------------------------------------------- codecs -- */

/* Compress(g) of Algorithm 1 (compute thread, line 9) / Sec. 3.2.
 *   TRUNC16: keep sign, exponent and 7 leading mantissa bits (toward zero).
 *   QUANT8 : per block of 4096 elements counted from src[0]: scale = max|x|;
 *            inv = 127/scale (one fp32 division, saturated at FLT_MAX);
 *            q = clamp(rint(x*inv), -127, 127), ties to even; scale 0 -> q 0.
 *   NONE   : copy.
 * src: DEVICE float[n].  payload: DEVICE, pipesgd_payload_bytes(mode,n) bytes.
 * scales: DEVICE float[pipesgd_num_scales(mode,n)], ignored unless QUANT8.
 * n may be 0 (nothing is enqueued).  src and payload must not overlap. */
int pipesgd_compress(int mode, const float *src, uint64_t n, void *payload, float *scales, void *stream);

/* Decompress(g^c) of Algorithm 1 (compute thread, line 4) / Sec. 3.2.
 *   TRUNC16: the 16 kept bits followed by 16 zero bits.
 *   QUANT8 : x = (float)q * (scale/127)  (one division per block, one multiply per element).
 * dst: DEVICE float[n]. */
int pipesgd_decompress(int mode, const void *payload, const float *scales, uint64_t n, float *dst, void *stream);

/* ------------------------------------------------------------------- ring -- */

typedef struct pipesgd_bucket {
    uint64_t start;      /* first element in the packed buffer; multiple of 4096 */
    uint64_t n;          /* elements */
} pipesgd_bucket;

/* One AllReduce over p simulated workers (Alg. 1, communication thread line 4:
 * g^c_sum <- sum of g^c_local).  Plain data; the caller fills it. */
typedef struct pipesgd_ring {
    int32_t  workers;                 /* p, 1..PIPESGD_MAX_WORKERS */
    int32_t  mode;                    /* PIPESGD_NONE / TRUNC16 / QUANT8 */
    uint64_t n;                       /* elements of each worker's (packed) vector */
    uint32_t num_buckets;             /* 0: the whole vector is one bucket {0, n} */
    uint32_t reserved;                /* must be 0 */
    const pipesgd_bucket *buckets;    /* HOST, num_buckets entries, ascending, non-overlapping */
    const float *g_local[PIPESGD_MAX_WORKERS];  /* DEVICE float[n]: worker r's local gradient */
    void        *g_sum_c[PIPESGD_MAX_WORKERS];  /* DEVICE payload of n elements: worker r's result
                                                   slot; also holds the hop payloads worker r sends
                                                   while the AllReduce is in progress */
    float       *scales[PIPESGD_MAX_WORKERS];   /* DEVICE float[num_scales]; QUANT8 only */
} pipesgd_ring;

/* Ring convention (the paper's Fig. 2(c) fixes none): worker r sends to worker
 * (r+1) mod p.  Chunk c starts its sum on worker c:
 *     P_0 = g_c[c];   P_j = D(C(P_{j-1})) + g_{(c+j) mod p}[c],  j = 1..p-1,
 * the local operand always in full fp32 precision, one IEEE add per element.
 * After the p-1 transmit-and-reduce rounds worker r owns chunk (r+1) mod p. */

/* Worker r compresses the chunk it sends in round 0 (chunk r) into its slot:
 * g_sum_c[r][chunk r] = C(g_local[r][chunk r]), all r in one launch.
 * With PIPESGD_NONE and p > 1 nothing is enqueued (round 0 then reads the
 * sender's gradient itself); with p == 1 this produces the whole result. */
int pipesgd_ring_first_send(const pipesgd_ring *ring, void *stream);

/* Transmit-and-reduce round `step` (0 <= step <= p-2) for all p workers in one
 * launch (Sec. 3.1; with compression: decompress, sum, compress -- Sec. 3.2):
 * worker r reads chunk j = (r-step-1) mod p from worker (r-1)'s slot, adds its
 * own g_local chunk j and writes C(sum) to chunk j of its own slot.  After
 * round p-2 worker r's slot holds the final C(P_{p-1}) of chunk (r+1) mod p.
 * Rounds must be enqueued in order after pipesgd_ring_first_send. */
int pipesgd_ring_reduce_scatter_step(const pipesgd_ring *ring, int step, void *stream);

/* Send-back round `step` (0 <= step <= p-2) for all p workers in one launch
 * (Sec. 3.1: the reduced blocks are sent on round the ring): worker r copies
 * chunk (r-step) mod p, payload bytes and scales verbatim, from worker (r-1)'s
 * slot into its own.  After round p-2 all p slots hold identical bytes. */
int pipesgd_ring_allgather_step(const pipesgd_ring *ring, int step, void *stream);

/* The whole AllReduce: first_send, p-1 reduce-scatter rounds, p-1 all-gather
 * rounds.  PIPESGD_STEPWISE enqueues exactly those launches.  PIPESGD_FUSED
 * enqueues one kernel that walks each chunk's chain in registers and writes
 * only the final payload to all p slots: same bits in g_sum_c/scales, fewer
 * bytes moved, for launch-bound (small or many-bucket) gradients. */
int pipesgd_allreduce_sim(const pipesgd_ring *ring, int schedule, void *stream);

/* Scratch that a schedule needs PER WORKER beyond the gradients and the result
 * slots; the caller allocates it (the library allocates nothing) and passes it
 * in a pipesgd_workspace.  HOST arithmetic.
 *   bytes[0]  payload-sized staging (stage), = pipesgd_payload_bytes(mode, n)
 *   bytes[1]  its per-block scales (stage_scales), QUANT8 only
 *   bytes[2]  fp32 partial sums (partial), halving-doubling with more than two workers
 * all zero for the ring schedules of pipesgd_allreduce_sim and for one worker.
 * Returns PIPESGD_ERR_MODE for an unknown mode or schedule, PIPESGD_ERR_ARG for
 * workers < 1 or a NULL table. */
#define PIPESGD_WS_RING              0   /* pipesgd_allreduce_sim, both schedules, and pipesgd_iteration_fused */
#define PIPESGD_WS_PIPELINED         1   /* pipesgd_allreduce_pipelined */
#define PIPESGD_WS_DIRECT            2   /* pipesgd_allreduce_direct */
#define PIPESGD_WS_HALVING_DOUBLING  3   /* pipesgd_allreduce_halving_doubling */
int pipesgd_workspace_bytes(int schedule, int mode, uint64_t n, int workers, uint64_t bytes[3]);

/* The scratch itself, as the three schedules above take it.  Plain data, HOST
 * struct; the three tables are HOST arrays of ring->workers DEVICE pointers.
 * Each *_bytes field is the size of EVERY buffer in its table; an entry point
 * returns PIPESGD_ERR_CAPACITY when a size it needs is below what
 * pipesgd_workspace_bytes states for (its schedule, ring->mode, ring->n,
 * ring->workers), PIPESGD_ERR_ARG / PIPESGD_ERR_ALIGN for a missing or
 * misaligned buffer it needs.  Tables and sizes a schedule or mode does not need
 * are ignored (stage_scales unless QUANT8; partial unless halving-doubling with
 * p > 2).  Contents are scratch: undefined after the call, nothing expected
 * before it. */
typedef struct pipesgd_workspace {
    void  *const *stage;           /* payload staging: receive buffers (pipelined) / send buffers */
    float *const *stage_scales;
    float *const *partial;
    uint64_t stage_bytes;
    uint64_t stage_scales_bytes;
    uint64_t partial_bytes;
} pipesgd_workspace;

/* A second AllReduce schedule, the one-exchange ("direct") schedule -- what an
 * 8-GPU node with a direct link between every pair of GPUs would run instead
 * of a ring (Sec. 3.1 notes that its analysis carries over to other AllReduce
 * algorithms).  Worker j owns chunk j.  Exchange 1: every worker k compresses
 * chunk j of its gradient for every j != k (into ws->stage[k], its send buffer).
 * Owner j then computes  P = g_j[j];  P = P + D(stage[(j+d) mod p][j]) for
 * d = 1..p-1 in this order;  and, exchange 2, writes C(P) into all p result
 * slots.  Two launches, two exchanges instead of 2(p-1), the same volume on the
 * links, and every value passes the codec twice instead of p times (less loss
 * than the ring; with PIPESGD_NONE the result bits equal the ring's).
 * ws: stage (and stage_scales with QUANT8), sized as PIPESGD_WS_DIRECT says; may
 * be NULL for one worker or an empty vector.  Buckets are supported. */
int pipesgd_allreduce_direct(const pipesgd_ring *ring, const pipesgd_workspace *ws, void *stream);

/* pipesgd_allreduce_direct for callers that cannot allocate device memory and
 * have none to spare for the send buffers: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  The send buffers live in a
 * device array of PIPESGD_STATIC_SCRATCH_BYTES bytes that is part of the
 * library's code object (each GPU the library runs on holds its own copy until
 * the process ends); the call allocates and frees nothing.  Same kernels and
 * same result bits as pipesgd_allreduce_direct.
 * The vector must fit:  p * (roundup256(pipesgd_payload_bytes(mode, n)) +
 * roundup256(4 * pipesgd_num_scales(mode, n))) <= PIPESGD_STATIC_SCRATCH_BYTES,
 * otherwise PIPESGD_ERR_CAPACITY (checked on the host before anything else).
 * Every call on one GPU uses that GPU's one array: calls that may overlap on a
 * GPU (different streams, different threads) race and must be ordered by the
 * caller.  Nothing in the array has to be zero on entry -- every cell that is
 * read was written earlier in the same call -- so it is never cleared and keeps
 * the previous call's contents.  The first call on a device looks the array's
 * address up (a query, no allocation); make that call outside graph capture. */
#define PIPESGD_STATIC_SCRATCH_BYTES  (32u << 20)
int pipesgd_allreduce_direct_static(const pipesgd_ring *ring, void *stream);

/* A third AllReduce schedule: recursive halving and doubling, one of the
 * algorithms Sec. 3.1's closing remark names beside the ring (reduce-scatter by
 * recursive halving, all-gather by recursive doubling, as published by Thakur,
 * Rabenseifner and Gropp, 2005).  ring->workers must be a power of two
 * (otherwise PIPESGD_ERR_ARG).  Chunks and codecs are the ring's.
 *   halving round with distance h = p/2, p/4, .., 1: worker r and partner r^h
 *   hold partial sums over the same 2h chunks; r keeps the h chunks whose index
 *   agrees with r in bit h, sends the other h compressed (into stage[r]) and
 *   computes  P = own + D(stage[r^h])  on the ones it keeps, own = the local
 *   gradient in the first round and the fp32 partial sum afterwards.  After the
 *   last round worker r holds chunk r and writes C(P) into its result slot.
 *   doubling round with distance d = 1, 2, .., p/2: r copies, byte for byte,
 *   the d chunks r^d holds.
 * For p = 4, chunk c:  P = (g_c + D(C(g_{c^2}))) + D(C(g_{c^1} + D(C(g_{c^3})))):
 * a codec chain of depth log2(p) (the ring's is p-1) and 2 log2(p) rounds.
 * 1 + log2(p) + log2(p) launches (one less without compression): a halving
 * round also compresses, in the same pass, the part of its sums that is sent
 * in the next round.
 * ws: stage = the p send buffers (stage_scales with QUANT8), partial = the fp32
 * partial sums (needed when p > 2), sized as PIPESGD_WS_HALVING_DOUBLING says.
 * Buckets are supported. */
int pipesgd_allreduce_halving_doubling(const pipesgd_ring *ring, const pipesgd_workspace *ws, void *stream);

/* Placement advice, HOST arithmetic.  MI355X interleaves its HBM channels within
 * 4 KiB; allocators hand out large buffers at multiples of 2 MiB, so the streams
 * that one workgroup reads and writes together (a worker's gradient, its slot and
 * its neighbour's slot; or slot, w and v of a replica) would all sit at the same
 * offset within that interleave and queue on one channel at a time.  Returns the
 * byte offset (a multiple of 256, below 4096) at which buffer `kind` of worker
 * `worker` (of `workers`) should start within a 4 KiB-aligned allocation so that
 * they do not (0 for arguments out of range):
 * measured, 2-2.5 % on the update kernel at 61M and 138M elements and 8 % on
 * power-of-two lengths.  Purely advisory: every entry point accepts any 16-byte
 * aligned pointer and results never depend on placement. */
#define PIPESGD_BUF_GRADIENT  0
#define PIPESGD_BUF_W         1
#define PIPESGD_BUF_V         2
#define PIPESGD_BUF_SLOT_A    3   /* result slots of even / odd iterations */
#define PIPESGD_BUF_SLOT_B    4
#define PIPESGD_BUF_SCALES_A  5
#define PIPESGD_BUF_SCALES_B  6
#define PIPESGD_BUF_STAGE     7   /* recv / stage */
#define PIPESGD_BUF_STAGE_SC  8
#define PIPESGD_BUF_PARTIAL   9
uint64_t pipesgd_placement_offset(int kind, int worker, int workers);


/* ---------------------------------------- pipelining within the AllReduce -- */

/* Host-side resources (HIP events) of the two-stream schedule below.  No device
 * memory.  Not thread-safe; one per concurrently used ring. */
typedef struct pipesgd_overlap pipesgd_overlap;
int  pipesgd_overlap_create(pipesgd_overlap **out);
void pipesgd_overlap_destroy(pipesgd_overlap *ov);

/* The AllReduce as a two-stage pipeline over `segments` sub-blocks of every
 * ring block (Sec. 3.2's pipelining inside the AllReduce, Fig. 3(b)): stage 1,
 * the compressed communication, copies a sub-block of the sender's payload into
 * the receiver's staging buffer recv[r] on `wire_stream`; stage 2, (decompress,
 * sum, compress), runs on `compute_stream` on what has arrived, while the next
 * sub-block is in transit.  The send-back rounds are communication only.
 * Same result bits as pipesgd_allreduce_sim.  Unlike the plain schedules, where
 * a receiver reads the sender's buffer in place, every hop payload here is
 * moved once more (the stand-in for the wire), so this costs bandwidth on one
 * GPU; it exists to measure how much of the codec time the transfer hides.
 * ws: stage = the p receive buffers recv[r] (stage_scales with QUANT8), sized
 * as PIPESGD_WS_PIPELINED says.  1 <= segments <= PIPESGD_MAX_SEGMENTS
 * (PIPESGD_ERR_CAPACITY above).
 * Buckets are supported (a sub-block is a range of the ring block's tiles, counted
 * across buckets).  On return both streams hold work; compute_stream
 * is made to wait for the end of it, and wire_stream for everything enqueued on
 * compute_stream before the call.  wire_stream may equal compute_stream (no
 * overlap: the sequential baseline).
 * wire_workgroups: 0 = every transfer runs at full memory speed.  k > 0 = each
 * worker's transfers are carried by only k workgroups that walk the sub-block:
 * a link of limited bandwidth that leaves the rest of the GPU to stage 2, which
 * is the situation of the paper (the network is slower than the reduction).
 * link_us_per_mib: 0 = none.  x > 0 = before every transfer lands in the staging
 * buffer the wire stream idles for x microseconds per MiB that one worker sends
 * in it (one wavefront, no memory traffic): the time the bytes spend on a network
 * of 1/x MiB/us -- Eq. 5's beta -- which, unlike a copy inside one HBM, competes
 * with nothing, so stage 2 of the previous sub-block runs beside it.  The delay
 * of one whole ring block may not pass one second (PIPESGD_ERR_ARG). */
#define PIPESGD_MAX_SEGMENTS 64
int pipesgd_allreduce_pipelined(const pipesgd_ring *ring, const pipesgd_workspace *ws,
                                int segments, int wire_workgroups, float link_us_per_mib, pipesgd_overlap *ov,
                                void *compute_stream, void *wire_stream);

/* ----------------------------------------------------------------- update -- */

/* Algorithm 1, compute thread lines 4-5, on one model replica:
 *     g = D(g_sum_c);  if grad_scale != 1: g = g * grad_scale;
 *     momentum != 0:  v = fma(momentum, v, g);  w = fma(-lr, v, w)
 *     momentum == 0:  w = fma(-lr, g, w)                (v may be NULL, untouched)
 * The pipelined method (width 2, staleness 1 -- Sec. 3.1) passes the result
 * slot of the PREVIOUS iteration's AllReduce; an all-zero slot (the initial
 * state of Alg. 1, communication thread line 1) leaves w unchanged.  Passing
 * the current iteration's slot gives decentralised synchronous SGD.
 * g_sum_c / scales: DEVICE payload of n elements.  w, v: DEVICE float[n]. */
int pipesgd_apply_update(int mode, const void *g_sum_c, const float *scales, uint64_t n,
                         float *w, float *v, float lr, float momentum, float grad_scale,
                         void *stream);

/* The same update on `replicas` model replicas (one per simulated worker) in a
 * single launch.  The four arrays are HOST arrays of DEVICE pointers;
 * v may be NULL iff momentum == 0. */
int pipesgd_apply_update_multi(int mode, int replicas, const void *const *g_sum_c,
                               const float *const *scales, uint64_t n, float *const *w,
                               float *const *v, float lr, float momentum, float grad_scale,
                               void *stream);

/* One whole width-2 iteration in a single launch: the AllReduce of ring->g_local
 * into ring->g_sum_c (fused schedule) together with the update of all
 * ring->workers replicas from the PREVIOUS iteration's slot set `stale_*`.  The
 * two halves touch disjoint buffers (the independence the paper's pipeline rests
 * on), so they share one grid.  For gradients so small that launch latency sets
 * the pace (a few MB, or many small buckets).  Same result bits as
 * pipesgd_allreduce_sim + pipesgd_apply_update_multi.  `stale_*`, w, v: HOST
 * arrays of ring->workers DEVICE pointers; the stale slot set must not be the
 * one the ring writes (PIPESGD_ERR_ARG). */
int pipesgd_iteration_fused(const pipesgd_ring *ring, const void *const *stale_g_sum_c,
                            const float *const *stale_scales, float *const *w, float *const *v,
                            float lr, float momentum, float grad_scale, void *stream);

/* -------------------------------------------------------------- bucketing -- */

/* Small-tensor fusion (not in the paper, which sends the gradient as one
 * segment -- L = 1 in Eq. 6): tensors in declaration order are packed greedily;
 * a bucket is closed when the next tensor would take it past bucket_elems; a
 * larger tensor gets a bucket of its own; every bucket starts at a multiple of
 * 4096 elements.  All arguments HOST.  Writes tensor_offsets[num_tensors]
 * (packed-buffer element offset of each tensor), up to max_buckets buckets and
 * *n_packed (packed length, multiple of 4096).  Returns the number of buckets,
 * or PIPESGD_ERR_CAPACITY if max_buckets is too small (nothing useful written). */
int pipesgd_bucket_plan(const uint64_t *numels, uint64_t num_tensors, uint64_t bucket_elems,
                        pipesgd_bucket *buckets, uint64_t max_buckets,
                        uint64_t *tensor_offsets, uint64_t *n_packed);

/* One tensor <-> packed-buffer copy.  32 bytes. */
typedef struct pipesgd_segment {
    float   *tensor;      /* DEVICE float[numel], 4-byte aligned is enough */
    float   *packed;      /* DEVICE: where the tensor lives in a packed buffer */
    uint64_t numel;
    uint64_t first_tile;  /* filled by pipesgd_segments_prepare */
} pipesgd_segment;

/* HOST: fills first_tile of each of the num segments (prefix sum of
 * ceil(numel/4096)) and returns the total tile count in *total_tiles.  The
 * caller then copies the table to the device. */
int pipesgd_segments_prepare(pipesgd_segment *segments, uint64_t num, uint64_t *total_tiles);

/* Gather (tensor -> packed) / scatter (packed -> tensor) all segments in one
 * launch.  segments: DEVICE table of num entries prepared as above. */
int pipesgd_pack(const pipesgd_segment *segments, uint64_t num, uint64_t total_tiles, void *stream);
int pipesgd_unpack(const pipesgd_segment *segments, uint64_t num, uint64_t total_tiles, void *stream);

/* ------------------------------------------------- Algorithm 1's two threads -- */

/* The per-worker runtime of Algorithm 1 for the p simulated workers at once:
 * the computation thread and the communication thread are two HIP streams of
 * default priority that the runtime owns, the "ready" marks are HIP events.
 * Indexing as elsewhere in this library: g[t] is the gradient evaluated at
 * w[t-1], A[t] = AllReduce(g[t]), w[t] = Update(w[t-1], A[t-1]) (Algorithm 1
 * counts the same steps one iteration later).  Iteration t enqueues
 *   comm stream:    wait "g[t] ready"; AllReduce (comm thread line 4); mark A[t] ready;
 *   compute stream: wait "A[t-1] ready"; decompress + update all replicas -> w[t]
 *                   (compute thread lines 3-5); the stand-in for batch / forward /
 *                   backward that yields g[t+1] (lines 6-8); mark it ready (line 10).
 * So the AllReduce of g[t] overlaps the update and the gradient computation that
 * follow it, and the time per iteration follows max(l_up + l_comp, l_comm)
 * (Eq. 4) as far as the two streams do not compete for the same resource.
 * width 1 is decentralised synchronous SGD: compute g[t], AllReduce, update with
 * A[t], one after the other (Eq. 2: l_up + l_comp + l_comm).
 * width K in 3..7 is Algorithm 1 with iteration dependency K: the update of
 * iteration t waits for and applies A[t-(K-1)] (Eq. 3's regime; the paper finds
 * K = 2 optimal).
 * The caller keeps K slot sets (two for width 1 and 2) and rotates them: `ring`
 * writes the slot set of iteration t, `stale_*` name the slot set of iteration
 * t-(K-1) (an all-zero set while t < K), `fresh_*` the set `ring` writes (width
 * 1 only).  With width >= 2 the stale set must not be the set `ring` writes
 * (PIPESGD_ERR_ARG): the two streams would race on it.
 * The caller must not change g_local while an AllReduce that reads it may still
 * be running (pipesgd_runtime_sync, or double-buffer the gradients).
 * pipesgd_runtime_iteration checks every field (the ring, the slot / w / v tables
 * of the update it will launch, both durations) before its first launch or event
 * record: after an error other than PIPESGD_ERR_HIP the runtime is as it was and
 * the same iteration can be issued again. */
typedef struct pipesgd_runtime pipesgd_runtime;

#define PIPESGD_RT_TIME_UPDATE 1

typedef struct pipesgd_runtime_iter {
    const pipesgd_ring *ring;            /* AllReduce of this iteration (HOST struct) */
    int32_t  schedule;                   /* PIPESGD_STEPWISE / PIPESGD_FUSED */
    int32_t  width;                      /* 2 = pipelined (staleness 1), 1 = synchronous, 3..7 = staleness width-1 */
    int32_t  replicas;                   /* model replicas to update (normally ring->workers) */
    int32_t  compute_workgroups;         /* workgroups the compute stand-in occupies (1..65535; below 1 is taken as 1) */
    float    compute_us;                 /* duration of the compute stand-in, microseconds (0 = none) */
    float    wire_us;                    /* extra delay on the comm stream after the AllReduce kernels: the time
                                            the payloads would spend on a network (Eq. 5's alpha and beta terms);
                                            it occupies one wavefront and no memory bandwidth (0 = none) */
    float    lr, momentum, grad_scale;
    int32_t  flags;                      /* 0, or PIPESGD_RT_TIME_UPDATE: bracket this iteration's update launch with
                                            timing events on the compute stream (see pipesgd_runtime_update_time) */
    const void  *const *stale_g_sum_c;   /* HOST arrays of DEVICE pointers, as for pipesgd_apply_update_multi */
    const float *const *stale_scales;
    const void  *const *fresh_g_sum_c;   /* width 1 only */
    const float *const *fresh_scales;
    float *const *w;
    float *const *v;
} pipesgd_runtime_iter;

int   pipesgd_runtime_create(pipesgd_runtime **out);
void  pipesgd_runtime_destroy(pipesgd_runtime *rt);       /* synchronises both streams first */
int   pipesgd_runtime_iteration(pipesgd_runtime *rt, const pipesgd_runtime_iter *it);
int   pipesgd_runtime_sync(pipesgd_runtime *rt);          /* host waits for both streams */
/* Waits for the compute stream, then returns the summed duration (milliseconds,
 * HIP events on the compute stream) and the number of the update launches that
 * were timed (PIPESGD_RT_TIME_UPDATE) since the previous call, and starts anew.
 * While the AllReduce runs beside it on the other stream an update takes longer
 * than alone: both draw on the same memory bandwidth.  At most 65536 timed
 * launches are kept between two read-outs; a further timed iteration is refused
 * with PIPESGD_ERR_CAPACITY (nothing enqueued). */
int   pipesgd_runtime_update_time(pipesgd_runtime *rt, double *total_ms, uint64_t *launches);
void *pipesgd_runtime_stream(pipesgd_runtime *rt, int which);   /* 0 = compute, 1 = comm: a hipStream_t */

/* The stand-in for forward + backward: `workgroups` workgroups of 64 threads
 * that do nothing for duration_us microseconds (0..1e6) and touch no memory. */
int pipesgd_synthetic_compute(float duration_us, int workgroups, void *stream);

/* ------------------------------------------------------------ timing models -- */

/* The paper's wall-clock models, HOST arithmetic only; times in any one unit.
 *   Eq. 2  synchronous:        T (l_up + l_comp + l_comm)
 *   Eq. 3  ideal pipeline:     T/K (l_up + l_comp + l_comm)
 *   Eq. 4  resource bound:     T max(l_up + l_comp, l_comm)     (any K >= 2)
 *   Eq. 5/6 ring AllReduce:    2(p-1) L alpha + 2((p-1)/p) n beta + ((p-1)/p) n gamma + L S
 *           (alpha latency per round, beta transfer time per byte, gamma reduction
 *            time per byte, S synchronisation, L gradient segments; L = 1 is Eq. 5)
 *   Eq. 7  scaling efficiency: (l_up + l_comp) / max(l_up + l_comp, l_comm)          */
double pipesgd_model_sync_time(double T, double l_up, double l_comp, double l_comm);
double pipesgd_model_pipe_ideal_time(double T, double K, double l_up, double l_comp, double l_comm);
double pipesgd_model_pipe_time(double T, double l_up, double l_comp, double l_comm);
double pipesgd_model_ring_comm_time(int p, double n_bytes, double alpha, double beta, double gamma,
                                    double S, int L);
double pipesgd_model_scaling_efficiency(double l_up, double l_comp, double l_comm);

/* ----------------------------------------------------------------- tuning -- */

/* Launch geometry of one kernel family for one compression mode.  Optional:
 * the built-in defaults are the measured best on MI355X for 60M-element
 * gradients.  A workgroup has `threads` threads, each handling `quads` groups of
 * 4 consecutive elements (for the all-gather copy: `quads` 16-byte vectors);
 * `lds_bytes` of LDS are reserved per workgroup for no other purpose than to cap
 * how many workgroups a compute unit holds at once (0 = no cap): HBM delivers
 * its best rate with fewer requests in flight than full occupancy issues.
 * Supported (threads, quads): (64,4) (128,2) (128,4) (256,1) (256,2) (256,4)
 * (512,1) (512,2) (1024,1); QUANT8 kernels that compute a block's range need
 * threads*quads == 1024; the all-gather copy needs threads*quads*16 bytes to
 * divide a tile's payload.  0 <= lds_bytes <= 162816 (159 KiB).
 * The table is process-global; each entry is read and written as one atomic
 * word, so a launch concurrent with a change uses the old or the new geometry.
 * Returns PIPESGD_ERR_ARG for an unsupported combination (the table is left
 * unchanged).  Results never depend on it. */
#define PIPESGD_K_FIRST_SEND      0
#define PIPESGD_K_REDUCE_SCATTER  1
#define PIPESGD_K_ALLGATHER       2
#define PIPESGD_K_FUSED           3
#define PIPESGD_K_UPDATE          4
#define PIPESGD_K_COMPRESS        5
#define PIPESGD_K_DECOMPRESS      6
#define PIPESGD_K_DIRECT_REDUCE   7   /* owner-side kernel of pipesgd_allreduce_direct(_static) */
int pipesgd_set_launch_config(int kernel, int mode, int threads, int quads, int lds_bytes);
int pipesgd_get_launch_config(int kernel, int mode, int *threads, int *quads, int *lds_bytes);

/* ------------------------------------------------------------ measurement -- */

/* Not part of the method: the update's memory streams with the arithmetic taken
 * out, to find what the memory system sustains for that access mix (the ceiling
 * the update kernel is measured against).  Runs over the update's own buffers
 * and grid (replicas x whole units of n; a ragged tail is left out), with the
 * update's cache policy, in the given launch geometry (see "tuning").
 *   PIPESGD_PROBE_READ   loads slot, w and v; stores nothing
 *   PIPESGD_PROBE_WRITE  stores finite bit patterns into w and v; loads nothing
 *   PIPESGD_PROBE_MIXED  loads slot, w and v; stores v's values into w and w's
 *                        into v: the update's bytes (TRUNC16: 10 read, 8 written
 *                        per element) without decode or multiply-adds
 *   PIPESGD_PROBE_COPY   loads w, stores it into v (the usual 1 : 1 copy figure)
 * Arguments as for pipesgd_apply_update_multi (v is always needed).  WRITE, MIXED
 * and COPY overwrite w and/or v. */
#define PIPESGD_PROBE_READ   0
#define PIPESGD_PROBE_WRITE  1
#define PIPESGD_PROBE_MIXED  2
#define PIPESGD_PROBE_COPY   3
int pipesgd_probe_stream(int kind, int mode, int replicas, const void *const *g_sum_c, float *const *w,
                         float *const *v, uint64_t n, int threads, int quads, int lds_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PIPESGD_H */
