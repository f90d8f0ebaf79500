// Host-only parts of libpipesgd: size rules, the bucket planner, error text.
// No device code and no HIP calls in this file.
#include "pipesgd.h"

namespace {
constexpr uint64_t kTile = PIPESGD_QBLOCK;
inline uint64_t round_up_tile(uint64_t x) { return (x + kTile - 1) / kTile * kTile; }
}  // namespace

extern "C" {

const char *pipesgd_strerror(int err)
{
    switch (err) {
    case PIPESGD_OK:           return "ok";
    case PIPESGD_ERR_ARG:      return "invalid argument (null pointer, or a count/index out of range)";
    case PIPESGD_ERR_ALIGN:    return "device pointer not 16-byte aligned, or bucket start not a multiple of 4096";
    case PIPESGD_ERR_MODE:     return "unknown compression mode or schedule";
    case PIPESGD_ERR_CAPACITY: return "too many workers, buckets or sub-blocks, or an output table or workspace buffer too small";
    case PIPESGD_ERR_HIP:      return "HIP runtime error at kernel launch";
    default:                   return "unknown pipesgd error";
    }
}

int pipesgd_version(void) { return PIPESGD_VERSION; }

// n/p of Eq. 5, rounded to whole quantisation blocks.
uint64_t pipesgd_chunk_elems(uint64_t n, int workers)
{
    if (workers < 1) return 0;
    const uint64_t p = static_cast<uint64_t>(workers);
    return round_up_tile((n + p - 1) / p);
}

uint64_t pipesgd_payload_bytes(int mode, uint64_t n)
{
    switch (mode) {
    case PIPESGD_NONE:    return 4 * n;
    case PIPESGD_TRUNC16: return 2 * n;     // the 2x of Sec. 4
    case PIPESGD_QUANT8:  return n;         // the 4x of Sec. 4 (plus one scale per block)
    default:              return 0;
    }
}

uint64_t pipesgd_num_scales(int mode, uint64_t n)
{
    return mode == PIPESGD_QUANT8 ? (n + kTile - 1) / kTile : 0;
}

uint64_t pipesgd_placement_offset(int kind, int worker, int workers)
{
    if (kind < PIPESGD_BUF_GRADIENT || kind > PIPESGD_BUF_PARTIAL || worker < 0 || workers < 1 || worker >= workers)
        return 0;
    // Ring neighbours must differ: colour the cycle of workers with two colours, and the
    // last worker of an odd ring with a third.
    const int colour = (workers > 1 && workers % 2 == 1 && worker == workers - 1) ? 2 : worker % 2;
    // Three positions per kind; kinds that one workgroup touches together get different
    // triples: gradient | slot | slot of the neighbour, and slot | w | v.  The staging
    // buffers of the other schedules reuse the triples of w and v, which no AllReduce
    // kernel touches; the tiny scale arrays share the last position.
    static const int base[10] = {0, 3, 6, 9, 12, 15, 15, 3, 15, 6};
    const int pos = base[kind] == 15 ? 15 : base[kind] + colour;
    return 256ull * static_cast<uint64_t>(pos);
}

int pipesgd_workspace_bytes(int schedule, int mode, uint64_t n, int workers, uint64_t bytes[3])
{
    if (mode != PIPESGD_NONE && mode != PIPESGD_TRUNC16 && mode != PIPESGD_QUANT8) return PIPESGD_ERR_MODE;
    if (schedule < PIPESGD_WS_RING || schedule > PIPESGD_WS_HALVING_DOUBLING) return PIPESGD_ERR_MODE;
    if (workers < 1 || !bytes) return PIPESGD_ERR_ARG;
    bytes[0] = bytes[1] = bytes[2] = 0;
    if (schedule == PIPESGD_WS_RING || workers == 1) return PIPESGD_OK;
    bytes[0] = pipesgd_payload_bytes(mode, n);
    bytes[1] = 4 * pipesgd_num_scales(mode, n);
    if (schedule == PIPESGD_WS_HALVING_DOUBLING && workers > 2) bytes[2] = 4 * n;
    return PIPESGD_OK;
}

int pipesgd_bucket_plan(const uint64_t *numels, uint64_t num_tensors, uint64_t bucket_elems,
                        pipesgd_bucket *buckets, uint64_t max_buckets,
                        uint64_t *tensor_offsets, uint64_t *n_packed)
{
    if ((!numels && num_tensors) || !buckets || !tensor_offsets || !n_packed || bucket_elems == 0)
        return PIPESGD_ERR_ARG;
    uint64_t nb = 0, start = 0, fill = 0;
    auto close_bucket = [&]() -> bool {
        if (nb >= max_buckets) return false;
        buckets[nb].start = start;
        buckets[nb].n = fill;
        ++nb;
        start = round_up_tile(start + fill);
        fill = 0;
        return true;
    };
    for (uint64_t i = 0; i < num_tensors; ++i) {
        if (fill > 0 && fill + numels[i] > bucket_elems) {
            if (!close_bucket()) return PIPESGD_ERR_CAPACITY;
        }
        tensor_offsets[i] = start + fill;
        fill += numels[i];
    }
    if (fill > 0 || nb == 0) {
        if (!close_bucket()) return PIPESGD_ERR_CAPACITY;
    }
    *n_packed = round_up_tile(buckets[nb - 1].start + buckets[nb - 1].n);
    if (nb > 0x7fffffffull) return PIPESGD_ERR_CAPACITY;
    return static_cast<int>(nb);
}

int pipesgd_segments_prepare(pipesgd_segment *segments, uint64_t num, uint64_t *total_tiles)
{
    if ((!segments && num) || !total_tiles) return PIPESGD_ERR_ARG;
    uint64_t tiles = 0;
    for (uint64_t i = 0; i < num; ++i) {
        if (segments[i].numel && (!segments[i].tensor || !segments[i].packed)) return PIPESGD_ERR_ARG;
        if ((reinterpret_cast<uintptr_t>(segments[i].tensor) | reinterpret_cast<uintptr_t>(segments[i].packed)) & 3)
            return PIPESGD_ERR_ALIGN;
        segments[i].first_tile = tiles;
        tiles += (segments[i].numel + kTile - 1) / kTile;
    }
    *total_tiles = tiles;
    return PIPESGD_OK;
}

// ---- the paper's timing models (Sec. 3.1 and 3.2): plain arithmetic ----

double pipesgd_model_sync_time(double T, double l_up, double l_comp, double l_comm)
{
    return T * (l_up + l_comp + l_comm);                                  // Eq. 2
}

double pipesgd_model_pipe_ideal_time(double T, double K, double l_up, double l_comp, double l_comm)
{
    return K > 0 ? T / K * (l_up + l_comp + l_comm) : 0.0;                // Eq. 3
}

double pipesgd_model_pipe_time(double T, double l_up, double l_comp, double l_comm)
{
    const double a = l_up + l_comp;
    return T * (a > l_comm ? a : l_comm);                                 // Eq. 4
}

double pipesgd_model_ring_comm_time(int p, double n_bytes, double alpha, double beta, double gamma,
                                    double S, int L)
{
    if (p < 1 || L < 1) return 0.0;
    const double f = static_cast<double>(p - 1) / p;
    // communication term of Eq. 5 (L = 1) / Eq. 6 (L segments)
    return 2.0 * (p - 1) * L * alpha + 2.0 * f * n_bytes * beta + f * n_bytes * gamma + L * S;
}

double pipesgd_model_scaling_efficiency(double l_up, double l_comp, double l_comm)
{
    const double a = l_up + l_comp;
    const double m = a > l_comm ? a : l_comm;
    return m > 0 ? a / m : 0.0;                                           // Eq. 7
}

}  // extern "C"
