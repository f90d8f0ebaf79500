// Parity of libpipesgd against the CPU oracle with nothing but the HIP runtime in
// between: the program allocates device memory itself, calls the library through
// its C ABI (include/pipesgd.h) and compares every output byte with the oracle's.
// TEST CODE: it links the oracle, which the product never does.
//
// What is compared (arXiv 1811.03619): the ring AllReduce with the compression of
// Sec. 3.2 on every hop (Sec. 3.1), in its stepwise, fused, one-exchange and
// halving-doubling schedules, and the decompress + momentum step of Algorithm 1
// (compute thread lines 4-5) applied to the previous result (width 2).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "pipesgd.h"

extern "C" {   // oracle/pipesgd_oracle.c
size_t orc_payload_bytes(int mode, size_t n);
size_t orc_num_scales(int mode, size_t n);
void orc_allreduce(int mode, int p, size_t n, const float *const *g_local, void *const *out_payload,
                   float *const *out_scales);
void orc_allreduce_direct(int mode, int p, size_t n, const float *const *g_local, void *const *out_payload,
                          float *const *out_scales, uint64_t *counters);
int orc_allreduce_hd(int mode, int p, size_t n, const float *const *g_local, void *const *out_payload,
                     float *const *out_scales, uint64_t *counters);
void orc_sgd_update(int mode, const void *g_sum_c, const float *scales, size_t n, float *w, float *v, float lr,
                    float momentum, float grad_scale);
}

#define HIP_OK(call)                                                                            \
    do {                                                                                        \
        hipError_t e_ = (call);                                                                 \
        if (e_ != hipSuccess) {                                                                 \
            std::fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, hipGetErrorString(e_));     \
            return 2;                                                                           \
        }                                                                                       \
    } while (0)
#define LIB_OK(call)                                                                            \
    do {                                                                                        \
        int rc_ = (call);                                                                       \
        if (rc_ != PIPESGD_OK) {                                                                \
            std::fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, pipesgd_strerror(rc_));     \
            return 2;                                                                           \
        }                                                                                       \
    } while (0)

// seeded synthetic values: splitmix64 -> sum of four uniforms (bell-shaped), scaled
static uint64_t mix(uint64_t &s)
{
    uint64_t z = (s += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
}
static void fill(std::vector<float> &x, uint64_t seed, float scale)
{
    uint64_t s = seed;
    for (float &v : x) {
        const uint64_t z = mix(s);
        double u = 0.0;
        for (int k = 0; k < 4; ++k) u += static_cast<double>((z >> (16 * k)) & 0xffff) / 65536.0 - 0.5;
        v = static_cast<float>(u * scale);
    }
}

struct Dev {   // p device buffers of `bytes` bytes each
    std::vector<void *> ptr;
    int alloc(int p, size_t bytes)
    {
        ptr.assign(p, nullptr);
        for (int r = 0; r < p; ++r) HIP_OK(hipMalloc(&ptr[r], bytes ? bytes : 16));
        return 0;
    }
    ~Dev() { for (void *q : ptr) (void)hipFree(q); }
};

static int run_case(int mode, int p, size_t n)
{
    const float lr = 0.01f, momentum = 0.9f;
    const size_t pb = orc_payload_bytes(mode, n), ns = orc_num_scales(mode, n);
    if (pb != pipesgd_payload_bytes(mode, n) || ns != pipesgd_num_scales(mode, n)) {
        std::fprintf(stderr, "size rules differ\n");
        return 1;
    }
    std::vector<std::vector<float>> g(p, std::vector<float>(n)), w(p, std::vector<float>(n)), v(p, std::vector<float>(n));
    for (int r = 0; r < p; ++r) {
        fill(g[r], 1000 * mode + 10 * r + 1, 2e-3f);
        fill(w[r], 77, 0.1f);                 // every replica starts from the same model (Alg. 1)
        fill(v[r], 78, 0.01f);
    }
    Dev dg, dslot, dsc, dstage, dstage_sc, dpartial, dw, dv;
    if (dg.alloc(p, 4 * n) || dslot.alloc(p, pb) || dsc.alloc(p, 4 * ns) || dstage.alloc(p, pb) ||
        dstage_sc.alloc(p, 4 * ns) || dpartial.alloc(p, 4 * n) || dw.alloc(p, 4 * n) || dv.alloc(p, 4 * n))
        return 2;
    for (int r = 0; r < p; ++r) HIP_OK(hipMemcpy(dg.ptr[r], g[r].data(), 4 * n, hipMemcpyHostToDevice));

    pipesgd_ring ring;
    std::memset(&ring, 0, sizeof ring);
    ring.workers = p; ring.mode = mode; ring.n = n;
    for (int r = 0; r < p; ++r) {
        ring.g_local[r] = static_cast<const float *>(dg.ptr[r]);
        ring.g_sum_c[r] = dslot.ptr[r];
        ring.scales[r] = mode == PIPESGD_QUANT8 ? static_cast<float *>(dsc.ptr[r]) : nullptr;
    }
    std::vector<float *> stage_sc(p), partial(p);
    for (int r = 0; r < p; ++r) { stage_sc[r] = static_cast<float *>(dstage_sc.ptr[r]); partial[r] = static_cast<float *>(dpartial.ptr[r]); }
    pipesgd_workspace ws;
    ws.stage = dstage.ptr.data(); ws.stage_scales = stage_sc.data(); ws.partial = partial.data();
    ws.stage_bytes = pb; ws.stage_scales_bytes = 4 * ns; ws.partial_bytes = 4 * n;

    std::vector<std::vector<unsigned char>> want(p, std::vector<unsigned char>(pb + 1)), got(p, std::vector<unsigned char>(pb + 1));
    std::vector<std::vector<float>> want_sc(p, std::vector<float>(ns + 1)), got_sc(p, std::vector<float>(ns + 1));
    std::vector<const float *> gp(p);
    std::vector<void *> wp(p);
    std::vector<float *> wsp(p);
    for (int r = 0; r < p; ++r) { gp[r] = g[r].data(); wp[r] = want[r].data(); wsp[r] = want_sc[r].data(); }

    const char *names[4] = {"stepwise", "fused", "one-exchange", "halving-doubling"};
    int schedules_run = 0;
    for (int sched = 0; sched < 4; ++sched) {
        if (sched == 3 && (p & (p - 1)) != 0) continue;     // needs a power-of-two worker count
        ++schedules_run;
        for (int r = 0; r < p; ++r) {                     // poison the result buffers
            HIP_OK(hipMemset(dslot.ptr[r], 0x55, pb));
            if (ns) HIP_OK(hipMemset(dsc.ptr[r], 0x55, 4 * ns));
        }
        switch (sched) {
        case 0: LIB_OK(pipesgd_allreduce_sim(&ring, PIPESGD_STEPWISE, nullptr)); break;
        case 1: LIB_OK(pipesgd_allreduce_sim(&ring, PIPESGD_FUSED, nullptr)); break;
        case 2: LIB_OK(pipesgd_allreduce_direct(&ring, &ws, nullptr)); break;
        default: LIB_OK(pipesgd_allreduce_halving_doubling(&ring, &ws, nullptr)); break;
        }
        HIP_OK(hipDeviceSynchronize());
        if (sched <= 1) orc_allreduce(mode, p, n, gp.data(), wp.data(), wsp.data());
        else if (sched == 2) orc_allreduce_direct(mode, p, n, gp.data(), wp.data(), wsp.data(), nullptr);
        else if (orc_allreduce_hd(mode, p, n, gp.data(), wp.data(), wsp.data(), nullptr) != 0) return 1;
        for (int r = 0; r < p; ++r) {
            HIP_OK(hipMemcpy(got[r].data(), dslot.ptr[r], pb, hipMemcpyDeviceToHost));
            if (ns) HIP_OK(hipMemcpy(got_sc[r].data(), dsc.ptr[r], 4 * ns, hipMemcpyDeviceToHost));
            if (std::memcmp(got[r].data(), want[r].data(), pb) != 0 ||
                (ns && std::memcmp(got_sc[r].data(), want_sc[r].data(), 4 * ns) != 0)) {
                std::fprintf(stderr, "MISMATCH mode %d p %d n %zu schedule %s worker %d\n", mode, p, n, names[sched], r);
                return 1;
            }
        }
    }
    // the update of every replica from the last result (the oracle's and the library's agree, checked above)
    for (int r = 0; r < p; ++r) {
        HIP_OK(hipMemcpy(dw.ptr[r], w[r].data(), 4 * n, hipMemcpyHostToDevice));
        HIP_OK(hipMemcpy(dv.ptr[r], v[r].data(), 4 * n, hipMemcpyHostToDevice));
    }
    std::vector<const void *> slots(p);
    std::vector<const float *> scs(p);
    std::vector<float *> dwp(p), dvp(p);
    for (int r = 0; r < p; ++r) {
        slots[r] = dslot.ptr[r]; scs[r] = static_cast<const float *>(dsc.ptr[r]);
        dwp[r] = static_cast<float *>(dw.ptr[r]); dvp[r] = static_cast<float *>(dv.ptr[r]);
    }
    LIB_OK(pipesgd_apply_update_multi(mode, p, slots.data(), mode == PIPESGD_QUANT8 ? scs.data() : nullptr, n, dwp.data(),
                                      dvp.data(), lr, momentum, 1.0f, nullptr));
    HIP_OK(hipDeviceSynchronize());
    std::vector<float> back(n);
    for (int r = 0; r < p; ++r) {
        orc_sgd_update(mode, want[r].data(), want_sc[r].data(), n, w[r].data(), v[r].data(), lr, momentum, 1.0f);
        HIP_OK(hipMemcpy(back.data(), dw.ptr[r], 4 * n, hipMemcpyDeviceToHost));
        if (std::memcmp(back.data(), w[r].data(), 4 * n) != 0) { std::fprintf(stderr, "MISMATCH w mode %d worker %d\n", mode, r); return 1; }
        HIP_OK(hipMemcpy(back.data(), dv.ptr[r], 4 * n, hipMemcpyDeviceToHost));
        if (std::memcmp(back.data(), v[r].data(), 4 * n) != 0) { std::fprintf(stderr, "MISMATCH v mode %d worker %d\n", mode, r); return 1; }
    }
    std::printf("ok: mode %d p %d n %zu (%d schedules + update, every byte)\n", mode, p, n, schedules_run);
    std::fflush(stdout);
    return 0;
}

int main()
{
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || count < 1) { std::fprintf(stderr, "no GPU\n"); return 3; }
    if (pipesgd_version() < 100) return 1;
    const struct { int p; size_t n; } cases[] = {{4, 4096 * 13 + 57}, {3, 50001}, {8, 4096 * 40}, {2, 5}, {1, 9000}};
    for (int mode = 0; mode < 3; ++mode)
        for (const auto &c : cases) {
            const int rc = run_case(mode, c.p, c.n);
            if (rc != 0) return rc;
        }
    std::printf("native parity ok\n");
    return 0;
}
