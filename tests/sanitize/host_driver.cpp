// Driver for an AddressSanitizer + UndefinedBehaviorSanitizer build of the library's host side
// (csrc/fq_api.cpp: validation, chunk planning, workspace layout, descriptor tables, plans), with
// the kernel launchers and the few HIP runtime calls it makes replaced by host stubs.  The stubs
// are not idle: the "device" is host memory, the table copy is a memcpy, and each stubbed launch
// checks what the kernels rely on -- every tensor's blocks, partial sums and slots lie inside the
// grid and inside the workspace the caller was told to provide, and consecutive tensors do not
// overlap there.  Exit status 0: clean.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/fq.h"
#include "../../paper_2511_12653_amd/csrc/fq_internal.h"

static int failures = 0;
#define EXPECT(cond)                                                        \
    do {                                                                    \
        if (!(cond)) {                                                      \
            std::printf("line %d: expectation failed: %s\n", __LINE__, #cond); \
            ++failures;                                                     \
        }                                                                   \
    } while (0)

// ---- what the launch stubs check against ------------------------------------------------------
static const char *g_ws = nullptr;          // workspace of the call in progress
static size_t g_ws_bytes = 0;
static int g_launches = 0;

static bool inside(const void *p, size_t bytes)
{
    const char *c = (const char *)p;
    return c >= g_ws && c + bytes <= g_ws + g_ws_bytes;
}

static void check_table(const fq::KArgs &a, unsigned blocks, bool backward)
{
    ++g_launches;
    const fq::DevTensor *t = a.table ? a.table : &a.one;
    const int n = a.table ? a.n : 1;
    if (a.table) EXPECT(inside(a.table, (size_t)n * sizeof(fq::DevTensor)));
    unsigned long long block = 0;
    const double *partial_end = nullptr;
    const unsigned long long *slot_end = nullptr;
    for (int i = 0; i < n; ++i) {
        const fq::DevTensor &d = t[i];
        const unsigned long long units = (unsigned long long)d.slabs * d.cps;
        const unsigned long long my_blocks = d.wave_units ? (units + 3) / 4 : units;
        EXPECT(d.block_begin == block);
        block += d.outer ? my_blocks : 0;
        if (d.outer) {
            EXPECT(d.cps >= 1 && d.chunk >= 1);
            EXPECT((unsigned long long)d.cps * d.chunk >= (unsigned long long)d.inner);            // chunks cover the slab
            EXPECT((unsigned long long)(d.cps - 1) * d.chunk < (unsigned long long)d.inner);       // and none is empty
            EXPECT(d.chunk % (16 / (d.dtype == 0 ? 2 : 4)) == 0);
            EXPECT(d.slabs == d.outer * d.channels);
        }
        if (backward && d.outer) {
            EXPECT(inside(d.partial, units * sizeof(double)));
            const unsigned long long slots = (unsigned long long)d.channels * (1 + d.sub);
            EXPECT(inside(d.slot, slots * sizeof(unsigned long long)));
            if (partial_end) EXPECT(d.partial >= partial_end);
            if (slot_end) EXPECT(d.slot >= slot_end);
            partial_end = d.partial + units;
            slot_end = d.slot + slots;
            for (unsigned long long s = 0; s < slots; ++s) EXPECT(d.slot[s] == 0);                 // zeroed workspace
        }
    }
    EXPECT(block == blocks);
}

namespace fq {
int launch_forward(const KArgs &a, unsigned blocks, bool, void *) { check_table(a, blocks, false); return 0; }
int launch_backward(const KArgs &a, unsigned blocks, bool, void *) { check_table(a, blocks, true); return 0; }
int launch_finalize(const KArgs &, unsigned, void *) { ++g_launches; return 0; }
int launch_scale_only(const KArgs &, unsigned, void *) { ++g_launches; return 0; }
int launch_fill_zero(void *p, size_t bytes, void *) { std::memset(p, 0, bytes); return 0; }
int launch_probe(int, const void *, const void *, void *, size_t, void *) { return 0; }
int static_scratch(void **ptr, void *)
{
    static std::vector<char> scratch(kStaticScratchBytes);
    *ptr = scratch.data();
    g_ws = scratch.data();
    g_ws_bytes = scratch.size();
    return 0;
}
}  // namespace fq

// ---- the HIP runtime calls of the staging ring, on host memory ---------------------------------
extern "C" {
hipError_t hipHostMalloc(void **p, size_t bytes, unsigned) { *p = std::malloc(bytes); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipHostFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned) { *e = (hipEvent_t)std::malloc(1); return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipMemcpyAsync(void *dst, const void *src, size_t bytes, hipMemcpyKind, hipStream_t)
{
    std::memcpy(dst, src, bytes);
    return hipSuccess;
}
}

// ---- cases -------------------------------------------------------------------------------------
static uint64_t rng_state = 0x2511126530ull;
static uint32_t rnd(uint32_t n)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(rng_state >> 33) % n;
}

// A descriptor over fake, far-apart device addresses (nothing dereferences them on the host).
static fq_tensor tensor(int64_t outer, int64_t channels, int64_t inner, int dtype, unsigned id)
{
    fq_tensor t;
    std::memset(&t, 0, sizeof t);
    t.outer = outer; t.channels = channels; t.inner = inner;
    t.dtype = dtype; t.qmin = -128; t.qmax = 127;
    t.eps = 0.0f; t.s_min = 1.17549435e-38f; t.s_max = INFINITY;
    const uintptr_t base = ((uintptr_t)(id + 1)) << 44;
    t.x = (const void *)(base + ((uintptr_t)1 << 40));
    t.y = (void *)(base + ((uintptr_t)2 << 40));
    t.gy = (const void *)(base + ((uintptr_t)3 << 40));
    t.gx = (void *)(base + ((uintptr_t)4 << 40));
    t.theta = (const float *)(base + ((uintptr_t)5 << 40));
    t.gtheta = (float *)(base + ((uintptr_t)6 << 40));
    return t;
}

static void run_list(const std::vector<fq_tensor> &ts, int mode)
{
    const int n = (int)ts.size();
    const size_t need = fq_workspace_bytes(ts.data(), n, mode);
    EXPECT(need >= 256 && need % 256 == 0);
    EXPECT(fq_validate(ts.data(), n, mode) == FQ_OK);
    // exactly the promised size (any write past it is an ASan report), aligned as the API asks
    char *ws = (char *)std::aligned_alloc(256, need);
    std::memset(ws, 0, need);
    g_ws = ws; g_ws_bytes = need;
    EXPECT(fq_multi_tensor(ts.data(), n, mode, ws, need, nullptr) == FQ_OK);
    EXPECT(fq_multi_tensor(ts.data(), n, mode, ws, need - 256, nullptr) == (n ? FQ_ERR_WORKSPACE : FQ_OK));
    EXPECT(fq_multi_tensor(ts.data(), n, mode, ws + 8, need, nullptr) == (n ? FQ_ERR_ALIGN : FQ_OK));
    fq_plan *plan = nullptr;
    EXPECT(fq_plan_create(ts.data(), n, mode, ws, need, nullptr, &plan) == FQ_OK);
    EXPECT(fq_plan_run(plan, nullptr) == FQ_OK);
    if (mode == FQ_MODE_BACKWARD) EXPECT(fq_plan_run_adam(plan, 3, nullptr) == FQ_OK);
    fq_plan_destroy(plan);
    if (n == 1 && mode == FQ_MODE_BACKWARD) {
        EXPECT(fq_backward(&ts[0], ws, need, nullptr) == FQ_OK);
        fq_layout_info info;
        EXPECT(fq_layout(&ts[0], &info) == FQ_OK);
        const fq_status st = fq_backward_static(&ts[0], nullptr);          // g_ws now names the stub's scratch array
        const bool fits = info.units_per_channel * ts[0].channels <= FQ_STATIC_MAX_UNITS &&
                          ts[0].channels * (1 + (int64_t)info.extra_slots) <= FQ_STATIC_MAX_SLOTS;
        EXPECT(st == (fits ? FQ_OK : FQ_ERR_WORKSPACE));
    }
    if (n == 1 && mode == FQ_MODE_FORWARD) EXPECT(fq_forward(&ts[0], nullptr) == FQ_OK);
    std::free(ws);
}

int main()
{
    // shapes around the planner's cases: empty, one element, short slabs (one wavefront per slab in
    // big launches), one to many chunks per slab, every combination protocol's unit count
    static const int64_t shapes[][3] = {
        {0, 4, 16}, {2, 0, 16}, {2, 4, 0}, {1, 1, 1}, {1, 1, 7}, {1, 384, 19200}, {15, 128, 19200}, {1, 1, 153600},
        {1, 1, 7372800}, {1, 384, 28800}, {1, 384, 22560}, {8, 384, 19200}, {9, 384, 19200}, {3, 4100, 40},
        {17, 4100, 40}, {257, 4100, 40}, {300, 4100, 40}, {384, 1, 3456}, {1, 384, 3456}, {1, 128, 1152}, {5, 3, 10241},
        {1, 70000, 9}, {70000, 1, 9}, {2, 2, 1280 * 8 + 1}, {1, 1, (int64_t)1 << 31}};
    for (const auto &s : shapes)
        for (int dtype = 0; dtype < 2; ++dtype)
            for (int mode = FQ_MODE_FORWARD; mode <= FQ_MODE_BACKWARD; ++mode) {
                std::vector<fq_tensor> one{tensor(s[0], s[1], s[2], dtype, 0)};
                run_list(one, mode);
            }
    // lists: empty, mixed, and a few hundred random tensors (enough blocks for the wavefront units)
    for (int mode = FQ_MODE_FORWARD; mode <= FQ_MODE_BACKWARD; ++mode) {
        run_list({}, mode);
        std::vector<fq_tensor> mixed;
        unsigned id = 0;
        for (const auto &s : shapes)
            if (s[0] * s[1] * s[2] < 40000000) mixed.push_back(tensor(s[0], s[1], s[2], (int)(id & 1), id)), ++id;
        run_list(mixed, mode);
        for (int round = 0; round < 20; ++round) {
            std::vector<fq_tensor> ts;
            const int n = 1 + (int)rnd(60);
            for (int i = 0; i < n; ++i) {
                const int64_t outer = 1 + rnd(rnd(4) ? 4 : 300), ch = 1 + rnd(rnd(3) ? 8 : 500), inner = rnd(rnd(3) ? 50 : 30000);
                fq_tensor t = tensor(outer, ch, inner, (int)rnd(2), (unsigned)i);
                if (rnd(4) == 0) t.flags |= FQ_FLAG_NO_DX;
                if (rnd(3) == 0) { t.qmin = -8; t.qmax = 7; }
                ts.push_back(t);
            }
            if (rnd(5) == 0) ts[0].flags |= FQ_FLAG_TWO_PASS;
            run_list(ts, mode);
        }
    }
    // rejections leave through their status codes
    {
        fq_tensor t = tensor(2, 3, 100, FQ_F16, 0);
        fq_tensor bad = t; bad.dtype = 9;
        EXPECT(fq_validate(&bad, 1, FQ_MODE_FORWARD) == FQ_ERR_DTYPE);
        bad = t; bad.outer = -1;
        EXPECT(fq_validate(&bad, 1, FQ_MODE_FORWARD) == FQ_ERR_SHAPE);
        bad = t; bad.inner = (int64_t)1 << 62;
        EXPECT(fq_validate(&bad, 1, FQ_MODE_FORWARD) == FQ_ERR_SHAPE);
        bad = t; bad.qmin = 1;
        EXPECT(fq_validate(&bad, 1, FQ_MODE_FORWARD) == FQ_ERR_QRANGE);
        bad = t; bad.s_min = 0.0f;
        EXPECT(fq_validate(&bad, 1, FQ_MODE_FORWARD) == FQ_ERR_SCALE_PARAMS);
        bad = t; bad.x = (const void *)((uintptr_t)t.x + 1);
        EXPECT(fq_validate(&bad, 1, FQ_MODE_FORWARD) == FQ_ERR_ALIGN);
        bad = t; bad.y = (void *)((uintptr_t)t.x + 2);
        EXPECT(fq_validate(&bad, 1, FQ_MODE_FORWARD) == FQ_ERR_ALIAS);
        EXPECT(fq_validate(&t, -1, FQ_MODE_FORWARD) == FQ_ERR_SHAPE);
        EXPECT(fq_validate(&t, 1, 7) == FQ_ERR_SHAPE);
        EXPECT(fq_validate(nullptr, 1, FQ_MODE_FORWARD) == FQ_ERR_NULL);
        EXPECT(fq_workspace_bytes(&bad, 1, FQ_MODE_FORWARD) == 0);
        EXPECT(fq_layout(nullptr, nullptr) == FQ_ERR_NULL);
        EXPECT(fq_backward_static(nullptr, nullptr) == FQ_ERR_NULL);
        for (int code = -12; code <= 1; ++code) EXPECT(fq_status_string((fq_status)code) != nullptr);
    }
    std::printf("host sanitizer run: %d stubbed launches checked, %d failures\n", g_launches, failures);
    return failures ? 1 : 0;
}
