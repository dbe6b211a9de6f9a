// Host side of libfq: argument validation, chunk planning, workspace layout and the C ABI
// declared in include/fq.h.  Validation and sizing are pure host code (no HIP call), so they can
// be exercised on a machine without a GPU.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/fq.h"
#include "fq_internal.h"

static_assert(FQ_STATIC_SCRATCH_BYTES == fq::kStaticScratchBytes && FQ_STATIC_MAX_SLOTS * 8 == fq::kStaticSlotBytes &&
                  FQ_STATIC_MAX_UNITS * 8 == fq::kStaticPartialBytes,
              "the limits stated in fq.h are the ones the library is built with");

namespace fq {
namespace {

constexpr size_t kAlign = 256;
constexpr long long kMaxBlocks = 0x7fffffffLL;
constexpr long long kWaveUnitsMinBlocks = 4096;   // 16 blocks per compute unit

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

// Partial overlap of [a, a+bytes) and [b, b+bytes) (identical ranges are fine).
bool partial_overlap(const void *a, const void *b, size_t bytes)
{
    if (!a || !b || a == b || bytes == 0) return false;
    uintptr_t pa = (uintptr_t)a, pb = (uintptr_t)b;
    return pa < pb ? (pb - pa) < bytes : (pa - pb) < bytes;
}

// Any overlap of [a, a+abytes) and [b, b+bbytes).
bool overlap(const void *a, size_t abytes, const void *b, size_t bbytes)
{
    if (!a || !b || abytes == 0 || bbytes == 0) return false;
    uintptr_t pa = (uintptr_t)a, pb = (uintptr_t)b;
    return pa < pb + bbytes && pb < pa + abytes;
}

struct Plan {
    long long numel = 0;
    unsigned slabs = 0, cps = 0, chunk = 0;
    unsigned sub = 0;            // extra slots per channel: pair slots (2) or first-level ticket slots (32)
    bool short_slabs = false;    // a slab fits one wavefront's chunk
    bool waves = false;          // short slabs in a launch with blocks to spare: one wavefront per slab,
                                 // four slabs to a block
    long long blocks = 0;        // grid blocks
    long long units = 0;         // partial sums: one per block, or one per slab with `waves'
};

// Slots a channel needs beside its own, by the number of units (blocks or wavefronts) that
// combine their sums for it: pair slots of the exchange tree, or first-level ticket slots.
unsigned extra_slots(long long units_per_channel)
{
    if (units_per_channel > (long long)kTicketManyUnits) return kTicketManySubSlots;
    if (units_per_channel > (long long)kTicketFanIn) return kTicketSubSlots;
    if (units_per_channel > 2 && units_per_channel <= (long long)kTreeBlocks) return 2u;
    return 0u;
}

// Split every [outer, channel] slab into cps equal chunks of at most kChunkVecs vectors each,
// chunk length a multiple of the vector width so all chunks of a slab share one alignment.
// A block's wavefront handles r = 1..5 rows of 64 vectors; among those five chunk sizes pick the
// one with the smallest estimated makespan: (blocks per compute unit, rounded up) x (rows per
// wavefront + 1 for the per-block prologue).  Large tensors end up with the biggest chunks, a
// tensor whose block count is a small multiple of the CU count avoids a mostly-empty last round.
fq_status plan_tensor(const fq_tensor &t, Plan &p, bool allow_waves)
{
    if (t.dtype != FQ_F16 && t.dtype != FQ_F32) return FQ_ERR_DTYPE;
    if (t.outer < 0 || t.channels < 0 || t.inner < 0) return FQ_ERR_SHAPE;
    if (t.channels > 0x7fffffffLL || t.outer > 0x7fffffffLL) return FQ_ERR_SHAPE;
    const long long slabs = t.outer * t.channels;
    if (slabs > 0x7fffffffLL) return FQ_ERR_SHAPE;
    if (t.inner > 0 && slabs > 0 && t.inner > (1LL << 62) / slabs) return FQ_ERR_SHAPE;
    p.numel = slabs * t.inner;
    p.slabs = (unsigned)slabs;
    if (p.numel == 0) {
        p.cps = 0; p.chunk = 0; p.blocks = 0;
        return FQ_OK;
    }
    const long long vec = kVecBytes / (t.dtype == FQ_F16 ? 2 : 4);
    const long long slab_vecs = (t.inner + vec - 1) / vec;
    // Slabs that one wavefront covers (320 vectors; one vector more than the aligned part can hold
    // is left for a misaligned head) go one to a wavefront: a block per slab would leave most of
    // its lanes idle and pay a block's prologue and reduction for a few KB.  Only where the launch
    // has blocks to spare (allow_waves): a small tensor on its own is bound by latency and is
    // better off spread over four times as many blocks.
    p.short_slabs = slab_vecs + 1 <= kWaveChunkVecs;
    if (allow_waves && p.short_slabs) {
        p.waves = true;
        p.cps = 1;
        p.chunk = (unsigned)((t.inner + vec - 1) / vec * vec);
        p.units = slabs;
        p.blocks = (slabs + kBlock / 64 - 1) / (kBlock / 64);
        p.sub = extra_slots(t.outer);
        return FQ_OK;
    }
    const int max_rows = kChunkVecs / kBlock;
    long long best_cps = 0, best_chunk = 0;
    double best_cost = 0.0;
    for (int r = max_rows; r >= 1; --r) {
        long long cps = (slab_vecs + (long long)kBlock * r - 1) / ((long long)kBlock * r);
        long long chunk = (t.inner + cps - 1) / cps;
        chunk = (chunk + vec - 1) / vec * vec;
        cps = (t.inner + chunk - 1) / chunk;
        const long long chunk_vecs = chunk / vec;
        const long long rows_per_wave = ((chunk_vecs + 63) / 64 + 3) / 4;
        const double blocks = (double)slabs * (double)cps;
        const double rounds = std::ceil(blocks / kComputeUnits);
        const double cost = rounds * (double)(rows_per_wave + 1);
        if (best_cps == 0 || cost < best_cost) {
            best_cost = cost; best_cps = cps; best_chunk = chunk;
        }
    }
    if (best_cps > kMaxBlocks || (double)slabs * (double)best_cps > (double)kMaxBlocks) return FQ_ERR_SHAPE;
    p.cps = (unsigned)best_cps;
    p.chunk = (unsigned)best_chunk;
    p.blocks = slabs * best_cps;
    p.units = p.blocks;
    const long long per_channel = t.outer * best_cps;                             // blocks per channel
    p.sub = extra_slots(per_channel);
    return FQ_OK;
}

fq_status validate_one(const fq_tensor &t, int mode, Plan &p)
{
    fq_status st = plan_tensor(t, p, false);
    if (st != FQ_OK) return st;
    if (!(t.qmin <= 0 && 0 <= t.qmax && t.qmin < t.qmax) || t.qmin < -32768 || t.qmax > 32768)
        return FQ_ERR_QRANGE;
    if (!std::isfinite(t.eps) || std::isnan(t.s_min) || std::isnan(t.s_max) || !(t.s_min > 0.0f) ||
        !std::isfinite(t.s_min) || !(t.s_max >= t.s_min))
        return FQ_ERR_SCALE_PARAMS;
    const size_t esz = t.dtype == FQ_F16 ? 2 : 4;
    const size_t bytes = (size_t)p.numel * esz;
    if (t.channels > 0 && !t.theta) return FQ_ERR_NULL;
    if (!aligned(t.theta, 4) || !aligned(t.s, 4) || !aligned(t.gs, 4) || !aligned(t.gtheta, 4))
        return FQ_ERR_ALIGN;
    if (p.numel > 0 && !t.x) return FQ_ERR_NULL;
    if (!aligned(t.x, esz)) return FQ_ERR_ALIGN;
    if (mode == FQ_MODE_FORWARD) {
        if (p.numel > 0 && !t.y && !t.q) return FQ_ERR_NULL;
        if (!aligned(t.y, esz)) return FQ_ERR_ALIGN;
        if (t.q && (t.qmin < -128 || t.qmax > 127)) return FQ_ERR_QRANGE;
        if (partial_overlap(t.x, t.y, bytes)) return FQ_ERR_ALIAS;
        // the codes are a different size per element: they may not share memory with x or y at all
        if (overlap(t.q, (size_t)p.numel, t.x, bytes) || overlap(t.q, (size_t)p.numel, t.y, bytes))
            return FQ_ERR_ALIAS;
    } else {
        const bool need_gx = !(t.flags & FQ_FLAG_NO_DX);
        if (p.numel > 0 && (!t.gy || (need_gx && !t.gx))) return FQ_ERR_NULL;
        if (!aligned(t.gy, esz) || (need_gx && !aligned(t.gx, esz))) return FQ_ERR_ALIGN;
        if (need_gx && (partial_overlap(t.gy, t.gx, bytes) || partial_overlap(t.x, t.gx, bytes)))
            return FQ_ERR_ALIAS;
        if (t.adam) {
            const fq_adam &a = *t.adam;
            if (a.step < 1 || !(a.beta1 >= 0.0 && a.beta1 < 1.0) || !(a.beta2 >= 0.0 && a.beta2 < 1.0) ||
                !std::isfinite(a.lr) || !std::isfinite(a.eps) || a.eps < 0.0)
                return FQ_ERR_OPTIMIZER;
            if (t.channels > 0 && (!a.m || !a.v || !a.theta_out)) return FQ_ERR_NULL;
            if (!aligned(a.m, 4) || !aligned(a.v, 4) || !aligned(a.theta_out, 4)) return FQ_ERR_ALIGN;
        }
    }
    return FQ_OK;
}

struct Layout {
    std::vector<Plan> plans;
    long long blocks = 0;        // grid of the main kernel
    long long channels = 0;      // grid of the finalize kernel
    long long slots = 0;         // 64-bit ticket / exchange slots (backward)
    long long partials = 0;      // doubles
    size_t table_bytes = 0, partial_off = 0, counter_off = 0, total = 0;
    bool any_empty_with_channels = false;
};

fq_status make_layout(const fq_tensor *ts, int n, int mode, Layout &L)
{
    if (mode != FQ_MODE_FORWARD && mode != FQ_MODE_BACKWARD) return FQ_ERR_SHAPE;
    if (n < 0) return FQ_ERR_SHAPE;
    if (n > 0 && !ts) return FQ_ERR_NULL;
    L.plans.resize((size_t)n);
    for (int i = 0; i < n; ++i) {
        fq_status st = validate_one(ts[i], mode, L.plans[(size_t)i]);
        if (st != FQ_OK) return st;
        L.blocks += L.plans[(size_t)i].blocks;
        L.partials += L.plans[(size_t)i].units;
        L.channels += ts[i].channels;
        L.slots += ts[i].channels * (1 + (long long)L.plans[(size_t)i].sub);
        if (L.plans[(size_t)i].numel == 0 && ts[i].channels > 0) L.any_empty_with_channels = true;
        if (L.blocks > kMaxBlocks || L.channels > kMaxBlocks || L.slots > 64 * kMaxBlocks) return FQ_ERR_SHAPE;
    }
    if (L.blocks >= kWaveUnitsMinBlocks) {
        // enough blocks to fill the chip many times over: short-slab tensors switch to one
        // wavefront per slab (fewer blocks, partial sums and slots; the limits above still hold)
        for (int i = 0; i < n; ++i) {
            Plan &p = L.plans[(size_t)i];
            if (!p.short_slabs || p.numel == 0) continue;
            L.blocks -= p.blocks;
            L.partials -= p.units;
            L.slots -= ts[i].channels * (1 + (long long)p.sub);
            (void)plan_tensor(ts[i], p, true);
            L.blocks += p.blocks;
            L.partials += p.units;
            L.slots += ts[i].channels * (1 + (long long)p.sub);
        }
    }
    L.table_bytes = round_up((size_t)n * sizeof(DevTensor), kAlign);
    L.partial_off = L.table_bytes;
    L.counter_off = L.partial_off;
    L.total = L.table_bytes;
    if (mode == FQ_MODE_BACKWARD) {
        L.counter_off = L.partial_off + round_up((size_t)L.partials * sizeof(double), kAlign);
        L.total = L.counter_off + round_up((size_t)L.slots * sizeof(unsigned long long), kAlign);
    }
    if (L.total < kAlign) L.total = kAlign;
    return FQ_OK;
}

// Where a tensor's share of a launch begins: grid block, finalize-grid channel, 64-bit slot and
// partial sum.
struct Cursor {
    long long block = 0, chan = 0, slot = 0, unit = 0;
};

// Device descriptor of one tensor; `partials` / `slots` are the launch's arrays of partial sums and
// of 64-bit slots (nullptr: forward, nothing is reduced).
DevTensor describe(const fq_tensor &t, const Plan &p, int mode, double *partials, unsigned long long *slots,
                   const Cursor &at)
{
    DevTensor d;
    std::memset(&d, 0, sizeof d);
    d.x = t.x; d.y = t.y; d.q = t.q; d.theta = t.theta; d.s = t.s;
    d.gy = t.gy; d.gx = t.gx; d.gs = t.gs; d.gtheta = t.gtheta;
    d.partial = partials ? partials + at.unit : nullptr;
    d.slot = slots ? slots + at.slot : nullptr;
    d.inner = t.inner;
    d.slabs = p.slabs;
    d.channels = (unsigned)t.channels;
    d.outer = p.numel ? (unsigned)t.outer : 0u;
    d.cps = p.cps;
    d.chunk = p.chunk;
    d.block_begin = (unsigned)at.block;
    d.chan_begin = (unsigned)at.chan;
    d.sub = p.sub;
    d.wave_units = p.waves ? 1u : 0u;
    d.dtype = t.dtype;
    d.lo = (float)t.qmin;
    d.hi = (float)t.qmax;
    d.eps = t.eps; d.s_min = t.s_min; d.s_max = t.s_max;
    d.flags = t.flags;
    if (mode == FQ_MODE_BACKWARD && t.adam && t.channels > 0) {   // validated for this mode only
        const fq_adam &a = *t.adam;
        d.adam_m = a.m; d.adam_v = a.v; d.adam_theta_out = a.theta_out;
        d.adam_lr = (float)a.lr;
        d.adam_beta1 = (float)a.beta1; d.adam_one_minus_beta1 = (float)(1.0 - a.beta1);
        d.adam_beta2 = (float)a.beta2; d.adam_one_minus_beta2 = (float)(1.0 - a.beta2);
        d.adam_eps = (float)a.eps;
        d.adam_bc1 = (float)(1.0 - std::pow(a.beta1, (double)a.step));
        d.adam_bc2 = (float)(1.0 - std::pow(a.beta2, (double)a.step));
    }
    return d;
}

// A tensor launched on its own gets a three-dimensional grid (chunks per slab, channels, outer)
// unless its slabs go one to a wavefront or an extent exceeds the grid's y/z limit.
void set_grid_shape(DevTensor &d)
{
    d.grid3 = (!d.wave_units && d.cps > 0 && d.channels > 0 && d.outer > 0 && d.channels <= 65535u &&
               d.outer <= 65535u) ? 1u : 0u;
}

// Fill the device descriptors; partial/counter pointers are carved out of the workspace.
void build_table(const fq_tensor *ts, int n, int mode, const Layout &L, char *workspace,
                 std::vector<DevTensor> &out)
{
    out.resize((size_t)n);
    double *partials = workspace ? (double *)(workspace + L.partial_off) : nullptr;
    unsigned long long *slots = workspace ? (unsigned long long *)(workspace + L.counter_off) : nullptr;
    Cursor at;
    for (int i = 0; i < n; ++i) {
        const fq_tensor &t = ts[i];
        const Plan &p = L.plans[(size_t)i];
        out[(size_t)i] = describe(t, p, mode, partials, slots, at);
        at.block += p.blocks;
        at.unit += p.units;
        at.chan += t.channels;
        at.slot += t.channels * (1 + (long long)p.sub);
    }
}

// Pinned staging slots for the descriptor table of fq_multi_tensor.  The async copy reads the
// slot after the call has returned, so a slot is reused only once its copy has completed.
class Staging {
public:
    int copy(void *dst, const void *src, size_t bytes, hipStream_t stream)
    {
        std::lock_guard<std::mutex> lock(mu_);
        Slot &s = slots_[next_];
        next_ = (next_ + 1) % kSlots;
        hipError_t e;
        if (s.busy) {
            if ((e = hipEventSynchronize(s.done)) != hipSuccess) return (int)e;
            s.busy = false;
        }
        if (s.cap < bytes) {
            if (s.host) (void)hipHostFree(s.host);
            s.host = nullptr; s.cap = 0;
            size_t cap = round_up(bytes, 4096);
            if ((e = hipHostMalloc(&s.host, cap, hipHostMallocDefault)) != hipSuccess) return (int)e;
            s.cap = cap;
        }
        if (!s.done && (e = hipEventCreateWithFlags(&s.done, hipEventDisableTiming)) != hipSuccess)
            return (int)e;
        std::memcpy(s.host, src, bytes);
        if ((e = hipMemcpyAsync(dst, s.host, bytes, hipMemcpyHostToDevice, stream)) != hipSuccess)
            return (int)e;
        if ((e = hipEventRecord(s.done, stream)) != hipSuccess) return (int)e;
        s.busy = true;
        return 0;
    }

private:
    static constexpr int kSlots = 8;
    struct Slot {
        void *host = nullptr;
        size_t cap = 0;
        hipEvent_t done = nullptr;
        bool busy = false;
    };
    Slot slots_[kSlots];
    int next_ = 0;
    std::mutex mu_;
};

Staging &staging()
{
    static Staging *s = new Staging();   // never destroyed: no HIP calls during process teardown
    return *s;
}

bool any_flag(const fq_tensor *ts, int n, unsigned flag)
{
    for (int i = 0; i < n; ++i)
        if (ts[i].flags & flag) return true;
    return false;
}

// Everything a launch needs once the descriptors have been validated and laid out.
struct Prepared {
    KArgs args;
    int mode = 0;
    long long blocks = 0, channels = 0;
    bool emit_q = false, two_pass = false, any_empty_with_channels = false;
    std::vector<DevTensor> table;     // host copy of the device descriptors
};

// Validate, plan, build the device descriptors and (for table launches) copy them to the head of
// the workspace.  Nothing is launched.
fq_status prepare(const fq_tensor *ts, int n, int mode, bool use_table, void *workspace, size_t ws_bytes,
                  void *stream, Prepared &P)
{
    Layout L;
    fq_status st = make_layout(ts, n, mode, L);
    if (st != FQ_OK) return st;
    std::memset(&P.args, 0, sizeof P.args);
    P.args.n = n;
    P.mode = mode;
    if (n == 0) return FQ_OK;
    const bool need_ws = use_table || mode == FQ_MODE_BACKWARD;
    if (need_ws) {
        if (!workspace || ws_bytes < L.total) return FQ_ERR_WORKSPACE;
        if (!aligned(workspace, kAlign)) return FQ_ERR_ALIGN;
    }
    std::vector<DevTensor> &table = P.table;
    build_table(ts, n, mode, L, (char *)workspace, table);
    if (use_table) {
        P.args.table = (const DevTensor *)workspace;
        if (copy_table_async(workspace, table.data(), (size_t)n * sizeof(DevTensor), stream) != 0)
            return FQ_ERR_LAUNCH;
    } else {
        P.args.one = table[0];
        set_grid_shape(P.args.one);
    }
    P.blocks = L.blocks;
    P.channels = L.channels;
    P.any_empty_with_channels = L.any_empty_with_channels;
    for (int i = 0; i < n; ++i) P.emit_q = P.emit_q || ts[i].q != nullptr;
    P.two_pass = any_flag(ts, n, FQ_FLAG_TWO_PASS) || L.any_empty_with_channels;
    return FQ_OK;
}

fq_status launch_prepared(const Prepared &P, void *stream)
{
    if (P.args.n == 0) return FQ_OK;
    if (P.mode == FQ_MODE_FORWARD) {
        if (P.blocks > 0 && launch_forward(P.args, (unsigned)P.blocks, P.emit_q, stream) != 0) return FQ_ERR_LAUNCH;
        // tensors without elements never reach a block: write the scales of all channels in a
        // separate small launch (same values as the main kernel writes)
        if (P.any_empty_with_channels && launch_scale_only(P.args, (unsigned)P.channels, stream) != 0)
            return FQ_ERR_LAUNCH;
        return FQ_OK;
    }
    if (P.blocks > 0 && launch_backward(P.args, (unsigned)P.blocks, !P.two_pass, stream) != 0) return FQ_ERR_LAUNCH;
    if (P.two_pass && P.channels > 0 && launch_finalize(P.args, (unsigned)P.channels, stream) != 0)
        return FQ_ERR_LAUNCH;
    return FQ_OK;
}

fq_status run(const fq_tensor *ts, int n, int mode, bool use_table, void *workspace, size_t ws_bytes,
              void *stream)
{
    Prepared P;
    fq_status st = prepare(ts, n, mode, use_table, workspace, ws_bytes, stream, P);
    if (st != FQ_OK) return st;
    return launch_prepared(P, stream);
}

// Plan of one tensor launched on its own, without any heap use: validation, the cut into units, and
// the switch to one wavefront per slab for short slabs in a launch with blocks to spare.
fq_status plan_single(const fq_tensor &t, int mode, Plan &p)
{
    fq_status st = validate_one(t, mode, p);
    if (st != FQ_OK) return st;
    if (p.blocks > kMaxBlocks || t.channels * (1 + (long long)p.sub) > 64 * kMaxBlocks) return FQ_ERR_SHAPE;
    if (p.short_slabs && p.numel > 0 && p.blocks >= kWaveUnitsMinBlocks) (void)plan_tensor(t, p, true);
    return FQ_OK;
}

// fq_backward with the partial sums and slots in the library's built-in scratch array.  Touches
// no allocator, host or device: one descriptor on the stack, passed by value to the kernel.
fq_status run_static(const fq_tensor &t, void *stream)
{
    Plan p;
    fq_status st = plan_single(t, FQ_MODE_BACKWARD, p);
    if (st != FQ_OK) return st;
    const long long slots = t.channels * (1 + (long long)p.sub);
    if ((unsigned long long)slots * sizeof(unsigned long long) > kStaticSlotBytes ||
        (unsigned long long)p.units * sizeof(double) > kStaticPartialBytes)
        return FQ_ERR_WORKSPACE;
    void *base = nullptr;
    if (static_scratch(&base, stream) != 0) return FQ_ERR_LAUNCH;
    Prepared P;                               // its table (a vector) stays empty: nothing is allocated
    std::memset(&P.args, 0, sizeof P.args);
    P.args.n = 1;
    P.args.one = describe(t, p, FQ_MODE_BACKWARD, (double *)((char *)base + kStaticSlotBytes),
                          (unsigned long long *)base, Cursor());
    set_grid_shape(P.args.one);
    P.mode = FQ_MODE_BACKWARD;
    P.blocks = p.blocks;
    P.channels = t.channels;
    P.any_empty_with_channels = p.numel == 0 && t.channels > 0;
    P.two_pass = (t.flags & FQ_FLAG_TWO_PASS) != 0 || P.any_empty_with_channels;
    return launch_prepared(P, stream);
}

}  // namespace

int copy_table_async(void *dst_device, const void *src_host, size_t bytes, void *stream)
{
    return staging().copy(dst_device, src_host, bytes, (hipStream_t)stream);
}

}  // namespace fq

extern "C" {

// Host containers may throw std::bad_alloc for absurd n; nothing may leave through the C ABI.
#define FQ_GUARDED(expr, on_throw) \
    try {                          \
        return (expr);             \
    } catch (...) {                \
        return (on_throw);         \
    }

size_t fq_workspace_bytes(const fq_tensor *ts, int n, int mode)
{
    try {
        fq::Layout L;
        if (fq::make_layout(ts, n, mode, L) != FQ_OK) return 0;
        return L.total;
    } catch (...) {
        return 0;
    }
}

fq_status fq_validate(const fq_tensor *ts, int n, int mode)
{
    try {
        fq::Layout L;
        return fq::make_layout(ts, n, mode, L);
    } catch (...) {
        return FQ_ERR_SHAPE;
    }
}

fq_status fq_layout(const fq_tensor *t, fq_layout_info *info)
{
    if (!t || !info) return FQ_ERR_NULL;
    fq::Plan p;
    fq_status st = fq::plan_tensor(*t, p, false);
    if (st == FQ_OK && p.short_slabs && p.blocks >= (long long)fq::kWaveUnitsMinBlocks) st = fq::plan_tensor(*t, p, true);
    if (st != FQ_OK) return st;
    info->blocks = p.blocks;
    info->units_per_channel = t->outer * (long long)p.cps;
    info->unit_elems = p.chunk;
    info->wave_units = p.waves ? 1 : 0;
    info->extra_slots = (int32_t)p.sub;
    return FQ_OK;
}

fq_status fq_workspace_init(void *workspace, size_t ws_bytes, void *hip_stream)
{
    if (!workspace) return FQ_ERR_WORKSPACE;
    if (!fq::aligned(workspace, 4) || ws_bytes % 4 != 0) return FQ_ERR_ALIGN;
    return fq::launch_fill_zero(workspace, ws_bytes, hip_stream) == 0 ? FQ_OK : FQ_ERR_LAUNCH;
}

fq_status fq_forward(const fq_tensor *t, void *hip_stream)
{
    if (!t) return FQ_ERR_NULL;
    FQ_GUARDED(fq::run(t, 1, FQ_MODE_FORWARD, false, nullptr, 0, hip_stream), FQ_ERR_LAUNCH)
}

fq_status fq_backward(const fq_tensor *t, void *workspace, size_t ws_bytes, void *hip_stream)
{
    if (!t) return FQ_ERR_NULL;
    FQ_GUARDED(fq::run(t, 1, FQ_MODE_BACKWARD, false, workspace, ws_bytes, hip_stream), FQ_ERR_LAUNCH)
}

fq_status fq_backward_static(const fq_tensor *t, void *hip_stream)
{
    if (!t) return FQ_ERR_NULL;
    FQ_GUARDED(fq::run_static(*t, hip_stream), FQ_ERR_LAUNCH)
}

fq_status fq_multi_tensor(const fq_tensor *ts, int n, int mode, void *workspace, size_t ws_bytes,
                          void *hip_stream)
{
    FQ_GUARDED(fq::run(ts, n, mode, true, workspace, ws_bytes, hip_stream), FQ_ERR_LAUNCH)
}

fq_status fq_probe_stream(int inputs, const void *a, const void *b, void *out, size_t bytes, void *hip_stream)
{
    if (inputs < 0 || inputs > 2 || bytes % fq::kVecBytes != 0 || bytes / fq::kVecBytes / fq::kChunkVecs > 0x7ffffffeull)
        return FQ_ERR_SHAPE;
    if (inputs >= 1 && bytes > 0 && (!a || !out || (inputs == 2 && !b))) return FQ_ERR_NULL;
    if (!fq::aligned(a, fq::kVecBytes) || !fq::aligned(b, fq::kVecBytes) || !fq::aligned(out, fq::kVecBytes))
        return FQ_ERR_ALIGN;
    return fq::launch_probe(inputs, a, b, out, bytes, hip_stream) == 0 ? FQ_OK : FQ_ERR_LAUNCH;
}

struct fq_plan {
    fq::Prepared prepared;
    void *workspace = nullptr;
    std::vector<double> beta1, beta2;     // per tensor; unused where the tensor has no Adam step
    std::vector<char> has_adam;
    int64_t step = 0;                      // Adam step the device table currently holds
};

static fq_status fill_plan(fq_plan *p, const fq_tensor *ts, int n, int mode, void *workspace, size_t ws_bytes,
                           void *hip_stream)
{
    fq_status st = fq::prepare(ts, n, mode, true, workspace, ws_bytes, hip_stream, p->prepared);
    if (st != FQ_OK) return st;
    p->workspace = workspace;
    p->beta1.resize((size_t)n); p->beta2.resize((size_t)n); p->has_adam.resize((size_t)n);
    bool first = true;
    for (int i = 0; i < n; ++i) {
        const bool on = mode == FQ_MODE_BACKWARD && ts[i].adam && ts[i].channels > 0;
        p->has_adam[(size_t)i] = on ? 1 : 0;
        if (on) {
            p->beta1[(size_t)i] = ts[i].adam->beta1;
            p->beta2[(size_t)i] = ts[i].adam->beta2;
            // descriptors created at different steps: no single step is in place, so the first
            // fq_plan_run_adam refreshes every tensor
            if (first) p->step = ts[i].adam->step;
            else if (p->step != ts[i].adam->step) p->step = 0;
            first = false;
        }
    }
    return FQ_OK;
}

fq_status fq_plan_create(const fq_tensor *ts, int n, int mode, void *workspace, size_t ws_bytes,
                         void *hip_stream, fq_plan **plan)
{
    if (!plan) return FQ_ERR_NULL;
    *plan = nullptr;
    fq_plan *p = new (std::nothrow) fq_plan();
    if (!p) return FQ_ERR_LAUNCH;
    fq_status st;
    try {
        st = fill_plan(p, ts, n, mode, workspace, ws_bytes, hip_stream);
    } catch (...) {
        st = FQ_ERR_LAUNCH;
    }
    if (st != FQ_OK) {
        delete p;
        return st;
    }
    *plan = p;
    return FQ_OK;
}

fq_status fq_plan_run(const fq_plan *plan, void *hip_stream)
{
    if (!plan) return FQ_ERR_NULL;
    return fq::launch_prepared(plan->prepared, hip_stream);
}

fq_status fq_plan_run_adam(fq_plan *plan, int64_t step, void *hip_stream)
{
    if (!plan) return FQ_ERR_NULL;
    if (step < 1) return FQ_ERR_OPTIMIZER;
    // (no container grows here: the table and the per-tensor vectors keep their size)
    if (step != plan->step) {
        bool any = false;
        std::vector<fq::DevTensor> &table = plan->prepared.table;
        for (size_t i = 0; i < table.size(); ++i) {
            if (!plan->has_adam[i]) continue;
            any = true;
            table[i].adam_bc1 = (float)(1.0 - std::pow(plan->beta1[i], (double)step));
            table[i].adam_bc2 = (float)(1.0 - std::pow(plan->beta2[i], (double)step));
        }
        if (any && fq::copy_table_async(plan->workspace, table.data(), table.size() * sizeof(fq::DevTensor),
                                        hip_stream) != 0)
            return FQ_ERR_LAUNCH;
        plan->step = step;
    }
    return fq::launch_prepared(plan->prepared, hip_stream);
}

void fq_plan_destroy(fq_plan *plan) { delete plan; }

const char *fq_status_string(fq_status status)
{
    switch (status) {
    case FQ_OK: return "ok";
    case FQ_ERR_NULL: return "a required pointer is NULL";
    case FQ_ERR_DTYPE: return "dtype must be FQ_F16 or FQ_F32";
    case FQ_ERR_SHAPE: return "bad extent, count, n or mode";
    case FQ_ERR_QRANGE: return "bad integer code range";
    case FQ_ERR_ALIGN: return "pointer not aligned";
    case FQ_ERR_WORKSPACE: return "workspace missing or too small";
    case FQ_ERR_SCALE_PARAMS: return "bad eps / s_min / s_max";
    case FQ_ERR_LAUNCH: return "HIP runtime error while enqueuing";
    case FQ_ERR_ALIAS: return "output partially overlaps an input";
    case FQ_ERR_OPTIMIZER: return "bad Adam parameters";
    }
    return "unknown status";
}

}  // extern "C"
