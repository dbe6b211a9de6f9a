// Internal interface between the host-side planner (fq_api.cpp) and the gfx950 kernels
// (fq_kernels.hip).  Not part of the C ABI.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace fq {

constexpr int kBlock = 256;          // threads per block: four 64-wide wavefronts
constexpr int kVecBytes = 16;        // one 128-bit global load/store per lane
constexpr int kChunkVecs = 1280;     // at most this many 128-bit vectors per block (20 KiB)
constexpr int kWaveChunkVecs = kChunkVecs / (kBlock / 64);   // what one wavefront covers: 320 vectors
constexpr int kComputeUnits = 256;   // MI355X; used by the host to balance blocks over the chip
// A single-tensor backward launch of at most this many blocks has all of them resident at once
// (three per compute unit) and takes the schedule made for one burst (backward_chunk, SHORT).
constexpr unsigned kShortLaunchBlocks = 3 * kComputeUnits;
// Units of a channel beyond kTicketFanIn draw their arrival tickets in two levels: that many
// atomics on one address queue up at the memory-side atomic unit (60 units on one slot cost a
// short-slab backward 17.4 us against 13.1 us with 16 first-level slots).
constexpr unsigned kTicketFanIn = 16;
constexpr unsigned kTicketSubSlots = 16;       // first-level slots per channel
constexpr unsigned kTicketManyUnits = 256;     // beyond this many units per channel ...
constexpr unsigned kTicketManySubSlots = 32;   // ... this many first-level slots
constexpr unsigned kTreeBlocks = 4;      // up to this many blocks per channel combine by atomic exchange alone

// Scratch memory built into the library for fq_backward_static: [slots][partial sums].
constexpr size_t kStaticScratchBytes = 1u << 20;                 // per GPU
constexpr size_t kStaticSlotBytes = 256u << 10;                  // 32768 64-bit slots
constexpr size_t kStaticPartialBytes = kStaticScratchBytes - kStaticSlotBytes;   // 98304 partial sums

// Device-side view of one tensor.  Built on the host; passed as a kernel argument for
// single-tensor calls, or as an array in device memory for the multi-tensor launch.
struct DevTensor {
    const void *x;
    void *y;
    int8_t *q;
    const float *theta;
    float *s;
    const void *gy;
    void *gx;
    float *gs;
    float *gtheta;
    double *partial;           // [slabs * cps] per-block partial sums of gy*t (backward)
    unsigned long long *slot;  // [channels] exchange slot / arrival tickets, then [channels][sub] first-level
                               // tickets; all zero between calls (backward)
    long long inner;           // elements per slab
    unsigned slabs;            // outer * channels
    unsigned channels;
    unsigned outer;
    unsigned cps;              // chunks per slab
    unsigned chunk;            // elements per chunk, a multiple of the vector width
    unsigned block_begin;      // first block of this tensor in the grid
    unsigned chan_begin;       // first channel of this tensor in the finalize grid
    unsigned wave_units;       // 1: slabs are short, every wavefront owns one (cps = 1, chunk = the slab);
                               // the tensor's blocks then number ceil(slabs / 4) and partial[] is per slab
    unsigned grid3;            // 1: launched alone with a grid of (cps, channels, outer) blocks (see own_chunk)
    unsigned sub;              // extra slots per channel after the [channels] main ones: 0, 2 (pair slots of
                               // the exchange tree, 3 or 4 blocks per channel) or kTicketSubSlots
    int dtype;                 // 0 = FP16, 1 = FP32
    float lo, hi;              // (float)qmin, (float)qmax
    float eps, s_min, s_max;
    unsigned flags;
    // fused Adam step on theta (backward); adam_m == nullptr: none
    float *adam_m, *adam_v, *adam_theta_out;
    float adam_lr, adam_beta1, adam_one_minus_beta1, adam_beta2, adam_one_minus_beta2, adam_eps;
    float adam_bc1, adam_bc2;      // 1 - beta1^t, 1 - beta2^t
};

struct KArgs {
    DevTensor one;             // used when table == nullptr
    const DevTensor *table;    // device array of n descriptors (multi-tensor launch)
    int n;
};

// Launchers; each returns the hipError_t value as int (0 = success).
int launch_forward(const KArgs &a, unsigned blocks, bool emit_q, void *stream);
int launch_backward(const KArgs &a, unsigned blocks, bool fused_finalize, void *stream);
int launch_finalize(const KArgs &a, unsigned total_channels, void *stream);
int launch_scale_only(const KArgs &a, unsigned total_channels, void *stream);
int launch_fill_zero(void *p, size_t bytes, void *stream);
int copy_table_async(void *dst_device, const void *src_host, size_t bytes, void *stream);
int static_scratch(void **ptr, void *stream);
int launch_probe(int inputs, const void *a, const void *b, void *out, size_t bytes, void *stream);

}  // namespace fq
