// Distillation loss between a student and a teacher feature map and its gradient with respect to
// the student (DPVO-QAT++ Sec. 3.2, Eq. (7): MSE plus lambda times one minus the cosine
// similarity over the channel axis, averaged over positions).  This is the producer of the
// upstream gradient that the fake-quantization backward consumes.
//
// [N, C, M] tensors; a "position" is one (n, m).  The reduction runs ACROSS the channel axis, whose
// stride is M elements, so the layout is read the way it lies in memory, without transposition and
// without atomics.  Two ways, chosen on the host:
//
// One read of the pair (fused kernel; channel counts up to 512, M a multiple of 4): a block owns a
// tile of all channels x one 128-byte run of positions (64 FP16 or 32 FP32 positions); a lane holds
// 4 consecutive positions of up to 16 channels IN REGISTERS, adds its four sums (a.b, a.a, b.b,
// (a-b)^2) per position, the block adds the lanes' sums through LDS in a fixed order, forms cos and
// the two gradient coefficients per position, and every lane then writes the gradient of the
// elements it still holds.  HBM traffic: read a, read b, write ga -- the algorithmic 3 bytes-widths
// per element.
//
// Two reads (any shape): a wavefront owns 64 lanes x V consecutive positions (one coalesced row per
// channel) and walks over a group of channels, every lane keeping the four sums of its V positions
// in binary64 registers:
//   stats kernel   one block per position tile, one wavefront per channel group (up to 16); the
//                  wavefronts add their sums through LDS in a fixed tree, then the block forms
//                  cos and the two coefficients of the gradient for its positions and leaves
//                  its sums of cos and of the squared error
//   grad kernel    elementwise: ga = k1 (a - b) - cB b + cA a, rounded once to the I/O type
// In both, the last small step adds the per-block sums in index order into the 3 results.
// All arithmetic is binary64 (two conversions and five fused multiply-adds per element pair, well
// under the memory time), so results do not depend on how the channels were grouped beyond
// rounding at the 1e-16 level, and are reproducible run to run.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/fq.h"
#include "fq_device.h"
#include "fq_internal.h"

namespace fq {

using namespace dev;

namespace {

constexpr int kThreads = 256;             // gradient kernel
constexpr int kWaves = kThreads / 64;
constexpr int kUnrollC = 8;               // channels in flight per wavefront (two loads each)
constexpr unsigned kTargetWaves = 2048;   // eight wavefronts per compute unit
constexpr unsigned kMaxGroups = 16;       // wavefronts of a statistics block (1024 threads)
constexpr unsigned kTreeSlots = 4;        // wavefronts that hand their sums over per round of the LDS tree
constexpr int kMaxVec = 4;                // positions per lane (a 1024-thread block has 128 VGPRs per lane)
constexpr long long kMinTiles = 256;      // prefer this many position tiles before narrowing the loads

struct DistillArgs {
    const void *a, *b;
    void *ga;
    double *coef;       // [positions][2]
    double *blocksum;   // [tiles][2]: per-block sums of cos and of (a-b)^2
    double *out;        // mse, cosim, loss
    long long M, P;     // positions per image, positions in total
    unsigned C, groups, per_group, tiles_per_n, tiles;
    double k1u, k2u, eps, lambda, inv_ncm, inv_nm;
};

template <typename T, int V> struct Pack {
    typedef T type __attribute__((ext_vector_type(V)));
    static __device__ __forceinline__ T get(const type &v, int i) { return v[i]; }
    static __device__ __forceinline__ void set(type &v, int i, T x) { v[i] = x; }
};
template <typename T> struct Pack<T, 1> {
    typedef T type;
    static __device__ __forceinline__ T get(const type &v, int) { return v; }
    static __device__ __forceinline__ void set(type &v, int, T x) { v = x; }
};

typedef double double2v __attribute__((ext_vector_type(2)));

// Which tile / channel group a wavefront works on, and where its lane's V positions start.
struct Where {
    bool active, valid;
    unsigned c0, c1;
    long long first;   // element offset of (n, c0, m0)
    long long p0;      // position index of the lane's first position
};

template <int V>
__device__ __forceinline__ Where locate(const DistillArgs &k, unsigned groups, unsigned per_group)
{
    Where w;
    const unsigned wid = blockIdx.x * kWaves + (threadIdx.x >> 6);
    w.active = wid < k.tiles * groups;
    const unsigned tile = w.active ? wid / groups : 0u;
    const unsigned g = w.active ? wid % groups : 0u;
    const unsigned n = tile / k.tiles_per_n;
    const unsigned tn = tile - n * k.tiles_per_n;
    long long m0 = ((long long)tn * 64 + (threadIdx.x & 63)) * V;
    w.valid = w.active && m0 < k.M;
    if (m0 >= k.M) m0 = k.M - V;            // lanes past the end re-read the last vector; results dropped
    w.c0 = g * per_group;
    w.c1 = w.c0 + per_group < k.C ? w.c0 + per_group : k.C;
    if (w.c0 > w.c1) w.c0 = w.c1;
    w.first = ((long long)n * k.C + w.c0) * k.M + m0;
    w.p0 = (long long)n * k.M + m0;
    return w;
}

// Sums of `u` and `v` over the block (any number of wavefronts up to 16) in a fixed order; valid
// in thread 0.  red: 32 doubles of LDS.
__device__ __forceinline__ void block_sum2(double &u, double &v, double *red)
{
    u = wave_sum(u);
    v = wave_sum(v);
    if ((threadIdx.x & 63) == kSumLane) {
        red[threadIdx.x >> 6] = u;
        red[16 + (threadIdx.x >> 6)] = v;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned waves = blockDim.x >> 6;
        u = v = 0.0;
        for (unsigned i = 0; i < waves; ++i) {
            u += red[i];
            v += red[16 + i];
        }
    }
}

// One block = one position tile; wavefront w takes channel group w.  Loads roll: as soon as a
// channel's pair of vectors has been consumed its registers are refilled with the channel
// kUnrollC further on, so 2 x kUnrollC loads stay in flight while the binary64 arithmetic runs.
// Dynamic LDS: min(kTreeSlots, max(1, p/2)) x 4V x 64 doubles, p = the number of wavefronts
// rounded up to a power of two.
template <typename T, int V>
__global__ __launch_bounds__(1024) void distill_stats_kernel(DistillArgs k)
{
    typedef typename Pack<T, V>::type VT;
    constexpr int U = V >= 4 ? kUnrollC : 2 * kUnrollC;   // narrow loads: more of them in flight
    constexpr int ES = V * 4;                         // sums per lane
    extern __shared__ double lds[];                   // [slot][ES][64]
    __shared__ double red[32];

    const unsigned wave = threadIdx.x >> 6, lane = threadIdx.x & 63, waves = blockDim.x >> 6;
    const unsigned tile = blockIdx.x;
    const unsigned n = tile / k.tiles_per_n, tn = tile - n * k.tiles_per_n;
    const long long tile_m = (long long)tn * 64 * V;  // first position of the tile in its image
    long long m0 = tile_m + (long long)lane * V;
    if (m0 >= k.M) m0 = k.M - V;                      // lanes past the end re-read the last vector
    const unsigned c0 = wave * k.per_group < k.C ? wave * k.per_group : k.C;
    const unsigned c1 = c0 + k.per_group < k.C ? c0 + k.per_group : k.C;
    const unsigned nch = c1 - c0;                     // 0 for a wavefront without a group
    const long long first = ((long long)n * k.C + (nch ? c0 : 0u)) * k.M + m0;
    const T *a = (const T *)k.a + first;
    const T *b = (const T *)k.b + first;

    double acc[ES];
#pragma unroll
    for (int i = 0; i < ES; ++i) acc[i] = 0.0;
    auto accumulate = [&](const VT &va, const VT &vb) {
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const double x = (double)(float)Pack<T, V>::get(va, e);
            const double y = (double)(float)Pack<T, V>::get(vb, e);
            const double d = x - y;
            acc[e * 4 + 0] = __builtin_fma(x, y, acc[e * 4 + 0]);
            acc[e * 4 + 1] = __builtin_fma(x, x, acc[e * 4 + 1]);
            acc[e * 4 + 2] = __builtin_fma(y, y, acc[e * 4 + 2]);
            acc[e * 4 + 3] = __builtin_fma(d, d, acc[e * 4 + 3]);
        }
    };

    if (nch) {
        VT ra[U], rb[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned cu = (unsigned)u < nch ? (unsigned)u : nch - 1;
            ra[u] = ld_global((const VT *)(a + (long long)cu * k.M));
            rb[u] = ld_global((const VT *)(b + (long long)cu * k.M));
        }
        unsigned c = 0;
        for (; c + U < nch; c += U) {                 // a next block exists, at least in part
#pragma unroll
            for (int u = 0; u < U; ++u) {
                accumulate(ra[u], rb[u]);
                unsigned nc = c + U + u;
                if (nc >= nch) nc = nch - 1;          // re-read of the last channel, never used
                ra[u] = ld_global((const VT *)(a + (long long)nc * k.M));
                rb[u] = ld_global((const VT *)(b + (long long)nc * k.M));
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (c + u < nch) accumulate(ra[u], rb[u]);
    }

    // Fixed tree over the wavefronts: w += w + stride for stride = 8, 4, 2, 1, at most kTreeSlots
    // wavefronts handing over per round so that the LDS footprint stays at 4 x 4V x 64 doubles.
    for (unsigned stride = kMaxGroups / 2; stride >= 1; stride >>= 1) {
        if (stride >= waves) continue;                // uniform over the block
        for (unsigned base = 0; base < stride; base += kTreeSlots) {
            const unsigned giver = stride + base;     // first wavefront that hands over in this round
            if (wave >= giver && wave < giver + kTreeSlots && wave < 2 * stride) {
#pragma unroll
                for (int i = 0; i < ES; ++i) lds[((wave - giver) * ES + i) * 64 + lane] = acc[i];
            }
            __syncthreads();
            if (wave >= base && wave < base + kTreeSlots && wave < stride && wave + stride < waves) {
#pragma unroll
                for (int i = 0; i < ES; ++i) acc[i] += lds[((wave - base) * ES + i) * 64 + lane];
            }
            __syncthreads();
        }
    }
    if (wave == 0) {
#pragma unroll
        for (int i = 0; i < ES; ++i) lds[i * 64 + lane] = acc[i];
    }
    __syncthreads();

    // One thread per position of the tile: cos, the coefficients of the gradient, block sums.
    double cos_sum = 0.0, sq_sum = 0.0;
    for (unsigned pp = threadIdx.x; pp < 64u * V; pp += blockDim.x) {
        const unsigned src = pp / V, e = pp % V;
        const long long m = tile_m + pp;
        if (m < k.M) {
            const double dot = lds[(e * 4 + 0) * 64 + src], na = lds[(e * 4 + 1) * 64 + src];
            const double nb = lds[(e * 4 + 2) * 64 + src], sq = lds[(e * 4 + 3) * 64 + src];
            const double ra = sqrt(na), rb = sqrt(nb);
            // a NaN norm stays NaN, so a non-finite input poisons its whole position visibly
            const double ca = ra < k.eps ? k.eps : ra, cb = rb < k.eps ? k.eps : rb;
            const double inv = 1.0 / (ca * cb);
            const double cosp = dot / (ca * cb);
            const double self = ra > k.eps ? cosp / na : 0.0;
            if (k.coef) {
                double2v o = {k.k2u * inv, k.k2u * self};
                st_global((double2v *)k.coef + ((long long)n * k.M + m), o);
            }
            cos_sum += cosp;
            sq_sum += sq;
        }
    }
    block_sum2(cos_sum, sq_sum, red);
    if (threadIdx.x == 0) {
        double2v o = {cos_sum, sq_sum};
        st_global((double2v *)k.blocksum + tile, o);
    }
}

// The three results from the per-block sums, added in a fixed order by one wavefront: lane l takes
// the sums l, l + 64, l + 128, ... (eight loads in flight at a time: thousands of tiles would
// otherwise be as many dependent round trips to memory), then the lanes are added by wave_sum.
__device__ __forceinline__ void finish(const DistillArgs &k)
{
    const unsigned lane = threadIdx.x & 63;
    double sc = 0.0, ss = 0.0;
    constexpr unsigned kBatch = 8;
    for (unsigned i0 = lane; i0 < k.tiles; i0 += 64 * kBatch) {
        double2v v[kBatch];
#pragma unroll
        for (unsigned j = 0; j < kBatch; ++j) {
            const unsigned i = i0 + 64 * j;
            v[j] = double2v{0.0, 0.0};
            if (i < k.tiles) v[j] = ld_global((const double2v *)k.blocksum + i);
        }
#pragma unroll
        for (unsigned j = 0; j < kBatch; ++j) {
            if (i0 + 64 * j < k.tiles) {
                sc += v[j][0];
                ss += v[j][1];
            }
        }
    }
    sc = wave_sum(sc);
    ss = wave_sum(ss);
    if (lane == kSumLane) {
        const double mse = ss * k.inv_ncm, cosim = sc * k.inv_nm;
        st_global(k.out + 0, mse);
        st_global(k.out + 1, cosim);
        st_global(k.out + 2, mse + k.lambda * (1.0 - cosim));
    }
}

// The same as a kernel of its own, by one block of 1024 threads: thread t takes the sums t,
// t + 1024, ..., the wavefronts add their lanes (wave_sum), thread 0 adds the sixteen wavefront
// sums in index order.
__global__ __launch_bounds__(1024) void distill_finish_kernel(DistillArgs k)
{
    __shared__ double part[2 * 16];
    double sc = 0.0, ss = 0.0;
    constexpr unsigned kBatch = 4;
    for (unsigned i0 = threadIdx.x; i0 < k.tiles; i0 += 1024 * kBatch) {
        double2v v[kBatch];
#pragma unroll
        for (unsigned j = 0; j < kBatch; ++j) {
            const unsigned i = i0 + 1024 * j;
            v[j] = double2v{0.0, 0.0};
            if (i < k.tiles) v[j] = ld_global((const double2v *)k.blocksum + i);
        }
#pragma unroll
        for (unsigned j = 0; j < kBatch; ++j) {
            if (i0 + 1024 * j < k.tiles) {
                sc += v[j][0];
                ss += v[j][1];
            }
        }
    }
    sc = wave_sum(sc);
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == kSumLane) {
        part[threadIdx.x >> 6] = sc;
        part[16 + (threadIdx.x >> 6)] = ss;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        sc = ss = 0.0;
        for (unsigned w = 0; w < 16; ++w) {
            sc += part[w];
            ss += part[16 + w];
        }
        const double mse = ss * k.inv_ncm, cosim = sc * k.inv_nm;
        st_global(k.out + 0, mse);
        st_global(k.out + 1, cosim);
        st_global(k.out + 2, mse + k.lambda * (1.0 - cosim));
    }
}

template <typename T, int V>
__global__ __launch_bounds__(kThreads) void distill_grad_kernel(DistillArgs k, unsigned groups, unsigned per_group)
{
    typedef typename Pack<T, V>::type VT;
    if (blockIdx.x == 0 && threadIdx.x < 64) finish(k);
    const Where w = locate<V>(k, groups, per_group);
    if (!w.active) return;
    const T *a = (const T *)k.a + w.first;
    const T *b = (const T *)k.b + w.first;
    T *ga = (T *)k.ga + w.first;
    double cb[V], ca[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
        const double2v v = ld_global((const double2v *)k.coef + w.p0 + e);
        cb[e] = v[0];
        ca[e] = v[1];
    }
    auto grad = [&](const VT &va, const VT &vb) {
        VT o;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const double x = (double)(float)Pack<T, V>::get(va, e);
            const double y = (double)(float)Pack<T, V>::get(vb, e);
            double g = k.k1u * (x - y);
            g = __builtin_fma(-cb[e], y, g);
            g = __builtin_fma(ca[e], x, g);
            Pack<T, V>::set(o, e, (T)(float)g);
        }
        return o;
    };
    constexpr int U = kUnrollC / 2;
    unsigned c = w.c0;
    for (; c + U <= w.c1; c += U) {
        VT ra[U], rb[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            ra[u] = ld_stream((const VT *)(a + (long long)u * k.M));
            rb[u] = ld_stream((const VT *)(b + (long long)u * k.M));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const VT o = grad(ra[u], rb[u]);
            if (w.valid) st_stream((VT *)(ga + (long long)u * k.M), o);
        }
        a += (long long)U * k.M;
        b += (long long)U * k.M;
        ga += (long long)U * k.M;
    }
    for (; c < w.c1; ++c) {
        const VT o = grad(ld_stream((const VT *)a), ld_stream((const VT *)b));
        if (w.valid) st_stream((VT *)ga, o);
        a += k.M;
        b += k.M;
        ga += k.M;
    }
}

// ---------------------------------------------------------------------------------------------
// One read of the pair.  Block: kFusedThreads threads = R rows of L lanes; lane l of row r holds
// positions 4l .. 4l+3 of the tile for channels r, r + R, r + 2R, ... (KCH of them at most).
constexpr int kFusedThreads = 512;
constexpr int kFusedVec = 4;                     // positions per lane
constexpr int kFusedMaxKch = 16;                 // channels per lane the registers hold (FP16; half for FP32)
// A tile's rows are 128 bytes of each channel, a whole cache line.  (Rows of 64 bytes would cut a
// 1x384x120x160 pair into 600 tiles instead of 300 and spread them more evenly over the 256
// compute units, but half-line accesses cost more than the balance gains: 24.4 us against 16.9.)
template <typename T> struct FusedShape {
    static constexpr int L = 128 / (kFusedVec * (int)sizeof(T));   // lanes per row: 16 (FP16), 8 (FP32)
    static constexpr int P = kFusedVec * L;                        // positions per tile: 64 / 32
    static constexpr int R = kFusedThreads / L;                    // channel rows: 32 / 64
};

template <typename T, int KCH, bool WANT_GRAD>
__global__ __launch_bounds__(kFusedThreads, 4) void distill_fused_kernel(DistillArgs k)
{
    typedef FusedShape<T> Shape;
    constexpr int V = kFusedVec, L = Shape::L, P = Shape::P, R = Shape::R;
    typedef typename Pack<T, V>::type VT;
    __shared__ double red[8 * kFusedThreads];     // half of the lanes' sums at a time: [value][thread]
    __shared__ double stat[P * 4];                // per position: a.b, a.a, b.b, (a-b)^2
    __shared__ double coefs[P * 2];               // per position: the two gradient coefficients

    const unsigned lane = threadIdx.x % L, row = threadIdx.x / L;
    const unsigned tile = blockIdx.x;
    const unsigned n = tile / k.tiles_per_n, tn = tile - n * k.tiles_per_n;
    const long long tile_m = (long long)tn * P;
    long long m0 = tile_m + (long long)lane * V;
    const bool lane_valid = m0 < k.M;
    if (!lane_valid) m0 = k.M - V;                // lanes past the end re-read the last quad; results dropped
    const long long base = (long long)n * k.C * k.M + m0;
    const T *a = (const T *)k.a + base;
    const T *b = (const T *)k.b + base;

    VT ra[KCH], rb[KCH];
#pragma unroll
    for (int j = 0; j < KCH; ++j) {
        unsigned c = row + (unsigned)j * R;
        c = c < k.C ? c : k.C - 1;                // rows past the last channel re-read it; results dropped
        ra[j] = ld_stream((const VT *)(a + (long long)c * k.M));
        rb[j] = ld_stream((const VT *)(b + (long long)c * k.M));
    }

    double acc[V * 4];
#pragma unroll
    for (int i = 0; i < V * 4; ++i) acc[i] = 0.0;
#pragma unroll
    for (int j = 0; j < KCH; ++j) {
        if (row + (unsigned)j * R < k.C) {
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const double x = (double)(float)ra[j][e];
                const double y = (double)(float)rb[j][e];
                const double d = x - y;
                acc[e * 4 + 0] = __builtin_fma(x, y, acc[e * 4 + 0]);
                acc[e * 4 + 1] = __builtin_fma(x, x, acc[e * 4 + 1]);
                acc[e * 4 + 2] = __builtin_fma(y, y, acc[e * 4 + 2]);
                acc[e * 4 + 3] = __builtin_fma(d, d, acc[e * 4 + 3]);
            }
        }
    }

    // Sum over the R rows, in row order, eight of the sixteen values at a time.
#pragma unroll
    for (int half = 0; half < 2; ++half) {
#pragma unroll
        for (int i = 0; i < 8; ++i) red[i * kFusedThreads + threadIdx.x] = acc[half * 8 + i];
        __syncthreads();
        if (threadIdx.x < 8 * L) {
            const unsigned i = threadIdx.x / L, l = threadIdx.x % L;
            double sum = 0.0;
            for (unsigned r = 0; r < (unsigned)R; ++r) sum += red[i * kFusedThreads + r * L + l];
            const unsigned value = half * 8 + i;                 // = e * 4 + which sum
            stat[(l * V + value / 4) * 4 + value % 4] = sum;
        }
        __syncthreads();
    }

    // One thread per position (all in the first wavefront): cos, the gradient's coefficients, and
    // the tile's sums of cos and of the squared error.
    if (threadIdx.x < 64) {
        double cos_sum = 0.0, sq_sum = 0.0;
        const unsigned pp = threadIdx.x;
        if (pp < (unsigned)P && tile_m + pp < k.M) {
            const double dot = stat[pp * 4 + 0], na = stat[pp * 4 + 1], nb = stat[pp * 4 + 2];
            const double ra_ = sqrt(na), rb_ = sqrt(nb);
            // a NaN norm stays NaN, so a non-finite input poisons its whole position visibly
            const double ca = ra_ < k.eps ? k.eps : ra_, cb = rb_ < k.eps ? k.eps : rb_;
            const double inv = 1.0 / (ca * cb);
            const double cosp = dot / (ca * cb);
            const double self = ra_ > k.eps ? cosp / na : 0.0;
            coefs[pp * 2 + 0] = k.k2u * inv;
            coefs[pp * 2 + 1] = k.k2u * self;
            cos_sum = cosp;
            sq_sum = stat[pp * 4 + 3];
        }
        cos_sum = wave_sum(cos_sum);
        sq_sum = wave_sum(sq_sum);
        if (threadIdx.x == kSumLane) {
            double2v o = {cos_sum, sq_sum};
            st_global((double2v *)k.blocksum + tile, o);
        }
    }
    if (!WANT_GRAD) return;
    __syncthreads();

    if (!lane_valid) return;
    double cb[V], ca[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
        cb[e] = coefs[(lane * V + e) * 2 + 0];
        ca[e] = coefs[(lane * V + e) * 2 + 1];
    }
    T *ga = (T *)k.ga + base;
#pragma unroll
    for (int j = 0; j < KCH; ++j) {
        const unsigned c = row + (unsigned)j * R;
        if (c < k.C) {
            VT o;
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const double x = (double)(float)ra[j][e];
                const double y = (double)(float)rb[j][e];
                double g = k.k1u * (x - y);
                g = __builtin_fma(-cb[e], y, g);
                g = __builtin_fma(ca[e], x, g);
                o[e] = (T)(float)g;
            }
            st_stream((VT *)(ga + (long long)c * k.M), o);
        }
    }
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct Plan {
    int vec;                 // elements per lane
    int fused_kch;           // > 0: the fused kernel with this many channels per lane; 0: two kernels
    unsigned tiles_per_n, tiles, groups, per_group, grad_groups, grad_per_group;
    size_t stats_lds, off_blocksum, bytes;
};

// Channels per lane the fused kernel would need for this pair, rounded up to a width it is built
// for; 0 if the pair does not qualify (positions not in whole quads, a pointer off the quad's
// alignment, or more channels than a lane's registers hold).
int fused_channels_per_lane(const fq_distill *d)
{
    const size_t esz = d->dtype == FQ_F16 ? 2 : 4;
    const uintptr_t addr_bits = (uintptr_t)d->student | (uintptr_t)d->teacher | (uintptr_t)d->gstudent;
    if (d->inner % kFusedVec || addr_bits % (kFusedVec * esz)) return 0;
    const long long rows = d->dtype == FQ_F16 ? FusedShape<_Float16>::R : FusedShape<float>::R;
    const long long need = (d->channels + rows - 1) / rows;
    const long long cap = d->dtype == FQ_F16 ? kFusedMaxKch : kFusedMaxKch / 2;
    if (need > cap) return 0;
    for (int kch : {2, 4, 6, 8, 12, 16})
        if (kch >= need) return kch;
    return 0;
}

fq_status make_plan(const fq_distill *d, Plan &pl)
{
    if (!d) return FQ_ERR_NULL;
    if (d->dtype != FQ_F16 && d->dtype != FQ_F32) return FQ_ERR_DTYPE;
    if (d->n < 0 || d->channels < 0 || d->inner < 0) return FQ_ERR_SHAPE;
    const size_t esz = d->dtype == FQ_F16 ? 2 : 4;
    // positions index 32-bit grids of 64-lane tiles; the element count must fit in 62 bits
    if (d->n > 0 && d->inner > (long long)0x7fffffff / d->n) return FQ_ERR_SHAPE;
    const long long P = d->n * d->inner;
    if (d->channels > 0x7fffffff) return FQ_ERR_SHAPE;
    if (P > 0 && d->channels > ((long long)1 << 60) / P) return FQ_ERR_SHAPE;
    if (!(d->lambda == d->lambda) || !(d->upstream == d->upstream) || !(d->eps >= 0.0f)) return FQ_ERR_SCALE_PARAMS;
    if (!d->out) return FQ_ERR_NULL;
    if ((uintptr_t)d->out % sizeof(double)) return FQ_ERR_ALIGN;
    const bool empty = P == 0 || d->channels == 0;
    if (!empty) {
        if (!d->student || !d->teacher) return FQ_ERR_NULL;
        if ((uintptr_t)d->student % esz || (uintptr_t)d->teacher % esz || (uintptr_t)d->gstudent % esz)
            return FQ_ERR_ALIGN;
        if (d->gstudent) {
            // exact in-place over the student is fine (each element is read before it is written
            // by the same lane); any other overlap is not
            const char *g0 = (const char *)d->gstudent, *g1 = g0 + (size_t)P * d->channels * esz;
            const void *ins[2] = {d->student, d->teacher};
            for (const void *in : ins) {
                const char *i0 = (const char *)in, *i1 = i0 + (size_t)P * d->channels * esz;
                if (g0 != i0 && g0 < i1 && i0 < g1) return FQ_ERR_ALIAS;
            }
        }
    }
    if (empty) {
        pl = Plan{};
        pl.vec = 1;
        pl.bytes = 256;
        return FQ_OK;
    }
    pl.fused_kch = fused_channels_per_lane(d);
    if (pl.fused_kch) {
        const long long per_tile = d->dtype == FQ_F16 ? FusedShape<_Float16>::P : FusedShape<float>::P;
        const long long tpn = (d->inner + per_tile - 1) / per_tile;
        if (tpn * d->n > 0x3fffffffLL) return FQ_ERR_SHAPE;
        pl.vec = kFusedVec;
        pl.tiles_per_n = (unsigned)tpn;
        pl.tiles = (unsigned)(tpn * d->n);
        pl.groups = pl.per_group = pl.grad_groups = pl.grad_per_group = 0;
        pl.stats_lds = 0;
        pl.off_blocksum = 0;                       // no per-position coefficients leave the block
        pl.bytes = align256((size_t)pl.tiles * 2 * sizeof(double));
        if (pl.bytes < 256) pl.bytes = 256;
        return FQ_OK;
    }
    const int full = (int)(kVecBytes / esz) < kMaxVec ? (int)(kVecBytes / esz) : kMaxVec;
    // Elements per lane: the widest load whose tiles (64 lanes x vec positions) are still many
    // enough to fill the chip without splitting the channels into many groups; a narrow load
    // still covers whole cache lines (64 lanes x 4 bytes = two lines).
    const uintptr_t addr_bits = (uintptr_t)d->student | (uintptr_t)d->teacher | (uintptr_t)d->gstudent;
    pl.vec = 1;
    for (int v = full; v > 1; v /= 2) {
        if (d->inner % v || addr_bits % (v * esz)) continue;
        pl.vec = v;
        if (d->n * ((d->inner + 64LL * v - 1) / (64LL * v)) >= kMinTiles) break;
    }
    const long long per_tile = 64LL * pl.vec;
    const long long tpn = empty ? 0 : (d->inner + per_tile - 1) / per_tile;
    if (tpn * d->n > 0x3fffffffLL) return FQ_ERR_SHAPE;
    pl.tiles_per_n = (unsigned)tpn;
    pl.tiles = (unsigned)(tpn * d->n);
    auto split = [&](unsigned want_waves, unsigned cap, unsigned &groups, unsigned &per_group) {
        unsigned g = pl.tiles ? (want_waves + pl.tiles - 1) / pl.tiles : 1u;
        if (g > cap) g = cap;
        if (g > (unsigned)d->channels) g = (unsigned)d->channels;
        if (g < 1u) g = 1u;
        per_group = empty ? 0u : ((unsigned)d->channels + g - 1) / g;
        groups = per_group ? ((unsigned)d->channels + per_group - 1) / per_group : 1u;
    };
    split(kTargetWaves, kMaxGroups, pl.groups, pl.per_group);
    split(2 * kTargetWaves, 1024u, pl.grad_groups, pl.grad_per_group);
    if ((unsigned long long)pl.tiles * pl.grad_groups > 0x3fffffffULL) {
        pl.grad_groups = pl.groups;
        pl.grad_per_group = pl.per_group;
    }
    unsigned pow2 = 1;
    while (pow2 < pl.groups) pow2 *= 2;
    unsigned slots = pow2 > 1 ? pow2 / 2 : 1;
    if (slots > kTreeSlots) slots = kTreeSlots;
    pl.stats_lds = (size_t)slots * 4 * pl.vec * 64 * sizeof(double);
    const size_t coef = align256((size_t)P * 2 * sizeof(double));
    const size_t blocksum = align256((size_t)pl.tiles * 2 * sizeof(double));
    pl.off_blocksum = coef;
    pl.bytes = coef + blocksum;
    if (pl.bytes < 256) pl.bytes = 256;
    return FQ_OK;
}

__global__ void distill_empty_kernel(double *out, bool has_positions)
{
    // a mean over no elements is 0/0; positions without channels have cos = 0 / eps^2 = 0
    const double nan = __builtin_nan("");
    out[0] = nan;
    out[1] = has_positions ? 0.0 : nan;
    out[2] = nan;
}

template <typename T, int V>
fq_status launch(const DistillArgs &k, const Plan &pl, bool want_grad, hipStream_t st)
{
    distill_stats_kernel<T, V><<<pl.tiles, 64 * pl.groups, pl.stats_lds, st>>>(k);
    if (want_grad) {
        const unsigned grad_blocks = (pl.tiles * pl.grad_groups + kWaves - 1) / kWaves;
        distill_grad_kernel<T, V><<<grad_blocks, kThreads, 0, st>>>(k, pl.grad_groups, pl.grad_per_group);
    } else {
        distill_finish_kernel<<<1, 1024, 0, st>>>(k);
    }
    return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_LAUNCH;
}

template <typename T, int KCH>
fq_status launch_fused(const DistillArgs &k, const Plan &pl, bool want_grad, hipStream_t st)
{
    if (want_grad) distill_fused_kernel<T, KCH, true><<<pl.tiles, kFusedThreads, 0, st>>>(k);
    else distill_fused_kernel<T, KCH, false><<<pl.tiles, kFusedThreads, 0, st>>>(k);
    distill_finish_kernel<<<1, 1024, 0, st>>>(k);
    return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_LAUNCH;
}

template <typename T>
fq_status launch_fused_width(const DistillArgs &k, const Plan &pl, bool want_grad, hipStream_t st)
{
    switch (pl.fused_kch) {
    case 2: return launch_fused<T, 2>(k, pl, want_grad, st);
    case 4: return launch_fused<T, 4>(k, pl, want_grad, st);
    case 6: return launch_fused<T, 6>(k, pl, want_grad, st);
    case 8: return launch_fused<T, 8>(k, pl, want_grad, st);
    default: break;
    }
    if (sizeof(T) == 2 && pl.fused_kch == 12) return launch_fused<_Float16, 12>(k, pl, want_grad, st);
    if (sizeof(T) == 2 && pl.fused_kch == 16) return launch_fused<_Float16, 16>(k, pl, want_grad, st);
    return FQ_ERR_SHAPE;                           // not reached: make_plan offers only the widths above
}

}  // namespace
}  // namespace fq

extern "C" {

int fq_distill_reads_of_pair(const fq_distill *d)
{
    fq::Plan pl;
    if (fq::make_plan(d, pl) != FQ_OK) return 0;
    if (d->n * d->inner == 0 || d->channels == 0) return 0;
    return pl.fused_kch ? 1 : (d->gstudent ? 2 : 1);
}

size_t fq_distill_workspace_bytes(const fq_distill *d)
{
    fq::Plan pl;
    return fq::make_plan(d, pl) == FQ_OK ? pl.bytes : 0;
}

fq_status fq_distill_loss(const fq_distill *d, void *workspace, size_t ws_bytes, void *hip_stream)
{
    using namespace fq;
    Plan pl;
    const fq_status v = make_plan(d, pl);
    if (v != FQ_OK) return v;
    hipStream_t st = (hipStream_t)hip_stream;
    if (d->n * d->inner == 0 || d->channels == 0) {
        distill_empty_kernel<<<1, 1, 0, st>>>(d->out, d->n * d->inner != 0);
        return hipGetLastError() == hipSuccess ? FQ_OK : FQ_ERR_LAUNCH;
    }
    if (!workspace || ws_bytes < pl.bytes) return FQ_ERR_WORKSPACE;
    if ((uintptr_t)workspace % 256) return FQ_ERR_ALIGN;

    DistillArgs k;
    k.a = d->student;
    k.b = d->teacher;
    k.ga = d->gstudent;
    k.coef = d->gstudent ? (double *)workspace : nullptr;
    k.blocksum = (double *)((char *)workspace + pl.off_blocksum);
    k.out = d->out;
    k.M = d->inner;
    k.P = d->n * d->inner;
    k.C = (unsigned)d->channels;
    k.groups = pl.groups;
    k.per_group = pl.per_group;
    k.tiles_per_n = pl.tiles_per_n;
    k.tiles = pl.tiles;
    const double ncm = (double)d->n * (double)d->channels * (double)d->inner;
    const double nm = (double)d->n * (double)d->inner;
    k.k1u = (double)d->upstream * (2.0 / ncm);
    k.k2u = (double)d->upstream * ((double)d->lambda / nm);
    k.eps = (double)d->eps;
    k.lambda = (double)d->lambda;
    k.inv_ncm = 1.0 / ncm;
    k.inv_nm = 1.0 / nm;
    const bool grad = d->gstudent != nullptr;
    if (pl.fused_kch) {
        k.coef = nullptr;
        return d->dtype == FQ_F16 ? launch_fused_width<_Float16>(k, pl, grad, st)
                                  : launch_fused_width<float>(k, pl, grad, st);
    }
    if (d->dtype == FQ_F16) {
        switch (pl.vec) {
        case 4: return launch<_Float16, 4>(k, pl, grad, st);
        case 2: return launch<_Float16, 2>(k, pl, grad, st);
        default: return launch<_Float16, 1>(k, pl, grad, st);
        }
    }
    switch (pl.vec) {
    case 4: return launch<float, 4>(k, pl, grad, st);
    case 2: return launch<float, 2>(k, pl, grad, st);
    default: return launch<float, 1>(k, pl, grad, st);
    }
}

}  // extern "C"
