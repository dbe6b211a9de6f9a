// gfx950 kernels for fused learnable-scale fake quantization (DPVO-QAT++ Sec. 3.2, Eq. (3)-(6),
// and the straight-through backward stated next to Eq. (5)).
//
// The work is HBM-bound elementwise traffic plus one per-channel reduction, so there is no MFMA
// here.  Each 256-thread block owns one chunk (at most 20 KiB of input) that lies inside a single
// [outer, channel] slab, so the scale is uniform over the block; lanes move 128-bit vectors
// (global_load/store_dwordx4, non-temporal), FP16 is widened/narrowed in registers.  Backward adds
// a DPP wavefront reduction, an LDS block reduction and a fixed-order combination of the blocks
// of a channel (direct, by atomic exchange, or by ticket: see combine); no float atomics.
// Tensors whose slabs are short are cut per wavefront instead (one slab per wavefront, four to a
// block, no barrier: forward_dispatch, backward_waves) when the launch has blocks to spare.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "fq_device.h"
#include "fq_internal.h"

namespace fq {

using namespace dev;

namespace {

template <typename T> struct VecOf;
template <> struct VecOf<float> {
    static constexpr int N = 4;
    typedef float type __attribute__((ext_vector_type(4)));
};
template <> struct VecOf<_Float16> {
    static constexpr int N = 8;
    typedef _Float16 type __attribute__((ext_vector_type(8)));
};

constexpr int kUnroll = kChunkVecs / kBlock;   // vectors per thread per chunk
static_assert(kChunkVecs % kBlock == 0, "chunk must be a whole number of block-wide vector rows");

// ---------------------------------------------------------------------------------------------
// Eq. (3)-(4): s = clip(softplus(theta) + eps, s_min, s_max).  Evaluated in binary64 and rounded
// to binary32 once, so the value does not depend on the accuracy of a binary32 exp/log.
struct Scale {
    float s;             // Eq. (3)-(4)
    bool clip_active;    // the clamp changed the value (its derivative is then zero)
    double sigmoid;      // d softplus / d theta
};

// What a block needs of its channel's scale (see block_params).
struct BlockScale {
    double rd;           // RN64(1 / s)
    double sigmoid;
    float s;
    unsigned clip_active;
};

// exp(-a) for a >= 0 in binary64, a few ulp: a = n ln2 + r with |r| <= ln2/2 (two-constant
// reduction, n ln2_hi is exact), exp(-r) by its Taylor polynomial of degree 13 (remainder below
// 2^-57), scaled by 2^-n.  Short on purpose: it sits in every block's prologue.
__device__ __forceinline__ double exp_neg(double a)
{
    if (!(a < 746.0)) return a != a ? a : 0.0;                   // underflows to 0; NaN stays NaN
    const double n = __builtin_rint(a * 1.4426950408889634074);      // a / ln2
    double r = __builtin_fma(-n, 6.93147180369123816490e-01, a);     // ln2_hi, 21 trailing zero bits
    r = __builtin_fma(-n, 1.90821492927058770002e-10, r);            // ln2_lo
    const double x = -r;
    double p = 1.0 / 6227020800.0;                                     // 1/13!
    p = __builtin_fma(p, x, 1.0 / 479001600.0);
    p = __builtin_fma(p, x, 1.0 / 39916800.0);
    p = __builtin_fma(p, x, 1.0 / 3628800.0);
    p = __builtin_fma(p, x, 1.0 / 362880.0);
    p = __builtin_fma(p, x, 1.0 / 40320.0);
    p = __builtin_fma(p, x, 1.0 / 5040.0);
    p = __builtin_fma(p, x, 1.0 / 720.0);
    p = __builtin_fma(p, x, 1.0 / 120.0);
    p = __builtin_fma(p, x, 1.0 / 24.0);
    p = __builtin_fma(p, x, 1.0 / 6.0);
    p = __builtin_fma(p, x, 0.5);
    p = __builtin_fma(p, x, 1.0);
    p = __builtin_fma(p, x, 1.0);
    return __builtin_ldexp(p, -(int)n);
}

// log(1 + e) for 0 <= e <= 1 in binary64, a few ulp: 2 atanh(z) with z = e / (2 + e) <= 1/3,
// odd series up to z^35 (next term below 2^-58 of the sum).  No cancellation for small e.
__device__ __forceinline__ double log1p_unit(double e)
{
    const double z = e / (2.0 + e);
    const double w = z * z;
    double p = 1.0 / 35.0;
    p = __builtin_fma(p, w, 1.0 / 33.0);
    p = __builtin_fma(p, w, 1.0 / 31.0);
    p = __builtin_fma(p, w, 1.0 / 29.0);
    p = __builtin_fma(p, w, 1.0 / 27.0);
    p = __builtin_fma(p, w, 1.0 / 25.0);
    p = __builtin_fma(p, w, 1.0 / 23.0);
    p = __builtin_fma(p, w, 1.0 / 21.0);
    p = __builtin_fma(p, w, 1.0 / 19.0);
    p = __builtin_fma(p, w, 1.0 / 17.0);
    p = __builtin_fma(p, w, 1.0 / 15.0);
    p = __builtin_fma(p, w, 1.0 / 13.0);
    p = __builtin_fma(p, w, 1.0 / 11.0);
    p = __builtin_fma(p, w, 1.0 / 9.0);
    p = __builtin_fma(p, w, 1.0 / 7.0);
    p = __builtin_fma(p, w, 1.0 / 5.0);
    p = __builtin_fma(p, w, 1.0 / 3.0);
    p = __builtin_fma(p, w, 1.0);
    return 2.0 * z * p;
}

// softplus(t) = max(t,0) + log1p(e) and sigmoid(t) = (t >= 0 ? 1 : e) / (1 + e), e = exp(-|t|):
// one exponential serves both.  The binary64 value is rounded to binary32 once; a few ulp of
// binary64 error move that rounding with probability ~1e-8 per channel.
template <bool NEED_SIGMOID>
__device__ __forceinline__ Scale compute_scale(float theta, float eps, float s_min, float s_max)
{
    const double t = (double)theta;
    const double e = exp_neg(__builtin_fabs(t));
    const double u = __builtin_fmax(t, 0.0) + log1p_unit(e) + (double)eps;
    const float uf = (float)u;
    Scale r;
    r.clip_active = !(uf >= s_min && uf <= s_max);
    float v = uf;
    v = v < s_min ? s_min : v;
    v = v > s_max ? s_max : v;
    r.s = v;
    r.sigmoid = NEED_SIGMOID ? (t >= 0.0 ? 1.0 : e) / (1.0 + e) : 0.0;
    return r;
}

// ---------------------------------------------------------------------------------------------
// Per-element arithmetic.
//
// Quotient.  v must be the correctly rounded binary32 value of x/s.  It is formed as
// (float)((double)x * rd) with rd = RN64(1/s): three full-rate instructions instead of the ~10 of
// the IEEE binary32 division expansion.  This rounds exactly like x/s: writing x = X*2^a and
// s = S*2^b with 24-bit integers X, S, the exact quotient is never half-way between two binary32
// values and its distance from the nearest half-way point is at least 1/(2S) > 2^-25 ulp, i.e.
// more than 2^-49 relative, while the binary64 product carries a relative error below 2^-52; so
// the final rounding to binary32 sees the same side of every rounding boundary.  Infinities, NaN,
// signed zeros and overflow behave as in x/s.  (Only a quotient in the binary32 subnormal range,
// |v| < 2^-126, may differ by one subnormal ulp; its code is 0 either way.)
//
// Clip + round.  v_med3_f32 returns lo for a NaN quotient, so NaN is put back afterwards
// (the per-operator definition propagates it: clamp and round keep NaN).
struct QParams {
    double rd;      // RN64(1 / s)
    float s, lo, hi;
    int ilo, ihi;   // the same bounds as integers (for the int8 codes)
};

__device__ __forceinline__ float quotient(float x, const QParams &p) { return (float)((double)x * p.rd); }

// y = s * round(clip(v)) for a quotient known not to be NaN (the clip would turn NaN into lo)
__device__ __forceinline__ float fq_value_finite(float v, const QParams &p)
{
    return __builtin_rintf(__builtin_amdgcn_fmed3f(v, p.lo, p.hi)) * p.s;
}

// forward value y = s * round(clip(v)); a NaN quotient gives NaN
__device__ __forceinline__ float fq_value(float v, const QParams &p)
{
    float q = __builtin_rintf(__builtin_amdgcn_fmed3f(v, p.lo, p.hi));
    float y = q * p.s;
    return v != v ? v : y;
}

// integer code clip(round(v)) (the same as round(clip(v)) for integer bounds), 0 for a NaN
// quotient.  v_cvt_i32_f32 itself maps NaN to 0 and saturates +-Inf and huge values, so no
// select is needed; it is written as an instruction because the C conversion of NaN/Inf is
// undefined.
__device__ __forceinline__ int fq_code(float v, const QParams &p)
{
    int c;
    asm("v_cvt_i32_f32 %0, %1" : "=v"(c) : "v"(__builtin_rintf(v)));
    c = c < p.ilo ? p.ilo : c;
    c = c > p.ihi ? p.ihi : c;
    return c;
}

// low bytes of four ints -> one dword (v_perm_b32 twice + or)
__device__ __forceinline__ unsigned pack_codes4(int c0, int c1, int c2, int c3)
{
    const unsigned lo = __builtin_amdgcn_perm((unsigned)c1, (unsigned)c0, 0x0c0c0400u);
    const unsigned hi = __builtin_amdgcn_perm((unsigned)c3, (unsigned)c2, 0x04000c0cu);
    return lo | hi;
}

// backward: returns t = dy/ds and whether the quotient is inside [lo, hi] (inclusive).
// in range: t = rint(v) - v;  below: lo;  above: hi;  NaN quotient: out of range, t = NaN.
__device__ __forceinline__ float ste_terms(float x, const QParams &p, bool &in_range, bool &is_nan)
{
    float v = quotient(x, p);
    float cl = __builtin_amdgcn_fmed3f(v, p.lo, p.hi);
    in_range = cl == v;                       // false for NaN
    is_nan = v != v;
    float r = __builtin_rintf(cl);            // the bound itself when clipped
    return r - (in_range ? v : 0.0f);
}

// Hold the wavefront until every vector memory operation it has issued (loads, stores, atomics)
// has been acknowledged; the "memory" clobber keeps the compiler from moving accesses across it.
__device__ __forceinline__ void wait_stores_acknowledged() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Finisher side of the tickets.  Every partial sum of the channel was acknowledged at agent scope
// before its unit drew a ticket, and the finisher has received the last ticket, so all of them are
// in memory when it starts reading.  It reads them with agent-scope atomic loads (global_load ...
// sc1), which are served from the level all XCDs share and never from a line cached by this XCD;
// the hardware issues a wavefront's memory operations in program order and the branch on the
// ticket's value needs the atomic's result, so the loads are issued after the ticket has returned.
// All that is left to enforce is that the compiler keeps them behind the ticket.  (An acquire
// fence at agent scope would also invalidate this XCD's L2 under the blocks still streaming
// through it: measured 41 -> 45 us on a 15x128x120x160 FP16 tensor, for nothing.)
__device__ __forceinline__ void acquire_partials() { asm volatile("" ::: "memory"); }

// Keeps the computation of a value at this point of the program: the compiler would otherwise
// sink it to its first use, behind the wait for a later load.  Emits no instruction.
__device__ __forceinline__ void pin_here(float &v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void pin_here(unsigned &v) { asm volatile("" : "+v"(v)); }

// Index of this wavefront in its block as a scalar: telling the compiler that it is uniform keeps
// everything derived from it (the unit's slab, channel, pointers, loop bounds) in SGPRs.
__device__ __forceinline__ unsigned wave_index() { return (unsigned)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

// ---------------------------------------------------------------------------------------------
// Chunk addressing shared by forward and backward.
struct Chunk {
    unsigned slab, channel;
    long long first;   // flat element index of the chunk's first element
    int n;             // elements in the chunk
};

__device__ __forceinline__ Chunk locate_chunk(const DevTensor &d, unsigned local_block)
{
    Chunk c;
    c.slab = local_block / d.cps;
    unsigned k = local_block - c.slab * d.cps;
    c.channel = c.slab % d.channels;
    long long e0 = (long long)k * d.chunk;
    long long rem = d.inner - e0;
    c.n = rem < (long long)d.chunk ? (int)rem : (int)d.chunk;
    c.first = (long long)c.slab * d.inner + e0;
    return c;
}

// The chunk of this block in a single-tensor launch.  Such a launch normally has a grid of
// (chunks per slab, channels, outer), which names the chunk without any division (two integer
// divisions sit between a block's start and its first load otherwise); tensors with more than
// 65535 channels or outer slices keep the linear grid.  `unit` receives the chunk's linear index.
__device__ __forceinline__ Chunk own_chunk(const DevTensor &d, unsigned &unit)
{
    if (!d.grid3) {
        unit = blockIdx.x;
        return locate_chunk(d, unit);
    }
    Chunk c;
    c.channel = blockIdx.y;
    c.slab = blockIdx.z * d.channels + blockIdx.y;
    unit = c.slab * d.cps + blockIdx.x;
    const long long e0 = (long long)blockIdx.x * d.chunk;
    const long long rem = d.inner - e0;
    c.n = rem < (long long)d.chunk ? (int)rem : (int)d.chunk;
    c.first = (long long)c.slab * d.inner + e0;
    return c;
}

// elements before the first 16-byte boundary of p
template <typename T> __device__ __forceinline__ int head_elems(const void *p, int n)
{
    int h = (int)(((kVecBytes - ((uintptr_t)p & (kVecBytes - 1))) & (kVecBytes - 1)) / sizeof(T));
    return h < n ? h : n;
}

// Scale of this group's channel (G = 256: the block; G = 64: one wavefront).  Callers issue their
// first global loads before this, so the evaluation sits in the shadow of the memory latency.
// A block lets one wavefront (rotating with the block index, so the work spreads over the four
// SIMDs of a compute unit) evaluate Eq. (3)-(4), about a hundred binary64 instructions, and the
// others read it from LDS after a barrier; a lone wavefront evaluates it for itself.
template <bool NEED_SIGMOID, int G>
__device__ __forceinline__ QParams block_params(const DevTensor &d, float theta, BlockScale &bs)
{
    if (G == 64) {
        const Scale sc = compute_scale<NEED_SIGMOID>(theta, d.eps, d.s_min, d.s_max);
        bs.s = sc.s;
        bs.rd = 1.0 / (double)sc.s;
        bs.sigmoid = sc.sigmoid;
        bs.clip_active = sc.clip_active ? 1u : 0u;
    } else {
        __shared__ BlockScale shared_scale;
        // (the block's linear index in the grid, whatever the grid's shape)
        const unsigned linear = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
        if ((threadIdx.x >> 6) == (linear & (kBlock / 64 - 1))) {
            const Scale sc = compute_scale<NEED_SIGMOID>(theta, d.eps, d.s_min, d.s_max);
            if ((threadIdx.x & 63) == 0) {
                shared_scale.s = sc.s;
                shared_scale.rd = 1.0 / (double)sc.s;
                shared_scale.sigmoid = sc.sigmoid;
                shared_scale.clip_active = sc.clip_active ? 1u : 0u;
            }
        }
        __syncthreads();
        bs = shared_scale;
    }
    QParams p;
    p.rd = bs.rd;
    p.s = bs.s;
    p.lo = d.lo;
    p.hi = d.hi;
    p.ilo = (int)d.lo;
    p.ihi = (int)d.hi;
    return p;
}

// ---------------------------------------------------------------------------------------------
// Forward.
template <typename T, bool WRITE_Y, bool EMIT_Q>
__device__ __forceinline__ void forward_elem(const T *x, T *y, int8_t *q, int i, const QParams &p)
{
    const float v = quotient((float)ld_global(x + i), p);
    if (WRITE_Y) st_global(y + i, (T)fq_value(v, p));
    if (EMIT_Q) st_global(q + i, (int8_t)fq_code(v, p));
}

// WRITE_Y: write the dequantized tensor y.  EMIT_Q: write the int8 codes, N per lane packed into
// one 64-bit (FP16 input) or 32-bit (FP32 input) store.  At least one of the two.
template <typename T, bool WRITE_Y, bool EMIT_Q, int G>
__device__ __forceinline__ void forward_chunk(const DevTensor &d, const Chunk &ck)
{
    typedef typename VecOf<T>::type VT;
    constexpr int N = VecOf<T>::N;
    typedef unsigned QV __attribute__((ext_vector_type(N / 4)));
    const T *x = (const T *)d.x + ck.first;
    T *y = WRITE_Y ? (T *)d.y + ck.first : nullptr;
    int8_t *q = EMIT_Q ? d.q + ck.first : nullptr;
    const int tid = threadIdx.x & (G - 1);
    const float theta = ld_uniform(d.theta + ck.channel);

    const bool vector_ok = !WRITE_Y || (((uintptr_t)x ^ (uintptr_t)y) & (kVecBytes - 1)) == 0;
    const int head = vector_ok ? head_elems<T>(x, ck.n) : ck.n;
    const int nvec = (ck.n - head) / N;
    const VT *xv = (const VT *)(x + head);
    VT *yv = WRITE_Y ? (VT *)(y + head) : nullptr;
    const bool q_packed = EMIT_Q && ((uintptr_t)(q + head) % N) == 0;

    // Issue the first row of loads (straight-line: out-of-range lanes re-read the last vector)
    // before the long binary64 scale evaluation, which then runs under the memory latency.
    VT r[kUnroll];
    if (nvec > 0) {
        const int last = nvec - 1;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            int v = u * G + tid;
            r[u] = ld_stream(xv + (v < last ? v : last));
        }
    }

    BlockScale bs;
    const QParams p = block_params<false, G>(d, theta, bs);
    if (d.s && ck.first == (long long)ck.channel * d.inner && tid == 0) st_global(d.s + ck.channel, p.s);

    for (int v0 = 0; v0 < nvec;) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            int v = v0 + u * G + tid;
            if (v < nvec) {
                float quot[N];
#pragma unroll
                for (int e = 0; e < N; ++e) quot[e] = quotient((float)r[u][e], p);
                if (WRITE_Y) {
                    // A NaN quotient must come out as NaN, and the clip swallows it.  Instead of a
                    // compare and a select per element, the row's quotients are tested in pairs
                    // (one unordered compare sees a NaN in either operand) and only a lane that
                    // has found one goes back over its row.
                    VT o;
                    bool any_nan = false;
#pragma unroll
                    for (int e = 0; e < N; e += 2) any_nan |= __builtin_isunordered(quot[e], quot[e + 1]);
#pragma unroll
                    for (int e = 0; e < N; ++e) o[e] = (T)fq_value_finite(quot[e], p);
                    if (__builtin_expect(any_nan, 0)) {
                        asm volatile("" ::: "memory");       // keep this a branch: it is almost never taken
#pragma unroll
                        for (int e = 0; e < N; ++e) o[e] = (T)fq_value(quot[e], p);
                    }
                    st_stream(yv + v, o);
                }
                if (EMIT_Q) {
                    int c[N];
#pragma unroll
                    for (int e = 0; e < N; ++e) c[e] = fq_code(quot[e], p);
                    if (q_packed) {
                        QV codes;
#pragma unroll
                        for (int g = 0; g < N / 4; ++g)
                            codes[g] = pack_codes4(c[4 * g], c[4 * g + 1], c[4 * g + 2], c[4 * g + 3]);
                        st_stream((QV *)(q + head + v * N), codes);
                    } else {
#pragma unroll
                        for (int e = 0; e < N; ++e) st_global(q + head + v * N + e, (int8_t)c[e]);
                    }
                }
            }
        }
        v0 += kUnroll * G;
        if (v0 >= nvec) break;
        const int last = nvec - 1;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            int v = v0 + u * G + tid;
            r[u] = ld_stream(xv + (v < last ? v : last));
        }
    }

    // scalar head (before the first 16-byte boundary, or the whole chunk if x and y are
    // misaligned relative to each other) and tail (after the last whole vector)
    for (int i = tid; i < head; i += G) forward_elem<T, WRITE_Y, EMIT_Q>(x, y, q, i, p);
    for (int i = head + nvec * N + tid; i < ck.n; i += G) forward_elem<T, WRITE_Y, EMIT_Q>(x, y, q, i, p);
}

// what one tensor asks of the forward pass: y only, y and codes, or codes only
template <typename T, int G>
__device__ __forceinline__ void forward_variants(const DevTensor &d, unsigned unit)
{
    const Chunk ck = locate_chunk(d, unit);
    if (!d.q) forward_chunk<T, true, false, G>(d, ck);
    else if (d.y) forward_chunk<T, true, true, G>(d, ck);
    else forward_chunk<T, false, true, G>(d, ck);
}

// Tensors whose slabs are short (d.wave_units) give every wavefront a slab of its own: four
// slabs to a block, no barrier.  Otherwise the block owns one chunk.
template <typename T>
__device__ __forceinline__ void forward_dispatch(const DevTensor &d, unsigned local_block)
{
    if (d.wave_units) {
        const unsigned unit = local_block * (kBlock / 64) + wave_index();
        if (unit < d.slabs * d.cps) forward_variants<T, 64>(d, unit);
    } else {
        forward_variants<T, kBlock>(d, local_block);
    }
}

// ---------------------------------------------------------------------------------------------
// Backward.
// gy*t is exact in binary64 (two 24-bit significands), so the per-channel sum differs from a
// sequential binary64 sum only by binary64 rounding, however badly the terms cancel.
template <typename T, bool WRITE_GX>
__device__ __forceinline__ double backward_elem(const T *x, const T *gy, T *gx, int i, const QParams &p,
                                                double acc)
{
    bool in_range, is_nan;
    T g = ld_global(gy + i);
    float t = ste_terms((float)ld_global(x + i), p, in_range, is_nan);
    if (WRITE_GX) st_global(gx + i, in_range ? g : (T)0.0f);
    acc = __builtin_fma((double)(float)g, (double)t, acc);
    return is_nan ? __builtin_nan("") : acc;
}

// Per-thread sum of gy*t over this thread's elements of the chunk (binary64).
template <typename T, bool WRITE_GX, int G>
__device__ __forceinline__ double backward_chunk(const DevTensor &d, const Chunk &ck, BlockScale &bs)
{
    typedef typename VecOf<T>::type VT;
    constexpr int N = VecOf<T>::N;
    const T *x = (const T *)d.x + ck.first;
    const T *gy = (const T *)d.gy + ck.first;
    T *gx = WRITE_GX ? (T *)d.gx + ck.first : nullptr;
    const int tid = threadIdx.x & (G - 1);
    const float theta = ld_uniform(d.theta + ck.channel);

    uintptr_t mis = (uintptr_t)x ^ (uintptr_t)gy;
    if (WRITE_GX) mis |= (uintptr_t)x ^ (uintptr_t)gx;
    const bool vector_ok = (mis & (kVecBytes - 1)) == 0;
    const int head = vector_ok ? head_elems<T>(x, ck.n) : ck.n;
    const int nvec = (ck.n - head) / N;
    const VT *xv = (const VT *)(x + head);
    const VT *gv = (const VT *)(gy + head);
    VT *ov = WRITE_GX ? (VT *)(gx + head) : nullptr;

    VT rx[kUnroll], rg[kUnroll];
    if (nvec > 0) {
        const int last = nvec - 1;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            int v = u * G + tid;
            v = v < last ? v : last;
            rx[u] = ld_stream(xv + v);
            rg[u] = ld_stream(gv + v);
        }
    }

    const QParams p = block_params<true, G>(d, theta, bs);

    double acc[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) acc[u] = 0.0;

    for (int v0 = 0; v0 < nvec;) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            int v = v0 + u * G + tid;
            if (v < nvec) {
                VT o;
                bool any_nan = false;
#pragma unroll
                for (int e = 0; e < N; ++e) {
                    bool in_range, is_nan;
                    float t = ste_terms((float)rx[u][e], p, in_range, is_nan);
                    o[e] = in_range ? rg[u][e] : (T)0.0f;
                    acc[u] = __builtin_fma((double)(float)rg[u][e], (double)t, acc[u]);
                    any_nan |= is_nan;
                }
                if (any_nan) acc[u] = __builtin_nan("");   // a NaN quotient poisons its channel
                if (WRITE_GX) st_stream(ov + v, o);
            }
        }
        v0 += kUnroll * G;
        if (v0 >= nvec) break;
        const int last = nvec - 1;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            int v = v0 + u * G + tid;
            v = v < last ? v : last;
            rx[u] = ld_stream(xv + v);
            rg[u] = ld_stream(gv + v);
        }
    }

    double sum = 0.0;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) sum += acc[u];
    for (int i = tid; i < head; i += G) sum = backward_elem<T, WRITE_GX>(x, gy, gx, i, p, sum);
    for (int i = head + nvec * N + tid; i < ck.n; i += G)
        sum = backward_elem<T, WRITE_GX>(x, gy, gx, i, p, sum);
    return sum;
}

// The same sum with the schedule for launches whose blocks are all resident at once (at most three
// per compute unit: the 1x384x120x160 FP16 tensor).  Such a launch is one burst: every wavefront asks
// for its whole chunk at the start, the data trickles in over the next microseconds, and whatever a
// wavefront still has to compute after its last row has landed is added to the kernel's duration,
// with nothing left to hide it.  So all x rows are requested before all gy rows; what depends on x
// alone (quotient, clip, round, t, the mask: two thirds of the arithmetic) is done as the x rows
// arrive, while the gy rows are still on their way; only the products and the selects wait for the
// last row; and gx is stored at the very end, in one run, so that no store sits between the loads
// in the memory pipeline.  The price is registers (every row's t is kept: 134 VGPRs instead of 71,
// three wavefronts per SIMD), which costs a large launch more than the schedule gains (a
// 15x128x120x160 FP16 tensor: 44.5 us instead of 40.7), so larger launches interleave as before.
// The arithmetic and its order are the same in both schedules; so are the bits.
template <typename T, bool WRITE_GX, int G>
__device__ __forceinline__ double backward_chunk_short(const DevTensor &d, const Chunk &ck, BlockScale &bs)
{
    typedef typename VecOf<T>::type VT;
    constexpr int N = VecOf<T>::N;
    const T *x = (const T *)d.x + ck.first;
    const T *gy = (const T *)d.gy + ck.first;
    T *gx = WRITE_GX ? (T *)d.gx + ck.first : nullptr;
    const int tid = threadIdx.x & (G - 1);
    const float theta = ld_uniform(d.theta + ck.channel);

    uintptr_t mis = (uintptr_t)x ^ (uintptr_t)gy;
    if (WRITE_GX) mis |= (uintptr_t)x ^ (uintptr_t)gx;
    const bool vector_ok = (mis & (kVecBytes - 1)) == 0;
    const int head = vector_ok ? head_elems<T>(x, ck.n) : ck.n;
    const int nvec = (ck.n - head) / N;
    const VT *xv = (const VT *)(x + head);
    const VT *gv = (const VT *)(gy + head);
    VT *ov = WRITE_GX ? (VT *)(gx + head) : nullptr;

    VT rx[kUnroll], rg[kUnroll];
    auto request = [&](int v0) {      // out-of-range lanes re-read the last vector
        const int last = nvec - 1;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int v = v0 + u * G + tid;
            rx[u] = ld_stream(xv + (v < last ? v : last));
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int v = v0 + u * G + tid;
            rg[u] = ld_stream(gv + (v < last ? v : last));
        }
    };
    if (nvec > 0) request(0);

    const QParams p = block_params<true, G>(d, theta, bs);

    double acc[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) acc[u] = 0.0;

    for (int v0 = 0; v0 < nvec;) {
        float t[kUnroll][N];
        unsigned inside[kUnroll], nan_row[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            inside[u] = 0u;
            nan_row[u] = 0u;
#pragma unroll
            for (int e = 0; e < N; ++e) {
                bool in_range, is_nan;
                t[u][e] = ste_terms((float)rx[u][e], p, in_range, is_nan);
                inside[u] |= in_range ? 1u << e : 0u;
                nan_row[u] |= is_nan ? 1u : 0u;
                pin_here(t[u][e]);
            }
            pin_here(inside[u]);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int v = v0 + u * G + tid;
            if (v < nvec) {
                VT o;
#pragma unroll
                for (int e = 0; e < N; ++e) {
                    o[e] = (inside[u] >> e & 1u) ? rg[u][e] : (T)0.0f;
                    acc[u] = __builtin_fma((double)(float)rg[u][e], (double)t[u][e], acc[u]);
                }
                if (nan_row[u]) acc[u] = __builtin_nan("");   // a NaN quotient poisons its channel
                rg[u] = o;
            }
        }
        if (WRITE_GX) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int v = v0 + u * G + tid;
                if (v < nvec) st_stream(ov + v, rg[u]);
            }
        }
        v0 += kUnroll * G;
        if (v0 >= nvec) break;
        request(v0);
    }

    double sum = 0.0;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) sum += acc[u];
    for (int i = tid; i < head; i += G) sum = backward_elem<T, WRITE_GX>(x, gy, gx, i, p, sum);
    for (int i = head + nvec * N + tid; i < ck.n; i += G)
        sum = backward_elem<T, WRITE_GX>(x, gy, gx, i, p, sum);
    return sum;
}

// Chain rule through Eq. (3)-(4) and the per-channel outputs of the backward pass.
__device__ __forceinline__ void write_channel_grads(const DevTensor &d, unsigned c, double total, const BlockScale &bs)
{
    const float g = bs.clip_active ? 0.0f : (float)(total * bs.sigmoid);
    if (d.gs) st_global(d.gs + c, (float)total);
    if (d.gtheta) st_global(d.gtheta + c, g);
    if (d.s) st_global(d.s + c, bs.s);
    if (d.adam_m) {
        // One Adam step on theta_c (Kingma & Ba, Algorithm 1), binary32, each operation rounded
        // on its own.  Every block of this channel has finished reading theta_c by now (this
        // code runs after all of them have handed in their sums), so theta may be updated in
        // place.  A non-finite gradient leaves m, v and theta as they are.
        const float theta = ld_global(d.theta + c);
        float out = theta;
        if (__builtin_isfinite(g)) {
            const float m = d.adam_beta1 * ld_global(d.adam_m + c) + d.adam_one_minus_beta1 * g;
            const float v = d.adam_beta2 * ld_global(d.adam_v + c) + (d.adam_one_minus_beta2 * g) * g;
            const float mhat = m / d.adam_bc1, vhat = v / d.adam_bc2;
            st_global(d.adam_m + c, m);
            st_global(d.adam_v + c, v);
            out = theta - (d.adam_lr * mhat) / (__builtin_sqrtf(vhat) + d.adam_eps);
        }
        st_global(d.adam_theta_out + c, out);
    }
}

// Sum the per-block partials of channel c in a fixed order (thread-strided binary64 sums, fixed
// tree).  Block-wide; lds holds kBlock/64 doubles.  Partials are read with agent-scope loads:
// they may have been written by a block running on another XCD, whose L2 is not this one.
__device__ __forceinline__ void finalize_channel(const DevTensor &d, unsigned c, const BlockScale &bs, double *lds)
{
    const unsigned bpc = d.outer * d.cps;
    double acc = 0.0;
    // thread t adds sums t, t+256, t+512, ... in that order; eight loads are kept in flight
    constexpr unsigned kBatch = 8;
    for (unsigned j0 = threadIdx.x; j0 < bpc; j0 += kBlock * kBatch) {
        double part[kBatch];
#pragma unroll
        for (unsigned i = 0; i < kBatch; ++i) {
            const unsigned j = j0 + i * kBlock;
            part[i] = 0.0;
            if (j < bpc) {
                const unsigned o = j / d.cps;
                const unsigned k = j - o * d.cps;
                const size_t idx = ((size_t)o * d.channels + c) * d.cps + k;
                part[i] = __hip_atomic_load(&d.partial[idx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
#pragma unroll
        for (unsigned i = 0; i < kBatch; ++i) acc += part[i];
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == kSumLane) lds[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double total = 0.0;
#pragma unroll
        for (int w = 0; w < kBlock / 64; ++w) total += lds[w];
        write_channel_grads(d, c, total, bs);
    }
    __syncthreads();
}

// value of v in the given lane, as a wavefront-uniform scalar
__device__ __forceinline__ double read_lane(double v, int lane)
{
    const unsigned long long bits = __builtin_bit_cast(unsigned long long, v);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)bits, lane);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(bits >> 32), lane);
    return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}

// The same sum, bit for bit, by a single wavefront (for tensors whose units are wavefronts): the
// block-wide version gives thread t the sums t, t+256, ... and adds wavefront 0's tree to
// wavefront 1's, 2's and 3's in that order; here the one wavefront plays the four in turn.
__device__ __forceinline__ void finalize_channel_wave(const DevTensor &d, unsigned c, const BlockScale &bs)
{
    const unsigned bpc = d.outer * d.cps;
    const unsigned lane = threadIdx.x & 63;
    double total = 0.0;
    for (unsigned w = 0; w < kBlock / 64; ++w) {
        double acc = 0.0;
        for (unsigned j = w * 64 + lane; j < bpc; j += kBlock) {
            const unsigned o = j / d.cps;
            const unsigned k = j - o * d.cps;
            const size_t idx = ((size_t)o * d.channels + c) * d.cps + k;
            acc += __hip_atomic_load(&d.partial[idx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        acc = wave_sum(acc);
        total += read_lane(acc, kSumLane);
    }
    if (lane == kSumLane) write_channel_grads(d, c, total, bs);
}

// How the units (blocks, or wavefronts of short-slab tensors) of a channel combine their sums
// (FUSED; no float atomics, fixed order):
//   1 unit per channel    the unit writes the channel's gradients itself;
//   2 units per channel   each swaps its sum into the channel's 64-bit slot; the one that finds
//                         its partner's sum there adds the two (a+b = b+a) and clears the slot:
//                         one atomic round trip, the payload travels in the atomic itself;
//   3 or 4                two rounds of that exchange, pairs first (two more slots per channel);
//   more                  each unit stores its sum, waits for that store, then draws a ticket
//                         from the slot; the unit with the last ticket has all sums re-read in
//                         index order and clears the slot.  Beyond kTicketFanIn units per channel
//                         the tickets are drawn in two levels (d.sub first-level slots).
// The slots are zero between calls.  (A sum of +0.0 is swapped in as -0.0 so that it differs from
// an empty slot; it adds the same.)
// Without FUSED the sums are only stored and finalize_kernel adds them in a second launch.
//
// Called by one lane per unit with the unit's total.  Returns 1 if the caller drew the last
// ticket, i.e. its block must now run finalize_channel for ck.channel.
template <bool FUSED>
__device__ __forceinline__ unsigned combine(const DevTensor &d, const Chunk &ck, unsigned unit, double total,
                                            const BlockScale &bs)
{
    const unsigned bpc = d.outer * d.cps;
    unsigned last = 0u;
    if (!FUSED) {
        __hip_atomic_store(&d.partial[unit], total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else if (bpc == 1u) {
        write_channel_grads(d, ck.channel, total, bs);
    } else if (bpc == 2u) {
        unsigned long long mine = __builtin_bit_cast(unsigned long long, total);
        if (mine == 0ull) mine = 0x8000000000000000ull;
        const unsigned long long theirs = __hip_atomic_exchange(&d.slot[ck.channel], mine, __ATOMIC_RELAXED,
                                                                __HIP_MEMORY_SCOPE_AGENT);
        if (theirs != 0ull) {
            __hip_atomic_store(&d.slot[ck.channel], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const double both = (__builtin_bit_cast(double, theirs) + total) + 0.0;
            write_channel_grads(d, ck.channel, both, bs);
        }
    } else if (bpc <= kTreeBlocks) {
        // Three or four units: two rounds of the same exchange, associated as finalize_channel
        // associates its sums, (p0 + p1) + (p2 + p3) with an absent p3 counting as +0.0, so the
        // bits equal those of the two-launch mode.  Unlike the tickets below this needs no wait
        // for the unit's own gx stores and no re-read of the partial sums.
        const unsigned o = ck.slab / d.channels;
        const unsigned j = o * d.cps + (unit - ck.slab * d.cps);
        double pair_sum = total + 0.0;                 // unit 2 of 3 has no partner
        bool carry_on = true;
        if (!(bpc == 3u && j == 2u)) {
            unsigned long long *pair = d.slot + d.channels + (size_t)ck.channel * 2u + (j >> 1);
            unsigned long long mine = __builtin_bit_cast(unsigned long long, total);
            if (mine == 0ull) mine = 0x8000000000000000ull;
            const unsigned long long theirs = __hip_atomic_exchange(pair, mine, __ATOMIC_RELAXED,
                                                                    __HIP_MEMORY_SCOPE_AGENT);
            carry_on = theirs != 0ull;
            if (carry_on) {
                __hip_atomic_store(pair, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                pair_sum = __builtin_bit_cast(double, theirs) + total;
            }
        }
        if (carry_on) {
            unsigned long long mine = __builtin_bit_cast(unsigned long long, pair_sum);
            if (mine == 0ull) mine = 0x8000000000000000ull;
            const unsigned long long theirs = __hip_atomic_exchange(&d.slot[ck.channel], mine, __ATOMIC_RELAXED,
                                                                    __HIP_MEMORY_SCOPE_AGENT);
            if (theirs != 0ull) {
                __hip_atomic_store(&d.slot[ck.channel], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const double all = (__builtin_bit_cast(double, theirs) + pair_sum) + 0.0;
                write_channel_grads(d, ck.channel, all, bs);
            }
        }
    } else {
        // Publish, then draw.  The sum goes out with an agent-scope store (global_store ... sc1:
        // written through to the memory level that all XCDs share).  Stores count in vmcnt on this
        // target and an agent-scope store is acknowledged only once it has reached that level, so
        // after s_waitcnt vmcnt(0) the sum is visible to every XCD; the ticket atomic is issued
        // after the wait and therefore reaches the memory side after the sum it announces.  A
        // release fence at agent scope would give the same order but also writes back the whole
        // L2 (the unit's gx stores), once per unit; only the partial has to be published.
        __hip_atomic_store(&d.partial[unit], total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        wait_stores_acknowledged();
        unsigned long long *top = &d.slot[ck.channel];
        unsigned long long expected = bpc;
        bool draw_top = true;
        if (d.sub) {
            // Hundreds of units drawing from one address queue up behind each other at the
            // memory-side atomic unit.  Unit j of the channel draws from sub-slot j mod sub
            // first; only the last arrival there goes on to the channel's own slot.
            const unsigned o = ck.slab / d.channels;
            const unsigned j = o * d.cps + (unit - ck.slab * d.cps);
            const unsigned k = j % d.sub;
            const unsigned long long arrivals = (bpc - k + d.sub - 1u) / d.sub;
            unsigned long long *first = d.slot + d.channels + (size_t)ck.channel * d.sub + k;
            const unsigned long long t1 = __hip_atomic_fetch_add(first, 1ull, __ATOMIC_RELAXED,
                                                                 __HIP_MEMORY_SCOPE_AGENT);
            draw_top = t1 == arrivals - 1ull;
            if (draw_top) __hip_atomic_store(first, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            expected = d.sub;                      // bpc > sub, so every sub-slot is in use
        }
        if (draw_top) {
            const unsigned long long ticket = __hip_atomic_fetch_add(top, 1ull, __ATOMIC_RELAXED,
                                                                     __HIP_MEMORY_SCOPE_AGENT);
            last = (ticket == expected - 1ull) ? 1u : 0u;
            if (last) __hip_atomic_store(top, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    return last;
}

// One block of the backward grid, owning one chunk of one slab.
template <typename T, bool FUSED, bool SHORT = false>
__device__ __forceinline__ void backward_block(const DevTensor &d, const Chunk &ck, unsigned local_block)
{
    __shared__ double wave_part[kBlock / 64];
    __shared__ double fin_part[kBlock / 64];
    __shared__ unsigned is_last;

    const bool write_gx = !(d.flags & 1u);
    BlockScale bs;
    double sum;
    if (SHORT) sum = write_gx ? backward_chunk_short<T, true, kBlock>(d, ck, bs) : backward_chunk_short<T, false, kBlock>(d, ck, bs);
    else sum = write_gx ? backward_chunk<T, true, kBlock>(d, ck, bs) : backward_chunk<T, false, kBlock>(d, ck, bs);

    sum = wave_sum(sum);
    if ((threadIdx.x & 63) == kSumLane) wave_part[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        double total = 0.0;
#pragma unroll
        for (int w = 0; w < kBlock / 64; ++w) total += wave_part[w];
        is_last = combine<FUSED>(d, ck, local_block, total, bs);
    }
    if (FUSED && d.outer * d.cps > kTreeBlocks) {
        __syncthreads();
        if (is_last) {
            acquire_partials();
            finalize_channel(d, ck.channel, bs, fin_part);
        }
    }
}

// One block of the backward grid for a tensor with short slabs: every wavefront owns a slab (a
// unit) of its own -- scale, sum, combination and, if it draws the last ticket of its channel,
// the final sum, all per wavefront; the block never meets at a barrier.
template <typename T, bool FUSED>
__device__ __forceinline__ void backward_waves(const DevTensor &d, unsigned local_block)
{
    const unsigned unit = local_block * (kBlock / 64) + wave_index();
    if (unit >= d.slabs * d.cps) return;
    const bool write_gx = !(d.flags & 1u);
    const Chunk ck = locate_chunk(d, unit);
    BlockScale bs;
    double sum = write_gx ? backward_chunk<T, true, 64>(d, ck, bs) : backward_chunk<T, false, 64>(d, ck, bs);
    sum = wave_sum(sum);
    unsigned last = 0u;
    if ((threadIdx.x & 63) == kSumLane) last = combine<FUSED>(d, ck, unit, sum, bs);
    if (FUSED && d.outer * d.cps > kTreeBlocks) {
        if (__builtin_amdgcn_readlane((int)last, kSumLane)) {
            acquire_partials();
            finalize_channel_wave(d, ck.channel, bs);
        }
    }
}

template <typename T, bool FUSED>
__device__ __forceinline__ void backward_dispatch(const DevTensor &d, unsigned local_block)
{
    if (d.wave_units) backward_waves<T, FUSED>(d, local_block);
    else backward_block<T, FUSED>(d, locate_chunk(d, local_block), local_block);
}

// ---------------------------------------------------------------------------------------------
// Multi-tensor grid: the table lives at the start of the workspace and is read through the scalar
// cache.  Block -> tensor: last entry whose first block is <= block.
__device__ __forceinline__ int find_by_block(const FQ_CONST DevTensor *table, int n, unsigned block)
{
    int lo = 0, hi = n - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (table[mid].block_begin <= block) lo = mid; else hi = mid - 1;
    }
    return lo;
}

__device__ __forceinline__ int find_by_channel(const FQ_CONST DevTensor *table, int n, unsigned chan)
{
    int lo = 0, hi = n - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (table[mid].chan_begin <= chan) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// copy one table entry into registers, word by word through the scalar cache
__device__ __forceinline__ DevTensor fetch(const DevTensor *table, int i)
{
    static_assert(sizeof(DevTensor) % 4 == 0, "descriptor is copied as 32-bit words");
    DevTensor d;
    const FQ_CONST unsigned *src = (const FQ_CONST unsigned *)(table + i);
    unsigned *dst = (unsigned *)&d;
#pragma unroll
    for (unsigned w = 0; w < sizeof(DevTensor) / 4; ++w) dst[w] = src[w];
    return d;
}

// Single tensor: descriptor in the kernel arguments (SGPRs), dtype fixed at compile time.
// WAVES: the tensor's slabs are short and every wavefront owns one (chosen by the launcher).
template <typename T, bool WRITE_Y, bool EMIT_Q, bool WAVES>
__global__ void __launch_bounds__(kBlock) forward_kernel(const DevTensor d)
{
    if (WAVES) {
        const unsigned unit = blockIdx.x * (kBlock / 64) + wave_index();
        if (unit < d.slabs * d.cps) forward_chunk<T, WRITE_Y, EMIT_Q, 64>(d, locate_chunk(d, unit));
    } else {
        unsigned unit;
        forward_chunk<T, WRITE_Y, EMIT_Q, kBlock>(d, own_chunk(d, unit));
    }
}

// ANY_Q = false: no tensor of the list wants codes (the usual case; keeps the kernel lean)
template <bool ANY_Q>
__global__ void __launch_bounds__(kBlock) forward_multi_kernel(const DevTensor *table, int n)
{
    const DevTensor d = fetch(table, find_by_block((const FQ_CONST DevTensor *)table, n, blockIdx.x));
    const unsigned local = blockIdx.x - d.block_begin;
    if (ANY_Q) {
        if (d.dtype == 0) forward_dispatch<_Float16>(d, local);
        else forward_dispatch<float>(d, local);
    } else {
        if (d.wave_units) {
            const unsigned unit = local * (kBlock / 64) + wave_index();
            if (unit < d.slabs * d.cps) {
                if (d.dtype == 0) forward_chunk<_Float16, true, false, 64>(d, locate_chunk(d, unit));
                else forward_chunk<float, true, false, 64>(d, locate_chunk(d, unit));
            }
        } else if (d.dtype == 0) {
            forward_chunk<_Float16, true, false, kBlock>(d, locate_chunk(d, local));
        } else {
            forward_chunk<float, true, false, kBlock>(d, locate_chunk(d, local));
        }
    }
}

// SHAPE: 0 = one chunk per block; 1 = one slab per wavefront (short slabs); 2 = one chunk per block
// in a launch of at most kShortLaunchBlocks blocks (see backward_chunk, SHORT).
template <typename T, bool FUSED, int SHAPE>
__global__ void __launch_bounds__(kBlock) backward_kernel(const DevTensor d)
{
    if (SHAPE == 1) {
        backward_waves<T, FUSED>(d, blockIdx.x);
    } else {
        unsigned unit;
        const Chunk ck = own_chunk(d, unit);
        backward_block<T, FUSED, SHAPE == 2>(d, ck, unit);
    }
}

template <bool FUSED>
__global__ void __launch_bounds__(kBlock) backward_multi_kernel(const DevTensor *table, int n)
{
    const DevTensor d = fetch(table, find_by_block((const FQ_CONST DevTensor *)table, n, blockIdx.x));
    const unsigned local = blockIdx.x - d.block_begin;
    if (d.dtype == 0) backward_dispatch<_Float16, FUSED>(d, local);
    else backward_dispatch<float, FUSED>(d, local);
}

// one block per channel: second pass of the two-pass backward, and the whole backward of tensors
// that have channels but no elements (their gradients are zero)
__global__ void __launch_bounds__(kBlock) finalize_kernel(const KArgs a)
{
    __shared__ double fin_part[kBlock / 64];
    const DevTensor d = a.table ? fetch(a.table, find_by_channel((const FQ_CONST DevTensor *)a.table, a.n, blockIdx.x))
                                : a.one;
    const unsigned c = blockIdx.x - d.chan_begin;
    BlockScale bs;
    block_params<true, kBlock>(d, ld_uniform(d.theta + c), bs);
    finalize_channel(d, c, bs, fin_part);
}

// s[c] for every channel; used when a tensor has channels but no elements (forward)
__global__ void __launch_bounds__(kBlock) scale_kernel(const KArgs a, unsigned total_channels)
{
    unsigned g = blockIdx.x * kBlock + threadIdx.x;
    if (g >= total_channels) return;
    const DevTensor *dp = a.table ? &a.table[find_by_channel((const FQ_CONST DevTensor *)a.table, a.n, g)] : &a.one;
    unsigned c = g - dp->chan_begin;
    if (dp->s) dp->s[c] = compute_scale<false>(dp->theta[c], dp->eps, dp->s_min, dp->s_max).s;
}

__global__ void __launch_bounds__(kBlock) fill_zero_kernel(unsigned *p, size_t words)
{
    size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (; i < words; i += stride) p[i] = 0u;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// Measurement aid (fq_probe_stream): streaming kernels with no arithmetic in the launch shape of the
// forward and backward kernels (256-thread blocks, one chunk of kChunkVecs 128-bit vectors each,
// every load issued before the first store, non-temporal).  What they take is what the memory
// system and the launch cost alone take for the same bytes.
namespace {
typedef unsigned probe_vec __attribute__((ext_vector_type(4)));

template <int INPUTS>
__global__ void __launch_bounds__(kBlock) probe_kernel(const probe_vec *a, const probe_vec *b, probe_vec *out, size_t nvec)
{
    constexpr int kRows = kChunkVecs / kBlock;
    if (INPUTS == 0) return;
    const size_t first = (size_t)blockIdx.x * kChunkVecs + threadIdx.x;
    probe_vec ra[kRows], rb[kRows];
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
        size_t v = first + (size_t)u * kBlock;
        v = v < nvec ? v : nvec - 1;
        ra[u] = ld_stream(a + v);
        if (INPUTS == 2) rb[u] = ld_stream(b + v);
    }
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
        const size_t v = first + (size_t)u * kBlock;
        if (v < nvec) st_stream(out + v, INPUTS == 2 ? ra[u] ^ rb[u] : ra[u]);
    }
}
}  // namespace

int launch_probe(int inputs, const void *a, const void *b, void *out, size_t bytes, void *stream)
{
    const size_t nvec = bytes / kVecBytes;
    if (nvec == 0) return 0;
    const unsigned blocks = (unsigned)((nvec + kChunkVecs - 1) / kChunkVecs);
    hipStream_t st = (hipStream_t)stream;
    const probe_vec *pa = (const probe_vec *)a, *pb = (const probe_vec *)b;
    probe_vec *po = (probe_vec *)out;
    if (inputs == 0) hipLaunchKernelGGL(probe_kernel<0>, dim3(blocks), dim3(kBlock), 0, st, pa, pb, po, nvec);
    else if (inputs == 1) hipLaunchKernelGGL(probe_kernel<1>, dim3(blocks), dim3(kBlock), 0, st, pa, pb, po, nvec);
    else hipLaunchKernelGGL(probe_kernel<2>, dim3(blocks), dim3(kBlock), 0, st, pa, pb, po, nvec);
    return (int)hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Built-in scratch memory for callers that cannot allocate (fq_backward_static).  One array per
// GPU, held from the moment the code object is loaded until the process ends.  In host code the
// array's name stands for the symbol, not for a device address: the address on the current
// device comes from hipGetSymbolAddress, once per device, and only that pointer is ever handed
// to kernels.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void *scratch_ptr[kMaxDevices];     // per device; nullptr until the first call on that device
}  // namespace

// Device address of the scratch array on the current device (0 = success, else a hipError_t).
// The first call on a device also zeroes the slot region with a fill kernel on `stream`; the
// loader has zeroed it already and every completed backward leaves it zero, this only makes the
// starting state explicit.
int static_scratch(void **ptr, void *stream)
{
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return (int)e;
    if (device < 0 || device >= kMaxDevices) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[device]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return (int)e;
        if (!p) return (int)hipErrorInvalidSymbol;
        const int rc = launch_fill_zero(p, kStaticSlotBytes, stream);
        if (rc != 0) return rc;
        scratch_ptr[device] = p;
    }
    *ptr = scratch_ptr[device];
    return 0;
}

// ---------------------------------------------------------------------------------------------
// Launchers.
template <typename K, typename... Args>
static void launch(K kernel, unsigned blocks, hipStream_t st, Args... args)
{
    hipLaunchKernelGGL(kernel, dim3(blocks), dim3(kBlock), 0, st, args...);
}

// Single-tensor launch: grid (chunks per slab, channels, outer) where d.grid3 says so.
template <typename K>
static void launch_tensor(K kernel, unsigned blocks, hipStream_t st, const DevTensor &d)
{
    const dim3 grid = d.grid3 ? dim3(d.cps, d.channels, d.outer) : dim3(blocks);
    hipLaunchKernelGGL(kernel, grid, dim3(kBlock), 0, st, d);
}

template <typename T, bool WAVES>
static void launch_forward_single(const DevTensor &d, unsigned blocks, hipStream_t st)
{
    if (!d.q) launch_tensor(forward_kernel<T, true, false, WAVES>, blocks, st, d);
    else if (d.y) launch_tensor(forward_kernel<T, true, true, WAVES>, blocks, st, d);
    else launch_tensor(forward_kernel<T, false, true, WAVES>, blocks, st, d);
}

int launch_forward(const KArgs &a, unsigned blocks, bool emit_q, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (a.table) {
        if (emit_q) launch(forward_multi_kernel<true>, blocks, st, a.table, a.n);
        else launch(forward_multi_kernel<false>, blocks, st, a.table, a.n);
    } else if (a.one.dtype == 0) {
        if (a.one.wave_units) launch_forward_single<_Float16, true>(a.one, blocks, st);
        else launch_forward_single<_Float16, false>(a.one, blocks, st);
    } else {
        if (a.one.wave_units) launch_forward_single<float, true>(a.one, blocks, st);
        else launch_forward_single<float, false>(a.one, blocks, st);
    }
    return (int)hipGetLastError();
}

template <typename T, int SHAPE>
static void launch_backward_typed(const DevTensor &d, unsigned blocks, bool fused_finalize, hipStream_t st)
{
    if (fused_finalize) launch_tensor(backward_kernel<T, true, SHAPE>, blocks, st, d);
    else launch_tensor(backward_kernel<T, false, SHAPE>, blocks, st, d);
}

template <typename T>
static void launch_backward_shaped(const DevTensor &d, unsigned blocks, bool fused_finalize, hipStream_t st)
{
    // The burst schedule stores gx at the very end of a chunk.  Channels that combine by tickets
    // must wait for their stores before they may draw one, so there it would lengthen the tail it
    // is meant to shorten (a 1x128x30x40 FP32 tensor with one scale: 6.7 us instead of 5.7).
    const bool tickets = fused_finalize && d.outer * d.cps > kTreeBlocks;
    if (d.wave_units) launch_backward_typed<T, 1>(d, blocks, fused_finalize, st);
    else if (blocks <= kShortLaunchBlocks && !tickets) launch_backward_typed<T, 2>(d, blocks, fused_finalize, st);
    else launch_backward_typed<T, 0>(d, blocks, fused_finalize, st);
}

static void launch_backward_single(const DevTensor &d, unsigned blocks, bool fused_finalize, hipStream_t st)
{
    if (d.dtype == 0) launch_backward_shaped<_Float16>(d, blocks, fused_finalize, st);
    else launch_backward_shaped<float>(d, blocks, fused_finalize, st);
}

int launch_backward(const KArgs &a, unsigned blocks, bool fused_finalize, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (a.table) {
        if (fused_finalize) launch(backward_multi_kernel<true>, blocks, st, a.table, a.n);
        else launch(backward_multi_kernel<false>, blocks, st, a.table, a.n);
    } else {
        launch_backward_single(a.one, blocks, fused_finalize, st);
    }
    return (int)hipGetLastError();
}

int launch_finalize(const KArgs &a, unsigned total_channels, void *stream)
{
    hipLaunchKernelGGL(finalize_kernel, dim3(total_channels), dim3(kBlock), 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

int launch_scale_only(const KArgs &a, unsigned total_channels, void *stream)
{
    unsigned blocks = (total_channels + kBlock - 1) / kBlock;
    hipLaunchKernelGGL(scale_kernel, dim3(blocks), dim3(kBlock), 0, (hipStream_t)stream, a, total_channels);
    return (int)hipGetLastError();
}

int launch_fill_zero(void *p, size_t bytes, void *stream)
{
    size_t words = bytes / 4;
    if (words == 0) return 0;
    size_t want = (words + kBlock - 1) / kBlock;
    unsigned blocks = (unsigned)(want < 4096 ? want : 4096);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(kBlock), 0, (hipStream_t)stream,
                       (unsigned *)p, words);
    return (int)hipGetLastError();
}

}  // namespace fq
