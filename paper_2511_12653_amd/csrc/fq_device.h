// Device helpers shared by the gfx950 kernels: the DPP wavefront reduction and the address-space
// qualified memory accesses.  Included by .hip files only; not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fq {
namespace dev {

// ---------------------------------------------------------------------------------------------
// Reductions, all in DPP (a binary64 value moves as its two 32-bit halves): butterflies inside
// rows of 16 lanes, then row_bcast15 / row_bcast31 carry the row sums across rows.  The sum of
// the whole wavefront ends in lanes 48..63 (kSumLane reads it); the order of additions is fixed.
template <int CTRL, int ROW_MASK> __device__ __forceinline__ double dpp_move(double v)
{
    typedef int i32x2 __attribute__((ext_vector_type(2)));
    i32x2 w = __builtin_bit_cast(i32x2, v);
    w[0] = __builtin_amdgcn_update_dpp(0, w[0], CTRL, ROW_MASK, 0xf, false);   // masked rows get 0
    w[1] = __builtin_amdgcn_update_dpp(0, w[1], CTRL, ROW_MASK, 0xf, false);
    return __builtin_bit_cast(double, w);
}

constexpr int kSumLane = 63;

__device__ __forceinline__ double wave_sum(double v)
{
    v += dpp_move<0xB1, 0xf>(v);    // quad_perm [1,0,3,2]
    v += dpp_move<0x4E, 0xf>(v);    // quad_perm [2,3,0,1]
    v += dpp_move<0x141, 0xf>(v);   // row_half_mirror
    v += dpp_move<0x140, 0xf>(v);   // row_mirror: every lane now holds its row's sum
    v += dpp_move<0x142, 0xa>(v);   // row_bcast15: rows 1 and 3 add the row before them
    v += dpp_move<0x143, 0xc>(v);   // row_bcast31: rows 2 and 3 add rows 0+1
    return v;
}

// ---------------------------------------------------------------------------------------------
// Memory access helpers.  Pointers inside the descriptor are generic; naming the address space
// gives global_load/global_store (not flat) for tensor data and scalar (SMEM) loads for values
// that are uniform over the block and never written while a kernel runs (theta, the table).
#define FQ_GLOBAL __attribute__((address_space(1)))
#define FQ_CONST __attribute__((address_space(4)))

template <typename U> __device__ __forceinline__ U ld_global(const U *p) { return *(const FQ_GLOBAL U *)p; }
template <typename U> __device__ __forceinline__ void st_global(U *p, U v) { *(FQ_GLOBAL U *)p = v; }

// Tensor data is touched exactly once per kernel: stream it (non-temporal hint) so it does not
// displace anything useful from the caches.
#ifndef FQ_NONTEMPORAL
#define FQ_NONTEMPORAL 1
#endif
template <typename U> __device__ __forceinline__ U ld_stream(const U *p)
{
#if FQ_NONTEMPORAL
    return __builtin_nontemporal_load((const FQ_GLOBAL U *)p);
#else
    return *(const FQ_GLOBAL U *)p;
#endif
}
template <typename U> __device__ __forceinline__ void st_stream(U *p, U v)
{
#if FQ_NONTEMPORAL
    __builtin_nontemporal_store(v, (FQ_GLOBAL U *)p);
#else
    *(FQ_GLOBAL U *)p = v;
#endif
}
template <typename U> __device__ __forceinline__ U ld_uniform(const U *p) { return *(const FQ_CONST U *)p; }

}  // namespace dev
}  // namespace fq
