// Pieces shared by the slab-streaming kernels (lmkan_slab.hip, lmkan_slab_f16.hip): kernel
// argument blocks, the LDS-direct load, small DPP helpers.
#pragma once

#include "lmkan_kernels.h"

namespace lmkan {

constexpr int kSlabTile = LMKAN_PACK_TILE;  // 64 outputs per workgroup tile

struct SlabArgs {
    const float *x_unused;
    const void *P;     // float32, or 16-bit storage converted while the slab is filled
    float *y;
    const int32_t *rec_node;
    const float *rec_u;
    const float *rec_v;
    CoefMap map;
    int64_t B;
    int n_out;
    int K;
    int W;             // G + 1
    int nodes;         // W * W
    int col_limit;     // columns >= col_limit do not exist in the coefficient tensor
    int packed;        // 1: packed layout, the slab of (pair, tile) is contiguous
    int pairs_per_split;
    int n_btiles;
    int n_jt;
    int n_split;
    int atomic_out;    // 1: add into y with atomics (split over pairs), 0: plain store
};

// 16 bytes per lane from global memory straight into LDS at lds_base + lane * 16
// (lds_base wave-uniform).  Written as inline assembly on purpose: the compiler does not
// track it, so it cannot make every later LDS read wait for loads that fill the *other*
// buffer; completion is awaited explicitly with s_waitcnt vmcnt(0) before the barrier.
__device__ __forceinline__ void lds_dma16(const void *gptr, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gptr), "s"(lds_base)
                 : "memory");
}

__device__ __forceinline__ unsigned lds_address(const void *p)
{
    return (unsigned)(size_t)(__attribute__((address_space(3))) const void *)p;
}

// Same, with the global address given as a wave-uniform base (scalar registers) plus a 32-bit
// per-lane byte offset: stepping through a contiguous slab then costs scalar instructions only.
__device__ __forceinline__ void lds_dma16_uniform(const void *gbase, unsigned lane_off, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_off), "s"(gbase), "s"(lds_base)
                 : "memory");
}

struct GradInArgs {
    const void *P;     // float32, or 16-bit storage converted while the slab is filled
    const float *gy;
    float *gx;  // transposed scratch [n_in][B], zero on entry
    const int32_t *rec_node;
    const float *rec_u;
    const float *rec_v;
    CoefMap map;
    GridTab tab;
    int64_t B;
    int n_in;
    int n_out;
    int K;
    int W;
    int nodes;
    int pairs_per_split;
    int n_btiles;
    int n_jt;
    int n_split;
    int col_limit;
    int packed;
};

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}

}  // namespace lmkan
