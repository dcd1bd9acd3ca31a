// Pieces shared by the slab-streaming kernels (lmkan_slab.hip, lmkan_slab_f16.hip): kernel
// argument blocks, the LDS-direct load, small DPP helpers.
#pragma once

#include "lmkan_kernels.h"

namespace lmkan {

constexpr int kSlabTile = LMKAN_PACK_TILE;  // 64 outputs per workgroup tile

struct SlabArgs {
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
    // Split over pairs without atomics: the workgroups of split 0 store into y, those of split
    // ks > 0 into y_part + (ks - 1) * part_elems, and a later pass adds the parts to y.
    float *y_part;     // NULL: use atomic_out
    int64_t part_elems;
};

// Pair splits for a launch of `tiles` workgroups over K pairs: double until 256 CUs have work,
// keeping at least four pairs per split.  A workgroup walks its pairs one after the other, a slab
// fill and a barrier each (about 3 us), so few workgroups with many pairs each are bound by that
// latency: with at least 32 pairs per split a 64 -> 64 layer on 4096 rows took 0.10 ms forward and
// 0.15 ms for grad_x whatever the batch, with four 0.034 and 0.044 ms.
// (the input-gradient launchers apply the same rule)
inline int pair_split_count(int tiles, int K)
{
    int split = 1;
    while (tiles * split < 256 && K / (split * 2) >= 4) split *= 2;
    return split;
}

// floats between the partial outputs of consecutive pair splits: a whole number of 16-byte pieces
inline int64_t partial_stride(int64_t elems) { return (elems + 3) & ~(int64_t)3; }

// How the splits of a forward launch combine: separate parts when the caller brought room for
// them, atomics on a cleared y otherwise.
inline void finish_split_setup(SlabArgs &a, const LayerShape &s, float *y, float *partials, hipStream_t stream)
{
    a.y_part = a.n_split > 1 ? partials : nullptr;
    a.part_elems = partial_stride((int64_t)s.batch * s.n_out);
    a.atomic_out = a.n_split > 1 && !a.y_part;
    if (a.atomic_out) launch_fill_zero(y, (size_t)s.batch * s.n_out, stream);
}

// four adjacent outputs of a sample leave the registers: one 16-byte store when every row of y
// starts on a multiple of four outputs, else element by element up to the last column
__device__ __forceinline__ void store_outputs(float *dst, const float *v, int n_out, int col, bool atomic)
{
    if (atomic) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (col + i < n_out) unsafeAtomicAdd(dst + i, v[i]);
    } else if ((n_out & 3) == 0) {
        *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (col + i < n_out) dst[i] = v[i];
    }
}

// where a forward workgroup of pair split ks stores, and whether it has to add atomically
__device__ __forceinline__ float *forward_out_base(const SlabArgs &a, int ks, bool &atomic)
{
    atomic = a.atomic_out && !a.y_part;
    return (a.y_part && ks > 0) ? a.y_part + (int64_t)(ks - 1) * a.part_elems : a.y;
}

// 16 bytes per lane from global memory straight into LDS at lds_base + lane * 16
// (lds_base wave-uniform).  Written as inline assembly on purpose: the compiler does not
// track it, so it cannot make every later LDS read wait for loads that fill the *other*
// buffer; completion is awaited explicitly with s_waitcnt vmcnt(0) before the barrier.
// m0 is overwritten without being listed as clobbered: it is a reserved register to this
// compiler, which rejects it in a clobber list and never keeps a value in it across
// statements (it sets m0 itself right before any instruction of its own that reads it).
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
    const float *gy;   // column c of row n at gy[(c >> 6) * gy_tile_stride + n * gy_row_stride + (c & 63)]
    int64_t gy_tile_stride;
    int64_t gy_row_stride;
    float *gx;  // transposed scratch [n_in][ld], zero on entry
    int64_t ld; // row stride of the scratch: B, or B rounded up to 64 with a permuted layout
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

// Layouts of a row of the transposed scratch gradient.  The slab kernels leave a set of 64
// samples spread over the lanes so that one atomic instruction holds every other run of 8
// (64-output tiles) or 2 (16-output tiles) samples; stored plainly, the instruction would touch
// 32- or 8-byte pieces with gaps.  Inside each aligned block of 64 samples the row is therefore
// permuted so that each instruction covers 128 contiguous bytes:
//   kScratchOct  (64-output tiles): sample s = 16 g + 8 h + i  sits at 32 h + 8 g + i
//   kScratchQuad (16-output tiles): sample s = 4 g + 2 h + i   sits at 32 h + 2 g + i
// Rows are padded to whole blocks.  The kernels that read the scratch undo the permutation.
enum ScratchLayout { kScratchPlain = 0, kScratchOct = 1, kScratchQuad = 2 };

__host__ __device__ inline int64_t scratch_position(int64_t n, int layout)
{
    if (layout == kScratchPlain) return n;
    const int s = (int)(n & 63);
    const int p = layout == kScratchOct ? ((s & 8) << 2) + ((s >> 4) << 3) + (s & 7)
                                        : ((s & 2) << 4) + ((s >> 2) << 1) + (s & 1);
    return (n & ~(int64_t)63) + p;
}

__host__ __device__ inline int64_t scratch_row_stride(int64_t batch, int layout)
{
    return layout == kScratchPlain ? batch : (batch + 63) & ~(int64_t)63;
}

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}

// Cross-lane sums of the 64-output input-gradient kernels, in three pieces (see grad_step in
// lmkan_slab.hip).  stage 1, lanes 8 apart: lanes 0-7 of a row keep d/dx1 (t1), lanes 8-15 d/dx2
// (t2).  A DPP add with a bank mask writes only the enabled quarter rows, so no select is needed.
__device__ __forceinline__ float grad_fold_halves(float t1, float t2)
{
    float v;
    asm("v_add_f32_dpp %0, %1, %1 row_ror:8 row_mask:0xf bank_mask:0x3" : "=v"(v) : "v"(t1));
    asm("v_add_f32_dpp %0, %1, %1 row_ror:8 row_mask:0xf bank_mask:0xc" : "+v"(v) : "v"(t2));
    return v;
}

// stage 2, lanes 4 apart: quarter rows 0 and 2 keep the even step (and add what the quarter row
// above holds of it), quarter rows 1 and 3 the odd one
__device__ __forceinline__ float grad_fold_steps(float even, float odd)
{
    float w;
    asm("v_add_f32_dpp %0, %1, %1 row_ror:12 row_mask:0xf bank_mask:0x5" : "=v"(w) : "v"(even));
    asm("v_add_f32_dpp %0, %1, %1 row_ror:4 row_mask:0xf bank_mask:0xa" : "+v"(w) : "v"(odd));
    return w;
}

// stages 3 and 4, lanes 2 and 1 apart: lanes with bit 1 clear keep the first pair of steps
__device__ __forceinline__ float grad_fold_pairs(float first, float second, bool second_half)
{
    const float keep = second_half ? second : first;
    const float send = second_half ? first : second;
    float z = keep + dpp_move<0x4E>(send);  // quad_perm [2,3,0,1]
    z += dpp_move<0xB1>(z);                 // quad_perm [1,0,3,2]
    return z;
}

}  // namespace lmkan
