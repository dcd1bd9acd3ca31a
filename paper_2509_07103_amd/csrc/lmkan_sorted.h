// The cell-sorted sample stream shared by the backward kernels (lmkan_backward.hip builds it,
// lmkan_backward.hip and lmkan_backward_fused.hip walk it), and the matrix-core pieces both use.
//
// For every pair k the samples are grouped by the cell their two inputs fall in (counting
// sort), every non-empty cell padded to whole chunks of four samples.  Inside a cell the
// gradients are small dense contractions over the samples of the cell (Alg. 1's four-term sum,
// differentiated), which is what lets them run on the matrix cores.
#pragma once

#include "lmkan_kernels.h"

namespace lmkan {

typedef float f4v __attribute__((ext_vector_type(4)));
typedef unsigned u2v __attribute__((ext_vector_type(2)));

constexpr int kChunk = 4;    // samples per chunk; a chunk never straddles two cells
constexpr int kUnroll = 16;  // chunks per trip of the walking kernels' main loops
constexpr int kSortSeg = 4096;       // samples per workgroup in the count and scatter passes
// A wave reads gy rows in the order of the sorted stream, i.e. all over the batch; as long as
// the 64-column slice of gy (256 bytes per sample) fits the L2 of an XCD next to the streams,
// the waves of that XCD share it.  Longer batches are cut into blocks of kBlockSamples samples,
// the stream of a pair is sorted by (block, cell), and all waves of an XCD work on one block
// at a time.
constexpr int kBlockSamples = 8192;  // 2 MiB of gy per block and 64-column tile
constexpr int kSegPerBlock = kBlockSamples / kSortSeg;

__host__ __device__ inline int stream_blocks(int64_t B)
{
    return B > kBlockSamples + kBlockSamples / 2 ? (int)((B + kBlockSamples - 1) / kBlockSamples) : 1;
}

// Entries per pair in the sorted stream: every non-empty (block, cell) is padded to whole
// chunks, every block to whole trips of kUnroll chunks, and the end is padded so that the
// walking kernels can prefetch up to three trips beyond the last one without bounds checks
// (the first trip of that padding holds valid filler entries, the rest is never dereferenced
// as a sample index).
__host__ __device__ inline int64_t stream_stride(int64_t B, int G)
{
    const int64_t blocks = stream_blocks(B);
    const int64_t body = B + blocks * ((int64_t)(kChunk - 1) * G * G + (int64_t)kChunk * kUnroll);
    return (body + kChunk - 1) / kChunk * kChunk + (int64_t)kChunk * (3 * kUnroll);
}

// One entry of the stream, 16 bytes: the local coordinates of Alg. 1's preamble
// (u, v: the four B-spline products are (1-u)(1-v), u(1-v), (1-u)v, uv), a factor that is 1 for
// a sample and 0 for a padding entry, and the sample index (bit pattern of an int32).  Padding
// entries repeat the index of a sample of the same cell, so that what they multiply is a value
// the cell sees anyway.
struct SortedStream {
    const f4v *rec;              // [K][S]
    const int32_t *chunk_cell;   // [K][S/4]  i1 << 8 | i2 of the cell each chunk belongs to,
                                 //           non-decreasing inside a block
    const int32_t *block_start;  // [K][blocks + 1]  first chunk of every block (multiples of
                                 //           kUnroll) and the number of chunks to process
    int64_t S;                   // stream_stride
    int n_blocks;
};

// Workspace carved up for the sort: the stream above plus the tables the sort passes hand to
// each other.
struct SortBuffers {
    f4v *rec;
    int32_t *chunk_cell;
    int32_t *block_start;
    int32_t *block_size;
    int32_t *seg_count;
    int32_t *cell_start;
    int32_t *cell_rep;
};
SortBuffers sort_buffers(const LayerShape &s, void *sorted);
// records = output of launch_preamble_records; fills the stream in `sorted`
// (sorted_records_bytes()) and returns its description
SortedStream launch_sort(const LayerShape &s, const void *records, void *sorted, hipStream_t stream);
// whether the batch is short enough for the 32-bit stream positions and 16-bit grid coordinates
bool sorted_batch_ok(const LayerShape &s);
// waves per (pair, output tile, block) of the walking kernels
int stream_run_split(const LayerShape &s);

// gy as the walking kernels gather it: the 64 columns of output tile t of row n start at
// base + t * tile_stride + n * row_stride (bytes).  The gradient as the caller holds it,
// [batch][n_out], is such a view with strides 256 and 4 n_out; but the rows of one tile then sit
// 4 n_out bytes apart, a power-of-two stride for the usual widths, and pile up on a few sets of
// the L2 (a 1 MB tile slice of a 4096-wide layer misses four times in ten).  For wide layers
// launch_gy_tiles copies gy once into [tiles][batch][64] (columns past n_out zero), where a tile
// slice is contiguous; for narrower ones it returns the view of gy itself.
struct GyView {
    const float *base;
    int64_t tile_stride;
    unsigned row_stride;
};
size_t gy_tiles_bytes(const LayerShape &s);
GyView launch_gy_tiles(const LayerShape &s, const float *gy, void *tiles, hipStream_t stream);
bool gy_offsets_fit_32_bits(const LayerShape &s, const GyView &gy);
// coefficient gradient alone (lmkan_backward.hip)
void launch_backward_coef_sorted(const LayerShape &s, const SortedStream &st, const GyView &gy, float *gcoef,
                                 bool accumulate, hipStream_t stream);

// input gradient, with the coefficient gradient when gcoef is not NULL (lmkan_backward_fused.hip).
// `partial` is scratch of fused_partial_bytes(); the result goes to gx [batch][n_in], or, when
// gx_transposed is not NULL, to that scratch as [n_in][batch] (for the convolution).
bool fused_backward_applicable(const LayerShape &s, const void *coef, const float *gy, const float *gcoef);
void launch_backward_fused(const LayerShape &s, const GridTab &tab, const SortedStream &st, const void *records,
                           const void *coef, const GyView &gy, float *gx, float *gcoef, bool accumulate,
                           void *partial, float *gx_transposed, hipStream_t stream);

// acc[i][q] += (product q of this group's sample) * gy[i] for the chunk whose products sit in
// quad SUB of every group of `w` (lane 16 g + 4 SUB + q holds product q of group g's sample).
// One MFMA is 16 independent 4x4 outer products, block b = lanes 4b .. 4b+3: the A operand of
// the four blocks of a group is taken from the group's block SUB (broadcast size 4 blocks),
// the B operand is the lane's own gy value, and row q of the result lands in register q of
// the same lane.
template <int SUB, bool FRESH>
__device__ __forceinline__ void chunk_fma(f4v (&acc)[4], float w, const f4v &g)
{
    // the first chunk of a cell starts from zero instead of clearing the accumulators
    const f4v zero = {0.f, 0.f, 0.f, 0.f};
    acc[0] = __builtin_amdgcn_mfma_f32_4x4x1f32(w, g.x, FRESH ? zero : acc[0], 2, SUB, 0);
    acc[1] = __builtin_amdgcn_mfma_f32_4x4x1f32(w, g.y, FRESH ? zero : acc[1], 2, SUB, 0);
    acc[2] = __builtin_amdgcn_mfma_f32_4x4x1f32(w, g.z, FRESH ? zero : acc[2], 2, SUB, 0);
    acc[3] = __builtin_amdgcn_mfma_f32_4x4x1f32(w, g.w, FRESH ? zero : acc[3], 2, SUB, 0);
}

// The four groups' partial sums acc[output i][corner q] -> f[i] of group r = total of corner r,
// output i.  Two rounds of "swap halves of two registers, add": the first pairs corner q
// with corner q + 2 across the 32-lane halves, the second pairs the results across odd and
// even 16-lane rows.
__device__ __forceinline__ void combine_groups(const f4v (&acc)[4], float (&f)[4])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float z[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            // upper half of acc[q] <-> lower half of acc[q + 2]
            const u2v s = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[i][q]),
                                                           __float_as_uint(acc[i][q + 2]), false, false);
            z[q] = __uint_as_float(s.x) + __uint_as_float(s.y);  // rows 0,1: corner q; rows 2,3: corner q + 2
        }
        // odd rows of z[0] <-> even rows of z[1]
        const u2v s = __builtin_amdgcn_permlane16_swap(__float_as_uint(z[0]), __float_as_uint(z[1]), false, false);
        f[i] = __uint_as_float(s.x) + __uint_as_float(s.y);
    }
}

// product q = (lane & 3) of an entry: ((1-u)(1-v), u(1-v), (1-u)v, uv)[q] times the entry's factor
__device__ __forceinline__ float entry_product(const f4v &e, int q)
{
    const float a = (q & 1) ? e.x : 1.0f - e.x;
    const float b = (q & 2) ? e.y : 1.0f - e.y;
    return a * b * e.z;
}

}  // namespace lmkan
