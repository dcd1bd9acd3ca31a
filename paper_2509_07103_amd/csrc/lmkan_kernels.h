// Host-callable launchers of the lmKAN kernels.  Every launcher enqueues on the given
// stream and returns; shapes have been validated by the caller (lmkan_api.hip).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lmkan_device.h"

namespace lmkan {

struct LayerShape {
    int64_t batch;
    int n_in;
    int n_out;
    int G;
    int dtype;   // lmkan_dtype
    int layout;  // lmkan_layout
    int pairs() const { return n_in / 2; }
    int nodes() const { return (G + 1) * (G + 1); }
    int out_tiles() const { return (n_out + LMKAN_PACK_TILE - 1) / LMKAN_PACK_TILE; }
};

CoefMap coef_map(const LayerShape &s);

// The tuned kernels move four adjacent outputs at a time.  That needs rows of the table that
// start on a multiple of four outputs: any n_out in the packed layout (rows padded to 64, the
// padding finite: lmkan_pack writes zeros), a multiple of four in the layout of Alg. 1.  When
// n_out itself is not a multiple of four (`ragged_outputs`), y and the coefficient gradient are
// written element by element in the last columns and gy is read through its tile-by-tile copy.
inline bool ragged_outputs(const LayerShape &s) { return (s.n_out & 3) != 0; }
inline bool outputs_by_four_ok(const LayerShape &s) { return !ragged_outputs(s) || s.layout == LMKAN_LAYOUT_PACKED; }

// Raises the dynamic LDS limit of a kernel on the current device, once per (device, kernel);
// safe to call from several host threads.  The first call for a kernel on a device talks to
// the runtime (hipFuncSetAttribute), so it must not happen inside a stream capture.
void allow_large_lds(const void *kernel, int bytes);


// Generic kernels: any shape, any dtype, both layouts; coefficient rows are read
// straight from global memory.
void launch_forward_generic(const LayerShape &s, const GridTab &tab, const float *x, const void *coef,
                            float *y, hipStream_t stream, const ConvGeom *conv = nullptr);
// with conv, grad_x is summed into gx with atomics: the caller clears it first
void launch_backward_generic(const LayerShape &s, const GridTab &tab, const float *x,
                             const void *coef, const float *gy, float *gx, float *gcoef,
                             hipStream_t stream, const ConvGeom *conv = nullptr);
void launch_locate(const LayerShape &s, const GridTab &tab, const float *x, int32_t *cell,
                   hipStream_t stream);
void launch_pack(const LayerShape &s, const void *src, void *dst, hipStream_t stream);
void launch_fill_zero(float *p, size_t n, hipStream_t stream);

// Tuned float32 forward (lmkan_slab.hip): preamble records in a workspace, coefficient
// slabs streamed through LDS.
size_t records_bytes(const LayerShape &s);
size_t slab_forward_lds_bytes(const LayerShape &s);
bool slab_forward_shape_ok(const LayerShape &s);
bool slab_tile_is_wide(const LayerShape &s);  // 64-output tiles (G <= 16) rather than 16-output ones
bool slab_forward_applicable(const LayerShape &s, const void *coef, const float *y);
void launch_preamble_records(const LayerShape &s, const GridTab &tab, const float *x, void *records,
                             hipStream_t stream, const ConvGeom *conv = nullptr);
// Measurement aid (lmkan_time_next_kernel): while armed, the main kernel of the chosen kind is
// bracketed by the caller's two events on its stream.  Put one in the scope of the launch.
enum TimedKernel { kTimeForward = 0, kTimeGradInput = 1, kTimeGradCoef = 2 };
struct KernelTiming {
    KernelTiming(hipStream_t stream, TimedKernel kind);
    ~KernelTiming();
    hipStream_t stream;
    bool on;
};

// Pair splits of the slab forward (1: none) and the bytes of the split - 1 partial outputs
// [batch][n_out] it then needs; `partials` = NULL makes the splits add into y atomically.
int slab_forward_split(const LayerShape &s);
size_t slab_forward_partial_bytes(const LayerShape &s);
// y[i] += sum over p of part[p][i], i < elems (a multiple of 4)
void launch_sum_partials(float *y, const float *part, int n_part, int64_t elems, hipStream_t stream);
void launch_forward_slab(const LayerShape &s, const void *coef, float *y, const void *records, float *partials,
                         hipStream_t stream);

bool slab_backward_input_shape_ok(const LayerShape &s);
bool slab_backward_input_takes_half_tiles(const LayerShape &s);  // 32-output tiles of a packed table kept as stored
bool slab_backward_input_applicable(const LayerShape &s, const void *coef, const float *gy, const float *gx);
size_t slab_backward_input_scratch_bytes(const LayerShape &s);
// gy as [batch][n_out] (gy_tile_stride = 64, gy_row_stride = n_out, in floats), or its tile-by-tile
// copy [tiles][batch][64] (batch * 64 and 64), which ragged output counts need
void launch_backward_input_slab(const LayerShape &s, const GridTab &tab, const void *coef, const float *gy,
                                int64_t gy_tile_stride, int64_t gy_row_stride, float *gx, const void *records,
                                void *scratch, hipStream_t stream, const ConvGeom *conv = nullptr);

// float16 tables kept as float16 in LDS (lmkan_slab_f16.hip); reached through the two slab
// launchers above when slab_f16_native_ok().  gx_scratch is the zero-filled transposed scratch.
bool slab_f16_native_ok(const LayerShape &s);
void launch_forward_slab_f16(const LayerShape &s, const void *coef, float *y, const void *records, float *partials,
                             hipStream_t stream);
void launch_backward_input_slab_f16(const LayerShape &s, const GridTab &tab, const void *coef, const float *gy,
                                    int64_t gy_tile_stride, int64_t gy_row_stride, float *gx_scratch,
                                    const void *records, hipStream_t stream);

// Layers with one output, or with at most kSmallMaxOut where no slab kernel applies
// (small_out_shape_ok; lmkan_small.hip): a lane is a sample.  All three use
// the preamble records; the input gradient goes to the transposed scratch [n_in][B] (every
// element written, no zero fill needed) and launch_transpose finishes it.
constexpr int kSmallMaxOut = 8;
bool small_out_shape_ok(const LayerShape &s);
bool small_coef_ok(const LayerShape &s);
void launch_forward_small(const LayerShape &s, const void *coef, float *y, const void *records, hipStream_t stream);
// Forward pass of a layer with one output on rows x[batch][n_in] (8-byte aligned): the tables sit
// in LDS and the kernel locates the inputs itself, so the call needs no records and no workspace.
// Applies when at least 64 pairs' tables (or all of them) fit LDS at once.
bool head_forward_shape_ok(const LayerShape &s);
void launch_forward_head(const LayerShape &s, const GridTab &tab, const float *x, const void *coef, float *y,
                         hipStream_t stream);
// its gradients, the same way: x, gy [batch] and grad_x 8-byte aligned rows; grad_coef float32 in
// the layout of Alg. 1
void launch_backward_input_head(const LayerShape &s, const GridTab &tab, const float *x, const void *coef,
                                const float *gy, float *gx, hipStream_t stream);
void launch_backward_coef_head(const LayerShape &s, const GridTab &tab, const float *x, const float *gy,
                               float *gcoef, bool accumulate, hipStream_t stream);
void launch_backward_input_small(const LayerShape &s, const GridTab &tab, const void *coef, const float *gy,
                                 float *gx_scratch, const void *records, hipStream_t stream);
void launch_backward_coef_small(const LayerShape &s, const void *records, const float *gy, float *gcoef,
                                bool accumulate, hipStream_t stream);
void launch_transpose(const float *in_t, float *out, int64_t batch, int n_in, hipStream_t stream);
// the transposed scratch [n_in][rows] -> grad_x: a transpose for a plain layer, for a convolution
// the sum over the patches that contain each input element
void launch_input_gradient_out(const float *in_t, float *gx, const LayerShape &s, const ConvGeom *conv,
                               hipStream_t stream, int scratch_layout = 0);

// Coefficient gradient by cell-sorted samples (lmkan_backward.hip).  `records` is the output
// of launch_preamble_records; `sorted` is scratch of sorted_records_bytes().  Needs n_out to be a
// multiple of 4 and 16-byte aligned gy and gcoef (coef_sorted_applicable); other shapes take the
// generic kernel with atomics on a zeroed gradient.
size_t sorted_records_bytes(const LayerShape &s);
bool sorted_shape_ok(const LayerShape &s);
bool coef_sorted_applicable(const LayerShape &s, const float *gy, const float *gcoef);
// per-tile partial sums of the input gradient from the sorted stream (lmkan_backward_fused.hip)
size_t fused_partial_bytes(const LayerShape &s);

// In-place inference folds of a float32 table (lmkan_fold.hip); absent terms are null pointers.
void launch_fold(const LayerShape &s, const GridTab &tab, float *coef, float gamma, const float *lin_w,
                 const float *lin_b, const float *scale, const float *shift, hipStream_t stream);

// Hessian regulariser (lmkan_hessian.hip): value (double, overwritten; may be null) and
// scale * gradient (float32, layout of Alg. 1; overwritten or added to; may be null).
void launch_hessian_reg(const LayerShape &s, const GridTab &tab, const void *coef, float scale, double *value,
                        float *grad, bool accumulate, hipStream_t stream);

}  // namespace lmkan
