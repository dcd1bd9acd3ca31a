// Host side of the C ABI declared in include/lmkan.h: argument validation, the
// grid table, kernel selection.  No entry point allocates or synchronises.
#include <math.h>
#include <string.h>

#include <mutex>
#include <set>
#include <utility>

#include "lmkan.h"
#include "lmkan_kernels.h"
#include "lmkan_sorted.h"

using namespace lmkan;

namespace {

size_t dtype_size(int dtype) { return dtype == LMKAN_F32 ? 4 : 2; }

size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// How a backward workspace is carved up; sizes depend on the shape and on which gradients are
// wanted only (pointer alignment, which also steers the choice of kernels, is not known when the
// caller asks for the size, so every path the shape admits is provided for).
struct BackwardWorkspace {
    size_t records, sorted, scratch, partial, gy_tiles;  // offsets
    size_t total;
};
BackwardWorkspace backward_workspace(const LayerShape &s, bool want_gx, bool want_gp)
{
    BackwardWorkspace w;
    // (mirrors backward_impl: the few-output kernels take the input gradient of such layers, and
    // their coefficient gradient too while a pair's slice of it fits LDS; everything else that
    // can be sorted is, for the coefficient gradient and for the walk that yields both)
    const bool small = small_out_shape_ok(s);
    const bool gp_small = small && small_coef_ok(s);
    const bool sorted = sorted_shape_ok(s) && ((want_gp && !gp_small) || (want_gx && !small));
    w.records = 0;
    w.sorted = align256(records_bytes(s));
    w.scratch = w.sorted + (sorted ? sorted_records_bytes(s) : 0);
    w.partial = w.scratch + (want_gx ? slab_backward_input_scratch_bytes(s) : 0);
    w.gy_tiles = w.partial + (want_gx && !small && sorted ? fused_partial_bytes(s) : 0);
    w.total = w.gy_tiles + (sorted || (want_gx && !small) ? gy_tiles_bytes(s) : 0);
    return w;
}

// Sec. 3.1 "Sigma grid" + App. B: real points where sigma crosses the levels k/G, with
// sigma from Eq. 5 (0.5 e^x on the left half, mirrored on the right), then the two ghost
// points.  Double precision, each entry rounded once to float32; the spacings are taken
// from the rounded points.
lmkan_status build_grid(int G, GridTab *tab)
{
    if (G < 3 || G > LMKAN_MAX_GRID) return LMKAN_ERR_SHAPE;
    double e[LMKAN_MAX_GRID + 1];
    for (int k = 1; k <= G - 1; ++k) {
        const int m = (2 * k <= G) ? k : G - k;
        const double left = log(2.0 * (double)m / (double)G);
        e[k] = (2 * k <= G) ? left : -left;
    }
    e[0] = e[1] - (e[2] - e[1]);
    e[G] = e[G - 1] + (e[G - 1] - e[G - 2]);
    memset(tab, 0, sizeof(*tab));
    tab->G = G;
    for (int k = 0; k <= G; ++k) tab->node[k] = (float)e[k];
    for (int i = 0; i < G; ++i)
        tab->inv_h[i] = (float)(1.0 / ((double)tab->node[i + 1] - (double)tab->node[i]));
    return LMKAN_OK;
}

lmkan_status check_desc(const lmkan_desc *d)
{
    if (d == nullptr) return LMKAN_ERR_NULL;
    if (d->n_in < 2 || (d->n_in & 1) || d->n_out < 1) return LMKAN_ERR_SHAPE;
    if (d->n_in > LMKAN_MAX_N_IN || d->n_out > LMKAN_MAX_N_OUT) return LMKAN_ERR_SHAPE;
    if (d->grid < 3 || d->grid > LMKAN_MAX_GRID) return LMKAN_ERR_SHAPE;
    if (d->spline_order != 2) return LMKAN_ERR_UNSUPPORTED;
    if (d->coef_dtype != LMKAN_F32 && d->coef_dtype != LMKAN_F16 && d->coef_dtype != LMKAN_BF16)
        return LMKAN_ERR_UNSUPPORTED;
    if (d->coef_layout != LMKAN_LAYOUT_PAPER && d->coef_layout != LMKAN_LAYOUT_PACKED)
        return LMKAN_ERR_UNSUPPORTED;
    if (d->flags & ~(LMKAN_FLAG_ACCUMULATE_GRAD_COEF | LMKAN_FLAG_WORKSPACE_HAS_RECORDS)) return LMKAN_ERR_UNSUPPORTED;
    return LMKAN_OK;
}

LayerShape shape_of(const lmkan_desc *d, int64_t batch)
{
    LayerShape s;
    s.batch = batch;
    s.n_in = d->n_in;
    s.n_out = d->n_out;
    s.G = d->grid;
    s.dtype = d->coef_dtype;
    s.layout = d->coef_layout;
    return s;
}

// Errors other code left behind on this host thread are not this call's: entry points that
// launch drop them first and report what their own launches produced.
void drop_stale_error() { (void)hipGetLastError(); }

lmkan_status launch_status()
{
    return hipGetLastError() == hipSuccess ? LMKAN_OK : LMKAN_ERR_HIP;
}

// lmkan_time_next_kernel: events of the calling host thread, and the kind of kernel the call
// in progress wants bracketed
struct TimingState {
    hipEvent_t start = nullptr, stop = nullptr;
    bool armed = false;
    int target = -1;
};
thread_local TimingState g_timing;

// scope of one compute call: chooses the kernel kind, disarms once the events were used
struct TimedCall {
    explicit TimedCall(int kind) { g_timing.target = g_timing.armed ? kind : -1; }
    ~TimedCall() { g_timing.target = -1; }
};

}  // namespace

namespace lmkan {
void allow_large_lds(const void *kernel, int bytes)
{
    static std::mutex mutex;
    static std::set<std::pair<int, const void *>> done;
    int dev = 0;
    (void)hipGetDevice(&dev);
    std::lock_guard<std::mutex> lock(mutex);
    if (done.insert(std::make_pair(dev, kernel)).second)
        (void)hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}
}  // namespace lmkan

KernelTiming::KernelTiming(hipStream_t s, TimedKernel kind) : stream(s), on(g_timing.armed && g_timing.target == (int)kind)
{
    if (on) (void)hipEventRecord(g_timing.start, stream);
}

KernelTiming::~KernelTiming()
{
    if (on) {
        (void)hipEventRecord(g_timing.stop, stream);
        g_timing.armed = false;
        g_timing.target = -1;
    }
}

extern "C" {

int lmkan_version(void) { return LMKAN_VERSION; }

const char *lmkan_status_string(lmkan_status status)
{
    switch (status) {
    case LMKAN_OK: return "ok";
    case LMKAN_ERR_NULL: return "required pointer is NULL";
    case LMKAN_ERR_SHAPE: return "invalid shape (n_in, n_out, grid or batch)";
    case LMKAN_ERR_UNSUPPORTED: return "unsupported spline order, dtype, layout or flag";
    case LMKAN_ERR_WORKSPACE: return "workspace too small";
    case LMKAN_ERR_ALIGN: return "misaligned pointer";
    case LMKAN_ERR_HIP: return "HIP runtime error at launch";
    case LMKAN_ERR_STATIC_LIMIT: return "batch needs more scratch than the library's static buffer holds";
    }
    return "unknown status";
}

lmkan_status lmkan_grid(int32_t grid, float *nodes_host, float *inv_h_host)
{
    GridTab tab;
    const lmkan_status st = build_grid(grid, &tab);
    if (st != LMKAN_OK) return st;
    if (nodes_host) memcpy(nodes_host, tab.node, sizeof(float) * (size_t)(grid + 1));
    if (inv_h_host) memcpy(inv_h_host, tab.inv_h, sizeof(float) * (size_t)grid);
    return LMKAN_OK;
}

size_t lmkan_packed_bytes(const lmkan_desc *desc)
{
    if (check_desc(desc) != LMKAN_OK) return 0;
    const LayerShape s = shape_of(desc, 0);
    return (size_t)s.out_tiles() * (size_t)s.pairs() * (size_t)s.nodes() * LMKAN_PACK_TILE *
           dtype_size(s.dtype);
}

size_t lmkan_workspace_bytes(const lmkan_desc *desc, int64_t batch, int32_t pass)
{
    if (check_desc(desc) != LMKAN_OK || batch <= 0) return 0;
    const LayerShape s = shape_of(desc, batch);
    // forward: preamble records, then the partial outputs of a forward split over the pairs
    if (pass == 0) {
        if (head_forward_shape_ok(s)) return 0;  // locates its inputs itself
        if (small_out_shape_ok(s)) return records_bytes(s);
        return slab_forward_shape_ok(s) ? align256(records_bytes(s)) + slab_forward_partial_bytes(s) : 0;
    }
    // backward (1: both gradients, 2: grad_x only, 3: grad_coef only): preamble records, their
    // cell-sorted copy, the per-tile partial sums of grad_x, and a transposed copy of grad_x for the
    // paths that finish with a transpose (small outputs, unaligned tables, convolutions)
    if (pass < 1 || pass > 3) return 0;
    const BackwardWorkspace w = backward_workspace(s, pass != 3, pass != 2);
    return w.total;
}

lmkan_status lmkan_pack(const lmkan_desc *desc, const void *coef_paper_dev, void *coef_packed_dev,
                        void *stream)
{
    const lmkan_status st = check_desc(desc);
    if (st != LMKAN_OK) return st;
    if (!coef_paper_dev || !coef_packed_dev) return LMKAN_ERR_NULL;
    const size_t es = dtype_size(desc->coef_dtype);
    if (!aligned(coef_paper_dev, es) || !aligned(coef_packed_dev, es)) return LMKAN_ERR_ALIGN;
    drop_stale_error();
    launch_pack(shape_of(desc, 0), coef_paper_dev, coef_packed_dev, static_cast<hipStream_t>(stream));
    return launch_status();
}

lmkan_status lmkan_locate(const lmkan_desc *desc, int64_t batch, const float *x_dev,
                          int32_t *cell_dev, void *stream)
{
    const lmkan_status st = check_desc(desc);
    if (st != LMKAN_OK) return st;
    if (batch < 0 || batch > LMKAN_MAX_BATCH) return LMKAN_ERR_SHAPE;
    if (batch == 0) return LMKAN_OK;
    if (!x_dev || !cell_dev) return LMKAN_ERR_NULL;
    if (!aligned(x_dev, 4) || !aligned(cell_dev, 4)) return LMKAN_ERR_ALIGN;
    drop_stale_error();
    GridTab tab;
    build_grid(desc->grid, &tab);
    launch_locate(shape_of(desc, batch), tab, x_dev, cell_dev, static_cast<hipStream_t>(stream));
    return launch_status();
}

}  // extern "C"

namespace {

// A plain layer on rows seen as a 1 x 1 convolution on a batch x 1 x 1 image: the window map of
// the kernels then reads and writes x element by element, which is what buffers that are only
// 4-byte aligned need (the row kernels move a pair of inputs, 8 bytes, at once).
ConvGeom rows_as_windows(const LayerShape &s)
{
    ConvGeom g;
    g.N = (int)s.batch, g.H = 1, g.W = 1, g.C = s.n_in, g.kh = 1, g.kw = 1, g.stride = 1, g.OH = 1, g.OW = 1;
    return g;
}

// conv == nullptr: rows x[batch][n_in]; otherwise the rows are the windows of an image
lmkan_status forward_impl(const lmkan_desc *desc, int64_t batch, const float *x_dev, const void *coef_dev,
                          float *y_dev, void *workspace_dev, size_t workspace_bytes, void *stream,
                          const ConvGeom *conv)
{
    const lmkan_status st = check_desc(desc);
    if (st != LMKAN_OK) return st;
    if (batch < 0 || batch > LMKAN_MAX_BATCH) return LMKAN_ERR_SHAPE;
    if (batch == 0) return LMKAN_OK;
    if (!x_dev || !coef_dev || !y_dev) return LMKAN_ERR_NULL;
    if (!aligned(x_dev, 4) || !aligned(y_dev, 4) || !aligned(coef_dev, dtype_size(desc->coef_dtype)))
        return LMKAN_ERR_ALIGN;
    ConvGeom plain;
    if (!conv && !aligned(x_dev, 8)) {
        plain = rows_as_windows(shape_of(desc, batch));
        conv = &plain;
    }
    const size_t need = lmkan_workspace_bytes(desc, batch, 0);
    if (need > 0 && (!workspace_dev || workspace_bytes < need)) return LMKAN_ERR_WORKSPACE;
    if (need > 0 && !aligned(workspace_dev, 256)) return LMKAN_ERR_ALIGN;
    GridTab tab;
    build_grid(desc->grid, &tab);
    const LayerShape s = shape_of(desc, batch);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    drop_stale_error();
    TimedCall timed(kTimeForward);
    // the records are written whenever the shape has a kernel that reads them, also when the
    // alignment of this call's pointers sends it to the generic kernel: a later call may rely on them
    if (need > 0 && !(desc->flags & LMKAN_FLAG_WORKSPACE_HAS_RECORDS))
        launch_preamble_records(s, tab, x_dev, workspace_dev, hs, conv);
    if (head_forward_shape_ok(s)) {
        // one output: no records (need == 0); windows and 4-byte aligned rows go the generic way
        if (!conv)
            launch_forward_head(s, tab, x_dev, coef_dev, y_dev, hs);
        else
            launch_forward_generic(s, tab, x_dev, coef_dev, y_dev, hs, conv);
    } else if (small_out_shape_ok(s)) {
        launch_forward_small(s, coef_dev, y_dev, workspace_dev, hs);
    } else if (slab_forward_applicable(s, coef_dev, y_dev)) {
        float *partials = slab_forward_partial_bytes(s) > 0
                              ? reinterpret_cast<float *>(static_cast<char *>(workspace_dev) + align256(records_bytes(s)))
                              : nullptr;
        launch_forward_slab(s, coef_dev, y_dev, workspace_dev, partials, hs);
    } else {
        launch_forward_generic(s, tab, x_dev, coef_dev, y_dev, hs, conv);
    }
    return launch_status();
}

lmkan_status backward_impl(const lmkan_desc *desc, int64_t batch, const float *x_dev, const void *coef_dev,
                           const float *grad_y_dev, float *grad_x_dev, float *grad_coef_dev, void *workspace_dev,
                           size_t workspace_bytes, void *stream, const ConvGeom *conv)
{
    const lmkan_status st = check_desc(desc);
    if (st != LMKAN_OK) return st;
    if (batch < 0 || batch > LMKAN_MAX_BATCH) return LMKAN_ERR_SHAPE;
    if (!grad_x_dev && !grad_coef_dev) return LMKAN_OK;
    const LayerShape s = shape_of(desc, batch);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const bool overwrite = !(desc->flags & LMKAN_FLAG_ACCUMULATE_GRAD_COEF);
    ConvGeom plain;
    if (!conv && batch > 0 && (!aligned(x_dev, 8) || (grad_x_dev && !aligned(grad_x_dev, 8)))) {
        plain = rows_as_windows(s);
        conv = &plain;
    }
    const size_t image_elems = conv ? (size_t)conv->N * conv->H * conv->W * conv->C : 0;
    drop_stale_error();
    if (batch == 0) {
        // an empty batch still defines the coefficient gradient: all zeros; an image too small for
        // one window still defines its gradient: all zeros
        if ((grad_coef_dev && !aligned(grad_coef_dev, 4)) || (grad_x_dev && !aligned(grad_x_dev, 4)))
            return LMKAN_ERR_ALIGN;
        if (grad_coef_dev && overwrite)
            launch_fill_zero(grad_coef_dev, (size_t)s.nodes() * s.pairs() * s.n_out, hs);
        if (grad_x_dev && image_elems) launch_fill_zero(grad_x_dev, image_elems, hs);
        return launch_status();
    }
    if (!x_dev || !grad_y_dev) return LMKAN_ERR_NULL;
    if (grad_x_dev && !coef_dev) return LMKAN_ERR_NULL;
    if (!aligned(x_dev, 4) || !aligned(grad_y_dev, 4) || (grad_x_dev && !aligned(grad_x_dev, 4)) ||
        (grad_coef_dev && !aligned(grad_coef_dev, 4)) ||
        (coef_dev && !aligned(coef_dev, dtype_size(desc->coef_dtype))))
        return LMKAN_ERR_ALIGN;
    const bool small = small_out_shape_ok(s);
    // one output on rows: kernels that keep the tables (or their gradient) in LDS and locate the
    // inputs themselves: no records, no scratch (windows and 4-byte aligned rows: the kernels below)
    const bool head = head_forward_shape_ok(s) && !conv;
    const bool gx_head = grad_x_dev && head;
    const bool gp_head = grad_coef_dev && head;
    const bool gx_small = grad_x_dev && small && !gx_head;
    const bool gp_small = grad_coef_dev && small && small_coef_ok(s) && !gp_head;
    // Input gradient.  Where a slab kernel applies (G <= 34) it is the faster one for the input
    // gradient alone.  The walk over the cell-sorted samples yields both gradients from one pass
    // over gy: it takes the grids too fine for any slab, and the 16-output slab range when both
    // gradients are wanted and cells hold enough samples for its chunks of four to fill (16 per
    // cell on average), except where the table is packed and two 32-output slabs fit LDS: that slab
    // kernel is as quick as its share of the walk, or quicker.  Whatever neither takes goes to the
    // generic kernel.
    const bool slab_ok = grad_x_dev && !small && slab_backward_input_applicable(s, coef_dev, grad_y_dev, grad_x_dev);
    const bool dense_cells = s.batch >= (int64_t)16 * s.G * s.G;
    const bool fused_pays = !slab_ok || (!slab_tile_is_wide(s) && grad_coef_dev && dense_cells &&
                                         !slab_backward_input_takes_half_tiles(s));
    const bool enough_work = s.batch >= 256 || (int64_t)s.pairs() * s.n_out >= 8192;  // as for the slab kernels
    const bool gx_fused = grad_x_dev && !small && enough_work && fused_pays &&
                          fused_backward_applicable(s, coef_dev, grad_y_dev, grad_coef_dev);
    const bool gx_slab = slab_ok && !gx_fused;
    const bool gp_sorted = grad_coef_dev && !gp_small && !gp_head && coef_sorted_applicable(s, grad_y_dev, grad_coef_dev);
    const bool need_records = gp_sorted || gx_fused || gx_slab || gx_small || gp_small;
    const BackwardWorkspace w = backward_workspace(s, grad_x_dev != nullptr, grad_coef_dev != nullptr);
    const size_t need = need_records ? w.total : 0;
    if (need > 0 && (!workspace_dev || workspace_bytes < need)) return LMKAN_ERR_WORKSPACE;
    if (need > 0 && !aligned(workspace_dev, 256)) return LMKAN_ERR_ALIGN;
    GridTab tab;
    build_grid(desc->grid, &tab);
    char *ws = static_cast<char *>(workspace_dev);
    char *ws_sorted = ws + w.sorted;
    float *ws_scratch = reinterpret_cast<float *>(ws + w.scratch);
    char *ws_partial = ws + w.partial;
    TimedCall timed(grad_x_dev ? kTimeGradInput : kTimeGradCoef);
    if (need_records && !(desc->flags & LMKAN_FLAG_WORKSPACE_HAS_RECORDS)) launch_preamble_records(s, tab, x_dev, ws, hs, conv);
    SortedStream stream_k{};
    GyView gy_k{};
    if (gp_sorted || gx_fused) stream_k = launch_sort(s, ws, ws_sorted, hs);
    // (the slab kernels read gy as it is, except with a ragged output count)
    if (gp_sorted || gx_fused || (gx_slab && ragged_outputs(s))) gy_k = launch_gy_tiles(s, grad_y_dev, ws + w.gy_tiles, hs);
    else gy_k = GyView{grad_y_dev, (int64_t)(LMKAN_PACK_TILE * sizeof(float)), (unsigned)(s.n_out * sizeof(float))};
    if (gp_head) {
        launch_backward_coef_head(s, tab, x_dev, grad_y_dev, grad_coef_dev, !overwrite, hs);
    } else if (gp_small) {
        launch_backward_coef_small(s, ws, grad_y_dev, grad_coef_dev, !overwrite, hs);
    } else if (gp_sorted && !gx_fused) {
        launch_backward_coef_sorted(s, stream_k, gy_k, grad_coef_dev, !overwrite, hs);
    } else if (grad_coef_dev && !gx_fused) {
        // odd output counts or unaligned buffers: atomics on a gradient that starts at zero
        if (overwrite) launch_fill_zero(grad_coef_dev, (size_t)s.nodes() * s.pairs() * s.n_out, hs);
        launch_backward_generic(s, tab, x_dev, coef_dev, grad_y_dev, nullptr, grad_coef_dev, hs, conv);
    }
    if (gx_head) {
        launch_backward_input_head(s, tab, x_dev, coef_dev, grad_y_dev, grad_x_dev, hs);
    } else if (gx_fused) {
        // one walk over the cell-sorted samples yields both gradients (the coefficient gradient
        // qualifies whenever the input gradient does)
        launch_backward_fused(s, tab, stream_k, ws, coef_dev, gy_k, grad_x_dev, grad_coef_dev, !overwrite, ws_partial,
                              conv ? ws_scratch : nullptr, hs);
        if (conv) launch_input_gradient_out(ws_scratch, grad_x_dev, s, conv, hs);
    } else if (gx_small) {
        launch_backward_input_small(s, tab, coef_dev, grad_y_dev, ws_scratch, ws, hs);
        launch_input_gradient_out(ws_scratch, grad_x_dev, s, conv, hs);
    } else if (gx_slab) {
        launch_backward_input_slab(s, tab, coef_dev, gy_k.base, gy_k.tile_stride / (int64_t)sizeof(float),
                                   gy_k.row_stride / sizeof(float), grad_x_dev, ws, ws_scratch, hs, conv);
    } else if (grad_x_dev) {
        if (conv) launch_fill_zero(grad_x_dev, image_elems, hs);  // the kernel sums into the image
        launch_backward_generic(s, tab, x_dev, coef_dev, grad_y_dev, grad_x_dev, nullptr, hs, conv);
    }
    return launch_status();
}

// window geometry from the public struct; false when it does not describe a convolution this layer fits
bool conv_geom(const lmkan_desc *desc, const lmkan_conv2d *c, ConvGeom *g)
{
    if (!desc || !c) return false;
    if (c->n < 0 || c->h < 1 || c->w < 1 || c->c_in < 1 || c->kh < 1 || c->kw < 1 || c->stride < 1) return false;
    if ((int64_t)c->kh * c->kw * c->c_in != desc->n_in) return false;
    if ((int64_t)c->n * c->h * c->w * c->c_in > (int64_t)1 << 40) return false;
    g->N = c->n, g->H = c->h, g->W = c->w, g->C = c->c_in, g->kh = c->kh, g->kw = c->kw, g->stride = c->stride;
    g->OH = c->h >= c->kh ? (c->h - c->kh) / c->stride + 1 : 0;
    g->OW = c->w >= c->kw ? (c->w - c->kw) / c->stride + 1 : 0;
    return true;
}

}  // namespace

extern "C" {

lmkan_status lmkan_forward(const lmkan_desc *desc, int64_t batch, const float *x_dev,
                           const void *coef_dev, float *y_dev, void *workspace_dev,
                           size_t workspace_bytes, void *stream)
{
    return forward_impl(desc, batch, x_dev, coef_dev, y_dev, workspace_dev, workspace_bytes, stream, nullptr);
}

lmkan_status lmkan_backward(const lmkan_desc *desc, int64_t batch, const float *x_dev,
                            const void *coef_dev, const float *grad_y_dev, float *grad_x_dev,
                            float *grad_coef_dev, void *workspace_dev, size_t workspace_bytes,
                            void *stream)
{
    return backward_impl(desc, batch, x_dev, coef_dev, grad_y_dev, grad_x_dev, grad_coef_dev, workspace_dev,
                         workspace_bytes, stream, nullptr);
}

}  // extern "C"

namespace {

// Workspace of lmkan_forward_static: part of the library's code object, one copy per GPU,
// kept until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the address kernels can use is looked up once per device.
__device__ __align__(256) unsigned char scratch[LMKAN_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];

// device address of `scratch` on the current device, or nullptr when the runtime refuses
void *static_scratch()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

lmkan_status lmkan_forward_static(const lmkan_desc *desc, int64_t batch, const float *x_dev, const void *coef_dev,
                                  float *y_dev, void *stream)
{
    const lmkan_status st = check_desc(desc);
    if (st != LMKAN_OK) return st;
    if (batch < 0 || batch > LMKAN_MAX_BATCH) return LMKAN_ERR_SHAPE;
    if (batch == 0) return LMKAN_OK;
    const size_t need = lmkan_workspace_bytes(desc, batch, 0);
    if (need > LMKAN_STATIC_SCRATCH_BYTES) return LMKAN_ERR_STATIC_LIMIT;
    if (!x_dev || !coef_dev || !y_dev) return LMKAN_ERR_NULL;
    void *ws = nullptr;
    if (need > 0) {
        ws = static_scratch();
        if (!ws) return LMKAN_ERR_HIP;
    }
    // every byte of the workspace a forward kernel reads was written earlier in the same call
    // (records by the preamble pass, partial outputs by the split workgroups), so what an
    // earlier call left behind needs no clearing
    return forward_impl(desc, batch, x_dev, coef_dev, y_dev, ws, need, stream, nullptr);
}

lmkan_status lmkan_time_next_kernel(void *start_event, void *stop_event)
{
    if ((start_event == nullptr) != (stop_event == nullptr)) return LMKAN_ERR_NULL;
    g_timing.start = static_cast<hipEvent_t>(start_event);
    g_timing.stop = static_cast<hipEvent_t>(stop_event);
    g_timing.armed = start_event != nullptr;
    g_timing.target = -1;
    return LMKAN_OK;
}

int64_t lmkan_conv2d_rows(const lmkan_conv2d *conv, int32_t *out_h, int32_t *out_w)
{
    if (!conv || conv->n < 0 || conv->h < 1 || conv->w < 1 || conv->kh < 1 || conv->kw < 1 || conv->stride < 1)
        return -1;
    const int32_t oh = conv->h >= conv->kh ? (conv->h - conv->kh) / conv->stride + 1 : 0;
    const int32_t ow = conv->w >= conv->kw ? (conv->w - conv->kw) / conv->stride + 1 : 0;
    if (out_h) *out_h = oh;
    if (out_w) *out_w = ow;
    return (int64_t)conv->n * oh * ow;
}

lmkan_status lmkan_conv2d_forward(const lmkan_desc *desc, const lmkan_conv2d *conv, const float *x_dev,
                                  const void *coef_dev, float *y_dev, void *workspace_dev, size_t workspace_bytes,
                                  void *stream)
{
    const lmkan_status st = check_desc(desc);
    if (st != LMKAN_OK) return st;
    if (!conv) return LMKAN_ERR_NULL;
    ConvGeom g;
    if (!conv_geom(desc, conv, &g)) return LMKAN_ERR_SHAPE;
    return forward_impl(desc, (int64_t)g.N * g.OH * g.OW, x_dev, coef_dev, y_dev, workspace_dev, workspace_bytes,
                        stream, &g);
}

lmkan_status lmkan_conv2d_backward(const lmkan_desc *desc, const lmkan_conv2d *conv, const float *x_dev,
                                   const void *coef_dev, const float *grad_y_dev, float *grad_x_dev,
                                   float *grad_coef_dev, void *workspace_dev, size_t workspace_bytes, void *stream)
{
    const lmkan_status st = check_desc(desc);
    if (st != LMKAN_OK) return st;
    if (!conv) return LMKAN_ERR_NULL;
    ConvGeom g;
    if (!conv_geom(desc, conv, &g)) return LMKAN_ERR_SHAPE;
    return backward_impl(desc, (int64_t)g.N * g.OH * g.OW, x_dev, coef_dev, grad_y_dev, grad_x_dev, grad_coef_dev,
                         workspace_dev, workspace_bytes, stream, &g);
}

lmkan_status lmkan_hessian_reg(const lmkan_desc *desc, const void *coef_dev, float scale, double *value_dev,
                               float *grad_coef_dev, void *stream)
{
    const lmkan_status st = check_desc(desc);
    if (st != LMKAN_OK) return st;
    if (!coef_dev) return LMKAN_ERR_NULL;
    if (!value_dev && !grad_coef_dev) return LMKAN_OK;
    if (!aligned(coef_dev, dtype_size(desc->coef_dtype)) || (value_dev && !aligned(value_dev, 8)) ||
        (grad_coef_dev && !aligned(grad_coef_dev, 4)))
        return LMKAN_ERR_ALIGN;
    drop_stale_error();
    GridTab tab;
    build_grid(desc->grid, &tab);
    launch_hessian_reg(shape_of(desc, 0), tab, coef_dev, scale, value_dev, grad_coef_dev,
                       (desc->flags & LMKAN_FLAG_ACCUMULATE_GRAD_COEF) != 0, static_cast<hipStream_t>(stream));
    return launch_status();
}

lmkan_status lmkan_fold(const lmkan_desc *desc, void *coef_dev, float gamma, const float *lin_w_dev,
                        const float *lin_b_dev, const float *out_scale_dev, const float *out_shift_dev,
                        void *stream)
{
    const lmkan_status st = check_desc(desc);
    if (st != LMKAN_OK) return st;
    if (desc->coef_dtype != LMKAN_F32) return LMKAN_ERR_UNSUPPORTED;  // fold first, round to 16 bits after
    if (!coef_dev) return LMKAN_ERR_NULL;
    if (!aligned(coef_dev, 4) || !aligned(lin_w_dev, 4) || !aligned(lin_b_dev, 4) || !aligned(out_scale_dev, 4) ||
        !aligned(out_shift_dev, 4))
        return LMKAN_ERR_ALIGN;
    drop_stale_error();
    GridTab tab;
    build_grid(desc->grid, &tab);
    launch_fold(shape_of(desc, 0), tab, static_cast<float *>(coef_dev), gamma, lin_w_dev, lin_b_dev, out_scale_dev,
                out_shift_dev, static_cast<hipStream_t>(stream));
    return launch_status();
}

}  // extern "C"
