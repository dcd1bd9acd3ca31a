/*
 * lmkan.h - C ABI of the MI355X (gfx950) implementation of the 2-D lmKAN layer
 * from "Lookup multivariate Kolmogorov-Arnold Networks" (arXiv 2509.07103).
 *
 * The layer (Sec. 3, Eq. 2; Alg. 1): inputs are taken in pairs; every
 * (pair k, output j) owns a bilinear spline table on the sigma grid, and
 *     y[n][j] = sum_k f_{kj}(x[n][2k], x[n][2k+1]).
 * Each f is parametrised by (G+1)^2 coefficients on second-order (piecewise
 * linear) B-splines (Sec. 3.1, Eq. 3); evaluating it needs one cell lookup per
 * pair, shared by all outputs, and four multiply-adds per output (Sec. 3.2).
 *
 * General rules for every entry point
 *   - Pointers whose name ends in _dev are device pointers on the current HIP
 *     device; pointers ending in _host are host pointers.  The caller owns all
 *     of them.  The library allocates no device memory, never synchronises and
 *     enqueues work only on the stream it is given.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Every function that can fail returns an lmkan_status.  Argument errors
 *     are found on the host before anything is launched, so nothing has been
 *     written when a status other than LMKAN_OK or LMKAN_ERR_HIP comes back.
 *   - batch == 0 is legal: nothing is read, and only lmkan_backward writes
 *     (an overwritten grad_coef becomes all zeros).
 *   - Alignment: every tensor its element size.  Faster kernels are chosen at
 *     run time when pointers and widths allow wider accesses (8 bytes for x_dev
 *     and grad_x_dev, 16 bytes for the other tensors).
 *   - Non-finite inputs are memory-safe: cell indices are always clamped to
 *     [0, G-1]; the affected outputs are whatever IEEE arithmetic gives.
 *   - Stream capture: every compute call may be recorded into a HIP graph (no
 *     allocation, no synchronisation, memory is cleared by fill kernels, not by
 *     memset nodes), with one proviso: the first launch, on a device, of a kernel
 *     that needs more than 64 KiB of LDS raises that kernel's limit with
 *     hipFuncSetAttribute, which is not a stream operation.  Make one ordinary
 *     call of the same shape on that device before capturing.
 *   - Host threads: calls may be made from several threads at once (the only
 *     shared host state, which kernels have had their LDS limit raised on which
 *     device and the address of the static scratch, is guarded by mutexes);
 *     lmkan_time_next_kernel arms the calling thread only.
 */
#ifndef LMKAN_H
#define LMKAN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LMKAN_VERSION 1

/* Largest number of grid intervals per axis.  The grid table travels to the
 * kernels by value; the paper's own experiments use G <= 40 (Sec. 3.4). */
#define LMKAN_MAX_GRID 64

/* Largest layer and batch: launch grids index pairs and output tiles with 16-bit
 * block coordinates and rows with 32-bit ones. */
#define LMKAN_MAX_N_IN 131070
#define LMKAN_MAX_N_OUT 4194240
#define LMKAN_MAX_BATCH 2147483647LL

/* Outputs per tile of the packed coefficient layout (see lmkan_pack). */
#define LMKAN_PACK_TILE 64

typedef enum {
    LMKAN_OK = 0,
    LMKAN_ERR_NULL = 1,        /* a required pointer is NULL                       */
    LMKAN_ERR_SHAPE = 2,       /* n_in odd or < 2, n_out < 1, G out of range, batch < 0,
                                  or a size above LMKAN_MAX_N_IN / _N_OUT / _BATCH     */
    LMKAN_ERR_UNSUPPORTED = 3, /* spline order, dtype, layout or flag not implemented  */
    LMKAN_ERR_WORKSPACE = 4,   /* workspace smaller than lmkan_workspace_bytes()   */
    LMKAN_ERR_ALIGN = 5,       /* a pointer is not aligned to its element size     */
    LMKAN_ERR_HIP = 6,         /* the HIP runtime reported an error at launch      */
    LMKAN_ERR_STATIC_LIMIT = 7 /* lmkan_forward_static: the batch needs more scratch
                                  than LMKAN_STATIC_SCRATCH_BYTES                     */
} lmkan_status;

/* Storage type of the coefficient tensor.  Half formats are storage only:
 * values are widened to float32 on load and all arithmetic, accumulation and
 * gradients are float32 (the paper's kernels are float32, Sec. 3.4). */
typedef enum { LMKAN_F32 = 0, LMKAN_F16 = 1, LMKAN_BF16 = 2 } lmkan_dtype;

typedef enum {
    LMKAN_LAYOUT_PAPER = 0, /* [G+1][G+1][n_in/2][n_out], last index fastest (Alg. 1) */
    LMKAN_LAYOUT_PACKED = 1 /* produced by lmkan_pack                                 */
} lmkan_layout;

#define LMKAN_FLAG_ACCUMULATE_GRAD_COEF 1 /* backward adds into grad_coef instead of overwriting */
/* The caller's promise that the workspace still holds the preamble records (cell and local
 * coordinates of every (sample, pair), Alg. 1 "Preamble") that an earlier lmkan_forward,
 * lmkan_backward or lmkan_conv2d_* call wrote for the same desc, batch (or geometry) and the same
 * contents of x: the call then skips the pass that computes them (a training step runs forward
 * and backward on the same x).  It holds only if that earlier call was given a workspace of at
 * least lmkan_workspace_bytes() for its pass, that size was not zero (a call whose size is zero
 * writes no records), the call returned LMKAN_OK,
 * and nothing has written to the first lmkan_workspace_bytes(desc, batch, 0) bytes since
 * (the forward pass's partial outputs lie behind the records and do not matter).  The library
 * cannot check the promise: with stale or foreign contents the records are garbage used as
 * table indices, which is as undefined as a wrong pointer. */
#define LMKAN_FLAG_WORKSPACE_HAS_RECORDS 2

/* Description of one layer (Alg. 1 "Require"). */
typedef struct {
    int32_t n_in;         /* input width, even, 2 .. LMKAN_MAX_N_IN (Eq. 2 with d = 2)   */
    int32_t n_out;        /* output width, 1 .. LMKAN_MAX_N_OUT                          */
    int32_t grid;         /* G: grid intervals per axis, 3 <= G <= LMKAN_MAX_GRID.
                             G-1 real grid points plus two ghost points (App. B)        */
    int32_t spline_order; /* must be 2: the paper's second-order (piecewise linear)
                             B-splines, two non-zero per axis (Sec. 3.1)                 */
    int32_t coef_dtype;   /* lmkan_dtype of the coefficient tensor                       */
    int32_t coef_layout;  /* lmkan_layout of the coefficient tensor                      */
    int32_t flags;        /* LMKAN_FLAG_* or 0                                           */
} lmkan_desc;

/* Library version (LMKAN_VERSION it was built with). */
int lmkan_version(void);

/* Static, human-readable name of a status code. */
const char *lmkan_status_string(lmkan_status status);

/*
 * The extended grid of Sec. 3.1 / App. B as the kernels use it, on the host.
 *   nodes_host [G+1]: nodes[1..G-1] are the real grid points, where
 *       sigma(x) = k/G with sigma from App. B Eq. 5; nodes[0] and nodes[G] are
 *       the ghost points first-(second-first) and its mirror image.  Computed
 *       in double and rounded once to float32.
 *   inv_h_host [G]: 1 / (nodes[i+1] - nodes[i]) of the float32 nodes, rounded to
 *       float32.  Either pointer may be NULL to skip that output.
 * The cell of an input x is defined on this table: i = number of real grid
 * points <= x, which is floor(sigma(x) G) of Sec. 3.1 in exact arithmetic.
 */
lmkan_status lmkan_grid(int32_t grid, float *nodes_host, float *inv_h_host);

/*
 * Bytes of the packed coefficient tensor for this layer: n_out is padded to a
 * multiple of LMKAN_PACK_TILE and the tensor is stored as
 * [n_out_tiles][n_in/2][(G+1)^2][LMKAN_PACK_TILE] in desc->coef_dtype, so the
 * table rows one workgroup needs for one pair are contiguous.  0 on bad desc.
 * The tuned kernels move four adjacent outputs at a time: they take any n_out
 * with a packed table (padding columns must hold finite values; lmkan_pack
 * writes zeros), and n_out that is a multiple of four with a table in the
 * layout of Alg. 1; other layers in that layout run on slower general kernels.
 * A layer with one output is quickest with its table left in the layout of
 * Alg. 1 (contiguous over the pairs; packing pads it to 64 columns).
 */
size_t lmkan_packed_bytes(const lmkan_desc *desc);

/*
 * Repack a coefficient tensor from the layout of Alg. 1 into the packed
 * layout (same dtype; padding columns are zero).  desc->coef_layout is
 * ignored.  src and dst must not overlap.
 */
lmkan_status lmkan_pack(const lmkan_desc *desc, const void *coef_paper_dev, void *coef_packed_dev,
                        void *stream);

/*
 * Device scratch memory a call needs for this batch size; may be 0.
 *   pass = 0  lmkan_forward: the preamble records of Alg. 1 (cell and local coordinates
 *             per (sample, pair), 12 bytes each) and, when few samples and outputs
 *             leave compute units idle and the pairs are therefore split over several
 *             workgroups, one [batch][n_out] float32 partial output per extra split
 *             (summed in a fixed order: the forward result does not vary between
 *             runs, except where the kernels for very few outputs run (one output,
 *             or up to eight where no slab kernel applies): their splits add
 *             atomically).  Zero for a layer with one output whose tables fit on
 *             chip 64 pairs at a time (G <= 24, or fewer pairs): its forward kernel
 *             locates the inputs itself and writes no records.
 *   pass = 1  lmkan_backward with both gradients; 2: grad_x only; 3: grad_coef only.
 *             The same records; their copy sorted by cell (16 bytes per (sample,
 *             pair) plus per-pair tables) when a kernel that walks it can serve the
 *             shape; for grad_x a transposed float32 copy of it and, for grids too
 *             fine for the slab kernels, its per-output-tile partial sums (8 bytes
 *             per (sample, pair) and 64 outputs).  The size for pass = 1 covers the
 *             other two.
 * The contents are scratch: nothing is kept between calls, and two calls that share a
 * workspace must not overlap in time.  Any other pass gives 0.
 */
size_t lmkan_workspace_bytes(const lmkan_desc *desc, int64_t batch, int32_t pass);

/*
 * Cell lookup alone (the first two lines of Alg. 1's preamble):
 *   cell_dev[n][k] = i1 * G + i2 for the pair (x[n][2k], x[n][2k+1]),
 * int32, [batch][n_in/2] row-major, overwritten.  Only n_in and grid of the
 * descriptor are used.
 */
lmkan_status lmkan_locate(const lmkan_desc *desc, int64_t batch, const float *x_dev,
                          int32_t *cell_dev, void *stream);

/*
 * Layer forward (Alg. 1) for a batch.
 *   x_dev    [batch][n_in]  float32 row-major
 *   coef_dev coefficient tensor in desc->coef_dtype / desc->coef_layout
 *   y_dev    [batch][n_out] float32 row-major, overwritten
 *   workspace_dev / workspace_bytes: at least lmkan_workspace_bytes(desc, batch, 0)
 *            bytes of device memory, 256-byte aligned (NULL allowed when 0)
 */
lmkan_status lmkan_forward(const lmkan_desc *desc, int64_t batch, const float *x_dev,
                           const void *coef_dev, float *y_dev, void *workspace_dev,
                           size_t workspace_bytes, void *stream);

/*
 * lmkan_forward for callers that cannot bring a workspace because they cannot allocate
 * one: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same kernels and same result as lmkan_forward; the
 * preamble records and partial outputs live in a buffer of LMKAN_STATIC_SCRATCH_BYTES
 * that is part of the library itself (one copy on every GPU the library runs on, kept
 * until the process ends).  The call allocates nothing and frees nothing.
 *   - LMKAN_ERR_STATIC_LIMIT when lmkan_workspace_bytes(desc, batch, 0) exceeds the
 *     buffer (nothing is launched); LMKAN_ERR_HIP when the runtime cannot name the
 *     buffer's address.
 *   - All calls on one GPU share the buffer: two of them must not overlap in time
 *     (different streams, or host threads, without ordering between them race).
 *   - The first call on a device looks the buffer's address up
 *     (hipGetSymbolAddress); make it outside any stream capture.
 */
#define LMKAN_STATIC_SCRATCH_BYTES (32u << 20)
lmkan_status lmkan_forward_static(const lmkan_desc *desc, int64_t batch, const float *x_dev,
                                  const void *coef_dev, float *y_dev, void *stream);

/*
 * Layer backward: derivatives of Alg. 1's four-term sum.
 *   grad_y_dev    [batch][n_out] float32, gradient of the loss w.r.t. y
 *   grad_x_dev    [batch][n_in]  float32, overwritten; NULL skips it.  On a grid
 *                 point the derivative of the cell on its right is returned.
 *   grad_coef_dev float32 in the layout of Alg. 1, [G+1][G+1][n_in/2][n_out],
 *                 whatever the storage type and layout of coef_dev; overwritten
 *                 (entries no sample touches become exactly 0, cf. Sec. 3.5)
 *                 unless LMKAN_FLAG_ACCUMULATE_GRAD_COEF is set; NULL skips it.
 *   coef_dev      may be NULL when grad_x_dev is NULL.
 *   workspace_dev / workspace_bytes: at least lmkan_workspace_bytes(desc, batch, 1),
 *                 256-byte aligned.
 * Sums are float32.  Run-to-run variation: the counting sort by cell is stable
 * (samples of a cell stay in index order), so a grad_coef written by the
 * cell-sorted kernels repeats bit for bit when every (pair, 64-output tile) is
 * walked by one wave (batch <= 12288 rows and at least 4096 (pair, tile) streams,
 * e.g. 1024 -> 1024); shorter layers and longer batches cut the streams into
 * runs that meet through float32 atomics, and the generic kernels and the
 * kernels for very few outputs use atomics throughout: there the last bits can
 * differ.  grad_x repeats bit for bit on the
 * sorted walk (grids finer than 34 intervals) and in the kernels for very few
 * outputs (one output, or up to eight where no slab kernel applies); the slab
 * kernels (grids up to 34) add their output tiles with float32 atomics.
 */
lmkan_status lmkan_backward(const lmkan_desc *desc, int64_t batch, const float *x_dev,
                            const void *coef_dev, const float *grad_y_dev, float *grad_x_dev,
                            float *grad_coef_dev, void *workspace_dev, size_t workspace_bytes,
                            void *stream);

/*
 * Off-diagonal Hessian regulariser of the layer (Sec. 3.5, App. C).  For every 2-D
 * function (pair, output) and every table node with a full stencil (both indices
 * in [1, G-1]; ghost-node coefficients enter as neighbours) App. C's finite
 * differences on the non-uniform grid give D11, D22, D12 and
 * H = D11^2 + 2 D12^2 + D22^2; a function contributes the mean of H over those
 * (G-1)^2 nodes, the layer the sum over its functions.
 *   coef_dev      coefficients in desc->coef_dtype / desc->coef_layout
 *   value_dev     one double on the device, overwritten with the layer's value
 *                 (unscaled); NULL skips it
 *   grad_coef_dev float32 in the layout of Alg. 1: receives scale * d value / d coef,
 *                 overwritten, or added to when LMKAN_FLAG_ACCUMULATE_GRAD_COEF is
 *                 set (so it can share the buffer lmkan_backward wrote); NULL skips it
 * The value is a sum of per-wave partial sums through a double atomic: its last
 * bits can differ from run to run.  No workspace.
 */
lmkan_status lmkan_hessian_reg(const lmkan_desc *desc, const void *coef_dev, float scale, double *value_dev,
                               float *grad_coef_dev, void *stream);

/*
 * Inference-time folds, in place on a float32 table (App. E Eq. 4b, App. F.1).
 * The ReLU-first preconditioned layer followed by an evaluation-mode batch
 * normalisation,
 *     y'_j = s_j (gamma lmKAN(x) + Linear(ReLU(x)))_j + t_j,
 * becomes a plain lmKAN layer with
 *     P'[a][b][k][j] = s_j (gamma P[a][b][k][j] + Wl[j][2k] max(E[a],0) + Wl[j][2k+1] max(E[b],0))
 *                      + [k == 0] (s_j bias_j + t_j).
 * The ReLU part is exact only when 0 is a grid point (grid even); the library does
 * not check this, and the other terms are exact for any grid.
 *   coef_dev       float32 table in desc->coef_layout, overwritten
 *                  (LMKAN_ERR_UNSUPPORTED for 16-bit tables: fold first, round after)
 *   gamma          weight of the lmKAN term (1 leaves it as it is)
 *   lin_w_dev      [n_out][n_in] float32 row-major, weight of Linear; NULL = no such term
 *   lin_b_dev      [n_out] bias of Linear; NULL = none
 *   out_scale_dev  [n_out] s_j; NULL = 1
 *   out_shift_dev  [n_out] t_j; NULL = 0
 */
lmkan_status lmkan_fold(const lmkan_desc *desc, void *coef_dev, float gamma, const float *lin_w_dev,
                        const float *lin_b_dev, const float *out_scale_dev, const float *out_shift_dev,
                        void *stream);

/*
 * For callers that measure (benchmarks; not part of the paper's method): the next
 * lmkan_forward / lmkan_backward / lmkan_conv2d_* call made by this host thread records
 * start_event on its stream right before its main kernel and stop_event right after it,
 * leaving out the passes around it (preamble records, sorting, zero fills, transposes,
 * partial sums).  The main kernel is the forward kernel; for a backward call the
 * input-gradient kernel when grad_x is requested, else the coefficient-gradient kernel.
 * Both are hipEvent_t created by the caller with timing enabled; the pair is used once.
 * Two NULLs disarm; one NULL is LMKAN_ERR_NULL.  A call that launches no such kernel
 * (empty batch, argument error) leaves the events armed for the next call.
 */
lmkan_status lmkan_time_next_kernel(void *start_event, void *stop_event);

/*
 * For callers that measure (not part of the paper's method): what this machine delivers on the
 * primitive streams the kernels are made of, to be quoted next to the published peaks.
 *   which         LMKAN_MICROBENCH_*: HBM copy and read (GB/s, bytes read + written), independent
 *                 float32 multiply-adds on the vector pipe and as 4x4x1 MFMAs (multiply-adds per
 *                 clock and compute unit, at the nominal clock the runtime reports), 16-byte
 *                 LDS reads and writes (bytes per clock and compute unit), gathers of 256-byte
 *                 rows from a 2 MiB table (bytes per clock and compute unit)
 *   scratch_dev   at least 64 MiB of device memory, 256-byte aligned, contents destroyed
 *   result_host   one double on the host
 * Unlike every other entry point this one creates two HIP events and waits for its kernels
 * (about ten short launches on `stream`) before it returns.
 */
#define LMKAN_MICROBENCH_COPY_GBPS 0
#define LMKAN_MICROBENCH_READ_GBPS 1
#define LMKAN_MICROBENCH_FMA_PER_CLK_CU 2
#define LMKAN_MICROBENCH_MFMA_FMA_PER_CLK_CU 3
#define LMKAN_MICROBENCH_LDS_READ_B_PER_CLK_CU 4
#define LMKAN_MICROBENCH_LDS_WRITE_B_PER_CLK_CU 5
#define LMKAN_MICROBENCH_GATHER_B_PER_CLK_CU 6
#define LMKAN_MICROBENCH_NOMINAL_CLOCK_GHZ 7 /* no kernel: the clock the "per clock" figures refer to */
#define LMKAN_MICROBENCH_COUNT 8
lmkan_status lmkan_microbench(int32_t which, void *scratch_dev, size_t scratch_bytes, double *result_host,
                              void *stream);

/*
 * Convolution (Sec. 5, "lmKAN-based Convolutional Neural Networks"): a kh x kw
 * convolution is the layer R^{kh kw c_in} -> R^{n_out} applied to every window of a
 * channels-last image.  The paper reshapes the windows into rows first; here the rows
 * are never written out: the kernels read the image through the window map.
 *   image   x[n][h][w][c_in] float32, no padding
 *   window  (oy, ox) covers rows oy*stride .. oy*stride + kh - 1 and columns
 *           ox*stride .. ox*stride + kw - 1;  out_h = (h - kh) / stride + 1 (floor),
 *           out_w likewise (0 when the image is smaller than the window)
 *   input   e = (ky*kw + kx)*c_in + c of the layer is x[img][oy*stride+ky][ox*stride+kx][c];
 *           desc->n_in must equal kh*kw*c_in (even); with an odd c_in the two inputs of
 *           a pair can come from neighbouring pixels
 *   output  y[n][out_h][out_w][n_out]
 */
typedef struct lmkan_conv2d {
    int32_t n, h, w, c_in;
    int32_t kh, kw, stride;
} lmkan_conv2d;

/* Rows of the equivalent fully connected layer, n*out_h*out_w (the `batch` to pass to
 * lmkan_workspace_bytes); writes out_h / out_w when not NULL.  -1 for an invalid struct. */
int64_t lmkan_conv2d_rows(const lmkan_conv2d *conv, int32_t *out_h, int32_t *out_w);

/*
 * Forward and backward of the convolution.  Arguments as for lmkan_forward /
 * lmkan_backward with batch = lmkan_conv2d_rows(conv): grad_y_dev is
 * [n][out_h][out_w][n_out]; grad_x_dev has the shape of the image and is
 * overwritten (every element gets the sum over the windows that contain it, zero
 * where no window does); grad_coef_dev as in lmkan_backward.  x_dev, grad_x_dev
 * need 4-byte alignment only.  workspace: lmkan_workspace_bytes(desc, rows, pass).
 * LMKAN_ERR_SHAPE when desc->n_in != kh*kw*c_in or a size is not positive.
 * For shapes the tuned kernels do not take, grad_x is summed with float32 atomics
 * (sum order, and so the last bits, can differ between runs).
 */
lmkan_status lmkan_conv2d_forward(const lmkan_desc *desc, const lmkan_conv2d *conv, const float *x_dev,
                                  const void *coef_dev, float *y_dev, void *workspace_dev, size_t workspace_bytes,
                                  void *stream);
lmkan_status lmkan_conv2d_backward(const lmkan_desc *desc, const lmkan_conv2d *conv, const float *x_dev,
                                   const void *coef_dev, const float *grad_y_dev, float *grad_x_dev,
                                   float *grad_coef_dev, void *workspace_dev, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LMKAN_H */
