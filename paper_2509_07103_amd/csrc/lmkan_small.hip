// Layers with very few outputs: a single output (regression heads), and up to eight outputs where
// the slab kernels do not apply (batches under 256 rows, grids finer than 34 intervals, tables in
// the layout of Alg. 1 whose output count is not a multiple of four).  From two outputs on the
// slab kernels are faster even with most of their 64-output tile empty (256 -> 8, 65536 rows:
// 0.44 ms for both gradients against 2.0 ms here; 256 -> 1: 0.46 against 0.37).
//
// With so few outputs the lanes cannot be outputs: here a lane is a sample and walks over the
// pairs, the preamble records (cell, local coordinates) arriving coalesced along the sample
// axis.  The table of such a layer is small ((G+1)^2 K n_out values) and is gathered from L2.
//   forward:        y[n][j] accumulated in registers over the pairs
//   input gradient: both derivatives of a (sample, pair) come from one lane, written once
//                   into the transposed scratch [n_in][B] (no atomics, no zero fill)
//   coefficient gradient: a workgroup owns a range of pairs whose table slice fits LDS, adds
//                   its samples into that slice with LDS atomics and then adds the slice into
//                   the zero-filled gradient (float32 atomics)
#include "lmkan_kernels.h"

namespace lmkan {

namespace {

constexpr int kSmallMax = kSmallMaxOut;
constexpr int kThreads = 256;

struct SmallArgs {
    const void *P;
    CoefMap map;
    const int32_t *rec_node;
    const float *rec_u;
    const float *rec_v;
    const float *gy;
    float *y;
    float *gx_t;   // transposed scratch [n_in][B]
    float *gP;     // layout of Alg. 1, float32
    GridTab tab;
    int64_t B;
    int n_out;
    int K;
    int W;
    int pairs_per_block;
    int atomic_out;
};

template <typename CT>
__global__ __launch_bounds__(kThreads) void forward_small_kernel(SmallArgs a)
{
    const int64_t n = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int k0 = blockIdx.y * a.pairs_per_block;
    const int k1 = min(a.K, k0 + a.pairs_per_block);
    if (n >= a.B) return;
    const CT *P = static_cast<const CT *>(a.P);
    const int64_t d_i1 = (int64_t)a.W * a.map.s_node, d_i2 = a.map.s_node;
    float acc[kSmallMax];
#pragma unroll
    for (int j = 0; j < kSmallMax; ++j) acc[j] = 0.f;
    for (int k = k0; k < k1; ++k) {
        const int64_t o = (int64_t)k * a.B + n;
        const int node = a.rec_node[o];
        const float u = a.rec_u[o], v = a.rec_v[o];
        const float a_lo = 1.0f - u, b_lo = 1.0f - v;
        const float w00 = a_lo * b_lo, w10 = u * b_lo, w01 = a_lo * v, w11 = u * v;
        const CT *row = P + (int64_t)node * a.map.s_node + (int64_t)k * a.map.s_pair;
#pragma unroll
        for (int j = 0; j < kSmallMax; ++j) {
            if (j < a.n_out) {
                acc[j] = fmaf(w00, widen(row[j]), acc[j]);
                acc[j] = fmaf(w10, widen(row[d_i1 + j]), acc[j]);
                acc[j] = fmaf(w01, widen(row[d_i2 + j]), acc[j]);
                acc[j] = fmaf(w11, widen(row[d_i1 + d_i2 + j]), acc[j]);
            }
        }
    }
    float *dst = a.y + n * a.n_out;
#pragma unroll
    for (int j = 0; j < kSmallMax; ++j) {
        if (j < a.n_out) {
            if (a.atomic_out)
                unsafeAtomicAdd(dst + j, acc[j]);
            else
                dst[j] = acc[j];
        }
    }
}

template <typename CT>
__global__ __launch_bounds__(kThreads) void backward_input_small_kernel(SmallArgs a)
{
    __shared__ float s_invh[LMKAN_MAX_GRID];
    for (int i = threadIdx.x; i < a.tab.G; i += blockDim.x) s_invh[i] = a.tab.inv_h[i];
    __syncthreads();
    const int64_t n = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int k0 = blockIdx.y * a.pairs_per_block;
    const int k1 = min(a.K, k0 + a.pairs_per_block);
    if (n >= a.B) return;
    const CT *P = static_cast<const CT *>(a.P);
    const int64_t d_i1 = (int64_t)a.W * a.map.s_node, d_i2 = a.map.s_node;
    float g[kSmallMax];
#pragma unroll
    for (int j = 0; j < kSmallMax; ++j) g[j] = j < a.n_out ? a.gy[n * a.n_out + j] : 0.f;
    for (int k = k0; k < k1; ++k) {
        const int64_t o = (int64_t)k * a.B + n;
        const int node = a.rec_node[o];
        const float u = a.rec_u[o], v = a.rec_v[o];
        const CT *row = P + (int64_t)node * a.map.s_node + (int64_t)k * a.map.s_pair;
        float s00 = 0.f, s10 = 0.f, s01 = 0.f, s11 = 0.f;
#pragma unroll
        for (int j = 0; j < kSmallMax; ++j) {
            if (j < a.n_out) {
                s00 = fmaf(g[j], widen(row[j]), s00);
                s10 = fmaf(g[j], widen(row[d_i1 + j]), s10);
                s01 = fmaf(g[j], widen(row[d_i2 + j]), s01);
                s11 = fmaf(g[j], widen(row[d_i1 + d_i2 + j]), s11);
            }
        }
        const int i1 = node / a.W, i2 = node - i1 * a.W;
        const float d1 = s_invh[i1] * ((s10 - s00) * (1.0f - v) + (s11 - s01) * v);
        const float d2 = s_invh[i2] * ((s01 - s00) * (1.0f - u) + (s11 - s10) * u);
        a.gx_t[(int64_t)(2 * k) * a.B + n] = d1;
        a.gx_t[(int64_t)(2 * k + 1) * a.B + n] = d2;
    }
}

// blockIdx.y: range of pairs [k0, k1) whose slice [(G+1)^2][k1-k0][n_out] sits in LDS;
// blockIdx.x: the samples n = blockIdx.x * 256 + tid, stepping by gridDim.x * 256
__global__ __launch_bounds__(kThreads) void backward_coef_small_kernel(SmallArgs a)
{
    extern __shared__ float s_tab[];
    const int k0 = blockIdx.y * a.pairs_per_block;
    const int k1 = min(a.K, k0 + a.pairs_per_block);
    const int kc = k1 - k0;
    const int nodes = a.W * a.W;
    const int slice = nodes * kc * a.n_out;
    for (int i = threadIdx.x; i < slice; i += blockDim.x) s_tab[i] = 0.f;
    __syncthreads();
    const int row_stride = kc * a.n_out;  // one node of the slice
    for (int64_t n = (int64_t)blockIdx.x * kThreads + threadIdx.x; n < a.B; n += (int64_t)gridDim.x * kThreads) {
        float g[kSmallMax];
#pragma unroll
        for (int j = 0; j < kSmallMax; ++j) g[j] = j < a.n_out ? a.gy[n * a.n_out + j] : 0.f;
        for (int k = k0; k < k1; ++k) {
            const int64_t o = (int64_t)k * a.B + n;
            const int node = a.rec_node[o];
            const float u = a.rec_u[o], v = a.rec_v[o];
            const float a_lo = 1.0f - u, b_lo = 1.0f - v;
            const float w00 = a_lo * b_lo, w10 = u * b_lo, w01 = a_lo * v, w11 = u * v;
            float *p = s_tab + node * row_stride + (k - k0) * a.n_out;
#pragma unroll
            for (int j = 0; j < kSmallMax; ++j) {
                if (j < a.n_out) {
                    atomicAdd(p + j, w00 * g[j]);
                    atomicAdd(p + a.W * row_stride + j, w10 * g[j]);
                    atomicAdd(p + row_stride + j, w01 * g[j]);
                    atomicAdd(p + (a.W + 1) * row_stride + j, w11 * g[j]);
                }
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < slice; i += blockDim.x) {
        const float v = s_tab[i];
        if (v != 0.f) {
            const int node = i / row_stride, r = i - node * row_stride;
            const int k = k0 + r / a.n_out, j = r - (r / a.n_out) * a.n_out;
            unsafeAtomicAdd(a.gP + (int64_t)node * a.map.s_node + (int64_t)k * a.map.s_pair + j, v);
        }
    }
}

// ---------------------------------------------------------------------------
// One output (a regression head): y[n] = sum_k f_k(x[n][2k], x[n][2k+1]) (Eq. 2 with a single q),
// its input gradient and its coefficient gradient.  With one output the table of a pair is
// (G+1)^2 floats, so the tables of a chunk of pairs (or, for the coefficient gradient, their
// gradient) sit in LDS as float32, [pair][node] with an odd pitch.  A group of `lps` lanes (a
// power of two, up to the whole wave) takes a sample with a lane per pair, so the two inputs of
// its pairs are one contiguous read of the sample's row (and the two derivatives one contiguous
// write), and locates them itself (Alg. 1 "Preamble"): no records are written or read.
//   kHeadForward    the products of a sample meet in a sum over its lanes
//   kHeadGradInput  d/dx1 = gy (1/h1) ((P10 - P00)(1 - v) + (P11 - P01) v), d/dx2 likewise
//   kHeadGradCoef   gP[corner] += w_corner gy with LDS atomics (the lanes of a sample are different
//                   pairs: their addresses never coincide), the LDS copy added to the zero-filled
//                   (or existing) gradient once at the end
// A wave has kHeadSamples such steps in flight and asks for the inputs of the next ones before it
// works on those it has.
// ---------------------------------------------------------------------------
enum HeadMode { kHeadForward = 0, kHeadGradInput = 1, kHeadGradCoef = 2 };

struct HeadArgs {
    const void *P;
    CoefMap map;           // of P; for kHeadGradCoef of the gradient
    const float *x;
    const float *gy;       // [B] (one output)
    float *y;
    float *gx;             // [B][n_in]
    float *gP;             // float32, layout of Alg. 1
    GridTab tab;
    int64_t B;
    int n_in;
    int K;
    int W;
    int nodes;
    int pitch;             // LDS floats per pair, odd
    int pairs_per_chunk;   // a multiple of 64 unless one chunk holds every pair
    int lps;               // lanes per sample
    int samples_per_block;
    int atomic_out;        // forward with several chunks: add into the zero-filled y
};

constexpr int kHeadSamples = 2;  // steps a wave has in flight (more gain nothing: the two locates of a step bound the kernel)
constexpr int kHeadFill = 12;    // table elements a thread has in flight while LDS is filled
constexpr int kHeadThreads = 1024;

template <typename CT, int MODE>
__device__ __forceinline__ void head_body(const HeadArgs &a)
{
    extern __shared__ __align__(16) float head_smem[];
    const int k0 = blockIdx.y * a.pairs_per_chunk;
    const int kc = min(a.K, k0 + a.pairs_per_chunk) - k0;
    float *s_tab = head_smem;
    float *s_node = head_smem + (int64_t)a.pairs_per_chunk * a.pitch;
    float *s_invh = s_node + LMKAN_MAX_GRID + 1;
    for (int i = threadIdx.x; i <= a.tab.G; i += blockDim.x) s_node[i] = a.tab.node[i];
    for (int i = threadIdx.x; i < a.tab.G; i += blockDim.x) s_invh[i] = a.tab.inv_h[i];
    const int total = kc * a.nodes;
    // element i = node * kc + kl (pairs along the threads: contiguous in the layout of Alg. 1 with
    // one output); a thread's elements lie blockDim.x apart: (node, kl) advance by
    // (step_node, step_kl) with a carry, without a division per element
    const int step_node = (int)blockDim.x / kc, step_kl = (int)blockDim.x - step_node * kc;
    if constexpr (MODE == kHeadGradCoef) {
        for (int i = threadIdx.x; i < a.pairs_per_chunk * a.pitch; i += blockDim.x) s_tab[i] = 0.0f;
    } else {
        // Every load is unconditional (the node clamped), so that kHeadFill of them are in flight
        // per thread.
        const CT *P = static_cast<const CT *>(a.P);
        int node = (int)threadIdx.x / kc, kl = (int)threadIdx.x - node * kc;
        for (int base = threadIdx.x; base < total; base += blockDim.x * kHeadFill) {
            CT raw[kHeadFill];
            int at[kHeadFill];
#pragma unroll
            for (int u = 0; u < kHeadFill; ++u) {
                const int node_rd = min(node, a.nodes - 1);   // past the end: the same pair of the last node again
                at[u] = kl * a.pitch + node_rd;
                raw[u] = P[(int64_t)node_rd * a.map.s_node + (int64_t)(k0 + kl) * a.map.s_pair];
                node += step_node;
                kl += step_kl;
                if (kl >= kc) {
                    kl -= kc;
                    ++node;
                }
            }
#pragma unroll
            for (int u = 0; u < kHeadFill; ++u) s_tab[at[u]] = widen(raw[u]);  // (a clamped one rewrites an element of the last node)
        }
    }
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
    const int per_step = 64 / a.lps;            // samples of a wave step
    const int sub = lane / a.lps, pl = lane - sub * a.lps;
    const int per_round = per_step * kHeadSamples;
    const int64_t n_begin = (int64_t)blockIdx.x * a.samples_per_block;
    const int64_t n_end = min(a.B, n_begin + a.samples_per_block);

    // inputs of (round starting at n, pairs kk ...): lanes past the chunk and samples past the block
    // repeat the last one, every load is in bounds and unconditional, what they yield is dropped
    auto request = [&](int64_t n, int kk, float2 (&xv)[kHeadSamples], float (&g)[kHeadSamples]) {
        const int kl = min(kk + pl, kc - 1);
#pragma unroll
        for (int s = 0; s < kHeadSamples; ++s) {
            const int64_t nn = min(n + s * per_step + sub, n_end - 1);
            xv[s] = *reinterpret_cast<const float2 *>(a.x + nn * a.n_in + 2 * (k0 + kl));
            if constexpr (MODE != kHeadForward) g[s] = a.gy[nn];
        }
    };

    int64_t n = n_begin + (int64_t)wave * per_round;
    float2 xv[kHeadSamples], xv_next[kHeadSamples];
    float g[kHeadSamples] = {}, g_next[kHeadSamples] = {};
    request(n, 0, xv_next, g_next);   // (a wave with no round of its own reads the block's last sample)
    while (n < n_end) {
        float acc[kHeadSamples];
#pragma unroll
        for (int s = 0; s < kHeadSamples; ++s) acc[s] = 0.0f;
        for (int kk = 0; kk < kc; kk += a.lps) {
#pragma unroll
            for (int s = 0; s < kHeadSamples; ++s) {
                xv[s] = xv_next[s];
                g[s] = g_next[s];
            }
            // the step after this one: more pairs of these samples, else the wave's next round
            // (past the end it repeats the block's last sample)
            const bool more = kk + a.lps < kc;
            request(more ? n : n + (int64_t)waves * per_round, more ? kk + a.lps : 0, xv_next, g_next);
            const bool on = kk + pl < kc;
            const int kl = min(kk + pl, kc - 1);
            float *t_pair = s_tab + kl * a.pitch;
#pragma unroll
            for (int s = 0; s < kHeadSamples; ++s) {
                const Preamble pr = preamble(s_node, s_invh, a.tab.G, xv[s].x, xv[s].y);
                const float u = pr.a_hi, v = pr.b_hi;
                const float a_lo = 1.0f - u, b_lo = 1.0f - v;
                float *t = t_pair + pr.node;
                const int64_t mine = n + s * per_step + sub;
                if constexpr (MODE == kHeadForward) {
                    float val = (a_lo * b_lo) * t[0];
                    val = fmaf(u * b_lo, t[a.W], val);
                    val = fmaf(a_lo * v, t[1], val);
                    val = fmaf(u * v, t[a.W + 1], val);
                    acc[s] += on ? val : 0.0f;
                } else if constexpr (MODE == kHeadGradInput) {
                    const float s00 = g[s] * t[0], s10 = g[s] * t[a.W], s01 = g[s] * t[1], s11 = g[s] * t[a.W + 1];
                    const float d1 = pr.rh1 * ((s10 - s00) * b_lo + (s11 - s01) * v);
                    const float d2 = pr.rh2 * ((s01 - s00) * a_lo + (s11 - s10) * u);
                    if (on && mine < n_end)
                        *reinterpret_cast<float2 *>(a.gx + mine * a.n_in + 2 * (k0 + kl)) = make_float2(d1, d2);
                } else {
                    if (on && mine < n_end) {
                        atomicAdd(t, (a_lo * b_lo) * g[s]);
                        atomicAdd(t + a.W, (u * b_lo) * g[s]);
                        atomicAdd(t + 1, (a_lo * v) * g[s]);
                        atomicAdd(t + a.W + 1, (u * v) * g[s]);
                    }
                }
            }
        }
        if constexpr (MODE == kHeadForward) {
#pragma unroll
            for (int s = 0; s < kHeadSamples; ++s) {
                float total_s = acc[s];
                for (int m = a.lps >> 1; m >= 1; m >>= 1) total_s += __shfl_xor(total_s, m, 64);
                const int64_t mine = n + s * per_step + sub;
                if (pl == 0 && mine < n_end) {
                    if (a.atomic_out)
                        unsafeAtomicAdd(a.y + mine, total_s);
                    else
                        a.y[mine] = total_s;
                }
            }
        }
        n += (int64_t)waves * per_round;
    }

    if constexpr (MODE == kHeadGradCoef) {
        // every wave comes here (none leaves early): the block's sums go to the gradient
        __syncthreads();
        int node = (int)threadIdx.x / kc, kl = (int)threadIdx.x - node * kc;
        for (int i = threadIdx.x; i < total; i += blockDim.x) {
            const float v = s_tab[kl * a.pitch + node];
            if (v != 0.0f) unsafeAtomicAdd(a.gP + (int64_t)node * a.map.s_node + (int64_t)(k0 + kl) * a.map.s_pair, v);
            node += step_node;
            kl += step_kl;
            if (kl >= kc) {
                kl -= kc;
                ++node;
            }
        }
    }
}

template <typename CT>
__global__ __launch_bounds__(kHeadThreads) void forward_head_kernel(HeadArgs a)
{
    head_body<CT, kHeadForward>(a);
}

template <typename CT>
__global__ __launch_bounds__(kHeadThreads) void backward_input_head_kernel(HeadArgs a)
{
    head_body<CT, kHeadGradInput>(a);
}

__global__ __launch_bounds__(kHeadThreads) void backward_coef_head_kernel(HeadArgs a)
{
    head_body<float, kHeadGradCoef>(a);
}

SmallArgs small_args(const LayerShape &s, const void *coef, const void *records)
{
    const size_t n = (size_t)s.pairs() * (size_t)s.batch;
    SmallArgs a = {};
    a.P = coef;
    a.map = coef_map(s);
    a.rec_node = static_cast<const int32_t *>(records);
    a.rec_u = reinterpret_cast<const float *>(a.rec_node + n);
    a.rec_v = a.rec_u + n;
    a.B = s.batch;
    a.n_out = s.n_out;
    a.K = s.pairs();
    a.W = s.G + 1;
    return a;
}

// enough blocks for 256 CUs: split the pairs when the batch alone gives too few
int pair_split(const LayerShape &s)
{
    const int64_t bblocks = (s.batch + kThreads - 1) / kThreads;
    int split = 1;
    while (bblocks * split < 512 && s.pairs() / (split * 2) >= 8) split *= 2;
    return split;
}

}  // namespace

bool small_out_shape_ok(const LayerShape &s)
{
    return s.n_out <= kSmallMax && (s.n_out == 1 || !slab_backward_input_shape_ok(s));
}

// LDS floats per pair of the one-output forward kernel, and the pairs one workgroup can hold
static int head_pitch(const LayerShape &s) { return s.nodes() | 1; }
static int head_chunk(const LayerShape &s)
{
    const int budget = (160 * 1024 - 1024) / (int)sizeof(float);  // 1 KB for the grid
    int kc = budget / head_pitch(s);
    if (kc >= s.pairs()) return s.pairs();
    return kc & ~63;
}

// One output, rows (not windows), and at least a wave of pairs fits LDS at a time (G <= 24, or few pairs)
bool head_forward_shape_ok(const LayerShape &s)
{
    return s.n_out == 1 && head_chunk(s) > 0;
}

// grid, LDS and per-block share of a launch of head_kernel over at most `max_blocks` workgroups
// per chunk of pairs
static HeadArgs head_args(const LayerShape &s, const GridTab &tab, const float *x, int max_blocks, dim3 *grid,
                          size_t *lds)
{
    HeadArgs a = {};
    a.x = x;
    a.tab = tab;
    a.B = s.batch;
    a.n_in = s.n_in;
    a.K = s.pairs();
    a.W = s.G + 1;
    a.nodes = s.nodes();
    a.pitch = head_pitch(s);
    a.pairs_per_chunk = head_chunk(s);
    const int chunks = (a.K + a.pairs_per_chunk - 1) / a.pairs_per_chunk;
    // a sample takes as many lanes as the chunk has pairs, rounded up to a power of two
    a.lps = 1;
    while (a.lps < 64 && a.lps < a.pairs_per_chunk) a.lps *= 2;
    *lds = ((size_t)a.pairs_per_chunk * a.pitch + 2 * LMKAN_MAX_GRID + 2) * sizeof(float);
    // every workgroup fills (or clears and later adds out) its LDS copy of the chunk's tables: a
    // workgroup should have at least two rounds of its 16 waves to spread that over
    const int64_t round = (int64_t)(kHeadThreads / 64) * kHeadSamples * (64 / a.lps);
    int64_t per_block = 2 * round;
    if ((s.batch + per_block - 1) / per_block > max_blocks)
        per_block = ((s.batch + max_blocks - 1) / max_blocks + round - 1) / round * round;
    a.samples_per_block = (int)per_block;
    *grid = dim3((unsigned)((s.batch + per_block - 1) / per_block), (unsigned)chunks);
    return a;
}

typedef void (*HeadKernel)(HeadArgs);

static void launch_head(HeadKernel kernel, const HeadArgs &a, dim3 grid, size_t lds, hipStream_t stream,
                        TimedKernel kind)
{
    if (lds > 64 * 1024) allow_large_lds(reinterpret_cast<const void *>(kernel), 160 * 1024);
    KernelTiming timing(stream, kind);
    kernel<<<grid, kHeadThreads, lds, stream>>>(a);
}

void launch_forward_head(const LayerShape &s, const GridTab &tab, const float *x, const void *coef, float *y,
                         hipStream_t stream)
{
    dim3 grid;
    size_t lds;
    HeadArgs a = head_args(s, tab, x, 256, &grid, &lds);   // 256 workgroups fill the chip
    a.P = coef;
    a.map = coef_map(s);
    a.y = y;
    a.atomic_out = grid.y > 1;
    if (a.atomic_out) launch_fill_zero(y, (size_t)s.batch, stream);
    const HeadKernel kernels[3] = {forward_head_kernel<float>, forward_head_kernel<_Float16>,
                                   forward_head_kernel<bf16_t>};
    launch_head(kernels[s.dtype], a, grid, lds, stream, kTimeForward);
}

void launch_backward_input_head(const LayerShape &s, const GridTab &tab, const float *x, const void *coef,
                                const float *gy, float *gx, hipStream_t stream)
{
    dim3 grid;
    size_t lds;
    HeadArgs a = head_args(s, tab, x, 256, &grid, &lds);
    a.P = coef;
    a.map = coef_map(s);
    a.gy = gy;
    a.gx = gx;   // every (sample, pair) is written by exactly one lane: no clearing, no atomics
    const HeadKernel kernels[3] = {backward_input_head_kernel<float>, backward_input_head_kernel<_Float16>,
                                   backward_input_head_kernel<bf16_t>};
    launch_head(kernels[s.dtype], a, grid, lds, stream, kTimeGradInput);
}

void launch_backward_coef_head(const LayerShape &s, const GridTab &tab, const float *x, const float *gy,
                               float *gcoef, bool accumulate, hipStream_t stream)
{
    dim3 grid;
    size_t lds;
    // (bound by the LDS atomics, about 3.5 clocks per lane and CU: every CU has to take part, although
    // every workgroup ends by adding its whole LDS copy to the gradient)
    HeadArgs a = head_args(s, tab, x, 256, &grid, &lds);
    LayerShape g = s;
    g.layout = LMKAN_LAYOUT_PAPER;
    a.map = coef_map(g);
    a.gy = gy;
    a.gP = gcoef;
    if (!accumulate) launch_fill_zero(gcoef, (size_t)s.nodes() * (size_t)s.pairs(), stream);
    launch_head(backward_coef_head_kernel, a, grid, lds, stream, kTimeGradCoef);
}

void launch_forward_small(const LayerShape &s, const void *coef, float *y, const void *records, hipStream_t stream)
{
    SmallArgs a = small_args(s, coef, records);
    a.y = y;
    const int split = pair_split(s);
    a.pairs_per_block = (a.K + split - 1) / split;
    a.atomic_out = split > 1;
    if (a.atomic_out) launch_fill_zero(y, (size_t)s.batch * s.n_out, stream);
    const dim3 grid((unsigned)((s.batch + kThreads - 1) / kThreads), (unsigned)split);
    KernelTiming timing(stream, kTimeForward);
    switch (s.dtype) {
    case LMKAN_F32: forward_small_kernel<float><<<grid, kThreads, 0, stream>>>(a); break;
    case LMKAN_F16: forward_small_kernel<_Float16><<<grid, kThreads, 0, stream>>>(a); break;
    default: forward_small_kernel<bf16_t><<<grid, kThreads, 0, stream>>>(a); break;
    }
}

void launch_backward_input_small(const LayerShape &s, const GridTab &tab, const void *coef, const float *gy,
                                 float *gx_scratch, const void *records, hipStream_t stream)
{
    SmallArgs a = small_args(s, coef, records);
    a.gy = gy;
    a.gx_t = gx_scratch;
    a.tab = tab;
    const int split = pair_split(s);
    a.pairs_per_block = (a.K + split - 1) / split;
    const dim3 grid((unsigned)((s.batch + kThreads - 1) / kThreads), (unsigned)split);
    KernelTiming timing(stream, kTimeGradInput);
    switch (s.dtype) {
    case LMKAN_F32: backward_input_small_kernel<float><<<grid, kThreads, 0, stream>>>(a); break;
    case LMKAN_F16: backward_input_small_kernel<_Float16><<<grid, kThreads, 0, stream>>>(a); break;
    default: backward_input_small_kernel<bf16_t><<<grid, kThreads, 0, stream>>>(a); break;
    }
}

void launch_backward_coef_small(const LayerShape &s, const void *records, const float *gy, float *gcoef,
                                bool accumulate, hipStream_t stream)
{
    SmallArgs a = small_args(s, nullptr, records);
    a.gy = gy;
    a.gP = gcoef;
    LayerShape g = s;
    g.layout = LMKAN_LAYOUT_PAPER;
    a.map = coef_map(g);
    // pairs per block: the slice must fit 64 KiB of LDS
    const int per_pair = s.nodes() * s.n_out * (int)sizeof(float);
    int kc = (64 * 1024) / per_pair;
    if (kc > a.K) kc = a.K;
    a.pairs_per_block = kc;  // >= 1: (G+1)^2 n_out 4 <= 65^2 * 8 * 4 bytes would not fit, see small_coef_ok
    const int groups = (a.K + kc - 1) / kc;
    int64_t bblocks = (s.batch + kThreads - 1) / kThreads;
    int64_t want = (1024 + groups - 1) / groups;  // about 1024 workgroups in all
    if (bblocks > want) bblocks = want;
    if (!accumulate) launch_fill_zero(gcoef, (size_t)s.nodes() * (size_t)s.pairs() * (size_t)s.n_out, stream);
    const dim3 grid((unsigned)bblocks, (unsigned)groups);
    KernelTiming timing(stream, kTimeGradCoef);
    backward_coef_small_kernel<<<grid, kThreads, (size_t)kc * per_pair, stream>>>(a);
}

bool small_coef_ok(const LayerShape &s)
{
    return small_out_shape_ok(s) && (size_t)s.nodes() * s.n_out * sizeof(float) <= 64 * 1024;
}

}  // namespace lmkan
