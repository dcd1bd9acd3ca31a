// Off-diagonal Hessian regulariser of a layer (Sec. 3.5, App. C): value and gradient with
// respect to the coefficients.
//
// For every 2-D function (pair k, output j) and every node (a, b) with a full stencil
// (a, b in [1, G-1]; ghost-node values enter as neighbours) App. C's finite differences on the
// non-uniform grid give D11, D22, D12 and H = D11^2 + 2 D12^2 + D22^2; the function's term is
// the mean of H over those nodes and the layer's value the sum over all functions.
//
// A thread owns one function and walks the table rows.  The tensor is read exactly once:
// consecutive threads are consecutive (k, j), which is the contiguous direction of both
// layouts, and a thread keeps a few rows of its function in a private slice of LDS: four
// rows of coefficients (three under the stencil, one being fetched) and three rows of
// gradient.  Along a row of centres the 3 x 3 neighbourhood and the 3 x 3 gradient
// contributions slide through registers, so a centre costs three LDS reads of coefficients
// and three read-modify-writes of gradient.  A gradient row leaves for HBM once the row of
// centres below it is done.  The kernel is bound by HBM: one read of the table, one write (or
// read-modify-write) of the gradient.
#include "lmkan_kernels.h"

namespace lmkan {

namespace {

constexpr int kThreads = 64;
constexpr int kGradRows = 3;  // ring of gradient rows

struct HessArgs {
    const void *P;
    CoefMap map;   // layout of P
    CoefMap gmap;  // layout of Alg. 1 (gradient)
    float *grad;   // may be null
    double *value;
    GridTab tab;
    float scale;
    int accumulate;
    int K;
    int n_out;
};

// W_CT = G + 1 when known at compile time: two coming rows then travel in registers while the
// current row of centres is worked on, so the loads of a wave overlap its arithmetic and the
// ring needs only the three rows under the stencil.  W_CT = 0: any grid, rows fetched one
// ahead straight into a ring of four (the fetch is waited for before the arithmetic starts).
template <int W_CT>
struct HessRing {
    static constexpr int kCoefRows = W_CT > 0 ? 3 : 4;
};

template <typename CT, int W_CT>
__global__ __launch_bounds__(kThreads) void hessian_reg_kernel(HessArgs a)
{
    extern __shared__ float s_dyn[];  // [kCoefRows + kGradRows][W][kThreads]: thread-private columns
    // per-axis stencil coefficients of centre i in [1, G-1]:
    //   second difference = cm[i] p(i-1) + c0[i] p(i) + cp[i] p(i+1),  mixed: r12[i] = 1 / (hl + hr)
    __shared__ float s_cm[LMKAN_MAX_GRID + 1], s_c0[LMKAN_MAX_GRID + 1], s_cp[LMKAN_MAX_GRID + 1],
        s_r12[LMKAN_MAX_GRID + 1];
    constexpr int kCoefRows = HessRing<W_CT>::kCoefRows;
    const int G = W_CT > 0 ? W_CT - 1 : a.tab.G, W = G + 1;
    for (int i = threadIdx.x; i <= G; i += blockDim.x) {
        float cm = 0.f, c0 = 0.f, cp = 0.f, r = 0.f;
        if (i >= 1 && i <= G - 1) {
            const float hl = a.tab.node[i] - a.tab.node[i - 1], hr = a.tab.node[i + 1] - a.tab.node[i];
            cm = 2.0f / (hl * (hl + hr));
            c0 = -2.0f / (hl * hr);
            cp = 2.0f / (hr * (hl + hr));
            r = 1.0f / (hl + hr);
        }
        s_cm[i] = cm;
        s_c0[i] = c0;
        s_cp[i] = cp;
        s_r12[i] = r;
    }
    __syncthreads();

    const int64_t col = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const bool live = col < (int64_t)a.K * a.n_out;
    const int k = live ? (int)(col / a.n_out) : 0;
    const int j = live ? (int)(col - (int64_t)k * a.n_out) : 0;
    // a dead thread (past the last function) reads function 0 and writes nothing
    const CT *P = static_cast<const CT *>(a.P) + (int64_t)k * a.map.s_pair + (int64_t)(j >> 6) * a.map.s_tile + (j & 63);
    float *gout = (a.grad && live) ? a.grad + (int64_t)k * a.gmap.s_pair + j : nullptr;
    float *pw = s_dyn + threadIdx.x;                             // coefficient rows
    float *gw = s_dyn + kCoefRows * W * kThreads + threadIdx.x;  // gradient rows
    auto prow = [&](int row) { return pw + (row % kCoefRows) * W * kThreads; };
    auto grow = [&](int row) { return gw + (row % kGradRows) * W * kThreads; };
    auto fetch_row = [&](int row) {  // global -> ring
        float *dst = prow(row);
        for (int b = 0; b <= G; ++b) dst[b * kThreads] = widen(P[(int64_t)(row * W + b) * a.map.s_node]);
    };
    auto store_row = [&](int row) {  // gradient row `row` is complete: write it, clear its slot
        float *src = grow(row);
#pragma unroll
        for (int b = 0; b < (W_CT > 0 ? W_CT : W); ++b) {
            const float v = src[b * kThreads];
            src[b * kThreads] = 0.f;
            if (gout) {
                float *dst = gout + (int64_t)(row * W + b) * a.gmap.s_node;
                *dst = a.accumulate ? *dst + v : v;
            }
        }
    };
    for (int i = 0; i < kGradRows * W; ++i) gw[i * kThreads] = 0.f;
    const float inv_n = 1.0f / ((float)(G - 1) * (float)(G - 1));
    const float gs = a.scale * inv_n;
    float h_sum = 0.f;

    // one row of centres; rows c-1, c, c+1 are in the ring
    auto centre_row = [&](int c) {
        const float *r0 = prow(c - 1), *r1 = prow(c), *r2 = prow(c + 1);
        float *g0 = grow(c - 1), *g1 = grow(c), *g2 = grow(c + 1);
        const float cm = s_cm[c], c0 = s_c0[c], cp = s_cp[c], rc = s_r12[c];
        // neighbourhood columns b-1, b, b+1 and the gradient pieces for them
        float p00 = r0[0], p10 = r1[0], p20 = r2[0];
        float p01 = r0[kThreads], p11 = r1[kThreads], p21 = r2[kThreads];
        float a00 = 0.f, a10 = 0.f, a20 = 0.f, a01 = 0.f, a11 = 0.f, a21 = 0.f;
#pragma unroll
        for (int b = 1; b <= (W_CT > 0 ? W_CT - 2 : G - 1); ++b) {
            const float p02 = r0[(b + 1) * kThreads], p12 = r1[(b + 1) * kThreads], p22 = r2[(b + 1) * kThreads];
            const float bm = s_cm[b], b0 = s_c0[b], bp = s_cp[b], rb = s_r12[b];
            const float d11 = cm * p01 + c0 * p11 + cp * p21;
            const float d22 = bm * p10 + b0 * p11 + bp * p12;
            const float rr = rc * rb;
            const float d12 = rr * (p22 - p20 - p02 + p00);
            h_sum += d11 * d11 + 2.0f * d12 * d12 + d22 * d22;
            const float e11 = 2.0f * gs * d11, e22 = 2.0f * gs * d22, e12 = 4.0f * gs * rr * d12;
            // column b-1 receives its last pieces and leaves the registers
            g0[(b - 1) * kThreads] += a00 + e12;
            g1[(b - 1) * kThreads] += a10 + bm * e22;
            g2[(b - 1) * kThreads] += a20 - e12;
            // column b
            a00 = a01 + cm * e11;
            a10 = a11 + c0 * e11 + b0 * e22;
            a20 = a21 + cp * e11;
            // column b+1 starts
            a01 = -e12;
            a11 = bp * e22;
            a21 = e12;
            p00 = p01; p10 = p11; p20 = p21;
            p01 = p02; p11 = p12; p21 = p22;
        }
        g0[(G - 1) * kThreads] += a00;
        g1[(G - 1) * kThreads] += a10;
        g2[(G - 1) * kThreads] += a20;
        g0[G * kThreads] += a01;
        g1[G * kThreads] += a11;
        g2[G * kThreads] += a21;
    };

    fetch_row(0);
    fetch_row(1);
    fetch_row(2);
    if constexpr (W_CT > 0) {
        // rows c+2 and c+3 in registers: `near` was requested an iteration ago and goes into the
        // ring slot that row c-1 leaves, `far` is requested now
        CT s0[W_CT], s1[W_CT];
        auto request = [&](CT(&st)[W_CT], int row) {
            if (row <= G) {
#pragma unroll
                for (int b = 0; b < W_CT; ++b) st[b] = P[(int64_t)(row * W + b) * a.map.s_node];
            }
        };
        auto deposit = [&](const CT(&st)[W_CT], int row) {
            if (row <= G) {
                float *dst = prow(row);
#pragma unroll
                for (int b = 0; b < W_CT; ++b) dst[b * kThreads] = widen(st[b]);
            }
        };
        auto step = [&](int c, CT(&near)[W_CT], CT(&far)[W_CT]) {
            request(far, c + 3);
            centre_row(c);
            store_row(c - 1);  // nothing below row c of centres reaches gradient row c-1
            deposit(near, c + 2);
        };
        request(s0, 3);
        for (int c = 1; c <= G - 1; c += 2) {
            step(c, s0, s1);
            if (c + 1 <= G - 1) step(c + 1, s1, s0);
        }
    } else {
        for (int c = 1; c <= G - 1; ++c) {
            if (c + 2 <= G) fetch_row(c + 2);
            centre_row(c);
            store_row(c - 1);
        }
    }
    store_row(G - 1);
    store_row(G);
    // value: sum over the wave, one double atomic per wave
    double part = live ? (double)h_sum * (double)inv_n : 0.0;
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) part += __shfl_down(part, d, 64);
    if ((threadIdx.x & 63) == 0 && a.value) atomicAdd(a.value, part);
}

}  // namespace

void launch_hessian_reg(const LayerShape &s, const GridTab &tab, const void *coef, float scale, double *value,
                        float *grad, bool accumulate, hipStream_t stream)
{
    HessArgs a;
    a.P = coef;
    a.map = coef_map(s);
    LayerShape g = s;
    g.layout = LMKAN_LAYOUT_PAPER;
    a.gmap = coef_map(g);
    a.grad = grad;
    a.value = value;
    a.tab = tab;
    a.scale = scale;
    a.accumulate = accumulate ? 1 : 0;
    a.K = s.pairs();
    a.n_out = s.n_out;
    if (value) launch_fill_zero(reinterpret_cast<float *>(value), 2, stream);
    const int64_t cols = (int64_t)s.pairs() * s.n_out;
    const unsigned grid = (unsigned)((cols + kThreads - 1) / kThreads);
    typedef void (*Kernel)(HessArgs);
    // kernels with the row length compiled in for the usual grids
    static const Kernel table[5][3] = {
        {hessian_reg_kernel<float, 0>, hessian_reg_kernel<_Float16, 0>, hessian_reg_kernel<bf16_t, 0>},
        {hessian_reg_kernel<float, 9>, hessian_reg_kernel<_Float16, 9>, hessian_reg_kernel<bf16_t, 9>},
        {hessian_reg_kernel<float, 13>, hessian_reg_kernel<_Float16, 13>, hessian_reg_kernel<bf16_t, 13>},
        {hessian_reg_kernel<float, 17>, hessian_reg_kernel<_Float16, 17>, hessian_reg_kernel<bf16_t, 17>},
        {hessian_reg_kernel<float, 33>, hessian_reg_kernel<_Float16, 33>, hessian_reg_kernel<bf16_t, 33>},
    };
    const int which = s.G == 8 ? 1 : s.G == 12 ? 2 : s.G == 16 ? 3 : s.G == 32 ? 4 : 0;
    const Kernel kernel = table[which][s.dtype];
    const size_t lds = (size_t)((which ? 3 : 4) + kGradRows) * (s.G + 1) * kThreads * sizeof(float);
    if (lds > 48 * 1024) allow_large_lds(reinterpret_cast<const void *>(kernel), 150 * 1024);
    kernel<<<grid, kThreads, lds, stream>>>(a);
}

}  // namespace lmkan
