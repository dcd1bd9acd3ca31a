// Off-diagonal Hessian regulariser of a layer (Sec. 3.5, App. C): value and gradient with
// respect to the coefficients.
//
// For every 2-D function (pair k, output j) and every node (a, b) with a full stencil
// (a, b in [1, G-1]; ghost-node values enter as neighbours) App. C's finite differences on the
// non-uniform grid give D11, D22, D12 and H = D11^2 + 2 D12^2 + D22^2; the function's term is
// the mean of H over those nodes and the layer's value the sum over all functions.
//
// A thread owns one function and walks the table rows a = 0 .. G.  The tensor is read exactly
// once: consecutive threads are consecutive (k, j), which is the contiguous direction of both
// layouts, and a thread keeps the last five rows of its function in a private slice of LDS.
// With rows a-2 .. a+2 present the gradient of row a is gathered: a node takes part in the
// stencils of at most 3 + 3 + 4 centres, whose second differences are recomputed from the
// window.  The kernel is bound by HBM: one read of the table, one write (or read-modify-write)
// of the gradient.
#include "lmkan_kernels.h"

namespace lmkan {

namespace {

constexpr int kThreads = 64;
constexpr int kRows = 5;

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

template <typename CT>
__global__ __launch_bounds__(kThreads) void hessian_reg_kernel(HessArgs a)
{
    extern __shared__ float s_win[];  // [kRows][W][kThreads]: thread-private columns
    // per-axis stencil coefficients of centre i in [1, G-1]:
    //   second difference = cm[i] p(i-1) + c0[i] p(i) + cp[i] p(i+1),  mixed: r12[i] = 1 / (hl + hr)
    __shared__ float s_cm[LMKAN_MAX_GRID + 1], s_c0[LMKAN_MAX_GRID + 1], s_cp[LMKAN_MAX_GRID + 1],
        s_r12[LMKAN_MAX_GRID + 1];
    const int G = a.tab.G, W = G + 1;
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
    const CT *P = static_cast<const CT *>(a.P) + (int64_t)k * a.map.s_pair + (int64_t)(j >> 6) * a.map.s_tile + (j & 63);
    float *gout = a.grad ? a.grad + (int64_t)k * a.gmap.s_pair + j : nullptr;
    float *win = s_win + threadIdx.x;
    auto at = [&](int row, int b) -> float & { return win[((row % kRows) * W + b) * kThreads]; };
    const float inv_n = 1.0f / ((float)(G - 1) * (float)(G - 1));

    // second differences at centre (ca, cb); zero where the stencil does not exist
    auto d11 = [&](int ca, int cb) {
        if (ca < 1 || ca > G - 1 || cb < 1 || cb > G - 1) return 0.f;
        return s_cm[ca] * at(ca - 1, cb) + s_c0[ca] * at(ca, cb) + s_cp[ca] * at(ca + 1, cb);
    };
    auto d22 = [&](int ca, int cb) {
        if (ca < 1 || ca > G - 1 || cb < 1 || cb > G - 1) return 0.f;
        return s_cm[cb] * at(ca, cb - 1) + s_c0[cb] * at(ca, cb) + s_cp[cb] * at(ca, cb + 1);
    };
    auto d12 = [&](int ca, int cb) {
        if (ca < 1 || ca > G - 1 || cb < 1 || cb > G - 1) return 0.f;
        return s_r12[ca] * s_r12[cb] *
               (at(ca + 1, cb + 1) - at(ca + 1, cb - 1) - at(ca - 1, cb + 1) + at(ca - 1, cb - 1));
    };

    float h_sum = 0.f;
    for (int a_in = 0; a_in <= G + 2; ++a_in) {
        if (a_in <= G && live) {
            for (int b = 0; b <= G; ++b) at(a_in, b) = widen(P[(int64_t)(a_in * W + b) * a.map.s_node]);
        }
        const int ao = a_in - 2;  // rows ao-2 .. ao+2 that exist are in the window
        if (ao < 0 || !live) continue;
        for (int b = 0; b <= G; ++b) {
            const float e11 = d11(ao, b), e22 = d22(ao, b), e12 = d12(ao, b);
            h_sum += e11 * e11 + 2.0f * e12 * e12 + e22 * e22;  // zero unless (ao, b) is a centre
            if (gout) {
                // node (ao, b) in the stencils of its neighbours: as p(i+1) of centre i-1 (cp), as
                // p(i) of centre i (c0), as p(i-1) of centre i+1 (cm); as one of the four corners of
                // the mixed difference of the four diagonal neighbours
                float g = 0.f;
                if (ao >= 2) g += s_cp[ao - 1] * d11(ao - 1, b);
                g += s_c0[ao] * e11;
                if (ao <= G - 2) g += s_cm[ao + 1] * d11(ao + 1, b);
                if (b >= 2) g += s_cp[b - 1] * d22(ao, b - 1);
                g += s_c0[b] * e22;
                if (b <= G - 2) g += s_cm[b + 1] * d22(ao, b + 1);
                float m = 0.f;
                if (ao >= 2 && b >= 2) m += s_r12[ao - 1] * s_r12[b - 1] * d12(ao - 1, b - 1);
                if (ao >= 2 && b <= G - 2) m -= s_r12[ao - 1] * s_r12[b + 1] * d12(ao - 1, b + 1);
                if (ao <= G - 2 && b >= 2) m -= s_r12[ao + 1] * s_r12[b - 1] * d12(ao + 1, b - 1);
                if (ao <= G - 2 && b <= G - 2) m += s_r12[ao + 1] * s_r12[b + 1] * d12(ao + 1, b + 1);
                const float v = a.scale * inv_n * (2.0f * g + 4.0f * m);
                float *dst = gout + (int64_t)(ao * W + b) * a.gmap.s_node;
                *dst = a.accumulate ? *dst + v : v;
            }
        }
    }
    // value: sum over the wave, one double atomic per wave
    double part = (double)h_sum * (double)inv_n;
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
    const size_t lds = (size_t)kRows * (s.G + 1) * kThreads * sizeof(float);
    typedef void (*Kernel)(HessArgs);
    const Kernel kernels[3] = {hessian_reg_kernel<float>, hessian_reg_kernel<_Float16>, hessian_reg_kernel<bf16_t>};
    const Kernel kernel = kernels[s.dtype];
    if (lds > 48 * 1024) {
        static bool attr_set[3] = {false, false, false};
        if (!attr_set[s.dtype]) {
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
            attr_set[s.dtype] = true;
        }
    }
    kernel<<<grid, kThreads, lds, stream>>>(a);
}

}  // namespace lmkan
