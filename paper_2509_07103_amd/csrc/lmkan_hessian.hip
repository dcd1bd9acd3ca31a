// Off-diagonal Hessian regulariser of a layer (Sec. 3.5, App. C): value and gradient with
// respect to the coefficients.
//
// For every 2-D function (pair k, output j) and every node (a, b) with a full stencil
// (a, b in [1, G-1]; ghost-node values enter as neighbours) App. C's finite differences on the
// non-uniform grid give D11, D22, D12 and H = D11^2 + 2 D12^2 + D22^2; the function's term is
// the mean of H over those nodes and the layer's value the sum over all functions.
//
// A lane owns one function: a workgroup takes pair k and 64 consecutive outputs j, the
// contiguous direction of both layouts, so every address is a wave-uniform base plus the lane.
// A wave owns a band of kBand columns of the table of those 64 functions; the bands are the
// waves of the workgroup.  A wave walks the table rows and
// keeps everything in registers: three rows of coefficients under the stencil (its own columns
// and two more on either side), three rows that are on their way from memory, and three rows of
// gradient for its own columns.  The gradient of a column takes pieces from the centres in the
// columns beside it, so a wave also evaluates the centre on either side of its band (two
// centres in eleven are computed twice; their loads hit the cache behind the neighbouring wave)
// and no wave ever adds into another wave's gradient.  Along a row the 3 x 3 neighbourhood and the
// 3 x 3 gradient pieces slide through registers.  A gradient row leaves for HBM once the row of
// centres below it is done.  The tensor is read from HBM once and the gradient written once
// (or read, added to and written).
#include "lmkan_kernels.h"

namespace lmkan {

namespace {

constexpr int kBand = 9;               // gradient columns a wave owns
constexpr int kCols = kBand + 4;       // coefficient columns it holds
constexpr int kCentres = kBand + 2;    // centres it evaluates per row
constexpr int kMaxBands = (LMKAN_MAX_GRID + 1 + kBand - 1) / kBand;

struct HessArgs {
    const void *P;
    CoefMap map;   // layout of P
    CoefMap gmap;  // layout of Alg. 1 (gradient)
    float *grad;   // null for the value alone
    double *value;
    GridTab tab;
    float scale;
    int K;
    int n_out;
};

// a value that is the same in every lane, moved to a scalar register
__device__ __forceinline__ float uniform(float v)
{
    return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v)));
}

// Per-axis stencil of centre i in [1, G-1] on the non-uniform grid:
//   second difference = cm p(i-1) + c0 p(i) + cp p(i+1),  mixed difference: r = 1 / (hl + hr) per axis
struct Stencil {
    float cm, c0, cp, r;
};
__device__ __forceinline__ Stencil stencil_of(const GridTab &tab, int i, int G)
{
    Stencil s = {0.f, 0.f, 0.f, 0.f};
    if (i >= 1 && i <= G - 1) {
        const float hl = tab.node[i] - tab.node[i - 1], hr = tab.node[i + 1] - tab.node[i];
        s.cm = 2.0f / (hl * (hl + hr));
        s.c0 = -2.0f / (hl * hr);
        s.cp = 2.0f / (hr * (hl + hr));
        s.r = 1.0f / (hl + hr);
    }
    return s;
}

// GRAD: 0 value only, 1 gradient written, 2 gradient added to what the buffer holds
template <typename CT, int GRAD>
__global__ __launch_bounds__(64 * kMaxBands) void hessian_reg_kernel(HessArgs a)
{
    // stencils of the rows, read once per row
    __shared__ float s_cm[LMKAN_MAX_GRID + 1], s_c0[LMKAN_MAX_GRID + 1], s_cp[LMKAN_MAX_GRID + 1],
        s_r[LMKAN_MAX_GRID + 1];
    const int G = a.tab.G, W = G + 1;
    for (int i = threadIdx.x; i <= G; i += blockDim.x) {
        const Stencil s = stencil_of(a.tab, i, G);
        s_cm[i] = s.cm;
        s_c0[i] = s.c0;
        s_cp[i] = s.cp;
        s_r[i] = s.r;
    }
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int band = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b_first = band * kBand;            // own columns [b_first, b_end)
    const int b_end = min(W, b_first + kBand);
    // Centre i of the wave sits in column b_first - 1 + i.  A column without a full stencil
    // (outside [1, G-1], or beyond the table for the last band) gets an all-zero stencil and a zero
    // factor on its row-direction difference: such a centre then contributes exact zeros.  The
    // middle weight of a second difference is minus the sum of the outer two, so two weights and
    // the mixed-difference factor per column are kept, in scalar registers.
    float col_cm[kCentres], col_cp[kCentres], col_r[kCentres];
    unsigned on_mask = 0;
#pragma unroll
    for (int i = 0; i < kCentres; ++i) {
        const int b = b_first - 1 + i;
        const Stencil s = stencil_of(a.tab, b, G);
        col_cm[i] = uniform(s.cm);
        col_cp[i] = uniform(s.cp);
        col_r[i] = uniform(s.r);
        if (b >= 1 && b <= G - 1) on_mask |= 1u << i;
    }

    // consecutive workgroups are the output tiles of one pair: next to each other in the gradient
    const int tile = blockIdx.x, k = blockIdx.y;
    const int j = tile * 64 + lane;
    const bool live = j < a.n_out;
    // A lane past the last output works on the last output once more: it reads the same values,
    // computes the same results and stores them to the same addresses in the same instructions
    // as the lane that owns that output, so nothing in the walk below depends on the lane.
    const int lane_rd = min(j, a.n_out - 1) & 63;
    const CT *P = static_cast<const CT *>(a.P) + (int64_t)k * a.map.s_pair + (int64_t)tile * a.map.s_tile;  // wave-uniform
    float *gout = a.grad + (int64_t)k * a.gmap.s_pair + tile * 64;                                          // wave-uniform

    // Coefficient column q of the wave is table column b_first - 2 + q.  Columns beyond the table
    // (only centres that are switched off look at them) read a neighbouring node instead: the node
    // index is clamped to the table, for every load, in scalar arithmetic.
    const int last_node = W * W - 1;
    auto node_ptr = [&](int row, int q) {
        const int node = min(max(row * W + b_first - 2 + q, 0), last_node);
        return P + (int64_t)node * a.map.s_node + lane_rd;
    };

    float p[3][kCols];     // rows c-1, c, c+1; row r lives in p[r % 3]
    CT raw[3][kCols];      // rows c+2, c+3, c+4 as loaded; row r lives in raw[r % 3]
    float g[3][kBand];     // gradient rows c-1, c, c+1 of the own columns; row r in g[r % 3]
#pragma unroll
    for (int r = 0; r < 3; ++r) {
#pragma unroll
        for (int t = 0; t < kBand; ++t) g[r][t] = 0.f;
#pragma unroll
        for (int q = 0; q < kCols; ++q) p[r][q] = widen(*node_ptr(r, q));  // G >= 3: rows 0..2 exist
    }
    // the rows under the first stencil have arrived before anything else is requested: the waits
    // inside the loop then only ever count the requests of the loop
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // (a request is never skipped: past the last row the clamp makes it read the last node again.
    // A skipped request would be a path with fewer loads in flight, and the waits the compiler
    // places count the loads of the shortest path.)
    auto request = [&](auto slot, int row) {
        constexpr int S = decltype(slot)::value;
#pragma unroll
        for (int q = 0; q < kCols; ++q) raw[S][q] = *node_ptr(row, q);
    };
    request(std::integral_constant<int, 0>{}, 3);
    request(std::integral_constant<int, 1>{}, 4);

    const float inv_n = 1.0f / ((float)(G - 1) * (float)(G - 1));
    const float gs = a.scale * inv_n;
    float h_sum = 0.f;

    // Gradient row `row` (complete: nothing below the current row of centres reaches it) leaves
    // the registers.  When the gradient is added to, the values it is added to were requested at
    // the top of the step (`old`), before the step's request of coefficients, so that waiting for
    // them leaves that request in flight.
    const int n_own = b_end - b_first;
    float old[kBand];
    auto grad_ptr = [&](int row, int t) {
        const int node = min(row * W + b_first + t, last_node);
        return gout + (int64_t)node * a.gmap.s_node + lane_rd;
    };
    auto request_old = [&](int row) {
        if constexpr (GRAD == 2) {
#pragma unroll
            for (int t = 0; t < kBand; ++t) old[t] = *grad_ptr(row, min(t, n_own - 1));
        }
    };
    auto store_row = [&](auto slot, int row) {
        constexpr int S = decltype(slot)::value;
        if constexpr (GRAD != 0) {
            if (n_own == kBand) {
#pragma unroll
                for (int t = 0; t < kBand; ++t) *grad_ptr(row, t) = GRAD == 2 ? old[t] + g[S][t] : g[S][t];
            } else {
#pragma unroll
                for (int t = 0; t < kBand; ++t)
                    if (t < n_own) *grad_ptr(row, t) = GRAD == 2 ? old[t] + g[S][t] : g[S][t];
            }
        }
#pragma unroll
        for (int t = 0; t < kBand; ++t) g[S][t] = 0.f;
    };

    // one row of centres: rows c-1, c, c+1 are in p[R0], p[R1], p[R2]
    auto centre_row = [&](auto r0c, int c) {
        constexpr int R0 = decltype(r0c)::value, R1 = (R0 + 1) % 3, R2 = (R0 + 2) % 3;
        const float cm = s_cm[c], c0 = s_c0[c], cp = s_cp[c], rc = s_r[c];
        // neighbourhood columns q-1, q, q+1 of the centre in column q, and the gradient pieces of
        // columns q-1 (all but the current centre's in) and q (the centres so far)
        float p00 = p[R0][0], p10 = p[R1][0], p20 = p[R2][0];
        float p01 = p[R0][1], p11 = p[R1][1], p21 = p[R2][1];
        float a00 = 0.f, a10 = 0.f, a20 = 0.f, a01 = 0.f, a11 = 0.f, a21 = 0.f;
#pragma unroll
        for (int i = 0; i < kCentres; ++i) {
            const float p02 = p[R0][i + 2], p12 = p[R1][i + 2], p22 = p[R2][i + 2];
            const float on = (on_mask >> i & 1) ? 1.0f : 0.0f;
            const float d11 = on * (cm * p01 + c0 * p11 + cp * p21);
            const float d22 = col_cm[i] * (p10 - p11) + col_cp[i] * (p12 - p11);
            const float rr = rc * col_r[i];
            const float d12 = rr * (p22 - p20 - p02 + p00);
            if (i >= 1 && i <= kBand) h_sum += d11 * d11 + 2.0f * d12 * d12 + d22 * d22;  // the wave's own centres
            if constexpr (GRAD == 0) {
                p00 = p01; p10 = p11; p20 = p21;
                p01 = p02; p11 = p12; p21 = p22;
                continue;
            }
            const float e11 = 2.0f * gs * d11, e22 = 2.0f * gs * d22, e12 = 4.0f * gs * rr * d12;
            const float e22m = col_cm[i] * e22, e22p = col_cp[i] * e22;
            // column q-1 receives its last pieces and leaves the sliding registers
            if (i >= 2) {
                g[R0][i - 2] += a00 + e12;
                g[R1][i - 2] += a10 + e22m;
                g[R2][i - 2] += a20 - e12;
            }
            // column q
            a00 = a01 + cm * e11;
            a10 = a11 + c0 * e11 - (e22m + e22p);
            a20 = a21 + cp * e11;
            // column q+1 starts
            a01 = -e12;
            a11 = e22p;
            a21 = e12;
            p00 = p01; p10 = p11; p20 = p21;
            p01 = p02; p11 = p12; p21 = p22;
        }
    };

    // Rows are walked three at a time so that every ring index is a compile-time constant:
    // c = 1 (mod 3) at the top, row c + d has rows c+d-1, c+d, c+d+1 in p[d], p[d+1], p[d+2] (mod 3).
    auto step = [&](auto dc, int c) {
        constexpr int D = decltype(dc)::value;
        request_old(c - 1);
        request(std::integral_constant<int, (D + 2) % 3>{}, c + 4);  // row c+4 -> raw[(c+4) % 3], free since row c+1 left it
        centre_row(dc, c);
        store_row(dc, c - 1);
        // row c+2 has arrived (it was requested two rows ago): it takes the place of row c-1
#pragma unroll
        for (int q = 0; q < kCols; ++q) p[D][q] = widen(raw[D][q]);
    };
    // (leaving the loop in the middle rather than skipping steps: no path through the loop body
    // then runs a step without the steps before it, see the note at `request`)
    for (int c3 = 1;; c3 += 3) {
        if (c3 > G - 1) break;
        step(std::integral_constant<int, 0>{}, c3);
        if (c3 + 1 > G - 1) break;
        step(std::integral_constant<int, 1>{}, c3 + 1);
        if (c3 + 2 > G - 1) break;
        step(std::integral_constant<int, 2>{}, c3 + 2);
    }
    // the last two gradient rows: row G-1 sits in g[(G-1) % 3]
    static_for(std::make_integer_sequence<int, 3>{}, [&](auto sc) {
        constexpr int S = decltype(sc)::value;
        if ((G - 1) % 3 == S) {
            request_old(G - 1);
            store_row(std::integral_constant<int, S>{}, G - 1);
            request_old(G);
            store_row(std::integral_constant<int, (S + 1) % 3>{}, G);
        }
    });
    // value: sum over the wave, one double atomic per wave
    double part = live ? (double)h_sum * (double)inv_n : 0.0;
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) part += __shfl_down(part, d, 64);
    if (lane == 0 && a.value) atomicAdd(a.value, part);
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
    a.K = s.pairs();
    a.n_out = s.n_out;
    if (value) launch_fill_zero(reinterpret_cast<float *>(value), 2, stream);
    const dim3 grid((unsigned)s.out_tiles(), (unsigned)s.pairs());
    const int bands = (s.G + 1 + kBand - 1) / kBand;
    typedef void (*Kernel)(HessArgs);
    static const Kernel table[3][3] = {
        {hessian_reg_kernel<float, 0>, hessian_reg_kernel<float, 1>, hessian_reg_kernel<float, 2>},
        {hessian_reg_kernel<_Float16, 0>, hessian_reg_kernel<_Float16, 1>, hessian_reg_kernel<_Float16, 2>},
        {hessian_reg_kernel<bf16_t, 0>, hessian_reg_kernel<bf16_t, 1>, hessian_reg_kernel<bf16_t, 2>},
    };
    table[s.dtype][grad ? (accumulate ? 2 : 1) : 0]<<<grid, 64 * bands, 0, stream>>>(a);
}

}  // namespace lmkan
