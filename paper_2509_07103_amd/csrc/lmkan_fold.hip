// Inference-time folds of a float32 table, in place (App. E Eq. 4b, App. F.1).
//
//   y' = s_j (gamma lmKAN(x) + Linear(ReLU(x)))_j + t_j
// is one lmKAN layer with coefficients
//   P'[a][b][k][j] = s_j (gamma P[a][b][k][j] + Wl[j][2k] max(E[a], 0) + Wl[j][2k+1] max(E[b], 0))
//                    + [k == 0] (s_j bias_j + t_j)
// (exact when 0 is a grid point, i.e. G even: a piecewise-linear table with a node at the
// kink reproduces ReLU; a per-output constant may sit in the table of any one pair because the
// four weights of a cell sum to one).  Elementwise over the table: one read, one write.
#include "lmkan_kernels.h"

namespace lmkan {

namespace {

struct FoldArgs {
    float *P;
    CoefMap map;
    GridTab tab;
    const float *lin_w;  // [n_out][n_in] or null
    const float *lin_b;  // [n_out] or null
    const float *scale;  // [n_out] or null
    const float *shift;  // [n_out] or null
    float gamma;
    int n_in;
    int n_out;
    int K;
};

// grid: x over (k, j) columns in units of 256 threads, y over the first node index; a thread
// walks the second one, so that its two linear weights and its per-output terms (strided,
// uncoalesced reads) are fetched once per table row rather than once per node
__global__ __launch_bounds__(256) void fold_kernel(FoldArgs a)
{
    const int64_t col = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (col >= (int64_t)a.K * a.n_out) return;
    const int k = (int)(col / a.n_out), j = (int)(col - (int64_t)k * a.n_out);
    const int W = a.tab.G + 1;
    const int ia = blockIdx.y;
    const float ra = fmaxf(a.tab.node[ia], 0.0f);
    const float wa = a.lin_w ? a.lin_w[(int64_t)j * a.n_in + 2 * k] : 0.0f;
    const float wb = a.lin_w ? a.lin_w[(int64_t)j * a.n_in + 2 * k + 1] : 0.0f;
    const float s = a.scale ? a.scale[j] : 1.0f;
    const float c = k == 0 ? s * (a.lin_b ? a.lin_b[j] : 0.0f) + (a.shift ? a.shift[j] : 0.0f) : 0.0f;
    float *p = a.P + (int64_t)ia * W * a.map.s_node + (int64_t)k * a.map.s_pair + (int64_t)(j >> 6) * a.map.s_tile + (j & 63);
    for (int ib = 0; ib < W; ++ib, p += a.map.s_node) {
        const float rb = fmaxf(a.tab.node[ib], 0.0f);
        float v = a.gamma * *p;
        if (a.lin_w) v += wa * ra + wb * rb;
        v *= s;
        if (k == 0) v += c;
        *p = v;
    }
}

}  // namespace

void launch_fold(const LayerShape &s, const GridTab &tab, float *coef, float gamma, const float *lin_w,
                 const float *lin_b, const float *scale, const float *shift, hipStream_t stream)
{
    FoldArgs a;
    a.P = coef;
    a.map = coef_map(s);
    a.tab = tab;
    a.lin_w = lin_w;
    a.lin_b = lin_b;
    a.scale = scale;
    a.shift = shift;
    a.gamma = gamma;
    a.n_in = s.n_in;
    a.n_out = s.n_out;
    a.K = s.pairs();
    const int64_t cols = (int64_t)s.pairs() * s.n_out;
    const dim3 grid((unsigned)((cols + 255) / 256), (unsigned)(s.G + 1));
    fold_kernel<<<grid, 256, 0, stream>>>(a);
}

}  // namespace lmkan
