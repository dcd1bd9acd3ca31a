// Coefficient gradient without atomics.
//
//   gP[a][b][k][j] = sum over samples n whose cell for pair k has (a,b) as a corner of
//                    B_ab(x_n) * gy[n][j]                  (derivative of Alg. 1's sum)
//
// Pass 1 (sort_records_kernel): for every pair k the samples are grouped by cell with a
// counting sort, and the four B-spline products are stored next to the sample index.
// Pass 2 (backward_coef_sorted_kernel): one wave owns (pair k, 64 outputs) and walks the
// cells in order.  Inside a cell the four corner sums live in registers (lanes = outputs,
// weights are wave-uniform scalars), so a value of gy feeds four multiply-adds.  Finished
// cells are added into a two-row window of the table kept in LDS (each lane only ever
// touches its own column, so no synchronisation is needed); a table row is written to
// global memory exactly once, when the walk has passed it.  Rows no sample touches are
// written as exact zeros, so no separate zero fill is needed.
#include "lmkan_kernels.h"

namespace lmkan {

namespace {

constexpr int kTile = LMKAN_PACK_TILE;
constexpr int kSortThreads = 1024;

// records_in: [3][K][B] (node, u, v) from the preamble pass.
// sorted:     [5][K][B] (sample index, w00, w10, w01, w11) grouped by cell i1*G+i2.
// cell_start: [K][G*G+1] exclusive prefix sums of the cell populations.
__global__ __launch_bounds__(kSortThreads) void sort_records_kernel(const int32_t *__restrict__ rec_node,
                                                                   const float *__restrict__ rec_u,
                                                                   const float *__restrict__ rec_v,
                                                                   int32_t *__restrict__ sorted_n,
                                                                   float *__restrict__ sorted_w,
                                                                   int32_t *__restrict__ cell_start,
                                                                   int64_t B, int K, int G)
{
    __shared__ int s_count[LMKAN_MAX_GRID * LMKAN_MAX_GRID + 1];
    __shared__ int s_wave_total[kSortThreads / 64];
    const int k = blockIdx.x;
    const int cells = G * G, W = G + 1;
    const int32_t *node_k = rec_node + (int64_t)k * B;
    const float *u_k = rec_u + (int64_t)k * B;
    const float *v_k = rec_v + (int64_t)k * B;
    const int64_t plane = (int64_t)K * B;

    for (int c = threadIdx.x; c <= cells; c += blockDim.x) s_count[c] = 0;
    __syncthreads();
    for (int64_t n = threadIdx.x; n < B; n += blockDim.x) {
        const int node = node_k[n];
        atomicAdd(&s_count[(node / W) * G + node % W], 1);
    }
    __syncthreads();
    // exclusive scan of s_count[0..cells) in chunks of blockDim.x
    int carry = 0;
    for (int base = 0; base < cells; base += blockDim.x) {
        const int c = base + threadIdx.x;
        const int v = c < cells ? s_count[c] : 0;
        int incl = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int t = __shfl_up(incl, d, 64);
            if ((threadIdx.x & 63) >= d) incl += t;
        }
        if ((threadIdx.x & 63) == 63) s_wave_total[threadIdx.x >> 6] = incl;
        __syncthreads();
        int wave_off = 0;
        for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) wave_off += s_wave_total[w];
        int chunk_total = 0;
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) chunk_total += s_wave_total[w];
        const int excl = carry + wave_off + incl - v;
        __syncthreads();
        if (c < cells) {
            s_count[c] = excl;  // becomes the running cursor of the scatter
            cell_start[(int64_t)k * (cells + 1) + c] = excl;
        }
        carry += chunk_total;
    }
    if (threadIdx.x == 0) cell_start[(int64_t)k * (cells + 1) + cells] = carry;
    __syncthreads();
    for (int64_t n = threadIdx.x; n < B; n += blockDim.x) {
        const int node = node_k[n];
        const float u = u_k[n], v = v_k[n];
        const int pos = atomicAdd(&s_count[(node / W) * G + node % W], 1);
        const int64_t o = (int64_t)k * B + pos;
        const float a_lo = 1.0f - u, b_lo = 1.0f - v;
        sorted_n[o] = (int32_t)n;
        sorted_w[o] = a_lo * b_lo;
        sorted_w[o + plane] = u * b_lo;
        sorted_w[o + 2 * plane] = a_lo * v;
        sorted_w[o + 3 * plane] = u * v;
    }
}

struct CoefGradArgs {
    const int32_t *sorted_n;
    const float *sorted_w;
    const int32_t *cell_start;
    const float *gy;
    float *gP;
    CoefMap gmap;  // layout of Alg. 1
    int64_t B;
    int n_out;
    int K;
    int G;
    int n_jt;
    int accumulate;
};

constexpr int kUnroll = 4;

__global__ __launch_bounds__(64) void backward_coef_sorted_kernel(CoefGradArgs a)
{
    extern __shared__ float win[];  // [2][G+1][64]: table rows i1 and i1+1 of this wave's columns
    const int lane = threadIdx.x;
    const int G = a.G, W = G + 1, cells = G * G;

    // Waves that run together on one XCD (ids congruent mod 8) take the same output tile, so
    // the 64-column slice of gy they all stream stays in that XCD's L2.
    int id = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int jt = id / a.K;
    const int k = id % a.K;

    const int col = jt * kTile + lane;
    const bool col_ok = col < a.n_out;
    const int64_t plane = (int64_t)a.K * a.B;
    const int32_t *sn = a.sorted_n + (int64_t)k * a.B;
    const float *sw = a.sorted_w + (int64_t)k * a.B;
    const int32_t *cs = a.cell_start + (int64_t)k * (cells + 1);
    const float *gy_col = a.gy + (col_ok ? col : 0);
    float *out = a.gP + (int64_t)k * a.gmap.s_pair + col;

    for (int i = 0; i < 2 * W; ++i) win[i * kTile + lane] = 0.0f;

    int beg = __builtin_amdgcn_readfirstlane(cs[0]);
    for (int i1 = 0; i1 < G; ++i1) {
        float *cur = win + (i1 & 1) * W * kTile;
        float *nxt = win + ((i1 + 1) & 1) * W * kTile;
        for (int i2 = 0; i2 < G; ++i2) {
            const int end = __builtin_amdgcn_readfirstlane(cs[i1 * G + i2 + 1]);
            if (end > beg) {
                float a00 = 0.f, a10 = 0.f, a01 = 0.f, a11 = 0.f;
                for (int pos = beg; pos < end; pos += kUnroll) {
                    float g[kUnroll], w00[kUnroll], w10[kUnroll], w01[kUnroll], w11[kUnroll];
#pragma unroll
                    for (int u = 0; u < kUnroll; ++u) {
                        const bool live = pos + u < end;
                        const int p = live ? pos + u : end - 1;
                        const int n = __builtin_amdgcn_readfirstlane(sn[p]);
                        w00[u] = live ? sw[p] : 0.0f;
                        w10[u] = live ? sw[p + plane] : 0.0f;
                        w01[u] = live ? sw[p + 2 * plane] : 0.0f;
                        w11[u] = live ? sw[p + 3 * plane] : 0.0f;
                        g[u] = gy_col[(int64_t)n * a.n_out];
                    }
#pragma unroll
                    for (int u = 0; u < kUnroll; ++u) {
                        a00 = fmaf(w00[u], g[u], a00);
                        a10 = fmaf(w10[u], g[u], a10);
                        a01 = fmaf(w01[u], g[u], a01);
                        a11 = fmaf(w11[u], g[u], a11);
                    }
                }
                cur[i2 * kTile + lane] += a00;
                cur[(i2 + 1) * kTile + lane] += a01;
                nxt[i2 * kTile + lane] += a10;
                nxt[(i2 + 1) * kTile + lane] += a11;
            }
            beg = end;
        }
        // table row i1 is complete: write it, then recycle its buffer for row i1 + 2
        for (int b = 0; b < W; ++b) {
            if (col_ok) {
                float *dst = out + (int64_t)(i1 * W + b) * a.gmap.s_node;
                const float v = cur[b * kTile + lane];
                *dst = a.accumulate ? *dst + v : v;
            }
            cur[b * kTile + lane] = 0.0f;
        }
    }
    const float *last = win + (G & 1) * W * kTile;
    for (int b = 0; b < W; ++b) {
        if (col_ok) {
            float *dst = out + (int64_t)(G * W + b) * a.gmap.s_node;
            const float v = last[b * kTile + lane];
            *dst = a.accumulate ? *dst + v : v;
        }
    }
}

}  // namespace

size_t sorted_records_bytes(const LayerShape &s)
{
    const size_t per_pair_cells = (size_t)s.G * s.G + 1;
    size_t bytes = (size_t)5 * s.pairs() * (size_t)s.batch * 4 + (size_t)s.pairs() * per_pair_cells * 4;
    return (bytes + 255) & ~(size_t)255;
}

void launch_backward_coef_sorted(const LayerShape &s, const void *records, void *sorted, const float *gy,
                                 float *gcoef, bool accumulate, hipStream_t stream)
{
    const size_t n = (size_t)s.pairs() * (size_t)s.batch;
    const int32_t *rec_node = static_cast<const int32_t *>(records);
    const float *rec_u = reinterpret_cast<const float *>(rec_node + n);
    const float *rec_v = rec_u + n;
    int32_t *sorted_n = static_cast<int32_t *>(sorted);
    float *sorted_w = reinterpret_cast<float *>(sorted_n + n);
    int32_t *cell_start = reinterpret_cast<int32_t *>(sorted_w + 4 * n);
    sort_records_kernel<<<s.pairs(), kSortThreads, 0, stream>>>(rec_node, rec_u, rec_v, sorted_n, sorted_w,
                                                               cell_start, s.batch, s.pairs(), s.G);
    CoefGradArgs a;
    a.sorted_n = sorted_n;
    a.sorted_w = sorted_w;
    a.cell_start = cell_start;
    a.gy = gy;
    a.gP = gcoef;
    LayerShape g = s;
    g.layout = LMKAN_LAYOUT_PAPER;
    a.gmap = coef_map(g);
    a.B = s.batch;
    a.n_out = s.n_out;
    a.K = s.pairs();
    a.G = s.G;
    a.n_jt = s.out_tiles();
    a.accumulate = accumulate ? 1 : 0;
    const unsigned lds = (unsigned)(2 * (s.G + 1) * kTile * sizeof(float));
    backward_coef_sorted_kernel<<<s.pairs() * s.out_tiles(), 64, lds, stream>>>(a);
}

}  // namespace lmkan
