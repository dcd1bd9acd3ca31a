// Coefficient gradient without atomics.
//
//   gP[a][b][k][j] = sum over samples n whose cell for pair k has (a,b) as a corner of
//                    B_ab(x_n) * gy[n][j]                  (derivative of Alg. 1's sum)
//
// Pass 1 (sort_records_kernel): for every pair k the samples are grouped by cell with a
// counting sort, and the four B-spline products are stored next to the sample index.
// Pass 2 (backward_coef_sorted_kernel): one wave owns (pair k, 64 outputs) and walks the
// sorted samples, cell after cell.  Inside a cell the four corner sums live in registers (lanes = outputs,
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

typedef float f4v __attribute__((ext_vector_type(4)));

// records_in: [3][K][B] (node, u, v) from the preamble pass.
// sorted_n / sorted_cell: [K][B] sample index and i1 << 8 | i2, grouped by cell in increasing
//             order of i1 * G + i2;  sorted_w: [K][B] the four products (w00, w10, w01, w11).
__global__ __launch_bounds__(kSortThreads) void sort_records_kernel(const int32_t *__restrict__ rec_node,
                                                                   const float *__restrict__ rec_u,
                                                                   const float *__restrict__ rec_v,
                                                                   int32_t *__restrict__ sorted_n,
                                                                   int32_t *__restrict__ sorted_cell,
                                                                   f4v *__restrict__ sorted_w, int64_t B,
                                                                   int G)
{
    __shared__ int s_count[LMKAN_MAX_GRID * LMKAN_MAX_GRID + 1];
    __shared__ int s_wave_total[kSortThreads / 64];
    const int k = blockIdx.x;
    const int cells = G * G, W = G + 1;
    const int32_t *node_k = rec_node + (int64_t)k * B;
    const float *u_k = rec_u + (int64_t)k * B;
    const float *v_k = rec_v + (int64_t)k * B;

    for (int c = threadIdx.x; c <= cells; c += blockDim.x) s_count[c] = 0;
    __syncthreads();
    for (int64_t n = threadIdx.x; n < B; n += blockDim.x) {
        const int node = node_k[n];
        atomicAdd(&s_count[(node / W) * G + node % W], 1);
    }
    __syncthreads();
    // exclusive scan of s_count[0..cells) in chunks of blockDim.x; the result is the running
    // cursor of the scatter below
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
        if (c < cells) s_count[c] = excl;
        carry += chunk_total;
    }
    __syncthreads();
    for (int64_t n = threadIdx.x; n < B; n += blockDim.x) {
        const int node = node_k[n];
        const float u = u_k[n], v = v_k[n];
        const int i1 = node / W, i2 = node % W;
        const int pos = atomicAdd(&s_count[i1 * G + i2], 1);
        const int64_t o = (int64_t)k * B + pos;
        const float a_lo = 1.0f - u, b_lo = 1.0f - v;
        sorted_n[o] = (int32_t)n;
        sorted_cell[o] = (i1 << 8) | i2;
        f4v w;
        w.x = a_lo * b_lo;
        w.y = u * b_lo;
        w.z = a_lo * v;
        w.w = u * v;
        sorted_w[o] = w;
    }
}

struct CoefGradArgs {
    const int32_t *sorted_n;
    const int32_t *sorted_cell;
    const f4v *sorted_w;
    const float *gy;
    float *gP;
    CoefMap gmap;  // layout of Alg. 1
    int64_t B;
    int n_out;
    int K;
    int G;
    int accumulate;
};

constexpr int kChunk = 4;  // samples per pipeline stage
constexpr int kDepth = 6;  // chunks of gy values in flight

__global__ __launch_bounds__(64) void backward_coef_sorted_kernel(CoefGradArgs a)
{
    extern __shared__ float win[];  // [2][G+1][64]: table rows r and r+1 of this wave's columns
    const int lane = threadIdx.x;
    const int G = a.G, W = G + 1;

    // Waves that run together on one XCD (ids congruent mod 8) take the same output tile, so
    // the 64-column slice of gy they all stream stays in that XCD's L2.
    int id = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int jt = id / a.K;
    const int k = id % a.K;

    const int col = jt * kTile + lane;
    const bool col_ok = col < a.n_out;
    // The sorted records are read through the scalar unit: positions are wave-uniform and the
    // weights are the same for all 64 outputs, so they belong in SGPRs.
    typedef __attribute__((address_space(4))) const int32_t *ScalarIntPtr;
    typedef __attribute__((address_space(4))) const f4v *ScalarWPtr;
    ScalarIntPtr sn = (ScalarIntPtr)(a.sorted_n + (int64_t)k * a.B);
    ScalarIntPtr sc = (ScalarIntPtr)(a.sorted_cell + (int64_t)k * a.B);
    ScalarWPtr sw = (ScalarWPtr)(a.sorted_w + (int64_t)k * a.B);
    const float *gy_col = a.gy + (col_ok ? col : 0);
    float *out = a.gP + (int64_t)k * a.gmap.s_pair + col;

    for (int i = 0; i < 2 * W; ++i) win[i * kTile + lane] = 0.0f;

    float a00 = 0.f, a10 = 0.f, a01 = 0.f, a11 = 0.f;
    int cur_cell = -1;    // (i1 << 8 | i2) of the cell the accumulators belong to
    int rows_done = 0;    // table rows [0, rows_done) have been written out

    // add the accumulators of the finished cell into the two-row window
    auto flush = [&]() {
        const int i1 = cur_cell >> 8, i2 = cur_cell & 255;
        float *cur = win + (i1 & 1) * W * kTile + i2 * kTile + lane;
        float *nxt = win + ((i1 + 1) & 1) * W * kTile + i2 * kTile + lane;
        cur[0] += a00;
        cur[kTile] += a01;
        nxt[0] += a10;
        nxt[kTile] += a11;
        a00 = a10 = a01 = a11 = 0.f;
    };
    // table rows below `upto` can receive nothing more: write them and recycle their buffers
    auto retire_rows = [&](int upto) {
        for (; rows_done < upto; ++rows_done) {
            float *row = win + (rows_done & 1) * W * kTile + lane;
            for (int b = 0; b < W; ++b) {
                if (col_ok) {
                    float *dst = out + (int64_t)(rows_done * W + b) * a.gmap.s_node;
                    const float v = row[b * kTile];
                    *dst = a.accumulate ? *dst + v : v;
                }
                row[b * kTile] = 0.0f;
            }
        }
    };
    auto consume = [&](int cell, f4v w, float g) {
        if (cell != cur_cell) {
            if (cur_cell >= 0) flush();
            retire_rows(cell >> 8);
            cur_cell = cell;
        }
        a00 = fmaf(w.x, g, a00);
        a10 = fmaf(w.y, g, a10);
        a01 = fmaf(w.z, g, a01);
        a11 = fmaf(w.w, g, a11);
    };

    // Software pipeline over chunks of kChunk samples.  The address of a gy value depends on
    // the sample index, so indices run kDepth+1 chunks ahead of the multiply-adds, the gy
    // loads kDepth chunks ahead (a register ring), weights and cell ids one chunk ahead.
    const int n_chunks = (int)(a.B / kChunk);
    int done = 0;  // chunks consumed
    if (n_chunks >= 2 * kDepth) {
        float g[kDepth][kChunk];
        int n_use[kChunk], cell_cur[kChunk];
        f4v w_cur[kChunk];
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
#pragma unroll
            for (int u = 0; u < kChunk; ++u) g[d][u] = gy_col[(int64_t)sn[d * kChunk + u] * a.n_out];
        }
#pragma unroll
        for (int u = 0; u < kChunk; ++u) {
            n_use[u] = sn[kDepth * kChunk + u];
            cell_cur[u] = sc[u];
            w_cur[u] = sw[u];
        }
        // chunks [0, limit) are consumed here; every load below stays inside [0, n_chunks)
        const int limit = ((n_chunks - kDepth - 1) / kDepth) * kDepth;
        for (int c = 0; c < limit; c += kDepth) {
#pragma unroll
            for (int p = 0; p < kDepth; ++p) {
                const int j = c + p;  // chunk consumed in this step; j + kDepth + 1 < n_chunks
                int n_load[kChunk], cell_nxt[kChunk];
                f4v w_nxt[kChunk];
#pragma unroll
                for (int u = 0; u < kChunk; ++u) {
                    n_load[u] = sn[(j + kDepth + 1) * kChunk + u];
                    cell_nxt[u] = sc[(j + 1) * kChunk + u];
                    w_nxt[u] = sw[(j + 1) * kChunk + u];
                }
#pragma unroll
                for (int u = 0; u < kChunk; ++u) consume(cell_cur[u], w_cur[u], g[p][u]);
#pragma unroll
                for (int u = 0; u < kChunk; ++u) {
                    g[p][u] = gy_col[(int64_t)n_use[u] * a.n_out];  // chunk j + kDepth
                    n_use[u] = n_load[u];
                    cell_cur[u] = cell_nxt[u];
                    w_cur[u] = w_nxt[u];
                }
            }
        }
        // drain: the ring holds chunks limit .. limit + kDepth - 1, w_cur / cell_cur chunk `limit`
#pragma unroll
        for (int p = 0; p < kDepth; ++p) {
#pragma unroll
            for (int u = 0; u < kChunk; ++u) {
                const int pos = (limit + p) * kChunk + u;
                consume(p == 0 ? cell_cur[u] : sc[pos], p == 0 ? w_cur[u] : sw[pos], g[p][u]);
            }
        }
        done = limit + kDepth;
    }
    for (int64_t pos = (int64_t)done * kChunk; pos < a.B; ++pos)
        consume(sc[pos], sw[pos], gy_col[(int64_t)sn[pos] * a.n_out]);
    if (cur_cell >= 0) flush();
    retire_rows(W);
}

}  // namespace

size_t sorted_records_bytes(const LayerShape &s)
{
    const size_t bytes = (size_t)s.pairs() * (size_t)s.batch * (2 * sizeof(int32_t) + sizeof(f4v));
    return (bytes + 255) & ~(size_t)255;
}

void launch_backward_coef_sorted(const LayerShape &s, const void *records, void *sorted, const float *gy,
                                 float *gcoef, bool accumulate, hipStream_t stream)
{
    const size_t n = (size_t)s.pairs() * (size_t)s.batch;
    const int32_t *rec_node = static_cast<const int32_t *>(records);
    const float *rec_u = reinterpret_cast<const float *>(rec_node + n);
    const float *rec_v = rec_u + n;
    f4v *sorted_w = static_cast<f4v *>(sorted);  // 16-byte items first, then the 8-byte ones
    int32_t *sorted_n = reinterpret_cast<int32_t *>(sorted_w + n);
    int32_t *sorted_cell = sorted_n + n;
    sort_records_kernel<<<s.pairs(), kSortThreads, 0, stream>>>(rec_node, rec_u, rec_v, sorted_n, sorted_cell,
                                                               sorted_w, s.batch, s.G);
    CoefGradArgs a;
    a.sorted_n = sorted_n;
    a.sorted_cell = sorted_cell;
    a.sorted_w = sorted_w;
    a.gy = gy;
    a.gP = gcoef;
    LayerShape g = s;
    g.layout = LMKAN_LAYOUT_PAPER;
    a.gmap = coef_map(g);
    a.B = s.batch;
    a.n_out = s.n_out;
    a.K = s.pairs();
    a.G = s.G;
    a.accumulate = accumulate ? 1 : 0;
    const unsigned lds = (unsigned)(2 * (s.G + 1) * kTile * sizeof(float));
    backward_coef_sorted_kernel<<<s.pairs() * s.out_tiles(), 64, lds, stream>>>(a);
}

}  // namespace lmkan
