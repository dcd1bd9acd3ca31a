// Coefficient gradient without atomics.
//
//   gP[a][b][k][j] = sum over samples n whose cell for pair k has (a,b) as a corner of
//                    B_ab(x_n) * gy[n][j]                  (derivative of Alg. 1's sum)
//
// Pass 1 (sort_records_kernel): for every pair k the samples are grouped by cell with a
// counting sort, each cell padded to whole chunks of four samples, and the four B-spline
// products are stored next to the sample index.
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

constexpr int kChunk = 4;  // samples per chunk; a chunk never straddles two cells
constexpr int kDepth = 6;  // chunks of gy values in flight

// Samples per pair in the sorted stream: every non-empty cell is padded to whole chunks with
// zero-weight entries, and the end is padded so that the pipeline below can run (and
// prefetch) over whole groups of kDepth chunks without bounds checks.
__host__ __device__ inline int64_t stream_stride(int64_t B, int G)
{
    const int64_t body = (B + (int64_t)(kChunk - 1) * G * G + kChunk - 1) / kChunk * kChunk;
    return body + (int64_t)kChunk * (3 * kDepth + 2);
}

// records_in: [3][K][B] (node, u, v) from the preamble pass.  Per pair k, with S = stream_stride:
//   sorted_n [K][S]      sample index (0 in padding entries)
//   sorted_w [K][S]      the four products (w00, w10, w01, w11), zero in padding entries
//   chunk_cell [K][S/4]  i1 << 8 | i2 of the cell each chunk belongs to, non-decreasing
//   n_chunks [K]         chunks to process, a multiple of kDepth
__global__ __launch_bounds__(kSortThreads) void sort_records_kernel(const int32_t *__restrict__ rec_node,
                                                                   const float *__restrict__ rec_u,
                                                                   const float *__restrict__ rec_v,
                                                                   int32_t *__restrict__ sorted_n,
                                                                   f4v *__restrict__ sorted_w,
                                                                   int32_t *__restrict__ chunk_cell,
                                                                   int32_t *__restrict__ n_chunks, int64_t B,
                                                                   int G)
{
    __shared__ int s_count[LMKAN_MAX_GRID * LMKAN_MAX_GRID];  // population, then scatter cursor
    __shared__ int s_start[LMKAN_MAX_GRID * LMKAN_MAX_GRID];  // first stream position of the cell
    __shared__ int s_wave_total[kSortThreads / 64];
    __shared__ int s_last_cell;
    const int k = blockIdx.x;
    const int cells = G * G, W = G + 1;
    const int64_t S = stream_stride(B, G);
    const int32_t *node_k = rec_node + (int64_t)k * B;
    const float *u_k = rec_u + (int64_t)k * B;
    const float *v_k = rec_v + (int64_t)k * B;
    int32_t *out_n = sorted_n + (int64_t)k * S;
    f4v *out_w = sorted_w + (int64_t)k * S;
    int32_t *out_cell = chunk_cell + (int64_t)k * (S / kChunk);

    for (int c = threadIdx.x; c < cells; c += blockDim.x) s_count[c] = 0;
    if (threadIdx.x == 0) s_last_cell = 0;
    __syncthreads();
    for (int64_t n = threadIdx.x; n < B; n += blockDim.x) {
        const int node = node_k[n];
        atomicAdd(&s_count[(node / W) * G + node % W], 1);
    }
    __syncthreads();
    // exclusive scan of the padded populations, in pieces of blockDim.x cells
    int carry = 0;
    for (int base = 0; base < cells; base += blockDim.x) {
        const int c = base + threadIdx.x;
        const int cnt = c < cells ? s_count[c] : 0;
        const int v = (cnt + kChunk - 1) / kChunk * kChunk;
        if (cnt > 0) atomicMax(&s_last_cell, c);
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
        int piece_total = 0;
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) piece_total += s_wave_total[w];
        if (c < cells) s_start[c] = carry + wave_off + incl - v;
        carry += piece_total;
        __syncthreads();
    }
    const int total = carry;  // padded samples of all cells, a multiple of kChunk
    // padding entries and the cell of every chunk
    for (int c = threadIdx.x; c < cells; c += blockDim.x) {
        const int cnt = s_count[c];
        if (cnt == 0) continue;
        const int first = s_start[c], padded = (cnt + kChunk - 1) / kChunk * kChunk;
        const f4v zero = {0.f, 0.f, 0.f, 0.f};
        for (int i = cnt; i < padded; ++i) {
            out_n[first + i] = 0;
            out_w[first + i] = zero;
        }
        const int code = ((c / G) << 8) | (c % G);
        for (int q = first / kChunk; q < (first + padded) / kChunk; ++q) out_cell[q] = code;
    }
    // tail: whole dummy chunks that belong to the last non-empty cell
    const int real_chunks = total / kChunk;
    const int run_chunks = (real_chunks + kDepth - 1) / kDepth * kDepth;
    const int tail_end = run_chunks + 2 * kDepth + 2;  // chunks the pipelines may touch
    {
        const int last = s_last_cell;
        const int code = ((last / G) << 8) | (last % G);
        const f4v zero = {0.f, 0.f, 0.f, 0.f};
        for (int i = total + threadIdx.x; i < tail_end * kChunk; i += blockDim.x) {
            out_n[i] = 0;
            out_w[i] = zero;
        }
        for (int q = real_chunks + threadIdx.x; q < tail_end; q += blockDim.x) out_cell[q] = code;
        if (threadIdx.x == 0) n_chunks[k] = run_chunks;
    }
    __syncthreads();
    for (int c = threadIdx.x; c < cells; c += blockDim.x) s_count[c] = 0;
    __syncthreads();
    for (int64_t n = threadIdx.x; n < B; n += blockDim.x) {
        const int node = node_k[n];
        const float u = u_k[n], v = v_k[n];
        const int c = (node / W) * G + node % W;
        const int pos = s_start[c] + atomicAdd(&s_count[c], 1);
        const float a_lo = 1.0f - u, b_lo = 1.0f - v;
        out_n[pos] = (int32_t)n;
        f4v w;
        w.x = a_lo * b_lo;
        w.y = u * b_lo;
        w.z = a_lo * v;
        w.w = u * v;
        out_w[pos] = w;
    }
}

struct CoefGradArgs {
    const int32_t *sorted_n;
    const f4v *sorted_w;
    const int32_t *chunk_cell;
    const int32_t *n_chunks;
    const float *gy;
    float *gP;
    CoefMap gmap;  // layout of Alg. 1
    int64_t B;
    int64_t S;     // stream_stride
    int n_out;
    int K;
    int G;
    int accumulate;
};

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
    ScalarIntPtr sn = (ScalarIntPtr)(a.sorted_n + (int64_t)k * a.S);
    ScalarWPtr sw = (ScalarWPtr)(a.sorted_w + (int64_t)k * a.S);
    ScalarIntPtr cc = (ScalarIntPtr)(a.chunk_cell + (int64_t)k * (a.S / kChunk));
    const int nch = ((ScalarIntPtr)a.n_chunks)[k];
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

    // Software pipeline over the chunks.  The address of a gy value depends on the sample
    // index, so indices run kDepth+1 chunks ahead of the multiply-adds, the gy loads kDepth
    // chunks ahead (a register ring), weights and the chunk's cell one chunk ahead.
    if (nch > 0) {
        float g[kDepth][kChunk];
        int n_use[kChunk];
        f4v w_cur[kChunk];
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
#pragma unroll
            for (int u = 0; u < kChunk; ++u) g[d][u] = gy_col[(int64_t)sn[d * kChunk + u] * a.n_out];
        }
#pragma unroll
        for (int u = 0; u < kChunk; ++u) {
            n_use[u] = sn[kDepth * kChunk + u];
            w_cur[u] = sw[u];
        }
        int cell_cur = cc[0];
        for (int c = 0; c < nch; c += kDepth) {
#pragma unroll
            for (int p = 0; p < kDepth; ++p) {
                const int j = c + p;
                int n_load[kChunk];
                f4v w_nxt[kChunk];
#pragma unroll
                for (int u = 0; u < kChunk; ++u) {
                    n_load[u] = sn[(j + kDepth + 1) * kChunk + u];
                    w_nxt[u] = sw[(j + 1) * kChunk + u];
                }
                const int cell_nxt = cc[j + 1];
                if (cell_cur != cur_cell) {
                    if (cur_cell >= 0) flush();
                    retire_rows(cell_cur >> 8);
                    cur_cell = cell_cur;
                }
#pragma unroll
                for (int u = 0; u < kChunk; ++u) {
                    a00 = fmaf(w_cur[u].x, g[p][u], a00);
                    a10 = fmaf(w_cur[u].y, g[p][u], a10);
                    a01 = fmaf(w_cur[u].z, g[p][u], a01);
                    a11 = fmaf(w_cur[u].w, g[p][u], a11);
                }
#pragma unroll
                for (int u = 0; u < kChunk; ++u) {
                    g[p][u] = gy_col[(int64_t)n_use[u] * a.n_out];  // chunk j + kDepth
                    n_use[u] = n_load[u];
                    w_cur[u] = w_nxt[u];
                }
                cell_cur = cell_nxt;
            }
        }
    }
    if (cur_cell >= 0) flush();
    retire_rows(W);
}

// Wide variant (n_out a multiple of 4, 16-byte aligned gy and gP): the wave works on the four
// samples of a chunk at once, one per 16-lane group, and a lane covers four adjacent outputs,
// so gy is read with 16-byte loads (the texture path moves 256-byte row pieces four times
// faster that way than as single dwords).  Weights and sample indices are per group and
// therefore come from vector loads.  When a cell ends, the four groups' partial sums are
// combined across the wave and group 0 adds them into the LDS window.
constexpr int kWideDepth = kDepth;  // chunks of gy values and weights in flight; indices run twice as far ahead

__global__ __launch_bounds__(64) void backward_coef_wide_kernel(CoefGradArgs a)
{
    extern __shared__ __align__(16) float win[];  // [2][G+1][64]
    const int lane = threadIdx.x;
    const int g = lane >> 4, l16 = lane & 15;
    const int G = a.G, W = G + 1;

    int id = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int jt = id / a.K;
    const int k = id % a.K;

    const int col = jt * kTile + l16 * 4;
    const bool col_ok = col < a.n_out;
    typedef __attribute__((address_space(4))) const int32_t *ScalarIntPtr;
    const int32_t *sn = a.sorted_n + (int64_t)k * a.S + g;  // this group's sample of each chunk
    const f4v *sw = a.sorted_w + (int64_t)k * a.S + g;
    ScalarIntPtr cc = (ScalarIntPtr)(a.chunk_cell + (int64_t)k * (a.S / kChunk));
    const int nch = ((ScalarIntPtr)a.n_chunks)[k];
    const float *gy_col = a.gy + (col_ok ? col : 0);
    float *out = a.gP + (int64_t)k * a.gmap.s_pair + col;

    for (int i = lane; i < 2 * W * kTile; i += 64) win[i] = 0.0f;

    f4v acc00 = {0.f, 0.f, 0.f, 0.f}, acc10 = acc00, acc01 = acc00, acc11 = acc00;
    int cur_cell = -1;
    int rows_done = 0;

    auto wave_sum = [&](f4v v) {
        f4v r;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float t = v[i];
            t += __shfl_xor(t, 16, 64);
            t += __shfl_xor(t, 32, 64);
            r[i] = t;
        }
        return r;
    };
    auto flush = [&]() {
        const int i1 = cur_cell >> 8, i2 = cur_cell & 255;
        const f4v s00 = wave_sum(acc00), s10 = wave_sum(acc10), s01 = wave_sum(acc01), s11 = wave_sum(acc11);
        if (g == 0) {
            f4v *cur = reinterpret_cast<f4v *>(win + (i1 & 1) * W * kTile + i2 * kTile) + l16;
            f4v *nxt = reinterpret_cast<f4v *>(win + ((i1 + 1) & 1) * W * kTile + i2 * kTile) + l16;
            cur[0] += s00;
            cur[kTile / 4] += s01;
            nxt[0] += s10;
            nxt[kTile / 4] += s11;
        }
        acc00 = acc10 = acc01 = acc11 = f4v{0.f, 0.f, 0.f, 0.f};
    };
    // four table rows entries per store instruction: group g takes b = 4 i + g
    auto retire_rows = [&](int upto) {
        for (; rows_done < upto; ++rows_done) {
            f4v *row = reinterpret_cast<f4v *>(win + (rows_done & 1) * W * kTile) + l16;
            for (int b = g; b < W; b += 4) {
                if (col_ok) {
                    f4v *dst = reinterpret_cast<f4v *>(out + (int64_t)(rows_done * W + b) * a.gmap.s_node);
                    const f4v v = row[b * (kTile / 4)];
                    *dst = a.accumulate ? *dst + v : v;
                }
                row[b * (kTile / 4)] = f4v{0.f, 0.f, 0.f, 0.f};
            }
        }
    };

    if (nch > 0) {
        // three-stage pipeline, all through in-order vector loads: at step j the sample index of
        // chunk j + 2 depth is requested, the index of chunk j + depth (requested depth steps ago)
        // addresses the gy and weight loads of that chunk, and chunk j is consumed
        f4v gq[kWideDepth], wq[kWideDepth];
        int nq[kWideDepth];
#pragma unroll
        for (int d = 0; d < kWideDepth; ++d) {
            gq[d] = *reinterpret_cast<const f4v *>(gy_col + (int64_t)sn[d * kChunk] * a.n_out);
            wq[d] = sw[d * kChunk];
            nq[d] = sn[(kWideDepth + d) * kChunk];
        }
        // cells of a whole group of chunks are fetched one group ahead (scalar loads return out
        // of order, so every use waits for all of them: keep them few and early)
        int cells_now[kWideDepth], cells_nxt[kWideDepth];
#pragma unroll
        for (int p = 0; p < kWideDepth; ++p) cells_now[p] = cc[p];
        for (int c = 0; c < nch; c += kWideDepth) {
#pragma unroll
            for (int p = 0; p < kWideDepth; ++p) cells_nxt[p] = cc[c + kWideDepth + p];
#pragma unroll
            for (int p = 0; p < kWideDepth; ++p) {
                const int j = c + p;
                const int cell_cur = cells_now[p];
                if (cell_cur != cur_cell) {
                    if (cur_cell >= 0) flush();
                    retire_rows(cell_cur >> 8);
                    cur_cell = cell_cur;
                }
                acc00 += wq[p].x * gq[p];
                acc10 += wq[p].y * gq[p];
                acc01 += wq[p].z * gq[p];
                acc11 += wq[p].w * gq[p];
                gq[p] = *reinterpret_cast<const f4v *>(gy_col + (int64_t)nq[p] * a.n_out);
                wq[p] = sw[(j + kWideDepth) * kChunk];
                nq[p] = sn[(j + 2 * kWideDepth) * kChunk];
            }
#pragma unroll
            for (int p = 0; p < kWideDepth; ++p) cells_now[p] = cells_nxt[p];
        }
    }
    if (cur_cell >= 0) flush();
    retire_rows(W);
}

}  // namespace

size_t sorted_records_bytes(const LayerShape &s)
{
    const size_t S = (size_t)stream_stride(s.batch, s.G);
    const size_t per_pair = S * (sizeof(f4v) + sizeof(int32_t)) + (S / kChunk) * sizeof(int32_t) + sizeof(int32_t);
    return ((size_t)s.pairs() * per_pair + 255) & ~(size_t)255;
}

void launch_backward_coef_sorted(const LayerShape &s, const void *records, void *sorted, const float *gy,
                                 float *gcoef, bool accumulate, hipStream_t stream)
{
    const size_t n = (size_t)s.pairs() * (size_t)s.batch;
    const size_t S = (size_t)stream_stride(s.batch, s.G);
    const size_t K = (size_t)s.pairs();
    const int32_t *rec_node = static_cast<const int32_t *>(records);
    const float *rec_u = reinterpret_cast<const float *>(rec_node + n);
    const float *rec_v = rec_u + n;
    f4v *sorted_w = static_cast<f4v *>(sorted);  // 16-byte items first, then the 4-byte ones
    int32_t *sorted_n = reinterpret_cast<int32_t *>(sorted_w + K * S);
    int32_t *chunk_cell = sorted_n + K * S;
    int32_t *n_chunks = chunk_cell + K * (S / kChunk);
    sort_records_kernel<<<s.pairs(), kSortThreads, 0, stream>>>(rec_node, rec_u, rec_v, sorted_n, sorted_w,
                                                               chunk_cell, n_chunks, s.batch, s.G);
    CoefGradArgs a;
    a.sorted_n = sorted_n;
    a.sorted_w = sorted_w;
    a.chunk_cell = chunk_cell;
    a.n_chunks = n_chunks;
    a.gy = gy;
    a.gP = gcoef;
    LayerShape g = s;
    g.layout = LMKAN_LAYOUT_PAPER;
    a.gmap = coef_map(g);
    a.B = s.batch;
    a.S = (int64_t)S;
    a.n_out = s.n_out;
    a.K = s.pairs();
    a.G = s.G;
    a.accumulate = accumulate ? 1 : 0;
    const unsigned lds = (unsigned)(2 * (s.G + 1) * kTile * sizeof(float));
    const bool wide = s.n_out % 4 == 0 &&
                      ((reinterpret_cast<uintptr_t>(gy) | reinterpret_cast<uintptr_t>(gcoef)) & 15) == 0;
    if (wide)
        backward_coef_wide_kernel<<<s.pairs() * s.out_tiles(), 64, lds, stream>>>(a);
    else
        backward_coef_sorted_kernel<<<s.pairs() * s.out_tiles(), 64, lds, stream>>>(a);
}

}  // namespace lmkan
