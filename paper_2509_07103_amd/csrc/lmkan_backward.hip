// Coefficient gradient without atomics.
//
//   gP[a][b][k][j] = sum over samples n whose cell for pair k has (a,b) as a corner of
//                    B_ab(x_n) * gy[n][j]                  (derivative of Alg. 1's sum)
//
// Pass 1 (sort_count / sort_layout / sort_scatter kernels): for every pair k the samples are
// grouped by cell with a counting sort, each cell padded to whole chunks of four samples, and
// the four B-spline products are stored next to the sample index.
// Pass 2 (backward_coef_stream_kernel): one wave owns (pair k, 64 outputs) and walks the
// sorted chunks, cell after cell.  The four samples of a chunk go to the four 16-lane
// groups of the wave and a lane covers four adjacent outputs, so gy is read with 16-byte
// loads.  Within a cell the update is a small dense contraction, (4 corners x samples) times
// (samples x outputs), and runs on the matrix cores: one 4x4x1 float32 MFMA (16 blocks)
// multiplies the four products of each group's sample with one gy value per lane, the
// block-broadcast control handing every block of a group the products of that group's sample.
// The 16 partial sums (4 corners x 4 outputs) live in the MFMA accumulators.  When the cell
// ends they are combined across the groups and added into a
// two-row window of the table kept in LDS; a table row is written to global memory exactly
// once, when the walk has passed it.  Rows no sample touches are written as exact zeros, so
// no separate zero fill is needed.
#include "lmkan_kernels.h"
#include "lmkan_sorted.h"

namespace lmkan {

namespace {

constexpr int kTile = LMKAN_PACK_TILE;
constexpr int kSortThreads = 1024;

constexpr int kDepth = 8;    // chunks of gy values in flight
constexpr int kPerW = 4;     // chunks whose entries one load instruction brings in
static_assert(kUnroll % kDepth == 0, "the gy ring must divide the unrolled trip");

// Counting sort of the samples of every pair by cell, in three launches so that long batches
// are spread over many workgroups.  records_in: [3][K][B] (node, u, v) from the preamble
// pass.  Per pair k, with S = stream_stride, the samples ordered by (block, cell):
//   rec [K][S]           (u, v, 1, index) of a sample, 16 bytes; padding entries are
//                        (0, 0, 0, index of a sample of the same cell)
//   chunk_cell [K][S/4]  i1 << 8 | i2 of the cell each chunk belongs to, non-decreasing
//                        inside a block
//   block_start [K][blocks+1]  first chunk of every block (multiples of kUnroll) and the
//                        number of chunks to process
// and as scratch between the launches, with nblk = ceil(B / kSortSeg) batch segments:
//   seg_count [K][nblk][G*G]  population of a cell inside a segment, then the offset of the
//                             segment's first sample of that cell within the cell
//   cell_start [K][blocks][G*G]  first stream position of the (block, cell)
//   cell_rep [K][G*G]         index of some sample of the cell (any one)
constexpr int kSortSegThreads = 256;
constexpr int kMaxCells = LMKAN_MAX_GRID * LMKAN_MAX_GRID;

__device__ __forceinline__ int cell_of_node(int node, int G) { return (node / (G + 1)) * G + node % (G + 1); }

// 1: histogram of one batch segment
__global__ __launch_bounds__(kSortSegThreads) void sort_count_kernel(const int32_t *__restrict__ rec_node,
                                                                    int32_t *__restrict__ seg_count,
                                                                    int32_t *__restrict__ cell_rep, int64_t B, int G)
{
    __shared__ int s_count[kMaxCells];
    __shared__ int s_rep[kMaxCells];
    const int blk = blockIdx.x, nblk = gridDim.x, k = blockIdx.y;
    const int cells = G * G;
    for (int c = threadIdx.x; c < cells; c += blockDim.x) s_count[c] = 0;
    __syncthreads();
    const int64_t n0 = (int64_t)blk * kSortSeg;
    const int64_t n1 = n0 + kSortSeg < B ? n0 + kSortSeg : B;
    const int32_t *node_k = rec_node + (int64_t)k * B;
    // all loads of the thread first: these passes are bound by the bytes in flight
    constexpr int kPer = kSortSeg / kSortSegThreads;
    int nd[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int64_t n = n0 + threadIdx.x + j * kSortSegThreads;
        nd[j] = n < n1 ? node_k[n] : -1;
    }
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        if (nd[j] >= 0) {
            const int c = cell_of_node(nd[j], G);
            atomicAdd(&s_count[c], 1);
            s_rep[c] = (int)(n0 + threadIdx.x + j * kSortSegThreads);  // any writer wins
        }
    }
    __syncthreads();
    int32_t *out = seg_count + ((int64_t)k * nblk + blk) * cells;
    for (int c = threadIdx.x; c < cells; c += blockDim.x) {
        const int cnt = s_count[c];
        out[c] = cnt;
        if (cnt > 0) cell_rep[(int64_t)k * cells + c] = s_rep[c];  // any segment wins
    }
}

// 1b: chunks of every (pair, block): cells padded to whole chunks, the block to whole trips
__global__ __launch_bounds__(kSortSegThreads) void sort_block_size_kernel(const int32_t *__restrict__ seg_count,
                                                                         int32_t *__restrict__ block_size, int64_t B,
                                                                         int G, int nseg)
{
    __shared__ int s_sum[kSortSegThreads / 64];
    const int k = blockIdx.x, blk = blockIdx.y;
    const int cells = G * G;
    const int blocks = stream_blocks(B);
    const int seg_per_block = blocks > 1 ? kSegPerBlock : nseg;
    const int b0 = blk * seg_per_block, b1 = min(nseg, b0 + seg_per_block);
    const int32_t *cnt_k = seg_count + (int64_t)k * nseg * cells;
    int mine = 0;
    for (int c = threadIdx.x; c < cells; c += blockDim.x) {
        int run = 0;
        for (int b = b0; b < b1; ++b) run += cnt_k[(int64_t)b * cells + c];
        mine += (run + kChunk - 1) / kChunk;
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) mine += __shfl_down(mine, d, 64);
    if ((threadIdx.x & 63) == 0) s_sum[threadIdx.x >> 6] = mine;
    __syncthreads();
    if (threadIdx.x == 0) {
        int total = 0;
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) total += s_sum[w];
        block_size[(int64_t)k * blocks + blk] = (total + kUnroll - 1) / kUnroll * kUnroll;
    }
}

// 2: per (pair, block): positions of the cells (each padded to whole chunks), the
// cell of every chunk, padding entries, dummy chunks that round the block up to whole trips
// (they belong to the block's last cell), and after the last block the tail
__global__ __launch_bounds__(kSortThreads) void sort_layout_kernel(int32_t *__restrict__ seg_count,
                                                                  int32_t *__restrict__ cell_start,
                                                                  const int32_t *__restrict__ cell_rep,
                                                                  f4v *__restrict__ rec,
                                                                  int32_t *__restrict__ chunk_cell,
                                                                  int32_t *__restrict__ block_start,
                                                                  const int32_t *__restrict__ block_size, int64_t B,
                                                                  int G, int nseg)
{
    __shared__ int s_count[kMaxCells];      // population of the cell in this block
    __shared__ int s_start[kMaxCells + 1];  // first stream position of the cell; [cells] = end
    __shared__ int s_wave_total[kSortThreads / 64];
    __shared__ int s_last_cell;
    const int k = blockIdx.x;
    const int cells = G * G;
    const int blocks = stream_blocks(B);
    const int seg_per_block = blocks > 1 ? kSegPerBlock : nseg;
    const int64_t S = stream_stride(B, G);
    f4v *out = rec + (int64_t)k * S;
    int32_t *out_cell = chunk_cell + (int64_t)k * (S / kChunk);
    int32_t *cnt_k = seg_count + (int64_t)k * nseg * cells;
    const int32_t *rep_k = cell_rep + (int64_t)k * cells;
    int32_t *bs_k = block_start + (int64_t)k * (blocks + 1);
    auto filler = [](int32_t n) { return f4v{0.f, 0.f, 0.f, __int_as_float(n)}; };

    const int blk = blockIdx.y;
    // stream position where this block starts (a multiple of kChunk * kUnroll)
    int base_pos = 0;
    for (int b = 0; b < blk; ++b) base_pos += block_size[(int64_t)k * blocks + b] * kChunk;
    {
        const int b0 = blk * seg_per_block, b1 = min(nseg, b0 + seg_per_block);
        if (threadIdx.x == 0) s_last_cell = 0;
        __syncthreads();
        // populations; the per-segment counts become offsets inside the (block, cell)
        for (int c = threadIdx.x; c < cells; c += blockDim.x) {
            int run = 0;
            for (int b = b0; b < b1; ++b) {
                const int v = cnt_k[(int64_t)b * cells + c];
                cnt_k[(int64_t)b * cells + c] = run;
                run += v;
            }
            s_count[c] = run;
            if (run > 0) atomicMax(&s_last_cell, c);
        }
        __syncthreads();
        // exclusive scan of the padded populations, in pieces of blockDim.x cells
        int carry = base_pos;
        for (int base = 0; base < cells; base += blockDim.x) {
            const int c = base + threadIdx.x;
            const int cnt = c < cells ? s_count[c] : 0;
            const int v = (cnt + kChunk - 1) / kChunk * kChunk;
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
        const int real_end = carry;  // end of the padded samples of this block
        const int block_chunks = ((real_end - base_pos) / kChunk + kUnroll - 1) / kUnroll * kUnroll;
        const int block_end = base_pos + block_chunks * kChunk;
        // the last block is followed by the chunks the pipelines may touch beyond the end
        const int fill_end = blk + 1 < blocks ? block_end : block_end + kUnroll * kChunk;
        for (int c = threadIdx.x; c < cells; c += blockDim.x)
            cell_start[((int64_t)k * blocks + blk) * cells + c] = s_start[c];
        const int last = s_last_cell;
        // the cell of every chunk: the highest cell whose start is <= the chunk's first position
        // (an empty cell shares its start with the next one, so the highest such cell is never
        // empty); chunks past the real ones belong to the block's last cell
        for (int q = base_pos / kChunk + threadIdx.x; q < fill_end / kChunk; q += blockDim.x) {
            int c = last;
            const int pos = q * kChunk;
            if (pos < real_end) {
                int lo = 0, hi = cells - 1;
                while (lo < hi) {
                    const int mid = (lo + hi + 1) >> 1;
                    if (s_start[mid] <= pos) lo = mid; else hi = mid - 1;
                }
                c = lo;
            }
            out_cell[q] = ((c / G) << 8) | (c % G);
        }
        // padding entries of every cell, then the dummy chunks: zero products, a sample of that cell
        for (int c = threadIdx.x; c < cells; c += blockDim.x) {
            const int cnt = s_count[c];
            if (cnt == 0) continue;
            const int first = s_start[c], padded = (cnt + kChunk - 1) / kChunk * kChunk;
            const f4v fill = filler(rep_k[c]);
            for (int i = cnt; i < padded; ++i) out[first + i] = fill;
        }
        {
            const f4v fill = filler(rep_k[last]);
            for (int i = real_end + threadIdx.x; i < fill_end; i += blockDim.x) out[i] = fill;
        }
        if (threadIdx.x == 0) {
            bs_k[blk] = base_pos / kChunk;
            if (blk + 1 == blocks) bs_k[blocks] = block_end / kChunk;
        }
    }
}

// 3: scatter of one batch segment.  The segment is first ordered by cell inside LDS, so that
// consecutive threads then write consecutive stream positions (the samples of one cell that
// lie in this segment form one contiguous run of the stream).
__host__ __device__ inline size_t scatter_lds_bytes(int G)
{
    return (size_t)((G * G * 3 + 3) & ~3) * sizeof(int) + (size_t)kSortSeg * (2 * sizeof(float) + 3 * sizeof(unsigned short));
}

__global__ __launch_bounds__(kSortSegThreads) void sort_scatter_kernel(const int32_t *__restrict__ rec_node,
                                                                      const float *__restrict__ rec_u,
                                                                      const float *__restrict__ rec_v,
                                                                      const int32_t *__restrict__ seg_count,
                                                                      const int32_t *__restrict__ cell_start,
                                                                      f4v *__restrict__ rec, int64_t B, int G,
                                                                      int stable)
{
    extern __shared__ __align__(16) int s_dyn[];
    __shared__ int s_wave[kSortSegThreads / 64];
    const int seg = blockIdx.x, nseg = gridDim.x, k = blockIdx.y;
    const int cells = G * G;
    int *s_cnt = s_dyn;              // population of the cell inside this segment
    int *s_lstart = s_cnt + cells;   // its first position in the segment's own cell order
    int *s_gbase = s_lstart + cells; // its first position in the stream
    float *s_u = reinterpret_cast<float *>(s_dyn + ((3 * cells + 3) & ~3));  // 16-byte aligned: s_order is read 16 bytes at a time
    float *s_v = s_u + kSortSeg;
    unsigned short *s_cell = reinterpret_cast<unsigned short *>(s_v + kSortSeg);
    unsigned short *s_rank = s_cell + kSortSeg;
    unsigned short *s_order = s_rank + kSortSeg;
    const int blocks = stream_blocks(B);
    const int blk = blocks > 1 ? seg / kSegPerBlock : 0;
    const int64_t S = stream_stride(B, G);
    const int32_t *off = seg_count + ((int64_t)k * nseg + seg) * cells;
    for (int c = threadIdx.x; c < cells; c += blockDim.x) {
        s_cnt[c] = 0;
        s_gbase[c] = cell_start[((int64_t)k * blocks + blk) * cells + c] + off[c];
    }
    __syncthreads();
    const int64_t n0 = (int64_t)seg * kSortSeg;
    const int count = (int)((n0 + kSortSeg < B ? n0 + kSortSeg : B) - n0);
    const int32_t *node_k = rec_node + (int64_t)k * B + n0;
    const float *u_k = rec_u + (int64_t)k * B + n0;
    const float *v_k = rec_v + (int64_t)k * B + n0;
    {
        constexpr int kPer = kSortSeg / kSortSegThreads;
        int nd[kPer];
        float uu[kPer], vv[kPer];
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int i = threadIdx.x + j * kSortSegThreads;
            nd[j] = -1;
            uu[j] = vv[j] = 0.f;
            if (i < count) {
                nd[j] = node_k[i];
                uu[j] = u_k[i];
                vv[j] = v_k[i];
            }
        }
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int i = threadIdx.x + j * kSortSegThreads;
            if (nd[j] >= 0) {
                const int c = cell_of_node(nd[j], G);
                s_cell[i] = (unsigned short)c;
                s_rank[i] = (unsigned short)atomicAdd(&s_cnt[c], 1);
                s_u[i] = uu[j];
                s_v[i] = vv[j];
            }
        }
    }
    __syncthreads();
    // exclusive scan of the populations: a run of consecutive cells per thread
    {
        const int per = (cells + kSortSegThreads - 1) / kSortSegThreads;
        const int c0 = threadIdx.x * per, c1 = min(cells, c0 + per);
        int mine = 0;
        for (int c = c0; c < c1; ++c) mine += s_cnt[c];
        int incl = mine;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int t = __shfl_up(incl, d, 64);
            if ((threadIdx.x & 63) >= d) incl += t;
        }
        if ((threadIdx.x & 63) == 63) s_wave[threadIdx.x >> 6] = incl;
        __syncthreads();
        int run = incl - mine;
        for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) run += s_wave[w];
        for (int c = c0; c < c1; ++c) {
            s_lstart[c] = run;
            run += s_cnt[c];
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < count; i += blockDim.x) s_order[s_lstart[s_cell[i]] + s_rank[i]] = (unsigned short)i;
    __syncthreads();
    // The ranks so far are in the order the atomics happened to be served.  Where the order of
    // the samples inside a cell reaches the result (a coefficient gradient summed cell by cell by
    // one wave), replace them by the order of the sample indices (rank = number of samples of the
    // same cell, in this segment, with a smaller index), so that the stream, and with it the
    // order of every float32 sum over the samples of a cell, is the same in every run.
    for (int i = threadIdx.x; stable && i < count; i += blockDim.x) {
        const int c = s_cell[i];
        // the run is read eight entries (16 bytes) at a time from an aligned position; entries
        // outside the run are masked
        const int first = s_lstart[c], end = first + s_cnt[c];
        int r = 0;
        for (int a = first & ~7; a < end; a += 8) {
            const uint4 w = *reinterpret_cast<const uint4 *>(s_order + a);
            const unsigned word[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int v = (int)((word[e >> 1] >> (16 * (e & 1))) & 0xffffu);
                r += (a + e >= first) & (a + e < end) & (v < i);
            }
        }
        s_rank[i] = (unsigned short)r;
    }
    __syncthreads();
    for (int i = threadIdx.x; stable && i < count; i += blockDim.x)
        s_order[s_lstart[s_cell[i]] + s_rank[i]] = (unsigned short)i;
    __syncthreads();
    f4v *out = rec + (int64_t)k * S;
    for (int lp = threadIdx.x; lp < count; lp += blockDim.x) {
        const int i = s_order[lp];
        const int c = s_cell[i];
        const int pos = s_gbase[c] + lp - s_lstart[c];
        out[pos] = f4v{s_u[i], s_v[i], 1.0f, __int_as_float((int32_t)(n0 + i))};
    }
}

struct CoefGradArgs {
    const f4v *rec;
    const int32_t *chunk_cell;
    const int32_t *block_start;  // [K][n_blocks + 1], in chunks
    GyView gy;
    float *gP;
    CoefMap gmap;  // layout of Alg. 1
    int64_t B;
    int64_t S;     // stream_stride
    int n_out;
    int K;
    int G;
    int accumulate;
    int n_blocks;  // locality blocks of the batch
    int n_sub;     // waves per (pair, output tile, block)
};

template <bool kOffset32>
__global__ __launch_bounds__(64) void backward_coef_stream_kernel(CoefGradArgs a)
{
    extern __shared__ __align__(16) float win[];  // [2][G+1][64]: table rows r and r+1 of this wave's columns
    const int lane = threadIdx.x;
    const int g = lane >> 4, l16 = lane & 15;
    const int G = a.G, W = G + 1;

    // Waves that run together on one XCD (ids congruent mod 8) take the same output tile and the
    // same block of the batch, so the piece of gy they all gather from stays in that XCD's L2.
    int id = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int sub = id % a.n_sub;
    id /= a.n_sub;
    const int k = id % a.K;
    id /= a.K;
    const int blk = id % a.n_blocks;
    const int jt = id / a.n_blocks;

    const int col = jt * kTile + l16 * 4;
    const bool col_ok = col < a.n_out;
    typedef __attribute__((address_space(4))) const int32_t *ScalarIntPtr;
    // With one block and one wave per (pair, tile) the wave owns its columns of the gradient and
    // writes every row once.  Otherwise (long batches; too few pairs x tiles to fill the chip)
    // a wave takes a run of whole trips of one block; a run may begin and end anywhere, even
    // inside a cell: every wave then adds what it has into a gradient that starts at zero.
    const bool split = a.n_blocks > 1 || a.n_sub > 1;
    ScalarIntPtr bs = (ScalarIntPtr)(a.block_start + (int64_t)k * (a.n_blocks + 1));
    int c_begin = bs[blk];
    int nch = bs[blk + 1] - c_begin;
    if (a.n_sub > 1) {
        const int trips = nch / kUnroll;
        const int per = (trips + a.n_sub - 1) / a.n_sub * kUnroll;
        const int skip = min(sub * per, nch);
        c_begin += skip;
        nch = min(per, nch - skip);
    }
    if (split && nch == 0) return;
    ScalarIntPtr cc = (ScalarIntPtr)(a.chunk_cell + (int64_t)k * (a.S / kChunk) + c_begin);
    float *out = a.gP + (int64_t)k * a.gmap.s_pair + col;

    // entries: lane (g, 4 j + q) fetches the entry of group g's sample of chunk c + j and will
    // form its product q, so one load brings in four chunks (256 contiguous bytes); sample
    // indices: lane (g, j) fetches the index of group g's sample of chunk c + j, sixteen chunks
    // per load
    const f4v *rec_k = a.rec + (int64_t)k * a.S + (int64_t)c_begin * kChunk;  // wave-uniform
    // The loads of the main loop are written as inline assembly, and so are the waits for them:
    // vector loads return in the order they were issued, and with the cell changes branching
    // inside the loop the compiler sizes its own waits for the worst path it can imagine, which
    // drains the ring of gy values at every step (it emitted vmcnt(0) ... vmcnt(6) where 9 loads
    // may stay in flight).  Every load below is issued at a fixed place of a trip, so the number
    // of younger loads at the point of use is known; loads the compiler adds on the rare paths
    // (row stores, atomics) only add to that number, which keeps the waits safe.
    const unsigned e_off = (unsigned)(((l16 >> 2) * kChunk + g) * sizeof(f4v));
    const unsigned n_off = (unsigned)((l16 * kChunk + g) * sizeof(f4v) + 12);
    // (operands are copied into locals first: a name used only as an asm operand is not captured)
    auto load_e = [&](f4v &dst, int chunk) {
        const f4v *base = rec_k + (int64_t)chunk * kChunk;
        const unsigned off = e_off;
        asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(dst) : "v"(off), "s"(base) : "memory");
    };
    auto load_n = [&](int &dst, int chunk) {
        const f4v *base = rec_k + (int64_t)chunk * kChunk;
        const unsigned off = n_off;
        asm volatile("global_load_dword %0, %1, %2" : "=v"(dst) : "v"(off), "s"(base) : "memory");
    };
    // blocks until at most N loads younger than the one that fills v are outstanding, i.e. until v has landed.
    // The compiler does not know that v is in flight between the load and this wait: were it to copy
    // or move v in between, it would copy stale data and hand the old register to something else for
    // the late load to overwrite.  The comment in the instruction names the register, so that the
    // generated code can be checked (check_codegen.py does, at every build): on every path from a
    // load, the first instruction that touches its destination must be this wait.
    auto landed = [](auto &v, auto nc) {
        asm volatile("s_waitcnt vmcnt(%1) ; landed %0" : "+v"(v) : "n"(decltype(nc)::value) : "memory");
    };

    const unsigned col_bytes = col_ok ? (unsigned)l16 * 16u : 0u;
    const unsigned row_bytes = a.gy.row_stride;
    const char *gy_tile = reinterpret_cast<const char *>(a.gy.base) + (int64_t)jt * a.gy.tile_stride;
    // what a lane keeps of the sixteen samples of a trip: the byte offset of the sample's row when
    // every offset fits 32 bits (one multiply per trip; the broadcast to the group then folds into
    // the add of the lane's column, a single DPP instruction per chunk), else the sample index
    auto row_offset = [&](int n) { return kOffset32 ? (int)__umul24((unsigned)n, row_bytes) : n; };
    auto load_gy = [&](f4v &dst, auto subc, int off16) {
        constexpr int SUB = decltype(subc)::value;
        if constexpr (kOffset32) {
            const unsigned off = (unsigned)row_bcast<SUB>(off16) + col_bytes;
            const char *base = gy_tile;
            asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(dst) : "v"(off), "s"(base) : "memory");
        } else {
            const char *ptr = gy_tile + ((int64_t)row_bcast<SUB>(off16) * row_bytes + col_bytes);
            asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(ptr) : "memory");
        }
    };

    for (int i = lane; i < 2 * W * kTile; i += 64) win[i] = 0.0f;

    f4v acc[4];  // [output i of the lane][corner q]
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = f4v{0.f, 0.f, 0.f, 0.f};
    int cur_cell = -1;  // (i1 << 8 | i2) of the cell the accumulators belong to
    int rows_done = 0;  // table rows [0, rows_done) have been written out

    // add the sums of the finished cell into the two-row window: group 0 holds corner
    // (i1, i2), group 1 (i1 + 1, i2), group 2 (i1, i2 + 1), group 3 (i1 + 1, i2 + 1)
    auto flush = [&]() {
        const int i1 = cur_cell >> 8, i2 = cur_cell & 255;
        float f[4];
        combine_groups(acc, f);
        const int row = (i1 + (g & 1)) & 1, b = i2 + (g >> 1);
        f4v *p = reinterpret_cast<f4v *>(win + (row * W + b) * kTile) + l16;
        f4v v = *p;
        v.x += f[0];
        v.y += f[1];
        v.z += f[2];
        v.w += f[3];
        *p = v;
    };
    // table rows below `upto` can receive nothing more: write them and recycle their buffers.
    // Owned columns: four table entries per store instruction, group g takes b = 4 i + g.
    // Shared gradient: one atomic instruction per entry, lanes on consecutive floats (256
    // contiguous bytes), entries this wave never touched left alone.
    const int out_col = jt * kTile + lane;
    float *out_lane = a.gP + (int64_t)k * a.gmap.s_pair + out_col;
    auto retire_rows = [&](int upto) {
        for (; rows_done < upto; ++rows_done) {
            if (split) {
                float *row = win + (rows_done & 1) * W * kTile + lane;
                for (int b = 0; b < W; ++b) {
                    const float v = row[b * kTile];
                    row[b * kTile] = 0.f;
                    if (v != 0.f && out_col < a.n_out)
                        unsafeAtomicAdd(out_lane + (int64_t)(rows_done * W + b) * a.gmap.s_node, v);
                }
            } else {
                f4v *row = reinterpret_cast<f4v *>(win + (rows_done & 1) * W * kTile) + l16;
                for (int b = g; b < W; b += 4) {
                    if (col_ok) {
                        float *dst = out + (int64_t)(rows_done * W + b) * a.gmap.s_node;
                        const f4v v = row[b * (kTile / 4)];
                        if ((a.n_out & 3) == 0) {
                            f4v *d4 = reinterpret_cast<f4v *>(dst);
                            *d4 = a.accumulate ? *d4 + v : v;
                        } else {
                            // rows of the gradient do not start on 16 bytes and the last one is short
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (col + e < a.n_out) dst[e] = a.accumulate ? dst[e] + v[e] : v[e];
                        }
                    }
                    row[b * (kTile / 4)] = f4v{0.f, 0.f, 0.f, 0.f};
                }
            }
        }
    };

    if (nch > 0) {
        // Software pipeline, all through in-order vector loads: at step P of a trip the chunk
        // c + P is consumed and the gy values of chunk c + P + kDepth are requested (their sample
        // indices were loaded a trip earlier); a register of products is refilled for the next
        // trip as soon as its fourth chunk has been consumed.  Order of issue in a trip: the
        // indices of the next trip, then per step one gy load, after every fourth step one load
        // of entries: 21 loads.
        f4v eq[kUnroll / kPerW];   // entries as loaded
        float wq[kUnroll / kPerW];  // their products, formed when the first of the four chunks is consumed
        f4v gq[kDepth];
        int n_now, n_nxt;
        // The fill is issued in the order the steady state leaves the loads in at the top of a
        // trip, so that the wait counts of the first steps are those of every other trip.
        load_n(n_now, 0);
        static_for(std::make_integer_sequence<int, kUnroll / kPerW>{}, [&](auto rc) {
            constexpr int r = decltype(rc)::value;
            if constexpr (r * kPerW < kUnroll - kDepth) load_e(eq[r], r * kPerW);
        });
        landed(n_now, std::integral_constant<int, (kUnroll - kDepth) / kPerW>{});
        n_now = row_offset(n_now);
        static_for(std::make_integer_sequence<int, kDepth>{}, [&](auto dc) {
            constexpr int d = decltype(dc)::value;
            constexpr int P = kUnroll - kDepth + d;  // the step that requests this chunk in later trips
            load_gy(gq[d], std::integral_constant<int, d>{}, n_now);
            if constexpr (P % kPerW == kPerW - 1) load_e(eq[P / kPerW], (P / kPerW) * kPerW);
        });
        // cells of a whole trip are fetched one trip ahead (scalar loads return out of order, so
        // every use waits for all of them: keep them few and early)
        int cells_now[kUnroll], cells_nxt[kUnroll];
#pragma unroll
        for (int p = 0; p < kUnroll; ++p) cells_now[p] = cc[p];
        if (split) rows_done = cells_now[0] >> 8;  // rows before the run's first cell are not this wave's
        for (int c = 0; c < nch; c += kUnroll) {
#pragma unroll
            for (int p = 0; p < kUnroll; ++p) cells_nxt[p] = cc[c + kUnroll + p];
            load_n(n_nxt, c + kUnroll);
            static_for(std::make_integer_sequence<int, kUnroll>{}, [&](auto pc) {
                constexpr int P = decltype(pc)::value;
                const int cell_cur = cells_now[P];
                // Younger loads at this point.  A gy value: the 7 gy loads after it and two loads
                // of entries (three in the first trip, four when the top of a trip lies between).
                // Entries: 16 (12 for the first register in the first trip).  Indices: 8 gy loads
                // and 2 loads of entries.
                if constexpr (P == kUnroll - kDepth) {
                    landed(n_nxt, std::integral_constant<int, kDepth + kDepth / kPerW>{});
                    n_nxt = row_offset(n_nxt);  // first needed below
                }
                if constexpr (P % kPerW == 0) {
                    landed(eq[P / kPerW], std::integral_constant<int, P == 0 ? 12 : 15>{});
                    wq[P / kPerW] = entry_product(eq[P / kPerW], l16 & 3);
                }
                landed(gq[P % kDepth], std::integral_constant<int, kDepth - 1 + kDepth / kPerW>{});
                if (cell_cur != cur_cell) {
                    if (cur_cell >= 0) flush();
                    retire_rows(cell_cur >> 8);
                    cur_cell = cell_cur;
                    chunk_fma<P % kPerW, true>(acc, wq[P / kPerW], gq[P % kDepth]);
                } else {
                    chunk_fma<P % kPerW, false>(acc, wq[P / kPerW], gq[P % kDepth]);
                }
                load_gy(gq[P % kDepth], std::integral_constant<int, (P + kDepth) % kUnroll>{},
                        P + kDepth < kUnroll ? n_now : n_nxt);
                if constexpr (P % kPerW == kPerW - 1) load_e(eq[P / kPerW], c + kUnroll + (P / kPerW) * kPerW);
            });
            n_now = n_nxt;
#pragma unroll
            for (int p = 0; p < kUnroll; ++p) cells_now[p] = cells_nxt[p];
        }
        // nothing may still be on its way to a register once the compiler is free to reuse it
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    if (cur_cell >= 0) flush();
    retire_rows(split ? min(W, (cur_cell >> 8) + 2) : W);
}

}  // namespace

size_t sorted_records_bytes(const LayerShape &s)
{
    const size_t S = (size_t)stream_stride(s.batch, s.G);
    const size_t nseg = ((size_t)s.batch + kSortSeg - 1) / kSortSeg;
    const size_t blocks = (size_t)stream_blocks(s.batch);
    const size_t cells = (size_t)s.G * s.G;
    const size_t per_pair = S * sizeof(f4v) + (S / kChunk) * sizeof(int32_t) + (2 * blocks + 1) * sizeof(int32_t) +
                            (nseg + blocks + 1) * cells * sizeof(int32_t);
    return ((size_t)s.pairs() * per_pair + 255) & ~(size_t)255;
}

// The cell-sorted paths index stream positions, and the launch grids batch segments, with 32-bit
// integers: the longest batch they take.  Longer ones go to the generic kernels.
bool sorted_batch_ok(const LayerShape &s)
{
    const int64_t nseg = (s.batch + kSortSeg - 1) / kSortSeg;
    return nseg <= 65535 && stream_blocks(s.batch) <= 65535 && stream_stride(s.batch, s.G) < ((int64_t)1 << 31);
}

// gy is gathered four columns at a time and the gradient leaves four columns at a time: with a
// ragged output count gy comes from its tile-by-tile copy and the last columns of the gradient are
// stored one by one, which any 4-byte aligned buffers allow
bool sorted_shape_ok(const LayerShape &s) { return sorted_batch_ok(s); }

bool coef_sorted_applicable(const LayerShape &s, const float *gy, const float *gcoef)
{
    if (!sorted_shape_ok(s)) return false;
    if (ragged_outputs(s)) return true;
    return ((reinterpret_cast<uintptr_t>(gy) | reinterpret_cast<uintptr_t>(gcoef)) & 15) == 0;
}

SortBuffers sort_buffers(const LayerShape &s, void *sorted)
{
    const size_t S = (size_t)stream_stride(s.batch, s.G);
    const size_t K = (size_t)s.pairs();
    const size_t nseg = ((size_t)s.batch + kSortSeg - 1) / kSortSeg;
    const size_t blocks = (size_t)stream_blocks(s.batch);
    const size_t cells = (size_t)s.G * s.G;
    SortBuffers b;
    b.rec = static_cast<f4v *>(sorted);  // 16-byte items first, then the 4-byte ones
    b.chunk_cell = reinterpret_cast<int32_t *>(b.rec + K * S);
    b.block_start = b.chunk_cell + K * (S / kChunk);
    b.block_size = b.block_start + K * (blocks + 1);
    b.seg_count = b.block_size + K * blocks;
    b.cell_start = b.seg_count + K * nseg * cells;
    b.cell_rep = b.cell_start + K * blocks * cells;
    return b;
}

SortedStream launch_sort(const LayerShape &s, const void *records, void *sorted, hipStream_t stream)
{
    // a fixed order inside the cells matters only where one wave sums a cell from start to end
    const bool stable = stream_blocks(s.batch) == 1 && stream_run_split(s) == 1;
    const size_t n = (size_t)s.pairs() * (size_t)s.batch;
    const size_t K = (size_t)s.pairs();
    const int32_t *rec_node = static_cast<const int32_t *>(records);
    const float *rec_u = reinterpret_cast<const float *>(rec_node + n);
    const float *rec_v = rec_u + n;
    const SortBuffers b = sort_buffers(s, sorted);
    const size_t nseg = ((size_t)s.batch + kSortSeg - 1) / kSortSeg;
    const size_t blocks = (size_t)stream_blocks(s.batch);
    const dim3 seg_grid((unsigned)nseg, (unsigned)K);
    sort_count_kernel<<<seg_grid, kSortSegThreads, 0, stream>>>(rec_node, b.seg_count, b.cell_rep, s.batch, s.G);
    const dim3 block_grid((unsigned)K, (unsigned)blocks);
    sort_block_size_kernel<<<block_grid, kSortSegThreads, 0, stream>>>(b.seg_count, b.block_size, s.batch, s.G,
                                                                       (int)nseg);
    sort_layout_kernel<<<block_grid, kSortThreads, 0, stream>>>(b.seg_count, b.cell_start, b.cell_rep, b.rec,
                                                              b.chunk_cell, b.block_start, b.block_size, s.batch, s.G,
                                                              (int)nseg);
    const size_t scatter_lds = scatter_lds_bytes(s.G);
    if (scatter_lds > 64 * 1024) allow_large_lds(reinterpret_cast<const void *>(sort_scatter_kernel), 160 * 1024 - 64);
    sort_scatter_kernel<<<seg_grid, kSortSegThreads, scatter_lds, stream>>>(rec_node, rec_u, rec_v, b.seg_count,
                                                                           b.cell_start, b.rec, s.batch,
                                                                           s.G, stable ? 1 : 0);
    SortedStream st;
    st.rec = b.rec;
    st.chunk_cell = b.chunk_cell;
    st.block_start = b.block_start;
    st.S = (int64_t)stream_stride(s.batch, s.G);
    st.n_blocks = (int)blocks;
    return st;
}

void launch_backward_coef_sorted(const LayerShape &s, const SortedStream &st, const GyView &gy, float *gcoef,
                                 bool accumulate, hipStream_t stream)
{
    CoefGradArgs a;
    a.rec = st.rec;
    a.chunk_cell = st.chunk_cell;
    a.block_start = st.block_start;
    a.gy = gy;
    a.gP = gcoef;
    LayerShape g = s;
    g.layout = LMKAN_LAYOUT_PAPER;
    a.gmap = coef_map(g);
    a.B = s.batch;
    a.S = st.S;
    a.n_out = s.n_out;
    a.K = s.pairs();
    a.G = s.G;
    a.accumulate = accumulate ? 1 : 0;
    const unsigned lds = (unsigned)(2 * (s.G + 1) * kTile * sizeof(float));
    const int n_sub = stream_run_split(s);
    a.n_blocks = st.n_blocks;
    a.n_sub = n_sub;
    if ((st.n_blocks > 1 || n_sub > 1) && !accumulate)
        launch_fill_zero(gcoef, (size_t)s.nodes() * (size_t)s.pairs() * (size_t)s.n_out, stream);
    const unsigned grid = (unsigned)((int64_t)s.pairs() * s.out_tiles() * st.n_blocks * n_sub);
    KernelTiming timing(stream, kTimeGradCoef);
    if (gy_offsets_fit_32_bits(s, gy))
        backward_coef_stream_kernel<true><<<grid, 64, lds, stream>>>(a);
    else
        backward_coef_stream_kernel<false><<<grid, 64, lds, stream>>>(a);
}

// Runs per (pair, tile, block).  One block: cut the stream when pairs x tiles cannot fill
// 256 CUs x 16 waves.  Several blocks: as many runs as it takes for the pairs of one (tile,
// block) to occupy an XCD (512 waves), so that the XCD works on one block at a time.  A run
// keeps at least four trips.
int stream_run_split(const LayerShape &s)
{
    const int64_t streams = (int64_t)s.pairs() * s.out_tiles();
    int n_sub = 1;
    if (stream_blocks(s.batch) == 1) {
        const int64_t trips = stream_stride(s.batch, s.G) / (kChunk * kUnroll);
        while (streams * n_sub < 4096 && trips / (n_sub * 2) >= 4 && n_sub < 64) n_sub *= 2;
    } else {
        const int64_t trips = kBlockSamples / (kChunk * kUnroll);
        while ((int64_t)s.pairs() * n_sub < 512 && trips / (n_sub * 2) >= 4 && n_sub < 32) n_sub *= 2;
    }
    return n_sub;
}

// 24-bit multiply and 32-bit byte offsets into gy when the tensor is small enough
bool gy_offsets_fit_32_bits(const LayerShape &s, const GyView &gy)
{
    return s.batch < (1 << 24) && gy.row_stride < (1u << 24) &&
           (int64_t)s.batch * gy.row_stride < ((int64_t)1 << 32);
}

namespace {

// out[t][n][c] = gy[n][64 t + c], zero past n_out; one thread per four columns, threads in the
// order of gy's rows
__global__ __launch_bounds__(256) void gy_tiles_kernel(const float *__restrict__ gy, float *__restrict__ out,
                                                       int64_t B, int n_out, int tiles)
{
    const int64_t per_row = (int64_t)tiles * (kTile / 4);
    const int64_t total = B * per_row;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t n = i / per_row;
        const int r = (int)(i - n * per_row);
        const int t = r / (kTile / 4), c = (r % (kTile / 4)) * 4;
        const int col = t * kTile + c;
        f4v v = {0.f, 0.f, 0.f, 0.f};
        if ((n_out & 3) == 0) {
            if (col < n_out) v = *reinterpret_cast<const f4v *>(gy + n * n_out + col);
        } else {
            // rows of gy do not start on 16 bytes
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (col + e < n_out) v[e] = gy[n * n_out + col + e];
        }
        *reinterpret_cast<f4v *>(out + ((int64_t)t * B + n) * kTile + c) = v;
    }
}

}  // namespace

// Measured: the copy pays from rows of 8 KiB on (at 4096 outputs the gathers' HBM reads fall from
// 62 GB to 18 GB and the coefficient gradient gains 9 %; at 1024 outputs it costs 2 %).
// A ragged output count needs the copy whatever the width: its rows are padded to whole tiles.
static bool gy_tiles_pay(const LayerShape &s) { return (size_t)s.n_out * sizeof(float) >= 8192 || ragged_outputs(s); }

size_t gy_tiles_bytes(const LayerShape &s)
{
    if (!gy_tiles_pay(s)) return 0;
    return ((size_t)s.out_tiles() * (size_t)s.batch * kTile * sizeof(float) + 255) & ~(size_t)255;
}

GyView launch_gy_tiles(const LayerShape &s, const float *gy, void *tiles, hipStream_t stream)
{
    GyView v;
    if (!gy_tiles_pay(s)) {
        v.base = gy, v.tile_stride = kTile * sizeof(float), v.row_stride = (unsigned)s.n_out * sizeof(float);
        return v;
    }
    const int64_t total = s.batch * (int64_t)s.out_tiles() * (kTile / 4);
    const unsigned grid = (unsigned)std::min<int64_t>((total + 255) / 256, 256 * 32);
    gy_tiles_kernel<<<grid, 256, 0, stream>>>(gy, static_cast<float *>(tiles), s.batch, s.n_out, s.out_tiles());
    v.base = static_cast<const float *>(tiles);
    v.tile_stride = s.batch * (int64_t)(kTile * sizeof(float));
    v.row_stride = kTile * sizeof(float);
    return v;
}

}  // namespace lmkan
