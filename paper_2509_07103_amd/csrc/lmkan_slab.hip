// Tuned float32 forward for layers whose table slab fits LDS twice.
//
// Work decomposition.  One workgroup owns a tile of samples x 64 outputs and
// walks over (a range of) the input pairs.  For pair k the (G+1)^2 x 64
// coefficient "slab" is streamed from global memory straight into LDS
// (double buffered, LDS-direct 16-byte loads), while the accumulators
// y[sample][output] stay in registers for the whole walk.
//
// Inside a wave the 64 lanes are 4 groups of 16; a group reads one 256-byte
// table row with one ds_read_b128 per lane (conflict-free, full LDS rate), so a
// wave processes 4 samples per step and each lane accumulates 4 outputs per
// sample.  The preamble of Alg. 1 (cell + weights) is computed once per
// (sample, pair) by a separate pass and stored as records; lane l of a wave
// fetches the record of sample l, and the group that processes that sample takes
// the weights directly from that lane's registers through the DPP row broadcast
// of v_fmac_f32, so the four multiply-adds of Alg. 1 cost exactly four VALU
// instructions per output quadruple.
#include <utility>

#include "lmkan_kernels.h"
#include "lmkan_slab_common.h"

namespace lmkan {

namespace {

constexpr int kTile = LMKAN_PACK_TILE;  // 64 outputs per workgroup tile
constexpr int kRowBytes = kTile * 4;    // one table row of a float32 slab in LDS

template <typename T>
struct is_bf16 {
    static constexpr bool value = false;
};
template <>
struct is_bf16<bf16_t> {
    static constexpr bool value = true;
};

// ---------------------------------------------------------------------------
// Preamble pass (Alg. 1 "Preamble"): records[field][pair][sample]
//   field 0: node = i1 (G+1) + i2 (int32), field 1: u, field 2: v  with
//   u = (x1 - node[i1]) / h1, v likewise; the four B-spline products are
//   (1-u)(1-v), u(1-v), (1-u)v, uv.
// A 64 x 32 (sample x pair) tile is read along the rows of x, transposed
// through LDS and written along the sample axis.
// ---------------------------------------------------------------------------
constexpr int kRecTile = 64;   // samples per tile
constexpr int kRecPairs = 32;  // pairs per tile: 25 KB of LDS, six workgroups per CU

template <bool CONV>
__global__ __launch_bounds__(256) void preamble_records_kernel(GridTab tab, const float *__restrict__ x,
                                                              int32_t *__restrict__ rec_node,
                                                              float *__restrict__ rec_u,
                                                              float *__restrict__ rec_v, int64_t B,
                                                              int n_in, ConvGeom cg)
{
    __shared__ float s_node[LMKAN_MAX_GRID + 1];
    __shared__ float s_invh[LMKAN_MAX_GRID];
    __shared__ int s_n[kRecPairs][kRecTile + 1];
    __shared__ float s_u[kRecPairs][kRecTile + 1];
    __shared__ float s_v[kRecPairs][kRecTile + 1];
    for (int i = threadIdx.x; i <= tab.G; i += blockDim.x) s_node[i] = tab.node[i];
    for (int i = threadIdx.x; i < tab.G; i += blockDim.x) s_invh[i] = tab.inv_h[i];

    const int K = n_in / 2;
    const int64_t n0 = (int64_t)blockIdx.x * kRecTile;
    const int k0 = blockIdx.y * kRecPairs;
    const int p = threadIdx.x % kRecPairs;  // pair within tile (fast axis of the read)
    const int r0 = threadIdx.x / kRecPairs;
    constexpr int kRowStep = 256 / kRecPairs, kPerThread = kRecTile / kRowStep;
    // convolution: offset of a row's window once per tile, offsets of this thread's two inputs
    // inside a window once per thread
    __shared__ int64_t s_base[CONV ? kRecTile : 1];
    int64_t e_off0 = 0, e_off1 = 0;
    if constexpr (CONV) {
        if (threadIdx.x < kRecTile && n0 + threadIdx.x < B) s_base[threadIdx.x] = conv_input_offset(cg, n0 + threadIdx.x, 0);
        if (k0 + p < K) {
            e_off0 = conv_input_offset(cg, 0, 2 * (k0 + p));
            e_off1 = conv_input_offset(cg, 0, 2 * (k0 + p) + 1);
        }
    }
    __syncthreads();
    // all loads of the thread first: the pass is bound by how many bytes are in flight
    const bool pair_ok = k0 + p < K;
    float2 xv[kPerThread];
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        const int r = r0 + kRowStep * i;
        const int64_t n = n0 + r;
        xv[i] = make_float2(0.f, 0.f);
        if (n < B && pair_ok) {
            if constexpr (CONV)
                xv[i] = make_float2(x[s_base[r] + e_off0], x[s_base[r] + e_off1]);
            else
                xv[i] = load_input_pair<false>(x, n, n_in, k0 + p, cg);
        }
    }
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        const int r = r0 + kRowStep * i;
        int node = 0;
        float u = 0.f, v = 0.f;
        if (n0 + r < B && pair_ok) {
            const Preamble pr = preamble(s_node, s_invh, tab.G, xv[i].x, xv[i].y);
            node = pr.node;
            u = pr.a_hi;
            v = pr.b_hi;
        }
        s_n[p][r] = node;
        s_u[p][r] = u;
        s_v[p][r] = v;
    }
    __syncthreads();
    const int r = threadIdx.x & 63;  // sample within tile (fast axis of the write)
    const int q0 = threadIdx.x >> 6;
    const int64_t n = n0 + r;
    if (n < B) {
        for (int q = q0; q < kRecPairs; q += 4) {
            if (k0 + q < K) {
                const int64_t o = (int64_t)(k0 + q) * B + n;
                rec_node[o] = s_n[q][r];
                rec_u[o] = s_u[q][r];
                rec_v[o] = s_v[q][r];
            }
        }
    }
}

// Stream the slab of (pair k, output tile jt) into LDS.  A wave instruction moves
// 4 table rows (one per 16-lane group, 16 bytes per lane); the 1 KiB it writes is
// contiguous in LDS.  Chunks are dealt round-robin to the waves.
// LPS = lanes per table row: 16 for 64-output tiles, 4 for 16-output tiles (a 1 KiB chunk is
// then 16 rows).
template <int WAVES, int LPS = 16>
__device__ __forceinline__ void issue_slab_load(const SlabArgs &a, float *slab, int k, int jt, int wave,
                                                int lane)
{
    constexpr int NG = 64 / LPS;  // rows per chunk
    const int g = lane / LPS, l16 = lane % LPS;
    const unsigned base = __builtin_amdgcn_readfirstlane(lds_address(slab));
    if (LPS == 16 && a.packed) {
        // the slab is one contiguous run of nodes x 256 bytes: chunk c sits at byte c * 1024
        const char *src = reinterpret_cast<const char *>(static_cast<const float *>(a.P) + (int64_t)k * a.map.s_pair +
                                                         (int64_t)jt * a.map.s_tile);
        const int full = a.nodes >> 2;  // chunks made of four rows
        const unsigned lane_off = (unsigned)lane * 16u;
        for (int c = wave; c < full; c += WAVES)
            lds_dma16_uniform(src + (size_t)c * (4 * kRowBytes), lane_off, base + c * (4 * kRowBytes));
        const int rest = a.nodes & 3;  // rows of the last, partial chunk
        if (rest != 0 && full % WAVES == wave && g < rest)
            lds_dma16_uniform(src + (size_t)full * (4 * kRowBytes), lane_off, base + full * (4 * kRowBytes));
        return;
    }
    const int col = jt * (LPS * 4) + l16 * 4;
    const float *src = static_cast<const float *>(a.P) + (int64_t)k * a.map.s_pair +
                       (int64_t)(col >> 6) * a.map.s_tile + (col & 63);
    const int chunks = (a.nodes + NG - 1) / NG;
    const bool col_ok = col < a.col_limit;  // never read past a table row
    for (int c = wave; c < chunks; c += WAVES) {
        const int node = c * NG + g;
        if (node < a.nodes && col_ok)
            lds_dma16(src + (int64_t)node * a.map.s_node,
                      __builtin_amdgcn_readfirstlane(base + c * (4 * kRowBytes)));
    }
}

// Filling a slab from 16-bit storage: the values travel through registers, are widened to
// float32 and written with ds_write_b128, so the slab in LDS and everything that reads it
// are those of the float32 path while the table costs half the bytes in HBM and L2.
// issue() requests the wave's chunks (8 bytes per lane: the lane's four outputs of one
// row), commit() converts and stores them; between the two the wave computes on the other
// buffer.  For float32 storage issue() is the LDS-direct load above and commit() is empty.
constexpr int kMaxSlabBytes = 80 * 1024;  // one of the two slab buffers

// A slab that has LDS to itself (up to 160 KiB) is filled in four phases of the same size.
template <typename CT, int WAVES, int LPS = 16, int PHASES = 2>
struct SlabFill {
    static constexpr int NG = 64 / LPS;  // rows per 1 KiB chunk
    static constexpr int kChunksPerWave = (PHASES / 2 * kMaxSlabBytes / 1024 + WAVES - 1) / WAVES;
    static constexpr int kPerPhase = (kChunksPerWave + PHASES - 1) / PHASES;  // phases keep the staging registers few
    uint2 v[kPerPhase];
    bool col_exists = true;  // the lane's four columns are inside the table (set by issue)

    template <int PHASE>
    __device__ __forceinline__ void issue(const SlabArgs &a, float *, int k, int jt, int wave, int lane)
    {
        const int g = lane / LPS, l16 = lane % LPS;
        const int col = jt * (LPS * 4) + l16 * 4;
        const bool col_ok = col < a.col_limit;
        const int col_rd = col_ok ? col : 0;
        const CT *src = static_cast<const CT *>(a.P) + (int64_t)k * a.map.s_pair + (int64_t)(col_rd >> 6) * a.map.s_tile +
                        (col_rd & 63);
#pragma unroll
        for (int i = 0; i < kPerPhase; ++i) {
            // Never skipped: a row or column outside the table reads an entry inside it; commit()
            // drops such a row and writes zeros for such a column.  (The compiler sizes a wait for a load by the path with
            // the fewest younger loads; a load that may be skipped makes every older load's wait
            // a wait for everything.)
            const int node = (wave + (PHASE * kPerPhase + i) * WAVES) * NG + g;
            v[i] = *reinterpret_cast<const uint2 *>(src + (int64_t)min(node, a.nodes - 1) * a.map.s_node);
        }
        col_exists = col_ok;
    }
    template <int PHASE>
    __device__ __forceinline__ void commit(const SlabArgs &a, float *slab, int wave, int lane)
    {
        const int g = lane / LPS;
#pragma unroll
        for (int i = 0; i < kPerPhase; ++i) {
            const int c = wave + (PHASE * kPerPhase + i) * WAVES;
            if (c * NG + g < a.nodes) {
                float4 f;
                if constexpr (!is_bf16<CT>::value) {
                    typedef _Float16 h2v __attribute__((ext_vector_type(2)));
                    const h2v lo = __builtin_bit_cast(h2v, v[i].x), hi = __builtin_bit_cast(h2v, v[i].y);
                    f = make_float4((float)lo.x, (float)lo.y, (float)hi.x, (float)hi.y);
                } else {
                    f = make_float4(__uint_as_float(v[i].x << 16), __uint_as_float(v[i].x & 0xffff0000u),
                                    __uint_as_float(v[i].y << 16), __uint_as_float(v[i].y & 0xffff0000u));
                }
                if (!col_exists) f = make_float4(0.f, 0.f, 0.f, 0.f);
                *reinterpret_cast<float4 *>(slab + c * (4 * kTile) + lane * 4) = f;
            }
        }
    }
};

template <int WAVES, int LPS, int PHASES>
struct SlabFill<float, WAVES, LPS, PHASES> {
    template <int PHASE>
    __device__ __forceinline__ void issue(const SlabArgs &a, float *slab, int k, int jt, int wave, int lane)
    {
        if constexpr (PHASE == 0) issue_slab_load<WAVES, LPS>(a, slab, k, jt, wave, lane);
    }
    template <int PHASE>
    __device__ __forceinline__ void commit(const SlabArgs &, float *, int, int)
    {
    }
};

// The four table rows of one step: corners (i1,i2), (i1,i2+1), (i1+1,i2), (i1+1,i2+1).
struct Corners {
    float4 c00, c01, c10, c11;
};

// lane_base = LDS address of the slab + this lane's column bytes; the broadcast of the
// sample's row offset folds into the one integer add that forms the address.  W_CT is G + 1
// when it is known at compile time (the second row pair then sits at an immediate offset),
// 0 otherwise.
typedef float f4raw __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float4 lds_load4(unsigned addr)
{
    const f4raw v = *reinterpret_cast<__attribute__((address_space(3))) const f4raw *>(addr);
    return make_float4(v.x, v.y, v.z, v.w);
}

template <int S, int W_CT>
__device__ __forceinline__ void load_corners(Corners &c, int lane_base, int off_bytes, int W)
{
    const unsigned addr = (unsigned)(row_bcast<S>(off_bytes) + lane_base);
    const int w = W_CT > 0 ? W_CT : W;
    c.c00 = lds_load4(addr);
    c.c01 = lds_load4(addr + kRowBytes);
    c.c10 = lds_load4(addr + w * kRowBytes);
    c.c11 = lds_load4(addr + w * kRowBytes + kRowBytes);
}

template <int S>
__device__ __forceinline__ void fma_corners(float *acc, const Corners &c, float w00, float w10, float w01,
                                            float w11)
{
    fmac_row_bcast<S>(acc[0], w00, c.c00.x);
    fmac_row_bcast<S>(acc[1], w00, c.c00.y);
    fmac_row_bcast<S>(acc[2], w00, c.c00.z);
    fmac_row_bcast<S>(acc[3], w00, c.c00.w);
    fmac_row_bcast<S>(acc[0], w10, c.c10.x);
    fmac_row_bcast<S>(acc[1], w10, c.c10.y);
    fmac_row_bcast<S>(acc[2], w10, c.c10.z);
    fmac_row_bcast<S>(acc[3], w10, c.c10.w);
    fmac_row_bcast<S>(acc[0], w01, c.c01.x);
    fmac_row_bcast<S>(acc[1], w01, c.c01.y);
    fmac_row_bcast<S>(acc[2], w01, c.c01.z);
    fmac_row_bcast<S>(acc[3], w01, c.c01.w);
    fmac_row_bcast<S>(acc[0], w11, c.c11.x);
    fmac_row_bcast<S>(acc[1], w11, c.c11.y);
    fmac_row_bcast<S>(acc[2], w11, c.c11.z);
    fmac_row_bcast<S>(acc[3], w11, c.c11.w);
}

// Software pipeline over the SETS * 16 steps of one pair: the rows of step T + AHEAD are
// requested from LDS before the multiply-adds of step T are issued.

template <int T, int END, int TOTAL, int AHEAD, int W_CT>
__device__ __forceinline__ void slab_pipeline(float *acc, Corners (&ring)[AHEAD + 1], int lane_base,
                                              const int *off, const float *w00, const float *w10,
                                              const float *w01, const float *w11, int W)
{
    if constexpr (T < END) {
        if constexpr (T + AHEAD < TOTAL)
            load_corners<(T + AHEAD) % 16, W_CT>(ring[(T + AHEAD) % (AHEAD + 1)], lane_base, off[(T + AHEAD) / 16], W);
        fma_corners<T % 16>(acc + 4 * T, ring[T % (AHEAD + 1)], w00[T / 16], w10[T / 16], w01[T / 16],
                            w11[T / 16]);
        slab_pipeline<T + 1, END, TOTAL, AHEAD, W_CT>(acc, ring, lane_base, off, w00, w10, w01, w11, W);
    }
}

// WAVES waves per workgroup, SETS x 64 samples per wave.
// Two waves per SIMD by construction (one workgroup per CU); telling the compiler lets
// it spend registers on keeping several LDS reads in flight.
// WAVES / 4 waves per SIMD by construction (one workgroup per CU); telling the compiler lets
// it spend exactly that share of the registers.  The multiply-add rate of a SIMD grows with
// the number of waves it can pick from (measured: DPP multiply-adds 49 per clock and CU with
// two waves per SIMD, 60 with four), hence 16 waves of 64 samples rather than 8 of 128 when
// the registers allow.
template <typename CT, int WAVES, int SETS, int AHEAD, int W_CT>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(WAVES / 4, WAVES / 4))) void forward_slab_kernel(
    SlabArgs a)
{
    extern __shared__ __align__(16) float smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform by construction
    const int l16 = lane & 15, g = lane >> 4;
    constexpr int kTileB = WAVES * SETS * 64;

    // Workgroup -> (output tile, pair split, sample tile).  Consecutive ids go round-robin
    // over the 8 XCDs, each with its own L2; workgroups that stream the same slabs
    // (same output tile and pair range, different sample tile) are placed on one XCD.
    int id = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int btile = id % a.n_btiles;
    const int rest = id / a.n_btiles;
    const int ks = rest % a.n_split;
    const int jt = rest / a.n_split;

    const int k_begin = ks * a.pairs_per_split;
    const int k_end = min(a.K, k_begin + a.pairs_per_split);
    const int slab_floats = a.nodes * kTile;
    float *slab0 = smem;
    float *slab1 = smem + slab_floats;

    const int64_t n_wave = (int64_t)btile * kTileB + (int64_t)wave * (SETS * 64);

    float acc[SETS * 64];
#pragma unroll
    for (int i = 0; i < SETS * 64; ++i) acc[i] = 0.0f;

    // record of (sample n_wave + set*64 + lane, pair k), fetched one pair ahead
    int nx_node[SETS];
    float nx_u[SETS], nx_v[SETS];
    auto fetch_records = [&](int k) {
#pragma unroll
        for (int s = 0; s < SETS; ++s) {
            const int64_t n = n_wave + s * 64 + lane;
            nx_node[s] = 0;
            nx_u[s] = 0.f;
            nx_v[s] = 0.f;
            if (n < a.B) {
                const int64_t o = (int64_t)k * a.B + n;
                nx_node[s] = a.rec_node[o];
                nx_u[s] = a.rec_u[o];
                nx_v[s] = a.rec_v[o];
            }
        }
    };

    SlabFill<CT, WAVES> fill;
    if (k_begin < k_end) {
        fill.template issue<0>(a, slab0, k_begin, jt, wave, lane);
        fill.template commit<0>(a, slab0, wave, lane);
        fill.template issue<1>(a, slab0, k_begin, jt, wave, lane);
        fill.template commit<1>(a, slab0, wave, lane);
        fetch_records(k_begin);
    }
    const int lane_bytes = l16 * 16;
    for (int k = k_begin; k < k_end; ++k) {
        const float *slab = ((k - k_begin) & 1) ? slab1 : slab0;
        float *slab_next = ((k - k_begin) & 1) ? slab0 : slab1;

        int off[SETS];
        float w00[SETS], w10[SETS], w01[SETS], w11[SETS];
#pragma unroll
        for (int s = 0; s < SETS; ++s) {
            const float u = nx_u[s], v = nx_v[s];
            const float a_lo = 1.0f - u, b_lo = 1.0f - v;
            off[s] = nx_node[s] * kRowBytes;
            w00[s] = a_lo * b_lo;
            w10[s] = u * b_lo;
            w01[s] = a_lo * v;
            w11[s] = u * v;
        }
        // this wave's slab loads for pair k have landed; after the barrier everybody's have,
        // and everybody has finished reading the other buffer (pair k-1)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (k + 1 < k_end) {
            fill.template issue<0>(a, slab_next, k + 1, jt, wave, lane);
            fetch_records(k + 1);
        }
#pragma unroll
        for (int s = 0; s < SETS; ++s) {
            // VALU results must not be read through DPP in the next two issue slots
            asm volatile("s_nop 1" : "+v"(w00[s]), "+v"(w10[s]), "+v"(w01[s]), "+v"(w11[s]));
        }
        Corners ring[AHEAD + 1];
        const int lane_base = (int)lds_address(slab) + lane_bytes;
        load_corners<0, W_CT>(ring[0], lane_base, off[0], a.W);
        if constexpr (AHEAD > 1) load_corners<1, W_CT>(ring[1], lane_base, off[0], a.W);
        // the steps of the pair in two halves; a 16-bit table is staged half a slab at a time
        constexpr int kHalf = SETS * 8;
        slab_pipeline<0, kHalf, SETS * 16, AHEAD, W_CT>(acc, ring, lane_base, off, w00, w10, w01, w11, a.W);
        if (k + 1 < k_end) {
            fill.template commit<0>(a, slab_next, wave, lane);
            fill.template issue<1>(a, slab_next, k + 1, jt, wave, lane);
        }
        slab_pipeline<kHalf, SETS * 16, SETS * 16, AHEAD, W_CT>(acc, ring, lane_base, off, w00, w10, w01, w11, a.W);
        if (k + 1 < k_end) fill.template commit<1>(a, slab_next, wave, lane);
    }

    // lane (g, l16) holds outputs jt*64 + 4*l16 .. +3 of samples n_wave + set*64 + 16*g + step
    const int col = jt * kTile + l16 * 4;
    bool atomic;
    float *ybase = forward_out_base(a, ks, atomic);
    if (col < a.n_out) {
#pragma unroll
        for (int s = 0; s < SETS; ++s) {
#pragma unroll
            for (int st = 0; st < 16; ++st) {
                const int64_t n = n_wave + s * 64 + g * 16 + st;
                if (n < a.B) store_outputs(ybase + n * a.n_out + col, acc + s * 64 + st * 4, a.n_out, col, atomic);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Input gradient with the same slab streaming.
//   s_ab(n,k) = sum_j gy[n][j] P[corner ab][k][j]
//   d/dx1 = (1/h1) ((s10 - s00)(1 - v) + (s11 - s01) v),  d/dx2 = (1/h2) ((s01 - s00)(1 - u) + (s11 - s10) u)
// The roles of the forward kernel are mirrored: gy[sample][4 outputs] stays in registers, a
// step forms the four partial dot products of its lane, combines them with the weights of
// the owning lane (DPP row broadcast) and sums over the 16 lanes that share the sample with
// DPP row operations.  The two derivatives travel together through the reduction: lanes
// 0-7 of a row end up with d/dx1, lanes 8-15 with d/dx2.  Results of eight steps are
// collected across the lanes and added into grad_x with one atomic instruction (the
// output tiles of a sample are spread over several workgroups).
// ---------------------------------------------------------------------------
// out[B][n_in] = in[n_in][B]
__global__ __launch_bounds__(256) void transpose_kernel(const float *__restrict__ in, float *__restrict__ out,
                                                       int64_t B, int n_in, int64_t ld, int layout)
{
    __shared__ float tile[64][65];
    const int64_t n0 = (int64_t)blockIdx.x * 64;
    const int c0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int64_t src = scratch_position(n0 + tx, layout);
    for (int r = ty; r < 64; r += 4)
        if (c0 + r < n_in && n0 + tx < B) tile[r][tx] = in[(int64_t)(c0 + r) * ld + src];
    __syncthreads();
    for (int r = ty; r < 64; r += 4)
        if (n0 + r < B && c0 + tx < n_in) out[(n0 + r) * n_in + c0 + tx] = tile[tx][r];
}


// d = (w of lane S of this row) * x
template <int S>
__device__ __forceinline__ float mul_row_bcast(float w, float x)
{
    float d;
    asm("v_mul_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf" : "=v"(d) : "v"(w), "v"(x), "n"(S));
    return d;
}

struct GradRecord {
    int off;
    float b_lo, b_hi;  // (1 - v) / h1, v / h1
    float a_lo, a_hi;  // (1 - u) / h2, u / h2
};

// The sum over the 16 lanes of a row (the 64 outputs of the tile) is taken for the two
// derivatives of eight steps together, halving the number of live values at every stage
// instead of summing every value over all lanes: a lane (bits b3 b2 b1 b0 of its position in
// the row) ends up with the derivative b3 (d/dx1 or d/dx2) of step 4 b0 + 2 b1 + b2 of the
// eight.  15 instructions per eight steps and derivative pair instead of 32.
//
// The stages are grad_fold_halves / _steps / _pairs in lmkan_slab_common.h.
template <int S>
__device__ __forceinline__ float grad_step(const float4 g, const Corners &c, const GradRecord &r)
{
    const float s00 = fmaf(g.w, c.c00.w, fmaf(g.z, c.c00.z, fmaf(g.y, c.c00.y, g.x * c.c00.x)));
    const float s10 = fmaf(g.w, c.c10.w, fmaf(g.z, c.c10.z, fmaf(g.y, c.c10.y, g.x * c.c10.x)));
    const float s01 = fmaf(g.w, c.c01.w, fmaf(g.z, c.c01.z, fmaf(g.y, c.c01.y, g.x * c.c01.x)));
    const float s11 = fmaf(g.w, c.c11.w, fmaf(g.z, c.c11.z, fmaf(g.y, c.c11.y, g.x * c.c11.x)));
    float t1 = mul_row_bcast<S>(r.b_lo, s10 - s00);
    fmac_row_bcast<S>(t1, r.b_hi, s11 - s01);
    float t2 = mul_row_bcast<S>(r.a_lo, s01 - s00);
    fmac_row_bcast<S>(t2, r.a_hi, s11 - s10);
    return grad_fold_halves(t1, t2);
}

template <typename CT, int WAVES, int SETS, int AHEAD, int W_CT>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(WAVES / 4, WAVES / 4))) void backward_input_slab_kernel(
    GradInArgs a)
{
    extern __shared__ __align__(16) float smem[];  // two slab buffers, then 1/h of the grid
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    constexpr int kTileB = WAVES * SETS * 64;
    constexpr int TOTAL = SETS * 16;
    int id = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int btile = id % a.n_btiles;
    const int rest = id / a.n_btiles;
    const int ks = rest % a.n_split;
    const int jt = rest / a.n_split;

    const int k_begin = ks * a.pairs_per_split;
    const int k_end = min(a.K, k_begin + a.pairs_per_split);
    const int slab_floats = a.nodes * kTile;
    float *slab0 = smem;
    float *slab1 = smem + slab_floats;
    float *s_invh = smem + 2 * slab_floats;
    for (int i = threadIdx.x; i < a.tab.G; i += blockDim.x) s_invh[i] = a.tab.inv_h[i];
    SlabArgs sa;  // only the fields issue_slab_load reads
    sa.P = a.P;
    sa.map = a.map;
    sa.nodes = a.nodes;
    sa.col_limit = a.col_limit;
    sa.packed = a.packed;

    const int64_t n_wave = (int64_t)btile * kTileB + (int64_t)wave * (SETS * 64);
    const int col = jt * kTile + l16 * 4;
    // the step of a block of eight whose result this lane ends up with (see grad_step)
    const int my_step = ((l16 & 1) << 2) | (l16 & 2) | ((l16 >> 2) & 1);

    // gy of (sample n_wave + set*64 + 16 g + step, outputs col .. col+3), resident for the walk
    float4 gyr[TOTAL];
#pragma unroll
    for (int t = 0; t < TOTAL; ++t) {
        const int64_t n = n_wave + (t / 16) * 64 + g * 16 + (t % 16);
        gyr[t] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (n < a.B && col < a.n_out)
            gyr[t] = *reinterpret_cast<const float4 *>(a.gy + (col >> 6) * a.gy_tile_stride + n * a.gy_row_stride + (col & 63));
    }

    int nx_node[SETS];
    float nx_u[SETS], nx_v[SETS];
    auto fetch_records = [&](int k) {
#pragma unroll
        for (int s = 0; s < SETS; ++s) {
            const int64_t n = n_wave + s * 64 + lane;
            nx_node[s] = 0;
            nx_u[s] = 0.f;
            nx_v[s] = 0.f;
            if (n < a.B) {
                const int64_t o = (int64_t)k * a.B + n;
                nx_node[s] = a.rec_node[o];
                nx_u[s] = a.rec_u[o];
                nx_v[s] = a.rec_v[o];
            }
        }
    };

    // columns past the end of a ragged output tile are never loaded: make them read as zero
    for (int i = threadIdx.x; i < 2 * slab_floats; i += blockDim.x) smem[i] = 0.0f;
    __syncthreads();  // zeros and s_invh in place before any slab load lands
    SlabFill<CT, WAVES> fill;
    if (k_begin < k_end) {
        fill.template issue<0>(sa, slab0, k_begin, jt, wave, lane);
        fill.template commit<0>(sa, slab0, wave, lane);
        fill.template issue<1>(sa, slab0, k_begin, jt, wave, lane);
        fill.template commit<1>(sa, slab0, wave, lane);
        fetch_records(k_begin);
    }
    const int lane_bytes = l16 * 16;
    // where this lane's collected results go: sample 16 g + my_step of each block of 8 steps,
    // input 2k (lanes 0-7) or 2k+1 (lanes 8-15).  The scratch gradient is stored transposed,
    // [n_in][ld], in the kScratchOct layout: the first block of 8 steps lands at 8 g + step,
    // the second 32 further, so an atomic instruction covers 128 contiguous bytes of each row.
    const int64_t n_lane = n_wave + g * 16 + my_step;
    float *gx_lane = a.gx + (int64_t)(l16 >> 3) * a.ld + n_wave + g * 8 + my_step;

    for (int k = k_begin; k < k_end; ++k) {
        const float *slab = ((k - k_begin) & 1) ? slab1 : slab0;
        float *slab_next = ((k - k_begin) & 1) ? slab0 : slab1;

        GradRecord rec[SETS];
#pragma unroll
        for (int s = 0; s < SETS; ++s) {
            const int node = nx_node[s];
            const float rh1 = s_invh[node / a.W], rh2 = s_invh[node % a.W];
            rec[s].off = node * kRowBytes;
            rec[s].b_lo = (1.0f - nx_v[s]) * rh1;
            rec[s].b_hi = nx_v[s] * rh1;
            rec[s].a_lo = (1.0f - nx_u[s]) * rh2;
            rec[s].a_hi = nx_u[s] * rh2;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (k + 1 < k_end) {
            fill.template issue<0>(sa, slab_next, k + 1, jt, wave, lane);
            fetch_records(k + 1);
        }
#pragma unroll
        for (int s = 0; s < SETS; ++s)
            asm volatile("s_nop 1" : "+v"(rec[s].b_lo), "+v"(rec[s].b_hi), "+v"(rec[s].a_lo), "+v"(rec[s].a_hi));

        Corners ring[AHEAD + 1];
        const int lane_base = (int)lds_address(slab) + lane_bytes;
        load_corners<0, W_CT>(ring[0], lane_base, rec[0].off, a.W);
        if constexpr (AHEAD > 1) load_corners<1, W_CT>(ring[1], lane_base, rec[0].off, a.W);
        float v_even = 0.0f, w_first = 0.0f, z_first = 0.0f;  // results waiting for their partners
        static_for(std::make_integer_sequence<int, TOTAL>{}, [&](auto tc) {
            constexpr int T = decltype(tc)::value;
            if constexpr (T + AHEAD < TOTAL)
                load_corners<(T + AHEAD) % 16, W_CT>(ring[(T + AHEAD) % (AHEAD + 1)], lane_base,
                                                     rec[(T + AHEAD) / 16].off, a.W);
            if constexpr (T == TOTAL / 2) {
                if (k + 1 < k_end) {
                    fill.template commit<0>(sa, slab_next, wave, lane);
                    fill.template issue<1>(sa, slab_next, k + 1, jt, wave, lane);
                }
            }
            const float v = grad_step<T % 16>(gyr[T], ring[T % (AHEAD + 1)], rec[T / 16]);
            if constexpr ((T & 1) == 0) {
                v_even = v;
            } else {
                const float w = grad_fold_steps(v_even, v);
                if constexpr ((T & 3) == 1) {
                    w_first = w;
                } else {
                    const float z = grad_fold_pairs(w_first, w, (l16 & 2) != 0);
                    if constexpr ((T & 7) == 3) {
                        z_first = z;
                    } else {
                        const float mine = (l16 & 1) ? z : z_first;
                        const int64_t n = n_lane + (T / 16) * 64 + ((T % 16) & ~7);
                        if (n < a.B)
                            unsafeAtomicAdd(gx_lane + (int64_t)(2 * k) * a.ld + ((T / 16) * 64 + ((T % 16) >> 3) * 32), mine);
                    }
                }
            }
        });
        if (k + 1 < k_end) fill.template commit<1>(sa, slab_next, wave, lane);
    }
}

// ---------------------------------------------------------------------------
// Input gradient with a lane per sample (float32 tables, 64-output tiles).  The lane keeps the 64
// gy values of its sample and tile in registers and reads the four corner rows of its own cell,
// 16 bytes at a time; the four dot products stay inside the lane, so nothing is exchanged between
// lanes and every multiply-add is a plain one.  All lanes reading piece j of their rows at once
// would meet on the same four banks; lane l reads piece (j + l) mod 16 instead and holds its gy
// pieces in that rotated order (a dot product does not care about the order of its terms): the 16
// lanes of every group of 16 are on 16 different bank groups whatever their rows, which is the
// best a 1 KiB read can do.  Instantiated for float32 tables only: with a 16-bit table the
// registers that stage its rows on their way to LDS push the kernel 16 registers over what four
// waves per SIMD leave it (it then spills in the main loop); those tables keep the kernel above.
// ---------------------------------------------------------------------------
template <typename CT, int W_CT>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(4, 4))) void backward_input_lane_kernel(GradInArgs a)
{
    extern __shared__ __align__(16) float smem[];  // two slab buffers, then 1/h of the grid
    constexpr int WAVES = 16;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l15 = lane & 15;
    int id = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int btile = id % a.n_btiles;
    const int rest = id / a.n_btiles;
    const int ks = rest % a.n_split;
    const int jt = rest / a.n_split;

    const int k_begin = ks * a.pairs_per_split;
    const int k_end = min(a.K, k_begin + a.pairs_per_split);
    const int slab_floats = a.nodes * kTile;
    float *slab0 = smem;
    float *slab1 = smem + slab_floats;
    float *s_invh = smem + 2 * slab_floats;
    for (int i = threadIdx.x; i < a.tab.G; i += blockDim.x) s_invh[i] = a.tab.inv_h[i];
    SlabArgs sa;  // only the fields issue_slab_load reads
    sa.P = a.P;
    sa.map = a.map;
    sa.nodes = a.nodes;
    sa.col_limit = a.col_limit;
    sa.packed = a.packed;

    const int64_t n = (int64_t)btile * (WAVES * 64) + wave * 64 + lane;
    const bool valid = n < a.B;
    const int64_t n_rd = valid ? n : a.B - 1;

    // register j: gy of outputs jt*64 + 4 p .. + 3 with p = (j + l15) mod 16
    float4 gyr[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const int col = jt * kTile + ((j + l15) & 15) * 4;
        gyr[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (valid && col < a.n_out)
            gyr[j] = *reinterpret_cast<const float4 *>(a.gy + (col >> 6) * a.gy_tile_stride + n * a.gy_row_stride + (col & 63));
    }

    // columns past the end of a ragged output tile are never loaded: make them read as zero
    for (int i = threadIdx.x; i < 2 * slab_floats; i += blockDim.x) smem[i] = 0.0f;
    __syncthreads();  // zeros and s_invh in place before any slab load lands
    SlabFill<CT, WAVES> fill;
    int nx_node = 0;
    float nx_u = 0.f, nx_v = 0.f;
    auto fetch_record = [&](int k) {
        const int64_t o = (int64_t)k * a.B + n_rd;
        nx_node = a.rec_node[o];
        nx_u = a.rec_u[o];
        nx_v = a.rec_v[o];
    };
    if (k_begin < k_end) {
        fill.template issue<0>(sa, slab0, k_begin, jt, wave, lane);
        fill.template commit<0>(sa, slab0, wave, lane);
        fill.template issue<1>(sa, slab0, k_begin, jt, wave, lane);
        fill.template commit<1>(sa, slab0, wave, lane);
        fetch_record(k_begin);
    }
    const int w = W_CT > 0 ? W_CT : a.W;
    float *gx_lane = a.gx + n;   // transposed scratch [n_in][ld], plain layout
    for (int k = k_begin; k < k_end; ++k) {
        const float *slab = ((k - k_begin) & 1) ? slab1 : slab0;
        float *slab_next = ((k - k_begin) & 1) ? slab0 : slab1;
        const int node = nx_node;
        const float u = nx_u, v = nx_v;
        const int i1 = node / w;
        const float rh1 = s_invh[i1], rh2 = s_invh[node - i1 * w];
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (k + 1 < k_end) {
            fill.template issue<0>(sa, slab_next, k + 1, jt, wave, lane);
            fetch_record(k + 1);
        }
        // piece (j + l15) mod 16 of the row: from `first` for j < 16 - l15, one row back after the wrap
        unsigned first = lds_address(slab) + (unsigned)node * kRowBytes + (unsigned)l15 * 16;
        // The derivative is made of differences between neighbouring corners, and on a smooth table
        // two dot products over all 64 outputs would agree in most of their digits before they are
        // subtracted.  So the four products are summed over the four outputs of a piece only and
        // their differences taken at once: dif_a = sum gy (P10 - P00), dif_b = sum gy (P11 - P01),
        // dif_c = sum gy (P01 - P00), dif_d = sum gy (P11 - P10).  (dif_d = dif_b + dif_c - dif_a
        // would save a register and four instructions per piece, but far outside the grid, where the
        // local coordinates are large, it costs accuracy: one more pair of roundings multiplied by u.)
        float dif_a = 0.f, dif_b = 0.f, dif_c = 0.f, dif_d = 0.f;
        // the rows of piece j + 1 are requested before the multiply-adds of piece j are issued
        Corners ring[2];
        auto request = [&](Corners &c, int j) {
            // (the empty statement ties the addresses to the sums so far, so that the compiler keeps
            // that order: left to itself it issues all 64 reads of a pair first and spills them, or
            // walks one corner at a time with a single read in flight)
            asm volatile("" : "+v"(first), "+v"(dif_a), "+v"(dif_b), "+v"(dif_c), "+v"(dif_d));
            const unsigned addr = (l15 + j >= 16 ? first - kRowBytes : first) + j * 16;
            c.c00 = lds_load4(addr);
            c.c01 = lds_load4(addr + kRowBytes);
            c.c10 = lds_load4(addr + w * kRowBytes);
            c.c11 = lds_load4(addr + w * kRowBytes + kRowBytes);
        };
        request(ring[0], 0);
        static_for(std::make_integer_sequence<int, 16>{}, [&](auto jc) {
            constexpr int j = decltype(jc)::value;
            if constexpr (j + 1 < 16) request(ring[(j + 1) & 1], j + 1);
            const Corners &c = ring[j & 1];
            const float4 g = gyr[j];
            float p00 = g.x * c.c00.x, p01 = g.x * c.c01.x, p10 = g.x * c.c10.x, p11 = g.x * c.c11.x;
            p00 = fmaf(g.y, c.c00.y, p00);
            p01 = fmaf(g.y, c.c01.y, p01);
            p10 = fmaf(g.y, c.c10.y, p10);
            p11 = fmaf(g.y, c.c11.y, p11);
            p00 = fmaf(g.z, c.c00.z, p00);
            p01 = fmaf(g.z, c.c01.z, p01);
            p10 = fmaf(g.z, c.c10.z, p10);
            p11 = fmaf(g.z, c.c11.z, p11);
            p00 = fmaf(g.w, c.c00.w, p00);
            p01 = fmaf(g.w, c.c01.w, p01);
            p10 = fmaf(g.w, c.c10.w, p10);
            p11 = fmaf(g.w, c.c11.w, p11);
            dif_a += p10 - p00;
            dif_b += p11 - p01;
            dif_c += p01 - p00;
            dif_d += p11 - p10;
            if constexpr (j == 7) {
                if (k + 1 < k_end) {
                    fill.template commit<0>(sa, slab_next, wave, lane);
                    fill.template issue<1>(sa, slab_next, k + 1, jt, wave, lane);
                }
            }
        });
        if (k + 1 < k_end) fill.template commit<1>(sa, slab_next, wave, lane);
        const float d1 = rh1 * (dif_a * (1.0f - v) + dif_b * v);
        const float d2 = rh2 * (dif_c * (1.0f - u) + dif_d * u);
        if (valid) {
            unsafeAtomicAdd(gx_lane + (int64_t)(2 * k) * a.ld, d1);
            unsafeAtomicAdd(gx_lane + (int64_t)(2 * k + 1) * a.ld, d2);
        }
    }
}

// ---------------------------------------------------------------------------
// Input gradient for 16-bit packed tables on grids too fine for 64-output slabs (17 <= G <= 34):
// 32-output tiles whose slab stays in LDS as it is stored (64 bytes per row, LDS-direct fill, two
// buffers), a lane per sample as in backward_input_lane_kernel, two samples per lane (2048 per
// workgroup, so that a slab serves twice as many).  A row is four pieces of eight outputs; lane l
// reads piece (j + l) mod 4 at step j and holds its gy in that order.  The stored values are
// widened in registers (a shift or a mask for bfloat16), the differences of neighbouring corners
// are taken per piece.
// ---------------------------------------------------------------------------
constexpr int kHalfTile = 32;
constexpr int kHalfRowBytes = kHalfTile * 2;

template <typename CT>
__device__ __forceinline__ void widen8(const uint4 raw, float (&f)[8])
{
    const unsigned d[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if constexpr (is_bf16<CT>::value) {
            f[2 * i] = __uint_as_float(d[i] << 16);
            f[2 * i + 1] = __uint_as_float(d[i] & 0xffff0000u);
        } else {
            typedef _Float16 h2v __attribute__((ext_vector_type(2)));
            const h2v h = __builtin_bit_cast(h2v, d[i]);
            f[2 * i] = (float)h.x;
            f[2 * i + 1] = (float)h.y;
        }
    }
}

typedef unsigned u4raw __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint4 lds_load_u4(unsigned addr)
{
    const u4raw v = *reinterpret_cast<__attribute__((address_space(3))) const u4raw *>(addr);
    return make_uint4(v.x, v.y, v.z, v.w);
}

struct CornersRaw {
    uint4 c00, c01, c10, c11;
};

// Forward on the same tiles: the 32 outputs of a sample's tile in registers (two samples per lane),
// the lane's own four weights, outputs kept and stored in the rotated order of the pieces.
template <typename CT>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(4, 4))) void forward_lane32_kernel(SlabArgs a)
{
    extern __shared__ __align__(16) char smem32[];  // two slab buffers
    constexpr int WAVES = 16, SETS = 2;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l3 = lane & 3;
    int id = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int btile = id % a.n_btiles;
    const int rest = id / a.n_btiles;
    const int ks = rest % a.n_split;
    const int jt = rest / a.n_split;   // 32-output tile

    const int k_begin = ks * a.pairs_per_split;
    const int k_end = min(a.K, k_begin + a.pairs_per_split);
    const unsigned slab_bytes = (unsigned)a.nodes * kHalfRowBytes;
    const unsigned base0 = __builtin_amdgcn_readfirstlane(lds_address(smem32));
    const unsigned base1 = base0 + slab_bytes;

    // packed table: the rows of (pair, 64-output tile jt / 2) lie 128 bytes apart, this tile is
    // their half jt & 1; a wave instruction moves 16 rows (four lanes x 16 bytes each)
    const CT *half = static_cast<const CT *>(a.P) + (int64_t)(jt >> 1) * a.map.s_tile + (jt & 1) * kHalfTile + (lane & 3) * 8;
    const int chunks = (a.nodes + 15) >> 4;
    auto issue_fill = [&](unsigned lds_base, int k) {
        const CT *src = half + (int64_t)k * a.map.s_pair;
        for (int c = wave; c < chunks; c += WAVES) {
            const int node = c * 16 + (lane >> 2);
            if (node < a.nodes) lds_dma16(src + (int64_t)node * a.map.s_node, __builtin_amdgcn_readfirstlane(lds_base + c * 1024));
        }
    };

    const int64_t n0 = (int64_t)btile * (WAVES * SETS * 64) + wave * (SETS * 64) + lane;
    // register block j of a sample: outputs jt*32 + 8 p .. + 7 with p = (j + l3) mod 4
    float acc[SETS][4][8];
#pragma unroll
    for (int s = 0; s < SETS; ++s)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[s][j][i] = 0.0f;

    // (a sample past the end of the batch reads the records of the last one; the records of a pair
    // start at a wave-uniform address, the sample is a 32-bit index into them)
    unsigned n_rec[SETS];
#pragma unroll
    for (int s = 0; s < SETS; ++s) n_rec[s] = (unsigned)min(n0 + s * 64, a.B - 1);
    int nx_node[SETS];
    float nx_u[SETS], nx_v[SETS];
    auto fetch_records = [&](int k) {
        const int32_t *r_node = a.rec_node + (int64_t)k * a.B;
        const float *r_u = a.rec_u + (int64_t)k * a.B, *r_v = a.rec_v + (int64_t)k * a.B;
#pragma unroll
        for (int s = 0; s < SETS; ++s) {
            nx_node[s] = r_node[n_rec[s]];
            nx_u[s] = r_u[n_rec[s]];
            nx_v[s] = r_v[n_rec[s]];
        }
    };
    if (k_begin < k_end) {
        issue_fill(base0, k_begin);
        fetch_records(k_begin);
    }

    for (int k = k_begin; k < k_end; ++k) {
        const unsigned cur = ((k - k_begin) & 1) ? base1 : base0;
        const unsigned nxt = ((k - k_begin) & 1) ? base0 : base1;
        unsigned first[SETS];
        float w00[SETS], w10[SETS], w01[SETS], w11[SETS];
#pragma unroll
        for (int s = 0; s < SETS; ++s) {
            const float u = nx_u[s], v = nx_v[s];
            const float a_lo = 1.0f - u, b_lo = 1.0f - v;
            w00[s] = a_lo * b_lo, w10[s] = u * b_lo, w01[s] = a_lo * v, w11[s] = u * v;
            // piece (j + l3) mod 4 of the row: from `first` for j < 4 - l3, one row back after the wrap
            first[s] = cur + (unsigned)nx_node[s] * kHalfRowBytes + (unsigned)l3 * 16;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (k + 1 < k_end) {
            issue_fill(nxt, k + 1);
            fetch_records(k + 1);
        }
        CornersRaw ring[2];
        auto request = [&](CornersRaw &c, int t, float &tie) {
            // (the empty statement ties the addresses to a sum of the piece before last: it keeps the
            // reads of a piece between the multiply-adds of the pieces before it)
            const int s = t >> 2, j = t & 3;
            asm volatile("" : "+v"(first[s]), "+v"(tie));
            const unsigned addr = (l3 + j >= 4 ? first[s] - kHalfRowBytes : first[s]) + j * 16;
            c.c00 = lds_load_u4(addr);
            c.c01 = lds_load_u4(addr + kHalfRowBytes);
            c.c10 = lds_load_u4(addr + a.W * kHalfRowBytes);
            c.c11 = lds_load_u4(addr + a.W * kHalfRowBytes + kHalfRowBytes);
        };
        request(ring[0], 0, acc[SETS - 1][3][7]);
        static_for(std::make_integer_sequence<int, SETS * 4>{}, [&](auto tc) {
            constexpr int t = decltype(tc)::value;
            constexpr int s = t >> 2, j = t & 3;
            constexpr int tp = t > 0 ? t - 1 : SETS * 4 - 1;   // the piece before this one
            if constexpr (t + 1 < SETS * 4) request(ring[(t + 1) & 1], t + 1, acc[tp >> 2][tp & 3][7]);
            const CornersRaw &c = ring[t & 1];
            float f[8];
            widen8<CT>(c.c00, f);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[s][j][i] = fmaf(w00[s], f[i], acc[s][j][i]);
            widen8<CT>(c.c10, f);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[s][j][i] = fmaf(w10[s], f[i], acc[s][j][i]);
            widen8<CT>(c.c01, f);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[s][j][i] = fmaf(w01[s], f[i], acc[s][j][i]);
            widen8<CT>(c.c11, f);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[s][j][i] = fmaf(w11[s], f[i], acc[s][j][i]);
        });
    }

    bool atomic;
    float *ybase = forward_out_base(a, ks, atomic);
#pragma unroll
    for (int s = 0; s < SETS; ++s) {
        const int64_t n = n0 + s * 64;
        if (n < a.B) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = jt * kHalfTile + ((j + l3) & 3) * 8;
                if (col < a.n_out) store_outputs(ybase + n * a.n_out + col, acc[s][j], a.n_out, col, atomic);
                if (col + 4 < a.n_out) store_outputs(ybase + n * a.n_out + col + 4, acc[s][j] + 4, a.n_out, col + 4, atomic);
            }
        }
    }
}

template <typename CT>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(4, 4))) void backward_input_lane32_kernel(GradInArgs a)
{
    extern __shared__ __align__(16) char smem32[];  // two slab buffers, then 1/h of the grid
    constexpr int WAVES = 16, SETS = 2;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l3 = lane & 3;
    int id = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int btile = id % a.n_btiles;
    const int rest = id / a.n_btiles;
    const int ks = rest % a.n_split;
    const int jt = rest / a.n_split;   // 32-output tile

    const int k_begin = ks * a.pairs_per_split;
    const int k_end = min(a.K, k_begin + a.pairs_per_split);
    const unsigned slab_bytes = (unsigned)a.nodes * kHalfRowBytes;
    const unsigned base0 = __builtin_amdgcn_readfirstlane(lds_address(smem32));
    const unsigned base1 = base0 + slab_bytes;
    float *s_invh = reinterpret_cast<float *>(smem32 + ((2 * slab_bytes + 15) & ~15u));
    for (int i = threadIdx.x; i < a.tab.G; i += blockDim.x) s_invh[i] = a.tab.inv_h[i];

    // packed table: the rows of (pair, 64-output tile jt / 2) lie 128 bytes apart, this tile is
    // their half jt & 1; a wave instruction moves 16 rows (four lanes x 16 bytes each)
    const CT *half = static_cast<const CT *>(a.P) + (int64_t)(jt >> 1) * a.map.s_tile + (jt & 1) * kHalfTile + (lane & 3) * 8;
    const int chunks = (a.nodes + 15) >> 4;
    auto issue_fill = [&](unsigned lds_base, int k) {
        const CT *src = half + (int64_t)k * a.map.s_pair;
        for (int c = wave; c < chunks; c += WAVES) {
            const int node = c * 16 + (lane >> 2);
            if (node < a.nodes) lds_dma16(src + (int64_t)node * a.map.s_node, __builtin_amdgcn_readfirstlane(lds_base + c * 1024));
        }
    };

    const int64_t n0 = (int64_t)btile * (WAVES * SETS * 64) + wave * (SETS * 64) + lane;
    // register block j of a sample: gy of outputs jt*32 + 8 p .. + 7 with p = (j + l3) mod 4
    float gyr[SETS][4][8];
#pragma unroll
    for (int s = 0; s < SETS; ++s) {
        const int64_t n = n0 + s * 64;
        const bool valid_s = n < a.B;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = jt * kHalfTile + ((j + l3) & 3) * 8;
            const float *src = a.gy + (col >> 6) * a.gy_tile_stride + n * a.gy_row_stride + (col & 63);
            float4 lo = make_float4(0.f, 0.f, 0.f, 0.f), hi = lo;
            if (valid_s && col < a.n_out) lo = *reinterpret_cast<const float4 *>(src);
            if (valid_s && col + 4 < a.n_out) hi = *reinterpret_cast<const float4 *>(src + 4);
            gyr[s][j][0] = lo.x, gyr[s][j][1] = lo.y, gyr[s][j][2] = lo.z, gyr[s][j][3] = lo.w;
            gyr[s][j][4] = hi.x, gyr[s][j][5] = hi.y, gyr[s][j][6] = hi.z, gyr[s][j][7] = hi.w;
        }
    }

    int nx_node[SETS];
    float nx_u[SETS], nx_v[SETS];
    // (a sample past the end of the batch reads the records of the last one; the records of a pair
    // start at a wave-uniform address, the sample is a 32-bit index into them)
    unsigned n_rec[SETS];
#pragma unroll
    for (int s = 0; s < SETS; ++s) n_rec[s] = (unsigned)min(n0 + s * 64, a.B - 1);
    auto fetch_records = [&](int k) {
        const int32_t *r_node = a.rec_node + (int64_t)k * a.B;
        const float *r_u = a.rec_u + (int64_t)k * a.B, *r_v = a.rec_v + (int64_t)k * a.B;
#pragma unroll
        for (int s = 0; s < SETS; ++s) {
            nx_node[s] = r_node[n_rec[s]];
            nx_u[s] = r_u[n_rec[s]];
            nx_v[s] = r_v[n_rec[s]];
        }
    };
    __syncthreads();  // s_invh in place
    if (k_begin < k_end) {
        issue_fill(base0, k_begin);
        fetch_records(k_begin);
    }

    for (int k = k_begin; k < k_end; ++k) {
        const unsigned cur = ((k - k_begin) & 1) ? base1 : base0;
        const unsigned nxt = ((k - k_begin) & 1) ? base0 : base1;
        int node[SETS];
        float u[SETS], v[SETS];
#pragma unroll
        for (int s = 0; s < SETS; ++s) node[s] = nx_node[s], u[s] = nx_u[s], v[s] = nx_v[s];
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (k + 1 < k_end) {
            issue_fill(nxt, k + 1);
            fetch_records(k + 1);
        }
        // piece (j + l3) mod 4 of the row: from `first` for j < 4 - l3, one row back after the wrap
        unsigned first[SETS];
#pragma unroll
        for (int s = 0; s < SETS; ++s) first[s] = cur + (unsigned)node[s] * kHalfRowBytes + (unsigned)l3 * 16;
        float dif_a = 0.f, dif_b = 0.f, dif_c = 0.f, dif_d = 0.f;   // as in backward_input_lane_kernel
        CornersRaw ring[2];
        auto request = [&](CornersRaw &c, int t) {
            // (the empty statement ties the addresses to the sums so far: it keeps the reads of a
            // piece between the multiply-adds of the pieces before it)
            const int s = t >> 2, j = t & 3;
            asm volatile("" : "+v"(first[s]), "+v"(dif_a), "+v"(dif_b), "+v"(dif_c), "+v"(dif_d));
            const unsigned addr = (l3 + j >= 4 ? first[s] - kHalfRowBytes : first[s]) + j * 16;
            c.c00 = lds_load_u4(addr);
            c.c01 = lds_load_u4(addr + kHalfRowBytes);
            c.c10 = lds_load_u4(addr + a.W * kHalfRowBytes);
            c.c11 = lds_load_u4(addr + a.W * kHalfRowBytes + kHalfRowBytes);
        };
        request(ring[0], 0);
        static_for(std::make_integer_sequence<int, SETS * 4>{}, [&](auto tc) {
            constexpr int t = decltype(tc)::value;
            constexpr int s = t >> 2, j = t & 3;
            if constexpr (t + 1 < SETS * 4) request(ring[(t + 1) & 1], t + 1);
            const CornersRaw &c = ring[t & 1];
            float f[8];
            float p00 = 0.f, p01 = 0.f, p10 = 0.f, p11 = 0.f;
            widen8<CT>(c.c00, f);
#pragma unroll
            for (int i = 0; i < 8; ++i) p00 = fmaf(gyr[s][j][i], f[i], p00);
            widen8<CT>(c.c01, f);
#pragma unroll
            for (int i = 0; i < 8; ++i) p01 = fmaf(gyr[s][j][i], f[i], p01);
            widen8<CT>(c.c10, f);
#pragma unroll
            for (int i = 0; i < 8; ++i) p10 = fmaf(gyr[s][j][i], f[i], p10);
            widen8<CT>(c.c11, f);
#pragma unroll
            for (int i = 0; i < 8; ++i) p11 = fmaf(gyr[s][j][i], f[i], p11);
            dif_a += p10 - p00;
            dif_b += p11 - p01;
            dif_c += p01 - p00;
            dif_d += p11 - p10;
            if constexpr (j == 3) {
                const int i1 = node[s] / a.W;
                const float rh1 = s_invh[i1], rh2 = s_invh[node[s] - i1 * a.W];
                const float d1 = rh1 * (dif_a * (1.0f - v[s]) + dif_b * v[s]);
                const float d2 = rh2 * (dif_c * (1.0f - u[s]) + dif_d * u[s]);
                if (n0 + s * 64 < a.B) {
                    float *dst = a.gx + (int64_t)(2 * k) * a.ld + n0 + s * 64;
                    unsafeAtomicAdd(dst, d1);
                    unsafeAtomicAdd(dst + a.ld, d2);
                }
                dif_a = dif_b = dif_c = dif_d = 0.f;
            }
        });
    }
}

// ---------------------------------------------------------------------------
// The same pair of kernels for float32 packed tables where two 32-output slabs of 128-byte rows fit
// LDS (17 <= G <= 24): eight pieces of four outputs per row, read in the order (j + l) mod 8.
// (The code below is written over the row's constants and would serve the 16-bit tables too; they
// keep the kernels above, whose loops the compiler schedules about 8 % faster than this form.)
// ---------------------------------------------------------------------------
struct HalfRowF32 {
    static constexpr int kBytes = kHalfTile * 4;         // a row of the slab
    static constexpr int kPieces = kBytes / 16;          // 16-byte pieces per row
    static constexpr int kPer = 4;                       // outputs per piece
    static constexpr int kRowsPerFill = 64 / kPieces;    // rows one wave instruction moves
    static constexpr int kPieceShift = 3;                // log2 of the two above
    static constexpr int kFillShift = 3;
};

__device__ __forceinline__ void piece_as_floats(const uint4 raw, float (&f)[4])
{
    f[0] = __uint_as_float(raw.x), f[1] = __uint_as_float(raw.y), f[2] = __uint_as_float(raw.z),
    f[3] = __uint_as_float(raw.w);
}

__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(4, 4))) void backward_input_lane32_f32_kernel(GradInArgs a)
{
    extern __shared__ __align__(16) char smem32[];  // two slab buffers, then 1/h of the grid
    typedef HalfRowF32 Row;
    constexpr int WAVES = 16, SETS = 2, PIECES = Row::kPieces, PER = Row::kPer, STEPS = SETS * PIECES;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lp = lane & (PIECES - 1);
    int id = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int btile = id % a.n_btiles;
    const int rest = id / a.n_btiles;
    const int ks = rest % a.n_split;
    const int jt = rest / a.n_split;   // 32-output tile

    const int k_begin = ks * a.pairs_per_split;
    const int k_end = min(a.K, k_begin + a.pairs_per_split);
    const unsigned slab_bytes = (unsigned)a.nodes * Row::kBytes;
    const unsigned base0 = __builtin_amdgcn_readfirstlane(lds_address(smem32));
    const unsigned base1 = base0 + slab_bytes;
    float *s_invh = reinterpret_cast<float *>(smem32 + ((2 * slab_bytes + 15) & ~15u));
    for (int i = threadIdx.x; i < a.tab.G; i += blockDim.x) s_invh[i] = a.tab.inv_h[i];

    // packed table: the rows of (pair, 64-output tile jt / 2) lie 64 elements apart, this tile is
    // their half jt & 1; a wave instruction moves 1024 bytes (PIECES lanes x 16 bytes per row)
    const float *half = static_cast<const float *>(a.P) + (int64_t)(jt >> 1) * a.map.s_tile + (jt & 1) * kHalfTile + lp * PER;
    const int chunks = (a.nodes + Row::kRowsPerFill - 1) >> Row::kFillShift;
    auto issue_fill = [&](unsigned lds_base, int k) {
        const float *src = half + (int64_t)k * a.map.s_pair;
        for (int c = wave; c < chunks; c += WAVES) {
            const int node = c * Row::kRowsPerFill + (lane >> Row::kPieceShift);
            if (node < a.nodes) lds_dma16(src + (int64_t)node * a.map.s_node, __builtin_amdgcn_readfirstlane(lds_base + c * 1024));
        }
    };

    const int64_t n0 = (int64_t)btile * (WAVES * SETS * 64) + wave * (SETS * 64) + lane;
    // register block j of a sample: gy of outputs jt*32 + PER p .. + PER - 1 with p = (j + lp) mod PIECES
    float gyr[SETS][PIECES][PER];
#pragma unroll
    for (int s = 0; s < SETS; ++s) {
        const int64_t n = n0 + s * 64;
        const bool valid_s = n < a.B;
#pragma unroll
        for (int j = 0; j < PIECES; ++j) {
            const int col = jt * kHalfTile + ((j + lp) & (PIECES - 1)) * PER;
            const float *src = a.gy + (col >> 6) * a.gy_tile_stride + n * a.gy_row_stride + (col & 63);
            float4 g = make_float4(0.f, 0.f, 0.f, 0.f);
            if (valid_s && col < a.n_out) g = *reinterpret_cast<const float4 *>(src);
            gyr[s][j][0] = g.x, gyr[s][j][1] = g.y, gyr[s][j][2] = g.z, gyr[s][j][3] = g.w;
        }
    }

    int nx_node[SETS];
    float nx_u[SETS], nx_v[SETS];
    // (a sample past the end of the batch reads the records of the last one; the records of a pair
    // start at a wave-uniform address, the sample is a 32-bit index into them)
    unsigned n_rec[SETS];
#pragma unroll
    for (int s = 0; s < SETS; ++s) n_rec[s] = (unsigned)min(n0 + s * 64, a.B - 1);
    auto fetch_records = [&](int k) {
        const int32_t *r_node = a.rec_node + (int64_t)k * a.B;
        const float *r_u = a.rec_u + (int64_t)k * a.B, *r_v = a.rec_v + (int64_t)k * a.B;
#pragma unroll
        for (int s = 0; s < SETS; ++s) {
            nx_node[s] = r_node[n_rec[s]];
            nx_u[s] = r_u[n_rec[s]];
            nx_v[s] = r_v[n_rec[s]];
        }
    };
    __syncthreads();  // s_invh in place
    if (k_begin < k_end) {
        issue_fill(base0, k_begin);
        fetch_records(k_begin);
    }

    for (int k = k_begin; k < k_end; ++k) {
        const unsigned cur = ((k - k_begin) & 1) ? base1 : base0;
        const unsigned nxt = ((k - k_begin) & 1) ? base0 : base1;
        int node[SETS];
        float u[SETS], v[SETS];
#pragma unroll
        for (int s = 0; s < SETS; ++s) node[s] = nx_node[s], u[s] = nx_u[s], v[s] = nx_v[s];
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (k + 1 < k_end) {
            issue_fill(nxt, k + 1);
            fetch_records(k + 1);
        }
        // piece (j + lp) mod PIECES of the row: from `first` for j < PIECES - lp, one row back after
        // the wrap
        unsigned first[SETS];
#pragma unroll
        for (int s = 0; s < SETS; ++s) first[s] = cur + (unsigned)node[s] * Row::kBytes + (unsigned)lp * 16;
        float dif_a = 0.f, dif_b = 0.f, dif_c = 0.f, dif_d = 0.f;   // as in backward_input_lane_kernel
        CornersRaw ring[2];
        auto request = [&](CornersRaw &c, int t) {
            // (the empty statement ties the addresses to the sums so far: it keeps the reads of a
            // piece between the multiply-adds of the pieces before it)
            const int s = t / PIECES, j = t % PIECES;
            asm volatile("" : "+v"(first[s]), "+v"(dif_a), "+v"(dif_b), "+v"(dif_c), "+v"(dif_d));
            const unsigned addr = (lp + j >= PIECES ? first[s] - Row::kBytes : first[s]) + j * 16;
            c.c00 = lds_load_u4(addr);
            c.c01 = lds_load_u4(addr + Row::kBytes);
            c.c10 = lds_load_u4(addr + a.W * Row::kBytes);
            c.c11 = lds_load_u4(addr + a.W * Row::kBytes + Row::kBytes);
        };
        request(ring[0], 0);
        static_for(std::make_integer_sequence<int, STEPS>{}, [&](auto tc) {
            constexpr int t = decltype(tc)::value;
            constexpr int s = t / PIECES, j = t % PIECES;
            if constexpr (t + 1 < STEPS) request(ring[(t + 1) & 1], t + 1);
            const CornersRaw &c = ring[t & 1];
            float f[PER];
            float p00 = 0.f, p01 = 0.f, p10 = 0.f, p11 = 0.f;
            piece_as_floats(c.c00, f);
#pragma unroll
            for (int i = 0; i < PER; ++i) p00 = fmaf(gyr[s][j][i], f[i], p00);
            piece_as_floats(c.c01, f);
#pragma unroll
            for (int i = 0; i < PER; ++i) p01 = fmaf(gyr[s][j][i], f[i], p01);
            piece_as_floats(c.c10, f);
#pragma unroll
            for (int i = 0; i < PER; ++i) p10 = fmaf(gyr[s][j][i], f[i], p10);
            piece_as_floats(c.c11, f);
#pragma unroll
            for (int i = 0; i < PER; ++i) p11 = fmaf(gyr[s][j][i], f[i], p11);
            dif_a += p10 - p00;
            dif_b += p11 - p01;
            dif_c += p01 - p00;
            dif_d += p11 - p10;
            if constexpr (j == PIECES - 1) {
                const int i1 = node[s] / a.W;
                const float rh1 = s_invh[i1], rh2 = s_invh[node[s] - i1 * a.W];
                const float d1 = rh1 * (dif_a * (1.0f - v[s]) + dif_b * v[s]);
                const float d2 = rh2 * (dif_c * (1.0f - u[s]) + dif_d * u[s]);
                if (n0 + s * 64 < a.B) {
                    float *dst = a.gx + (int64_t)(2 * k) * a.ld + n0 + s * 64;
                    unsafeAtomicAdd(dst, d1);
                    unsafeAtomicAdd(dst + a.ld, d2);
                }
                dif_a = dif_b = dif_c = dif_d = 0.f;
            }
        });
    }
}

// Forward on the same tiles: the 32 outputs of a sample's tile in registers, stored in the rotated
// order of the pieces.  Rows of 128 bytes alternate between the two halves of the LDS banks, and
// lanes l and l + 8 of a 16-lane group read the same piece of their rows.  Lanes 0-7 therefore
// start with whichever of their cell's rows r, r + 1 lies in the lower half and lanes 8-15 with
// the one in the upper half (rows r + W, r + W + 1 follow suit: they flip both or neither), and the
// four weights go to the rows as the lane reads them: no two lanes of a group meet on a bank.
// (The input gradient above does not do this: it is bound by its vector instructions, and the two
// extra address additions per piece cost it more than the conflicts do.)
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(4, 4))) void forward_lane32_f32_kernel(SlabArgs a)
{
    extern __shared__ __align__(16) char smem32[];  // two slab buffers
    typedef HalfRowF32 Row;
    constexpr int WAVES = 16, SETS = 2, PIECES = Row::kPieces, PER = Row::kPer, STEPS = SETS * PIECES;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lp = lane & (PIECES - 1);
    int id = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int btile = id % a.n_btiles;
    const int rest = id / a.n_btiles;
    const int ks = rest % a.n_split;
    const int jt = rest / a.n_split;   // 32-output tile

    const int k_begin = ks * a.pairs_per_split;
    const int k_end = min(a.K, k_begin + a.pairs_per_split);
    const unsigned slab_bytes = (unsigned)a.nodes * Row::kBytes;
    const unsigned base0 = __builtin_amdgcn_readfirstlane(lds_address(smem32));
    const unsigned base1 = base0 + slab_bytes;

    // packed table: the rows of (pair, 64-output tile jt / 2) lie 64 elements apart, this tile is
    // their half jt & 1; a wave instruction moves 1024 bytes (PIECES lanes x 16 bytes per row)
    const float *half = static_cast<const float *>(a.P) + (int64_t)(jt >> 1) * a.map.s_tile + (jt & 1) * kHalfTile + lp * PER;
    const int chunks = (a.nodes + Row::kRowsPerFill - 1) >> Row::kFillShift;
    auto issue_fill = [&](unsigned lds_base, int k) {
        const float *src = half + (int64_t)k * a.map.s_pair;
        for (int c = wave; c < chunks; c += WAVES) {
            const int node = c * Row::kRowsPerFill + (lane >> Row::kPieceShift);
            if (node < a.nodes) lds_dma16(src + (int64_t)node * a.map.s_node, __builtin_amdgcn_readfirstlane(lds_base + c * 1024));
        }
    };

    const int64_t n0 = (int64_t)btile * (WAVES * SETS * 64) + wave * (SETS * 64) + lane;
    // register block j of a sample: outputs jt*32 + PER p .. + PER - 1 with p = (j + lp) mod PIECES
    float acc[SETS][PIECES][PER];
#pragma unroll
    for (int s = 0; s < SETS; ++s)
#pragma unroll
        for (int j = 0; j < PIECES; ++j)
#pragma unroll
            for (int i = 0; i < PER; ++i) acc[s][j][i] = 0.0f;

    // (a sample past the end of the batch reads the records of the last one; the records of a pair
    // start at a wave-uniform address, the sample is a 32-bit index into them)
    unsigned n_rec[SETS];
#pragma unroll
    for (int s = 0; s < SETS; ++s) n_rec[s] = (unsigned)min(n0 + s * 64, a.B - 1);
    int nx_node[SETS];
    float nx_u[SETS], nx_v[SETS];
    auto fetch_records = [&](int k) {
        const int32_t *r_node = a.rec_node + (int64_t)k * a.B;
        const float *r_u = a.rec_u + (int64_t)k * a.B, *r_v = a.rec_v + (int64_t)k * a.B;
#pragma unroll
        for (int s = 0; s < SETS; ++s) {
            nx_node[s] = r_node[n_rec[s]];
            nx_u[s] = r_u[n_rec[s]];
            nx_v[s] = r_v[n_rec[s]];
        }
    };
    if (k_begin < k_end) {
        issue_fill(base0, k_begin);
        fetch_records(k_begin);
    }

    for (int k = k_begin; k < k_end; ++k) {
        const unsigned cur = ((k - k_begin) & 1) ? base1 : base0;
        const unsigned nxt = ((k - k_begin) & 1) ? base0 : base1;
        // rows as the lane reads them (A, B = r, r + 1, or swapped where that keeps lanes l and
        // l + 8 on different halves of the banks; C, D = A, B + W rows) and their weights
        unsigned first[SETS];
        int to_other[SETS];
        float w_a[SETS], w_b[SETS], w_c[SETS], w_d[SETS];
#pragma unroll
        for (int s = 0; s < SETS; ++s) {
            const float u = nx_u[s], v = nx_v[s];
            const float a_lo = 1.0f - u, b_lo = 1.0f - v;
            const float w00 = a_lo * b_lo, w10 = u * b_lo, w01 = a_lo * v, w11 = u * v;
            const unsigned sw = ((unsigned)nx_node[s] ^ (unsigned)(lane >> 3)) & 1u;
            w_a[s] = sw ? w01 : w00, w_b[s] = sw ? w00 : w01;
            w_c[s] = sw ? w11 : w10, w_d[s] = sw ? w10 : w11;
            // piece (j + lp) mod PIECES of the row: from `first` for j < PIECES - lp, one row back
            // after the wrap
            first[s] = cur + ((unsigned)nx_node[s] + sw) * Row::kBytes + (unsigned)lp * 16;
            to_other[s] = sw ? -Row::kBytes : Row::kBytes;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (k + 1 < k_end) {
            issue_fill(nxt, k + 1);
            fetch_records(k + 1);
        }
        CornersRaw ring[2];
        auto request = [&](CornersRaw &c, int t, float &tie) {
            // (the empty statement ties the addresses to a sum of the piece before last: it keeps the
            // reads of a piece between the multiply-adds of the pieces before it)
            const int s = t / PIECES, j = t % PIECES;
            asm volatile("" : "+v"(first[s]), "+v"(tie));
            const unsigned addr = (lp + j >= PIECES ? first[s] - Row::kBytes : first[s]) + j * 16;
            const unsigned other = addr + to_other[s];
            c.c00 = lds_load_u4(addr);
            c.c01 = lds_load_u4(other);
            c.c10 = lds_load_u4(addr + a.W * Row::kBytes);
            c.c11 = lds_load_u4(other + a.W * Row::kBytes);
        };
        request(ring[0], 0, acc[SETS - 1][PIECES - 1][PER - 1]);
        static_for(std::make_integer_sequence<int, STEPS>{}, [&](auto tc) {
            constexpr int t = decltype(tc)::value;
            constexpr int s = t / PIECES, j = t % PIECES;
            constexpr int tp = t > 0 ? t - 1 : STEPS - 1;   // the piece before this one
            if constexpr (t + 1 < STEPS) request(ring[(t + 1) & 1], t + 1, acc[tp / PIECES][tp % PIECES][PER - 1]);
            const CornersRaw &c = ring[t & 1];
            float f[PER];
            piece_as_floats(c.c00, f);
#pragma unroll
            for (int i = 0; i < PER; ++i) acc[s][j][i] = fmaf(w_a[s], f[i], acc[s][j][i]);
            piece_as_floats(c.c10, f);
#pragma unroll
            for (int i = 0; i < PER; ++i) acc[s][j][i] = fmaf(w_c[s], f[i], acc[s][j][i]);
            piece_as_floats(c.c01, f);
#pragma unroll
            for (int i = 0; i < PER; ++i) acc[s][j][i] = fmaf(w_b[s], f[i], acc[s][j][i]);
            piece_as_floats(c.c11, f);
#pragma unroll
            for (int i = 0; i < PER; ++i) acc[s][j][i] = fmaf(w_d[s], f[i], acc[s][j][i]);
        });
    }

    bool atomic;
    float *ybase = forward_out_base(a, ks, atomic);
#pragma unroll
    for (int s = 0; s < SETS; ++s) {
        const int64_t n = n0 + s * 64;
        if (n < a.B) {
#pragma unroll
            for (int j = 0; j < PIECES; ++j) {
                const int col = jt * kHalfTile + ((j + lp) & (PIECES - 1)) * PER;
                if (col < a.n_out) store_outputs(ybase + n * a.n_out + col, acc[s][j], a.n_out, col, atomic);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Forward for grids whose 64-output slab does not fit LDS twice (17 <= G <= 34): the same
// streaming with 16-output tiles.  A table row is then 64 bytes, read by four lanes, so a wave
// takes 16 samples per step and the sample's weights reach its four lanes through the DPP
// quad broadcast.  A wave owns SETS x 64 samples (512 with SETS = 8: a whole batch of 4096
// per workgroup, so that for such batches every slab is fetched exactly once); the records of
// a set are fetched three sets ahead into a ring of four.
// ---------------------------------------------------------------------------
template <int T>
__device__ __forceinline__ int quad_bcast(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, T * 0x55, 0xf, 0xf, true);
}

// acc += (w of lane T of this quad) * c
template <int T>
__device__ __forceinline__ void fmac_quad_bcast(float &acc, float w, float c)
{
    asm("v_fmac_f32_dpp %0, %1, %2 quad_perm:[%3,%3,%3,%3] row_mask:0xf bank_mask:0xf"
        : "+v"(acc)
        : "v"(w), "v"(c), "n"(T));
}

constexpr int kNarrowTile = 16;               // outputs per workgroup tile
constexpr int kNarrowRowBytes = kNarrowTile * 4;

template <int T>
__device__ __forceinline__ void load_corners_quad(Corners &c, const float *slab, int off_bytes, int lane_bytes, int W)
{
    const float *rowp =
        reinterpret_cast<const float *>(reinterpret_cast<const char *>(slab) + quad_bcast<T>(off_bytes) + lane_bytes);
    c.c00 = *reinterpret_cast<const float4 *>(rowp);
    c.c01 = *reinterpret_cast<const float4 *>(rowp + kNarrowTile);
    c.c10 = *reinterpret_cast<const float4 *>(rowp + W * kNarrowTile);
    c.c11 = *reinterpret_cast<const float4 *>(rowp + W * kNarrowTile + kNarrowTile);
}

template <int T>
__device__ __forceinline__ void fma_corners_quad(float *acc, const Corners &c, float w00, float w10, float w01,
                                                 float w11)
{
    fmac_quad_bcast<T>(acc[0], w00, c.c00.x);
    fmac_quad_bcast<T>(acc[1], w00, c.c00.y);
    fmac_quad_bcast<T>(acc[2], w00, c.c00.z);
    fmac_quad_bcast<T>(acc[3], w00, c.c00.w);
    fmac_quad_bcast<T>(acc[0], w10, c.c10.x);
    fmac_quad_bcast<T>(acc[1], w10, c.c10.y);
    fmac_quad_bcast<T>(acc[2], w10, c.c10.z);
    fmac_quad_bcast<T>(acc[3], w10, c.c10.w);
    fmac_quad_bcast<T>(acc[0], w01, c.c01.x);
    fmac_quad_bcast<T>(acc[1], w01, c.c01.y);
    fmac_quad_bcast<T>(acc[2], w01, c.c01.z);
    fmac_quad_bcast<T>(acc[3], w01, c.c01.w);
    fmac_quad_bcast<T>(acc[0], w11, c.c11.x);
    fmac_quad_bcast<T>(acc[1], w11, c.c11.y);
    fmac_quad_bcast<T>(acc[2], w11, c.c11.z);
    fmac_quad_bcast<T>(acc[3], w11, c.c11.w);
}

// SINGLE: the slab fits LDS only once (35 <= G <= 48): no slab is fetched while another is
// walked; the wave waits for its part of the fill and for the others' at the top of every pair.
template <typename CT, int WAVES, int SETS, bool SINGLE = false>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(WAVES / 4, WAVES / 4))) void forward_slab_narrow_kernel(
    SlabArgs a)
{
    extern __shared__ __align__(16) float smem[];
    constexpr int LPS = 4;             // lanes per sample
    constexpr int STEPS = SETS * LPS;  // steps per pair, 16 samples each
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int sub = lane & 3, grp = lane >> 2;
    constexpr int kTileB = WAVES * SETS * 64;

    int id = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int btile = id % a.n_btiles;
    const int rest = id / a.n_btiles;
    const int ks = rest % a.n_split;
    const int jt = rest / a.n_split;

    const int k_begin = ks * a.pairs_per_split;
    const int k_end = min(a.K, k_begin + a.pairs_per_split);
    const int slab_floats = a.nodes * kNarrowTile;
    float *slab0 = smem;
    float *slab1 = SINGLE ? smem : smem + slab_floats;
    const int64_t n_wave = (int64_t)btile * kTileB + (int64_t)wave * (SETS * 64);

    float acc[SETS * 16];
#pragma unroll
    for (int i = 0; i < SETS * 16; ++i) acc[i] = 0.0f;

    // Record ring, one slot per set: slot s holds (node, u, v) of sample n_wave + s * 64 + lane.
    // A slot is refilled for the next pair as soon as its set has started, a whole pair before
    // it is needed again.  Vector loads return in order, so a wait for a record also waits for
    // every older load: the order of issue below keeps the slab loads (long latency, straight
    // from HBM) younger than any record that is waited for before they are due.
    int r_node[SETS];
    float r_u[SETS], r_v[SETS];
    // No load of the main loop is ever skipped (the compiler sizes the wait for a load by the
    // path with the fewest younger loads, so a load that may be skipped turns the waits for all
    // older ones into waits for everything): a sample past the batch reads the last sample's
    // record (its results are not stored), the step past the last pair reads the last pair again.
    auto fetch_record = [&](int slot, int k) {
        const int64_t n = min(n_wave + slot * 64 + lane, a.B - 1);
        const int64_t o = (int64_t)min(k, k_end - 1) * a.B + n;
        r_node[slot] = a.rec_node[o];
        r_u[slot] = a.rec_u[o];
        r_v[slot] = a.rec_v[o];
    };

    SlabFill<CT, WAVES, LPS, SINGLE ? 4 : 2> fill;
    auto fill_whole = [&](int k) {  // every phase, one after the other
        static_for(std::make_integer_sequence<int, SINGLE ? 4 : 2>{}, [&](auto pc) {
            fill.template issue<decltype(pc)::value>(a, slab0, k, jt, wave, lane);
            fill.template commit<decltype(pc)::value>(a, slab0, wave, lane);
        });
    };
    if (k_begin < k_end) {
#pragma unroll
        for (int s = 0; s < SETS; ++s) fetch_record(s, k_begin);
        fill_whole(k_begin);
    }
    const int lane_bytes = sub * 16;
    for (int k = k_begin; k < k_end; ++k) {
        const float *slab = ((k - k_begin) & 1) ? slab1 : slab0;
        float *slab_next = ((k - k_begin) & 1) ? slab0 : slab1;
        if constexpr (SINGLE) {
            if (k > k_begin) {
                __syncthreads();  // nobody reads the slab of pair k - 1 any more
                fill_whole(k);
            }
        }
        // a float32 table arrives by LDS-direct loads, which nothing but this wait tracks
        if constexpr (sizeof(CT) == 4) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();  // the slab of pair k is complete, nobody reads the other buffer any more
        // (16-bit tables: the last pair fetches its own slab once more, for nobody; the LDS-direct
        // loads of a float32 table are not tracked by the compiler's waits and are simply left out)
        const int k_next = min(k + 1, k_end - 1);
        if constexpr (!SINGLE)
            if (sizeof(CT) != 4 || k + 1 < k_end) fill.template issue<0>(a, slab_next, k_next, jt, wave, lane);

        constexpr int kNear = 1;  // LDS reads run one step ahead (registers are short here)
        Corners ring[kNear + 1];
        int off_cur = r_node[0] * kNarrowRowBytes, off_nxt = 0;
        float w00 = 0.f, w10 = 0.f, w01 = 0.f, w11 = 0.f;
        load_corners_quad<0>(ring[0], slab, off_cur, lane_bytes, a.W);
        static_for(std::make_integer_sequence<int, STEPS>{}, [&](auto fc) {
            constexpr int F = decltype(fc)::value;
            constexpr int set = F / LPS, t = F % LPS;
            if constexpr (t == 0) {
                if constexpr (set == SETS / 2 && !SINGLE) {
                    fill.template commit<0>(a, slab_next, wave, lane);
                    fill.template issue<1>(a, slab_next, k_next, jt, wave, lane);
                }
                // weights of this set, offsets of the next one; then the slot is free
                const float u = r_u[set], v = r_v[set];
                const float a_lo = 1.0f - u, b_lo = 1.0f - v;
                w00 = a_lo * b_lo;
                w10 = u * b_lo;
                w01 = a_lo * v;
                w11 = u * v;
                if constexpr (set > 0) off_cur = off_nxt;
                if constexpr (set + 1 < SETS) off_nxt = r_node[set + 1] * kNarrowRowBytes;
                // VALU results must not be read through DPP in the next two issue slots
                asm volatile("s_nop 1" : "+v"(w00), "+v"(w10), "+v"(w01), "+v"(w11), "+v"(off_cur), "+v"(off_nxt));
                fetch_record(set, k + 1);
            }
            if constexpr (F + kNear < STEPS) {
                constexpr int F2 = F + kNear;
                load_corners_quad<F2 % LPS>(ring[F2 % (kNear + 1)], slab, (F2 / LPS == set) ? off_cur : off_nxt,
                                            lane_bytes, a.W);
            }
            fma_corners_quad<t>(acc + 4 * F, ring[F % (kNear + 1)], w00, w10, w01, w11);
        });
        if constexpr (!SINGLE) fill.template commit<1>(a, slab_next, wave, lane);
    }

    // lane (grp, sub) holds outputs jt*16 + 4*sub .. +3 of samples n_wave + set*64 + 4*grp + t
    const int col = jt * kNarrowTile + sub * 4;
    bool atomic;
    float *ybase = forward_out_base(a, ks, atomic);
    if (col < a.n_out) {
#pragma unroll
        for (int F = 0; F < STEPS; ++F) {
            const int64_t n = n_wave + (F / LPS) * 64 + grp * LPS + (F % LPS);
            if (n < a.B) store_outputs(ybase + n * a.n_out + col, acc + 4 * F, a.n_out, col, atomic);
        }
    }
}

// ---------------------------------------------------------------------------
// Input gradient with 16-output slabs (the mirror of forward_slab_narrow_kernel): gy of the
// wave's SETS x 64 samples stays in registers, a step forms the four partial dot products of
// 16 samples, applies each sample's weights by the DPP quad broadcast and sums over the four
// lanes of the sample with two quad permutations.  Lanes 0-1 of a quad end up with d/dx1,
// lanes 2-3 with d/dx2; over the four steps of a set every lane keeps two results, which
// leave with two atomic instructions per set into the transposed scratch.
// ---------------------------------------------------------------------------
template <int T>
__device__ __forceinline__ float mul_quad_bcast(float w, float x)
{
    float d;
    asm("v_mul_f32_dpp %0, %1, %2 quad_perm:[%3,%3,%3,%3] row_mask:0xf bank_mask:0xf"
        : "=v"(d)
        : "v"(w), "v"(x), "n"(T));
    return d;
}

template <int T>
__device__ __forceinline__ float grad_step_quad(const float4 g, const Corners &c, float b_lo, float b_hi, float a_lo,
                                                float a_hi, bool upper)
{
    const float s00 = fmaf(g.w, c.c00.w, fmaf(g.z, c.c00.z, fmaf(g.y, c.c00.y, g.x * c.c00.x)));
    const float s10 = fmaf(g.w, c.c10.w, fmaf(g.z, c.c10.z, fmaf(g.y, c.c10.y, g.x * c.c10.x)));
    const float s01 = fmaf(g.w, c.c01.w, fmaf(g.z, c.c01.z, fmaf(g.y, c.c01.y, g.x * c.c01.x)));
    const float s11 = fmaf(g.w, c.c11.w, fmaf(g.z, c.c11.z, fmaf(g.y, c.c11.y, g.x * c.c11.x)));
    float t1 = mul_quad_bcast<T>(b_lo, s10 - s00);
    fmac_quad_bcast<T>(t1, b_hi, s11 - s01);
    float t2 = mul_quad_bcast<T>(a_lo, s01 - s00);
    fmac_quad_bcast<T>(t2, a_hi, s11 - s10);
    const float keep = upper ? t2 : t1;
    const float send = upper ? t1 : t2;
    float v = keep + dpp_move<0x4E>(send);  // quad_perm [2,3,0,1]
    v += dpp_move<0xB1>(v);                 // quad_perm [1,0,3,2]
    return v;
}

template <typename CT, int WAVES, int SETS>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(WAVES / 4, WAVES / 4))) void backward_input_slab_narrow_kernel(
    GradInArgs a)
{
    extern __shared__ __align__(16) float smem[];  // two slab buffers, then 1/h of the grid
    constexpr int LPS = 4;
    constexpr int STEPS = SETS * LPS;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int sub = lane & 3, grp = lane >> 2;
    constexpr int kTileB = WAVES * SETS * 64;
    int id = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int btile = id % a.n_btiles;
    const int rest = id / a.n_btiles;
    const int ks = rest % a.n_split;
    const int jt = rest / a.n_split;

    const int k_begin = ks * a.pairs_per_split;
    const int k_end = min(a.K, k_begin + a.pairs_per_split);
    const int slab_floats = a.nodes * kNarrowTile;
    float *slab0 = smem;
    float *slab1 = smem + slab_floats;
    float *s_invh = smem + 2 * slab_floats;
    for (int i = threadIdx.x; i < a.tab.G; i += blockDim.x) s_invh[i] = a.tab.inv_h[i];
    SlabArgs sa;  // only the fields the slab fill reads
    sa.P = a.P;
    sa.map = a.map;
    sa.nodes = a.nodes;
    sa.col_limit = a.col_limit;
    sa.packed = a.packed;

    const int64_t n_wave = (int64_t)btile * kTileB + (int64_t)wave * (SETS * 64);
    const int col = jt * kNarrowTile + sub * 4;
    const bool upper = (sub & 2) != 0;
    const float inv_w = 1.0f / (float)a.W;

    // gy of (sample n_wave + set*64 + 4 grp + t, outputs col .. col+3), resident for the walk
    float4 gyr[STEPS];
#pragma unroll
    for (int F = 0; F < STEPS; ++F) {
        const int64_t n = n_wave + (F / LPS) * 64 + grp * LPS + (F % LPS);
        gyr[F] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (n < a.B && col < a.n_out)
            gyr[F] = *reinterpret_cast<const float4 *>(a.gy + (col >> 6) * a.gy_tile_stride + n * a.gy_row_stride + (col & 63));
    }

    int r_node[SETS];
    float r_u[SETS], r_v[SETS];
    // (never skipped, like every load of the main loop: see forward_slab_narrow_kernel; a sample
    // past the batch has gy = 0 and adds nothing)
    auto fetch_record = [&](int slot, int k) {
        const int64_t n = min(n_wave + slot * 64 + lane, a.B - 1);
        const int64_t o = (int64_t)k * a.B + n;
        r_node[slot] = a.rec_node[o];
        r_u[slot] = a.rec_u[o];
        r_v[slot] = a.rec_v[o];
    };

    // columns past the end of a ragged output tile are never loaded: the staged fill writes
    // zeros there, the LDS-direct loads of a float32 table leave them as they are, so they are
    // cleared first; s_invh must be in place before the first set
    if constexpr (sizeof(CT) == 4) {
        for (int i = threadIdx.x; i < 2 * slab_floats; i += blockDim.x) smem[i] = 0.0f;
        __syncthreads();
    }
    // Workgroups that differ only in their output tile add into the same entries of the
    // gradient.  Each starts its walk over the pairs at a different one, so that at any moment
    // they are on different pairs and their atomics go to different cache lines.
    const int n_k = k_end - k_begin;
    const int rot = n_k > 0 ? (int)(((int64_t)jt * n_k) / a.n_jt) : 0;
    auto pair_at = [&](int i) {  // pair of step i of the walk; past its end the last pair once more, for nobody
        const int r = min(i, n_k - 1) + rot;
        return k_begin + (r >= n_k ? r - n_k : r);
    };
    SlabFill<CT, WAVES, LPS> fill;
    if (n_k > 0) {
        const int k0 = pair_at(0);
#pragma unroll
        for (int s = 0; s < SETS; ++s) fetch_record(s, k0);
        fill.template issue<0>(sa, slab0, k0, jt, wave, lane);
        fill.template commit<0>(sa, slab0, wave, lane);
        fill.template issue<1>(sa, slab0, k0, jt, wave, lane);
        fill.template commit<1>(sa, slab0, wave, lane);
    }
    const int lane_bytes = sub * 16;
    // where this lane's two results of a set go: samples 4 grp + (sub & 1) and + 2 more, input
    // 2k (lanes 0-1 of the quad) or 2k + 1 (lanes 2-3)
    // (kScratchQuad layout of the scratch rows: the first two land at 2 grp + (sub & 1), the others 32 further)
    const int64_t n_lane = n_wave + grp * LPS + (sub & 1);
    float *gx_lane = a.gx + (int64_t)(sub >> 1) * a.ld + n_wave + grp * 2 + (sub & 1);

    for (int step = 0; step < n_k; ++step) {
        const int k = pair_at(step), k_next = pair_at(step + 1);
        const float *slab = (step & 1) ? slab1 : slab0;
        float *slab_next = (step & 1) ? slab0 : slab1;
        if constexpr (sizeof(CT) == 4) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (sizeof(CT) != 4 || step + 1 < n_k) fill.template issue<0>(sa, slab_next, k_next, jt, wave, lane);

        constexpr int kNear = 1;
        Corners ring[kNear + 1];
        int off_cur = r_node[0] * kNarrowRowBytes, off_nxt = 0;
        float b_lo = 0.f, b_hi = 0.f, a_lo = 0.f, a_hi = 0.f;
        float stash_a = 0.f, stash_b = 0.f;
        load_corners_quad<0>(ring[0], slab, off_cur, lane_bytes, a.W);
        static_for(std::make_integer_sequence<int, STEPS>{}, [&](auto fc) {
            constexpr int F = decltype(fc)::value;
            constexpr int set = F / LPS, t = F % LPS;
            if constexpr (t == 0) {
                if constexpr (set == SETS / 2) {
                    fill.template commit<0>(sa, slab_next, wave, lane);
                    fill.template issue<1>(sa, slab_next, k_next, jt, wave, lane);
                }
                const int node = r_node[set];
                const int i1 = (int)(((float)node + 0.5f) * inv_w);  // node / W, exact for these sizes
                const float rh1 = s_invh[i1], rh2 = s_invh[node - i1 * a.W];
                const float u = r_u[set], v = r_v[set];
                b_lo = (1.0f - v) * rh1;
                b_hi = v * rh1;
                a_lo = (1.0f - u) * rh2;
                a_hi = u * rh2;
                if constexpr (set > 0) off_cur = off_nxt;
                if constexpr (set + 1 < SETS) off_nxt = r_node[set + 1] * kNarrowRowBytes;
                asm volatile("s_nop 1" : "+v"(b_lo), "+v"(b_hi), "+v"(a_lo), "+v"(a_hi), "+v"(off_cur), "+v"(off_nxt));
                fetch_record(set, k_next);
            }
            if constexpr (F + kNear < STEPS) {
                constexpr int F2 = F + kNear;
                load_corners_quad<F2 % LPS>(ring[F2 % (kNear + 1)], slab, (F2 / LPS == set) ? off_cur : off_nxt,
                                            lane_bytes, a.W);
            }
            const float v = grad_step_quad<t>(gyr[F], ring[F % (kNear + 1)], b_lo, b_hi, a_lo, a_hi, upper);
            if ((sub & 1) == (t & 1)) {
                if constexpr (t < 2) stash_a = v; else stash_b = v;
            }
            if constexpr (t == LPS - 1) {
                const int64_t n = n_lane + set * 64;
                float *dst = gx_lane + (int64_t)(2 * k) * a.ld + set * 64;
                if (n < a.B) unsafeAtomicAdd(dst, stash_a);
                if (n + 2 < a.B) unsafeAtomicAdd(dst + 32, stash_b);
            }
        });
        fill.template commit<1>(sa, slab_next, wave, lane);
    }
}

}  // namespace

size_t slab_forward_lds_bytes(const LayerShape &s)
{
    return (size_t)2 * s.nodes() * kRowBytes;
}

size_t records_bytes(const LayerShape &s)
{
    return (size_t)3 * (size_t)s.pairs() * (size_t)s.batch * 4;
}

void launch_preamble_records(const LayerShape &s, const GridTab &tab, const float *x, void *records,
                             hipStream_t stream, const ConvGeom *conv)
{
    const size_t n = (size_t)s.pairs() * (size_t)s.batch;
    int32_t *rec_node = static_cast<int32_t *>(records);
    float *rec_u = reinterpret_cast<float *>(rec_node + n);
    float *rec_v = rec_u + n;
    const dim3 grid((unsigned)((s.batch + kRecTile - 1) / kRecTile),
                    (unsigned)((s.pairs() + kRecPairs - 1) / kRecPairs));
    if (conv)
        preamble_records_kernel<true><<<grid, 256, 0, stream>>>(tab, x, rec_node, rec_u, rec_v, s.batch, s.n_in, *conv);
    else
        preamble_records_kernel<false><<<grid, 256, 0, stream>>>(tab, x, rec_node, rec_u, rec_v, s.batch, s.n_in,
                                                                ConvGeom{});
}

// 64-output tiles: the float32 slab fits LDS twice (G <= 16)
// Streaming every slab of the table through LDS pays from 256 rows on for any layer, and for any
// batch once a row is some work: pairs x outputs >= 8192 (e.g. 128 -> 128) for the input
// gradient, >= 1024 (64 -> 32) for the forward pass.  A single row of a 1024 -> 1024 layer takes
// 0.13 ms forward and 0.16 ms for grad_x here, about what it takes to read the table, against
// 0.68 and 2.8 ms on the generic kernels; 64 rows of 128 -> 32 take 0.029 ms forward against
// 0.109, but 0.037 ms for grad_x against 0.043; a 16 -> 16 layer is quicker on the generic kernels.
static bool slab_batch_ok(const LayerShape &s, bool forward)
{
    return s.batch >= 256 || (int64_t)s.pairs() * s.n_out >= (forward ? 1024 : 8192);
}

// which tile a shape takes when it takes a slab kernel at all
static bool slab_wide_fits(const LayerShape &s)
{
    return outputs_by_four_ok(s) && slab_forward_lds_bytes(s) <= 160 * 1024;
}

// 16-output tiles for larger grids (G <= 34)
static bool slab_narrow_fits(const LayerShape &s)
{
    return outputs_by_four_ok(s) && !slab_wide_fits(s) && (size_t)2 * s.nodes() * kNarrowRowBytes <= 160 * 1024;
}

// forward only: one 16-output slab at a time (35 <= G <= 48)
static bool slab_narrow_single_fits(const LayerShape &s)
{
    return outputs_by_four_ok(s) && !slab_wide_fits(s) && !slab_narrow_fits(s) &&
           (size_t)s.nodes() * kNarrowRowBytes <= 160 * 1024 - 512;
}

bool slab_forward_shape_ok(const LayerShape &s)
{
    return slab_batch_ok(s, true) && (slab_wide_fits(s) || slab_narrow_fits(s) || slab_narrow_single_fits(s));
}
bool slab_tile_is_wide(const LayerShape &s) { return slab_wide_fits(s); }

// Packed tables on the grids that stream two 16-output slabs, where two 32-output slabs as stored
// fit LDS as well (16-bit: all of those grids, float32: G <= 24): the lane32 kernels
static size_t half_tile_row_bytes(const LayerShape &s) { return (size_t)kHalfTile * (s.dtype == LMKAN_F32 ? 4 : 2); }
static bool slab_half_tiles_fit(const LayerShape &s)
{
    return slab_narrow_fits(s) && s.layout == LMKAN_LAYOUT_PACKED &&
           (size_t)2 * s.nodes() * half_tile_row_bytes(s) + LMKAN_MAX_GRID * sizeof(float) <= 160 * 1024;
}
bool slab_forward_takes_half_tiles(const LayerShape &s)
{
    return slab_batch_ok(s, true) && slab_half_tiles_fit(s);
}

// Samples per forward workgroup: 1024 with 64-output tiles, 4096 with 16-output tiles, 2048 with
// 32-output tiles.
int slab_forward_split(const LayerShape &s)
{
    if (!slab_forward_shape_ok(s)) return 1;
    const bool wide = slab_wide_fits(s);
    const bool half = slab_forward_takes_half_tiles(s);
    const int64_t tile_b = wide ? 1024 : half ? 2048 : 4096;
    const int64_t n_jt = wide ? s.out_tiles() : half ? (s.n_out + 31) / 32 : (s.n_out + 15) / 16;
    return pair_split_count((int)(((s.batch + tile_b - 1) / tile_b) * n_jt), s.pairs());
}

size_t slab_forward_partial_bytes(const LayerShape &s)
{
    const size_t parts = (size_t)slab_forward_split(s) - 1;
    return (parts * (size_t)partial_stride((int64_t)s.batch * s.n_out) * sizeof(float) + 255) & ~(size_t)255;
}

namespace {
// y[i] += sum over p of part[p * stride + i]; stride is a multiple of four, y and part 16-byte aligned
__global__ __launch_bounds__(256) void sum_partials_kernel(float *__restrict__ y, const float *__restrict__ part,
                                                          int n_part, int64_t elems, int64_t stride)
{
    const int64_t quads = elems / 4;
    const int64_t step = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < quads; i += step) {
        float4 v = reinterpret_cast<float4 *>(y)[i];
        for (int p = 0; p < n_part; ++p) {
            const float4 w = reinterpret_cast<const float4 *>(part + (int64_t)p * stride)[i];
            v.x += w.x;
            v.y += w.y;
            v.z += w.z;
            v.w += w.w;
        }
        reinterpret_cast<float4 *>(y)[i] = v;
    }
    // the last one to three elements of a tensor whose size is not a multiple of four
    const int64_t t = quads * 4 + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t < elems) {
        float v = y[t];
        for (int p = 0; p < n_part; ++p) v += part[(int64_t)p * stride + t];
        y[t] = v;
    }
}
}  // namespace

void launch_sum_partials(float *y, const float *part, int n_part, int64_t elems, hipStream_t stream)
{
    const int64_t quads = elems / 4;
    int64_t blocks = (quads + 255) / 256;
    if (blocks < 1) blocks = 1;
    sum_partials_kernel<<<(unsigned)(blocks < 8192 ? blocks : 8192), 256, 0, stream>>>(y, part, n_part, elems,
                                                                                      partial_stride(elems));
}

bool slab_forward_applicable(const LayerShape &s, const void *coef, const float *y)
{
    if (!slab_forward_shape_ok(s)) return false;
    return ((reinterpret_cast<uintptr_t>(coef) | reinterpret_cast<uintptr_t>(y)) & 15) == 0;
}

static void launch_forward_slab_narrow(const LayerShape &s, const void *coef, float *y, const void *records,
                                       float *partials, hipStream_t stream)
{
    constexpr int WAVES = 8, SETS = 8;
    constexpr int kTileB = WAVES * SETS * 64;
    typedef void (*Kernel)(SlabArgs);
    if (slab_forward_takes_half_tiles(s)) {
        const Kernel k32 = s.dtype == LMKAN_F32   ? forward_lane32_f32_kernel
                           : s.dtype == LMKAN_F16 ? forward_lane32_kernel<_Float16>
                                                  : forward_lane32_kernel<bf16_t>;
        allow_large_lds(reinterpret_cast<const void *>(k32), 160 * 1024);
        const size_t nrec = (size_t)s.pairs() * (size_t)s.batch;
        SlabArgs a;
        a.P = coef;
        a.y = y;
        a.rec_node = static_cast<const int32_t *>(records);
        a.rec_u = reinterpret_cast<const float *>(a.rec_node + nrec);
        a.rec_v = a.rec_u + nrec;
        a.map = coef_map(s);
        a.B = s.batch;
        a.n_out = s.n_out;
        a.K = s.pairs();
        a.W = s.G + 1;
        a.nodes = s.nodes();
        a.col_limit = s.out_tiles() * kTile;
        a.packed = 1;
        a.n_btiles = (int)((s.batch + 2047) / 2048);
        a.n_jt = (s.n_out + kHalfTile - 1) / kHalfTile;
        const int tiles32 = a.n_btiles * a.n_jt;
        const int split32 = slab_forward_split(s);   // what the workspace was sized for
        a.n_split = split32;
        a.pairs_per_split = (a.K + split32 - 1) / split32;
        finish_split_setup(a, s, y, partials, stream);
        {
            KernelTiming timing(stream, kTimeForward);
            k32<<<tiles32 * split32, 1024, ((size_t)2 * s.nodes() * half_tile_row_bytes(s) + 15) & ~(size_t)15, stream>>>(a);
        }
        if (a.y_part) launch_sum_partials(y, a.y_part, split32 - 1, (int64_t)s.batch * s.n_out, stream);
        return;
    }
    // a float32 table needs no staging registers: 16 waves of 256 samples instead of 8 of 512
    const bool single = slab_narrow_single_fits(s);
    const Kernel kernels[6] = {forward_slab_narrow_kernel<float, 2 * WAVES, SETS / 2>,
                               forward_slab_narrow_kernel<_Float16, WAVES, SETS>,
                               forward_slab_narrow_kernel<bf16_t, WAVES, SETS>,
                               forward_slab_narrow_kernel<float, 2 * WAVES, SETS / 2, true>,
                               forward_slab_narrow_kernel<_Float16, WAVES, SETS, true>,
                               forward_slab_narrow_kernel<bf16_t, WAVES, SETS, true>};
    const Kernel kernel = kernels[s.dtype + (single ? 3 : 0)];
    const int waves = s.dtype == LMKAN_F32 ? 2 * WAVES : WAVES;
    allow_large_lds(reinterpret_cast<const void *>(kernel), 160 * 1024);
    const size_t n = (size_t)s.pairs() * (size_t)s.batch;
    SlabArgs a;
    a.P = coef;
    a.y = y;
    a.rec_node = static_cast<const int32_t *>(records);
    a.rec_u = reinterpret_cast<const float *>(a.rec_node + n);
    a.rec_v = a.rec_u + n;
    a.map = coef_map(s);
    a.B = s.batch;
    a.n_out = s.n_out;
    a.K = s.pairs();
    a.W = s.G + 1;
    a.nodes = s.nodes();
    a.col_limit = s.layout == LMKAN_LAYOUT_PACKED ? s.out_tiles() * kTile : s.n_out;
    a.packed = s.layout == LMKAN_LAYOUT_PACKED;
    a.n_btiles = (int)((s.batch + kTileB - 1) / kTileB);
    a.n_jt = (s.n_out + kNarrowTile - 1) / kNarrowTile;
    const int tiles = a.n_btiles * a.n_jt;
    const int split = pair_split_count(tiles, a.K);
    a.n_split = split;
    a.pairs_per_split = (a.K + split - 1) / split;
    finish_split_setup(a, s, y, partials, stream);
    {
        KernelTiming timing(stream, kTimeForward);
        kernel<<<tiles * split, waves * 64, (size_t)(single ? 1 : 2) * s.nodes() * kNarrowRowBytes, stream>>>(a);
    }
    if (a.y_part) launch_sum_partials(y, a.y_part, split - 1, (int64_t)s.batch * s.n_out, stream);
}

void launch_forward_slab(const LayerShape &s, const void *coef, float *y, const void *records, float *partials,
                         hipStream_t stream)
{
    if (!slab_wide_fits(s)) {
        launch_forward_slab_narrow(s, coef, y, records, partials, stream);
        return;
    }
    if (slab_f16_native_ok(s)) {
        launch_forward_slab_f16(s, coef, y, records, partials, stream);
        return;
    }
    // 1024 samples per workgroup either way: 16 waves x 64 samples for float32 tables, 8 x 128 for
    // 16-bit tables (their staging registers do not fit the smaller register share)
    constexpr int kTileB = 1024;
    typedef void (*Kernel)(SlabArgs);
    // G = 16 (the usual grid) gets a kernel with the row stride folded into the LDS offsets
    const Kernel kernels[3] = {forward_slab_kernel<float, 16, 1, 1, 0>,
                               forward_slab_kernel<_Float16, 8, 2, 2, 0>, forward_slab_kernel<bf16_t, 8, 2, 2, 0>};
    const Kernel kernels17[3] = {forward_slab_kernel<float, 16, 1, 1, 17>,
                                 forward_slab_kernel<_Float16, 8, 2, 2, 17>, forward_slab_kernel<bf16_t, 8, 2, 2, 17>};
    const Kernel kernel = s.G == 16 ? kernels17[s.dtype] : kernels[s.dtype];
    const int waves = s.dtype == LMKAN_F32 ? 16 : 8;
    allow_large_lds(reinterpret_cast<const void *>(kernel), 160 * 1024);
    const size_t n = (size_t)s.pairs() * (size_t)s.batch;
    SlabArgs a;
    a.P = coef;
    a.y = y;
    a.rec_node = static_cast<const int32_t *>(records);
    a.rec_u = reinterpret_cast<const float *>(a.rec_node + n);
    a.rec_v = a.rec_u + n;
    a.map = coef_map(s);
    a.B = s.batch;
    a.n_out = s.n_out;
    a.K = s.pairs();
    a.W = s.G + 1;
    a.nodes = s.nodes();
    a.col_limit = s.layout == LMKAN_LAYOUT_PACKED ? s.out_tiles() * kTile : s.n_out;
    a.packed = s.layout == LMKAN_LAYOUT_PACKED;
    a.n_btiles = (int)((s.batch + kTileB - 1) / kTileB);
    a.n_jt = s.out_tiles();
    // split the pairs over several workgroups when the tiles alone cannot fill 256 CUs
    const int tiles = a.n_btiles * a.n_jt;
    const int split = pair_split_count(tiles, a.K);
    a.n_split = split;
    a.pairs_per_split = (a.K + split - 1) / split;
    finish_split_setup(a, s, y, partials, stream);
    {
        KernelTiming timing(stream, kTimeForward);
        kernel<<<tiles * split, waves * 64, slab_forward_lds_bytes(s), stream>>>(a);
    }
    if (a.y_part) launch_sum_partials(y, a.y_part, split - 1, (int64_t)s.batch * s.n_out, stream);
}

}  // namespace lmkan

namespace lmkan {

bool slab_backward_input_shape_ok(const LayerShape &s)
{
    return slab_batch_ok(s, false) && (slab_wide_fits(s) || slab_narrow_fits(s));
}

// the input gradient on 32-output tiles kept in LDS as they are stored (backward_input_lane32_kernel)
bool slab_backward_input_takes_half_tiles(const LayerShape &s)
{
    return slab_backward_input_shape_ok(s) && slab_half_tiles_fit(s);
}

bool slab_backward_input_applicable(const LayerShape &s, const void *coef, const float *gy, const float *gx)
{
    if (!slab_backward_input_shape_ok(s)) return false;
    // (with a ragged output count gy is read through its tile-by-tile copy, which is aligned)
    if ((reinterpret_cast<uintptr_t>(coef) & 15) != 0 || (reinterpret_cast<uintptr_t>(gx) & 3) != 0) return false;
    return ragged_outputs(s) || (reinterpret_cast<uintptr_t>(gy) & 15) == 0;
}

namespace {

// gx[img][y][x][c] = sum over the windows that contain (y, x) of the patch gradient
// in_t[(ky kw + kx) C + c][row of that window]; elements no window covers get zero
__global__ __launch_bounds__(256) void conv_input_gradient_kernel(const float *__restrict__ in_t,
                                                                 float *__restrict__ gx, ConvGeom cg, int64_t ld,
                                                                 int layout)
{
    const int64_t total = (int64_t)cg.N * cg.H * cg.W * cg.C;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int c = (int)(i % cg.C);
    const int xw = (int)((i / cg.C) % cg.W);
    const int yh = (int)((i / ((int64_t)cg.C * cg.W)) % cg.H);
    const int64_t img = i / ((int64_t)cg.C * cg.W * cg.H);
    float sum = 0.f;
    for (int ky = 0; ky < cg.kh; ++ky) {
        const int ty = yh - ky;
        if (ty < 0 || ty % cg.stride != 0) continue;
        const int oy = ty / cg.stride;
        if (oy >= cg.OH) continue;
        for (int kx = 0; kx < cg.kw; ++kx) {
            const int tx = xw - kx;
            if (tx < 0 || tx % cg.stride != 0) continue;
            const int ox = tx / cg.stride;
            if (ox >= cg.OW) continue;
            const int64_t row = (img * cg.OH + oy) * cg.OW + ox;
            sum += in_t[(int64_t)((ky * cg.kw + kx) * cg.C + c) * ld + scratch_position(row, layout)];
        }
    }
    gx[i] = sum;
}

// Windows that do not overlap (stride >= window): every image element belongs to at most one
// window, so the transposed scratch is scattered straight into the image, 64 rows x 64 inputs per
// block through an LDS tile: reads run along the rows, writes along the channels of a pixel.
__global__ __launch_bounds__(256) void conv_input_gradient_scatter_kernel(const float *__restrict__ in_t,
                                                                         float *__restrict__ gx, ConvGeom cg,
                                                                         int64_t rows, int n_in, int64_t ld, int layout)
{
    __shared__ float tile[64][65];
    __shared__ int64_t s_base[64];
    const int64_t n0 = (int64_t)blockIdx.x * 64;
    const int e0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    if (threadIdx.x < 64 && n0 + tx < rows) s_base[tx] = conv_input_offset(cg, n0 + tx, 0);
    const int64_t src = scratch_position(n0 + tx, layout);
    for (int r = ty; r < 64; r += 4)
        if (e0 + r < n_in && n0 + tx < rows) tile[r][tx] = in_t[(int64_t)(e0 + r) * ld + src];
    __syncthreads();
    const int e = e0 + tx;
    if (e >= n_in) return;
    const int c = e % cg.C, kx = (e / cg.C) % cg.kw, ky = e / (cg.C * cg.kw);
    const int64_t e_off = ((int64_t)ky * cg.W + kx) * cg.C + c;
    for (int r = ty; r < 64; r += 4)
        if (n0 + r < rows) gx[s_base[r] + e_off] = tile[tx][r];
}

}  // namespace

void launch_input_gradient_out(const float *in_t, float *gx, const LayerShape &s, const ConvGeom *conv,
                               hipStream_t stream, int scratch_layout)
{
    const int64_t ld = scratch_row_stride(s.batch, scratch_layout);
    if (!conv) {
        const dim3 grid((unsigned)((s.batch + 63) / 64), (unsigned)((s.n_in + 63) / 64));
        transpose_kernel<<<grid, 256, 0, stream>>>(in_t, gx, s.batch, s.n_in, ld, scratch_layout);
        return;
    }
    const ConvGeom &cg = *conv;
    const int64_t total = (int64_t)cg.N * cg.H * cg.W * cg.C;
    if (cg.stride >= cg.kh && cg.stride >= cg.kw) {
        const bool covered = cg.stride == cg.kh && cg.stride == cg.kw && cg.OH * cg.kh == cg.H && cg.OW * cg.kw == cg.W;
        if (!covered) launch_fill_zero(gx, (size_t)total, stream);  // gaps between or beyond the windows
        const dim3 grid((unsigned)((s.batch + 63) / 64), (unsigned)((s.n_in + 63) / 64));
        conv_input_gradient_scatter_kernel<<<grid, 256, 0, stream>>>(in_t, gx, cg, s.batch, s.n_in, ld, scratch_layout);
        return;
    }
    conv_input_gradient_kernel<<<(unsigned)((total + 255) / 256), 256, 0, stream>>>(in_t, gx, cg, ld, scratch_layout);
}

void launch_transpose(const float *in_t, float *out, int64_t batch, int n_in, hipStream_t stream)
{
    const dim3 grid((unsigned)((batch + 63) / 64), (unsigned)((n_in + 63) / 64));
    transpose_kernel<<<grid, 256, 0, stream>>>(in_t, out, batch, n_in, batch, kScratchPlain);
}

size_t slab_backward_input_scratch_bytes(const LayerShape &s)
{
    // rows padded to whole blocks of 64 samples (the quad layout permutes inside such blocks)
    return ((((size_t)s.batch + 63) & ~(size_t)63) * s.n_in * sizeof(float) + 255) & ~(size_t)255;
}

void launch_backward_input_slab(const LayerShape &s, const GridTab &tab, const void *coef, const float *gy,
                                int64_t gy_tile_stride, int64_t gy_row_stride, float *gx, const void *records,
                                void *scratch, hipStream_t stream, const ConvGeom *conv)
{
    if (slab_wide_fits(s) && slab_f16_native_ok(s)) {
        launch_fill_zero(static_cast<float *>(scratch), (size_t)scratch_row_stride(s.batch, kScratchPlain) * s.n_in,
                         stream);
        launch_backward_input_slab_f16(s, tab, coef, gy, gy_tile_stride, gy_row_stride, static_cast<float *>(scratch),
                                       records, stream);
        launch_input_gradient_out(static_cast<float *>(scratch), gx, s, conv, stream, kScratchPlain);
        return;
    }
    constexpr int WAVES = 8, SETS = 2;
    constexpr int kTileB = WAVES * SETS * 64;
    typedef void (*Kernel)(GradInArgs);
    const bool narrow = !slab_wide_fits(s);
    // packed tables on the grids of the 16-output tiles: 32-output tiles kept as stored where two fit
    const bool lane32 = slab_backward_input_takes_half_tiles(s);
    if (lane32) {
        const Kernel k32 = s.dtype == LMKAN_F32   ? backward_input_lane32_f32_kernel
                           : s.dtype == LMKAN_F16 ? backward_input_lane32_kernel<_Float16>
                                                  : backward_input_lane32_kernel<bf16_t>;
        allow_large_lds(reinterpret_cast<const void *>(k32), 160 * 1024);
        const size_t nrec = (size_t)s.pairs() * (size_t)s.batch;
        GradInArgs a;
        a.P = coef;
        a.gy = gy;
        a.gy_tile_stride = gy_tile_stride;
        a.gy_row_stride = gy_row_stride;
        a.gx = static_cast<float *>(scratch);
        a.rec_node = static_cast<const int32_t *>(records);
        a.rec_u = reinterpret_cast<const float *>(a.rec_node + nrec);
        a.rec_v = a.rec_u + nrec;
        a.map = coef_map(s);
        a.tab = tab;
        a.B = s.batch;
        a.n_in = s.n_in;
        a.n_out = s.n_out;
        a.K = s.pairs();
        a.W = s.G + 1;
        a.nodes = s.nodes();
        a.col_limit = s.out_tiles() * kTile;
        a.packed = 1;
        a.n_btiles = (int)((s.batch + 2047) / 2048);
        a.n_jt = (s.n_out + kHalfTile - 1) / kHalfTile;
        const int tiles32 = a.n_btiles * a.n_jt;
        int split32 = 1;
        while (tiles32 * split32 < 256 && a.K / (split32 * 2) >= 4) split32 *= 2;
        a.n_split = split32;
        a.pairs_per_split = (a.K + split32 - 1) / split32;
        a.ld = scratch_row_stride(s.batch, kScratchPlain);
        launch_fill_zero(a.gx, (size_t)a.ld * s.n_in, stream);
        const size_t lds = (((size_t)2 * s.nodes() * half_tile_row_bytes(s) + 15) & ~(size_t)15) + LMKAN_MAX_GRID * sizeof(float);
        {
            KernelTiming timing(stream, kTimeGradInput);
            k32<<<tiles32 * split32, 1024, lds, stream>>>(a);
        }
        launch_input_gradient_out(a.gx, gx, s, conv, stream, kScratchPlain);
        return;
    }
    constexpr int kNarrowSets = 8;
    constexpr int kWavesF32 = 16;  // float32 tables need no staging registers: 16 waves of 64 samples
    // (float32 tables on 64-output tiles: the kernel with a lane per sample)
    const Kernel kernels[9] = {backward_input_lane_kernel<float, 0>,
                               backward_input_slab_kernel<_Float16, WAVES, SETS, 2, 0>,
                               backward_input_slab_kernel<bf16_t, WAVES, SETS, 2, 0>,
                               backward_input_slab_narrow_kernel<float, 2 * WAVES, kNarrowSets / 2>,
                               backward_input_slab_narrow_kernel<_Float16, WAVES, kNarrowSets>,
                               backward_input_slab_narrow_kernel<bf16_t, WAVES, kNarrowSets>,
                               backward_input_lane_kernel<float, 17>,
                               backward_input_slab_kernel<_Float16, WAVES, SETS, 2, 17>,
                               backward_input_slab_kernel<bf16_t, WAVES, SETS, 2, 17>};
    const int which = s.dtype + (narrow ? 3 : (s.G == 16 ? 6 : 0));
    const Kernel kernel = kernels[which];
    allow_large_lds(reinterpret_cast<const void *>(kernel), 160 * 1024);
    const size_t n = (size_t)s.pairs() * (size_t)s.batch;
    GradInArgs a;
    a.P = coef;
    a.gy = gy;
    a.gy_tile_stride = gy_tile_stride;
    a.gy_row_stride = gy_row_stride;
    a.gx = static_cast<float *>(scratch);
    a.rec_node = static_cast<const int32_t *>(records);
    a.rec_u = reinterpret_cast<const float *>(a.rec_node + n);
    a.rec_v = a.rec_u + n;
    a.map = coef_map(s);
    a.tab = tab;
    a.B = s.batch;
    a.n_in = s.n_in;
    a.n_out = s.n_out;
    a.K = s.pairs();
    a.W = s.G + 1;
    a.nodes = s.nodes();
    a.col_limit = s.layout == LMKAN_LAYOUT_PACKED ? s.out_tiles() * kTile : s.n_out;
    a.packed = s.layout == LMKAN_LAYOUT_PACKED;
    const int tile_b = narrow ? WAVES * kNarrowSets * 64 : kTileB;
    a.n_btiles = (int)((s.batch + tile_b - 1) / tile_b);
    a.n_jt = narrow ? (s.n_out + kNarrowTile - 1) / kNarrowTile : s.out_tiles();
    const int tiles = a.n_btiles * a.n_jt;
    int split = 1;
    while (tiles * split < 256 && a.K / (split * 2) >= 4) split *= 2;
    a.n_split = split;
    a.pairs_per_split = (a.K + split - 1) / split;
    const bool lane_kernel = !narrow && s.dtype == LMKAN_F32;   // its lanes are consecutive samples
    const int layout = lane_kernel ? kScratchPlain : narrow ? kScratchQuad : kScratchOct;
    a.ld = scratch_row_stride(s.batch, layout);
    launch_fill_zero(a.gx, (size_t)a.ld * s.n_in, stream);
    const size_t slabs = narrow ? (size_t)2 * s.nodes() * kNarrowRowBytes : slab_forward_lds_bytes(s);
    const int waves = s.dtype == LMKAN_F32 ? (narrow ? 2 * WAVES : kWavesF32) : WAVES;
    {
        KernelTiming timing(stream, kTimeGradInput);
        kernel<<<tiles * split, waves * 64, slabs + LMKAN_MAX_GRID * sizeof(float), stream>>>(a);
    }
    launch_input_gradient_out(a.gx, gx, s, conv, stream, layout);
}

}  // namespace lmkan
