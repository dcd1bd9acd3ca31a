// Slab kernels for float16 tables that keep the slab in LDS as float16.
//
// Same decomposition as the float32 slab kernels (lmkan_slab.hip): a workgroup owns 1024
// samples x 64 outputs, 16 waves of 64 samples, and streams the (G+1)^2 x 64 slab of each pair
// through LDS, double buffered.  Here a table row is 128 bytes in LDS and arrives by LDS-direct
// loads of the stored values as they are; a lane reads four outputs of a corner row with one
// ds_read_b64, and the float16 values enter the float32 multiply-adds directly (v_fma_mix_f32
// widens an operand on the fly), so nothing is converted in a separate instruction.  Per
// multiply-add the kernels move half the LDS and L2 bytes of the float32 path.  Forward: lanes
// are outputs; the mixed multiply-add has no DPP form, so the sample's four weights are copied
// into the lanes of its group with four DPP moves per step.  Input gradient: a lane is a sample
// and reads the rows of its own cell in a per-lane rotated order.  (The forward pass with a lane
// per sample was measured too: 0.76 against 0.80 ms on cfg3, but slower on long batches of
// narrow layers, 0.58 against 0.53 ms for 262144 rows of 128 -> 128, where the rotated 16-byte
// stores of y weigh more; it is not kept.)
#include <utility>

#include "lmkan_kernels.h"
#include "lmkan_slab_common.h"

namespace lmkan {

namespace {

constexpr int kTile = kSlabTile;
constexpr int kRowBytesH = kTile * 2;  // one table row of a float16 slab in LDS
constexpr int kWaves = 16;             // waves per workgroup, 64 samples each
constexpr int kAheadH = 2;             // LDS reads run two steps ahead

typedef _Float16 h4v __attribute__((ext_vector_type(4)));

// Stream the float16 slab of (pair k, output tile jt) into LDS.  A wave instruction moves
// 8 table rows (8 lanes x 16 bytes per row); the 1 KiB it writes is contiguous in LDS.
__device__ __forceinline__ void issue_slab_load_h(const SlabArgs &a, unsigned lds_base, int k, int jt, int wave, int lane)
{
    const _Float16 *P = static_cast<const _Float16 *>(a.P);
    const int row = lane >> 3, l8 = lane & 7;
    const int full = a.nodes >> 3;  // chunks made of eight rows
    const int rest = a.nodes & 7;
    if (a.packed) {
        // the slab is one contiguous run of nodes x 128 bytes
        const char *src = reinterpret_cast<const char *>(P + (int64_t)k * a.map.s_pair + (int64_t)jt * a.map.s_tile);
        const unsigned lane_off = (unsigned)lane * 16u;
        for (int c = wave; c < full; c += kWaves) lds_dma16_uniform(src + (size_t)c * 1024, lane_off, lds_base + c * 1024);
        if (rest != 0 && full % kWaves == wave && row < rest)
            lds_dma16_uniform(src + (size_t)full * 1024, lane_off, lds_base + full * 1024);
        return;
    }
    const int col = jt * kTile + l8 * 8;
    const _Float16 *src = P + (int64_t)k * a.map.s_pair + (int64_t)(col >> 6) * a.map.s_tile + (col & 63);
    const bool col_ok = col < a.col_limit;  // never read past a table row (n_out is a multiple of 8 here)
    const int chunks = full + (rest != 0);
    for (int c = wave; c < chunks; c += kWaves) {
        const int node = c * 8 + row;
        if (node < a.nodes && col_ok)
            lds_dma16(src + (int64_t)node * a.map.s_node, __builtin_amdgcn_readfirstlane(lds_base + c * 1024));
    }
}

// The four table rows of one step: corners (i1,i2), (i1,i2+1), (i1+1,i2), (i1+1,i2+1).
struct CornersH {
    h4v c00, c01, c10, c11;
};

__device__ __forceinline__ h4v lds_load_h4(unsigned addr)
{
    return *reinterpret_cast<__attribute__((address_space(3))) const h4v *>(addr);
}

template <int S>
__device__ __forceinline__ void load_corners_h(CornersH &c, int lane_base, int off_bytes, int W)
{
    const unsigned addr = (unsigned)(row_bcast<S>(off_bytes) + lane_base);
    c.c00 = lds_load_h4(addr);
    c.c01 = lds_load_h4(addr + kRowBytesH);
    c.c10 = lds_load_h4(addr + W * kRowBytesH);
    c.c11 = lds_load_h4(addr + W * kRowBytesH + kRowBytesH);
}

template <int S>
__device__ __forceinline__ float bcast_f(float v)
{
    return __int_as_float(row_bcast<S>(__float_as_int(v)));
}

template <int S>
__device__ __forceinline__ void fma_corners_h(float *acc, const CornersH &c, float w00, float w10, float w01, float w11)
{
    const float a = bcast_f<S>(w00), b = bcast_f<S>(w10), d = bcast_f<S>(w01), e = bcast_f<S>(w11);
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = fmaf(a, (float)c.c00[i], acc[i]);
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = fmaf(b, (float)c.c10[i], acc[i]);
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = fmaf(d, (float)c.c01[i], acc[i]);
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = fmaf(e, (float)c.c11[i], acc[i]);
}

__global__ __launch_bounds__(kWaves * 64) __attribute__((amdgpu_waves_per_eu(4, 4))) void forward_slab_f16_kernel(SlabArgs a)
{
    extern __shared__ __align__(16) char smem_h[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    constexpr int kTileB = kWaves * 64;

    int id = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int btile = id % a.n_btiles;
    const int rest = id / a.n_btiles;
    const int ks = rest % a.n_split;
    const int jt = rest / a.n_split;

    const int k_begin = ks * a.pairs_per_split;
    const int k_end = min(a.K, k_begin + a.pairs_per_split);
    const unsigned slab_bytes = (unsigned)a.nodes * kRowBytesH;
    const unsigned base0 = __builtin_amdgcn_readfirstlane(lds_address(smem_h));
    const unsigned base1 = base0 + slab_bytes;
    const int64_t n_wave = (int64_t)btile * kTileB + (int64_t)wave * 64;

    float acc[64];
#pragma unroll
    for (int i = 0; i < 64; ++i) acc[i] = 0.0f;

    // record of (sample n_wave + lane, pair k), fetched one pair ahead
    int nx_node = 0;
    float nx_u = 0.f, nx_v = 0.f;
    auto fetch_record = [&](int k) {
        const int64_t n = n_wave + lane;
        nx_node = 0;
        nx_u = 0.f;
        nx_v = 0.f;
        if (n < a.B) {
            const int64_t o = (int64_t)k * a.B + n;
            nx_node = a.rec_node[o];
            nx_u = a.rec_u[o];
            nx_v = a.rec_v[o];
        }
    };

    if (k_begin < k_end) {
        issue_slab_load_h(a, base0, k_begin, jt, wave, lane);
        fetch_record(k_begin);
    }
    const int lane_bytes = l16 * 8;
    for (int k = k_begin; k < k_end; ++k) {
        const unsigned cur = ((k - k_begin) & 1) ? base1 : base0;
        const unsigned nxt = ((k - k_begin) & 1) ? base0 : base1;
        const float u = nx_u, v = nx_v;
        const float a_lo = 1.0f - u, b_lo = 1.0f - v;
        const int off = nx_node * kRowBytesH;
        const float w00 = a_lo * b_lo, w10 = u * b_lo, w01 = a_lo * v, w11 = u * v;
        // this wave's slab loads for pair k have landed; after the barrier everybody's have,
        // and everybody has finished reading the other buffer (pair k-1)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (k + 1 < k_end) {
            issue_slab_load_h(a, nxt, k + 1, jt, wave, lane);
            fetch_record(k + 1);
        }
        CornersH ring[kAheadH + 1];
        const int lane_base = (int)cur + lane_bytes;
        load_corners_h<0>(ring[0], lane_base, off, a.W);
        load_corners_h<1>(ring[1], lane_base, off, a.W);
        static_for(std::make_integer_sequence<int, 16>{}, [&](auto tc) {
            constexpr int T = decltype(tc)::value;
            if constexpr (T + kAheadH < 16)
                load_corners_h<T + kAheadH>(ring[(T + kAheadH) % (kAheadH + 1)], lane_base, off, a.W);
            fma_corners_h<T>(acc + 4 * T, ring[T % (kAheadH + 1)], w00, w10, w01, w11);
        });
    }

    // lane (g, l16) holds outputs jt*64 + 4*l16 .. +3 of samples n_wave + 16*g + step
    const int col = jt * kTile + l16 * 4;
    bool atomic;
    float *ybase = forward_out_base(a, ks, atomic);
    if (col < a.n_out) {
#pragma unroll
        for (int st = 0; st < 16; ++st) {
            const int64_t n = n_wave + g * 16 + st;
            if (n < a.B) store_outputs(ybase + n * a.n_out + col, acc + st * 4, a.n_out, col, atomic);
        }
    }
}

// acc += gy . c over the four outputs of a piece (v_fma_mix_f32 widens the float16 operand)
__device__ __forceinline__ float fma4_h(const float4 g, const h4v c, float acc)
{
    return fmaf(g.w, (float)c[3], fmaf(g.z, (float)c[2], fmaf(g.y, (float)c[1], fmaf(g.x, (float)c[0], acc))));
}

// Input gradient with a lane per sample (see backward_input_lane_kernel in lmkan_slab.hip for
// the scheme): the 64 gy values of the lane's sample and tile in registers, the four corner rows
// of its cell read eight bytes (four float16 outputs) at a time, lane l taking piece
// (j + l) mod 16 at step j so that the 16 lanes of a group never meet on a bank; the four dot
// products stay inside the lane, the differences of neighbouring corners are taken per piece,
// and the two derivatives go to the transposed scratch (plain layout) with one atomic each.
// W_CT: G + 1 when known at compile time (the corner offsets are then immediates), else 0
template <int W_CT>
__global__ __launch_bounds__(kWaves * 64) __attribute__((amdgpu_waves_per_eu(4, 4))) void backward_input_slab_f16_kernel(
    GradInArgs a)
{
    extern __shared__ __align__(16) char smem_h[];  // two slab buffers, then 1/h of the grid
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l15 = lane & 15;
    const int w = W_CT > 0 ? W_CT : a.W;
    constexpr int kTileB = kWaves * 64;
    int id = blockIdx.x;
    const int total = gridDim.x;
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int btile = id % a.n_btiles;
    const int rest = id / a.n_btiles;
    const int ks = rest % a.n_split;
    const int jt = rest / a.n_split;

    const int k_begin = ks * a.pairs_per_split;
    const int k_end = min(a.K, k_begin + a.pairs_per_split);
    const unsigned slab_bytes = (unsigned)a.nodes * kRowBytesH;
    const unsigned base0 = __builtin_amdgcn_readfirstlane(lds_address(smem_h));
    const unsigned base1 = base0 + slab_bytes;
    const unsigned slabs_end = (2 * slab_bytes + 15) & ~15u;
    float *s_invh = reinterpret_cast<float *>(smem_h + slabs_end);
    for (int i = threadIdx.x; i < a.tab.G; i += blockDim.x) s_invh[i] = a.tab.inv_h[i];
    SlabArgs sa;  // only the fields issue_slab_load_h reads
    sa.P = a.P;
    sa.map = a.map;
    sa.nodes = a.nodes;
    sa.col_limit = a.col_limit;
    sa.packed = a.packed;

    const int64_t n = (int64_t)btile * kTileB + (int64_t)wave * 64 + lane;
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

    int nx_node = 0;
    float nx_u = 0.f, nx_v = 0.f;
    auto fetch_record = [&](int k) {
        const int64_t o = (int64_t)k * a.B + n_rd;
        nx_node = a.rec_node[o];
        nx_u = a.rec_u[o];
        nx_v = a.rec_v[o];
    };

    // columns past the end of a ragged output tile are never loaded: make them read as zero
    for (unsigned i = threadIdx.x * 16u; i < 2 * slab_bytes; i += blockDim.x * 16u)
        *reinterpret_cast<float4 *>(smem_h + i) = make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();  // zeros and s_invh in place before any slab load lands
    if (k_begin < k_end) {
        issue_slab_load_h(sa, base0, k_begin, jt, wave, lane);
        fetch_record(k_begin);
    }
    float *gx_lane = a.gx + n;   // transposed scratch [n_in][ld], plain layout

    for (int k = k_begin; k < k_end; ++k) {
        const unsigned cur = ((k - k_begin) & 1) ? base1 : base0;
        const unsigned nxt = ((k - k_begin) & 1) ? base0 : base1;
        const int node = nx_node;
        const float u = nx_u, v = nx_v;
        const int i1 = node / w;
        const float rh1 = s_invh[i1], rh2 = s_invh[node - i1 * w];
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (k + 1 < k_end) {
            issue_slab_load_h(sa, nxt, k + 1, jt, wave, lane);
            fetch_record(k + 1);
        }
        // piece (j + l15) mod 16 of the row: from `first` for j < 16 - l15, one row back after the wrap
        unsigned first = cur + (unsigned)node * kRowBytesH + (unsigned)l15 * 8;
        // dif_a = sum gy (P10 - P00), dif_b = sum gy (P11 - P01), dif_c = sum gy (P01 - P00),
        // dif_d = sum gy (P11 - P10): the four products summed over the four outputs of a piece
        // only, their differences taken at once
        float dif_a = 0.f, dif_b = 0.f, dif_c = 0.f, dif_d = 0.f;
        CornersH ring[kAheadH + 1];
        auto request = [&](CornersH &c, int j) {
            // (the empty statement ties the addresses to the sums so far: it keeps the reads of a
            // piece between the multiply-adds of the pieces before it)
            asm volatile("" : "+v"(first), "+v"(dif_a), "+v"(dif_b), "+v"(dif_c), "+v"(dif_d));
            const unsigned addr = (l15 + j >= 16 ? first - kRowBytesH : first) + j * 8;
            c.c00 = lds_load_h4(addr);
            c.c01 = lds_load_h4(addr + kRowBytesH);
            c.c10 = lds_load_h4(addr + w * kRowBytesH);
            c.c11 = lds_load_h4(addr + w * kRowBytesH + kRowBytesH);
        };
        request(ring[0], 0);
        request(ring[1], 1);
        static_for(std::make_integer_sequence<int, 16>{}, [&](auto jc) {
            constexpr int j = decltype(jc)::value;
            if constexpr (j + kAheadH < 16) request(ring[(j + kAheadH) % (kAheadH + 1)], j + kAheadH);
            const CornersH &c = ring[j % (kAheadH + 1)];
            const float p00 = fma4_h(gyr[j], c.c00, 0.0f), p01 = fma4_h(gyr[j], c.c01, 0.0f);
            const float p10 = fma4_h(gyr[j], c.c10, 0.0f), p11 = fma4_h(gyr[j], c.c11, 0.0f);
            dif_a += p10 - p00;
            dif_b += p11 - p01;
            dif_c += p01 - p00;
            dif_d += p11 - p10;
        });
        const float d1 = rh1 * (dif_a * (1.0f - v) + dif_b * v);
        const float d2 = rh2 * (dif_c * (1.0f - u) + dif_d * u);
        if (valid) {
            unsafeAtomicAdd(gx_lane + (int64_t)(2 * k) * a.ld, d1);
            unsafeAtomicAdd(gx_lane + (int64_t)(2 * k + 1) * a.ld, d2);
        }
    }
}

}  // namespace

// float16 table, slab fits LDS twice as float16 would always hold when it fits as float32;
// the direct loads need 16-byte pieces of a row: packed layout, or n_out a multiple of 8
bool slab_f16_native_ok(const LayerShape &s)
{
    if (s.dtype != LMKAN_F16) return false;
    if (s.layout != LMKAN_LAYOUT_PACKED && s.n_out % 8 != 0) return false;
    return true;
}

void launch_forward_slab_f16(const LayerShape &s, const void *coef, float *y, const void *records, float *partials,
                             hipStream_t stream)
{
    constexpr int kTileB = kWaves * 64;
    allow_large_lds(reinterpret_cast<const void *>(forward_slab_f16_kernel), 160 * 1024);
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
    const int tiles = a.n_btiles * a.n_jt;
    const int split = pair_split_count(tiles, a.K);
    a.n_split = split;
    a.pairs_per_split = (a.K + split - 1) / split;
    finish_split_setup(a, s, y, partials, stream);
    {
        KernelTiming timing(stream, kTimeForward);
        forward_slab_f16_kernel<<<tiles * split, kWaves * 64, (size_t)2 * s.nodes() * kRowBytesH, stream>>>(a);
    }
    if (a.y_part) launch_sum_partials(y, a.y_part, split - 1, (int64_t)s.batch * s.n_out, stream);
}

void launch_backward_input_slab_f16(const LayerShape &s, const GridTab &tab, const void *coef, const float *gy,
                                    int64_t gy_tile_stride, int64_t gy_row_stride, float *gx_scratch,
                                    const void *records, hipStream_t stream)
{
    constexpr int kTileB = kWaves * 64;
    void (*const kernel)(GradInArgs) = s.G == 16 ? backward_input_slab_f16_kernel<17> : backward_input_slab_f16_kernel<0>;
    allow_large_lds(reinterpret_cast<const void *>(kernel), 160 * 1024);
    const size_t n = (size_t)s.pairs() * (size_t)s.batch;
    GradInArgs a;
    a.P = coef;
    a.gy = gy;
    a.gy_tile_stride = gy_tile_stride;
    a.gy_row_stride = gy_row_stride;
    a.gx = gx_scratch;
    a.rec_node = static_cast<const int32_t *>(records);
    a.rec_u = reinterpret_cast<const float *>(a.rec_node + n);
    a.rec_v = a.rec_u + n;
    a.map = coef_map(s);
    a.tab = tab;
    a.B = s.batch;
    a.ld = scratch_row_stride(s.batch, kScratchPlain);
    a.n_in = s.n_in;
    a.n_out = s.n_out;
    a.K = s.pairs();
    a.W = s.G + 1;
    a.nodes = s.nodes();
    a.col_limit = s.layout == LMKAN_LAYOUT_PACKED ? s.out_tiles() * kTile : s.n_out;
    a.packed = s.layout == LMKAN_LAYOUT_PACKED;
    a.n_btiles = (int)((s.batch + kTileB - 1) / kTileB);
    a.n_jt = s.out_tiles();
    const int tiles = a.n_btiles * a.n_jt;
    int split = 1;
    while (tiles * split < 256 && a.K / (split * 2) >= 4) split *= 2;
    a.n_split = split;
    a.pairs_per_split = (a.K + split - 1) / split;
    const size_t lds = (((size_t)2 * s.nodes() * kRowBytesH + 15) & ~(size_t)15) + LMKAN_MAX_GRID * sizeof(float);
    KernelTiming timing(stream, kTimeGradInput);
    kernel<<<tiles * split, kWaves * 64, lds, stream>>>(a);
}

}  // namespace lmkan
