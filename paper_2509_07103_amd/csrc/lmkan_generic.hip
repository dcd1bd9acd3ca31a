// Generic lmKAN kernels: correct for every shape, storage type and layout.
// Lanes are outputs, so every coefficient access is a coalesced row segment
// read from (or atomically added to) global memory.
#include "lmkan_kernels.h"

namespace lmkan {

namespace {

constexpr int kTile = LMKAN_PACK_TILE;  // outputs per tile = lanes per wave
constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ void stage_grid(const GridTab &tab, float *s_node, float *s_invh)
{
    for (int i = threadIdx.x; i <= tab.G; i += blockDim.x) s_node[i] = tab.node[i];
    for (int i = threadIdx.x; i < tab.G; i += blockDim.x) s_invh[i] = tab.inv_h[i];
    __syncthreads();
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

__device__ __forceinline__ float bcast(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ int bcast(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }

// ---------------------------------------------------------------------------
// Forward (Alg. 1).  Block = 4 waves x 8 samples, one 64-wide output tile.
// Pairs are processed in chunks: the block first writes the preamble records of
// (32 samples x 16 pairs) to LDS, then every wave walks its samples.
// ---------------------------------------------------------------------------
constexpr int kFwdSamplesPerWave = 8;
constexpr int kFwdTileB = kWaves * kFwdSamplesPerWave;
constexpr int kFwdPairChunk = 16;

template <typename CT, bool CONV>
__global__ __launch_bounds__(kThreads) void forward_generic_kernel(GridTab tab, CoefMap map,
                                                                  const float *__restrict__ x,
                                                                  const CT *__restrict__ P,
                                                                  float *__restrict__ y, int64_t B,
                                                                  int n_in, int n_out, ConvGeom cg)
{
    __shared__ float s_node[LMKAN_MAX_GRID + 1];
    __shared__ float s_invh[LMKAN_MAX_GRID];
    __shared__ int s_rec_node[kFwdTileB][kFwdPairChunk];
    __shared__ float4 s_rec_w[kFwdTileB][kFwdPairChunk];
    stage_grid(tab, s_node, s_invh);

    const int G = tab.G, W = G + 1, K = n_in / 2;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t n0 = (int64_t)blockIdx.x * kFwdTileB;
    const int jt = blockIdx.y;
    const int j = jt * kTile + lane;
    const bool j_ok = j < n_out;
    const int64_t col = (int64_t)jt * map.s_tile + lane;
    const int64_t d_i2 = map.s_node, d_i1 = (int64_t)W * map.s_node;

    float acc[kFwdSamplesPerWave];
#pragma unroll
    for (int s = 0; s < kFwdSamplesPerWave; ++s) acc[s] = 0.0f;

    for (int k0 = 0; k0 < K; k0 += kFwdPairChunk) {
        __syncthreads();
        for (int r = threadIdx.x; r < kFwdTileB * kFwdPairChunk; r += kThreads) {
            const int s = r / kFwdPairChunk, kk = r % kFwdPairChunk;
            const int64_t n = n0 + s;
            int node = 0;
            float4 w = make_float4(0.f, 0.f, 0.f, 0.f);
            if (n < B && k0 + kk < K) {
                const float2 xv = load_input_pair<CONV>(x, n, n_in, k0 + kk, cg);
                const Preamble p = preamble(s_node, s_invh, G, xv.x, xv.y);
                node = p.node;
                w = make_float4(p.a_lo * p.b_lo, p.a_hi * p.b_lo, p.a_lo * p.b_hi, p.a_hi * p.b_hi);
            }
            s_rec_node[s][kk] = node;
            s_rec_w[s][kk] = w;
        }
        __syncthreads();
        const int kmax = min(kFwdPairChunk, K - k0);
        for (int kk = 0; kk < kmax; ++kk) {
#pragma unroll
            for (int s = 0; s < kFwdSamplesPerWave; ++s) {
                const int sw = wave * kFwdSamplesPerWave + s;
                const int node = s_rec_node[sw][kk];
                const float4 w = s_rec_w[sw][kk];
                if (j_ok) {
                    const CT *row = P + ((int64_t)node * map.s_node + (int64_t)(k0 + kk) * map.s_pair + col);
                    const float c00 = widen(row[0]);
                    const float c10 = widen(row[d_i1]);
                    const float c01 = widen(row[d_i2]);
                    const float c11 = widen(row[d_i1 + d_i2]);
                    acc[s] = fmaf(w.x, c00, acc[s]);
                    acc[s] = fmaf(w.y, c10, acc[s]);
                    acc[s] = fmaf(w.z, c01, acc[s]);
                    acc[s] = fmaf(w.w, c11, acc[s]);
                }
            }
        }
    }
    if (j_ok) {
#pragma unroll
        for (int s = 0; s < kFwdSamplesPerWave; ++s) {
            const int64_t n = n0 + wave * kFwdSamplesPerWave + s;
            if (n < B) y[n * n_out + j] = acc[s];
        }
    }
}

// ---------------------------------------------------------------------------
// Backward.  One wave per sample.  For a chunk of 64 pairs lane l computes the
// preamble of pair k0+l; the records are then broadcast one pair at a time while
// the lanes sweep the outputs.
//   grad_x : s_ab = sum_j gy[j] P[corner ab][j] (wave reduction), then
//            d/dx1 = (1/h1) ((s10-s00) b_lo + (s11-s01) b_hi), d/dx2 alike.
//   grad_P : gP[corner ab][j] += w_ab gy[j]  with float32 atomics.
// ---------------------------------------------------------------------------
template <typename CT, bool DO_GX, bool DO_GP, bool CONV>
__global__ __launch_bounds__(kThreads) void backward_generic_kernel(
    GridTab tab, CoefMap map, CoefMap gmap, const float *__restrict__ x, const CT *__restrict__ P,
    const float *__restrict__ gy, float *__restrict__ gx, float *__restrict__ gP, int64_t B, int n_in,
    int n_out, ConvGeom cg)
{
    __shared__ float s_node[LMKAN_MAX_GRID + 1];
    __shared__ float s_invh[LMKAN_MAX_GRID];
    stage_grid(tab, s_node, s_invh);

    const int G = tab.G, W = G + 1, K = n_in / 2;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t n = (int64_t)blockIdx.x * kWaves + wave;
    if (n >= B) return;  // whole wave leaves together; no block-wide barrier follows
    const float *gyr = gy + n * n_out;
    const int tiles = (n_out + kTile - 1) / kTile;
    const int64_t d_i2 = map.s_node, d_i1 = (int64_t)W * map.s_node;
    const int64_t g_i2 = gmap.s_node, g_i1 = (int64_t)W * gmap.s_node;

    for (int k0 = 0; k0 < K; k0 += 64) {
        Preamble mine;
        mine.node = 0;
        mine.a_lo = mine.a_hi = mine.b_lo = mine.b_hi = mine.rh1 = mine.rh2 = 0.0f;
        if (k0 + lane < K) {
            const float2 xv = load_input_pair<CONV>(x, n, n_in, k0 + lane, cg);
            mine = preamble(s_node, s_invh, G, xv.x, xv.y);
        }
        float my_d1 = 0.0f, my_d2 = 0.0f;
        const int kmax = min(64, K - k0);
        for (int kk = 0; kk < kmax; ++kk) {
            const int node = bcast(mine.node, kk);
            const float a_lo = bcast(mine.a_lo, kk), a_hi = bcast(mine.a_hi, kk);
            const float b_lo = bcast(mine.b_lo, kk), b_hi = bcast(mine.b_hi, kk);
            float s00 = 0.f, s10 = 0.f, s01 = 0.f, s11 = 0.f;
            for (int jt = 0; jt < tiles; ++jt) {
                const int j = jt * kTile + lane;
                if (j < n_out) {
                    const float g = gyr[j];
                    if (DO_GX) {
                        const CT *row = P + ((int64_t)node * map.s_node +
                                             (int64_t)(k0 + kk) * map.s_pair + (int64_t)jt * map.s_tile + lane);
                        s00 = fmaf(g, widen(row[0]), s00);
                        s10 = fmaf(g, widen(row[d_i1]), s10);
                        s01 = fmaf(g, widen(row[d_i2]), s01);
                        s11 = fmaf(g, widen(row[d_i1 + d_i2]), s11);
                    }
                    if (DO_GP) {
                        float *grow = gP + ((int64_t)node * gmap.s_node +
                                            (int64_t)(k0 + kk) * gmap.s_pair + (int64_t)jt * gmap.s_tile + lane);
                        unsafeAtomicAdd(grow, a_lo * b_lo * g);
                        unsafeAtomicAdd(grow + g_i1, a_hi * b_lo * g);
                        unsafeAtomicAdd(grow + g_i2, a_lo * b_hi * g);
                        unsafeAtomicAdd(grow + g_i1 + g_i2, a_hi * b_hi * g);
                    }
                }
            }
            if (DO_GX) {
                s00 = wave_sum(s00);
                s10 = wave_sum(s10);
                s01 = wave_sum(s01);
                s11 = wave_sum(s11);
                if (lane == kk) {
                    my_d1 = mine.rh1 * ((s10 - s00) * mine.b_lo + (s11 - s01) * mine.b_hi);
                    my_d2 = mine.rh2 * ((s01 - s00) * mine.a_lo + (s11 - s10) * mine.a_hi);
                }
            }
        }
        if (DO_GX && k0 + lane < K) {
            if constexpr (CONV) {
                // windows may overlap: an image element collects from every window that holds it
                atomicAdd(gx + conv_input_offset(cg, n, 2 * (k0 + lane)), my_d1);
                atomicAdd(gx + conv_input_offset(cg, n, 2 * (k0 + lane) + 1), my_d2);
            } else {
                *reinterpret_cast<float2 *>(gx + n * n_in + 2 * (k0 + lane)) = make_float2(my_d1, my_d2);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Cell lookup alone, packing, zero fill
// ---------------------------------------------------------------------------
template <bool PAIRED>  // PAIRED: x is 8-byte aligned, the two inputs of a pair are read at once
__global__ __launch_bounds__(kThreads) void locate_kernel(GridTab tab, const float *__restrict__ x,
                                                         int32_t *__restrict__ cell, int64_t total,
                                                         int K)
{
    __shared__ float s_node[LMKAN_MAX_GRID + 1];
    __shared__ float s_invh[LMKAN_MAX_GRID];
    stage_grid(tab, s_node, s_invh);
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < total; r += stride) {
        float2 xv;  // x[n][2k], x[n][2k+1]
        if constexpr (PAIRED)
            xv = reinterpret_cast<const float2 *>(x)[r];
        else
            xv = make_float2(x[2 * r], x[2 * r + 1]);
        cell[r] = locate(s_node, tab.G, xv.x) * tab.G + locate(s_node, tab.G, xv.y);
    }
    (void)K;
}

template <typename U>
__global__ __launch_bounds__(kThreads) void pack_kernel(const U *__restrict__ src, U *__restrict__ dst,
                                                       int K, int n_out, int nodes, int64_t total)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t d = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; d < total; d += stride) {
        const int jl = (int)(d % kTile);
        int64_t r = d / kTile;
        const int node = (int)(r % nodes);
        r /= nodes;
        const int k = (int)(r % K);
        const int jt = (int)(r / K);
        const int j = jt * kTile + jl;
        dst[d] = j < n_out ? src[((int64_t)node * K + k) * n_out + j] : (U)0;
    }
}

__global__ __launch_bounds__(kThreads) void fill_zero_kernel(float *__restrict__ p, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0.0f;
}

int blocks_for(int64_t work_items, int per_block, int cap)
{
    int64_t b = (work_items + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return (int)b;
}

}  // namespace

CoefMap coef_map(const LayerShape &s)
{
    CoefMap m;
    if (s.layout == LMKAN_LAYOUT_PACKED) {
        m.s_node = kTile;
        m.s_pair = (int64_t)s.nodes() * kTile;
        m.s_tile = (int64_t)s.pairs() * s.nodes() * kTile;
    } else {
        m.s_node = (int64_t)s.pairs() * s.n_out;
        m.s_pair = s.n_out;
        m.s_tile = kTile;
    }
    return m;
}

template <typename CT>
static void forward_generic_dispatch(const LayerShape &s, const GridTab &tab, const float *x, const CT *coef,
                                     float *y, hipStream_t stream, const ConvGeom *conv)
{
    const dim3 grid((unsigned)((s.batch + kFwdTileB - 1) / kFwdTileB), (unsigned)s.out_tiles());
    const CoefMap map = coef_map(s);
    KernelTiming timing(stream, kTimeForward);
    if (conv)
        forward_generic_kernel<CT, true><<<grid, kThreads, 0, stream>>>(tab, map, x, coef, y, s.batch, s.n_in,
                                                                        s.n_out, *conv);
    else
        forward_generic_kernel<CT, false><<<grid, kThreads, 0, stream>>>(tab, map, x, coef, y, s.batch, s.n_in,
                                                                         s.n_out, ConvGeom{});
}

void launch_forward_generic(const LayerShape &s, const GridTab &tab, const float *x, const void *coef,
                            float *y, hipStream_t stream, const ConvGeom *conv)
{
    switch (s.dtype) {
    case LMKAN_F32: forward_generic_dispatch(s, tab, x, static_cast<const float *>(coef), y, stream, conv); break;
    case LMKAN_F16: forward_generic_dispatch(s, tab, x, static_cast<const _Float16 *>(coef), y, stream, conv); break;
    default: forward_generic_dispatch(s, tab, x, static_cast<const bf16_t *>(coef), y, stream, conv); break;
    }
}

template <typename CT, bool CONV>
static void backward_generic_dispatch(const LayerShape &s, const GridTab &tab, const float *x,
                                      const CT *coef, const float *gy, float *gx, float *gcoef,
                                      hipStream_t stream, const ConvGeom &cg)
{
    const dim3 grid((unsigned)((s.batch + kWaves - 1) / kWaves));
    const CoefMap map = coef_map(s);
    LayerShape g = s;
    g.layout = LMKAN_LAYOUT_PAPER;  // the gradient is always in the layout of Alg. 1
    const CoefMap gmap = coef_map(g);
    KernelTiming timing(stream, gx ? kTimeGradInput : kTimeGradCoef);
    if (gx && gcoef)
        backward_generic_kernel<CT, true, true, CONV><<<grid, kThreads, 0, stream>>>(
            tab, map, gmap, x, coef, gy, gx, gcoef, s.batch, s.n_in, s.n_out, cg);
    else if (gx)
        backward_generic_kernel<CT, true, false, CONV><<<grid, kThreads, 0, stream>>>(
            tab, map, gmap, x, coef, gy, gx, gcoef, s.batch, s.n_in, s.n_out, cg);
    else if (gcoef)
        backward_generic_kernel<CT, false, true, CONV><<<grid, kThreads, 0, stream>>>(
            tab, map, gmap, x, coef, gy, gx, gcoef, s.batch, s.n_in, s.n_out, cg);
}

template <typename CT>
static void backward_generic_conv_or_rows(const LayerShape &s, const GridTab &tab, const float *x, const CT *coef,
                                          const float *gy, float *gx, float *gcoef, hipStream_t stream,
                                          const ConvGeom *conv)
{
    if (conv)
        backward_generic_dispatch<CT, true>(s, tab, x, coef, gy, gx, gcoef, stream, *conv);
    else
        backward_generic_dispatch<CT, false>(s, tab, x, coef, gy, gx, gcoef, stream, ConvGeom{});
}

void launch_backward_generic(const LayerShape &s, const GridTab &tab, const float *x,
                             const void *coef, const float *gy, float *gx, float *gcoef,
                             hipStream_t stream, const ConvGeom *conv)
{
    switch (s.dtype) {
    case LMKAN_F32:
        backward_generic_conv_or_rows(s, tab, x, static_cast<const float *>(coef), gy, gx, gcoef, stream, conv);
        break;
    case LMKAN_F16:
        backward_generic_conv_or_rows(s, tab, x, static_cast<const _Float16 *>(coef), gy, gx, gcoef, stream, conv);
        break;
    default:
        backward_generic_conv_or_rows(s, tab, x, static_cast<const bf16_t *>(coef), gy, gx, gcoef, stream, conv);
        break;
    }
}

void launch_locate(const LayerShape &s, const GridTab &tab, const float *x, int32_t *cell,
                   hipStream_t stream)
{
    const int64_t total = s.batch * s.pairs();
    if ((reinterpret_cast<uintptr_t>(x) & 7) == 0)
        locate_kernel<true><<<blocks_for(total, kThreads, 65536), kThreads, 0, stream>>>(tab, x, cell, total, s.pairs());
    else
        locate_kernel<false><<<blocks_for(total, kThreads, 65536), kThreads, 0, stream>>>(tab, x, cell, total, s.pairs());
}

void launch_pack(const LayerShape &s, const void *src, void *dst, hipStream_t stream)
{
    const int64_t total = (int64_t)s.out_tiles() * s.pairs() * s.nodes() * kTile;
    const int blocks = blocks_for(total, kThreads, 1 << 20);
    if (s.dtype == LMKAN_F32)
        pack_kernel<uint32_t><<<blocks, kThreads, 0, stream>>>(static_cast<const uint32_t *>(src),
                                                              static_cast<uint32_t *>(dst), s.pairs(),
                                                              s.n_out, s.nodes(), total);
    else
        pack_kernel<uint16_t><<<blocks, kThreads, 0, stream>>>(static_cast<const uint16_t *>(src),
                                                              static_cast<uint16_t *>(dst), s.pairs(),
                                                              s.n_out, s.nodes(), total);
}

void launch_fill_zero(float *p, size_t n, hipStream_t stream)
{
    fill_zero_kernel<<<blocks_for((int64_t)n, kThreads * 8, 1 << 16), kThreads, 0, stream>>>(p, n);
}

}  // namespace lmkan
