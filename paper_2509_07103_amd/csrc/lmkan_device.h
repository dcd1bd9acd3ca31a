// Device-side pieces shared by every lmKAN kernel: the grid table, the cell
// lookup and the four weights of Alg. 1's preamble, and coefficient decoding.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <utility>

#include "lmkan.h"

namespace lmkan {

// Extended grid (Sec. 3.1, App. B "Edge cases") as float32, passed to kernels by value.
// node[1..G-1] are the real grid points, node[0] / node[G] the ghost points;
// inv_h[i] = 1 / (node[i+1] - node[i]).
struct GridTab {
    float node[LMKAN_MAX_GRID + 1];
    float inv_h[LMKAN_MAX_GRID];
    int G;
};

// Convolution as a fully connected layer on windows (Sec. 5, "lmKAN-based Convolutional Neural
// Networks"): channels-last image x[N][H][W][C], kh x kw window, no padding; row r of the layer =
// output pixel (img, oy, ox), r = (img OH + oy) OW + ox; input e = (ky kw + kx) C + c of that row is
// x[img][oy stride + ky][ox stride + kx][c].  The patches are never written out: every kernel that
// reads x goes through this map.  C == 0 stands for a plain layer on rows x[n][n_in].
struct ConvGeom {
    int N, H, W, C, kh, kw, stride, OH, OW;
};

// offset, in elements, of input e of row n
__host__ __device__ inline int64_t conv_input_offset(const ConvGeom &cg, int64_t n, int e)
{
    const int c = e % cg.C, kx = (e / cg.C) % cg.kw, ky = e / (cg.C * cg.kw);
    const int ox = (int)(n % cg.OW), oy = (int)((n / cg.OW) % cg.OH);
    const int64_t img = n / ((int64_t)cg.OW * cg.OH);
    return ((img * cg.H + (oy * cg.stride + ky)) * cg.W + (ox * cg.stride + kx)) * cg.C + c;
}

// the two inputs of pair k of row n (with an odd channel count they can sit in two pixels)
template <bool CONV>
__device__ inline float2 load_input_pair(const float *__restrict__ x, int64_t n, int n_in, int k, const ConvGeom &cg)
{
    if constexpr (!CONV) {
        return *reinterpret_cast<const float2 *>(x + n * n_in + 2 * k);
    } else {
        const int64_t o0 = conv_input_offset(cg, n, 2 * k);
        const int64_t o1 = (cg.C & 1) ? conv_input_offset(cg, n, 2 * k + 1) : o0 + 1;
        return make_float2(x[o0], x[o1]);
    }
}

// Where coefficient (node, pair k, output tile jt, column jl) lives, in elements:
//   node * s_node + k * s_pair + jt * s_tile + jl,
// and moving one node along the second axis adds s_node, along the first (G+1) * s_node.
// Covers both the layout of Alg. 1 and the packed layout.
struct CoefMap {
    int64_t s_node;
    int64_t s_pair;
    int64_t s_tile;
};

// One record per (sample, pair): Alg. 1's preamble output.
struct Preamble {
    int node;    // i1 * (G+1) + i2 : table node of the cell's lower-left corner
    int cell;    // i1 * G + i2
    float a_lo;  // (node[i1+1] - x1) / h1 : factor of B_{i1}
    float a_hi;  // (x1 - node[i1]) / h1   : factor of B_{i1+1}
    float b_lo;  // same along the second axis
    float b_hi;
    float rh1;   // 1 / h1, 1 / h2 : needed by the input gradient
    float rh2;
};

// App. B Eq. 5 the way Alg. 2 evaluates it: one exponential of -|x|.
__device__ __forceinline__ float sigma(float x)
{
    float t = __expf(-fabsf(x));
    return x > 0.0f ? 1.0f - 0.5f * t : 0.5f * t;
}

// Cell index.  The candidate floor(sigma(x) G) of Sec. 3.1 is corrected against the
// float32 grid table so that the result is exactly "number of real grid points <= x"
// whatever the accuracy of the exponential.  node points to LDS or kernel arguments.
__device__ __forceinline__ int locate(const float *node, int G, float x)
{
    int i = (int)(sigma(x) * (float)G);
    i = min(max(i, 0), G - 1);
    while (i > 0 && x < node[i]) --i;
    while (i < G - 1 && x >= node[i + 1]) ++i;
    return i;
}

__device__ __forceinline__ Preamble preamble(const float *node, const float *inv_h, int G, float x1,
                                             float x2)
{
    Preamble r;
    int i1 = locate(node, G, x1);
    int i2 = locate(node, G, x2);
    r.node = i1 * (G + 1) + i2;
    r.cell = i1 * G + i2;
    r.rh1 = inv_h[i1];
    r.rh2 = inv_h[i2];
    r.a_lo = (node[i1 + 1] - x1) * r.rh1;
    r.a_hi = (x1 - node[i1]) * r.rh1;
    r.b_lo = (node[i2 + 1] - x2) * r.rh2;
    r.b_hi = (x2 - node[i2]) * r.rh2;
    return r;
}

// Stored coefficient -> float32.
__device__ __forceinline__ float widen(float v) { return v; }
__device__ __forceinline__ float widen(_Float16 v) { return (float)v; }
struct bf16_t {
    uint16_t bits;
};
__device__ __forceinline__ float widen(bf16_t v) { return __uint_as_float((uint32_t)v.bits << 16); }

// ---------------------------------------------------------------------------
// DPP helpers.  row_newbcast:S makes every lane of a 16-lane row read lane S of
// that row.
// ---------------------------------------------------------------------------
template <int S>
__device__ __forceinline__ int row_bcast(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, 0x150 + S, 0xf, 0xf, true);
}

// acc += (w of lane S of this row) * c
template <int S>
__device__ __forceinline__ void fmac_row_bcast(float &acc, float w, float c)
{
    asm("v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
        : "+v"(acc)
        : "v"(w), "v"(c), "n"(S));
}

template <int... Ts, class F>
__device__ __forceinline__ void static_for(std::integer_sequence<int, Ts...>, F &&f)
{
    (f(std::integral_constant<int, Ts>{}), ...);
}

}  // namespace lmkan
