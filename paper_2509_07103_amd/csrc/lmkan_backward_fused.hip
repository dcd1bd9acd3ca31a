// Input gradient, alone or together with the coefficient gradient, from the cell-sorted stream.
//
//   s_c(n,k)  = sum_j gy[n][j] P[corner c of the cell of (n,k)][k][j]
//   d/dx1     = (1/h1) ((s10 - s00)(1 - v) + (s11 - s01) v)
//   d/dx2     = (1/h2) ((s01 - s00)(1 - u) + (s11 - s10) u)        (derivative of Alg. 1's sum)
//   gP[corner][k][j] += B_corner(x_n) gy[n][j]
//
// For the samples of one cell both are small dense contractions that share one operand, the
// gy rows of those samples: s = GY P_cell^T (long in j) and gP_cell = W^T GY (long in the
// samples).  One wave owns (pair k, 64 outputs) and walks the sorted chunks of four samples;
// every gy row piece it gathers (256 bytes, the expensive part: it comes from all over the
// batch through L2) feeds eight 4x4x1 float32 MFMAs, four for each gradient.
//
// Coefficient gradient: as in lmkan_backward.hip (the four samples of a chunk in the four
// 16-lane groups, block-broadcast products, two-row window of the table in LDS).
//
// Input gradient: the MFMA wants the four samples of a chunk in the four lanes of a block,
// which is not how a coalesced load leaves them, so the rows of four chunks go through LDS
// (written as loaded, 16 bytes per lane, read back 16 bytes per lane in the other order; LDS
// reads cost no vector-ALU issue slot).  Block (q, o) of an MFMA then holds chunk q and the
// o-th quarter of the 64 outputs: B = gy of the chunk's four samples at one output, A = the
// four corner coefficients of the chunk's cell at that output (the 4 x 64 corner rows of a
// cell are staged in LDS once per cell), D[corner][sample] accumulates over the 16 outputs of
// the quarter; two row rotations add the four quarters.  The weights of the two derivatives
// are applied per lane, and the two sums of a sample over this tile's 64 outputs go to
// partial[tile][k][position in the stream]: consecutive lanes, consecutive addresses.
// gx_combine_kernel adds the tiles in a fixed order, multiplies by 1/h and writes grad_x.
// No atomics and no zero fill on this path: grad_x is the same in every run.
#include <type_traits>

#include "lmkan_kernels.h"
#include "lmkan_slab_common.h"
#include "lmkan_sorted.h"

namespace lmkan {

namespace {

constexpr int kTile = LMKAN_PACK_TILE;
constexpr int kDepth = 8;                    // chunks of gy in flight
constexpr int kCellDepth = 8;                // chunks ahead at which the rows of a new cell are requested
constexpr int kGroup = 4;                    // chunks per MFMA group of the input gradient
constexpr int kGroups = kUnroll / kGroup;    // groups per trip
constexpr int kStageBytes = kGroup * 1024;   // gy rows of one group in LDS
constexpr int kCellSlots = 5;                // coefficient rows of the cells a group can touch (4 new + 1 carried over)
constexpr int kFusedLdsFixed = kStageBytes + kCellSlots * 1024;
static_assert(kUnroll % kDepth == 0 && kDepth % kGroup == 0 && kUnroll % kCellDepth == 0, "rings must divide the trip");

struct FusedArgs {
    const f4v *rec;
    const int32_t *chunk_cell;
    const int32_t *block_start;
    GyView gy;
    const void *P;
    float *gP;        // NULL: input gradient only
    float2 *partial;  // [tiles][K][S]
    CoefMap pmap;     // layout of P
    CoefMap gmap;     // layout of Alg. 1 (gP)
    int64_t B;
    int64_t S;
    int n_out;
    int K;
    int G;
    int accumulate;
    int n_blocks;
    int n_sub;
    int col_limit;    // columns >= col_limit do not exist in P
};

// Four adjacent coefficients of a row as they are stored, and their float32 values.  The two are
// kept apart on purpose: a row is requested several chunks before its cell begins, and a
// conversion written next to the load would wait for the load right there.
template <typename CT>
struct CoefRow {
    typedef typename std::conditional<sizeof(CT) == 4, f4v, uint2>::type raw;
};

template <typename CT>
__device__ __forceinline__ typename CoefRow<CT>::raw load_coef4(const CT *p)
{
    return *reinterpret_cast<const typename CoefRow<CT>::raw *>(p);
}

template <typename CT>
__device__ __forceinline__ f4v widen_coef4(const typename CoefRow<CT>::raw &v)
{
    if constexpr (sizeof(CT) == 4) {
        return v;
    } else if constexpr (std::is_same<CT, _Float16>::value) {
        typedef _Float16 h2v __attribute__((ext_vector_type(2)));
        const h2v lo = __builtin_bit_cast(h2v, v.x), hi = __builtin_bit_cast(h2v, v.y);
        return f4v{(float)lo.x, (float)lo.y, (float)hi.x, (float)hi.y};
    } else {
        return f4v{__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u), __uint_as_float(v.y << 16),
                   __uint_as_float(v.y & 0xffff0000u)};
    }
}

template <typename CT, bool DO_GP, bool kOffset32, bool RAGGED>
__global__ __launch_bounds__(64) void backward_fused_kernel(FusedArgs a)
{
    // [gy rows of the four chunks of a group][coefficient rows of up to kCellSlots cells][gP window: 2 table rows]
    extern __shared__ __align__(16) float smem[];
    char *lds = reinterpret_cast<char *>(smem);
    float *win = smem + kFusedLdsFixed / 4;
    const int lane = threadIdx.x;
    const int g = lane >> 4, l16 = lane & 15;              // as loaded: row g of a load, 16-byte piece l16
    const int q = lane >> 4, og = (lane >> 2) & 3, j = lane & 3;  // as multiplied: chunk, output quarter, sample / corner
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
    if (nch == 0) return;
    ScalarIntPtr cc = (ScalarIntPtr)(a.chunk_cell + (int64_t)k * (a.S / kChunk) + c_begin);

    // Stream entries in two lane orders, one load per group of four chunks each:
    //   for the products and the gy addresses, lane (g, 4 j' + q') takes the entry of sample g of
    //   chunk j' (and forms product q' of it);
    //   for the weights of the input gradient, lane (q, o, j) takes (u, v) of sample j of chunk q.
    const f4v *rec_k = a.rec + (int64_t)k * a.S + (int64_t)c_begin * kChunk;
    const f4v *e_ptr = rec_k + (l16 >> 2) * kChunk + g;
    auto load_e = [&](int chunk) { return e_ptr[(int64_t)chunk * kChunk]; };

    const unsigned col_bytes = col_ok ? (unsigned)l16 * 16u : 0u;
    const unsigned row_bytes = a.gy.row_stride;
    const char *gy_tile = reinterpret_cast<const char *>(a.gy.base) + (int64_t)jt * a.gy.tile_stride;
    // gy row piece of sample g of the chunk whose row offset sits in lane (g, 4 SUB) of off16
    // (the byte offset of the sample's row when it fits 32 bits, else the sample index)
    auto row_offset = [&](int n) { return kOffset32 ? (int)__umul24((unsigned)n, row_bytes) : n; };
    auto load_gy = [&](auto subc, int off16) {
        constexpr int SUB = decltype(subc)::value;
        if constexpr (kOffset32) {
            // one instruction: (offset of lane 4 SUB of this row) + this lane's column bytes
            const unsigned off = (unsigned)__builtin_amdgcn_update_dpp(0, off16, 0x150 + 4 * SUB, 0xf, 0xf, true) + col_bytes;
            return *reinterpret_cast<const f4v *>(gy_tile + off);
        } else {
            const int n = row_bcast<4 * SUB>(off16);
            return *reinterpret_cast<const f4v *>(gy_tile + ((int64_t)n * row_bytes + col_bytes));
        }
    };
    // Rows of a cell as the input gradient wants them: the derivative along the first axis pairs
    // corner (i1+1, .) with (i1, .), the one along the second axis (., i2+1) with (., i2), and
    // taking the differences of the coefficients before the sum over j keeps neighbouring
    // coefficients of a smooth table from cancelling inside a long float32 sum:
    //   d0 = P10 - P00, d1 = P11 - P01, d2 = P01 - P00, d3 = P11 - P10   (corner c = (c & 1, c >> 1))
    // lane (r, l16) loads 4 outputs of both rows of difference r; the subtraction happens when
    // the rows are staged in LDS.  Columns the table does not have count as zero.
    const bool pcol_ok = col < a.col_limit;
    const int ca = g == 0 ? 1 : g == 2 ? 2 : 3, cb = g == 0 ? 0 : g == 1 ? 2 : g == 2 ? 0 : 1;
    const CT *p_tile = static_cast<const CT *>(a.P) + (int64_t)k * a.pmap.s_pair + (int64_t)jt * a.pmap.s_tile +
                       (pcol_ok ? l16 * 4 : 0);
    const CT *pa_lane = p_tile + (int64_t)((ca & 1) * W + (ca >> 1)) * a.pmap.s_node;
    const CT *pb_lane = p_tile + (int64_t)((cb & 1) * W + (cb >> 1)) * a.pmap.s_node;
    auto corner_offset = [&](int cell) { return (int64_t)((cell >> 8) * W + (cell & 255)) * a.pmap.s_node; };

    // LDS byte offsets.  Rows are 256 bytes; the 16-byte pieces of a row are rotated by the row's
    // number so that both the writes (16 lanes: one row, 16 pieces) and the reads (16 lanes: 4
    // rows, 4 pieces 4 apart) touch every bank once.  The coefficient rows of a cell sit in one of
    // kCellSlots slots after the gy rows, in the same arrangement.
    const int wr_off = g * 256 + ((l16 + g) & 15) * 16;  // + chunk-in-group * 1024 (gy) or slot * 1024 (coefficients)
    int rd_off[4];                                       // piece 4 og + t of row j; + q * 1024 (gy) or slot * 1024
    const char *gy_rd[4];                                // the same for the gy rows of chunk q
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        rd_off[t] = j * 256 + ((4 * og + t + j) & 15) * 16;
        gy_rd[t] = lds + q * 1024 + rd_off[t];
    }

    float *out = DO_GP ? a.gP + (int64_t)k * a.gmap.s_pair + col : nullptr;
    if constexpr (DO_GP)
        for (int i = lane; i < 2 * W * kTile; i += 64) win[i] = 0.0f;

    f4v acc[4];  // coefficient gradient of the current cell: [output i of the lane][corner]
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = f4v{0.f, 0.f, 0.f, 0.f};
    int cur_cell = -1;  // (i1 << 8 | i2) of the cell being accumulated
    int rows_done = 0;  // gP table rows [0, rows_done) have been written out
    int cur_slot = 0;    // LDS slot of the current cell's coefficient rows
    unsigned slots = 0;  // slot of each chunk of the current group, one byte each

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
    const int out_col = jt * kTile + lane;
    float *out_lane = DO_GP ? a.gP + (int64_t)k * a.gmap.s_pair + out_col : nullptr;
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

    // lane (q, og, j) keeps the result of sample j of chunk q of group og of a trip; one store per trip
    float2 *part = a.partial + ((int64_t)jt * a.K + k) * a.S + (int64_t)c_begin * kChunk + ((og * kGroup + q) * kChunk + j);
    // where that sample's (u, v) sit in the entries as loaded: lane (g = j, 4 q)
    const int uv_src = (16 * j + 4 * q) * 4;
    // Lines of the table a few cells ahead of the walk, touched once per trip so that the rows of
    // coming cells are in L2 when they are asked for.  Vector memory operations of a wave return
    // in order: one load that has to go to HBM holds back every gy piece requested after it, so
    // everything that streams from HBM is requested in one burst at the top of a trip.
    const int touch_row = (lane >= 16 ? W : 0) + 4 + ((lane & 15) >> 1);
    // (two touches per row: its first column and its middle one, where the table has that column)
    const int touch_col = (lane & 1) != 0 && jt * kTile + kTile / 2 < a.col_limit ? kTile / 2 : 0;
    const char *touch_base = reinterpret_cast<const char *>(static_cast<const CT *>(a.P) + (int64_t)k * a.pmap.s_pair +
                                                            (int64_t)jt * a.pmap.s_tile + touch_col);
    const int last_node = W * W - 1;
    auto touch_ahead = [&](int cell) {
        int v = 0;
        if (lane < 32) {
            const int r = min((cell >> 8) * W + (cell & 255) + touch_row, last_node);
            v = *reinterpret_cast<const int *>(touch_base + (int64_t)r * a.pmap.s_node * (int64_t)sizeof(CT));
        }
        return v;
    };

    // Per group of four chunks: products (coefficient gradient) and sample indices in the first
    // lane order, (u, v) in the second.  "now" belongs to the trip being consumed, "nxt" to the
    // next one: its entries are requested at the top of a trip and unpacked half a trip later,
    // just before the gy loads issued kDepth chunks ahead need its sample indices.
    float prod_now[kGroups], prod_nxt[kGroups];
    int n_now[kGroups], n_nxt[kGroups];
    float2 uv_now[kGroups], uv_nxt[kGroups];
    f4v raw[kGroups];
    float2 res = make_float2(0.f, 0.f);  // results of this lane's sample of the trip
    int touched = 0;
    f4v gq[kDepth];         // gy row pieces
    typename CoefRow<CT>::raw pqa[kCellDepth];  // both rows of this lane's coefficient difference, as stored,
    typename CoefRow<CT>::raw pqb[kCellDepth];  // for the chunks that start a cell

    auto unpack = [&](const f4v &e, float &prod, int &n, float2 &uv) {
        prod = DO_GP ? entry_product(e, l16 & 3) : 0.f;
        n = row_offset(__float_as_int(e.w));
        // (u, v) into the lane order of the multiplications, through the LDS crossbar
        uv.x = __int_as_float(__builtin_amdgcn_ds_bpermute(uv_src, __float_as_int(e.x)));
        uv.y = __int_as_float(__builtin_amdgcn_ds_bpermute(uv_src, __float_as_int(e.y)));
    };

    int cells_now[kUnroll], cells_nxt[kUnroll];
#pragma unroll
    for (int p = 0; p < kUnroll; ++p) cells_now[p] = cc[p];
    if (DO_GP && split) rows_done = cells_now[0] >> 8;  // rows before the run's first cell are not this wave's

    // prologue: entries of trip 0, gy of the first kDepth chunks, coefficient rows of the first kCellDepth
#pragma unroll
    for (int r = 0; r < kGroups; ++r) unpack(load_e(r * kGroup), prod_now[r], n_now[r], uv_now[r]);
    static_for(std::make_integer_sequence<int, kDepth>{}, [&](auto dc) {
        constexpr int d = decltype(dc)::value;
        gq[d] = load_gy(std::integral_constant<int, d % kGroup>{}, n_now[d / kGroup]);
        if constexpr (d < kCellDepth) {
            if (d == 0 || cells_now[d] != cells_now[d > 0 ? d - 1 : 0]) {
                const int64_t off = corner_offset(cells_now[d]);
                pqa[d] = load_coef4<CT>(pa_lane + off);
                pqb[d] = load_coef4<CT>(pb_lane + off);
            }
        }
    });

    for (int c = 0; c < nch; c += kUnroll) {
#pragma unroll
        for (int p = 0; p < kUnroll; ++p) cells_nxt[p] = cc[c + kUnroll + p];
        // the burst: entries of the next trip, table lines ahead of the walk (the value loaded a
        // trip ago only has to have arrived), results of the trip before
        asm volatile("" ::"v"(touched));
#pragma unroll
        for (int r = 0; r < kGroups; ++r) raw[r] = load_e(c + kUnroll + r * kGroup);
        touched = touch_ahead(cells_now[0]);
        if (c > 0) part[(int64_t)(c - kUnroll) * kChunk] = res;
        static_for(std::make_integer_sequence<int, kUnroll>{}, [&](auto pc) {
            constexpr int P = decltype(pc)::value;
            constexpr int R = P / kGroup, SUB = P % kGroup;
            if constexpr (P == kUnroll - kDepth - 1) {
#pragma unroll
                for (int r = 0; r < kGroups; ++r) unpack(raw[r], prod_nxt[r], n_nxt[r], uv_nxt[r]);
            }
            const int cell_cur = cells_now[P];
            const bool changed = cell_cur != cur_cell;
            if (changed) {
                if constexpr (DO_GP) {
                    if (cur_cell >= 0) flush();
                    retire_rows(cell_cur >> 8);
                }
                cur_cell = cell_cur;
                cur_slot = cur_slot + 1 == kCellSlots ? 0 : cur_slot + 1;
                f4v d = widen_coef4<CT>(pqa[P % kCellDepth]) - widen_coef4<CT>(pqb[P % kCellDepth]);
                if (RAGGED && !pcol_ok) d = f4v{0.f, 0.f, 0.f, 0.f};
                *reinterpret_cast<f4v *>(lds + kStageBytes + cur_slot * 1024 + wr_off) = d;
                // this chunk and the rest of its group take the new slot
                constexpr unsigned kept = SUB == 0 ? 0u : (1u << (8 * SUB)) - 1u;
                slots = (slots & kept) | (((unsigned)cur_slot * 0x01010101u) & ~kept);
            }
            if constexpr (DO_GP) {
                if (changed)
                    chunk_fma<SUB, true>(acc, prod_now[R], gq[P % kDepth]);
                else
                    chunk_fma<SUB, false>(acc, prod_now[R], gq[P % kDepth]);
            }
            *reinterpret_cast<f4v *>(lds + SUB * 1024 + wr_off) = gq[P % kDepth];
            // refill the ring slots just consumed: gy of chunk c + P + kDepth, rows of the cell that
            // chunk c + P + kCellDepth starts
            {
                constexpr int PN = (P + kDepth) % kUnroll;
                const int n16 = P + kDepth < kUnroll ? n_now[PN / kGroup] : n_nxt[PN / kGroup];
                gq[P % kDepth] = load_gy(std::integral_constant<int, PN % kGroup>{}, n16);
                constexpr int PC = (P + kCellDepth) % kUnroll, PB = (P + kCellDepth - 1) % kUnroll;
                const int cell_new = P + kCellDepth < kUnroll ? cells_now[PC] : cells_nxt[PC];
                const int cell_before = P + kCellDepth - 1 < kUnroll ? cells_now[PB] : cells_nxt[PB];
                if (cell_new != cell_before) {
                    const int64_t off = corner_offset(cell_new);
                    pqa[P % kCellDepth] = load_coef4<CT>(pa_lane + off);
                    pqb[P % kCellDepth] = load_coef4<CT>(pb_lane + off);
                }
            }
            if constexpr (SUB == kGroup - 1) {
                // the four chunks of group R are in LDS: 16 MFMAs, block (q, og) = chunk q, outputs
                // 16 og .. 16 og + 15, then the sum over og and the weights
                const int a_base = kStageBytes + (int)((slots >> (8 * q)) & 0xffu) * 1024;
                f4v bv[4], av[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    bv[t] = *reinterpret_cast<const f4v *>(gy_rd[t]);
                    av[t] = *reinterpret_cast<const f4v *>(lds + a_base + rd_off[t]);
                }
                // two accumulators, so that consecutive MFMAs do not wait for each other
                const f4v zero = {0.f, 0.f, 0.f, 0.f};
                f4v dx0 = zero, dx1 = zero;
#pragma unroll
                for (int t = 0; t < 4; t += 2) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        dx0 = __builtin_amdgcn_mfma_f32_4x4x1f32(av[t][i], bv[t][i], (t == 0 && i == 0) ? zero : dx0, 0, 0, 0);
                        dx1 = __builtin_amdgcn_mfma_f32_4x4x1f32(av[t + 1][i], bv[t + 1][i], (t == 0 && i == 0) ? zero : dx1, 0, 0, 0);
                    }
                }
                float s[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float v = dx0[r] + dx1[r];
                    v += dpp_move<0x128>(v);  // row_ror:8
                    v += dpp_move<0x124>(v);  // row_ror:4
                    s[r] = v;                 // sum over the tile's 64 outputs of gy * d_r, sample j of chunk q
                }
                const float2 uv = uv_now[R];
                const float g1 = fmaf(uv.y, s[1] - s[0], s[0]);  // (s10 - s00)(1 - v) + (s11 - s01) v
                const float g2 = fmaf(uv.x, s[3] - s[2], s[2]);  // (s01 - s00)(1 - u) + (s11 - s10) u
                // every lane of a row has the sums of chunk q; the quarter og == R keeps them
                if (og == R) res = make_float2(g1, g2);
                slots = (unsigned)cur_slot * 0x01010101u;  // the next group starts in the current cell
            }
        });
#pragma unroll
        for (int r = 0; r < kGroups; ++r) {
            prod_now[r] = prod_nxt[r];
            n_now[r] = n_nxt[r];
            uv_now[r] = uv_nxt[r];
        }
#pragma unroll
        for (int p = 0; p < kUnroll; ++p) cells_now[p] = cells_nxt[p];
    }
    part[(int64_t)(nch - kUnroll) * kChunk] = res;
    asm volatile("" ::"v"(touched));
    if constexpr (DO_GP) {
        if (cur_cell >= 0) flush();
        retire_rows(split ? min(W, (cur_cell >> 8) + 2) : W);
    }
}

// grad_x[n][2k], [2k+1] = (1/h1, 1/h2) * sum over the output tiles of partial[tile][k][position of n].
// Threads walk the stream positions of a pair, so every tile's partial sums are read as one
// contiguous run; the sample index and the cell (for 1/h) come from the stream itself, and the
// two derivatives of a sample are written where they belong in grad_x (8 bytes per sample and
// pair; padding entries are skipped).  With `ld` > 0 the result goes to a transposed scratch
// [n_in][ld] instead (the convolution scatters it into the image from there).  The tiles are
// added in a fixed order.
constexpr int kCombinePer = 4;  // positions per thread

__global__ __launch_bounds__(256) void gx_combine_kernel(const float2 *__restrict__ partial, const f4v *__restrict__ rec,
                                                        const int32_t *__restrict__ chunk_cell,
                                                        const int32_t *__restrict__ block_start, GridTab tab,
                                                        float *__restrict__ gx, int64_t S, int K, int n_tiles,
                                                        int n_in, int n_blocks, int64_t ld, int vec2)
{
    __shared__ float s_invh[LMKAN_MAX_GRID];
    for (int i = threadIdx.x; i < tab.G; i += blockDim.x) s_invh[i] = tab.inv_h[i];
    __syncthreads();
    const int k = blockIdx.y;
    const int used = block_start[(int64_t)k * (n_blocks + 1) + n_blocks] * kChunk;  // entries of this pair's stream
    const f4v *rec_k = rec + (int64_t)k * S;
    const int32_t *cell_k = chunk_cell + (int64_t)k * (S / kChunk);
    const float2 *part_k = partial + (int64_t)k * S;
    const int64_t tile_stride = (int64_t)K * S;
    const int p0 = blockIdx.x * (256 * kCombinePer) + threadIdx.x;
    f4v e[kCombinePer];
    int cell[kCombinePer];
    float sx[kCombinePer], sy[kCombinePer];
#pragma unroll
    for (int i = 0; i < kCombinePer; ++i) {
        const int pos = p0 + i * 256;
        e[i] = f4v{0.f, 0.f, 0.f, 0.f};
        cell[i] = 0;
        sx[i] = sy[i] = 0.f;
        if (pos < used) {
            e[i] = rec_k[pos];
            cell[i] = cell_k[pos / kChunk];
        }
    }
    for (int t = 0; t < n_tiles; ++t) {
#pragma unroll
        for (int i = 0; i < kCombinePer; ++i) {
            const int pos = p0 + i * 256;
            if (pos < used) {
                const float2 p = part_k[t * tile_stride + pos];
                sx[i] += p.x;
                sy[i] += p.y;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < kCombinePer; ++i) {
        if (e[i].z == 0.f) continue;  // padding entry, or beyond the stream
        const int64_t n = __float_as_int(e[i].w);
        const float gx1 = sx[i] * s_invh[cell[i] >> 8], gx2 = sy[i] * s_invh[cell[i] & 255];
        if (ld > 0) {
            gx[(int64_t)(2 * k) * ld + n] = gx1;
            gx[(int64_t)(2 * k + 1) * ld + n] = gx2;
        } else if (vec2) {
            *reinterpret_cast<float2 *>(gx + n * n_in + 2 * k) = make_float2(gx1, gx2);
        } else {
            gx[n * n_in + 2 * k] = gx1;
            gx[n * n_in + 2 * k + 1] = gx2;
        }
    }
}

}  // namespace

bool fused_backward_applicable(const LayerShape &s, const void *coef, const float *gy, const float *gcoef)
{
    if (!outputs_by_four_ok(s) || !sorted_batch_ok(s)) return false;
    const uintptr_t coef_align = s.dtype == LMKAN_F32 ? 15 : 7;
    // rows of the table must keep that alignment too: every stride is a multiple of n_out (4 | n_out) or of 64
    if ((reinterpret_cast<uintptr_t>(coef) & coef_align) != 0) return false;
    if (ragged_outputs(s)) return true;  // gy through its tile-by-tile copy, gradient columns one by one
    return ((reinterpret_cast<uintptr_t>(gy) | reinterpret_cast<uintptr_t>(gcoef)) & 15) == 0;
}

size_t fused_partial_bytes(const LayerShape &s)
{
    const size_t S = (size_t)stream_stride(s.batch, s.G);
    return ((size_t)s.out_tiles() * s.pairs() * S * sizeof(float2) + 255) & ~(size_t)255;
}

void launch_backward_fused(const LayerShape &s, const GridTab &tab, const SortedStream &st, const void *records,
                           const void *coef, const GyView &gy, float *gx, float *gcoef, bool accumulate,
                           void *partial, float *gx_transposed, hipStream_t stream)
{
    FusedArgs a;
    a.rec = st.rec;
    a.chunk_cell = st.chunk_cell;
    a.block_start = st.block_start;
    a.gy = gy;
    a.P = coef;
    a.gP = gcoef;
    a.partial = static_cast<float2 *>(partial);
    a.pmap = coef_map(s);
    LayerShape g = s;
    g.layout = LMKAN_LAYOUT_PAPER;
    a.gmap = coef_map(g);
    a.B = s.batch;
    a.S = st.S;
    a.n_out = s.n_out;
    a.K = s.pairs();
    a.G = s.G;
    a.accumulate = accumulate ? 1 : 0;
    a.col_limit = s.layout == LMKAN_LAYOUT_PACKED ? s.out_tiles() * kTile : s.n_out;
    const int n_sub = stream_run_split(s);
    a.n_blocks = st.n_blocks;
    a.n_sub = n_sub;
    if (gcoef && (st.n_blocks > 1 || n_sub > 1) && !accumulate)
        launch_fill_zero(gcoef, (size_t)s.nodes() * (size_t)s.pairs() * (size_t)s.n_out, stream);
    const unsigned lds = (unsigned)(kFusedLdsFixed + (gcoef ? 2 * (s.G + 1) * kTile * sizeof(float) : 0));
    const unsigned grid = (unsigned)((int64_t)s.pairs() * s.out_tiles() * st.n_blocks * n_sub);
    typedef void (*Kernel)(FusedArgs);
#define LMKAN_FUSED_ROW(CT, GP)                                                                       \
    {                                                                                                 \
        {backward_fused_kernel<CT, GP, false, false>, backward_fused_kernel<CT, GP, false, true>},    \
        {                                                                                             \
            backward_fused_kernel<CT, GP, true, false>, backward_fused_kernel<CT, GP, true, true>     \
        }                                                                                             \
    }
    static const Kernel kernels[3][2][2][2] = {{LMKAN_FUSED_ROW(float, false), LMKAN_FUSED_ROW(float, true)},
                                               {LMKAN_FUSED_ROW(_Float16, false), LMKAN_FUSED_ROW(_Float16, true)},
                                               {LMKAN_FUSED_ROW(bf16_t, false), LMKAN_FUSED_ROW(bf16_t, true)}};
#undef LMKAN_FUSED_ROW
    // the last tile is ragged when the table has fewer columns than whole tiles
    const bool ragged = a.col_limit % kTile != 0;
    const Kernel kernel = kernels[s.dtype][gcoef ? 1 : 0][gy_offsets_fit_32_bits(s, gy) ? 1 : 0][ragged ? 1 : 0];
    {
        KernelTiming timing(stream, kTimeGradInput);
        kernel<<<grid, 64, lds, stream>>>(a);
    }
    const bool transposed = gx_transposed != nullptr;
    const dim3 cgrid((unsigned)((st.S + 256 * kCombinePer - 1) / (256 * kCombinePer)), (unsigned)s.pairs());
    gx_combine_kernel<<<cgrid, 256, 0, stream>>>(a.partial, st.rec, st.chunk_cell, st.block_start, tab,
                                                transposed ? gx_transposed : gx, st.S, s.pairs(), s.out_tiles(),
                                                s.n_in, st.n_blocks, transposed ? s.batch : 0,
                                                (reinterpret_cast<uintptr_t>(gx) & 7) == 0 ? 1 : 0);
}

}  // namespace lmkan
