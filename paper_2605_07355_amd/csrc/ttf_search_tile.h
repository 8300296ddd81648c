// Device-side pieces shared by the matrix-core window-search kernels (bf16 and fp32 input): the
// geometry of a workgroup's strip, the epilogue that turns finished 16x16 products into cosines,
// arg max, gate and outputs (Section 3, "Pointwise Matching with Local Window Search" and "Threshold
// Gating"), and the LDS-only workgroup barrier.
#pragma once

#include "ttf_device.h"

namespace ttf {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr float kNegInf = -__builtin_inff();

// Geometry of one workgroup's problem: a strip of 32 grid cells (two source tiles of 16).
// CT = 1: grid (tile row) 16 wide, the strip is two rows.  CT = 2: 32 wide, the strip is one row.
// CT = 3: any wider grid; the strip is 32 consecutive columns of one row starting at column tile
// c0 (even), and the anchor tiles fetched are column tiles c0-1 .. c0+2 of the rows around it.
template <int CT, int RAD>
struct Shape {
    static_assert(CT >= 1 && CT <= 3, "1: 16 wide, 2: 32 wide, 3: wider");
    static constexpr int W = CT == 1 ? 16 : 32;              // cells per strip row
    static constexpr int ROWS = 2 * RAD + 1;
    // anchor tiles fetched per K-step: CT==1: rows y0-RAD .. y0+1+RAD; CT==2: rows y-RAD .. y+RAD, 2 columns;
    // CT==3: the same rows, 4 columns
    static constexpr int NA = CT == 1 ? 2 * RAD + 2 : (CT == 2 ? 2 : 4) * ROWS;
    // anchor tiles paired with each source tile (CT==3: the column tile itself and both neighbours)
    static constexpr int NPS = CT == 1 ? ROWS : (CT == 2 ? 2 : 3) * ROWS;
    // source frames per workgroup and anchor fragment prefetch distance: sized so accumulators
    // (4*NPS VGPRs per source tile), source fragments (4 per tile and K-step) and the anchor
    // ring (4*NA per K-step) fit the 256 VGPRs of a wave at two waves per SIMD
    static constexpr int FR = NPS <= 3 ? 4 : 2;
    // waves per SIMD the register budget is planned for (512 registers per lane and SIMD)
    static constexpr int OCC = NPS <= 6 ? 2 : 1;
    static constexpr int PF = 1;
    // source tiles whose partial products go through LDS together (<= 48 KiB)
    static constexpr int RT = NPS <= 3 ? 4 : (NPS <= 6 ? 2 : 1);
    // fetched anchor tile that pair q of source tile u (tile within the strip) uses
    __device__ static constexpr int pair_tile(int u, int q)
    {
        return CT == 1 ? u + q : (CT == 2 ? q : (q / 3) * 4 + u + q % 3);
    }
    // fetched anchor tile a: row offset from ylo, column tile relative to the strip's first
    __device__ static constexpr int tile_row(int a) { return CT == 1 ? a : (CT == 2 ? a / 2 : a / 4); }
    __device__ static constexpr int tile_col(int a) { return CT == 1 ? 0 : (CT == 2 ? a % 2 : a % 4 - 1); }
    // pair q of source tile u: anchor row offset from the source row - RAD, and anchor column tile
    // relative to the strip's first column tile
    __device__ static constexpr int pair_row(int u, int q) { return CT == 1 ? q : (CT == 2 ? q / 2 : q / 3); }
    __device__ static constexpr int pair_col(int u, int q) { return CT == 1 ? 0 : (CT == 2 ? q % 2 : u - 1 + q % 3); }
};

constexpr int kNoArg = 0x7fffffff;       // "no candidate yet" while reducing (so that min() breaks ties)

// One step of an arg max over the 16 lanes of a DPP row: every lane looks at the lane the DPP
// control pairs it with and keeps the larger value, the lower index on equal values.  NaN never
// wins a comparison, so it never displaces a number.
template <int DPP_CTRL>
__device__ __forceinline__ void row_argmax_step(float& best, int& arg)
{
    const float ob = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, best),
                                                                           DPP_CTRL, 0xf, 0xf, false));
    const int oa = __builtin_amdgcn_update_dpp(0, arg, DPP_CTRL, 0xf, 0xf, false);
    const bool take = (ob > best) | ((ob == best) & (oa < arg));
    best = take ? ob : best;
    arg = take ? oa : arg;
}

// Final step for one source tile (16 tokens of one frame): v[q] are the complete 16x16 products
// with the NPS anchor tiles paired with it (MFMA result layout: lane = anchor column n + 16*g,
// element j = source token 4g+j), nn[j] the squared norms of tokens 4g+j, ai_tile[a] this lane's
// anchor inverse norm in anchor tile a.  Forms the cosines,
// masks the band |dx| <= RAD and the rows outside the grid, takes the arg max (lowest anchor
// index on ties), applies the threshold and writes s^, dst, the fuse map and the tile's 16 keep
// bits.  Straight-line code: no divergent branches.
// ALL (tied-batch mode): instead of the arg max, every in-window cosine is stored to
// win_sim[b][k][(dy+RAD)*(2*RAD+1) + (dx+RAD)][i] and nothing else is written.
// PAD: the grid is Wg <= W tokens wide (columns Wg..W-1 of every tile row are padding): flat
// indices use Wg, padding columns never win nor get written, H may be odd, and the keep bits are
// packed afterwards by k_pack_keep (tiles are no longer aligned to 16-bit pieces of keep words).
template <int CT, int RAD, bool ALL, bool PAD = false>
__device__ __forceinline__ void finish_tile(const f32x4* v, const float* nn, int s, bool live, int si, int a, int b,
                                            int F, int H, int i0, float t, const float* ai_tile,
                                            int32_t* __restrict__ fuse_map, float* __restrict__ best_sim,
                                            int32_t* __restrict__ best_idx, uint16_t* __restrict__ keep16,
                                            float* __restrict__ win_sim, int lane, int Wg = Shape<CT, RAD>::W,
                                            int c0 = 0)
{
    static_assert(PAD || CT <= 2, "wider grids only through the padded path");
    using S = Shape<CT, RAD>;
    constexpr int W = S::W, NPS = S::NPS;
    const int N = PAD ? H * Wg : H * W;
    const int m = lane & 15, g = lane >> 4;
    const int u = s % 2;                                     // tile within the frame
    const int y0 = i0 / W;
    float sinv[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) sinv[j] = nn[j] > 0.f ? __builtin_amdgcn_rsqf(nn[j]) : 0.f;
    float best[4] = {kNegInf, kNegInf, kNegInf, kNegInf};
    int arg[4] = {kNoArg, kNoArg, kNoArg, kNoArg};
    const int ysrc = y0 + (CT == 1 ? u : 0);
    const int xsrc0 = CT == 1 ? 0 : 16 * (c0 + u);           // c0 = 0 unless CT == 3
    if constexpr (ALL) {
        constexpr int K1 = 2 * RAD + 1;
        const int kk = si + (si >= a ? 1 : 0);
        // flat index of source token (4g + 0) of this tile inside the frame
        const size_t cell0 = PAD ? (size_t)ysrc * Wg + xsrc0 + 4 * g : (size_t)i0 + 16 * u + 4 * g;
        const size_t tok0 = ((size_t)b * F + kk) * (K1 * K1) * N + cell0;   // slot 0 of token 4g+0
        const bool src_row_ok = !PAD || ysrc < H;
#pragma unroll
        for (int q = 0; q < NPS; ++q) {
            const int yy = ysrc - RAD + S::pair_row(u, q);
            const int xa_col = 16 * (c0 + S::pair_col(u, q)) + m;
            const bool row_ok = (yy >= 0) & (yy < H) & (!PAD || ((xa_col >= 0) & (xa_col < Wg)));
            const float ai = ai_tile[S::pair_tile(u, q)];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int xs = xsrc0 + 4 * g + j;
                const int dx = xa_col - xs;
                if (live & src_row_ok & row_ok & (dx >= -RAD) & (dx <= RAD) & (!PAD || xs < Wg))
                    win_sim[tok0 + (size_t)((yy - ysrc + RAD) * K1 + dx + RAD) * N + j] = v[q][j] * sinv[j] * ai;
            }
        }
        return;
    }
#pragma unroll
    for (int q = 0; q < NPS; ++q) {
        // anchor tile of pair q: CT==1: row ysrc-RAD+q; CT==2: row ylo + q/2, column tile q%2;
        // CT==3: row ylo + q/3, column tile c0 + u - 1 + q%3
        const int yy = ysrc - RAD + S::pair_row(u, q);
        const int xa_col = 16 * (c0 + S::pair_col(u, q)) + m;     // this lane's anchor column
        const bool row_ok = PAD ? (yy >= 0) & (yy < H) & (xa_col >= 0) & (xa_col < Wg) : (yy >= 0) & (yy < H);
        const int ja = min(max(yy, 0), H - 1) * (PAD ? Wg : W) + xa_col;
        const float ai = ai_tile[S::pair_tile(u, q)];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int dx = xa_col - (xsrc0 + 4 * g + j);          // anchor column - source column
            const bool in_band = row_ok & (dx >= -RAD) & (dx <= RAD);
            const float sim = in_band ? v[q][j] * sinv[j] * ai : kNegInf;
            const bool take = sim > best[j];                      // ascending ja per lane: first maximum
            best[j] = take ? sim : best[j];
            arg[j] = take ? ja : arg[j];
        }
    }
    // arg max across the 16 anchor columns held by the 16 lanes of a row; lowest index on ties
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        row_argmax_step<0xB1>(best[j], arg[j]);       // lanes i <-> i^1
        row_argmax_step<0x4E>(best[j], arg[j]);       // lanes i <-> i^2
        row_argmax_step<0x141>(best[j], arg[j]);      // mirror inside each half row (8 lanes)
        row_argmax_step<0x140>(best[j], arg[j]);      // mirror inside the row (16 lanes)
        arg[j] = arg[j] == kNoArg ? -1 : arg[j];
    }
    const int k = si + (si >= a ? 1 : 0);
    if constexpr (PAD) {
        const size_t row0 = ((size_t)b * F + k) * N + (size_t)ysrc * Wg;
        if (m == 0 && live && ysrc < H) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int xs = xsrc0 + 4 * g + j;
                if (xs < Wg) {
                    const bool fused = best[j] > t;               // keep = 1[s^ <= t]
                    fuse_map[row0 + xs] = fused ? arg[j] : -1;
                    if (best_sim) best_sim[row0 + xs] = best[j];
                    if (best_idx) best_idx[row0 + xs] = arg[j];
                }
            }
        }
        return;
    }
    const size_t o0 = ((size_t)b * F + k) * N + i0 + 16 * u;
    unsigned keep = 0;
    if (m == 0) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const size_t o = o0 + 4 * g + j;
            const bool fused = best[j] > t;                   // keep = 1[s^ <= t]
            if (live) {
                fuse_map[o] = fused ? arg[j] : -1;
                if (best_sim) best_sim[o] = best[j];
                if (best_idx) best_idx[o] = arg[j];
            }
            if (!fused) keep |= 1u << (4 * g + j);
        }
    }
    keep |= __shfl_xor(keep, 16, 64);
    keep |= __shfl_xor(keep, 32, 64);
    if (lane == 0 && live) keep16[o0 / 16] = (uint16_t)keep;
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load of the wave (its fence covers global memory), which would drain the
// source fragments requested a pass ahead; the data exchanged here lives in LDS alone.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

}  // namespace
}  // namespace ttf
