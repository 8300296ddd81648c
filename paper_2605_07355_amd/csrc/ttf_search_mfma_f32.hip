// Window search and gate for fp32 tokens with windows up to 5x5 on any grid (Section 3, "Pointwise
// Matching with Local Window Search" and "Threshold Gating"), on the gfx950 matrix cores.
//
// fp32 products at matrix-core speed: every value is cut into three bf16 pieces, v = hi + mid + lo
// (24 significant bits, the subtractions that form mid and lo are exact), and a dot product is the
// sum of the six piece products whose weight is at least 2^-16 of the leading one:
//   <x, a> ~ xh.ah + xh.am + xm.ah + xm.am + xh.al + xl.ah        (dropped: xm.al, xl.am, xl.al <= 2^-24)
// each a 16x16x32 bf16 MFMA with fp32 accumulation, smallest terms first.  Six MFMAs per source tile,
// anchor tile and 32 channels cost 96 cycles of one SIMD's matrix pipe per 2 KiB of source data -- a
// third of what streaming those bytes from HBM takes -- where the plain fp32 MFMA (16x16x4) would
// need 256 cycles and bind before HBM does.  The split costs 5.5 vector instructions per element
// (v_cvt_pk_bf16_f32, shift / mask, subtract).
//
// Layout: that of k_search_mfma_shared.  A workgroup of 4 waves owns a 32-cell strip in 4*FW
// consecutive source frames (FW per wave, whole channel axis, wave-local epilogue) and shares the
// anchor fragments (three planes per tile and K-step, prepared per clip by k_anchor_prepare_f32)
// through LDS.  A pass is one K-step of 32 channels: 128 bytes per token, read as two coalesced
// 16-byte loads per lane (lane l: token l/4, floats 4(l%4).. of each 64-byte half) and moved to
// operand order (lane = token + 16*group) by eight ds_bpermute; inside a K-step the operand lane of
// group g holds channels 4g..4g+3 and 16+4g..16+4g+3, the anchor planes use the same order.  Loads
// run two passes ahead of their use (three register buffers), anchor fragments one pass ahead in a
// double LDS buffer.
#include "ttf_device.h"
#include "ttf_internal.h"
#include "ttf_search_tile.h"

#include <algorithm>

namespace ttf {
namespace {

typedef __attribute__((ext_vector_type(2))) float f32x2;

// hi / mid / lo bf16 pieces of two fp32 values, each pair packed into one word (round to nearest even;
// both subtractions are exact in fp32)
__device__ __forceinline__ void split_bf16x3(float a, float b, uint32_t& hi, uint32_t& mid, uint32_t& lo)
{
    hi = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
    const float ra = a - __builtin_bit_cast(float, hi << 16), rb = b - __builtin_bit_cast(float, hi & 0xffff0000u);
    mid = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{ra, rb}, bf16x2));
    const float sa = ra - __builtin_bit_cast(float, mid << 16), sb = rb - __builtin_bit_cast(float, mid & 0xffff0000u);
    lo = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{sa, sb}, bf16x2));
}

// PAD: grids that are not exactly 16*CT wide or whose height leaves partial strips (see finish_tile).
// ALL: tied-batch mode, every in-window cosine is stored instead of the arg max.
// (Two workgroups per CU wherever two double buffers of anchor planes fit the 160 KiB of LDS; the 5x5
// window on wide grids stages 60 KiB per pass and gets the whole register file instead.)
template <int CT, int RAD, int FW, bool ALL, bool PAD>
__global__ __launch_bounds__(256, (Shape<CT, RAD>::NA * 6 > 80 ? 1 : 2)) void k_search_mfma_f32(
    const float* __restrict__ x, const uint16_t* __restrict__ anchor_frag, const int32_t* __restrict__ anchor_index,
    const float* __restrict__ anchor_inv, int32_t* __restrict__ fuse_map, float* __restrict__ best_sim,
    int32_t* __restrict__ best_idx, uint16_t* __restrict__ keep16, float* __restrict__ win_sim, int F, int H, int C,
    float t, int groups, int Wg)
{
    using S = Shape<CT, RAD>;
    constexpr int W = S::W, NA = S::NA, NPS = S::NPS;
    constexpr int NS = 2 * FW;                               // source tiles per wave (FW frames)
    constexpr int FRG = 4 * FW;                              // frames per workgroup
    constexpr int NFR = 3 * NA;                              // 1-KiB anchor fragments per pass (3 planes per tile)
    constexpr int GL = (NFR + 3) / 4;                        // fragments each wave stages per pass
    extern __shared__ u32x4 frag_lds[];                      // [2][NA][3][64]
    static_assert(PAD || CT <= 2, "wider grids only through the padded path");
    const int N = PAD ? H * Wg : H * W;                      // tokens per frame
    const int CTt = CT <= 2 ? CT : (Wg + 15) / 16;           // column tiles per grid row
    const int NT = PAD ? H * CTt : N / 16;                   // anchor tiles per frame
    const int spr = (CTt + 1) / 2;                           // strips per grid row (CT == 3)
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int m = lane & 15, g = lane >> 4;
    const int tpf = PAD ? (CT == 1 ? (H + 1) / 2 : (CT == 2 ? H : H * spr)) : N / 32;   // 32-cell strips per frame
    int tp, grp, b;                                          // XCD-aware mapping as in k_search_mfma
    if ((tpf & 7) == 0) {
        const int chunk = tpf >> 3;
        const int idx = blockIdx.x >> 3;
        tp = (blockIdx.x & 7) * chunk + idx % chunk;
        grp = (idx / chunk) % groups;
        b = idx / chunk / groups;
    } else {
        tp = blockIdx.x % tpf;
        grp = (blockIdx.x / tpf) % groups;
        b = blockIdx.x / tpf / groups;
    }
    const int a_in = anchor_index[b];
    const int a = a_in < 0 ? 0x7fffffff : a_in;              // < 0: the anchor frame lies outside x (segment mode)
    const int nsrc = a_in < 0 ? F : F - 1;
    const int y0 = CT == 3 ? tp / spr : tp * 32 / W;
    const int c0 = CT == 3 ? 2 * (tp % spr) : 0;
    const int i0 = CT == 3 ? y0 * W : tp * 32;
    const int ylo = y0 - RAD;
    const int KS = C / 32;                                   // K-steps = passes

    const float* sp[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int si = min(grp * FRG + wave * FW + s / 2, nsrc - 1);
        const int k = si + (si >= a ? 1 : 0);
        size_t cell = i0 + 16 * (s % 2) + (lane >> 2);       // flat token index inside the frame
        if constexpr (PAD) {                                 // padding cells read a valid token; results are dropped
            const int ys = min(y0 + (CT == 1 ? s % 2 : 0), H - 1);
            const int xs = min((CT == 1 ? 0 : 16 * (c0 + s % 2)) + (lane >> 2), Wg - 1);
            cell = (size_t)ys * Wg + xs;
        }
        sp[s] = x + (((size_t)b * F + k) * N + cell) * (size_t)C + (lane & 3) * 4;
    }
    const int bperm = (4 * m + g) * 4;
    // this wave's share of a pass's anchor fragments: fragment e = wave + 4*i is (tile e / 3, plane e % 3)
    const uint16_t* gbase = anchor_frag + (size_t)b * NT * KS * 1536 + lane * 8;
    size_t goff[GL];
    int gslot[GL];
#pragma unroll
    for (int i = 0; i < GL; ++i) {
        const int e = min(wave + 4 * i, NFR - 1), q = e / 3, pl = e % 3;
        const int yy = min(max(ylo + S::tile_row(q), 0), H - 1);
        const int tile = yy * CTt + min(max(c0 + S::tile_col(q), 0), CTt - 1);   // outside the grid: clamped, masked later
        goff[i] = (size_t)tile * KS * 1536 + pl * 512;
        gslot[i] = (q * 3 + pl) * 64;
    }

    f32x4 acc[NS][NPS];
    float nv[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        nv[s] = 0.f;
#pragma unroll
        for (int q = 0; q < NPS; ++q) acc[s][q] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    u32x4 A[3][NS][2];                                       // native vectors: plain SSA values, never memory
    u32x4 G[GL];
    // (macros, not lambdas: captured by a lambda the staged fragments were kept in scratch memory)
#define TTF_REQUEST_ANCHOR(pass_)                                                                             \
    do {                                                                                                      \
        const int pq = min((pass_), KS - 1);                                                                  \
        _Pragma("unroll") for (int i = 0; i < GL; ++i)                                                        \
            G[i] = *reinterpret_cast<const u32x4*>(gbase + goff[i] + (size_t)pq * 1536);                      \
    } while (0)
#define TTF_REQUEST_SOURCE(pass_, Abuf)                                                                       \
    do {                                                                                                      \
        const int pq = min((pass_), KS - 1);                                                                  \
        _Pragma("unroll") for (int h = 0; h < 2; ++h) {                                                       \
            _Pragma("unroll") for (int s = 0; s < NS; ++s)                                                    \
                Abuf[s][h] = *reinterpret_cast<const u32x4*>(sp[s] + pq * 32 + h * 16);                       \
        }                                                                                                     \
    } while (0)
#define TTF_STAGE(buf_)                                                                                       \
    do {                                                                                                      \
        _Pragma("unroll") for (int i = 0; i < GL; ++i)                                                        \
            if (wave + 4 * i < NFR) frag_lds[(buf_) * (NFR * 64) + gslot[i] + lane] = G[i];                   \
    } while (0)

    // The LDS round trips of a pass (lane permutations, anchor planes) are requested ahead of the
    // arithmetic that hides them: with two waves per SIMD nothing else covers an exposed LDS wait.
    auto compute = [&](int buf, const u32x4 (&Abuf)[NS][2]) {
        const u32x4* fr = frag_lds + buf * (NFR * 64) + lane;
        // phase 1: squared norms, and every lane permutation of the pass in flight at once
        uint32_t f[NS][8];
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const uint32_t r[8] = {Abuf[s][0][0], Abuf[s][0][1], Abuf[s][0][2], Abuf[s][0][3],
                                   Abuf[s][1][0], Abuf[s][1][1], Abuf[s][1][2], Abuf[s][1][3]};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float v = __builtin_bit_cast(float, r[e]);
                nv[s] = fmaf(v, v, nv[s]);
                f[s][e] = (uint32_t)__builtin_amdgcn_ds_bpermute(bperm, (int)r[e]);
            }
        }
        u32x4 bq[2][3];                                      // anchor planes of the current and the next tile
#pragma unroll
        for (int pl = 0; pl < 3; ++pl) bq[0][pl] = fr[pl * 64];
        __builtin_amdgcn_sched_barrier(0);
        // phase 2: the three bf16 pieces of every source tile, in operand order
        bf16x8 ah[NS], am[NS], al[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            uint32_t hi[4], mid[4], lo[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                split_bf16x3(__builtin_bit_cast(float, f[s][2 * e]), __builtin_bit_cast(float, f[s][2 * e + 1]), hi[e],
                             mid[e], lo[e]);
            ah[s] = __builtin_bit_cast(bf16x8, uint4{hi[0], hi[1], hi[2], hi[3]});
            am[s] = __builtin_bit_cast(bf16x8, uint4{mid[0], mid[1], mid[2], mid[3]});
            al[s] = __builtin_bit_cast(bf16x8, uint4{lo[0], lo[1], lo[2], lo[3]});
        }
        __builtin_amdgcn_sched_barrier(0);
        // phase 3: one anchor tile at a time, the next tile's planes requested before this tile's products
#pragma unroll
        for (int qa = 0; qa < NA; ++qa) {
            if (qa + 1 < NA) {
#pragma unroll
                for (int pl = 0; pl < 3; ++pl) bq[(qa + 1) & 1][pl] = fr[((qa + 1) * 3 + pl) * 64];
            }
            const bf16x8 bh = __builtin_bit_cast(bf16x8, bq[qa & 1][0]);
            const bf16x8 bm = __builtin_bit_cast(bf16x8, bq[qa & 1][1]);
            const bf16x8 bl = __builtin_bit_cast(bf16x8, bq[qa & 1][2]);
            // the six piece products, smallest first; term by term over every accumulator that uses this
            // anchor tile, so that consecutive MFMAs do not wait for each other's result
#pragma unroll
            for (int term = 0; term < 6; ++term) {
                const bf16x8 bb = term == 0 ? bh : (term == 1 ? bl : (term == 2 ? bm : (term == 3 ? bh : (term == 4 ? bm : bh))));
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    const bf16x8 aa = term == 0 ? al[s] : (term == 2 || term == 3 ? am[s] : ah[s]);
#pragma unroll
                    for (int q = 0; q < NPS; ++q) {              // the pair (if any) of this source tile that uses tile qa
                        if (S::pair_tile(s % 2, q) == qa)
                            acc[s][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aa, bb, acc[s][q], 0, 0, 0);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // State at the top of pass p: LDS buffer p%2 holds the anchor fragments of pass p; the source
    // fragments of passes p and p+1 (A[p%3], A[(p+1)%3]) and the anchor fragments of pass p+1 (G) are
    // already requested.  The anchor loads waited for are always older than the source loads that may
    // still be in flight, which therefore stay in flight across the wait.
    TTF_REQUEST_ANCHOR(0);
    TTF_REQUEST_SOURCE(0, A[0]);
    TTF_STAGE(0);
    lds_barrier();
    TTF_REQUEST_ANCHOR(1);
    TTF_REQUEST_SOURCE(1, A[1]);
#define TTF_PASS(j)                                                   \
    do {                                                              \
        const int pp = pass + (j);                                    \
        TTF_STAGE((pp + 1) & 1);                                      \
        TTF_REQUEST_ANCHOR(pp + 2);                                   \
        TTF_REQUEST_SOURCE(pp + 2, A[((j) + 2) % 3]);                 \
        __builtin_amdgcn_sched_barrier(0);                            \
        compute(pp & 1, A[(j)]);                                      \
        __builtin_amdgcn_sched_barrier(0);                            \
        lds_barrier();                                                \
    } while (0)
    for (int pass = 0; pass < KS; pass += 3) {
        TTF_PASS(0);
        if (pass + 1 < KS) TTF_PASS(1);                      // wave-uniform
        if (pass + 2 < KS) TTF_PASS(2);
    }
#undef TTF_PASS
#undef TTF_REQUEST_ANCHOR
#undef TTF_REQUEST_SOURCE
#undef TTF_STAGE

#pragma unroll
    for (int s = 0; s < NS; ++s) {
        nv[s] += __shfl_xor(nv[s], 1, 64);
        nv[s] += __shfl_xor(nv[s], 2, 64);
    }
    float ai_tile[NA];                                       // this lane's anchor inverse norms (epilogue only)
#pragma unroll
    for (int q = 0; q < NA; ++q) {
        const int yy = min(max(ylo + S::tile_row(q), 0), H - 1);
        ai_tile[q] = anchor_inv[(size_t)b * NT * 16 + 16 * (yy * CTt + min(max(c0 + S::tile_col(q), 0), CTt - 1)) + m];
    }
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        float nn[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) nn[j] = __shfl(nv[s], 4 * (4 * g + j), 64);
        const int si = grp * FRG + wave * FW + s / 2;
        finish_tile<CT, RAD, ALL, PAD>(acc[s], nn, s, si < nsrc, min(si, nsrc - 1), a, b, F, H, i0, t, ai_tile, fuse_map,
                                       best_sim, best_idx, keep16, win_sim, lane, Wg, c0);
    }
}

template <int CT, int RAD>
hipError_t launch_f32(const ttf_params& p, const void* x, bool external_anchor, const Workspace& w,
                      const int32_t* anchor_index, int32_t* fuse_map, float* best_sim, int32_t* best_idx,
                      float* win_sim, hipStream_t s)
{
    using S = Shape<CT, RAD>;
    const int nsrc = external_anchor ? p.F : p.F - 1;
    if (nsrc < 1) return hipSuccess;                         // no source frame: the anchor rows are all there is
    constexpr int FWS = S::NPS <= 3 ? 2 : 1;                 // frames per wave: as many as the accumulators leave room for
    const bool pad = !mfma_f32_aligned(p);
    const int groups = (nsrc + 4 * FWS - 1) / (4 * FWS);
    const int N = p.H * p.W;
    const int strips = !pad ? N / 32
                     : CT == 1 ? (p.H + 1) / 2 : (CT == 2 ? p.H : p.H * (((p.W + 15) / 16 + 1) / 2));
    const size_t wgs = (size_t)p.B * groups * strips;
    const size_t lds = 2 * 3 * (size_t)S::NA * 1024;
    auto go = [&](auto kernel) {
        hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kernel), lds);
        if (e != hipSuccess) return e;
        kernel<<<(unsigned)wgs, 256, lds, s>>>(static_cast<const float*>(x), w.anchor_frag, anchor_index, w.anchor_inv,
                                               fuse_map, best_sim, best_idx, reinterpret_cast<uint16_t*>(w.keep_bits),
                                               win_sim, p.F, p.H, p.C, p.t, groups, p.W);
        return hipGetLastError();
    };
    if constexpr (CT == 3) {
        return win_sim ? go(k_search_mfma_f32<CT, RAD, FWS, true, true>) : go(k_search_mfma_f32<CT, RAD, FWS, false, true>);
    } else {
        if (pad)
            return win_sim ? go(k_search_mfma_f32<CT, RAD, FWS, true, true>)
                           : go(k_search_mfma_f32<CT, RAD, FWS, false, true>);
        return win_sim ? go(k_search_mfma_f32<CT, RAD, FWS, true, false>) : go(k_search_mfma_f32<CT, RAD, FWS, false, false>);
    }
}

}  // namespace

// Grids exactly 16 or 32 wide with whole 64-token keep words: the search writes the keep bits itself.
bool mfma_f32_aligned(const ttf_params& p)
{
    return (p.W == 16 && p.H % 4 == 0) || (p.W == 32 && p.H % 2 == 0);
}

// True when the matrix-core kernels for fp32 tokens take this problem: radius <= 2, whole 32-channel
// K-steps, and enough workgroups.  A workgroup walks the channel axis one K-step per pass (about 1.6 us
// each on an idle chip), so a handful of them is slower than the wave-per-token kernels, which spread
// the same tokens over hundreds of waves (measured: B1 F16 16x16 C2048, 16 workgroups, 0.104 against
// 0.033 ms; B4 F16 16x16 C1024, 64 workgroups, 0.059 against 0.069 ms).
bool mfma_search_f32_supported(const ttf_params& p)
{
    if (p.dtype != TTF_F32 || p.r > 2 || p.C % 32 != 0) return false;
    const int ct = p.W <= 16 ? 1 : (p.W <= 32 ? 2 : 3);
    const int nps = (ct == 1 ? 1 : ct) * (2 * p.r + 1);              // anchor tiles paired with a source tile
    const int frames_per_wg = nps <= 3 ? 8 : 4;
    const long long groups = (std::max(p.F - 1, 1) + frames_per_wg - 1) / frames_per_wg;
    const long long strips = mfma_f32_aligned(p) ? (long long)p.H * p.W / 32
                           : ct == 1 ? (p.H + 1) / 2 : (ct == 2 ? p.H : (long long)p.H * (((p.W + 15) / 16 + 1) / 2));
    return (long long)p.B * groups * strips >= 48;
}

hipError_t launch_window_search_mfma_f32(const ttf_params& p, const void* x, bool external_anchor, const Workspace& w,
                                         const int32_t* anchor_index, int32_t* fuse_map, float* best_sim,
                                         int32_t* best_idx, float* win_sim, hipStream_t s)
{
    const int ct = p.W <= 16 ? 1 : (p.W <= 32 ? 2 : 3);
    hipError_t e = hipErrorInvalidValue;
#define TTF_FCASE(CT, RAD)                          \
    if (ct == CT && p.r == RAD)                     \
    e = launch_f32<CT, RAD>(p, x, external_anchor, w, anchor_index, fuse_map, best_sim, best_idx, win_sim, s)
    TTF_FCASE(1, 0);
    TTF_FCASE(1, 1);
    TTF_FCASE(1, 2);
    TTF_FCASE(2, 0);
    TTF_FCASE(2, 1);
    TTF_FCASE(2, 2);
    TTF_FCASE(3, 0);
    TTF_FCASE(3, 1);
    TTF_FCASE(3, 2);
#undef TTF_FCASE
    if (e != hipSuccess) return e;
    // padded tile rows: the keep words are packed from the fuse map afterwards (tied-batch mode: the tie
    // kernel forms them)
    if (!mfma_f32_aligned(p) && !win_sim) return launch_pack_keep(p, fuse_map, anchor_index, w, s);
    return hipSuccess;
}

}  // namespace ttf
