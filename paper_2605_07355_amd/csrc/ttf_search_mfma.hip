// Window search and gate for bf16 tokens with windows up to 5x5 on any grid (Section 3, "Pointwise
// Matching with Local Window Search" and "Threshold Gating"), on the gfx950 matrix cores.  Grids
// exactly 16 or 32 tokens wide with whole 64-token keep words take k_search_mfma (the 5x5 window on
// large 32-wide inputs k_search_mfma_shared); every other grid runs k_search_mfma_shared on tile rows
// padded to whole 16-column tiles.
//
// Why matrix cores for a banded product: the (2r+1)^2 dot products per source token cost
// 2(2r+1)^2 C + 2C flops per 2C input bytes.  On the plain vector ALUs (78.6 TFLOP/s fp32
// without packed math) that arithmetic alone would take as long as streaming the tokens from
// HBM at its peak rate, before any bf16 unpacking or cross-lane reduction.  A 16x16x32 bf16
// MFMA computes a source tile (16 consecutive tokens of a grid row) against an anchor tile (16
// consecutive anchor tokens) with fp32 accumulation at a small fraction of that cost; only the
// band |dx| <= r of each 16x16 result is used.  The kernel is then bound by HBM, as intended.
//
// Data movement is what the design is about:
//  * Source tokens are read exactly once, with coalesced 16-byte loads (lane l reads chunk l%4 of
//    token l/4: four tokens x 64 contiguous bytes per quarter-wave), and moved into MFMA operand
//    order (lane = token + 16*chunk) by four ds_bpermute per fragment.  Loading straight in
//    operand order would make every lane of a quarter-wave touch a different cache line, which
//    the texture path serves at one line per clock.
//  * Anchor tokens are re-used by every source frame, so their inverse norms and a copy of the
//    anchor frame in fragment order (1 KiB per tile and K-step, lane-major) are prepared once
//    per clip (ttf_anchor.hip); the search streams those fragments from L2 fully coalesced.
//  * One workgroup owns the same 32 grid cells (two source tiles) in FR
//    consecutive source frames, so every anchor fragment fetched from L2 feeds FR frames.
//  * Large problems: one wavefront per workgroup walks the whole channel axis, so its 16x16
//    products are final and the epilogue is wave-local.  Small problems: the channel axis is split
//    across 4 wavefronts and the partial products are added through LDS in wave order (fixed
//    order: reproducible).  The 5x5 window on 32-wide grids (10 anchor tiles per K-step) has its
//    own layout, k_search_mfma_shared: 4 waves with one frame each share the anchor fragments
//    through LDS.  In every layout one wave per source tile forms the cosines, masks the band,
//    takes the arg max (lowest anchor index on ties), applies the threshold and writes s^, dst,
//    the fuse map and 16 keep bits.
//  * Source squared norms: v_dot2 on the loaded fragments (one VGPR per tile), reduced with the
//    products.
#include "ttf_device.h"
#include "ttf_internal.h"
#include "ttf_search_tile.h"

namespace ttf {
namespace {

constexpr size_t kSimds = 256 * 4;             // SIMDs of the chip: wave slots per unit of occupancy

// B operand that picks 16 of the 32 channels of a K-step: E_h[k][n] = 1 iff k == 16h + n (operand
// order: lane n + 16g holds rows k = 8g .. 8g+7 of column n).  A source tile times E_h is that
// tile's tokens x channels 16h .. 16h+15 in the MFMA result layout, i.e. a lane then holds four
// TOKENS of one channel: the form in which a sum over tokens is cheap.
__device__ __forceinline__ bf16x8 channel_picker(int h, int lane)
{
    const int n = lane & 15, g = lane >> 4;
    const bool mine = g == 2 * h + (n >> 3);
    const int e = n & 7;
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = (mine && (e >> 1) == i) ? ((e & 1) ? 0x3F800000u : 0x00003F80u) : 0u;
    return __builtin_bit_cast(bf16x8, uint4{w[0], w[1], w[2], w[3]});
}

// FRO: source frames per workgroup, 0 = the shape's default.  Small inputs use 1 frame and long
// passes (more workgroups, fewer dependent rounds of loads per workgroup).
// SPEC 0: the plain search.  SPEC 1: the search of the speculative pass -- the anchor in
// anchor_index may be a guess, so every frame of the clip, the anchor frame included, is walked
// (its outputs are not written) and the sum over the 32 tokens of every (frame, strip) is written to
// strip_sum[b][k][strip][channel], from which the exact anchor rule is evaluated afterwards.  The
// sums come from two extra MFMAs per source tile and K-step (channel_picker) whose accumulators add
// the two tiles of a strip; four in-lane adds and two cross-row steps finish them.
// SPEC 2: the plain search for the clips marked in spec[b][2] only (guess refuted); other clips exit.
// RAG: the K-steps need not divide over the waves and passes.  The passes are dealt to the waves in
// contiguous runs of nearly equal length (a wave may get none); the wave that owns the end of the
// channel axis finishes with a pass of the K-steps left over.
template <int CT, int RAD, int KSW, int NW, bool ALL, int FRO = 0, int SPEC = 0, bool RAG = false>
__global__ __launch_bounds__(NW * 64, (Shape<CT, RAD>::OCC)) void k_search_mfma(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ anchor_frag,
    const int32_t* __restrict__ anchor_index, const float* __restrict__ anchor_inv,
    int32_t* __restrict__ fuse_map, float* __restrict__ best_sim, int32_t* __restrict__ best_idx,
    uint16_t* __restrict__ keep16, float* __restrict__ win_sim, int F, int H, int C, float t, int passes, int groups,
    const int32_t* __restrict__ spec, float* __restrict__ strip_sum)
{
    using S = Shape<CT, RAD>;
    constexpr int W = S::W, NA = S::NA, NPS = S::NPS, PF = S::PF;
    constexpr int FR = FRO ? FRO : S::FR;
    constexpr int NS = 2 * FR;                               // source tiles of the workgroup
    constexpr int RT = S::RT < NS ? S::RT : NS;              // source tiles per LDS round
    constexpr int NB = PF + 1;                               // anchor fragment ring
    const int N = H * W;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: per-wave offsets stay scalar
    const int m = lane & 15, g = lane >> 4;
    const int tpf = N / 32;                                  // workgroups per frame group
    // Workgroup -> (clip, frame group, 32-cell strip).  Workgroups are dealt to the 8 XCDs round
    // robin and every XCD has its own L2, so when the strips divide evenly each XCD owns tpf/8
    // ADJACENT strips (for every clip and frame group): the anchor rows its workgroups re-read
    // overlap and stay resident in that L2 instead of being fetched again by every frame group.
    int tp, grp, b;
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
    if constexpr (SPEC == 1) {
        if (spec[4 * b + 1] == 0) return;                    // no trusted guess: the clip takes the two-pass route
    }
    if constexpr (SPEC == 2) {
        if (spec[4 * b + 2] == 0) return;                    // guess confirmed: nothing to redo
    }
    const int a_in = anchor_index[b];                        // < 0: the anchor frame lies outside x (segment mode)
    // frame slot -> frame: the anchor frame is skipped, except in the speculative pass, which walks
    // every frame (a_skip beyond every frame index)
    const int a_skip = (SPEC == 1 || a_in < 0) ? 0x7fffffff : a_in;
    const int i0 = tp * 32;                                  // first grid cell of this workgroup

    const int y0 = i0 / W;                                   // first (or only) source row
    const int ylo = y0 - RAD;
    // (speculative pass: C % 128 == 0, so the K-step count is even and a ragged split only hands the waves
    // different numbers of whole two-step passes; the one-step pass below never runs there)
    static_assert(!(RAG && SPEC == 1) || KSW == 2, "strip sums are stored per pair of K-steps");
    const int KS = C / 32;                                   // K-steps per token
    // first K-step of this wave and how many it has.  RAG: the ceil(KS / KSW) passes are dealt to the
    // waves as evenly as whole passes allow, so only the last wave can end on a short pass; a wave left
    // without any starts at K-step 0, where its pointers stay inside the row (it loads nothing)
    const int units = (KS + KSW - 1) / KSW;
    const int kfirst = RAG ? (wave * units / NW) * KSW : wave * (KS / NW);
    const int ks_mine = RAG ? min(KS, ((wave + 1) * units / NW) * KSW) - kfirst : KS / NW;
    const int kbase = (RAG && ks_mine == 0) ? 0 : kfirst;
    const int nsrc = (SPEC == 1 || a_in < 0) ? F : F - 1;    // frames walked per clip (>= 1 here)

    // source frame of slot f: the f-th walked frame of this group, the last one repeated past the end
    // (plain 64-bit addresses: the same loads through buffer descriptors, with one shared per-lane
    // offset and scalar per-tile offsets, freed 22 registers but ran 10 % slower)
    const uint16_t* sp[NS];                                  // load order: lane -> token lane/4, chunk lane%4
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int si = min(grp * FR + s / 2, nsrc - 1);
        const int k = si + (si >= a_skip ? 1 : 0);
        sp[s] = x + (((size_t)b * F + k) * N + i0 + 16 * (s % 2) + (lane >> 2)) * (size_t)C +
                kbase * 32 + (lane & 3) * 8;
    }
    const int bperm = (4 * m + g) * 4;                       // operand lane (token m, chunk g) <- load lane 4m+g
    const uint16_t* ap[NA];
    float ai_tile[NA];
#pragma unroll
    for (int q = 0; q < NA; ++q) {
        const int yy = min(max(ylo + S::tile_row(q), 0), H - 1);      // rows outside the grid: clamped, masked later
        const int tile = yy * CT + S::tile_col(q);
        ap[q] = anchor_frag + (((size_t)b * (N / 16) + tile) * KS + kbase) * 512 + lane * 8;
        ai_tile[q] = anchor_inv[(size_t)b * N + 16 * tile + m];       // requested now, used in the epilogue
    }

    f32x4 acc[NS][NPS];
    float nv[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        nv[s] = 0.f;
#pragma unroll
        for (int q = 0; q < NPS; ++q) acc[s][q] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // speculative pass: the channel pickers, and where this lane's strip sums go (lanes 0..31 hold the
    // 32 channels of a K-step after the reduction)
    bf16x8 pick0, pick1;
    float* sums = nullptr;
    float held[FR];                                          // first K-step's totals until the second's are there
    if constexpr (SPEC == 1) {
        static_assert(KSW <= 2, "strip sums are stored once per pass from the two halves of a wave");
        pick0 = channel_picker(0, lane);
        pick1 = channel_picker(1, lane);
        sums = strip_sum + ((((size_t)b * F + (size_t)grp * FR) * tpf + tp) * (size_t)C) + kbase * 32 +
               (KSW == 2 ? lane : (lane & 31));
    }

    // One source tile's share of the strip sums (speculative pass).  Even tile of a frame: start the two
    // token x channel accumulators; odd tile: add to them, finish the strip and store it.
    //   lane n + 16g of d0 / d1: tokens 4g..4g+3 (both tiles) of channel n / 16 + n; four in-lane adds;
    //   the four row groups are added by an fp32 MFMA against a matrix of ones (K = the row group), after
    //   which every lane n + 16g holds the strip's total of its channel (rows 0, 2 keep channel n, rows
    //   1, 3 channel 16 + n);
    //   one 256-byte store per frame and pass: lanes 0..31 the first K-step's 32 channels, lanes 32..63
    //   the second's.  A slot past the clip's end repeats the last frame and stores the same values to
    //   the same place again.
    f32x4 d0, d1;
#define TTF_STRIP_SUM_STEP(av_, s_, ks_, ks0_)                                                                \
    do {                                                                                                      \
        const f32x4 zero_ = {0.f, 0.f, 0.f, 0.f};                                                             \
        if ((s_) % 2 == 0) {                                                                                  \
            d0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av_, pick0, zero_, 0, 0, 0);                         \
            d1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av_, pick1, zero_, 0, 0, 0);                         \
        } else {                                                                                              \
            d0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av_, pick0, d0, 0, 0, 0);                            \
            d1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av_, pick1, d1, 0, 0, 0);                            \
            const float t0_ = (d0[0] + d0[1]) + (d0[2] + d0[3]);                                              \
            const float t1_ = (d1[0] + d1[1]) + (d1[2] + d1[3]);                                              \
            const f32x4 r0_ = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, t0_, zero_, 0, 0, 0);                \
            const f32x4 r1_ = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, t1_, zero_, 0, 0, 0);                \
            const float mine_ = (g & 1) ? r1_[0] : r0_[0];                                                    \
            if (KSW == 1 || (ks_) == KSW - 1) {                                                               \
                const float v_ = (KSW == 2 && lane < 32) ? held[(s_) / 2] : mine_;                            \
                sums[(size_t)min((s_) / 2, F - 1 - grp * FR) * tpf * C + (ks0_) * 32] = v_;                   \
            } else {                                                                                          \
                held[(s_) / 2] = mine_;                                                                       \
            }                                                                                                 \
        }                                                                                                     \
    } while (0)

    // One pass over KN_ (<= KSW) K-steps starting at this wave's K-step ks0_.  (A macro on purpose: with
    // the body in a lambda the same code ran 10 % slower.)
    //  * Anchor fragments run PF K-steps ahead of their use in a ring of PF+1 buffers; the first PF are
    //    requested before the source loads (loads complete in issue order).
    //  * Every source load of the pass is issued before any product (the scheduler would otherwise sink
    //    them to their uses and serialise on HBM latency).
    //  * Fragments are kept as four plain 32-bit words: v_dot2 on elements extracted from a bit-cast
    //    vector was observed to read element 0 four times.
#define TTF_SEARCH_PASS(KN_, ks0_)                                                                            \
    do {                                                                                                      \
        const int ks0 = (ks0_);                                                                               \
        bf16x8 Bt[NB][NA];                                                                                    \
        _Pragma("unroll") for (int d = 0; d < PF && d < (KN_); ++d) {                                         \
            _Pragma("unroll") for (int q = 0; q < NA; ++q)                                                    \
                Bt[d][q] = __builtin_bit_cast(bf16x8,                                                         \
                                              *reinterpret_cast<const u32x4*>(ap[q] + (size_t)(ks0 + d) * 512)); \
        }                                                                                                     \
        u32x4 A[NS][(KN_)];                                                                                   \
        _Pragma("unroll") for (int ks = 0; ks < (KN_); ++ks) {                                                \
            _Pragma("unroll") for (int s = 0; s < NS; ++s)                                                    \
                A[s][ks] = *reinterpret_cast<const u32x4*>(sp[s] + (ks0 + ks) * 32);                          \
        }                                                                                                     \
        __builtin_amdgcn_sched_barrier(0);                                                                    \
        _Pragma("unroll") for (int ks = 0; ks < (KN_); ++ks) {                                                \
            if (ks + PF < (KN_)) {                                                                            \
                _Pragma("unroll") for (int q = 0; q < NA; ++q)                                                \
                    Bt[(ks + PF) % NB][q] = __builtin_bit_cast(                                               \
                        bf16x8, *reinterpret_cast<const u32x4*>(ap[q] + (size_t)(ks0 + ks + PF) * 512));      \
            }                                                                                                 \
            __builtin_amdgcn_sched_barrier(0);                                                                \
            _Pragma("unroll") for (int s = 0; s < NS; ++s) {                                                  \
                uint32_t r[4] = {A[s][ks][0], A[s][ks][1], A[s][ks][2], A[s][ks][3]};                         \
                _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                               \
                    const bf16x2 p = __builtin_bit_cast(bf16x2, r[e]);                                        \
                    nv[s] = __builtin_amdgcn_fdot2_f32_bf16(p, p, nv[s], false);                              \
                }                                                                                             \
                _Pragma("unroll") for (int e = 0; e < 4; ++e)                                                 \
                    r[e] = (uint32_t)__builtin_amdgcn_ds_bpermute(bperm, (int)r[e]);                          \
                const bf16x8 av = __builtin_bit_cast(bf16x8, uint4{r[0], r[1], r[2], r[3]});                  \
                _Pragma("unroll") for (int q = 0; q < NPS; ++q)                                               \
                    acc[s][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(                                      \
                        av, Bt[ks % NB][S::pair_tile(s % 2, q)], acc[s][q], 0, 0, 0);                         \
                if constexpr (SPEC == 1) TTF_STRIP_SUM_STEP(av, s, ks, ks0);                                  \
            }                                                                                                 \
            __builtin_amdgcn_sched_barrier(0);                                                                \
        }                                                                                                     \
    } while (0)

    if constexpr (RAG) {
        static_assert(KSW == 2, "one leftover K-step at most");
        const int whole = ks_mine / KSW;                     // wave-uniform
        for (int pass = 0; pass < whole; ++pass) TTF_SEARCH_PASS(KSW, pass * KSW);
        if (ks_mine % KSW) TTF_SEARCH_PASS(1, whole * KSW);
    } else {
        for (int pass = 0; pass < passes; ++pass) TTF_SEARCH_PASS(KSW, pass * KSW);
    }

#undef TTF_SEARCH_PASS
#undef TTF_STRIP_SUM_STEP

    // squared-norm partials: lanes 4i..4i+3 hold the four chunks of token i
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        nv[s] += __shfl_xor(nv[s], 1, 64);
        nv[s] += __shfl_xor(nv[s], 2, 64);
    }
    // a slot is live when it is a real frame of the clip whose outputs this search owns (in the
    // speculative pass the anchor frame is walked for its sums only)
    auto slot_live = [&](int s) {
        const int si = grp * FR + s / 2;
        return si < nsrc && (SPEC != 1 || si != a_in);
    };
    if constexpr (NW == 1) {
        // one wave owns the whole channel axis: its sums are final, the epilogue needs no LDS
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            float nn[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) nn[j] = __shfl(nv[s], 4 * (4 * g + j), 64);
            finish_tile<CT, RAD, ALL>(acc[s], nn, s, slot_live(s), min(grp * FR + s / 2, nsrc - 1),
                                      a_skip, b, F, H, i0, t, ai_tile, fuse_map, best_sim, best_idx, keep16, win_sim, lane);
        }
    } else {
        // ---- add the channel slices through LDS (wave order), RT source tiles per round ----
        __shared__ f32x4 red[NW][RT][NPS][64];
        __shared__ float rnv[NW][RT][64];
#pragma unroll
        for (int round = 0; round < NS / RT; ++round) {
#pragma unroll
            for (int sl = 0; sl < RT; ++sl) {
                const int s = round * RT + sl;
                rnv[wave][sl][lane] = nv[s];
#pragma unroll
                for (int q = 0; q < NPS; ++q) red[wave][sl][q][lane] = acc[s][q];
            }
            __syncthreads();
            if (wave < RT) {
                // (straight-line code from here on: one wave runs this while the others wait, so
                // every divergent branch would be paid in full)
                const int sl = wave;
                const int s = round * RT + sl;                   // wave-uniform
                float nn[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    nn[j] = rnv[0][sl][4 * (4 * g + j)];
#pragma unroll
                    for (int w = 1; w < NW; ++w) nn[j] += rnv[w][sl][4 * (4 * g + j)];
                }
                f32x4 v[NPS];
#pragma unroll
                for (int q = 0; q < NPS; ++q) {
                    v[q] = red[0][sl][q][lane];
#pragma unroll
                    for (int w = 1; w < NW; ++w) {
                        const f32x4 p = red[w][sl][q][lane];
                        v[q][0] += p[0]; v[q][1] += p[1]; v[q][2] += p[2]; v[q][3] += p[3];
                    }
                }
                finish_tile<CT, RAD, ALL>(v, nn, s, slot_live(s), min(grp * FR + s / 2, nsrc - 1),
                                          a_skip, b, F, H, i0, t, ai_tile, fuse_map, best_sim, best_idx, keep16, win_sim,
                                          lane);
            }
            __syncthreads();
        }
    }
}

// Variant for shapes with many anchor tiles per source tile (5x5 window on a 32-wide grid: 10 anchor
// tiles per K-step).  With two frames per wave the accumulators leave room for one wave per SIMD
// only and nothing hides memory latency; with one frame per one-wave workgroup every workgroup
// would fetch five times its source bytes in anchor fragments.  Here the 4 waves of a workgroup
// work on the same 32-cell strip in 4*FW consecutive source frames (FW frames each, whole channel
// axis, wave-local epilogue) and share the anchor fragments through LDS, which keeps the register
// count at two waves per SIMD.  Loads complete in issue order, so the pipeline is arranged such
// that the loads a wave has to wait for are always its oldest: per pass of KSW K-steps a wave
// stores the anchor fragments it requested one pass ago to the idle LDS buffer, requests its share
// of the anchor fragments of the pass after next and then the source fragments two passes ahead,
// and computes the current pass from LDS and registers.
// PAD: grids narrower than the tile row (Wg <= 16*CT) and of any height; see finish_tile.
// SPEC: as for k_search_mfma (1: speculative pass -- every frame walked, strip sums written, clips
// without a trusted guess skipped; 2: second search of the marked clips only).
// RAG: the K-step count need not be a multiple of KSW; the slots of the last pass beyond it read the
// last K-step again (valid memory) with the source fragment replaced by zeros.
template <int CT, int RAD, int KSW, int FW, bool ALL, bool PAD = false, int SPEC = 0, bool RAG = false>
__global__ __launch_bounds__(256, 2) void k_search_mfma_shared(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ anchor_frag,
    const int32_t* __restrict__ anchor_index, const float* __restrict__ anchor_inv,
    int32_t* __restrict__ fuse_map, float* __restrict__ best_sim, int32_t* __restrict__ best_idx,
    uint16_t* __restrict__ keep16, float* __restrict__ win_sim, int F, int H, int C, float t, int groups, int Wg,
    const int32_t* __restrict__ spec, float* __restrict__ strip_sum)
{
    static_assert(SPEC == 0 || (!ALL && KSW <= 2 && !RAG), "speculative pass: plain outputs, whole passes");
    using S = Shape<CT, RAD>;
    constexpr int W = S::W, NA = S::NA, NPS = S::NPS;
    constexpr int NS = 2 * FW;                               // source tiles per wave (FW frames)
    constexpr int FRG = 4 * FW;                              // frames per workgroup
    constexpr int GL = KSW * NA / 4;                         // anchor fragments each wave stages per pass
    static_assert((KSW * NA) % 4 == 0, "anchor fragments divide over the four waves");
    extern __shared__ u32x4 frag_lds[];                      // [2][KSW][NA][64]
    static_assert(PAD || CT <= 2, "wider grids only through the padded path");
    const int N = PAD ? H * Wg : H * W;                      // tokens per frame
    const int CTt = CT <= 2 ? CT : (Wg + 15) / 16;           // column tiles per grid row
    const int NT = H * CTt;                                  // anchor tiles per frame (tile rows x column tiles)
    const int spr = (CTt + 1) / 2;                           // strips per grid row (CT == 3)
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: keeps per-wave offsets scalar
    const int m = lane & 15, g = lane >> 4;
    const int tpf = PAD ? (CT == 1 ? (H + 1) / 2 : (CT == 2 ? H : H * spr)) : N / 32;   // 32-cell strips per frame
    int tp, grp, b;                                          // same XCD-aware mapping as k_search_mfma
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
    if constexpr (SPEC == 1) {
        if (spec[4 * b + 1] == 0) return;                    // no trusted guess: the clip takes the two-pass route
    }
    if constexpr (SPEC == 2) {
        if (spec[4 * b + 2] == 0) return;                    // guess confirmed: nothing to redo
    }
    const int a_in = anchor_index[b];
    const int a = (SPEC == 1 || a_in < 0) ? 0x7fffffff : a_in;   // the speculative pass walks the anchor frame too
    const int nsrc = (SPEC == 1 || a_in < 0) ? F : F - 1;
    // first source row y0 and first column tile c0 of the strip; i0 = y0 * W is what finish_tile decodes
    const int y0 = CT == 3 ? tp / spr : tp * 32 / W;
    const int c0 = CT == 3 ? 2 * (tp % spr) : 0;
    const int i0 = CT == 3 ? y0 * W : tp * 32;
    const int ylo = y0 - RAD;
    const int KS = C / 32;
    const int passes = RAG ? (KS + KSW - 1) / KSW : KS / KSW;

    const uint16_t* sp[NS];
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
        sp[s] = x + (((size_t)b * F + k) * N + cell) * (size_t)C + (lane & 3) * 8;
    }
    const int bperm = (4 * m + g) * 4;
    // this wave's share of a pass's anchor fragments: fragment e = wave + 4*i is (K-step e / NA, tile
    // e % NA); offsets are wave-uniform (scalar registers), the lane part is added at the access
    const uint16_t* gbase = anchor_frag + (size_t)b * NT * KS * 512 + lane * 8;
    int goff[GL], gslot[GL];
#pragma unroll
    for (int i = 0; i < GL; ++i) {
        const int e = wave + 4 * i, ks = e / NA, q = e % NA;
        const int yy = min(max(ylo + S::tile_row(q), 0), H - 1);
        const int tile = yy * CTt + min(max(c0 + S::tile_col(q), 0), CTt - 1);   // outside the grid: clamped, masked later
        goff[i] = RAG ? tile * KS : (tile * KS + ks) * 512;      // RAG: in K-steps, the pass's K-step is added (clamped) at the access
        gslot[i] = (ks * NA + q) * 64;
    }

    f32x4 acc[NS][NPS];
    float nv[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        nv[s] = 0.f;
#pragma unroll
        for (int q = 0; q < NPS; ++q) acc[s][q] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    u32x4 A[3][NS][KSW];                                     // native vectors: plain SSA values, never memory
    u32x4 G[GL];
    // (macros, not lambdas: captured by a lambda the staged fragments were kept in scratch memory)
#define TTF_REQUEST_ANCHOR(pass_)                                                                             \
    do {                                                                                                      \
        const int pq = min((pass_), passes - 1);                                                              \
        _Pragma("unroll") for (int i = 0; i < GL; ++i)                                                        \
            G[i] = *reinterpret_cast<const u32x4*>(                                                           \
                gbase + (RAG ? (goff[i] + min(pq * KSW + (wave + 4 * i) / NA, KS - 1)) * 512                  \
                             : goff[i] + pq * (KSW * 512)));                                                  \
    } while (0)
#define TTF_REQUEST_SOURCE(pass_, Abuf)                                                                       \
    do {                                                                                                      \
        const int pq = min((pass_), passes - 1);                                                              \
        _Pragma("unroll") for (int ks = 0; ks < KSW; ++ks) {                                                  \
            _Pragma("unroll") for (int s = 0; s < NS; ++s)                                                    \
                Abuf[s][ks] = *reinterpret_cast<const u32x4*>(                                                \
                    sp[s] + (RAG ? min(pq * KSW + ks, KS - 1) : pq * KSW + ks) * 32);                         \
        }                                                                                                     \
    } while (0)
#define TTF_STAGE(buf_)                                                                                       \
    do {                                                                                                      \
        _Pragma("unroll") for (int i = 0; i < GL; ++i)                                                        \
            frag_lds[(buf_) * (KSW * NA * 64) + gslot[i] + lane] = G[i];                                      \
    } while (0)
    // speculative pass: channel pickers, where this lane's strip sums go (as in k_search_mfma; here a
    // wave owns whole frames and the whole channel axis), and the first K-step's totals of a pass
    bf16x8 pick0, pick1;
    float* sums = nullptr;
    float held[FW];
    bool pad_cell[2] = {false, false};                       // PAD: operand lane m of tile kind u holds a padding cell
    if constexpr (SPEC == 1) {
        pick0 = channel_picker(0, lane);
        pick1 = channel_picker(1, lane);
        const int k0 = min(grp * FRG + wave * FW, F - 1);
        sums = strip_sum + ((((size_t)b * F + k0) * tpf + tp) * (size_t)C) + (KSW == 2 ? lane : (lane & 31));
        if constexpr (PAD) {
            // padding cells were pointed at a real token (their results are dropped); in the strip sums
            // they must count as zero
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int ys = y0 + (CT == 1 ? u : 0);
                const int xs = (CT == 1 ? 0 : 16 * (c0 + u)) + m;
                pad_cell[u] = ys >= H || xs >= Wg;
            }
        }
    }
    auto compute = [&](int buf, const u32x4 (&Abuf)[NS][KSW], int ks0) {
#pragma unroll
        for (int ks = 0; ks < KSW; ++ks) {
            bf16x8 av[NS];                                   // source tiles in operand order
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                uint32_t r[4] = {Abuf[s][ks][0], Abuf[s][ks][1], Abuf[s][ks][2], Abuf[s][ks][3]};
                if constexpr (RAG) {                             // a slot past the last K-step adds nothing
                    const bool real = ks0 + ks < KS;             // wave-uniform
#pragma unroll
                    for (int e = 0; e < 4; ++e) r[e] = real ? r[e] : 0u;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bf16x2 p = __builtin_bit_cast(bf16x2, r[e]);
                    nv[s] = __builtin_amdgcn_fdot2_f32_bf16(p, p, nv[s], false);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) r[e] = (uint32_t)__builtin_amdgcn_ds_bpermute(bperm, (int)r[e]);
                if constexpr (PAD && SPEC == 1) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) r[e] = pad_cell[s % 2] ? 0u : r[e];
                }
                av[s] = __builtin_bit_cast(bf16x8, uint4{r[0], r[1], r[2], r[3]});
            }
            // one anchor tile at a time from LDS, used by every source tile paired with it
#pragma unroll
            for (int qa = 0; qa < NA; ++qa) {
                const bf16x8 bt = __builtin_bit_cast(bf16x8, frag_lds[buf * (KSW * NA * 64) + (ks * NA + qa) * 64 + lane]);
#pragma unroll
                for (int s = 0; s < NS; ++s) {
#pragma unroll
                    for (int q = 0; q < NPS; ++q) {              // the pair (if any) of this source tile that uses tile qa
                        if (S::pair_tile(s % 2, q) == qa)
                            acc[s][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[s], bt, acc[s][q], 0, 0, 0);
                    }
                }
            }
            if constexpr (SPEC == 1) {
                // strip sums of this K-step: tokens x channels of both tiles of a frame through the channel
                // pickers, four in-lane adds, the four row groups by an fp32 MFMA against ones; one
                // 256-byte store per frame and pass (lanes 0..31 first K-step, 32..63 second).  A slot past
                // the clip's end repeats the last frame and stores the same values to the same place.
#pragma unroll
                for (int f = 0; f < FW; ++f) {
                    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
                    f32x4 d0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[2 * f], pick0, zero, 0, 0, 0);
                    f32x4 d1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[2 * f], pick1, zero, 0, 0, 0);
                    d0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[2 * f + 1], pick0, d0, 0, 0, 0);
                    d1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[2 * f + 1], pick1, d1, 0, 0, 0);
                    const float t0 = (d0[0] + d0[1]) + (d0[2] + d0[3]);
                    const float t1 = (d1[0] + d1[1]) + (d1[2] + d1[3]);
                    const f32x4 r0 = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, t0, zero, 0, 0, 0);
                    const f32x4 r1 = __builtin_amdgcn_mfma_f32_16x16x4f32(1.0f, t1, zero, 0, 0, 0);
                    const float mine = (g & 1) ? r1[0] : r0[0];
                    if (KSW == 1 || ks == KSW - 1) {
                        const float v = (KSW == 2 && lane < 32) ? held[f] : mine;
                        const int k0 = min(grp * FRG + wave * FW, F - 1);
                        sums[(size_t)(min(k0 + f, F - 1) - k0) * tpf * C + ks0 * 32] = v;
                    } else {
                        held[f] = mine;
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);               // keep the K-steps apart: bounded live ranges
        }
    };

    // State at the top of pass p: LDS buffer p%2 holds the anchor fragments of pass p; the source
    // fragments of passes p and p+1 (A[p%3], A[(p+1)%3]) and the anchor fragments of pass p+1 (G) are
    // already requested.  Every value is used in a later iteration than the one that requested it,
    // so no load can be moved next to its use; the anchor loads waited for are always older than
    // the source loads that may still be in flight, which therefore stay in flight (two passes of
    // source data per wave) across the wait.
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
        compute(pp & 1, A[(j)], pp * KSW);                            \
        __builtin_amdgcn_sched_barrier(0);                            \
        lds_barrier();                                                \
    } while (0)
    for (int pass = 0; pass < passes; pass += 3) {
        TTF_PASS(0);
        if (pass + 1 < passes) TTF_PASS(1);                  // wave-uniform
        if (pass + 2 < passes) TTF_PASS(2);
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
        // (in the speculative pass the anchor frame is walked for its sums only)
        finish_tile<CT, RAD, ALL, PAD>(acc[s], nn, s, si < nsrc && (SPEC != 1 || si != a_in), min(si, nsrc - 1), a, b, F,
                                       H, i0, t, ai_tile, fuse_map, best_sim, best_idx, keep16, win_sim, lane, Wg, c0);
    }
}

// True when launch_shape<CT, RAD> runs k_search_mfma (and not the LDS-shared kernel) on this
// problem: the kernel that can also write strip sums.
template <int CT, int RAD>
bool shape_uses_plain_kernel(const ttf_params& p, int nsrc)
{
    using S = Shape<CT, RAD>;
    if constexpr (S::NPS > 6) {
        const int groups8 = (nsrc + 3) / 4;
        const size_t wgs = (size_t)p.B * groups8 * (p.H * p.W / 32);
        if (wgs >= 2 * 256 && (p.C / 32) % 2 == 0) return false;
    }
    return true;
}

// spec_mode 0: plain search.  1: speculative pass (every frame walked, strip sums written).  2: plain
// search restricted to the clips marked for a second search.
template <int CT, int RAD>
hipError_t launch_shape(const ttf_params& p, const void* x, bool external_anchor, const Workspace& w,
                        const int32_t* anchor_index, int32_t* fuse_map, float* best_sim, int32_t* best_idx,
                        float* win_sim, int spec_mode, hipStream_t s)
{
    using S = Shape<CT, RAD>;
    const int nsrc = (external_anchor || spec_mode == 1) ? p.F : p.F - 1;   // frames walked per clip
    if (nsrc < 1) return hipSuccess;                         // no source frame: the anchor rows are all there is
    const uint16_t* xs = static_cast<const uint16_t*>(x);
    const int N = p.H * p.W;
    const int groups = (nsrc + S::FR - 1) / S::FR;           // groups of source frames per clip
    const size_t blocks = (size_t)p.B * groups * (N / 32);
    const unsigned grid = (unsigned)blocks;
    const int ks_total = p.C / 32;                           // K-steps per token
    uint16_t* keep16 = reinterpret_cast<uint16_t*>(w.keep_bits);
    if (spec_mode != 0 && shape_uses_plain_kernel<CT, RAD>(p, p.F - 1)) {
        // the speculative path is for large inputs: the two layouts that serve those, nothing else
        if (win_sim) return hipErrorInvalidValue;
#define TTF_LAUNCH_SPEC(KSW, NW, SPEC)                                                                            \
    k_search_mfma<CT, RAD, KSW, NW, false, 0, SPEC><<<grid, NW * 64, 0, s>>>(                                     \
        xs, w.anchor_frag, anchor_index, w.anchor_inv, fuse_map, best_sim, best_idx, keep16, nullptr, p.F, p.H, p.C, \
        p.t, ks_total / (NW * KSW), groups, w.spec, w.strip_sum)
#define TTF_LAUNCH_SPEC_AS(KSW, NW)                        \
    do {                                                   \
        if (spec_mode == 1) TTF_LAUNCH_SPEC(KSW, NW, 1);   \
        else TTF_LAUNCH_SPEC(KSW, NW, 2);                  \
    } while (0)
#define TTF_LAUNCH_SPEC_RAG(SPEC)                                                                                 \
    k_search_mfma<CT, RAD, 2, 4, false, 0, SPEC, true><<<grid, 256, 0, s>>>(                                      \
        xs, w.anchor_frag, anchor_index, w.anchor_inv, fuse_map, best_sim, best_idx, keep16, nullptr, p.F, p.H, p.C, \
        p.t, 0 /* passes: the waves count their own */, groups, w.spec, w.strip_sum)
        if (blocks >= 3 * kSimds * S::OCC && ks_total % 2 == 0) TTF_LAUNCH_SPEC_AS(2, 1);
        else if (ks_total % 8 == 0) TTF_LAUNCH_SPEC_AS(2, 4);
        else if (spec_mode == 1) TTF_LAUNCH_SPEC_RAG(1);     // (C % 256 == 128: passes dealt unevenly, none short)
        else TTF_LAUNCH_SPEC_RAG(2);
#undef TTF_LAUNCH_SPEC_RAG
#undef TTF_LAUNCH_SPEC_AS
#undef TTF_LAUNCH_SPEC
        return hipGetLastError();
    }
    if constexpr (S::NPS > 6) {
        // many anchor tiles per source tile (32-wide grid, 5x5 window): workgroups of 4 waves x 1 frame
        // sharing the anchor fragments in LDS, as soon as there are enough of them to cover the chip
        // twice (measured on B4 F64 32x32 C4096 r2: 0.48-0.52 ms against 0.58-0.60 ms for one-wave
        // workgroups; for the smaller windows the split-channel kernel below is as fast or faster)
        constexpr int FWS = 1;                               // frames per wave
        const int nsrc_plain = external_anchor ? p.F : p.F - 1;   // (the route does not depend on the pass kind)
        const int groups8 = (nsrc_plain + 4 * FWS - 1) / (4 * FWS);
        const size_t wgs = (size_t)p.B * groups8 * (N / 32);
        constexpr int KSWS = 2;                              // K-steps per pass of the shared-anchor kernel
        if (wgs >= 2 * 256 && ks_total % KSWS == 0) {
            const size_t lds = 2 * KSWS * (size_t)S::NA * 1024;
            auto go = [&](auto kernel, int frames) {
                const int groups_ = (frames + 4 * FWS - 1) / (4 * FWS);
                const size_t wgs_ = (size_t)p.B * groups_ * (N / 32);
                hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kernel), lds);
                if (e != hipSuccess) return e;
                kernel<<<(unsigned)wgs_, 256, lds, s>>>(xs, w.anchor_frag, anchor_index, w.anchor_inv, fuse_map,
                                                        best_sim, best_idx, keep16, win_sim, p.F, p.H, p.C, p.t, groups_,
                                                        p.W, w.spec, w.strip_sum);
                return hipGetLastError();
            };
            if (spec_mode == 1) return go(k_search_mfma_shared<CT, RAD, KSWS, FWS, false, false, 1>, p.F);
            if (spec_mode == 2) return go(k_search_mfma_shared<CT, RAD, KSWS, FWS, false, false, 2>, p.F - 1);
            return win_sim ? go(k_search_mfma_shared<CT, RAD, KSWS, FWS, true>, nsrc)
                           : go(k_search_mfma_shared<CT, RAD, KSWS, FWS, false>, nsrc);
        }
    }
#define TTF_LAUNCH_AS(KSW, NW, ALL)                                                                           \
    k_search_mfma<CT, RAD, KSW, NW, ALL><<<grid, NW * 64, 0, s>>>(xs, w.anchor_frag, anchor_index, w.anchor_inv,  \
                                                                  fuse_map, best_sim, best_idx, keep16, win_sim,  \
                                                                  p.F, p.H, p.C, p.t, ks_total / (NW * KSW), groups,  \
                                                                  nullptr, nullptr)
#define TTF_LAUNCH(KSW, NW)                   \
    do {                                      \
        if (win_sim) TTF_LAUNCH_AS(KSW, NW, true); \
        else TTF_LAUNCH_AS(KSW, NW, false);   \
    } while (0)
    // (ragged: each wave takes ceil(K-steps / NW) K-steps, in passes of KSW)
#define TTF_LAUNCH_RAG_AS(KSW, NW, ALL)                                                                       \
    k_search_mfma<CT, RAD, KSW, NW, ALL, 0, 0, true><<<grid, NW * 64, 0, s>>>(                                    \
        xs, w.anchor_frag, anchor_index, w.anchor_inv, fuse_map, best_sim, best_idx, keep16, win_sim, p.F, p.H,   \
        p.C, p.t, 0 /* passes: the waves count their own */, groups, nullptr, nullptr)
#define TTF_LAUNCH_RAG(KSW, NW)                       \
    do {                                              \
        if (win_sim) TTF_LAUNCH_RAG_AS(KSW, NW, true); \
        else TTF_LAUNCH_RAG_AS(KSW, NW, false);       \
    } while (0)
    // With several rounds of workgroups per wave slot, one wave per workgroup walks the whole
    // channel axis (no cross-wave sum, no LDS).  With fewer, such long-running single waves
    // leave SIMDs unevenly loaded (measured: 0.24 ms against 0.20 ms on 1024 workgroups), so the
    // channels are split over four waves instead.
    if (blocks < 256 && ks_total % 32 == 0) {
        // fewer workgroups than CUs: one source frame per workgroup (up to FR times the workgroups)
        // and 8 K-steps per pass, so that a workgroup waits for memory C/1024 times instead of C/256
        // times (B1 F32 16x16 C2048: 0.024 -> 0.013 ms; anchor fragments come from L2 either way)
        const unsigned grid1 = (unsigned)((size_t)p.B * nsrc * (N / 32));
        if (win_sim)
            k_search_mfma<CT, RAD, 8, 4, true, 1><<<grid1, 256, 0, s>>>(xs, w.anchor_frag, anchor_index, w.anchor_inv,
                                                                        fuse_map, best_sim, best_idx, keep16, win_sim,
                                                                        p.F, p.H, p.C, p.t, ks_total / 32, nsrc, nullptr,
                                                                        nullptr);
        else
            k_search_mfma<CT, RAD, 8, 4, false, 1><<<grid1, 256, 0, s>>>(xs, w.anchor_frag, anchor_index, w.anchor_inv,
                                                                         fuse_map, best_sim, best_idx, keep16, win_sim,
                                                                         p.F, p.H, p.C, p.t, ks_total / 32, nsrc, nullptr,
                                                                        nullptr);
    } else if (blocks >= 3 * kSimds * S::OCC && S::OCC == 1 && ks_total % 4 == 0) TTF_LAUNCH(4, 1);
    else if (blocks >= 3 * kSimds * S::OCC && ks_total % 2 == 0) TTF_LAUNCH(2, 1);
    else if (blocks >= 3 * kSimds * S::OCC) TTF_LAUNCH_RAG(2, 1);     // odd K-step count
    else if (ks_total % 8 == 0) TTF_LAUNCH(2, 4);
    else TTF_LAUNCH_RAG(2, 4);                                       // K-steps that do not divide into 4 waves x 2-step passes
#undef TTF_LAUNCH
#undef TTF_LAUNCH_AS
#undef TTF_LAUNCH_RAG
#undef TTF_LAUNCH_RAG_AS
    return hipGetLastError();
}

// Keep words from the fuse map (padded grids): bit i of frame (b,k) is set iff the token is an
// anchor token or was not fused.  One wave per 64-token word.
__global__ __launch_bounds__(256) void k_pack_keep(const int32_t* __restrict__ fuse_map,
                                                   const int32_t* __restrict__ anchor_index,
                                                   uint64_t* __restrict__ keep_bits, int F, int N, int NW, size_t words)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t wd = (size_t)blockIdx.x * 4 + wave;
    if (wd >= words) return;
    const size_t frame = wd / NW;
    const int i = (int)(wd % NW) * 64 + lane;
    const int b = (int)(frame / F), k = (int)(frame % F);
    const bool keep = i < N && (k == anchor_index[b] || fuse_map[frame * (size_t)N + i] < 0);
    const uint64_t bits = __ballot(keep);
    if (lane == 0) keep_bits[wd] = bits;
}

// Grids that are not exactly 16 or 32 wide (or whose height does not make whole keep words): the
// LDS-shared kernel on tile rows padded to whole 16-column tiles.
template <int CT, int RAD>
hipError_t launch_padded(const ttf_params& p, const void* x, bool external_anchor, const Workspace& w,
                         const int32_t* anchor_index, int32_t* fuse_map, float* best_sim, int32_t* best_idx,
                         float* win_sim, int spec_mode, hipStream_t s)
{
    using S = Shape<CT, RAD>;
    const int nsrc = (external_anchor || spec_mode == 1) ? p.F : p.F - 1;   // frames walked per clip
    const int N = p.H * p.W, NW = (N + 63) / 64;
    const size_t words = (size_t)p.B * p.F * NW;
    if (nsrc >= 1) {
        constexpr int FWS = S::NPS <= 3 ? 2 : 1, KSWS = 2;
        const int groups = (nsrc + 4 * FWS - 1) / (4 * FWS);
        const int strips = CT == 1 ? (p.H + 1) / 2 : (CT == 2 ? p.H : p.H * (((p.W + 15) / 16 + 1) / 2));
        const size_t wgs = (size_t)p.B * groups * strips;
        const size_t lds = 2 * KSWS * (size_t)S::NA * 1024;
        auto go = [&](auto kernel) {
            hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kernel), lds);
            if (e != hipSuccess) return e;
            kernel<<<(unsigned)wgs, 256, lds, s>>>(static_cast<const uint16_t*>(x), w.anchor_frag, anchor_index,
                                                   w.anchor_inv, fuse_map, best_sim, best_idx, nullptr, win_sim, p.F,
                                                   p.H, p.C, p.t, groups, p.W, w.spec, w.strip_sum);
            return hipGetLastError();
        };
        const bool ragged = (p.C / 32) % KSWS != 0;          // odd K-step count: the variant with a guarded last pass
        {
            // speculative pass (every frame walked, strip sums written; the keep words are packed after the
            // last search of the call), and the second search of the clips it leaves
            if (spec_mode == 1) return (win_sim || ragged) ? hipErrorInvalidValue
                                                           : go(k_search_mfma_shared<CT, RAD, KSWS, FWS, false, true, 1>);
            if (spec_mode == 2) {
                if (win_sim || ragged) return hipErrorInvalidValue;
                const hipError_t e2 = go(k_search_mfma_shared<CT, RAD, KSWS, FWS, false, true, 2>);
                if (e2 != hipSuccess) return e2;
                k_pack_keep<<<(unsigned)((words + 3) / 4), 256, 0, s>>>(fuse_map, anchor_index, w.keep_bits, p.F, N, NW,
                                                                        words);
                return hipGetLastError();
            }
        }
        if (spec_mode != 0) return hipErrorInvalidValue;
        const hipError_t e =
            ragged ? (win_sim ? go(k_search_mfma_shared<CT, RAD, KSWS, FWS, true, true, 0, true>)
                              : go(k_search_mfma_shared<CT, RAD, KSWS, FWS, false, true, 0, true>))
                   : (win_sim ? go(k_search_mfma_shared<CT, RAD, KSWS, FWS, true, true>)
                              : go(k_search_mfma_shared<CT, RAD, KSWS, FWS, false, true>));
        if (e != hipSuccess) return e;
    }
    if (win_sim) return hipSuccess;                          // tied-batch mode: the tie kernel forms the keep words
    k_pack_keep<<<(unsigned)((words + 3) / 4), 256, 0, s>>>(fuse_map, anchor_index, w.keep_bits, p.F, N, NW, words);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_pack_keep(const ttf_params& p, const int32_t* fuse_map, const int32_t* anchor_index,
                            const Workspace& w, hipStream_t s)
{
    const int N = p.H * p.W, NW = (N + 63) / 64;
    const size_t words = (size_t)p.B * p.F * NW;
    k_pack_keep<<<(unsigned)((words + 3) / 4), 256, 0, s>>>(fuse_map, anchor_index, w.keep_bits, p.F, N, NW, words);
    return hipGetLastError();
}

// True when the matrix-core kernels cover this problem: bf16, grid width 16 or 32, radius <= 2,
// channel count a multiple of 32 (whole K-steps; where they do not divide over waves and passes the
// ragged variants run), and a token count per frame that is a multiple of 64 so that 64-bit keep
// words are whole.
bool mfma_search_supported(const ttf_params& p)
{
    if (p.dtype != TTF_BF16 || p.r > 2 || p.C % 32 != 0) return false;
    if (p.W == 16) return p.H % 4 == 0;
    if (p.W == 32) return p.H % 2 == 0;
    return false;
}

// Same element type, radius and channel conditions, but any grid: served by the padded-tile
// kernels.
bool mfma_search_padded(const ttf_params& p)
{
    if (p.dtype != TTF_BF16 || p.r > 2 || p.C % 32 != 0) return false;
    // the padded kernels index a clip's anchor fragments with 32-bit offsets
    const long long padded_tokens = (long long)p.H * ((p.W + 15) / 16) * 16;
    if (padded_tokens * p.C >= (1ll << 31)) return false;
    return !mfma_search_supported(p);
}

// True when the speculative anchor path can run this problem's search.
bool mfma_search_speculative(const ttf_params& p)
{
    return (mfma_search_supported(p) || mfma_search_padded(p)) && speculation_shape(p) && p.F >= 2;
}

hipError_t launch_window_search_mfma(const ttf_params& p, const void* x, bool external_anchor, const Workspace& w,
                                     const int32_t* anchor_index, int32_t* fuse_map, float* best_sim,
                                     int32_t* best_idx, float* win_sim, int spec_mode, hipStream_t s)
{
    if (mfma_search_padded(p)) {
        const int ct = p.W <= 16 ? 1 : (p.W <= 32 ? 2 : 3);
#define TTF_PCASE(CT, RAD)                              \
    if (ct == CT && p.r == RAD)                         \
    return launch_padded<CT, RAD>(p, x, external_anchor, w, anchor_index, fuse_map, best_sim, best_idx, win_sim, \
                                  spec_mode, s)
        TTF_PCASE(1, 0);
        TTF_PCASE(1, 1);
        TTF_PCASE(1, 2);
        TTF_PCASE(2, 0);
        TTF_PCASE(2, 1);
        TTF_PCASE(2, 2);
        TTF_PCASE(3, 0);
        TTF_PCASE(3, 1);
        TTF_PCASE(3, 2);
#undef TTF_PCASE
        return hipErrorInvalidValue;
    }
#define TTF_CASE(CT, RAD)             \
    if (p.W == 16 * CT && p.r == RAD) \
    return launch_shape<CT, RAD>(p, x, external_anchor, w, anchor_index, fuse_map, best_sim, best_idx, win_sim, \
                                 spec_mode, s)
    TTF_CASE(1, 0);
    TTF_CASE(1, 1);
    TTF_CASE(1, 2);
    TTF_CASE(2, 0);
    TTF_CASE(2, 1);
    TTF_CASE(2, 2);
#undef TTF_CASE
    return hipErrorInvalidValue;
}

}  // namespace ttf
