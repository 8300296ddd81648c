// Anchor frame selection (Section 3, "Anchor Frame Selection"):
//   a* = argmax_k cos( (1/N) sum_i x_{k,i} , (1/(FN)) sum_{k',i} x_{k',i} )
// The cosine does not change when either argument is scaled, so the kernels work with plain
// sums: frame sums in fp32 (one streaming pass over X, the only large read of this stage),
// everything after that in fp64 on [B,F,C] numbers.  The last kernel of the stage picks the arg
// max (lowest k on ties) and computes 1/||x_{a,j}|| for the anchor tokens, which the window
// search uses as the anchor half of every cosine denominator.
#include <type_traits>

#include "ttf_device.h"
#include "ttf_internal.h"

namespace ttf {
namespace {

constexpr int kAnchorGiven = -2;   // "fixed_anchor" value: the anchor of every clip is already in anchor_index

// One block = one frame x one slice of 64*V channels.  Wave w adds rows w, w+4, ...; the four
// partial sums are combined through LDS in wave order, so the result is order-stable.
// `spec` (may be null): per clip {guessed anchor, guess trusted, ...}; clips with a trusted guess get
// their exact sums from the search and are skipped here.
template <typename T, int V>
__global__ __launch_bounds__(256) void k_frame_sums(const T* __restrict__ x, float* __restrict__ frame_sum,
                                                    int N, int C, int F, const int32_t* __restrict__ spec)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t frame = blockIdx.x;
    if (spec && spec[4 * (frame / F) + 1]) return;
    const int c0 = (blockIdx.y * 64 + lane) * V;
    __shared__ float part[4][64 * V];
    float acc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = 0.f;
    if (c0 < C) {
        const T* base = x + frame * (size_t)N * C + c0;
        int i = wave;
        for (; i + 12 < N; i += 16) {          // four rows in flight per wave
            RowVec<T, V> r0, r1, r2, r3;
            r0.template load<true>(base + (size_t)i * C);
            r1.template load<true>(base + (size_t)(i + 4) * C);
            r2.template load<true>(base + (size_t)(i + 8) * C);
            r3.template load<true>(base + (size_t)(i + 12) * C);
#pragma unroll
            for (int e = 0; e < V; ++e) acc[e] += r0.v[e];
#pragma unroll
            for (int e = 0; e < V; ++e) acc[e] += r1.v[e];
#pragma unroll
            for (int e = 0; e < V; ++e) acc[e] += r2.v[e];
#pragma unroll
            for (int e = 0; e < V; ++e) acc[e] += r3.v[e];
        }
        for (; i < N; i += 4) {
            RowVec<T, V> r0;
            r0.template load<true>(base + (size_t)i * C);
#pragma unroll
            for (int e = 0; e < V; ++e) acc[e] += r0.v[e];
        }
    }
#pragma unroll
    for (int e = 0; e < V; ++e) part[wave][lane * V + e] = acc[e];
    __syncthreads();
    if (wave == 0 && c0 < C) {
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const int q = lane * V + e;
            frame_sum[frame * (size_t)C + c0 + e] = ((part[0][q] + part[1][q]) + part[2][q]) + part[3][q];
        }
    }
}

// The same sums for rows that are whole 4 KiB slabs: a block owns one frame and one slab, every
// thread its 16 bytes of the slab for all N rows (eight rows in flight), so the four waves of a block
// read 4 KiB of one row together and no cross-wave sum is needed.
template <typename T, int V>
__global__ __launch_bounds__(256) void k_frame_sums_slab(const T* __restrict__ x, float* __restrict__ frame_sum,
                                                         int N, int C, int F, const int32_t* __restrict__ spec)
{
    const size_t frame = blockIdx.x;
    if (spec && spec[4 * (frame / F) + 1]) return;
    const int c0 = (blockIdx.y * 256 + threadIdx.x) * V;
    const T* base = x + frame * (size_t)N * C + c0;
    float acc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = 0.f;
    int i = 0;
    for (; i + 8 <= N; i += 8) {
        RowVec<T, V> r[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) r[u].template load<true>(base + (size_t)(i + u) * C);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
#pragma unroll
            for (int e = 0; e < V; ++e) acc[e] += r[u].v[e];
        }
    }
    for (; i < N; ++i) {
        RowVec<T, V> r0;
        r0.template load<true>(base + (size_t)i * C);
#pragma unroll
        for (int e = 0; e < V; ++e) acc[e] += r0.v[e];
    }
#pragma unroll
    for (int e = 0; e < V; ++e) frame_sum[frame * (size_t)C + c0 + e] = acc[e];
}

// Per clip and 256-channel slice, in fp64: the clip sum g = sum_k frame_sum[k] (k ascending inside
// each of sixteen interleaved groups, groups added in order), then for every frame the slice's share
// of <frame_sum_k, g> and |frame_sum_k|^2, and the slice's share of |g|^2.  The cosine of the
// anchor rule is assembled from these shares by pick_anchor().
// STRIPS: a frame sum is not stored as such but as `strips` partial sums (one per 32-token strip, as
// the window search writes them: fs[k][strip][C]); they are added in ascending strip order (fp32)
// as they are loaded.  UN: frames in flight per wave.
template <int UN, bool STRIPS>
__device__ __forceinline__ void anchor_partials_body(const float* __restrict__ fs, double* __restrict__ score_part,
                                                     double* __restrict__ clip_part, size_t b, int slice, int fg,
                                                     int F, int C, int S, int FG, int strips, double (*gsh)[256])
{
    // Long clips: FG blocks share a (clip, slice); each forms the clip sum itself (frame sums come
    // from L2) and scores its own run of frames, so that few clips still fill the chip.
    constexpr int NWV = 16;                             // waves per block
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int per = (F + FG - 1) / FG;                  // frames scored by one block
    const int k_lo = fg * per, k_hi = min(F, k_lo + per);
    const size_t fstride = STRIPS ? (size_t)strips * C : (size_t)C;   // floats between consecutive frames
    int c[4];
    bool ok[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        c[e] = slice * 256 + lane * 4 + e;             // four consecutive channels per lane: one 16-byte load
        ok[e] = c[e] < C;
    }
    // this lane's four channels of one frame sum: one 16-byte load when the row allows it
    const bool vec = (C % 4 == 0) && ok[3];
    auto load4 = [&](const float* row, float* out) {
        if constexpr (STRIPS) {                        // (C % 128 == 0 on this path: always 16-byte loads)
            if (!ok[3]) return;                        // the last slice may reach beyond C
            for (int s0 = 0; s0 < strips; s0 += 8) {
                float4 q[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (s0 + u < strips) q[u] = *reinterpret_cast<const float4*>(row + (size_t)(s0 + u) * C + c[0]);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (s0 + u < strips) { out[0] += q[u].x; out[1] += q[u].y; out[2] += q[u].z; out[3] += q[u].w; }
            }
        } else if (vec) {
            const float4 q = *reinterpret_cast<const float4*>(row + c[0]);
            out[0] = q.x; out[1] = q.y; out[2] = q.z; out[3] = q.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (ok[e]) out[e] = row[c[e]];
        }
    };
    // short clips: every wave's frames fit its registers, so the second pass re-uses the first's loads
    const bool resident = F <= NWV * UN && FG == 1;
    float v[UN][4];
    double gp[4] = {0.0, 0.0, 0.0, 0.0};
    for (int k0 = wave; k0 < F; k0 += NWV * UN) {
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int k = k0 + NWV * u;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[u][e] = 0.f;
            if (k < F) load4(fs + (size_t)k * fstride, v[u]);
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
#pragma unroll
            for (int e = 0; e < 4; ++e) gp[e] += (double)v[u][e];
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) gsh[wave][lane * 4 + e] = gp[e];
    __syncthreads();
    double g[4], vv = 0.0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int q = lane * 4 + e;
        double t = gsh[0][q];
#pragma unroll
        for (int w = 1; w < NWV; ++w) t += gsh[w][q];
        g[e] = t;
        vv += t * t;
    }
    vv = wave_sum(vv);
    if (threadIdx.x == 0 && fg == 0) clip_part[b * S + slice] = vv;
    for (int k0 = k_lo + wave; k0 < k_hi; k0 += NWV * UN) {
        if (!resident) {
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int k = k0 + NWV * u;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[u][e] = 0.f;
                if (k < k_hi) load4(fs + (size_t)k * fstride, v[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int k = k0 + NWV * u;
            double uv = 0.0, uu = 0.0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const double x = (double)v[u][e];
                uv += x * g[e];
                uu += x * x;
            }
            uv = wave_sum(uv);
            uu = wave_sum(uu);
            if (lane == 0 && k < k_hi) {
                double* o = score_part + ((b * S + slice) * (size_t)F + k) * 2;
                o[0] = uv;
                o[1] = uu;
            }
        }
    }
}

// MIXED: clips with a trusted anchor guess (spec[b][1]) have their frame sums as strip sums
// (strip_sum [B,F,strips,C]), the other clips in frame_sum [B,F,C]; otherwise every clip in frame_sum.
template <bool MIXED>
__global__ __launch_bounds__(1024) void k_anchor_partials(const float* __restrict__ frame_sum,
                                                         double* __restrict__ score_part,
                                                         double* __restrict__ clip_part, int F, int C, int S,
                                                         int FG, int strips, const float* __restrict__ strip_sum,
                                                         const int32_t* __restrict__ spec)
{
    const int fg = blockIdx.x % FG;
    const int slice = (blockIdx.x / FG) % S;
    const size_t b = blockIdx.x / FG / S;
    __shared__ double gsh[16][256];
    if (MIXED && spec[4 * b + 1] != 0)                   // block-uniform
        anchor_partials_body<2, true>(strip_sum + b * (size_t)F * strips * C, score_part, clip_part, b, slice, fg, F,
                                      C, S, FG, strips, gsh);
    else
        anchor_partials_body<8, false>(frame_sum + b * (size_t)F * C, score_part, clip_part, b, slice, fg, F, C, S, FG,
                                       1, gsh);
}

// Strip sums -> frame sums for the clips with a trusted anchor guess (grids with many strips per
// frame: a plain streaming reduction ahead of k_anchor_partials<false> keeps the chip full, where the
// fused form has too few blocks).  Block (frame, 1024-channel slab): thread t adds its four channels
// over the strips in ascending order, eight loads in flight.
__global__ __launch_bounds__(256) void k_reduce_strips(const float* __restrict__ strip_sum,
                                                       float* __restrict__ frame_sum,
                                                       const int32_t* __restrict__ spec, int F, int C, int strips)
{
    const size_t frame = blockIdx.x;
    if (!spec[4 * (frame / F) + 1]) return;             // this clip's frame sums come from k_frame_sums
    const int c = (blockIdx.y * 256 + threadIdx.x) * 4;
    if (c >= C) return;
    const float* row = strip_sum + frame * (size_t)strips * C + c;
    float4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < strips; s0 += 8) {
        float4 q[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (s0 + u < strips) q[u] = *reinterpret_cast<const float4*>(row + (size_t)(s0 + u) * C);
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (s0 + u < strips) { acc.x += q[u].x; acc.y += q[u].y; acc.z += q[u].z; acc.w += q[u].w; }
    }
    *reinterpret_cast<float4*>(frame_sum + frame * (size_t)C + c) = acc;
}

// Anchor guess, step 1 (bf16 rows): sums over the tokens of a frame of the kGuessChannels guess
// channels only (kGuessSegments runs of 128 bytes per token row).  Block (frame, part) covers tokens
// part*per .. (part+1)*per - 1: thread t reads 16-byte piece t%32 of the guess channels of its tokens
// t/32, t/32 + 8, ...; the eight token groups are added through LDS in order.  The parts of a frame
// are added by guess_pick_block.
__global__ __launch_bounds__(256) void k_guess_sums(const uint16_t* __restrict__ x, float* __restrict__ guess_sum,
                                                    int N, int C, int parts)
{
    static_assert(kGuessSegChannels == 64 && kGuessSegments * 8 == 32, "32 sixteen-byte pieces per token");
    const size_t frame = blockIdx.x / parts;
    const int part = blockIdx.x % parts;
    const int per = (N + parts - 1) / parts;
    const int n_lo = part * per, n_hi = min(N, n_lo + per);
    const int ts = threadIdx.x >> 5, q = threadIdx.x & 31;
    const int ch = guess_segment_start(C, q >> 3) + (q & 7) * 8;
    const uint16_t* base = x + frame * (size_t)N * C + ch;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (int i0 = n_lo + ts; i0 < n_hi; i0 += 64) {
        RowVec<bf16_t, 8> r[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + 8 * u;
            if (i < n_hi) r[u].template load<true>(reinterpret_cast<const bf16_t*>(base + (size_t)i * C));
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (i0 + 8 * u < n_hi) {
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] += r[u].v[e];
            }
        }
    }
    __shared__ float part_s[8][kGuessChannels];
#pragma unroll
    for (int e = 0; e < 8; ++e) part_s[ts][q * 8 + e] = acc[e];
    __syncthreads();
    float t = part_s[0][threadIdx.x];
#pragma unroll
    for (int w = 1; w < 8; ++w) t += part_s[w][threadIdx.x];
    guess_sum[(size_t)blockIdx.x * kGuessChannels + threadIdx.x] = t;
}

// Anchor guess, step 2: the anchor rule evaluated on the guess channels alone (fp64 from the fp32
// sums of step 1), by all NWV waves of a block together (every thread must call it; it synchronises
// the block).  The guess is trusted when its score beats the runner-up's by at least kGuessMinGap and
// no score is NaN; the search then runs against it before the exact rule has been evaluated, and the
// exact rule (from sums the search produces on the side) confirms it or triggers a second search.
// Returns the guessed frame (lowest k on ties) and whether it is trusted, to every thread.
constexpr double kGuessMinGap = 0.1;
template <int NWV>
__device__ __forceinline__ void guess_pick_block(const float* __restrict__ guess_sum, int b, int F, int parts,
                                                 int& guess, bool& trusted)
{
    constexpr int UN = 8;                               // frames in flight per wave
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t fstride = (size_t)parts * kGuessChannels;
    const float* gs = guess_sum + (size_t)b * F * fstride + lane * 4;
    // this lane's four guess channels of frame k: its parts added in order
    auto load4 = [&](int k) {
        float4 v = *reinterpret_cast<const float4*>(gs + (size_t)k * fstride);
        for (int pp = 1; pp < parts; ++pp) {
            const float4 q = *reinterpret_cast<const float4*>(gs + (size_t)k * fstride + (size_t)pp * kGuessChannels);
            v.x += q.x; v.y += q.y; v.z += q.z; v.w += q.w;
        }
        return v;
    };
    __shared__ double gsh[NWV][kGuessChannels];
    __shared__ double s_best[NWV], s_second[NWV];
    __shared__ int s_arg[NWV], s_nan[NWV];
    __shared__ int s_out[2];
    // clips of up to NWV*UN frames: every wave's frames stay in its registers for the second pass
    const bool resident = F <= NWV * UN;
    float4 v[UN];
    double gp[4] = {0.0, 0.0, 0.0, 0.0};
    for (int k0 = wave; k0 < F; k0 += NWV * UN) {
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int k = k0 + NWV * u;
            v[u] = float4{0.f, 0.f, 0.f, 0.f};
            if (k < F) v[u] = load4(k);
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            gp[0] += (double)v[u].x; gp[1] += (double)v[u].y; gp[2] += (double)v[u].z; gp[3] += (double)v[u].w;
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) gsh[wave][lane * 4 + e] = gp[e];
    __syncthreads();
    double g[4], vv = 0.0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        double t = gsh[0][lane * 4 + e];
#pragma unroll
        for (int w = 1; w < NWV; ++w) t += gsh[w][lane * 4 + e];
        g[e] = t;
        vv += t * t;
    }
    vv = wave_sum(vv);
    double best = -1.0e300, second = -1.0e300;          // wave-uniform running top two of this wave's frames
    int arg = 0x7fffffff, nan = 0;
    for (int k0 = wave; k0 < F; k0 += NWV * UN) {       // ascending k per wave: strict > keeps the lowest on ties
        if (!resident) {
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int k = k0 + NWV * u;
                v[u] = float4{0.f, 0.f, 0.f, 0.f};
                if (k < F) v[u] = load4(k);
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int k = k0 + NWV * u;
            const double xv[4] = {(double)v[u].x, (double)v[u].y, (double)v[u].z, (double)v[u].w};
            double uv = 0.0, uu = 0.0;
#pragma unroll
            for (int e = 0; e < 4; ++e) { uv += xv[e] * g[e]; uu += xv[e] * xv[e]; }
            uv = wave_sum(uv);
            uu = wave_sum(uu);
            const double den = sqrt(uu) * sqrt(vv);
            const double score = den > 0.0 ? uv / den : 0.0;
            if (k < F) {                                // wave-uniform
                if (!(score == score)) nan = 1;
                if (score > best) { second = best; best = score; arg = k; }
                else if (score > second) second = score;
            }
        }
    }
    if (lane == 0) { s_best[wave] = best; s_second[wave] = second; s_arg[wave] = arg; s_nan[wave] = nan; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double bb = -1.0e300, sec = -1.0e300;
        int aa = 0x7fffffff, nn = 0;
        for (int w = 0; w < NWV; ++w) {
            nn |= s_nan[w];
            if (s_best[w] > bb || (s_best[w] == bb && s_arg[w] < aa)) {
                sec = fmax(sec, bb);
                bb = s_best[w];
                aa = s_arg[w];
            } else {
                sec = fmax(sec, s_best[w]);
            }
            sec = fmax(sec, s_second[w]);
        }
        s_out[0] = aa == 0x7fffffff ? 0 : aa;
        s_out[1] = (!nn && aa != 0x7fffffff && (F == 1 || bb - sec >= kGuessMinGap)) ? 1 : 0;
    }
    __syncthreads();
    guess = s_out[0];
    trusted = s_out[1] != 0;
}

// Arg max over k of cos(frame_sum_k, clip_sum), assembled in fp64 from the per-slice shares
// (slices added in order); 0 when a norm is 0.  Computed by one wave, every lane gets the result;
// lowest k on ties; frame 0 if every score is NaN.
__device__ __forceinline__ int pick_anchor(const double* __restrict__ score_part,
                                           const double* __restrict__ clip_part, int b, int F, int S, int lane)
{
    double vv = 0.0;
#pragma unroll 8
    for (int s = 0; s < S; ++s) vv += clip_part[(size_t)b * S + s];
    double best = -1.0e300;
    int arg = 0x7fffffff;
    for (int k = lane; k < F; k += 64) {                // ascending k per lane: strict > keeps the lowest
        double uv = 0.0, uu = 0.0;
#pragma unroll 8
        for (int s = 0; s < S; ++s) {
            const double2 o = *reinterpret_cast<const double2*>(score_part + (((size_t)b * S + s) * F + k) * 2);
            uv += o.x;
            uu += o.y;
        }
        const double den = sqrt(uu) * sqrt(vv);
        const double score = den > 0.0 ? uv / den : 0.0;
        if (score > best) { best = score; arg = k; }
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        const double ob = __shfl_xor(best, m, 64);
        const int oa = __shfl_xor(arg, m, 64);
        if (ob > best || (ob == best && oa < arg)) { best = ob; arg = oa; }
    }
    return arg == 0x7fffffff ? 0 : arg;
}

// Batch-tied anchor (tied-batch mode): the frame whose anchor score, averaged over the B clips
// (fp64), is largest; lowest k on ties.  A fixed frame is simply broadcast.  One workgroup of 16
// waves: wave w adds the scores of clips w, w+16, ... (ascending) for 64 frames at a time, wave 0
// adds the 16 partial sums in wave order and keeps the running arg max; the shared index is
// written to every entry of anchor_index.
__global__ __launch_bounds__(1024) void k_tied_anchor(const double* __restrict__ score_part,
                                                      const double* __restrict__ clip_part,
                                                      int32_t* __restrict__ anchor_index, int B, int F, int S,
                                                      int fixed_anchor)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __shared__ double part[16][64];
    __shared__ int s_arg;
    int arg = fixed_anchor;
    if (fixed_anchor < 0) {
        double best = -1.0e300;
        arg = 0x7fffffff;
        for (int k0 = 0; k0 < F; k0 += 64) {
            const int k = k0 + lane;
            double acc = 0.0;
            for (int b = wave; b < B && k < F; b += 16) {
                double vv = 0.0, uv = 0.0, uu = 0.0;
#pragma unroll 8
                for (int s = 0; s < S; ++s) {
                    vv += clip_part[(size_t)b * S + s];
                    const double2 o = *reinterpret_cast<const double2*>(score_part + (((size_t)b * S + s) * F + k) * 2);
                    uv += o.x;
                    uu += o.y;
                }
                const double den = sqrt(uu) * sqrt(vv);
                acc += den > 0.0 ? uv / den : 0.0;
            }
            part[wave][lane] = acc;
            __syncthreads();
            if (wave == 0 && k < F) {
                double sum = part[0][lane];
#pragma unroll
                for (int w = 1; w < 16; ++w) sum += part[w][lane];
                const double score = sum / (double)B;
                if (score > best) { best = score; arg = k; }   // ascending k per lane: strict > keeps the lowest
            }
            __syncthreads();
        }
        if (wave == 0) {
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) {
                const double ob = __shfl_xor(best, m, 64);
                const int oa = __shfl_xor(arg, m, 64);
                if (ob > best || (ob == best && oa < arg)) { best = ob; arg = oa; }
            }
            if (arg == 0x7fffffff) arg = 0;
            if (lane == 0) s_arg = arg;
        }
        __syncthreads();
        arg = s_arg;
    }
    for (int b = threadIdx.x; b < B; b += 1024) anchor_index[b] = arg;
}

// Picks the anchor of clip b (arg max of frame_score, lowest k on ties, or the fixed frame),
// publishes it, and writes 1/||x_{a,j}|| for the anchor tokens.  One wave per anchor token.
template <typename T, int V>
__global__ __launch_bounds__(256) void k_anchor_norms(const T* __restrict__ x, const T* __restrict__ ext_anchor,
                                                      const double* __restrict__ score_part,
                                                      const double* __restrict__ clip_part,
                                                      int32_t* __restrict__ anchor_index,
                                                      float* __restrict__ anchor_inv,
                                                      int F, int N, int C, int S, int fixed_anchor, int groups)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = blockIdx.x / groups;
    const int j = (blockIdx.x % groups) * 4 + wave;
    // the anchor is a frame of x (fixed, picked here, or already chosen: kAnchorGiven), or frame b
    // of ext_anchor (published as -1)
    const int a = ext_anchor ? -1
                : fixed_anchor >= 0 ? fixed_anchor
                : fixed_anchor == kAnchorGiven ? anchor_index[b]
                                               : pick_anchor(score_part, clip_part, b, F, S, lane);
    if (fixed_anchor != kAnchorGiven && blockIdx.x % groups == 0 && threadIdx.x == 0) anchor_index[b] = a;
    if (j >= N) return;
    const T* row = (ext_anchor ? ext_anchor + (size_t)b * N * C : x + ((size_t)b * F + a) * N * C) + (size_t)j * C;
    float ss = 0.f;
    for (int c = lane * V; c < C; c += 64 * V) {
        RowVec<T, V> r;
        r.load(row + c);
#pragma unroll
        for (int e = 0; e < V; ++e) ss = fmaf(r.v[e], r.v[e], ss);
    }
    ss = wave_sum(ss);
    if (lane == 0) anchor_inv[(size_t)b * N + j] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
}

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// Matrix-core path.  One workgroup (8 waves) per anchor tile of 16 tokens: picks the anchor,
// writes the anchor-frame rows of the per-token outputs (never fused, all keep bits set), reads
// the tile once with coalesced loads (lane l: chunk l%4 of token l/4), accumulates squared
// norms, permutes every 16x64-byte block into MFMA operand order (lane = token + 16*chunk) and
// stores it as one contiguous KiB: anchor_frag[b][tile][K-step][lane][8 bf16].
// PAD: the grid is Wg <= 16*CT tokens wide; a tile is 16 columns of one grid row, columns at and
// beyond Wg are padding (zero fragments, inverse norm 0), and tiles are numbered row * CT + column
// tile.  Without PAD a tile is 16 consecutive flat tokens (the same thing when Wg == 16*CT).
template <bool PAD>
__global__ __launch_bounds__(512) void k_anchor_prepare(const uint16_t* __restrict__ x,
                                                        const uint16_t* __restrict__ ext_anchor,
                                                        const double* __restrict__ score_part,
                                                        const double* __restrict__ clip_part,
                                                        int32_t* __restrict__ anchor_index,
                                                        float* __restrict__ anchor_inv,
                                                        uint16_t* __restrict__ anchor_frag,
                                                        int32_t* __restrict__ fuse_map, float* __restrict__ best_sim,
                                                        int32_t* __restrict__ best_idx, uint16_t* __restrict__ keep16,
                                                        int F, int N, int C, int S, int fixed_anchor, int tiles,
                                                        int Wg, int CT, int32_t* __restrict__ spec, int spec_mode,
                                                        const float* __restrict__ guess_sum, int guess_parts)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = blockIdx.x / tiles, tile = blockIdx.x % tiles;
    // the anchor is a frame of x (fixed, picked here, or already chosen: kAnchorGiven), or frame b
    // of ext_anchor (published as -1)
    int a;
    if (spec_mode == 0) {
        a = ext_anchor ? -1
          : fixed_anchor >= 0 ? fixed_anchor
          : fixed_anchor == kAnchorGiven ? anchor_index[b]
                                         : pick_anchor(score_part, clip_part, b, F, S, lane);
    } else if (spec_mode == 1) {
        // speculative pass: the guess (anchor rule on a few channels), evaluated by every block of the
        // clip for itself.  A trusted guess stands in for the anchor until the search has produced exact
        // frame sums; a clip without one is only summed by the coming search, so nothing is prepared.
        bool trusted;
        guess_pick_block<8>(guess_sum, b, F, guess_parts, a, trusted);
        if (tile == 0 && threadIdx.x == 0) {
            spec[4 * b + 0] = a;
            spec[4 * b + 1] = trusted ? 1 : 0;
            spec[4 * b + 2] = 0;
            spec[4 * b + 3] = 0;
        }
        if (!trusted) return;
    } else {
        // after the search: the exact rule.  A trusted guess it confirms: nothing to do.  Otherwise
        // publish the exact anchor, mark the clip for the second search and prepare its anchor.
        a = pick_anchor(score_part, clip_part, b, F, S, lane);
        const bool redo = !spec[4 * b + 1] || a != spec[4 * b];
        if (tile == 0 && threadIdx.x == 0) spec[4 * b + 2] = redo ? 1 : 0;
        if (!redo) return;
    }
    if (fixed_anchor != kAnchorGiven && tile == 0 && threadIdx.x == 0) anchor_index[b] = a;
    // flat index of the tile's first token, and how many of its 16 columns exist
    const int first = PAD ? (tile / CT) * Wg + 16 * (tile % CT) : 16 * tile;
    const int ncol = PAD ? min(16, Wg - 16 * (tile % CT)) : 16;
    if (a >= 0 && fuse_map && (int)threadIdx.x < ncol) {     // anchor tokens are always retained
        const size_t o = ((size_t)b * F + a) * N + first + threadIdx.x;
        fuse_map[o] = -1;
        if (best_sim) best_sim[o] = 1.0f;
        if (best_idx) best_idx[o] = first + (int)threadIdx.x;
        if (!PAD && threadIdx.x == 0) keep16[o / 16] = 0xffffu;
    }
    const int KS = C / 32;
    const uint16_t* frame = ext_anchor ? ext_anchor + (size_t)b * N * C : x + ((size_t)b * F + a) * N * C;
    const bool real = (lane >> 2) < ncol;                    // this lane's token exists (padding reads the tile's first)
    const uint16_t* src = frame + (size_t)(first + (real ? lane >> 2 : 0)) * C + (lane & 3) * 8;
    uint16_t* dst = anchor_frag + ((size_t)b * tiles + tile) * (size_t)KS * 512 + lane * 8;
    const int bperm = (4 * (lane & 15) + (lane >> 4)) * 4;
    float nn = 0.f;
    constexpr int UN = 8;                                   // K-steps in flight per wave
    for (int k0 = wave; k0 < KS; k0 += 8 * UN) {
        uint4 v[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int ks = k0 + 8 * u;
            if (ks < KS) {
                v[u] = *reinterpret_cast<const uint4*>(src + (size_t)ks * 32);
                if (PAD && !real) v[u] = uint4{0u, 0u, 0u, 0u};
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int ks = k0 + 8 * u;
            if (ks < KS) {
                uint32_t r[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bf16x2 p = __builtin_bit_cast(bf16x2, r[e]);
                    nn = __builtin_amdgcn_fdot2_f32_bf16(p, p, nn, false);
                    r[e] = (uint32_t)__builtin_amdgcn_ds_bpermute(bperm, (int)r[e]);
                }
                *reinterpret_cast<uint4*>(dst + (size_t)ks * 512) = uint4{r[0], r[1], r[2], r[3]};
            }
        }
    }
    nn += __shfl_xor(nn, 1, 64);
    nn += __shfl_xor(nn, 2, 64);
    __shared__ float part[8][16];
    if ((lane & 3) == 0) part[wave][lane >> 2] = nn;
    __syncthreads();
    if (threadIdx.x < 16) {
        float ss = part[0][threadIdx.x];
#pragma unroll
        for (int w = 1; w < 8; ++w) ss += part[w][threadIdx.x];
        anchor_inv[((size_t)b * tiles + tile) * 16 + threadIdx.x] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
    }
}

// The three bf16 pieces of two fp32 values, each pair packed into one 32-bit word: hi = bf16(v),
// mid = bf16(v - hi), lo = bf16(v - hi - mid), round to nearest even.  Both subtractions are exact in
// fp32, so hi + mid + lo carries 24 significant bits of v.
typedef __attribute__((ext_vector_type(2))) float f32x2;
__device__ __forceinline__ void split_bf16x3(float a, float b, uint32_t& hi, uint32_t& mid, uint32_t& lo)
{
    hi = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
    const float ra = a - __builtin_bit_cast(float, hi << 16), rb = b - __builtin_bit_cast(float, hi & 0xffff0000u);
    mid = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{ra, rb}, bf16x2));
    const float sa = ra - __builtin_bit_cast(float, mid << 16), sb = rb - __builtin_bit_cast(float, mid & 0xffff0000u);
    lo = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{sa, sb}, bf16x2));
}

// Matrix-core path for fp32 tokens.  As k_anchor_prepare, but the anchor frame is stored as three
// bf16 planes (hi, mid, lo pieces of every value) per tile and K-step of 32 channels:
// anchor_frag[b][tile][K-step][plane][lane][8 bf16], 3 KiB per tile and K-step.  Inside a K-step the
// operand lane (token n, group g) holds channels 4g..4g+3 and 16+4g..16+4g+3: the order in which two
// coalesced 16-byte loads per lane (lane l: token l/4, floats 4(l%4).. of each 64-byte half) arrive
// after one lane permutation.  The search splits and orders its source fragments the same way.
template <bool PAD>
__global__ __launch_bounds__(512) void k_anchor_prepare_f32(const float* __restrict__ x,
                                                            const float* __restrict__ ext_anchor,
                                                            const double* __restrict__ score_part,
                                                            const double* __restrict__ clip_part,
                                                            int32_t* __restrict__ anchor_index,
                                                            float* __restrict__ anchor_inv,
                                                            uint16_t* __restrict__ anchor_frag,
                                                            int32_t* __restrict__ fuse_map,
                                                            float* __restrict__ best_sim,
                                                            int32_t* __restrict__ best_idx,
                                                            uint16_t* __restrict__ keep16, int F, int N, int C, int S,
                                                            int fixed_anchor, int tiles, int Wg, int CT)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = blockIdx.x / tiles, tile = blockIdx.x % tiles;
    const int a = ext_anchor ? -1
                : fixed_anchor >= 0 ? fixed_anchor
                : fixed_anchor == kAnchorGiven ? anchor_index[b]
                                               : pick_anchor(score_part, clip_part, b, F, S, lane);
    if (fixed_anchor != kAnchorGiven && tile == 0 && threadIdx.x == 0) anchor_index[b] = a;
    const int first = PAD ? (tile / CT) * Wg + 16 * (tile % CT) : 16 * tile;
    const int ncol = PAD ? min(16, Wg - 16 * (tile % CT)) : 16;
    if (a >= 0 && fuse_map && (int)threadIdx.x < ncol) {     // anchor tokens are always retained
        const size_t o = ((size_t)b * F + a) * N + first + threadIdx.x;
        fuse_map[o] = -1;
        if (best_sim) best_sim[o] = 1.0f;
        if (best_idx) best_idx[o] = first + (int)threadIdx.x;
        if (!PAD && threadIdx.x == 0) keep16[o / 16] = 0xffffu;
    }
    const int KS = C / 32;
    const float* frame = ext_anchor ? ext_anchor + (size_t)b * N * C : x + ((size_t)b * F + a) * N * C;
    const bool real = (lane >> 2) < ncol;                    // this lane's token exists (padding reads the tile's first)
    const float* src = frame + (size_t)(first + (real ? lane >> 2 : 0)) * C + (lane & 3) * 4;
    uint16_t* dst = anchor_frag + ((size_t)b * tiles + tile) * (size_t)KS * 1536 + lane * 8;
    const int bperm = (4 * (lane & 15) + (lane >> 4)) * 4;
    float nn = 0.f;
    constexpr int UN = 4;                                   // K-steps in flight per wave
    for (int k0 = wave; k0 < KS; k0 += 8 * UN) {
        uint4 v[UN][2];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int ks = k0 + 8 * u;
            if (ks < KS) {
                v[u][0] = *reinterpret_cast<const uint4*>(src + (size_t)ks * 32);
                v[u][1] = *reinterpret_cast<const uint4*>(src + (size_t)ks * 32 + 16);
                if (PAD && !real) v[u][0] = v[u][1] = uint4{0u, 0u, 0u, 0u};
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int ks = k0 + 8 * u;
            if (ks < KS) {
                uint32_t r[8] = {v[u][0].x, v[u][0].y, v[u][0].z, v[u][0].w, v[u][1].x, v[u][1].y, v[u][1].z, v[u][1].w};
                float f[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float t = __builtin_bit_cast(float, r[e]);
                    nn = fmaf(t, t, nn);
                    f[e] = __builtin_bit_cast(float, (uint32_t)__builtin_amdgcn_ds_bpermute(bperm, (int)r[e]));
                }
                uint32_t hi[4], mid[4], lo[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) split_bf16x3(f[2 * e], f[2 * e + 1], hi[e], mid[e], lo[e]);
                uint16_t* o = dst + (size_t)ks * 1536;
                *reinterpret_cast<uint4*>(o) = uint4{hi[0], hi[1], hi[2], hi[3]};
                *reinterpret_cast<uint4*>(o + 512) = uint4{mid[0], mid[1], mid[2], mid[3]};
                *reinterpret_cast<uint4*>(o + 1024) = uint4{lo[0], lo[1], lo[2], lo[3]};
            }
        }
    }
    nn += __shfl_xor(nn, 1, 64);
    nn += __shfl_xor(nn, 2, 64);
    __shared__ float part[8][16];
    if ((lane & 3) == 0) part[wave][lane >> 2] = nn;
    __syncthreads();
    if (threadIdx.x < 16) {
        float ss = part[0][threadIdx.x];
#pragma unroll
        for (int w = 1; w < 8; ++w) ss += part[w][threadIdx.x];
        anchor_inv[((size_t)b * tiles + tile) * 16 + threadIdx.x] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
    }
}

template <typename F>
hipError_t by_layout(const ttf_params& p, F&& f)
{
    // 16-byte vector loads need rows that start 16-byte aligned: C*sizeof(T) % 16 == 0.
    if (p.dtype == TTF_BF16) {
        if (p.C % 8 == 0) return f(bf16_t{}, std::integral_constant<int, 8>{});
        return f(bf16_t{}, std::integral_constant<int, 1>{});
    }
    if (p.C % 4 == 0) return f(float{}, std::integral_constant<int, 4>{});
    return f(float{}, std::integral_constant<int, 1>{});
}

}  // namespace

hipError_t launch_frame_sums(const ttf_params& p, const void* x, const Workspace& w, bool skip_trusted, hipStream_t s)
{
    const int N = p.H * p.W;
    const int32_t* spec = skip_trusted ? w.spec : nullptr;
    return by_layout(p, [&](auto tag, auto vtag) {
        using T = decltype(tag);
        constexpr int V = decltype(vtag)::value;
        if (V > 1 && p.C % (256 * V) == 0 && (size_t)p.B * p.F * (p.C / (256 * V)) >= 512) {
            dim3 slabs((unsigned)(p.B * p.F), (unsigned)(p.C / (256 * V)));
            k_frame_sums_slab<T, V><<<slabs, 256, 0, s>>>(static_cast<const T*>(x), w.frame_sum, N, p.C, p.F, spec);
            return hipGetLastError();
        }
        dim3 grid((unsigned)(p.B * p.F), (unsigned)((p.C + 64 * V - 1) / (64 * V)));
        k_frame_sums<T, V><<<grid, 256, 0, s>>>(static_cast<const T*>(x), w.frame_sum, N, p.C, p.F, spec);
        return hipGetLastError();
    });
}

// mixed: clips with a trusted anchor guess take their frame sums from the strip sums the search wrote
// (w.strip_sum), the others from w.frame_sum; otherwise every clip from w.frame_sum.
hipError_t launch_anchor_scores(const ttf_params& p, const Workspace& w, bool mixed, hipStream_t s)
{
    const int S = (p.C + 255) / 256;
    // runs of at least 32 frames, and no more blocks than fill the chip a few times
    int FG = 1;
    while (FG < 16 && (size_t)S * p.B * FG < 512 && p.F >= 64 * FG) FG *= 2;
    const unsigned grid = (unsigned)((size_t)S * p.B * FG);
    const int strips = (int)spec_strips(p);
    if (mixed && strips > 8) {
        k_reduce_strips<<<dim3((unsigned)(p.B * p.F), (unsigned)((p.C + 1023) / 1024)), 256, 0, s>>>(
            w.strip_sum, w.frame_sum, w.spec, p.F, p.C, strips);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (mixed && strips <= 8)
        k_anchor_partials<true><<<grid, 1024, 0, s>>>(w.frame_sum, w.score_part, w.clip_part, p.F, p.C, S, FG, strips,
                                                      w.strip_sum, w.spec);
    else
        k_anchor_partials<false><<<grid, 1024, 0, s>>>(w.frame_sum, w.score_part, w.clip_part, p.F, p.C, S, FG, 1,
                                                       nullptr, nullptr);
    return hipGetLastError();
}

// Frame sums over the guess channels only (w.guess_sum), from which the anchor is guessed.
hipError_t launch_guess_sums(const ttf_params& p, const void* x, const Workspace& w, hipStream_t s)
{
    const int parts = guess_parts(p);
    k_guess_sums<<<(unsigned)(p.B * p.F * parts), 256, 0, s>>>(static_cast<const uint16_t*>(x), w.guess_sum, p.H * p.W,
                                                               p.C, parts);
    return hipGetLastError();
}

static int fixed_frame(const ttf_params& p)
{
    if (p.anchor_mode != TTF_ANCHOR_FIXED) return -1;
    return p.anchor_index < 0 ? p.anchor_index + p.F : p.anchor_index;
}

hipError_t launch_tied_anchor(const ttf_params& p, const Workspace& w, int32_t* anchor_index, hipStream_t s)
{
    k_tied_anchor<<<1, 1024, 0, s>>>(w.score_part, w.clip_part, anchor_index, p.B, p.F, (p.C + 255) / 256,
                                     fixed_frame(p));
    return hipGetLastError();
}

hipError_t launch_anchor_norms(const ttf_params& p, const void* x, const void* ext_anchor, const Workspace& w,
                               int32_t* anchor_index, bool anchor_given, hipStream_t s)
{
    const int N = p.H * p.W;
    const int groups = (N + 3) / 4;
    const int fixed = anchor_given ? kAnchorGiven : fixed_frame(p);
    return by_layout(p, [&](auto tag, auto vtag) {
        using T = decltype(tag);
        constexpr int V = decltype(vtag)::value;
        k_anchor_norms<T, V><<<(unsigned)(p.B * groups), 256, 0, s>>>(
            static_cast<const T*>(x), static_cast<const T*>(ext_anchor), w.score_part, w.clip_part, anchor_index,
            w.anchor_inv, p.F, N, p.C,
            (p.C + 255) / 256, fixed, groups);
        return hipGetLastError();
    });
}

hipError_t launch_anchor_prepare_mfma(const ttf_params& p, const void* x, const void* ext_anchor, const Workspace& w,
                                      int32_t* anchor_index, int32_t* fuse_map, float* best_sim,
                                      int32_t* best_idx, bool anchor_given, int spec_mode, hipStream_t s)
{
    const int N = p.H * p.W;
    const int fixed = anchor_given ? kAnchorGiven : fixed_frame(p);
    const bool pad = mfma_search_padded(p);
    const int CT = (p.W + 15) / 16;                          // column tiles per grid row
    const int tiles = pad ? p.H * CT : N / 16;
    auto go = [&](auto kernel) {
        kernel<<<(unsigned)(p.B * tiles), 512, 0, s>>>(static_cast<const uint16_t*>(x),
                                                       static_cast<const uint16_t*>(ext_anchor), w.score_part,
                                                       w.clip_part, anchor_index, w.anchor_inv, w.anchor_frag, fuse_map,
                                                       best_sim, best_idx, reinterpret_cast<uint16_t*>(w.keep_bits),
                                                       p.F, N, p.C, (p.C + 255) / 256, fixed, tiles, p.W, CT,
                                                       spec_mode ? w.spec : nullptr, spec_mode, w.guess_sum,
                                                       guess_parts(p));
        return hipGetLastError();
    };
    return pad ? go(k_anchor_prepare<true>) : go(k_anchor_prepare<false>);
}

hipError_t launch_anchor_prepare_mfma_f32(const ttf_params& p, const void* x, const void* ext_anchor,
                                          const Workspace& w, int32_t* anchor_index, int32_t* fuse_map,
                                          float* best_sim, int32_t* best_idx, bool anchor_given, hipStream_t s)
{
    const int N = p.H * p.W;
    const int fixed = anchor_given ? kAnchorGiven : fixed_frame(p);
    const bool pad = !mfma_f32_aligned(p);
    const int CT = (p.W + 15) / 16;                          // column tiles per grid row
    const int tiles = pad ? p.H * CT : N / 16;
    auto go = [&](auto kernel) {
        kernel<<<(unsigned)(p.B * tiles), 512, 0, s>>>(static_cast<const float*>(x), static_cast<const float*>(ext_anchor),
                                                       w.score_part, w.clip_part, anchor_index, w.anchor_inv,
                                                       w.anchor_frag, fuse_map, best_sim, best_idx,
                                                       reinterpret_cast<uint16_t*>(w.keep_bits), p.F, N, p.C,
                                                       (p.C + 255) / 256, fixed, tiles, p.W, CT);
        return hipGetLastError();
    };
    return pad ? go(k_anchor_prepare_f32<true>) : go(k_anchor_prepare_f32<false>);
}

}  // namespace ttf
