// Window search and gate, general form (any grid, radius, channel count, fp32 or bf16 input):
// Section 3 "Pointwise Matching with Local Window Search" and "Threshold Gating".
//
// For a source token (k,i) at grid cell (y,x) the clamped offsets of Delta_r land exactly on the
// cells [max(0,y-r), min(H-1,y+r)] x [max(0,x-r), min(W-1,x+r)], each counted once after the
// duplicate masking the paper prescribes; walking those cells in ascending flat index and
// keeping the first maximum is the row-major arg max over offsets.  One wavefront handles one
// token at a time: lanes stride over channels, products accumulate in fp32, a butterfly adds the
// lanes.  Candidates are taken in groups of G so the source row is read once per group.  A
// workgroup is 16 wavefronts with TPW tokens each: 4 (one workgroup per 64-token keep word) on
// large inputs, 1 (a quarter word per workgroup, four times the workgroups) on small ones, where
// the serial walk of a wave over its tokens is the whole run time.
#include <type_traits>

#include "ttf_device.h"
#include "ttf_internal.h"

namespace ttf {
namespace {

constexpr int G = 9;                 // candidates per pass over the channels (a 3x3 window in one pass)
constexpr float kNegInf = -__builtin_inff();

// ALL = false: arg max and gate per token.  ALL = true (tied-batch mode): every window similarity
// is written to win_sim[token][(dy+r)*(2r+1) + (dx+r)] instead and nothing else is produced.
template <typename T, int V, bool ALL, int TPW>
__global__ __launch_bounds__(1024) void k_search_generic(
    const T* __restrict__ x, const T* __restrict__ ext_anchor, const int32_t* __restrict__ anchor_index,
    const float* __restrict__ anchor_inv,
    int32_t* __restrict__ fuse_map, float* __restrict__ best_sim, int32_t* __restrict__ best_idx,
    uint64_t* __restrict__ keep_bits, float* __restrict__ win_sim, int F, int H, int W, int C, int r, float t,
    int NW)
{
    const int N = H * W;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int PARTS = 4 / TPW;                    // workgroups per keep word
    const int part = blockIdx.x % PARTS;
    const int word = (blockIdx.x / PARTS) % NW;       // 64-token group inside the frame
    const size_t frame = blockIdx.x / PARTS / NW;     // b*F + k
    const int b = (int)(frame / F), k = (int)(frame % F);
    const int a = anchor_index[b];                    // < 0: the anchor frames are in ext_anchor [B,N,C]
    __shared__ unsigned long long keep_word;
    if (threadIdx.x == 0) keep_word = 0ull;
    __syncthreads();

    const T* anchor = a < 0 ? ext_anchor + (size_t)b * N * C : x + ((size_t)b * F + a) * (size_t)N * C;
    const float* ainv = anchor_inv + (size_t)b * N;

    for (int q = 0; q < TPW; ++q) {
        const int i = word * 64 + part * (16 * TPW) + wave * TPW + q;   // wave-uniform
        if (i >= N) break;
        const size_t o = frame * (size_t)N + i;
        if (k == a) {                                 // anchor tokens are always retained
            if (!ALL && lane == 0) {
                fuse_map[o] = -1;
                if (best_sim) best_sim[o] = 1.0f;
                if (best_idx) best_idx[o] = i;
                atomicOr(&keep_word, 1ull << (i & 63));
            }
            continue;
        }
        const int y = i / W, xx = i % W;
        const int y0 = max(0, y - r), y1 = min(H - 1, y + r);
        const int x0 = max(0, xx - r), x1 = min(W - 1, xx + r);
        const int ww = x1 - x0 + 1;
        const int ncand = (y1 - y0 + 1) * ww;
        const T* src = x + o * (size_t)C;

        float best = kNegInf, src_inv = 0.f;
        int arg = -1;
        for (int c0 = 0; c0 < ncand; c0 += G) {
            int cand[G];
            const T* arow[G];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const int cc = min(c0 + g, ncand - 1);     // pad the last group with its last candidate
                cand[g] = (y0 + cc / ww) * W + x0 + cc % ww;
                arow[g] = anchor + (size_t)cand[g] * C;
            }
            float dot[G], nn = 0.f;
#pragma unroll
            for (int g = 0; g < G; ++g) dot[g] = 0.f;
            for (int c = lane * V; c < C; c += 64 * V) {
                RowVec<T, V> s;
                s.load(src + c);
#pragma unroll
                for (int e = 0; e < V; ++e) nn = fmaf(s.v[e], s.v[e], nn);
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    RowVec<T, V> av;
                    av.load(arow[g] + c);
#pragma unroll
                    for (int e = 0; e < V; ++e) dot[g] = fmaf(s.v[e], av.v[e], dot[g]);
                }
            }
            if (c0 == 0) {
                nn = wave_sum(nn);
                src_inv = nn > 0.f ? 1.0f / sqrtf(nn) : 0.f;
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float d = wave_sum(dot[g]);
                if (c0 + g < ncand) {
                    const float sim = d * src_inv * ainv[cand[g]];
                    if constexpr (ALL) {
                        const int slot = (cand[g] / W - y + r) * (2 * r + 1) + (cand[g] % W - xx + r);
                        if (lane == 0) win_sim[o * (size_t)((2 * r + 1) * (2 * r + 1)) + slot] = sim;
                    } else if (sim > best) {                         // ascending index, strict: first maximum
                        best = sim;
                        arg = cand[g];
                    }
                }
            }
        }
        if (!ALL && lane == 0) {
            const bool fused = best > t;                  // keep = 1[s^ <= t]
            fuse_map[o] = fused ? arg : -1;
            if (best_sim) best_sim[o] = best;
            if (best_idx) best_idx[o] = arg;
            if (!fused) atomicOr(&keep_word, 1ull << (i & 63));
        }
    }
    __syncthreads();
    if (!ALL && threadIdx.x == 0) {
        if constexpr (TPW == 4) {
            keep_bits[frame * (size_t)NW + word] = keep_word;
        } else {                                      // this workgroup's 16 bits of the word
            uint16_t* keep16 = reinterpret_cast<uint16_t*>(keep_bits);
            keep16[(frame * (size_t)NW + word) * 4 + part] = (uint16_t)(keep_word >> (16 * part));
        }
    }
}

}  // namespace

hipError_t launch_window_search_generic(const ttf_params& p, const void* x, const void* ext_anchor, const Workspace& w,
                                        const int32_t* anchor_index, int32_t* fuse_map, float* best_sim,
                                        int32_t* best_idx, float* win_sim, hipStream_t s)
{
    const int N = p.H * p.W, NW = (N + 63) / 64;
    const size_t words = (size_t)p.B * p.F * NW;
    const bool small = words < 2048;                  // fewer than two workgroups per CU at 4 tokens per wave
    const unsigned grid = (unsigned)(small ? 4 * words : words);
    auto go = [&](auto tag, auto vtag) {
        using T = decltype(tag);
        constexpr int V = decltype(vtag)::value;
#define TTF_GEN(ALL, TPW)                                                                                       \
    k_search_generic<T, V, ALL, TPW><<<grid, 1024, 0, s>>>(                                                     \
        static_cast<const T*>(x), static_cast<const T*>(ext_anchor), anchor_index, w.anchor_inv, fuse_map,      \
        best_sim, best_idx, w.keep_bits, win_sim, p.F, p.H, p.W, p.C, p.r, p.t, NW)
        if (win_sim) { if (small) TTF_GEN(true, 1); else TTF_GEN(true, 4); }
        else { if (small) TTF_GEN(false, 1); else TTF_GEN(false, 4); }
#undef TTF_GEN
        return hipGetLastError();
    };
    if (p.dtype == TTF_BF16)
        return p.C % 8 == 0 ? go(bf16_t{}, std::integral_constant<int, 8>{})
                            : go(bf16_t{}, std::integral_constant<int, 1>{});
    return p.C % 4 == 0 ? go(float{}, std::integral_constant<int, 4>{})
                        : go(float{}, std::integral_constant<int, 1>{});
}

}  // namespace ttf
