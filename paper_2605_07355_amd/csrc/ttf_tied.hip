// Tied-batch matching and gating (Section 3, the B > 1 remark after the s^/dst equations and the
// gating paragraph): the B elements share one candidate cell per source position -- the cell whose
// cosines average highest over the elements -- each element reports its own cosine there, and a
// position is dropped only if all elements exceed the threshold.
//
// The window search has left every element's cosines of the whole window in
// win_sim[b][k][(dy+r)*(2r+1) + (dx+r)][i] (entries of cells outside the grid are never written
// nor read; the position index i is innermost so that a wave's reads are contiguous).  One
// workgroup of four waves owns one 64-position keep word of the shared mask and one lane of each
// wave owns position (k,i).  Wave w takes the window cells w, w+4, ... in row-major order --
// ascending anchor index, each in-grid cell once, which is the paper's duplicate masking --
// averages the B cosines of each (summed in ascending b) and keeps its first maximum; the four
// candidates are merged through LDS, the lower cell winning ties, so the result is the first
// maximum of the whole window.  Then wave w reads the cosines of elements w, w+4, ... at that
// cell, and the position is fused only if every one of the B exceeds t.
#include "ttf_device.h"
#include "ttf_internal.h"

namespace ttf {
namespace {

constexpr float kNegInf = -__builtin_inff();

__global__ __launch_bounds__(256) void k_tie(const float* __restrict__ win_sim,
                                             const int32_t* __restrict__ anchor_index,
                                             int32_t* __restrict__ fuse_map, float* __restrict__ best_sim,
                                             int32_t* __restrict__ best_idx, float* __restrict__ mean_sim,
                                             uint64_t* __restrict__ keep_bits,
                                             int B, int F, int H, int W, int r, float t, int NW)
{
    __shared__ float cand_mean[4][64];
    __shared__ int cand_slot[4][64];
    __shared__ int all_above[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wd = blockIdx.x;                                // keep word of the shared mask
    const int N = H * W, K1 = 2 * r + 1, K = K1 * K1;
    const int k = wd / NW, word = wd % NW;
    const int i = word * 64 + lane;
    const int a = anchor_index[0];
    const size_t FN = (size_t)F * N;
    const size_t o = (size_t)k * N + i;
    if (k == a) {                                             // anchor tokens are always retained
        if (i < N) {
            if (wave == 0) {
                fuse_map[o] = -1;
                if (best_idx) best_idx[o] = i;
                if (mean_sim) mean_sim[o] = 1.0f;
            }
            if (best_sim)
                for (int b = wave; b < B; b += 4) best_sim[b * FN + o] = 1.0f;
        }
        if (threadIdx.x == 0) keep_bits[wd] = N - word * 64 >= 64 ? ~0ull : (1ull << (N - word * 64)) - 1;
        return;
    }
    const int y = i / W, x = i % W;
    const size_t frame = (size_t)K * N;                       // one (b,k) block of win_sim
    const float* base = win_sim + (size_t)k * frame + i;
    float best = kNegInf;
    int slot_hat = -1;
    for (int slot = wave; slot < K; slot += 4) {
        const int yy = y + slot / K1 - r, xx = x + slot % K1 - r;
        if (i >= N || yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
        const float* cell = base + (size_t)slot * N;
        float sum = 0.f;
        for (int b0 = 0; b0 < B; b0 += 16) {                  // 16 loads in flight, then summed in order
            float v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = b0 + u < B ? cell[(b0 + u) * F * frame] : 0.f;
#pragma unroll
            for (int u = 0; u < 16; ++u)
                if (b0 + u < B) sum += v[u];
        }
        const float m = sum / (float)B;
        if (m > best) { best = m; slot_hat = slot; }          // first maximum of this wave's cells
    }
    cand_mean[wave][lane] = best;
    cand_slot[wave][lane] = slot_hat;
    __syncthreads();
    best = kNegInf;
    slot_hat = -1;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const float m = cand_mean[w][lane];
        const int sl = cand_slot[w][lane];
        if (sl >= 0 && (m > best || (m == best && sl < slot_hat))) { best = m; slot_hat = sl; }
    }
    int above = 1;
    for (int b = wave; b < B; b += 4) {
        const float s = slot_hat >= 0 ? base[(size_t)b * F * frame + (size_t)slot_hat * N] : kNegInf;
        if (best_sim && i < N) best_sim[b * FN + o] = s;
        above &= (s > t) ? 1 : 0;                             // keep = union over the batch of 1[s^ <= t]
    }
    all_above[wave][lane] = above;
    __syncthreads();
    if (wave != 0) return;
    bool keep = false;
    if (i < N) {
        const bool fused = slot_hat >= 0 && (all_above[0][lane] & all_above[1][lane] & all_above[2][lane] & all_above[3][lane]);
        const int arg = slot_hat >= 0 ? (y + slot_hat / K1 - r) * W + x + slot_hat % K1 - r : -1;
        fuse_map[o] = fused ? arg : -1;
        if (best_idx) best_idx[o] = arg;
        if (mean_sim) mean_sim[o] = best;
        keep = !fused;
    }
    const uint64_t bits = __ballot(keep);
    if (lane == 0) keep_bits[wd] = bits;
}

}  // namespace

hipError_t launch_tie(const ttf_params& p, const Workspace& w, const float* win_sim, const int32_t* anchor_index,
                      int32_t* fuse_map, float* best_sim, int32_t* best_idx, float* mean_sim, hipStream_t s)
{
    const int N = p.H * p.W, NW = (N + 63) / 64;
    const int words = p.F * NW;
    k_tie<<<(unsigned)words, 256, 0, s>>>(win_sim, anchor_index, fuse_map, best_sim, best_idx, mean_sim,
                                                      w.keep_bits, p.B, p.F, p.H, p.W, p.r, p.t, NW);
    return hipGetLastError();
}

}  // namespace ttf
