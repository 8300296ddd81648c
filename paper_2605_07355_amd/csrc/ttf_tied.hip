// Tied-batch matching and gating (Section 3: for B > 1 one offset per source position is chosen by
// maximising the mean similarity across the batch elements, every element reads its s^ at that
// offset, and the preserve rule unites the keep masks over the batch).
//
// The window search has left every element's cosines of the whole window in
// win_sim[b][k][i][(dy+r)*(2r+1) + (dx+r)] (entries of cells outside the grid are never written
// nor read).  Here one lane owns one position (k,i): it walks the in-grid cells of the window in
// row-major order -- ascending anchor index, each cell once, which is the paper's duplicate
// masking -- averages the B cosines of each (summed in ascending b), keeps the first maximum,
// reads the B cosines at that cell and fuses the position only if every one of them exceeds t.
#include "ttf_device.h"
#include "ttf_internal.h"

namespace ttf {
namespace {

constexpr float kNegInf = -__builtin_inff();

// One wave per 64-token keep word of the shared mask [F,NW].
__global__ __launch_bounds__(256) void k_tie(const float* __restrict__ win_sim,
                                             const int32_t* __restrict__ anchor_index,
                                             int32_t* __restrict__ fuse_map, float* __restrict__ best_sim,
                                             int32_t* __restrict__ best_idx, float* __restrict__ mean_sim,
                                             uint64_t* __restrict__ keep_bits,
                                             int B, int F, int H, int W, int r, float t, int NW)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wd = blockIdx.x * 4 + wave;                     // keep word of the shared mask
    if (wd >= F * NW) return;
    const int N = H * W, K1 = 2 * r + 1, K = K1 * K1;
    const int k = wd / NW, word = wd % NW;
    const int i = word * 64 + lane;
    const int a = anchor_index[0];
    const size_t FN = (size_t)F * N;
    bool keep = false;
    if (i < N) {
        const size_t o = (size_t)k * N + i;
        if (k == a) {                                         // anchor tokens are always retained
            fuse_map[o] = -1;
            if (best_idx) best_idx[o] = i;
            if (mean_sim) mean_sim[o] = 1.0f;
            if (best_sim)
                for (int b = 0; b < B; ++b) best_sim[b * FN + o] = 1.0f;
            keep = true;
        } else {
            const int y = i / W, x = i % W;
            float best = kNegInf;
            int slot_hat = -1, arg = -1;
            for (int dy = -r; dy <= r; ++dy) {
                const int yy = y + dy;
                if (yy < 0 || yy >= H) continue;
                for (int dx = -r; dx <= r; ++dx) {
                    const int xx = x + dx;
                    if (xx < 0 || xx >= W) continue;
                    const int slot = (dy + r) * K1 + dx + r;
                    float sum = 0.f;
                    for (int b = 0; b < B; ++b) sum += win_sim[(b * FN + o) * K + slot];
                    const float m = sum / (float)B;
                    if (m > best) { best = m; slot_hat = slot; arg = yy * W + xx; }   // first maximum
                }
            }
            bool fused = slot_hat >= 0;
            for (int b = 0; b < B; ++b) {
                const float s = slot_hat >= 0 ? win_sim[(b * FN + o) * K + slot_hat] : kNegInf;
                if (best_sim) best_sim[b * FN + o] = s;
                fused = fused && (s > t);                     // keep = union over the batch of 1[s^ <= t]
            }
            fuse_map[o] = fused ? arg : -1;
            if (best_idx) best_idx[o] = arg;
            if (mean_sim) mean_sim[o] = best;
            keep = !fused;
        }
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
    k_tie<<<(unsigned)((words + 3) / 4), 256, 0, s>>>(win_sim, anchor_index, fuse_map, best_sim, best_idx, mean_sim,
                                                      w.keep_bits, p.B, p.F, p.H, p.W, p.r, p.t, NW);
    return hipGetLastError();
}

}  // namespace ttf
