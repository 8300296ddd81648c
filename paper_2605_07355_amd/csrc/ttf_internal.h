// Internal declarations of the TTF library for gfx950: workspace layout and the launch
// functions behind ttf_compress.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "ttf.h"

namespace ttf {

constexpr int kWave = 64;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// A launch may not have 2^32 threads or more: the most blocks of up to 256 threads.  Kernels that take
// a block per row are launched with at most this many blocks and walk on by the grid size.
constexpr size_t kMaxBlocks256 = (1u << 24) - 1;

// Lets `kernel` use `bytes` of dynamic LDS.  The limit is a property of the function on a device, so it
// is raised once (per function, device and size reached) and not on every launch.
hipError_t allow_dynamic_lds(const void* kernel, size_t bytes);
// fp32 tokens on the matrix cores (ttf_search_mfma_f32.hip): can this problem take them; is its grid one
// whose keep words the search writes itself (exactly 16 or 32 wide, whole 64-token words)
bool mfma_search_f32_supported(const ttf_params& p);
bool mfma_f32_aligned(const ttf_params& p);

// Device scratch carved out of the caller's workspace.  All sections are 256-byte aligned.
struct Workspace {
    float*    frame_sum;     // [B,F,C]  sum over the N tokens of every frame (anchor rule, inner sum)
    double*   score_part;    // [B,S,F,2] per 256-channel slice: <frame sum, clip sum> and |frame sum|^2
    double*   clip_part;     // [B,S]    per slice: |clip sum|^2          (S = ceil(C/256))
    float*    anchor_inv;    // [B,NP]   1/||x_{a,j}|| of every anchor token (0 for a zero token); NP = token count
                             //          of the grid with rows padded to whole 16-column tiles (N when W % 16 == 0)
    uint16_t* anchor_frag;   // [B,NP/16,C/32,64,8] bf16 anchor frame in MFMA fragment order (matrix-core path)
    uint64_t* keep_bits;     // [B,F,NW] bit i%64 of word i/64 set iff token i is kept (NW=ceil(N/64))
    int32_t*  frame_base;    // [B,F]    output row of the first kept token of every frame
    int32_t*  src_row;       // [B*F*N]  input token (flat over clips and frames) that output row r copies
    // Speculative anchor (single pass over the input, see ttf_api.hip); sized 0 where it cannot apply
    float*    guess_sum;     // [B,F,P,kGuessChannels] frame sums over the guess channels only, in P = guess_parts()
                             // shares (one per run of tokens)
    int32_t*  spec;          // [B,4]    guessed anchor, guess trusted (1/0), second search needed (1/0), unused
    float*    strip_sum;     // [B,F,spec_strips(),C] sum of every 32-cell strip of every frame, written by the search
    size_t    bytes;
};

// Channels the anchor guess looks at: kGuessSegments runs of kGuessSegChannels channels, run j starting
// at channel (2j+1)*C/(2*kGuessSegments) rounded down to a multiple of kGuessSegChannels.
constexpr int kGuessSegments = 4;
constexpr int kGuessSegChannels = 64;
constexpr int kGuessChannels = kGuessSegments * kGuessSegChannels;
__host__ __device__ inline int guess_segment_start(int C, int j)
{
    return (int)(((long long)(2 * j + 1) * C / (2 * kGuessSegments)) / kGuessSegChannels * kGuessSegChannels);
}
// The guess sums of a frame are formed by this many blocks, each over a run of the frame's tokens (more
// blocks for big grids, so that few frames still fill the chip), and added when the guess is picked.
inline int guess_parts(const ttf_params& p)
{
    const long long n = (long long)p.H * p.W;
    return n >= 2048 ? 8 : (n >= 1024 ? 4 : (n >= 256 ? 2 : 1));   // (16x16 grids: 23 -> 16 us with two)
}
// 32-cell strips per frame as the matrix-core search cuts them: aligned grids N/32; padded tile rows: two
// grid rows per strip up to 16 columns, one row per strip up to 32, ceil(column tiles / 2) per row beyond.
inline long long spec_strips(const ttf_params& p)
{
    const bool aligned = (p.W == 16 && p.H % 4 == 0) || (p.W == 32 && p.H % 2 == 0);
    if (aligned) return (long long)p.H * p.W / 32;
    if (p.W <= 16) return (p.H + 1) / 2;
    return (long long)p.H * (((p.W + 15) / 16 + 1) / 2);
}
// Shapes the speculative anchor path exists for: the matrix-core search kernels (bf16, C % 128 == 0) on
// grids whose tokens fill at least 70 % of the padded 32-cell strips (the strip sums are stored per
// padded strip: 12..16, 23..32, 45..64 columns, ...), with at least 1024 channels, so that the guess
// channels are a small part of a row.  The radius is not looked at (the workspace must not depend on it).
inline bool speculation_shape(const ttf_params& p)
{
    if (p.dtype != TTF_BF16 || p.C % 128 != 0 || p.C < 1024 || p.F < 2) return false;
    return 10ll * p.H * p.W >= 7ll * 32 * spec_strips(p);
}

inline Workspace carve(const ttf_params& p, void* base)
{
    const size_t B = p.B, F = p.F, N = (size_t)p.H * p.W, C = p.C, NW = (N + 63) / 64;
    const size_t NP = (size_t)p.H * ((p.W + 15) / 16) * 16;   // grid rows padded to whole 16-column tiles
    size_t off = 0;
    auto take = [&](size_t n) { size_t o = off; off = align_up(off + n, 256); return o; };
    const size_t o_fs = take(B * F * C * sizeof(float));
    const size_t S = (C + 255) / 256;
    const size_t o_sp = take(B * S * F * 2 * sizeof(double));
    const size_t o_cp = take(B * S * sizeof(double));
    const size_t o_ai = take(B * NP * sizeof(float));
    // anchor frame in fragment order: bf16 as is, fp32 as three bf16 planes (where the matrix-core path can run)
    const size_t o_af = take(p.dtype == TTF_BF16 ? B * NP * C * sizeof(uint16_t)
                                                 : (C % 32 == 0 ? 3 * B * NP * C * sizeof(uint16_t) : 0));
    const size_t o_kb = take(B * F * NW * sizeof(uint64_t));
    const size_t o_fb = take(B * F * sizeof(int32_t));
    const size_t o_sr = take(B * F * N * sizeof(int32_t));
    const bool spec = speculation_shape(p);
    const size_t o_gs = take(spec ? B * F * guess_parts(p) * kGuessChannels * sizeof(float) : 0);
    const size_t o_sp2 = take(spec ? B * 4 * sizeof(int32_t) : 0);
    const size_t o_ss = take(spec ? B * F * (size_t)spec_strips(p) * C * sizeof(float) : 0);
    char* c = static_cast<char*>(base);
    Workspace w;
    w.frame_sum   = reinterpret_cast<float*>(c + o_fs);
    w.score_part  = reinterpret_cast<double*>(c + o_sp);
    w.clip_part   = reinterpret_cast<double*>(c + o_cp);
    w.anchor_inv  = reinterpret_cast<float*>(c + o_ai);
    w.anchor_frag = reinterpret_cast<uint16_t*>(c + o_af);
    w.keep_bits   = reinterpret_cast<uint64_t*>(c + o_kb);
    w.frame_base  = reinterpret_cast<int32_t*>(c + o_fb);
    w.src_row     = reinterpret_cast<int32_t*>(c + o_sr);
    w.guess_sum   = reinterpret_cast<float*>(c + o_gs);
    w.spec        = reinterpret_cast<int32_t*>(c + o_sp2);
    w.strip_sum   = reinterpret_cast<float*>(c + o_ss);
    w.bytes = off;
    return w;
}

// Stage launchers.  Each enqueues on `s` and returns the launch status.
// `skip_trusted`: clips with a trusted anchor guess (w.spec) are left out.
hipError_t launch_frame_sums(const ttf_params& p, const void* x, const Workspace& w, bool skip_trusted, hipStream_t s);
// Per-slice shares of the anchor scores from w.frame_sum; `mixed`: from w.strip_sum for the clips with a
// trusted anchor guess.
hipError_t launch_anchor_scores(const ttf_params& p, const Workspace& w, bool mixed, hipStream_t s);
// Frame sums over the guess channels only (w.guess_sum).
hipError_t launch_guess_sums(const ttf_params& p, const void* x, const Workspace& w, hipStream_t s);
// `ext_anchor` (here and below): nullptr when the anchor is a frame of x; otherwise the anchor
// frames [B,N,C] of a segment, in which case anchor_index is written as -1 and every frame of x
// is a source frame.
// `anchor_given`: the anchor of every clip is already in anchor_index (tied-batch mode); it is
// read, not chosen.
hipError_t launch_anchor_norms(const ttf_params& p, const void* x, const void* ext_anchor, const Workspace& w,
                               int32_t* anchor_index, bool anchor_given, hipStream_t s);
// Matrix-core path: anchor choice, inverse norms, the anchor frame re-laid in fragment order, and
// the anchor-frame rows of fuse_map / best_sim / best_idx / keep bits.
// spec_mode 0: the plain rule (fixed, given, or the arg max of the exact scores).  1: speculative pass --
// the anchor is guessed from w.guess_sum; w.spec[b] = {guess, trusted, 0, 0} is written and only clips
// with a trusted guess are prepared.  2: after the speculative search -- the exact rule from the
// scores; clips whose guess it confirms are left alone, the others are marked in w.spec[b][2],
// get the exact anchor published and prepared.
hipError_t launch_anchor_prepare_mfma(const ttf_params& p, const void* x, const void* ext_anchor, const Workspace& w,
                                      int32_t* anchor_index, int32_t* fuse_map, float* best_sim,
                                      int32_t* best_idx, bool anchor_given, int spec_mode, hipStream_t s);
// The same for fp32 tokens: the anchor frame as three bf16 planes per tile and K-step (no speculative modes).
hipError_t launch_anchor_prepare_mfma_f32(const ttf_params& p, const void* x, const void* ext_anchor,
                                          const Workspace& w, int32_t* anchor_index, int32_t* fuse_map,
                                          float* best_sim, int32_t* best_idx, bool anchor_given, hipStream_t s);
bool mfma_search_supported(const ttf_params& p);   // grids exactly 16 or 32 wide with whole keep words
bool mfma_search_padded(const ttf_params& p);      // every other grid (tile rows padded to 16 columns)
hipError_t launch_window_search(const ttf_params& p, const void* x, const void* ext_anchor, const Workspace& w,
                                const int32_t* anchor_index, int32_t* fuse_map, float* best_sim,
                                int32_t* best_idx, float* win_sim, hipStream_t s);
// Keep words rebuilt from the fuse map (for searches whose work units do not line up with keep words).
hipError_t launch_pack_keep(const ttf_params& p, const int32_t* fuse_map, const int32_t* anchor_index,
                            const Workspace& w, hipStream_t s);
hipError_t launch_offsets_scan(const ttf_params& p, const Workspace& w, const int32_t* anchor_index,
                               int32_t* kept_count, int32_t* row_offsets, bool tied, hipStream_t s);
// `total_rows`: device address of the number of output rows (of one clip's share in tied-batch mode),
// as the offsets scan has left it.
hipError_t launch_emit_rows(const ttf_params& p, const void* x, const Workspace& w,
                            const int32_t* total_rows, void* tokens_out, int32_t* pos_ids,
                            int32_t* src_index, int frame_offset, bool tied, hipStream_t s);

// Tied-batch mode.  Workspace behind the common sections: every window similarity of every
// element, and the two row offsets of the shared mask.
struct TiedWorkspace {
    Workspace base;
    float*    win_sim;       // [B,F,(2r+1)^2,N]
    int32_t*  row_offsets;   // [2]
    size_t    bytes;
};
inline TiedWorkspace carve_tied(const ttf_params& p, void* base)
{
    TiedWorkspace t;
    t.base = carve(p, base);
    const size_t K = (size_t)(2 * p.r + 1) * (2 * p.r + 1);
    const size_t o_ws = t.base.bytes;
    const size_t o_ro = align_up(o_ws + (size_t)p.B * p.F * p.H * p.W * K * sizeof(float), 256);
    char* c = static_cast<char*>(base);
    t.win_sim = reinterpret_cast<float*>(c + o_ws);
    t.row_offsets = reinterpret_cast<int32_t*>(c + o_ro);
    t.bytes = o_ro + 256;
    return t;
}
// The shared anchor (batch-mean score, or the fixed frame) written to every entry of anchor_index.
hipError_t launch_tied_anchor(const ttf_params& p, const Workspace& w, int32_t* anchor_index, hipStream_t s);
// Shared offset, per-element s^, united keep mask (keep bits [F,NW] at the start of w.keep_bits).
hipError_t launch_tie(const ttf_params& p, const Workspace& w, const float* win_sim, const int32_t* anchor_index,
                      int32_t* fuse_map, float* best_sim, int32_t* best_idx, float* mean_sim, hipStream_t s);

// Restoration: map from every original token to the compressed row that stands for it, and the
// gather that rebuilds the full layout.
hipError_t launch_restore_map(const ttf_params& p, const int32_t* fuse_map, const int32_t* row_offsets,
                              const int32_t* src_index, int32_t* restore_map, hipStream_t s);
hipError_t launch_restore_rows(const ttf_params& p, const void* tokens, long long rows,
                               const int32_t* restore_map, void* restored, hipStream_t s);
// Adaptive threshold: exact order statistic of the source similarities per clip, and the gate
// redone from stored similarities (fills fuse_map and the keep bits).
// keep_fraction = 1 - requested fused fraction (double); the rank is formed per clip on the device,
// from the clip's own number of source tokens.
hipError_t launch_select_threshold(const ttf_params& p, const float* best_sim, const int32_t* anchor_index,
                                   double keep_fraction, float* thresholds, hipStream_t s);
hipError_t launch_regate(const ttf_params& p, const Workspace& w, const float* best_sim, const int32_t* best_idx,
                         const int32_t* anchor_index, const float* thresholds, int32_t* fuse_map, hipStream_t s);

}  // namespace ttf
