// C ABI of the TTF library: argument checks, workspace carving, the launch sequence of
// Section 3 (anchor selection -> window search + gate -> offsets -> row emission) and the
// optional per-stage event timing.  Nothing here allocates device memory.
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <atomic>
#include <map>
#include <mutex>
#include <utility>

#include "ttf_internal.h"

namespace ttf {

hipError_t launch_window_search_generic(const ttf_params& p, const void* x, const void* ext_anchor, const Workspace& w,
                                        const int32_t* anchor_index, int32_t* fuse_map, float* best_sim,
                                        int32_t* best_idx, float* win_sim, hipStream_t s);

hipError_t launch_window_search_mfma(const ttf_params& p, const void* x, bool external_anchor, const Workspace& w,
                                     const int32_t* anchor_index, int32_t* fuse_map, float* best_sim,
                                     int32_t* best_idx, float* win_sim, int spec_mode, hipStream_t s);
bool mfma_search_speculative(const ttf_params& p);
hipError_t launch_window_search_mfma_f32(const ttf_params& p, const void* x, bool external_anchor, const Workspace& w,
                                         const int32_t* anchor_index, int32_t* fuse_map, float* best_sim,
                                         int32_t* best_idx, float* win_sim, hipStream_t s);

// bf16 and fp32 tokens with r <= 2 and C % 32 == 0 take the matrix-core kernels (grids exactly 16 or 32
// wide with whole keep words the aligned ones, every other grid the padded-tile ones); larger radii and
// other channel counts take the general wave-per-token kernel.  The environment variable TTF_SEARCH=general, read once per process, forces
// the general kernels (for comparisons).
bool use_mfma_path(const ttf_params& p)
{
    static const bool general = [] {
        const char* force = std::getenv("TTF_SEARCH");
        return force && std::strcmp(force, "general") == 0;
    }();
    return !general && (mfma_search_supported(p) || mfma_search_padded(p) || mfma_search_f32_supported(p));
}

// Anchor preparation of the matrix-core path for the element type at hand (fp32: three bf16 planes).
hipError_t launch_anchor_prepare_any(const ttf_params& p, const void* x, const void* ext_anchor, const Workspace& w,
                                     int32_t* anchor_index, int32_t* fuse_map, float* best_sim, int32_t* best_idx,
                                     bool anchor_given, int spec_mode, hipStream_t s)
{
    if (p.dtype == TTF_F32)
        return launch_anchor_prepare_mfma_f32(p, x, ext_anchor, w, anchor_index, fuse_map, best_sim, best_idx,
                                              anchor_given, s);
    return launch_anchor_prepare_mfma(p, x, ext_anchor, w, anchor_index, fuse_map, best_sim, best_idx, anchor_given,
                                      spec_mode, s);
}

hipError_t launch_window_search(const ttf_params& p, const void* x, const void* ext_anchor, const Workspace& w,
                                const int32_t* anchor_index, int32_t* fuse_map, float* best_sim,
                                int32_t* best_idx, float* win_sim, hipStream_t s)
{
    if (use_mfma_path(p)) {
        if (p.dtype == TTF_F32)
            return launch_window_search_mfma_f32(p, x, ext_anchor != nullptr, w, anchor_index, fuse_map, best_sim,
                                                 best_idx, win_sim, s);
        return launch_window_search_mfma(p, x, ext_anchor != nullptr, w, anchor_index, fuse_map, best_sim, best_idx,
                                         win_sim, 0, s);
    }
    return launch_window_search_generic(p, x, ext_anchor, w, anchor_index, fuse_map, best_sim, best_idx, win_sim, s);
}

hipError_t allow_dynamic_lds(const void* kernel, size_t bytes)
{
    static std::mutex mutex;
    static std::map<std::pair<const void*, int>, size_t> granted;   // (function, device) -> bytes allowed so far
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mutex);
    size_t& have = granted[{kernel, dev}];
    if (bytes <= have) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) have = bytes;
    return e;
}

namespace {

thread_local int g_last_hip_error = 0;

// Speculative anchor: -1 never, 0 for inputs of at least kSpeculationMinBytes in clips of at most
// kSpeculationMaxFrames frames, 1 whenever the shape allows.  (Long clips: the more frames, the closer the
// best two anchor scores; at 256 frames no guess of the synthetic workloads clears the trust gap, every
// clip falls back to the two-pass kernels and the guess costs 0.05 ms for nothing.)
std::atomic<int> g_speculation{0};
constexpr unsigned long long kSpeculationMinBytes = 256ull << 20;
constexpr int kSpeculationMaxFrames = 128;

// Event sets for stage timing: `slots` sets of TTF_NUM_STAGES+1 events, used round-robin by
// successive profiled calls so that a benchmark can time many calls and read them afterwards.
struct Profile {
    int slots = 0;                 // 0 = profiling off
    int created = 0;               // event sets that exist
    long long calls = 0;           // profiled calls since enabling
    hipEvent_t ev[TTF_PROFILE_MAX_SLOTS][TTF_NUM_STAGES + 1];
};
thread_local Profile g_prof;

ttf_status check_params(const ttf_params* p)
{
    if (!p) return TTF_ERR_INVALID_ARG;
    if (p->B < 1 || p->F < 1 || p->H < 1 || p->W < 1 || p->C < 1) return TTF_ERR_INVALID_ARG;
    const long long tokens = (long long)p->B * p->F * p->H * p->W;
    if ((long long)p->H * p->W >= (1ll << 31) || tokens >= (1ll << 31)) return TTF_ERR_INVALID_ARG;
    if (p->C > (1 << 21)) return TTF_ERR_INVALID_ARG;       // keeps every launch grid inside HIP limits
    // every launch stays below 2^32 threads: the densest grids take a 256-thread block per 16 tokens of a
    // frame rounded up to whole 64-token keep words, or per 4 anchor tokens
    if ((long long)p->B * p->F * (((long long)p->H * p->W + 63) / 64) * 64 >= (1ll << 25)) return TTF_ERR_INVALID_ARG;
    if (p->r < 0) return TTF_ERR_INVALID_ARG;
    if (!std::isfinite(p->t)) return TTF_ERR_INVALID_ARG;
    if (p->anchor_mode != TTF_ANCHOR_AUTO && p->anchor_mode != TTF_ANCHOR_FIXED) return TTF_ERR_INVALID_ARG;
    if (p->anchor_mode == TTF_ANCHOR_FIXED && (p->anchor_index < -p->F || p->anchor_index >= p->F))
        return TTF_ERR_INVALID_ARG;
    if (p->dtype != TTF_BF16 && p->dtype != TTF_F32) return TTF_ERR_UNSUPPORTED;
    return TTF_OK;
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace
}  // namespace ttf

using namespace ttf;

extern "C" {

ttf_status ttf_workspace_size(const ttf_params* params, size_t* bytes)
{
    if (!bytes) return TTF_ERR_INVALID_ARG;
    const ttf_status st = check_params(params);
    if (st != TTF_OK) return st;
    *bytes = carve(*params, nullptr).bytes;
    return TTF_OK;
}

// The launch sequence behind ttf_compress (ext_anchor == nullptr) and ttf_compress_segment.
static ttf_status run_pass(const ttf_params* params, const void* features, const void* ext_anchor,
                           int frame_offset, void* workspace, size_t workspace_bytes, const ttf_outputs* out,
                           void* hip_stream)
{
    const ttf_status st = check_params(params);
    if (st != TTF_OK) return st;
    if (!features || !workspace || !out) return TTF_ERR_INVALID_ARG;
    if (!out->tokens_out || !out->pos_ids || !out->src_index || !out->row_offsets || !out->kept_count ||
        !out->anchor_index || !out->fuse_map)
        return TTF_ERR_INVALID_ARG;
    if (!aligned(features, 16) || !aligned(out->tokens_out, 16) || !aligned(workspace, 256))
        return TTF_ERR_UNSUPPORTED;
    if (ext_anchor && !aligned(ext_anchor, 16)) return TTF_ERR_UNSUPPORTED;

    ttf_params p = *params;
    p.r = p.r > (p.H > p.W ? p.H : p.W) ? (p.H > p.W ? p.H : p.W) : p.r;   // beyond the grid = whole grid
    const Workspace w = carve(p, workspace);
    if (workspace_bytes < w.bytes) return TTF_ERR_WORKSPACE_TOO_SMALL;
    const bool pick = !ext_anchor && p.anchor_mode == TTF_ANCHOR_AUTO;       // the automatic anchor rule runs

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    Profile& prof = g_prof;
    const bool timing = prof.slots > 0;
    hipEvent_t* ev = timing ? prof.ev[prof.calls % prof.slots] : nullptr;
    hipError_t e = hipSuccess;
    int stage = 0;
    auto mark = [&]() {
        if (timing && e == hipSuccess) e = hipEventRecord(ev[stage], s);
        ++stage;
    };
#define TTF_STEP(call)                 \
    do {                               \
        if (e == hipSuccess) e = (call); \
    } while (0)

    // The automatic anchor rule needs the sum of every frame, i.e. a pass over the whole input before
    // the search can start.  Large inputs on the aligned matrix-core path avoid that pass: the rule is
    // first evaluated on a few channels only (4 x 128 bytes of every token row); where that guess wins
    // clearly the search runs against it at once and adds up, on the side, the exact sums of every
    // 32-token strip it reads.  The exact rule is then evaluated from those sums: it confirms the
    // guess (the usual case: nothing else to do) or refutes it, and then the clip's anchor is prepared
    // again and its search repeated.  A clip whose guess is not clear-cut sits out the first search; its
    // frame sums are then formed the two-pass way and it is searched with the refuted clips.  Either way
    // every output is what the exact rule gives.
    const int spec_pref = g_speculation.load(std::memory_order_relaxed);
    const unsigned long long in_bytes = (unsigned long long)p.B * p.F * p.H * p.W * p.C * 2ull;
    const bool spec = pick && use_mfma_path(p) && mfma_search_speculative(p) &&
                      (spec_pref > 0 ||
                       (spec_pref == 0 && in_bytes >= kSpeculationMinBytes && p.F <= kSpeculationMaxFrames));

    mark();                                                    // start of stage 0
    if (spec) TTF_STEP(launch_guess_sums(p, features, w, s));
    else if (pick) TTF_STEP(launch_frame_sums(p, features, w, false, s));
    mark();
    if (pick && !spec) TTF_STEP(launch_anchor_scores(p, w, false, s));
    mark();
    if (use_mfma_path(p))
        TTF_STEP(launch_anchor_prepare_any(p, features, ext_anchor, w, out->anchor_index, out->fuse_map,
                                           out->best_sim, out->best_idx, false, spec ? 1 : 0, s));
    else TTF_STEP(launch_anchor_norms(p, features, ext_anchor, w, out->anchor_index, false, s));
    mark();
    if (spec)
        TTF_STEP(launch_window_search_mfma(p, features, false, w, out->anchor_index, out->fuse_map, out->best_sim,
                                           out->best_idx, nullptr, 1, s));
    else
        TTF_STEP(launch_window_search(p, features, ext_anchor, w, out->anchor_index, out->fuse_map, out->best_sim,
                                      out->best_idx, nullptr, s));
    mark();
    if (spec) {
        TTF_STEP(launch_frame_sums(p, features, w, true, s));     // clips without a trusted guess only
        TTF_STEP(launch_anchor_scores(p, w, true, s));
        TTF_STEP(launch_anchor_prepare_mfma(p, features, nullptr, w, out->anchor_index, out->fuse_map,
                                            out->best_sim, out->best_idx, false, 2, s));
        TTF_STEP(launch_window_search_mfma(p, features, false, w, out->anchor_index, out->fuse_map, out->best_sim,
                                           out->best_idx, nullptr, 2, s));
    }
    mark();
    TTF_STEP(launch_offsets_scan(p, w, out->anchor_index, out->kept_count, out->row_offsets, false, s));
    mark();
    TTF_STEP(launch_emit_rows(p, features, w, out->row_offsets + p.B, out->tokens_out, out->pos_ids,
                              out->src_index, frame_offset, false, s));
    mark();                                                    // end of the last stage
    if (out->host_counts) {
        TTF_STEP(hipMemcpyAsync(out->host_counts, out->kept_count, sizeof(int32_t) * p.B,
                                hipMemcpyDeviceToHost, s));
        TTF_STEP(hipMemcpyAsync(out->host_counts + p.B, out->row_offsets, sizeof(int32_t) * (p.B + 1),
                                hipMemcpyDeviceToHost, s));
    }
#undef TTF_STEP
    if (e != hipSuccess) {
        g_last_hip_error = static_cast<int>(e);
        return TTF_ERR_HIP;
    }
    if (timing) ++prof.calls;
    return TTF_OK;
}

ttf_status ttf_compress(const ttf_params* params, const void* features, void* workspace,
                        size_t workspace_bytes, const ttf_outputs* out, void* hip_stream)
{
    return run_pass(params, features, nullptr, 0, workspace, workspace_bytes, out, hip_stream);
}

// Workspace of ttf_compress_static.  In host code this name is only a handle for the runtime's symbol
// lookup, never a device address: host code uses the pointer hipGetSymbolAddress returns for the
// current device (every GPU holds its own copy of the array at its own address).
static __device__ __align__(256) unsigned char scratch[TTF_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` per device, looked up once
}  // namespace

ttf_status ttf_compress_static(const ttf_params* params, const void* features, const ttf_outputs* out,
                               void* hip_stream)
{
    const ttf_status st = check_params(params);
    if (st != TTF_OK) return st;
    if (!features || !out) return TTF_ERR_INVALID_ARG;
    if (carve(*params, nullptr).bytes > (size_t)TTF_STATIC_WORKSPACE_BYTES) return TTF_ERR_WORKSPACE_TOO_SMALL;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && (dev < 0 || dev >= kMaxDevices)) e = hipErrorInvalidDevice;
    void* ptr = nullptr;
    if (e == hipSuccess) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void* found = nullptr;
            e = hipGetSymbolAddress(&found, HIP_SYMBOL(scratch));
            if (e == hipSuccess && !found) e = hipErrorInvalidSymbol;
            if (e == hipSuccess) g_scratch_ptr[dev] = found;
        }
        ptr = g_scratch_ptr[dev];
    }
    if (e != hipSuccess) {
        g_last_hip_error = static_cast<int>(e);
        return TTF_ERR_HIP;
    }
    return run_pass(params, features, nullptr, 0, ptr, (size_t)TTF_STATIC_WORKSPACE_BYTES, out, hip_stream);
}

ttf_status ttf_compress_segment(const ttf_params* params, const void* features, const void* anchor_frame,
                                int32_t frame_offset, void* workspace, size_t workspace_bytes,
                                const ttf_outputs* out, void* hip_stream)
{
    if (!anchor_frame) return TTF_ERR_INVALID_ARG;
    if (params && (long long)frame_offset + params->F > 0x7fffffffll) return TTF_ERR_INVALID_ARG;
    return run_pass(params, features, anchor_frame, frame_offset, workspace, workspace_bytes, out, hip_stream);
}

// Largest radius of the tied-batch mode: its workspace keeps all (2r+1)^2 similarities per token.
static constexpr int kTiedMaxRadius = 3;

ttf_status ttf_tied_workspace_size(const ttf_params* params, size_t* bytes)
{
    if (!bytes) return TTF_ERR_INVALID_ARG;
    const ttf_status st = check_params(params);
    if (st != TTF_OK) return st;
    if (params->r > kTiedMaxRadius) return TTF_ERR_UNSUPPORTED;
    *bytes = carve_tied(*params, nullptr).bytes;
    return TTF_OK;
}

ttf_status ttf_compress_tied(const ttf_params* params, const void* features, void* workspace,
                             size_t workspace_bytes, const ttf_tied_outputs* out, void* hip_stream)
{
    const ttf_status st = check_params(params);
    if (st != TTF_OK) return st;
    if (!features || !workspace || !out) return TTF_ERR_INVALID_ARG;
    if (!out->tokens_out || !out->pos_ids || !out->src_index || !out->kept_count || !out->anchor_index ||
        !out->fuse_map)
        return TTF_ERR_INVALID_ARG;
    if (params->r > kTiedMaxRadius) return TTF_ERR_UNSUPPORTED;
    if (!aligned(features, 16) || !aligned(out->tokens_out, 16) || !aligned(workspace, 256))
        return TTF_ERR_UNSUPPORTED;
    const ttf_params& p = *params;
    const TiedWorkspace tw = carve_tied(p, workspace);
    if (workspace_bytes < tw.bytes) return TTF_ERR_WORKSPACE_TOO_SMALL;
    const Workspace& w = tw.base;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipError_t e = hipSuccess;
#define TTF_STEP(call)                 \
    do {                               \
        if (e == hipSuccess) e = (call); \
    } while (0)
    if (p.anchor_mode == TTF_ANCHOR_AUTO) {
        TTF_STEP(launch_frame_sums(p, features, w, false, s));
        TTF_STEP(launch_anchor_scores(p, w, false, s));
    }
    TTF_STEP(launch_tied_anchor(p, w, out->anchor_index, s));
    if (use_mfma_path(p))
        TTF_STEP(launch_anchor_prepare_any(p, features, nullptr, w, out->anchor_index, nullptr, nullptr, nullptr,
                                           true, 0, s));
    else TTF_STEP(launch_anchor_norms(p, features, nullptr, w, out->anchor_index, true, s));
    TTF_STEP(launch_window_search(p, features, nullptr, w, out->anchor_index, nullptr, nullptr, nullptr,
                                  tw.win_sim, s));
    TTF_STEP(launch_tie(p, w, tw.win_sim, out->anchor_index, out->fuse_map, out->best_sim, out->best_idx,
                        out->mean_sim, s));
    TTF_STEP(launch_offsets_scan(p, w, out->anchor_index, out->kept_count, tw.row_offsets, true, s));
    TTF_STEP(launch_emit_rows(p, features, w, tw.row_offsets + 1, out->tokens_out, out->pos_ids, out->src_index, 0,
                              true, s));
    if (out->host_counts)
        TTF_STEP(hipMemcpyAsync(out->host_counts, out->kept_count, sizeof(int32_t), hipMemcpyDeviceToHost, s));
#undef TTF_STEP
    if (e != hipSuccess) {
        g_last_hip_error = static_cast<int>(e);
        return TTF_ERR_HIP;
    }
    return TTF_OK;
}

ttf_status ttf_restore_map(const ttf_params* params, const int32_t* fuse_map, const int32_t* row_offsets,
                           const int32_t* src_index, int32_t* restore_map, void* hip_stream)
{
    const ttf_status st = check_params(params);
    if (st != TTF_OK) return st;
    if (!fuse_map || !row_offsets || !src_index || !restore_map) return TTF_ERR_INVALID_ARG;
    const hipError_t e = launch_restore_map(*params, fuse_map, row_offsets, src_index, restore_map,
                                            static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) {
        g_last_hip_error = static_cast<int>(e);
        return TTF_ERR_HIP;
    }
    return TTF_OK;
}

ttf_status ttf_restore(const ttf_params* params, const void* tokens, int64_t rows,
                       const int32_t* restore_map, void* restored, void* hip_stream)
{
    const ttf_status st = check_params(params);
    if (st != TTF_OK) return st;
    if (!tokens || !restore_map || !restored || rows < 0) return TTF_ERR_INVALID_ARG;
    if (!aligned(tokens, 16) || !aligned(restored, 16)) return TTF_ERR_UNSUPPORTED;
    const hipError_t e = launch_restore_rows(*params, tokens, rows, restore_map, restored,
                                             static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) {
        g_last_hip_error = static_cast<int>(e);
        return TTF_ERR_HIP;
    }
    return TTF_OK;
}

ttf_status ttf_decode_alignment(int64_t l_prime, int64_t text_tokens, int64_t step,
                                int64_t* l_pre, int64_t* position, int64_t* mask_length)
{
    if (l_prime < 0 || text_tokens < 0 || step < 0) return TTF_ERR_INVALID_ARG;
    const int64_t pre = l_prime + text_tokens;
    if (l_pre) *l_pre = pre;
    if (position) *position = pre + step;
    if (mask_length) *mask_length = pre + step + 1;
    return TTF_OK;
}

ttf_status ttf_select_threshold(const ttf_params* params, const float* best_sim,
                                const int32_t* anchor_index, float fused_fraction,
                                float* thresholds, void* hip_stream)
{
    const ttf_status st = check_params(params);
    if (st != TTF_OK) return st;
    if (!best_sim || !anchor_index || !thresholds) return TTF_ERR_INVALID_ARG;
    if (!(fused_fraction >= 0.0f && fused_fraction <= 1.0f)) return TTF_ERR_INVALID_ARG;
    const hipError_t e = launch_select_threshold(*params, best_sim, anchor_index, 1.0 - (double)fused_fraction,
                                                 thresholds,
                                                 static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) {
        g_last_hip_error = static_cast<int>(e);
        return TTF_ERR_HIP;
    }
    return TTF_OK;
}

ttf_status ttf_regate(const ttf_params* params, const void* features, const float* thresholds,
                      void* workspace, size_t workspace_bytes, const ttf_outputs* out, void* hip_stream)
{
    const ttf_status st = check_params(params);
    if (st != TTF_OK) return st;
    if (!features || !workspace || !out) return TTF_ERR_INVALID_ARG;
    if (!out->tokens_out || !out->pos_ids || !out->src_index || !out->row_offsets || !out->kept_count ||
        !out->anchor_index || !out->fuse_map || !out->best_sim || !out->best_idx)
        return TTF_ERR_INVALID_ARG;
    if (!aligned(features, 16) || !aligned(out->tokens_out, 16) || !aligned(workspace, 256))
        return TTF_ERR_UNSUPPORTED;
    const ttf_params& p = *params;
    const Workspace w = carve(p, workspace);
    if (workspace_bytes < w.bytes) return TTF_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipError_t e = launch_regate(p, w, out->best_sim, out->best_idx, out->anchor_index, thresholds,
                                 out->fuse_map, s);
    if (e == hipSuccess)
        e = launch_offsets_scan(p, w, out->anchor_index, out->kept_count, out->row_offsets, false, s);
    if (e == hipSuccess)
        e = launch_emit_rows(p, features, w, out->row_offsets + p.B, out->tokens_out, out->pos_ids, out->src_index, 0,
                             false, s);
    if (e == hipSuccess && out->host_counts) {
        e = hipMemcpyAsync(out->host_counts, out->kept_count, sizeof(int32_t) * p.B, hipMemcpyDeviceToHost, s);
        if (e == hipSuccess)
            e = hipMemcpyAsync(out->host_counts + p.B, out->row_offsets, sizeof(int32_t) * (p.B + 1),
                               hipMemcpyDeviceToHost, s);
    }
    if (e != hipSuccess) {
        g_last_hip_error = static_cast<int>(e);
        return TTF_ERR_HIP;
    }
    return TTF_OK;
}

ttf_status ttf_search_route(const ttf_params* params, int* route)
{
    if (!route) return TTF_ERR_INVALID_ARG;
    const ttf_status st = check_params(params);
    if (st != TTF_OK) return st;
    const ttf_params& p = *params;
    *route = !use_mfma_path(p)              ? TTF_ROUTE_GENERAL
           : p.dtype == TTF_F32             ? TTF_ROUTE_MFMA_F32
           : mfma_search_supported(p)       ? TTF_ROUTE_MFMA_BF16
                                            : TTF_ROUTE_MFMA_BF16_PADDED;
    return TTF_OK;
}

ttf_status ttf_set_speculation(int mode)
{
    if (mode < -1 || mode > 1) return TTF_ERR_INVALID_ARG;
    g_speculation.store(mode, std::memory_order_relaxed);
    return TTF_OK;
}

const char* ttf_status_string(ttf_status status)
{
    switch (status) {
        case TTF_OK: return "ok";
        case TTF_ERR_INVALID_ARG: return "invalid argument";
        case TTF_ERR_UNSUPPORTED: return "unsupported dtype or alignment";
        case TTF_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case TTF_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

int ttf_last_hip_error(void) { return g_last_hip_error; }

ttf_status ttf_profile_enable(int slots)
{
    Profile& prof = g_prof;
    if (slots < 0 || slots > TTF_PROFILE_MAX_SLOTS) return TTF_ERR_INVALID_ARG;
    for (; prof.created < slots; ++prof.created) {
        for (int i = 0; i <= TTF_NUM_STAGES; ++i) {
            const hipError_t e = hipEventCreate(&prof.ev[prof.created][i]);
            if (e != hipSuccess) {
                for (int j = 0; j < i; ++j) (void)hipEventDestroy(prof.ev[prof.created][j]);
                g_last_hip_error = static_cast<int>(e);
                return TTF_ERR_HIP;
            }
        }
    }
    prof.slots = slots;
    prof.calls = 0;
    return TTF_OK;
}

ttf_status ttf_profile_read(int call, float* ms_out, int n)
{
    Profile& prof = g_prof;
    if (!ms_out || n < 0 || prof.slots <= 0) return TTF_ERR_INVALID_ARG;
    if (call < 0 || call >= prof.calls || call < prof.calls - prof.slots) return TTF_ERR_INVALID_ARG;
    hipEvent_t* ev = prof.ev[call % prof.slots];
    hipError_t e = hipEventSynchronize(ev[TTF_NUM_STAGES]);
    for (int i = 0; i < n && i < TTF_NUM_STAGES && e == hipSuccess; ++i)
        e = hipEventElapsedTime(&ms_out[i], ev[i], ev[i + 1]);
    if (e != hipSuccess) {
        g_last_hip_error = static_cast<int>(e);
        return TTF_ERR_HIP;
    }
    return TTF_OK;
}

const char* ttf_stage_name(int stage)
{
    static const char* names[TTF_NUM_STAGES] = {"frame_sums", "anchor_scores", "anchor_norms", "window_search",
                                                "anchor_verify", "offsets_scan", "emit_rows"};
    return (stage >= 0 && stage < TTF_NUM_STAGES) ? names[stage] : "";
}

}  // extern "C"
