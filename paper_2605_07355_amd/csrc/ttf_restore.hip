// Token restoration (Discussion D4: the full spatio-temporal layout is rebuilt from the compressed
// sequence through the matching map dst(k,i)) and the scalar bookkeeping of cache-aware decode
// alignment (Section 3: L_pre = L' + T, decode position and mask length).
//
// The restoration map says, for every original token, which row of the compressed sequence
// stands for it: a retained token is its own row; a fused token is represented by the anchor
// token it was matched to, and because the stacked X' starts with the N anchor rows in grid
// order, anchor token j of clip b is row row_offsets[b] + j.
#include "ttf_device.h"
#include "ttf_internal.h"

namespace ttf {
namespace {

// Thread (b, j), j < F*N.  Two disjoint sets of entries are written: fused tokens (from fuse_map)
// and retained tokens (row j of the clip names the token it was copied from in src_index).
__global__ __launch_bounds__(256) void k_restore_map(const int32_t* __restrict__ fuse_map,
                                                     const int32_t* __restrict__ row_offsets,
                                                     const int32_t* __restrict__ src_index,
                                                     int32_t* __restrict__ restore_map, int FN, int per_clip)
{
    const int b = blockIdx.x / per_clip;
    const int j = (blockIdx.x % per_clip) * 256 + threadIdx.x;
    if (j >= FN) return;
    const int first = row_offsets[b], rows = row_offsets[b + 1] - first;
    int32_t* out = restore_map + (size_t)b * FN;
    const int d = fuse_map[(size_t)b * FN + j];
    if (d >= 0) out[j] = first + d;
    if (j < rows) {
        const int tok = src_index[first + j];
        if (tok >= 0 && tok < FN) out[tok] = first + j;
    }
}

// One wave per original token: copies the row that represents it.  Entries outside [0, rows)
// (a map that does not belong to `tokens`) produce a zero row instead of a wild read.
template <int U>
__global__ __launch_bounds__(256) void k_restore_rows(const char* __restrict__ tokens,
                                                      const int32_t* __restrict__ restore_map,
                                                      char* __restrict__ restored, size_t total,
                                                      size_t row_bytes, long long rows)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t tok = (size_t)blockIdx.x * 4 + wave;
    if (tok >= total) return;
    const long long row = restore_map[tok];
    char* dst = restored + tok * row_bytes;
    if (row >= 0 && row < rows) {
        copy_row<U, false>(tokens + (size_t)row * row_bytes, dst, row_bytes, lane);   // rows are read many times
    } else {
        for (size_t q = lane * (size_t)U; q < row_bytes; q += 64 * (size_t)U)
            for (int e = 0; e < U; ++e) dst[q + e] = 0;
    }
}

// Long rows: one block per original token (blocks beyond the launch limit walk on by the grid size),
// the whole block copies the row: many small blocks with one or two 16-byte pieces per thread is the
// copy shape that runs fastest on this chip.
__global__ __launch_bounds__(256) void k_restore_row_blocks(const char* __restrict__ tokens,
                                                            const int32_t* __restrict__ restore_map,
                                                            char* __restrict__ restored, size_t row_bytes,
                                                            long long rows, size_t total)
{
    for (size_t tok = blockIdx.x; tok < total; tok += gridDim.x) {
        const long long row = restore_map[tok];
        uint4* d = reinterpret_cast<uint4*>(restored + tok * row_bytes);
        const int n = (int)(row_bytes / 16);
        const int step = (int)blockDim.x;
        int q = threadIdx.x;
        if (row >= 0 && row < rows) {
            const uint4* s = reinterpret_cast<const uint4*>(tokens + (size_t)row * row_bytes);
            for (; q + step < n; q += 2 * step) {
                const uint4 v0 = s[q], v1 = s[q + step];      // cached loads: anchor rows are read many times
                store16_stream(d + q, v0);
                store16_stream(d + q + step, v1);
            }
            if (q < n) store16_stream(d + q, s[q]);
        } else {
            for (; q < n; q += step) store16_stream(d + q, uint4{0u, 0u, 0u, 0u});
        }
    }
}

}  // namespace

hipError_t launch_restore_map(const ttf_params& p, const int32_t* fuse_map, const int32_t* row_offsets,
                              const int32_t* src_index, int32_t* restore_map, hipStream_t s)
{
    const int FN = p.F * p.H * p.W;
    const int per_clip = (FN + 255) / 256;
    k_restore_map<<<(unsigned)((size_t)p.B * per_clip), 256, 0, s>>>(fuse_map, row_offsets, src_index, restore_map,
                                                                     FN, per_clip);
    return hipGetLastError();
}

hipError_t launch_restore_rows(const ttf_params& p, const void* tokens, long long rows,
                               const int32_t* restore_map, void* restored, hipStream_t s)
{
    const size_t total = (size_t)p.B * p.F * p.H * p.W;
    const size_t row_bytes = (size_t)p.C * (p.dtype == TTF_BF16 ? 2 : 4);
    const unsigned grid = (unsigned)((total + 3) / 4);
    const char* in = static_cast<const char*>(tokens);
    char* out = static_cast<char*>(restored);
    constexpr size_t kRowBlockMin = 2048;
    if (row_bytes % 16 == 0 && row_bytes >= kRowBlockMin)
        k_restore_row_blocks<<<(unsigned)(total < kMaxBlocks256 ? total : kMaxBlocks256),
                               (unsigned)(row_bytes >= 4096 ? 256 : 128), 0, s>>>(in, restore_map, out, row_bytes, rows,
                                                                                   total);
    else if (row_bytes % 16 == 0)
        k_restore_rows<16><<<grid, 256, 0, s>>>(in, restore_map, out, total, row_bytes, rows);
    else if (row_bytes % 4 == 0)
        k_restore_rows<4><<<grid, 256, 0, s>>>(in, restore_map, out, total, row_bytes, rows);
    else
        k_restore_rows<2><<<grid, 256, 0, s>>>(in, restore_map, out, total, row_bytes, rows);
    return hipGetLastError();
}

}  // namespace ttf
