// Sequence compaction and positional alignment (Section 3: stacked X' = [anchor rows ; kept
// source rows], retention mask m_{k,i}, gather of X and P by I_keep, L' = N + P).
//
// The search leaves one keep bit per token.  A single small block turns per-frame popcounts
// into output row offsets (anchor frame first inside each clip, clips packed one after the
// other); the emit kernel then copies every kept row bit-exactly and writes its original
// (k, y, x) triple and flat index.
#include "ttf_device.h"
#include "ttf_internal.h"

namespace ttf {
namespace {

// Exclusive scan over the sequence  [N, c(b,0), ..., c(b,F-1)]  for b = 0..B-1, where c(b,k) is
// the number of kept tokens of source frame k and 0 for the anchor frame.  The entry in front
// of each clip places its N anchor rows first.
__global__ __launch_bounds__(1024) void k_offsets_scan(const uint64_t* __restrict__ keep_bits,
                                                       const int32_t* __restrict__ anchor_index,
                                                       int32_t* __restrict__ frame_base,
                                                       int32_t* __restrict__ kept_count,
                                                       int32_t* __restrict__ row_offsets,
                                                       int B, int F, int N, int NW)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    __shared__ int wave_tot[16];
    __shared__ int carry_s;
    if (tid == 0) carry_s = 0;
    __syncthreads();
    const long long E = (long long)B * (F + 1);
    for (long long e0 = 0; e0 < E; e0 += 1024) {
        const long long e = e0 + tid;
        int v = 0, b = 0, s = 0, a = 0;
        if (e < E) {
            b = (int)(e / (F + 1));
            s = (int)(e % (F + 1));
            a = anchor_index[b];                       // < 0: the anchor frame is not part of the clip
            if (s == 0) {
                v = a < 0 ? 0 : N;
            } else if (s - 1 != a) {
                const uint64_t* kb = keep_bits + ((size_t)b * F + (s - 1)) * NW;
                for (int q = 0; q < NW; ++q) v += __popcll(kb[q]);
            }
        }
        int inc = v;                                   // inclusive scan inside the wave
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int o = __shfl_up(inc, d, 64);
            if (lane >= d) inc += o;
        }
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();
        int pre = carry_s;
        for (int q = 0; q < wave; ++q) pre += wave_tot[q];
        const int excl = pre + inc - v;
        if (e < E) {
            if (s == 0) {
                row_offsets[b] = excl;
                if (a >= 0) frame_base[(size_t)b * F + a] = excl;
            } else if (s - 1 != a) {
                frame_base[(size_t)b * F + (s - 1)] = excl;
            }
        }
        __syncthreads();
        if (tid == 1023) carry_s = excl + v;
        __syncthreads();
    }
    if (tid == 0) row_offsets[B] = carry_s;
    __syncthreads();
    for (int b = tid; b < B; b += 1024) kept_count[b] = row_offsets[b + 1] - row_offsets[b];
}

// One block = 16 tokens (a quarter of a 64-token keep word) of one frame; its kept tokens are dealt
// to the four waves by rank.  tied_rows > 0 (tied-batch mode): keep bits and frame bases are shared
// by all clips ([F,NW] and [F]), clip b writes its rows at row b*tied_rows + shared row, and only
// clip 0 writes the shared position ids and source indices.  Small blocks matter: a wave copies its rows one after the other, so
// the fewer rows per wave, the more copies are in flight across the chip.
template <int U>
__global__ __launch_bounds__(256) void k_emit_rows(const char* __restrict__ x,
                                                   const uint64_t* __restrict__ keep_bits,
                                                   const int32_t* __restrict__ frame_base,
                                                   char* __restrict__ tokens_out,
                                                   int32_t* __restrict__ pos_ids,
                                                   int32_t* __restrict__ src_index,
                                                   int F, int N, int W, int NW, size_t row_bytes, size_t cap,
                                                   int frame_offset, size_t tied_rows)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int quarter = blockIdx.x & 3;
    const int word = (blockIdx.x >> 2) % NW;
    const size_t frame = (blockIdx.x >> 2) / NW;
    const int k = (int)(frame % F);
    const size_t meta = tied_rows ? (size_t)k : frame;        // which frame's bits and base to use
    const size_t row0 = tied_rows ? (frame / F) * tied_rows : 0;
    const bool ids = !tied_rows || frame < (size_t)F;
    const uint64_t* kb = keep_bits + meta * (size_t)NW;
    const uint64_t wbits = kb[word];
    const uint64_t bits = wbits & (0xffffull << (16 * quarter));
    if (bits == 0) return;
    int before = frame_base[meta];
    for (int q = 0; q < word; ++q) before += __popcll(kb[q]);
    before += __popcll(wbits & ((1ull << (16 * quarter)) - 1ull));
    uint64_t rem = bits;
    for (int rank = 0; rem != 0; ++rank) {
        const int bit = __ffsll((unsigned long long)rem) - 1;
        rem &= rem - 1;
        if ((rank & 3) != wave) continue;
        const int i = word * 64 + bit;
        const size_t row = (size_t)before + rank;
        copy_row<U>(x + (frame * (size_t)N + i) * row_bytes, tokens_out + (row0 + row) * row_bytes, row_bytes, lane);
        if (ids && lane == 0) {
            pos_ids[row] = k + frame_offset;
            pos_ids[cap + row] = i / W;
            pos_ids[2 * cap + row] = i % W;
            src_index[row] = k * N + i;
        }
    }
}

// Rows of 1 KiB and more are emitted in two steps, so that the copy runs in the shape a plain device
// copy is fastest in on this chip -- many small blocks, a whole block on one row, one or two 16-byte
// pieces per thread (measured on 1 GiB: 6.4-6.5 TB/s against 5.8 for eight pieces per lane in a
// loop) -- without launching blocks for fused tokens (a block per input token costs 0.17 ms of
// launches alone on 262 144 tokens of which 17 % are kept).
//
// Step 1, one wave per keep word: the ids of every kept token and, in src_row[r], the input token
// that output row r copies.  tied_rows > 0: the mask is the shared one ([F,NW]); ids and src_row
// are those of one clip.
__global__ __launch_bounds__(256) void k_emit_ids(const uint64_t* __restrict__ keep_bits,
                                                  const int32_t* __restrict__ frame_base,
                                                  int32_t* __restrict__ pos_ids, int32_t* __restrict__ src_index,
                                                  int32_t* __restrict__ src_row, int F, int N, int W, int NW,
                                                  size_t words, size_t cap, int frame_offset)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t wd = (size_t)blockIdx.x * 4 + wave;
    if (wd >= words) return;
    const int word = (int)(wd % NW);
    const size_t frame = wd / NW;
    const int k = (int)(frame % F);
    const uint64_t* kb = keep_bits + frame * (size_t)NW;
    const uint64_t wbits = kb[word];
    if (((wbits >> lane) & 1ull) == 0) return;
    int before = frame_base[frame];
    for (int q = 0; q < word; ++q) before += __popcll(kb[q]);
    const size_t row = (size_t)before + __popcll(wbits & ((1ull << lane) - 1ull));
    const int i = word * 64 + lane;
    pos_ids[row] = k + frame_offset;
    pos_ids[cap + row] = i / W;
    pos_ids[2 * cap + row] = i % W;
    src_index[row] = k * N + i;
    src_row[row] = (int32_t)(frame * (size_t)N + i);
}

// Step 2: block j copies output rows j, j + gridDim.x, ... below *total_rows.  blockIdx.y = clip in
// tied-batch mode (input tokens src_clip_stride apart, output rows dst_clip_stride apart), 0 otherwise.
__global__ __launch_bounds__(256) void k_copy_rows(const char* __restrict__ x, const int32_t* __restrict__ src_row,
                                                   const int32_t* __restrict__ total_rows,
                                                   char* __restrict__ tokens_out, size_t row_bytes,
                                                   size_t src_clip_stride, size_t dst_clip_stride)
{
    const int total = *total_rows;
    const int n = (int)(row_bytes / 16);
    const int step = (int)blockDim.x;
    const char* xs = x + blockIdx.y * src_clip_stride * row_bytes;
    char* out = tokens_out + blockIdx.y * dst_clip_stride * row_bytes;
    for (int r = blockIdx.x; r < total; r += gridDim.x) {
        const uint4* s = reinterpret_cast<const uint4*>(xs + (size_t)src_row[r] * row_bytes);
        uint4* d = reinterpret_cast<uint4*>(out + (size_t)r * row_bytes);
        int q = threadIdx.x;
        for (; q + step < n; q += 2 * step) {
            const uint4 v0 = load16_stream(s + q), v1 = load16_stream(s + q + step);
            store16_stream(d + q, v0);
            store16_stream(d + q + step, v1);
        }
        if (q < n) store16_stream(d + q, load16_stream(s + q));
    }
}

}  // namespace

hipError_t launch_offsets_scan(const ttf_params& p, const Workspace& w, const int32_t* anchor_index,
                               int32_t* kept_count, int32_t* row_offsets, bool tied, hipStream_t s)
{
    const int N = p.H * p.W, NW = (N + 63) / 64;
    // tied-batch mode: one shared mask, i.e. the scan of a single clip
    k_offsets_scan<<<1, 1024, 0, s>>>(w.keep_bits, anchor_index, w.frame_base, kept_count, row_offsets,
                                      tied ? 1 : p.B, p.F, N, NW);
    return hipGetLastError();
}

hipError_t launch_emit_rows(const ttf_params& p, const void* x, const Workspace& w,
                            const int32_t* total_rows, void* tokens_out, int32_t* pos_ids,
                            int32_t* src_index, int frame_offset, bool tied, hipStream_t s)
{
    const int N = p.H * p.W, NW = (N + 63) / 64;
    const size_t row_bytes = (size_t)p.C * (p.dtype == TTF_BF16 ? 2 : 4);
    const size_t tied_rows = tied ? (size_t)p.F * N : 0;
    const size_t cap = tied ? tied_rows : (size_t)p.B * p.F * N;  // length of one pos_ids plane
    const unsigned grid = (unsigned)((size_t)p.B * p.F * NW * 4);
    const char* xs = static_cast<const char*>(x);
    char* out = static_cast<char*>(tokens_out);
    constexpr size_t kRowBlockMin = 1024;
    if (row_bytes % 16 == 0 && row_bytes >= kRowBlockMin && (!tied || p.B <= 65535)) {   // (clips ride on gridDim.y)
        const size_t words = (size_t)(tied ? 1 : p.B) * p.F * NW;
        k_emit_ids<<<(unsigned)((words + 3) / 4), 256, 0, s>>>(w.keep_bits, w.frame_base, pos_ids, src_index, w.src_row,
                                                              p.F, N, p.W, NW, words, cap, frame_offset);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        // a quarter as many blocks as there could be rows: at the usual kept fractions every block has
        // one to four rows; 64 threads per KiB of row, at most 256
        const unsigned threads = (unsigned)(row_bytes >= 4096 ? 256 : row_bytes / 1024 * 64);
        const size_t want = (cap + 3) / 4;
        const unsigned blocks = (unsigned)(want < kMaxBlocks256 ? want : kMaxBlocks256);
        k_copy_rows<<<dim3(blocks, tied ? p.B : 1), threads, 0, s>>>(xs, w.src_row, total_rows, out, row_bytes,
                                                                     tied_rows, tied_rows);
        return hipGetLastError();
    }
    if (row_bytes % 16 == 0)
        k_emit_rows<16><<<grid, 256, 0, s>>>(xs, w.keep_bits, w.frame_base, out, pos_ids, src_index,
                                             p.F, N, p.W, NW, row_bytes, cap, frame_offset, tied_rows);
    else if (row_bytes % 4 == 0)
        k_emit_rows<4><<<grid, 256, 0, s>>>(xs, w.keep_bits, w.frame_base, out, pos_ids, src_index,
                                            p.F, N, p.W, NW, row_bytes, cap, frame_offset, tied_rows);
    else
        k_emit_rows<2><<<grid, 256, 0, s>>>(xs, w.keep_bits, w.frame_base, out, pos_ids, src_index,
                                            p.F, N, p.W, NW, row_bytes, cap, frame_offset, tied_rows);
    return hipGetLastError();
}

}  // namespace ttf
