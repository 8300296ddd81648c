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

// Long rows (at least 4 KiB): one block per token; the block of a kept token copies the row
// together, two 16-byte pieces per thread in flight, and the blocks of fused tokens leave at once.
// Many small blocks with little work per thread is the shape in which a plain device copy runs
// fastest on this chip (measured on 1 GiB: one or two pieces per thread 6.4-6.5 TB/s, eight pieces
// per lane in a loop 5.8; against the wave-per-row kernel above on 8 KiB rows: 0.138 -> 0.123 ms at
// 35 % kept rows, 0.345 -> 0.303 ms at 90 %; 2, 4, 8 or 16 tokens per block, 128 or 512 threads and
// rows split over two blocks were all slower).  Meaning of tied_rows as in k_emit_rows.
__global__ __launch_bounds__(256) void k_emit_row_blocks(const char* __restrict__ x,
                                                         const uint64_t* __restrict__ keep_bits,
                                                         const int32_t* __restrict__ frame_base,
                                                         char* __restrict__ tokens_out,
                                                         int32_t* __restrict__ pos_ids,
                                                         int32_t* __restrict__ src_index,
                                                         int F, int N, int W, int NW, size_t row_bytes, size_t cap,
                                                         int frame_offset, size_t tied_rows)
{
    const int bit = blockIdx.x & 63;
    const int word = (blockIdx.x >> 6) % NW;
    const size_t frame = (blockIdx.x >> 6) / NW;
    const int k = (int)(frame % F);
    const size_t meta = tied_rows ? (size_t)k : frame;
    const uint64_t* kb = keep_bits + meta * (size_t)NW;
    const uint64_t wbits = kb[word];
    if (((wbits >> bit) & 1ull) == 0) return;
    int before = frame_base[meta];
    for (int q = 0; q < word; ++q) before += __popcll(kb[q]);
    before += __popcll(wbits & ((1ull << bit) - 1ull));
    const int i = word * 64 + bit;
    const size_t row = (size_t)before;
    const size_t row0 = tied_rows ? (frame / F) * tied_rows : 0;
    const uint4* s = reinterpret_cast<const uint4*>(x + (frame * (size_t)N + i) * row_bytes);
    uint4* d = reinterpret_cast<uint4*>(tokens_out + (row0 + row) * row_bytes);
    const int n = (int)(row_bytes / 16);
    const int step = (int)blockDim.x;                         // 64..256 threads
    int q = threadIdx.x;
    for (; q + step < n; q += 2 * step) {
        const uint4 v0 = load16_stream(s + q), v1 = load16_stream(s + q + step);
        store16_stream(d + q, v0);
        store16_stream(d + q + step, v1);
    }
    if (q < n) store16_stream(d + q, load16_stream(s + q));
    if (threadIdx.x == 0 && (!tied_rows || frame < (size_t)F)) {
        pos_ids[row] = k + frame_offset;
        pos_ids[cap + row] = i / W;
        pos_ids[2 * cap + row] = i % W;
        src_index[row] = k * N + i;
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
                            const int32_t* anchor_index, void* tokens_out, int32_t* pos_ids,
                            int32_t* src_index, int frame_offset, bool tied, hipStream_t s)
{
    (void)anchor_index;
    const int N = p.H * p.W, NW = (N + 63) / 64;
    const size_t row_bytes = (size_t)p.C * (p.dtype == TTF_BF16 ? 2 : 4);
    const size_t tied_rows = tied ? (size_t)p.F * N : 0;
    const size_t cap = tied ? tied_rows : (size_t)p.B * p.F * N;  // length of one pos_ids plane
    const unsigned grid = (unsigned)((size_t)p.B * p.F * NW * 4);
    const char* xs = static_cast<const char*>(x);
    char* out = static_cast<char*>(tokens_out);
    // rows of 6 KiB and more: one block per token (below that the launch of the blocks of fused tokens
    // costs more than the denser copy gains; measured cross-over between 5 and 6 KiB at 35 % kept rows)
    constexpr size_t kRowBlockMin = 6144;
    const unsigned threads = (unsigned)(row_bytes / 16 >= 256 ? 256 : (row_bytes / 16 + 63) / 64 * 64);
    if (row_bytes % 16 == 0 && row_bytes >= kRowBlockMin)
        k_emit_row_blocks<<<(unsigned)((size_t)p.B * p.F * NW * 64), threads, 0, s>>>(
            xs, w.keep_bits, w.frame_base, out, pos_ids, src_index, p.F, N, p.W, NW, row_bytes, cap, frame_offset,
            tied_rows);
    else if (row_bytes % 16 == 0)
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
