// Video-adaptive threshold (Discussion D1): the threshold of a clip is read off the empirical
// distribution of its best-match similarities {s^(k,i)}, and the gate, the offsets and the row
// emission are redone at the new threshold from the stored s^ and dst, without another window
// search.
//
// The selection rule is an order statistic: for a requested fused fraction phi of the
// M = (F-1) N source tokens, t = the rank-th smallest s^ with rank = clamp(ceil((1-phi) M), 1, M);
// only tokens strictly above it are fused, so at most floor(phi M) are.  It is found exactly by a
// most-significant-digit-first radix selection over an order-preserving integer image of the
// floats: four passes of 256-bin counting, one workgroup per clip, integer LDS counters only
// (counts do not depend on the order of the additions).
#include "ttf_device.h"
#include "ttf_internal.h"

namespace ttf {
namespace {

// Monotone map float -> uint32: a < b as reals  <=>  key(a) < key(b)  (-0 sorts just below +0).
__device__ __forceinline__ uint32_t order_key(float v)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_value(uint32_t k)
{
    const uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __builtin_bit_cast(float, u);
}

__global__ __launch_bounds__(1024) void k_select_threshold(const float* __restrict__ best_sim,
                                                           const int32_t* __restrict__ anchor_index,
                                                           float* __restrict__ thresholds,
                                                           int F, int N, double keep_fraction)
{
    const int b = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int a = anchor_index[b];                   // < 0 (segment outputs): every frame is a source frame
    // rank of the order statistic among the clip's M source tokens: clamp(ceil((1 - phi) M), 1, M)
    const long long M = (long long)(a < 0 ? F : F - 1) * N;
    if (M == 0) {                                    // no source token: the documented default
        if (threadIdx.x == 0) thresholds[b] = 1.0f;
        return;
    }
    long long rank = (long long)ceil(keep_fraction * (double)M);
    rank = rank < 1 ? 1 : (rank > M ? M : rank);
    const float* sim = best_sim + (size_t)b * F * N;
    const long long FN = (long long)F * N;
    const long long skip_lo = (long long)a * N, skip_hi = skip_lo + N;   // the anchor frame is not a source
    __shared__ unsigned hist[16][256];               // one histogram per wave: no cross-wave contention
    __shared__ unsigned total[256];
    __shared__ uint32_t s_prefix;
    __shared__ long long s_k;
    if (threadIdx.x == 0) { s_prefix = 0u; s_k = rank - 1; }
    uint32_t mask = 0u;
    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int q = lane; q < 256; q += 64) hist[wave][q] = 0u;
        __syncthreads();
        const uint32_t prefix = s_prefix;
        // eight independent loads in flight per thread before their counts are added
        for (long long j0 = threadIdx.x; j0 < FN; j0 += 8 * 1024) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const long long j = j0 + 1024 * u;
                v[u] = j < FN ? sim[j] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const long long j = j0 + 1024 * u;
                const uint32_t key = order_key(v[u]);
                const bool act = j < FN && (j < skip_lo || j >= skip_hi) && (key & mask) == prefix;
                const uint32_t bin = (key >> shift) & 255u;
                if (shift == 24) {
                    // leading digit (sign and high exponent bits): similarities crowd into a few bins,
                    // so lanes with equal bins are counted together and one lane adds the count
                    uint64_t todo = __ballot(act);
                    while (todo) {
                        const int leader = __ffsll((unsigned long long)todo) - 1;
                        const uint32_t lb = (uint32_t)__shfl((int)bin, leader, 64);
                        const uint64_t same = __ballot(act && bin == lb);
                        if (lane == leader) hist[wave][lb] += (unsigned)__popcll(same);
                        todo &= ~same;
                    }
                } else if (act) {
                    atomicAdd(&hist[wave][bin], 1u);
                }
            }
        }
        __syncthreads();
        if (threadIdx.x < 256) {
            unsigned c = 0;
#pragma unroll
            for (int w = 0; w < 16; ++w) c += hist[w][threadIdx.x];
            total[threadIdx.x] = c;
        }
        __syncthreads();
        if (wave == 0) {
            // find the bin that holds the k-th remaining key: lane l owns bins 4l..4l+3, a wave scan
            // of the lane sums locates the lane, which then walks its four bins
            const long long k = s_k;
            unsigned c[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) c[e] = total[4 * lane + e];
            const long long mine = (long long)c[0] + c[1] + c[2] + c[3];
            long long incl = mine;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const long long o = __shfl_up(incl, d, 64);
                if (lane >= d) incl += o;
            }
            const uint64_t hit = __ballot(k < incl);          // never empty: k < number of remaining keys
            const int owner = hit ? __ffsll((unsigned long long)hit) - 1 : 63;
            if (lane == owner) {
                long long rest = k - (incl - mine);
                int e = 0;
                while (e < 3 && rest >= (long long)c[e]) { rest -= c[e]; ++e; }
                s_k = rest;
                s_prefix = prefix | ((uint32_t)(4 * lane + e) << shift);
            }
        }
        mask |= 255u << shift;
        __syncthreads();
    }
    if (threadIdx.x == 0) thresholds[b] = key_value(s_prefix);
}

// Gate from stored similarities: one wave per 64-token keep word.
__global__ __launch_bounds__(256) void k_regate(const float* __restrict__ best_sim,
                                                const int32_t* __restrict__ best_idx,
                                                const int32_t* __restrict__ anchor_index,
                                                const float* __restrict__ thresholds, float t_all,
                                                int32_t* __restrict__ fuse_map, uint64_t* __restrict__ keep_bits,
                                                int F, int N, int NW, size_t words)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t wd = (size_t)blockIdx.x * 4 + wave;          // global keep word
    if (wd >= words) return;
    const int word = (int)(wd % NW);
    const size_t frame = wd / NW;
    const int b = (int)(frame / F), k = (int)(frame % F);
    const float t = thresholds ? thresholds[b] : t_all;
    const int i = word * 64 + lane;
    bool keep = false;
    if (i < N) {
        const size_t o = frame * (size_t)N + i;
        const bool fused = k != anchor_index[b] && best_sim[o] > t;   // keep = 1[s^ <= t]
        fuse_map[o] = fused ? best_idx[o] : -1;
        keep = !fused;
    }
    const uint64_t bits = __ballot(keep);
    if (lane == 0) keep_bits[wd] = bits;
}

}  // namespace

hipError_t launch_select_threshold(const ttf_params& p, const float* best_sim, const int32_t* anchor_index,
                                   double keep_fraction, float* thresholds, hipStream_t s)
{
    k_select_threshold<<<(unsigned)p.B, 1024, 0, s>>>(best_sim, anchor_index, thresholds, p.F, p.H * p.W,
                                                      keep_fraction);
    return hipGetLastError();
}

hipError_t launch_regate(const ttf_params& p, const Workspace& w, const float* best_sim, const int32_t* best_idx,
                         const int32_t* anchor_index, const float* thresholds, int32_t* fuse_map, hipStream_t s)
{
    const int N = p.H * p.W, NW = (N + 63) / 64;
    const size_t words = (size_t)p.B * p.F * NW;
    k_regate<<<(unsigned)((words + 3) / 4), 256, 0, s>>>(best_sim, best_idx, anchor_index, thresholds, p.t,
                                                         fuse_map, w.keep_bits, p.F, N, NW, words);
    return hipGetLastError();
}

}  // namespace ttf
