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
// is written to win_sim[b][k][(dy+r)*(2r+1) + (dx+r)][i] instead and nothing else is produced.
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
                        if (lane == 0) win_sim[(frame * (size_t)((2 * r + 1) * (2 * r + 1)) + slot) * N + i] = sim;
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


// acc + sum over the 16 bytes of a[i]*b[i]: four packed dot products for bf16 (exact products,
// fp32 accumulation), four FMAs for fp32.
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
template <typename T>
__device__ __forceinline__ float dot16(u32x4 a, u32x4 b, float acc)
{
    // (elements are copied to plain words first: arithmetic on elements extracted from a bit-cast
    // vector has been seen to read the wrong element)
    const uint32_t aw[4] = {a[0], a[1], a[2], a[3]}, bw[4] = {b[0], b[1], b[2], b[3]};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if constexpr (sizeof(T) == 2)
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, aw[i]), __builtin_bit_cast(bf16x2, bw[i]), acc, false);
        else
            acc = fmaf(__builtin_bit_cast(float, aw[i]), __builtin_bit_cast(float, bw[i]), acc);
    }
    return acc;
}

// Tiled form of the same search for large inputs with r <= RMAX (1 or 2) and 16-byte row pieces.
// A workgroup (8 waves) owns a patch of 8 rows x PT columns of source tokens of one frame (PT = 8
// for the 3x3 window, 4 for the 5x5 window, where every token needs 25 partial sums); the anchor
// cells its windows can touch (the patch plus RMAX cells on every side) are staged in LDS one
// 64*V-channel chunk at a time (16 bytes per lane and cell), so an anchor row is fetched once per
// patch instead of once per source token that has it in its window, whatever the grid width.
// Wave w owns patch row w: it keeps the partial dot products of its PT tokens with their
// candidates in registers across the chunks and reduces them over the lanes once at the end.
// The halo pieces of the next chunk are requested into registers before the current chunk is
// computed and are written to LDS at the top of the next iteration, so those loads overlap the
// arithmetic.  Patches do not line up with keep words; the words are packed from the fuse map
// afterwards.
template <int RMAX>
struct Patch {
    static constexpr int ROWS = 8;                    // one per wave
    static constexpr int PT = RMAX == 1 ? 8 : 4;      // tokens per wave
    static constexpr int HW = PT + 2 * RMAX, HH = ROWS + 2 * RMAX, CELLS = HW * HH;
    static constexpr int K1 = 2 * RMAX + 1, G = K1 * K1;
};
template <typename T, int V, int RMAX, bool ALL>
__global__ __launch_bounds__(512) void k_search_tiled(
    const T* __restrict__ x, const T* __restrict__ ext_anchor, const int32_t* __restrict__ anchor_index,
    const float* __restrict__ anchor_inv,
    int32_t* __restrict__ fuse_map, float* __restrict__ best_sim, int32_t* __restrict__ best_idx,
    float* __restrict__ win_sim, int F, int H, int W, int C, int r, float t, int tiles_x, int tiles)
{
    using P = Patch<RMAX>;
    constexpr int PT = P::PT, HW = P::HW, K1 = P::K1, G = P::G;
    constexpr int HP = (P::CELLS + 7) / 8;            // halo cells a wave stages per chunk
    extern __shared__ u32x4 halo[];                   // [halo cell][lane]
    const int N = H * W;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tile = blockIdx.x % tiles;
    const size_t frame = blockIdx.x / tiles;
    const int b = (int)(frame / F), k = (int)(frame % F);
    const int a = anchor_index[b];
    const int ty0 = (tile / tiles_x) * P::ROWS, tx0 = (tile % tiles_x) * PT;
    const int y = ty0 + wave;                         // this wave's grid row
    if (k == a) {                                     // anchor tokens are always retained
        if (!ALL && lane < PT && y < H && tx0 + lane < W) {
            const int i = y * W + tx0 + lane;
            const size_t o = frame * (size_t)N + i;
            fuse_map[o] = -1;
            if (best_sim) best_sim[o] = 1.0f;
            if (best_idx) best_idx[o] = i;
        }
        return;
    }
    const T* anchor = a < 0 ? ext_anchor + (size_t)b * N * C : x + ((size_t)b * F + a) * (size_t)N * C;
    const float* ainv = anchor_inv + (size_t)b * N;
    const T* src = x + (frame * (size_t)N + (size_t)min(y, H - 1) * W + tx0) * (size_t)C;
    const int ntok = y < H ? min(PT, W - tx0) : 0;    // tokens of this wave

    // this wave's halo cells: cell j = wave + 8*h is grid cell (ty0 - RMAX + j / HW, tx0 - RMAX + j % HW)
    int hoff[HP];                                     // token index in the anchor frame, -1 outside the grid
#pragma unroll
    for (int h = 0; h < HP; ++h) {
        const int j = wave + 8 * h;
        const int hy = ty0 - RMAX + j / HW, hx = tx0 - RMAX + j % HW;
        hoff[h] = (j < P::CELLS && hy >= 0 && hy < H && hx >= 0 && hx < W) ? hy * W + hx : -1;
    }
    float dot[PT][G], nn[PT];
#pragma unroll
    for (int q = 0; q < PT; ++q) {
        nn[q] = 0.f;
#pragma unroll
        for (int g = 0; g < G; ++g) dot[q][g] = 0.f;
    }
    const int chunks = (C + 64 * V - 1) / (64 * V);
    u32x4 hreg[HP];                                   // halo pieces of the chunk in flight
#pragma unroll
    for (int h = 0; h < HP; ++h) {
        hreg[h] = u32x4{0u, 0u, 0u, 0u};
        if (hoff[h] >= 0 && lane * V < C) hreg[h] = *reinterpret_cast<const u32x4*>(anchor + (size_t)hoff[h] * C + lane * V);
    }
    for (int ch = 0; ch < chunks; ++ch) {
#pragma unroll
        for (int h = 0; h < HP; ++h) {
            const int j = wave + 8 * h;
            if (j < P::CELLS) halo[j * 64 + lane] = hreg[h];
        }
        __syncthreads();
        {                                             // next chunk's halo pieces: consumed at the top of the next iteration
            const int cn = (min(ch + 1, chunks - 1) * 64 + lane) * V;
#pragma unroll
            for (int h = 0; h < HP; ++h) {
                hreg[h] = u32x4{0u, 0u, 0u, 0u};
                if (hoff[h] >= 0 && cn < C) hreg[h] = *reinterpret_cast<const u32x4*>(anchor + (size_t)hoff[h] * C + cn);
            }
        }
        const int c = (ch * 64 + lane) * V;
        u32x4 s[PT];
#pragma unroll
        for (int q = 0; q < PT; ++q) {
            s[q] = u32x4{0u, 0u, 0u, 0u};
            if (q < ntok && c < C) s[q] = *reinterpret_cast<const u32x4*>(src + (size_t)q * C + c);
        }
#pragma unroll
        for (int q = 0; q < PT; ++q) nn[q] = dot16<T>(s[q], s[q], nn[q]);
        // every halo cell of the K1 rows around this wave's row is read once and multiplied with the
        // (up to K1) tokens that have it in their window; cells outside the grid hold zeros and pieces
        // of absent tokens are zeros, so nothing needs a branch here -- candidates that do not exist
        // are left out when the arg max is taken
#pragma unroll
        for (int hr = 0; hr < K1; ++hr) {
#pragma unroll
            for (int hc = 0; hc < HW; ++hc) {
                const u32x4 cell = halo[((wave + hr) * HW + hc) * 64 + lane];
#pragma unroll
                for (int q = 0; q < PT; ++q) {
                    const int dx = hc - RMAX - q;         // column offset of this cell from token q
                    if (dx >= -RMAX && dx <= RMAX)
                        dot[q][hr * K1 + dx + RMAX] = dot16<T>(s[q], cell, dot[q][hr * K1 + dx + RMAX]);
                }
            }
        }
        __syncthreads();
    }

#pragma unroll
    for (int q = 0; q < PT; ++q) {
        if (q < ntok) {
            const int xx = tx0 + q;
            const int i = y * W + xx;
            const size_t o = frame * (size_t)N + i;
            const float ss = wave_sum(nn[q]);
            const float src_inv = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
            float best = kNegInf;
            int arg = -1;
#pragma unroll
            for (int dy = -RMAX; dy <= RMAX; ++dy) {
                if (dy < -r || dy > r || y + dy < 0 || y + dy >= H) continue;
#pragma unroll
                for (int dx = -RMAX; dx <= RMAX; ++dx) {
                    if (dx < -r || dx > r || xx + dx < 0 || xx + dx >= W) continue;
                    const int cand = (y + dy) * W + xx + dx;
                    const float sim = wave_sum(dot[q][(dy + RMAX) * K1 + dx + RMAX]) * src_inv * ainv[cand];
                    if constexpr (ALL) {
                        if (lane == 0)
                            win_sim[(frame * (size_t)((2 * r + 1) * (2 * r + 1)) + (dy + r) * (2 * r + 1) + dx + r) * N + i] = sim;
                    } else if (sim > best) {          // ascending index, strict: first maximum
                        best = sim;
                        arg = cand;
                    }
                }
            }
            if (!ALL && lane == 0) {
                const bool fused = best > t;          // keep = 1[s^ <= t]
                fuse_map[o] = fused ? arg : -1;
                if (best_sim) best_sim[o] = best;
                if (best_idx) best_idx[o] = arg;
            }
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
        if constexpr (V > 1) {
            // large inputs, windows up to 5x5: patches of source tokens with their anchor halo staged in LDS
            if (!small && p.r <= 2) {
                auto tiled = [&](auto kernel, auto patch) {
                    using P = decltype(patch);
                    const int tiles_x = (p.W + P::PT - 1) / P::PT, tiles = tiles_x * ((p.H + P::ROWS - 1) / P::ROWS);
                    const size_t lds = (size_t)P::CELLS * 1024;
                    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kernel), lds);
                    if (e != hipSuccess) return e;
                    kernel<<<(unsigned)((size_t)p.B * p.F * tiles), 512, lds, s>>>(
                        static_cast<const T*>(x), static_cast<const T*>(ext_anchor), anchor_index, w.anchor_inv,
                        fuse_map, best_sim, best_idx, win_sim, p.F, p.H, p.W, p.C, p.r, p.t, tiles_x, tiles);
                    return hipGetLastError();
                };
                hipError_t e;
                if (p.r <= 1) e = win_sim ? tiled(k_search_tiled<T, V, 1, true>, Patch<1>{}) : tiled(k_search_tiled<T, V, 1, false>, Patch<1>{});
                else e = win_sim ? tiled(k_search_tiled<T, V, 2, true>, Patch<2>{}) : tiled(k_search_tiled<T, V, 2, false>, Patch<2>{});
                if (e != hipSuccess || win_sim) return e;               // tied-batch mode: the tie kernel forms the keep words
                return launch_pack_keep(p, fuse_map, anchor_index, w, s);
            }
        }
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
