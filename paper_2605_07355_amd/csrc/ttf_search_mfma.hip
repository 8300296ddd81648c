// Window search and gate for bf16 tokens on grids 16 or 32 tokens wide (Section 3, "Pointwise
// Matching with Local Window Search" and "Threshold Gating"), on the gfx950 matrix cores.
//
// Why matrix cores for a banded product: the (2r+1)^2 dot products per source token cost
// 2(2r+1)^2 C + 2C flops per 2C input bytes.  On the plain vector ALUs (78.6 TFLOP/s fp32
// without packed math) that arithmetic alone would take as long as streaming the tokens from
// HBM at its peak rate, before any bf16 unpacking or cross-lane reduction.  A 16x16x32 bf16
// MFMA computes a source tile (16 consecutive tokens of a grid row) against an anchor tile (16
// consecutive anchor tokens) with fp32 accumulation at a small fraction of that cost; only the
// band |dx| <= r of each 16x16 result is used.  The kernel is then bound by HBM, as intended.
//
// Work split.  One workgroup of 8 wavefronts owns 32 consecutive tokens of one source frame
// (two source tiles: two grid rows when W = 16, one grid row when W = 32).  The channel axis is
// split across the wavefronts: wave w owns channels [w*C/8, (w+1)*C/8).  Each wave loads its
// slice of both source tiles straight from HBM into registers in MFMA operand layout (16 rows x
// 64 bytes per load; the dot product is invariant under any permutation of channels applied to
// both operands, so the natural 8-channel groups per lane are used), streams the matching
// slices of the anchor tiles from L2, and accumulates partial 16x16 products.  The partials of
// the 8 waves are added through LDS in wave order (fixed order: results are reproducible),
// then one wave per source tile forms the cosines, masks the band, takes the arg max (lowest
// anchor index on ties), applies the threshold and writes s^, dst, the fuse map and 16 keep bits.
//
// Source squared norms come from the diagonal of tile x tile^T on the matrix cores; anchor
// inverse norms are precomputed per clip.
#include "ttf_device.h"
#include "ttf_internal.h"

namespace ttf {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kWaves = 8;                 // wavefronts per workgroup = channel slices
constexpr int kGroup = 7;                 // result tiles reduced through LDS per round (7*8 KiB)
constexpr float kNegInf = -__builtin_inff();

// Geometry of one workgroup's problem.  CT = W/16 column tiles per grid row.
template <int CT, int RAD>
struct Shape {
    static_assert(CT == 1 || CT == 2, "grids of width 16 or 32");
    static constexpr int W = 16 * CT;
    static constexpr int ROWS = (2 * RAD + 1);
    // anchor tiles held per K-step: CT==1: rows y0-RAD .. y0+1+RAD; CT==2: rows y-RAD .. y+RAD, 2 columns
    static constexpr int NA = CT == 1 ? 2 * RAD + 2 : 2 * ROWS;
    // anchor tiles paired with each source tile
    static constexpr int NPS = CT == 1 ? ROWS : 2 * ROWS;
    // anchor tile index of pair q of source tile s
    __device__ static constexpr int pair_tile(int s, int q) { return CT == 1 ? s + q : q; }
    __device__ static constexpr int tile_row(int a) { return CT == 1 ? a : a / 2; }   // offset from ylo
    __device__ static constexpr int tile_col(int a) { return CT == 1 ? 0 : a % 2; }
    __device__ static constexpr int src_col(int s) { return CT == 1 ? 0 : s; }
    __device__ static constexpr int src_row(int s) { return CT == 1 ? s : 0; }       // offset from first row
    // K-steps of both source tiles a wave keeps in registers at once; bounded by the 256 VGPRs a
    // wave may use at two waves per SIMD (accumulators take 8*(NPS+1), anchor fragments 4*NA)
    static constexpr int MAXK = NPS <= 3 ? 16 : (NPS <= 6 ? 8 : 4);
    // K-steps of anchor fragments requested ahead of use (ring of PF+1 buffers, 4*NA VGPRs each)
    static constexpr int PF = NA <= 4 ? 3 : (NA <= 6 ? 2 : 1);
};

__device__ __forceinline__ bf16x8 load_frag(const uint16_t* p)
{
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p));
}

template <int CT, int RAD, int KSW, int PF>
__global__ __launch_bounds__(kWaves * 64) void k_search_mfma(
    const uint16_t* __restrict__ x, const int32_t* __restrict__ anchor_index,
    const float* __restrict__ anchor_inv, int32_t* __restrict__ fuse_map, float* __restrict__ best_sim,
    int32_t* __restrict__ best_idx, uint16_t* __restrict__ keep16, int F, int H, int C, float t, int passes)
{
    using S = Shape<CT, RAD>;
    constexpr int W = S::W, NA = S::NA, NPS = S::NPS;
    constexpr int NB = PF + 1;                               // anchor fragment ring
    const int N = H * W;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int tpf = N / 32;                                  // workgroups per frame
    const int tp = blockIdx.x % tpf;
    const size_t frame = blockIdx.x / tpf;                   // b*F + k
    const int b = (int)(frame / F), k = (int)(frame % F);
    const int a = anchor_index[b];
    const int i0 = tp * 32;                                  // first token of this workgroup
    const size_t o0 = frame * (size_t)N + i0;

    if (k == a) {                                            // anchor tokens are always retained
        if (threadIdx.x < 32) {
            fuse_map[o0 + threadIdx.x] = -1;
            if (best_sim) best_sim[o0 + threadIdx.x] = 1.0f;
            if (best_idx) best_idx[o0 + threadIdx.x] = i0 + threadIdx.x;
        }
        if (threadIdx.x < 2) keep16[o0 / 16 + threadIdx.x] = 0xffffu;
        return;
    }

    const int y0 = i0 / W;                                   // first (or only) source row
    const int ylo = y0 - RAD;
    const int slice = C / kWaves;                            // channels per wave
    const uint16_t* xf = x + frame * (size_t)N * C;
    const uint16_t* xa = x + ((size_t)b * F + a) * (size_t)N * C;
    const int kofs = wave * slice + g * 8;

    const uint16_t* sp[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) sp[s] = xf + (size_t)(i0 + 16 * s + m) * C + kofs;
    const uint16_t* ap[NA];
#pragma unroll
    for (int q = 0; q < NA; ++q) {
        const int yy = min(max(ylo + S::tile_row(q), 0), H - 1);      // rows outside the grid: clamped, masked later
        ap[q] = xa + (size_t)(yy * W + 16 * S::tile_col(q) + m) * C + kofs;
    }

    f32x4 acc[2][NPS], nrm[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        nrm[s] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int q = 0; q < NPS; ++q) acc[s][q] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    for (int pass = 0; pass < passes; ++pass) {
        const int off = pass * KSW * 32;
        // Anchor fragments run PF K-steps ahead of their use in a ring of PF+1 buffers.  Their
        // first PF K-steps are requested before the source loads: loads complete in issue order,
        // so products can start as soon as the first source fragments land.
        bf16x8 Bt[NB][NA];
#pragma unroll
        for (int d = 0; d < PF && d < KSW; ++d) {
#pragma unroll
            for (int q = 0; q < NA; ++q) Bt[d][q] = load_frag(ap[q] + off + d * 32);
        }
        bf16x8 A[2][KSW];
#pragma unroll
        for (int ks = 0; ks < KSW; ++ks) {
#pragma unroll
            for (int s = 0; s < 2; ++s) A[s][ks] = load_frag(sp[s] + off + ks * 32);
        }
        // all source loads of the pass go out before any product: that many bytes in flight per
        // wave is what hides HBM latency (the scheduler would otherwise sink them to their uses)
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < KSW; ++ks) {
            if (ks + PF < KSW) {
#pragma unroll
                for (int q = 0; q < NA; ++q) Bt[(ks + PF) % NB][q] = load_frag(ap[q] + off + (ks + PF) * 32);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                nrm[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[s][ks], A[s][ks], nrm[s], 0, 0, 0);
#pragma unroll
                for (int q = 0; q < NPS; ++q)
                    acc[s][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[s][ks], Bt[ks % NB][S::pair_tile(s, q)],
                                                                        acc[s][q], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // ---- add the 8 channel slices through LDS (wave order), one source tile at a time ----
    __shared__ f32x4 red[kWaves][kGroup][64];
    const float* ainv = anchor_inv + (size_t)b * N;

#pragma unroll
    for (int s = 0; s < 2; ++s) {
        float best[4] = {kNegInf, kNegInf, kNegInf, kNegInf};
        int arg[4] = {-1, -1, -1, -1};
        float sinv[4] = {0.f, 0.f, 0.f, 0.f};
        // tile slot 0 is the norm tile, slots 1..NPS the pair tiles; groups of kGroup slots
#pragma unroll
        for (int base = 0; base <= NPS; base += kGroup) {
#pragma unroll
            for (int u = 0; u < kGroup; ++u) {
                const int slot = base + u;
                if (slot <= NPS) red[wave][u][lane] = slot == 0 ? nrm[s] : acc[s][slot == 0 ? 0 : slot - 1];
            }
            __syncthreads();
            if (wave == s) {
#pragma unroll
                for (int u = 0; u < kGroup; ++u) {
                    const int slot = base + u;
                    if (slot > NPS) continue;
                    f32x4 v = red[0][u][lane];
#pragma unroll
                    for (int w = 1; w < kWaves; ++w) {
                        const f32x4 p = red[w][u][lane];
                        v[0] += p[0]; v[1] += p[1]; v[2] += p[2]; v[3] += p[3];
                    }
                    if (slot == 0) {
                        // ||x_{k,i}||^2 of token 4g+j sits on the diagonal: lane 16g + 4g + j, element j
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const float nn = __shfl(v[j], (lane & 48) + 4 * g + j, 64);
                            sinv[j] = nn > 0.f ? 1.0f / sqrtf(nn) : 0.f;
                        }
                    } else {
                        const int q = slot - 1;
                        const int tile = S::pair_tile(s, q);
                        const int yy = ylo + S::tile_row(tile);
                        const int xa_col = 16 * S::tile_col(tile) + m;          // this lane's anchor column
                        const bool row_ok = yy >= 0 && yy < H &&
                                            yy >= y0 + S::src_row(s) - RAD && yy <= y0 + S::src_row(s) + RAD;
                        const int ja = yy * W + xa_col;
                        const float ai = row_ok ? ainv[ja] : 0.f;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int xs_col = 16 * S::src_col(s) + 4 * g + j;  // source token's column
                            const int dx = xa_col - xs_col;
                            if (row_ok && dx >= -RAD && dx <= RAD) {
                                const float sim = v[j] * sinv[j] * ai;
                                if (sim > best[j]) { best[j] = sim; arg[j] = ja; }   // ascending ja per lane
                            }
                        }
                    }
                }
            }
            __syncthreads();
        }
        if (wave == s) {
            // arg max across the 16 anchor columns held by the 16 lanes of a group; lowest index on ties
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int d = 1; d < 16; d <<= 1) {
                    const float ob = __shfl_xor(best[j], d, 64);
                    const int oa = __shfl_xor(arg[j], d, 64);
                    if (ob > best[j] || (ob == best[j] && oa >= 0 && (arg[j] < 0 || oa < arg[j]))) {
                        best[j] = ob;
                        arg[j] = oa;
                    }
                }
            }
            unsigned keep = 0;
            if (m == 0) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const size_t o = o0 + 16 * s + 4 * g + j;
                    const bool fused = best[j] > t;                   // keep = 1[s^ <= t]
                    fuse_map[o] = fused ? arg[j] : -1;
                    if (best_sim) best_sim[o] = best[j];
                    if (best_idx) best_idx[o] = arg[j];
                    if (!fused) keep |= 1u << (4 * g + j);
                }
            }
            keep |= __shfl_xor(keep, 16, 64);
            keep |= __shfl_xor(keep, 32, 64);
            if (lane == 0) keep16[o0 / 16 + s] = (uint16_t)keep;
        }
    }
}

template <int CT, int RAD>
hipError_t launch_shape(const ttf_params& p, const void* x, const Workspace& w, const int32_t* anchor_index,
                        int32_t* fuse_map, float* best_sim, int32_t* best_idx, hipStream_t s)
{
    const int N = p.H * p.W;
    const unsigned grid = (unsigned)((size_t)p.B * p.F * (N / 32));
    const int ksw_total = p.C / (kWaves * 32);               // K-steps per wave
    const uint16_t* xs = static_cast<const uint16_t*>(x);
    uint16_t* keep16 = reinterpret_cast<uint16_t*>(w.keep_bits);
#define TTF_LAUNCH(KSW)                                                                                   \
    k_search_mfma<CT, RAD, KSW, Shape<CT, RAD>::PF><<<grid, kWaves * 64, 0, s>>>(xs, anchor_index, w.anchor_inv, fuse_map,    \
                                                             best_sim, best_idx, keep16, p.F, p.H, p.C,   \
                                                             p.t, ksw_total / KSW)
    constexpr int MAXK = Shape<CT, RAD>::MAXK;
    if (MAXK >= 16 && ksw_total % 16 == 0) TTF_LAUNCH(16);
    else if (MAXK >= 8 && ksw_total % 8 == 0) TTF_LAUNCH(8);
    else if (ksw_total % 4 == 0) TTF_LAUNCH(4);
    else if (ksw_total % 2 == 0) TTF_LAUNCH(2);
    else TTF_LAUNCH(1);
#undef TTF_LAUNCH
    return hipGetLastError();
}

}  // namespace

// True when the matrix-core kernel covers this problem: bf16, grid width 16 (even height) or 32,
// radius <= 2, channel count a multiple of 256 (8 wave slices of whole 32-channel K-steps), and a
// token count per frame that is a multiple of 64 so keep words are whole.
bool mfma_search_supported(const ttf_params& p)
{
    if (p.dtype != TTF_BF16 || p.r > 2 || p.C % 256 != 0) return false;
    if (p.W == 16) return p.H % 4 == 0;
    if (p.W == 32) return p.H % 2 == 0;
    return false;
}

hipError_t launch_window_search_mfma(const ttf_params& p, const void* x, const Workspace& w,
                                     const int32_t* anchor_index, int32_t* fuse_map, float* best_sim,
                                     int32_t* best_idx, hipStream_t s)
{
#define TTF_CASE(CT, RAD) \
    if (p.W == 16 * CT && p.r == RAD) return launch_shape<CT, RAD>(p, x, w, anchor_index, fuse_map, best_sim, best_idx, s)
    TTF_CASE(1, 0);
    TTF_CASE(1, 1);
    TTF_CASE(1, 2);
    TTF_CASE(2, 0);
    TTF_CASE(2, 1);
    TTF_CASE(2, 2);
#undef TTF_CASE
    return hipErrorInvalidValue;
}

}  // namespace ttf
