// Device-side helpers shared by the TTF kernels: element widening, vector row loads and
// fixed-order wavefront reductions (64 lanes).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ttf {

struct bf16_t { uint16_t bits; };

// 16-byte accesses marked non-temporal: token rows are streamed (each byte is used once per pass),
// so they should not displace the anchor data and small arrays that are re-read from cache.
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
__device__ __forceinline__ uint4 load16_stream(const void* p)
{
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return uint4{v[0], v[1], v[2], v[3]};
}
__device__ __forceinline__ void store16_stream(void* p, uint4 v)
{
    __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4*>(p));
}

__device__ __forceinline__ float widen(bf16_t v)
{
    return __builtin_bit_cast(float, static_cast<uint32_t>(v.bits) << 16);
}
__device__ __forceinline__ float widen(float v) { return v; }

// V consecutive elements of a row, widened to fp32.  V*sizeof(T) is 16 (vector path, needs a
// 16-byte aligned address) or sizeof(T) (scalar path, any C).
template <typename T, int V>
struct RowVec {
    float v[V];
    template <bool STREAM = false>
    __device__ __forceinline__ void load(const T* p)
    {
        if constexpr (V == 1) {
            v[0] = widen(p[0]);
        } else if constexpr (sizeof(T) == 2) {
            static_assert(V == 8, "bf16 vector path is 8 elements");
            const uint4 q = STREAM ? load16_stream(p) : *reinterpret_cast<const uint4*>(p);
            const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[2 * i]     = __builtin_bit_cast(float, w[i] << 16);
                v[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xffff0000u);
            }
        } else {
            static_assert(V == 4, "fp32 vector path is 4 elements");
            const uint4 u = STREAM ? load16_stream(p) : *reinterpret_cast<const uint4*>(p);
            const float4 q = __builtin_bit_cast(float4, u);
            v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
        }
    }
};

// Bit-exact copy of one token row by one wavefront.  U = bytes moved per lane per step: 16 (row
// bytes % 16 == 0, both addresses 16-byte aligned), 4 or 2.
template <int U, bool STREAM = true>
__device__ __forceinline__ void copy_row(const char* __restrict__ src, char* __restrict__ dst,
                                         size_t row_bytes, int lane)
{
    if constexpr (U == 16) {
        // STREAM: the source row is read once (no reason to keep it in cache); otherwise plain loads
        auto ld = [](const uint4* p) { return STREAM ? load16_stream(p) : *p; };
        const uint4* s = reinterpret_cast<const uint4*>(src);
        uint4* d = reinterpret_cast<uint4*>(dst);
        const int n = (int)(row_bytes / 16);
        int q = lane;
        for (; q + 448 < n; q += 512) {                // eight 16-byte pieces in flight per lane
            uint4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = ld(s + q + 64 * u);
#pragma unroll
            for (int u = 0; u < 8; ++u) store16_stream(d + q + 64 * u, v[u]);
        }
        for (; q + 192 < n; q += 256) {
            const uint4 v0 = ld(s + q), v1 = ld(s + q + 64),
                        v2 = ld(s + q + 128), v3 = ld(s + q + 192);
            store16_stream(d + q, v0); store16_stream(d + q + 64, v1);
            store16_stream(d + q + 128, v2); store16_stream(d + q + 192, v3);
        }
        for (; q < n; q += 64) store16_stream(d + q, ld(s + q));
    } else if constexpr (U == 4) {
        const uint32_t* s = reinterpret_cast<const uint32_t*>(src);
        uint32_t* d = reinterpret_cast<uint32_t*>(dst);
        const int n = (int)(row_bytes / 4);
        for (int q = lane; q < n; q += 64) d[q] = s[q];
    } else {
        const uint16_t* s = reinterpret_cast<const uint16_t*>(src);
        uint16_t* d = reinterpret_cast<uint16_t*>(dst);
        const int n = (int)(row_bytes / 2);
        for (int q = lane; q < n; q += 64) d[q] = s[q];
    }
}

// Sum over the 64 lanes of a wavefront, butterfly order (identical on every call); every
// lane ends with the total.
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1)
        v += __shfl_xor(v, m, 64);
    return v;
}
// The lane each DPP control pairs a lane with inside its row of 16: i^1, i^2, mirror in the half
// row (i <-> 7-i), mirror in the row (i <-> 15-i).  Four such steps leave every lane of a row with
// the row's total; they run at VALU rate, unlike ds_bpermute.
template <int DPP_CTRL>
__device__ __forceinline__ double dpp_partner(double v)
{
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)u, DPP_CTRL, 0xf, 0xf, false);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(u >> 32), DPP_CTRL, 0xf, 0xf, false);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ double wave_sum(double v)
{
    v += dpp_partner<0xB1>(v);
    v += dpp_partner<0x4E>(v);
    v += dpp_partner<0x141>(v);
    v += dpp_partner<0x140>(v);
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    return v;
}

}  // namespace ttf
