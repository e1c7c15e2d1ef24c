// Small pieces shared by the staged kernels and the single-launch kernel: the paged KV cache's
// addressing, access to the G logits of a recalled key, and a few sizes.
#pragma once
#include "arith.hpp"

namespace ctkvr {

constexpr int kWinSplit = 8;   // blocks per unit of the resident window's attention (window_attn_kernel)

struct Paged {
    const void *pages;            // [num_pages][g][page][128]
    const int32_t *block_table;   // [batch][max_pages]
    int max_pages, page_shift;
};

// physical row (in units of 128 elements) of token t of sequence b, KV head kv
__device__ __forceinline__ uint32_t row_of(const int32_t *block_table, int max_pages, int page_shift, int g, int b,
                                           int kv, int t)
{
    int page = block_table[(size_t)b * max_pages + (t >> page_shift)];
    return (uint32_t)((page * g + kv) << page_shift) + (uint32_t)(t & ((1 << page_shift) - 1));
}

constexpr int kSelLds = 2048 + 64;   // words block_select_topk needs

// the G scores of candidate i (rows of G floats, 4G-byte aligned)
template <int G> __device__ __forceinline__ void load_z(const float *zb, int i, float (&v)[G])
{
    if constexpr (G == 1) {
        v[0] = zb[i];
    } else if constexpr (G == 2) {
        float2 t = reinterpret_cast<const float2 *>(zb)[i];
        v[0] = t.x; v[1] = t.y;
    } else {
#pragma unroll
        for (int c = 0; c < G / 4; ++c) {
            float4 t = reinterpret_cast<const float4 *>(zb)[(size_t)i * (G / 4) + c];
            v[4 * c] = t.x; v[4 * c + 1] = t.y; v[4 * c + 2] = t.z; v[4 * c + 3] = t.w;
        }
    }
}
template <int G> __device__ __forceinline__ void store_z(float *zb, int i, const float (&v)[G])
{
    if constexpr (G == 1) {
        zb[i] = v[0];
    } else if constexpr (G == 2) {
        reinterpret_cast<float2 *>(zb)[i] = make_float2(v[0], v[1]);
    } else {
#pragma unroll
        for (int c = 0; c < G / 4; ++c)
            reinterpret_cast<float4 *>(zb)[(size_t)i * (G / 4) + c] = make_float4(v[4 * c], v[4 * c + 1], v[4 * c + 2], v[4 * c + 3]);
    }
}

}  // namespace ctkvr
