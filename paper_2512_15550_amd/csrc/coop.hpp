// Pieces shared by the kernels whose blocks cooperate within one launch (the single-launch decode
// step, and the selection + attention stage of the staged step): accesses that are coherent across
// the chip without a fence, ordered compaction, and the attention of one block over a list of picks.
//
// Coherence rule: a word that another block reads within the same launch is written with an
// agent-scope atomic store or read-modify-write (written through to memory) and read with an
// agent-scope atomic load (never served from a stale cache line).  Measured on this part: such a
// store followed by a wait costs 0.36 us, such a load 0.21 us, both about what plain accesses cost;
// a release fence at agent scope (write-back of the whole L2) costs 1.3 us and more.
#pragma once
#include "arith.hpp"
#include "common.hpp"

namespace ctkvr {

// ---- coherent accesses (see the header comment) -------------------------------------------------
template <typename V> __device__ __forceinline__ V ldc(const V *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
template <typename V> __device__ __forceinline__ void stc(V *p, V v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Gives every thread whose `pred` holds its place, in thread order, behind `base` earlier entries, and
// returns the new fill level to every thread: no atomic decides an order, so the result is the same in
// every run.  All threads of the block call it.  s_cnt: NT / 64 words.
template <int NT> __device__ __forceinline__ int block_ordered_slot(bool pred, int base, uint32_t *s_cnt, int &slot)
{
    const int wv = threadIdx.x >> 6, ln = threadIdx.x & 63;
    const uint64_t m = __ballot(pred);
    if (ln == 0) s_cnt[wv] = (uint32_t)__popcll(m);
    __syncthreads();
    uint32_t before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) {
        const uint32_t c = s_cnt[w];
        before += w < wv ? c : 0u;
        tot += c;
    }
    slot = base + (int)before + __popcll(m & ((1ull << ln) - 1ull));
    __syncthreads();
    return base + (int)tot;
}

// Attention of one block over n picks (staging positions of the unit, in s_pick): per head the
// maximum logit (returned in mx[], the same in every thread), and per wave w its partial sums
// relative to that maximum, left in shared memory: s_red[(w * G + hh) * 129 + dim] = sum over the
// wave's picks of exp(z - mx) v[dim], and at dim = 128 the sum of exp(z - mx); attend_sum() adds
// the waves up.  One pick per 16-lane group at a time, four in flight; z and the row numbers are
// read coherently (they may be another block's).  s_red: (NT / 64) * G * 129 words.  Barriers
// inside; the caller places one before s_red is written again.
template <typename T, int G, int NT>
__device__ __forceinline__ void attend_picks(int n, const int32_t *s_pick, const float *zb, const uint32_t *rb, const T *V,
                                             float *s_red, float (&mx)[G])
{
    const int tid = threadIdx.x, wv = tid >> 6, ln = tid & 63, lane16 = tid & 15, grp = tid >> 4;
    const int myh = lane16 & (G - 1);
    constexpr int NG = NT / 16;   // 16-lane groups
    // pass A: maxima per head
#pragma unroll
    for (int hh = 0; hh < G; ++hh) mx[hh] = -__builtin_huge_valf();
    for (int t = tid; t < n; t += NT) {
        const int i = s_pick[t];
#pragma unroll
        for (int hh = 0; hh < G; ++hh) mx[hh] = fmaxf(mx[hh], ldc(zb + (size_t)i * G + hh));
    }
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        float v = mx[hh];
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
        if (ln == 0) s_red[wv * G + hh] = v;
    }
    __syncthreads();
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        float v = s_red[hh];
#pragma unroll
        for (int w = 1; w < NT / 64; ++w) v = fmaxf(v, s_red[w * G + hh]);
        mx[hh] = v;
    }
    __syncthreads();
    // pass B: weighted value rows
    float acc[G][8], lsum = 0.0f;   // lsum: lane l < G of a group carries head l's share of the denominators
#pragma unroll
    for (int hh = 0; hh < G; ++hh)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[hh][e] = 0.0f;
    for (int t0 = 0; t0 < n; t0 += NG * 4) {
        int pi[4];
        uint32_t row[4];
        float zme[4];
        Chunk<T> cv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) pi[u] = s_pick[min(t0 + u * NG + grp, n - 1)];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            row[u] = ldc(rb + pi[u]);
            zme[u] = ldc(zb + (size_t)pi[u] * G + myh);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) cv[u] = load_chunk(V + (size_t)row[u] * kD, lane16);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (t0 + u * NG + wv * 4 >= n) continue;   // nothing for this wave (uniform)
            const bool live = t0 + u * NG + grp < n;
            float vx[8];
            unpack(cv[u], vx);
            // lane (l mod G) of the group holds head l's logit: exp once per head, then handed round
            float pme = live ? __expf(zme[u] - mx[myh]) : 0.0f;
            if (lane16 < G) lsum += pme;
#pragma unroll
            for (int hh = 0; hh < G; ++hh) {
                const float p = __shfl(pme, (ln & 48) | hh);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[hh][e] = __fmaf_rn(p, vx[e], acc[hh][e]);
            }
        }
    }
    // the four groups of a wave; the waves are added up by attend_sum
#pragma unroll
    for (int hh = 0; hh < G; ++hh)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = acc[hh][e];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            acc[hh][e] = v;
        }
    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);
    if (ln < 16) {
#pragma unroll
        for (int hh = 0; hh < G; ++hh)
#pragma unroll
            for (int e = 0; e < 8; ++e) s_red[(wv * G + hh) * (kD + 1) + lane16 * 8 + e] = acc[hh][e];
        if (lane16 < G) s_red[(wv * G + lane16) * (kD + 1) + kD] = lsum;
    }
    __syncthreads();
}

// element `dim` (128: the denominator) of head hh after attend_picks: the waves' partial sums added in order
template <int G, int NT> __device__ __forceinline__ float attend_sum(const float *s_red, int hh, int dim)
{
    float v = 0.0f;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) v += s_red[(w * G + hh) * (kD + 1) + dim];
    return v;
}

template <int G> __device__ __forceinline__ float pick_head(const float (&v)[G], int hh)
{
    float r = v[0];
#pragma unroll
    for (int c = 1; c < G; ++c) r = hh == c ? v[c] : r;
    return r;
}

}  // namespace ctkvr
