// k-means centroid mode of the index build (replaces Algorithm 1 line 1 only; the
// paper itself takes the last C prompt queries).  Per (sequence, KV head) the s
// prompt positions are clustered; a point is the concatenation of the G query-head
// vectors of the group at one position (G*128 numbers, contiguous in q_prefill).
// Lloyd iteration = half-norms -> assignment on the matrix cores (which also counts the
// members of every centre) -> counting sort of the positions by centre -> one block per
// centre sums its members in fixed point and writes the new centre.  The centres live in the index's centroid table
// [b][h][c_max][128] all along: head hh of centre c is one 128-element row.
#pragma once
#include "kernels.hpp"

namespace ctkvr {

struct KmeansArgs {
    int g, h, c_max, s_max;
    const int32_t *n_cent, *ctx_lens;
    const int32_t *first_row;      // [batch] row of position 0 of each sequence in q_prefill
    const bf16_t *q;               // [rows][h][128]
    bf16_t *centroids;             // [batch][h][c_max][128]
    const int32_t *init_pos;       // [batch][g][c_max]
    float *half_norm;              // [batch*g][c_max]
    int32_t *assign;               // [batch*g][s_max]
    uint32_t *counts;              // [batch*g][c_max] members per centre (zero before the assignment)
    uint32_t *start;               // [batch*g][c_max] first slot of each centre in `order`
    uint32_t *cursor;              // [batch*g][c_max] next free slot while scattering
    int32_t *order;                // [batch*g][s_max] positions grouped by centre
};

// centres start as the prompt queries at init_pos; grid (c_max, h, batch), 128 threads
__global__ void kmeans_init_kernel(KmeansArgs a, int G)
{
    const int j = blockIdx.x, hd = blockIdx.y, b = blockIdx.z;
    if (j >= a.n_cent[b]) return;
    const int kv = hd / G;
    int pos = a.init_pos[((size_t)b * a.g + kv) * a.c_max + j];
    pos = max(0, min(pos, a.ctx_lens[b] - 1));
    const bf16_t *src = a.q + ((size_t)(a.first_row[b] + pos) * a.h + hd) * kD;
    a.centroids[(((size_t)b * a.h + hd) * a.c_max + j) * kD + threadIdx.x] = src[threadIdx.x];
}

// half_norm[c] = |mu_c|^2 / 2 (heads summed in order); grid (ceil(c_max/16), batch*g), 256 threads
template <int G> __global__ __launch_bounds__(256) void kmeans_halfnorm_kernel(KmeansArgs a)
{
    const int ul = blockIdx.y, b = ul / a.g, kv = ul - b * a.g;
    const int C = a.n_cent[b];
    const int lane16 = threadIdx.x & 15, grp = threadIdx.x >> 4;
    const int c = blockIdx.x * 16 + grp;
    if (blockIdx.x * 16 >= C) return;
    const int cc = c < C ? c : C - 1;
    float n2 = 0.0f;
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        float x[8];
        unpack(load_chunk(a.centroids + (((size_t)b * a.h + kv * G + hh) * a.c_max + cc) * kD, lane16), x);
        n2 = n2 + group16_sum(lane_partial(x, x));
    }
    if (c < C && lane16 == 0) a.half_norm[(size_t)ul * a.c_max + c] = 0.5f * n2;
}

// assignment: argmax_c (x . mu_c - |mu_c|^2/2), ties to the lowest c.  A = 32 centres x 16 dims,
// B = 16 dims x 32 points per v_mfma_f32_32x32x16_bf16.  A block owns 256 points, a wave 32 of
// them with their B fragments resident in registers (G <= 4); the centres are walked 128 at a
// time, and each 128-centre x 64-dim piece of the centre table goes through shared memory once
// for the eight waves (double-buffered, requested two pieces ahead; rows padded to 144 bytes so that the 16-byte fragment reads of a
// wave spread over the banks).  With G = 8 the fragments do not fit the registers and are
// re-read from memory.  Counts the members of every centre as it goes.
// grid (ceil(s_max/256), batch*g), 512 threads; dynamic shared memory: c_max rounded up to 128, floats.
// The accumulators start from -|mu_c|^2/2, so the result tile is the score itself.
template <int G> __global__ __launch_bounds__(512) void kmeans_assign_kernel(KmeansArgs a)
{
    extern __shared__ __align__(16) float s_hn[];   // c_max rounded up to 128 floats
    constexpr int KS = 8 * G;                 // k-steps of 16 dims
    constexpr bool REG_B = (G <= 4);
    constexpr int ROWB = 144;                 // bytes per staged centre row (64 dims + padding)
    __shared__ __align__(16) unsigned char s_a[2][128 * ROWB];
    const int ul = blockIdx.y, b = ul / a.g, kv = ul - b * a.g;
    const int C = a.n_cent[b], s = a.ctx_lens[b];
    if ((int)blockIdx.x * 256 >= s) return;
    const int tid = threadIdx.x, wv = tid >> 6, ln = tid & 63, col = ln & 31, half = ln >> 5;
    // -|mu_c|^2 / 2, the value every accumulator starts from; -inf for the padding up to a whole tile
    for (int c = tid; c < ((C + 127) & ~127); c += 512)
        s_hn[c] = c < C ? -a.half_norm[(size_t)ul * a.c_max + c] : -__builtin_huge_valf();
    const int p0 = blockIdx.x * 256 + wv * 32;
    const int t = min(p0 + col, s - 1);
    const bf16_t *xrow = a.q + ((size_t)(a.first_row[b] + t) * a.h + kv * G) * kD + 8 * half;
    bf16x8_t bfrag[REG_B ? KS : 1];
    if constexpr (REG_B) {
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) bfrag[kk] = *reinterpret_cast<const bf16x8_t *>(xrow + kk * 16);
    }
    // staging: thread t moves a quarter row (32 bytes) of piece (c0, kc): centre c0 + t/4, head kc/2,
    // dims 64*(kc%2) + 16*(t%4) ..
    constexpr int NKC = 2 * G;                // 64-dim pieces per 128-centre tile
    static_assert(NKC % 2 == 0, "piece parity must carry over from one centre tile to the next");
    const int srow = tid >> 2, sq = tid & 3;
    const bf16_t *cbase = a.centroids + ((size_t)b * a.h + kv * G) * a.c_max * kD;
    // two pieces ahead in registers: piece i+2 is requested while piece i feeds the matrix cores
    // and piece i+1 waits to be written to the other buffer
    // (named variables: an array indexed through the helpers would be kept in private memory)
    uint4 st0a, st0b, st1a, st1b;
    auto fetch = [&](uint4 &x, uint4 &y, int c0, int kc) {
        const int c = min(c0 + srow, C - 1);
        const uint4 *src = reinterpret_cast<const uint4 *>(cbase + ((size_t)(kc >> 1) * a.c_max + c) * kD + (kc & 1) * 64 + sq * 16);
        x = src[0];
        y = src[1];
    };
    auto put = [&](const uint4 &x, const uint4 &y, int buf) {
        uint4 *dst = reinterpret_cast<uint4 *>(&s_a[buf][srow * ROWB + sq * 32]);
        dst[0] = x;
        dst[1] = y;
    };
    float best = -__builtin_huge_valf();
    int bi = 0;
    fetch(st0a, st0b, 0, 0);
    fetch(st1a, st1b, 0, 1);
    put(st0a, st0b, 0);
    __syncthreads();
    for (int c0 = 0; c0 < C; c0 += 128) {
        f32x16_t acc[4];
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const float4 v = *reinterpret_cast<const float4 *>(&s_hn[c0 + ct * 32 + 8 * rq + 4 * half]);
                acc[ct][4 * rq + 0] = v.x;
                acc[ct][4 * rq + 1] = v.y;
                acc[ct][4 * rq + 2] = v.z;
                acc[ct][4 * rq + 3] = v.w;
            }
#pragma unroll
        for (int kc = 0; kc < NKC; ++kc) {
            const int buf = kc & 1;
            {   // piece i + 2
                const int c2 = kc + 2 < NKC ? c0 : c0 + 128, k2 = kc + 2 < NKC ? kc + 2 : kc + 2 - NKC;
                if (c2 < C) {
                    if ((kc & 1) == 0) fetch(st0a, st0b, c2, k2);
                    else fetch(st1a, st1b, c2, k2);
                }
            }
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                bf16x8_t bf;
                if constexpr (REG_B) bf = bfrag[kc * 4 + ks];
                else bf = *reinterpret_cast<const bf16x8_t *>(xrow + (kc * 4 + ks) * 16);
#pragma unroll
                for (int ct = 0; ct < 4; ++ct) {
                    bf16x8_t af = *reinterpret_cast<const bf16x8_t *>(&s_a[buf][(ct * 32 + col) * ROWB + ks * 32 + half * 16]);
                    acc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bf, acc[ct], 0, 0, 0);
                }
            }
            if (kc + 1 < NKC || c0 + 128 < C) {   // piece i + 1
                if (((kc + 1) & 1) == 0) put(st0a, st0b, buf ^ 1);
                else put(st1a, st1b, buf ^ 1);
            }
            __syncthreads();
        }
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int c = c0 + ct * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                if (acc[ct][r] > best) { best = acc[ct][r]; bi = c; }
            }
    }
    float ob = __shfl_xor(best, 32);
    int oi = __shfl_xor(bi, 32);
    if (ob > best || (ob == best && oi < bi)) bi = oi;
    if (half == 0 && (p0 + col) < s) {
        a.assign[(size_t)ul * a.s_max + p0 + col] = bi;
        atomicAdd(&a.counts[(size_t)ul * a.c_max + bi], 1u);
    }
}

// start[c] = number of positions assigned to centres below c; cursor[c] = start[c].
// grid batch*g, 1024 threads (C <= 8192: eight centres per thread)
__global__ __launch_bounds__(1024) void kmeans_offsets_kernel(KmeansArgs a)
{
    __shared__ uint32_t s_tmp[32];
    const int ul = blockIdx.x, b = ul / a.g;
    const int C = a.n_cent[b], tid = threadIdx.x;
    uint32_t c[8], mine = 0;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        int j = tid * 8 + q;
        c[q] = j < C ? a.counts[(size_t)ul * a.c_max + j] : 0u;
        mine += c[q];
    }
    uint32_t tot;
    uint32_t before = block_excl_scan<1024>(mine, s_tmp, &tot);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        int j = tid * 8 + q;
        if (j < C) {
            a.start[(size_t)ul * a.c_max + j] = before;
            a.cursor[(size_t)ul * a.c_max + j] = before;
        }
        before += c[q];
    }
}

// order[cursor[assign[t]]++] = t.  The order inside a centre's range is whatever the atomics give:
// the sums taken over it are integer sums.  grid (ceil(s_max/256), batch*g), 256 threads
__global__ __launch_bounds__(256) void kmeans_scatter_kernel(KmeansArgs a)
{
    const int ul = blockIdx.y, b = ul / a.g;
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= a.ctx_lens[b]) return;
    const int c = a.assign[(size_t)ul * a.s_max + t];
    const uint32_t pos = atomicAdd(&a.cursor[(size_t)ul * a.c_max + c], 1u);
    a.order[(size_t)ul * a.s_max + pos] = t;
}

// One block per centre: sum_c = sum of llrint(x * 2^20) over its members (int64 per element, in
// registers), mu_c = sum / count (fp64 divide, rounded to fp32, then to bf16 nearest-even); an
// empty centre keeps its place.  Four groups of 128 threads take the members eight at a time in
// turn (their ids are requested one round ahead of their rows); thread e of a group owns the G
// consecutive elements e*G .. e*G+G-1 of the G*128-element point, and the groups' integer sums
// are added through shared memory.  Clears the count for the next iteration.
// grid (c_max, batch*g), 512 threads
template <int G> __global__ __launch_bounds__(512) void kmeans_reduce_kernel(KmeansArgs a)
{
    __shared__ long long s_part[3][128][G];
    const int ul = blockIdx.y, b = ul / a.g, kv = ul - b * a.g;
    const int c = blockIdx.x;
    if (c >= a.n_cent[b]) return;
    const uint32_t n = a.counts[(size_t)ul * a.c_max + c];
    const uint32_t st = a.start[(size_t)ul * a.c_max + c];
    const int32_t *ord = a.order + (size_t)ul * a.s_max + st;
    const int e = threadIdx.x & 127, grp = threadIdx.x >> 7;
    const bf16_t *base = a.q + ((size_t)a.first_row[b] * a.h + kv * G) * kD + e * G;
    const size_t rstride = (size_t)a.h * kD;
    long long acc[G];
#pragma unroll
    for (int r = 0; r < G; ++r) acc[r] = 0;
    int t[8];
    if (n) {
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = ord[min((uint32_t)(grp * 8 + u), n - 1)];
    }
    for (uint32_t m0 = grp * 8; m0 < n; m0 += 32) {
        int tn[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) tn[u] = ord[min(m0 + 32 + u, n - 1)];
        bf16_t x[8][G];
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int r = 0; r < G; ++r) x[u][r] = base[(size_t)t[u] * rstride + r];
        // x * 2^20 is exact in fp32 (a bf16 value, an exponent shift); below 2^30 it converts with
        // the one-instruction fp32 -> int32 rounding, and the wave checks that together
        bool small = true;
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int r = 0; r < G; ++r) small = small && ((uint32_t)x[u][r] & 0x7fffu) < 0x4480u;   // |x| < 1024
        if (__all(small)) {
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (m0 + u < n) {
#pragma unroll
                    for (int r = 0; r < G; ++r)
                        acc[r] += (long long)__float2int_rn(__uint_as_float((uint32_t)x[u][r] << 16) * 1048576.0f);
                }
        } else {
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (m0 + u < n) {
#pragma unroll
                    for (int r = 0; r < G; ++r)
                        acc[r] += __float2ll_rn(__uint_as_float((uint32_t)x[u][r] << 16) * 1048576.0f);
                }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = tn[u];
    }
    if (grp) {
#pragma unroll
        for (int r = 0; r < G; ++r) s_part[grp - 1][e][r] = acc[r];
    }
    __syncthreads();
    if (grp == 0 && n) {
#pragma unroll
        for (int r = 0; r < G; ++r) {
            const long long tot = acc[r] + s_part[0][e][r] + s_part[1][e][r] + s_part[2][e][r];
            const int ee = e * G + r, hh = ee >> 7, dim = ee & 127;
            float m = (float)((double)tot * (1.0 / 1048576.0) / (double)n);
            uint32_t u = __float_as_uint(m);
            u += 0x7fffu + ((u >> 16) & 1u);
            a.centroids[(((size_t)b * a.h + kv * G + hh) * a.c_max + c) * kD + dim] = (bf16_t)(u >> 16);
        }
    }
    if (threadIdx.x == 0) a.counts[(size_t)ul * a.c_max + c] = 0u;
}

}  // namespace ctkvr
