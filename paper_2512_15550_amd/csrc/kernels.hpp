// gfx950 kernels of the CTkvr path.  Decode (Algorithm 2): centroid_cos ->
// recall (probe select + list gather/dedup) -> score -> denom -> rerank_select ->
// sparse_attn -> attn_merge.  The exact index build (Algorithm 1 lines 2-4) runs
// score -> denom -> rerank_select with "the recalled set" = all s keys and the
// centroid in the role of the query, which is literally the same formula.
#pragma once
#include "arith.hpp"

namespace ctkvr {

// A "unit" is what one selection is made for: in a decode step a (sequence, KV
// head) pair; in the build a (sequence, KV head, centroid) triple.
struct Units {
    int g, G, h;
    int build;               // 0: unit = b*g + kv            1: unit = unit0 + local = (b*g + kv)*c_max + j
    int unit0, c_max;
    const int32_t *n_cent;   // [batch] centroids per sequence
};

__device__ __forceinline__ bool decode_unit(const Units &u, int local, int &b, int &kv, int &j)
{
    if (!u.build) {
        b = local / u.g;
        kv = local - b * u.g;
        j = 0;
        return true;
    }
    int id = u.unit0 + local;
    int bk = id / u.c_max;
    j = id - bk * u.c_max;
    b = bk / u.g;
    kv = bk - b * u.g;
    return j < u.n_cent[b];
}

struct Paged {
    const void *pages;            // [num_pages][g][page][128]
    const int32_t *block_table;   // [batch][max_pages]
    int max_pages, page_shift;
};

__device__ __forceinline__ uint32_t row_of(const Paged &pg, int g, int b, int kv, int t)
{
    int page = pg.block_table[(size_t)b * pg.max_pages + (t >> pg.page_shift)];
    return (uint32_t)((page * g + kv) << pg.page_shift) + (uint32_t)(t & ((1 << pg.page_shift) - 1));
}

// ------------------------------------------------------------------------------
// small utilities
// ------------------------------------------------------------------------------
__global__ void fill_u32_kernel(uint32_t *p, uint32_t v, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// Algorithm 1 line 1: centroid j of sequence b, head hd = prompt query at position s_b - C_b + j.
// q_prefill rows [row0_b + off_b + j][h][128] -> centroids [b][h][c_max][128]
template <typename T>
__global__ void copy_centroids_kernel(const T *q_prefill, const int32_t *first_row /*[batch]*/, const int32_t *n_cent,
                                      int h, int c_max, T *centroids)
{
    int j = blockIdx.x, hd = blockIdx.y, b = blockIdx.z;
    if (j >= n_cent[b]) return;
    const T *src = q_prefill + ((size_t)(first_row[b] + j) * h + hd) * kD;
    T *dst = centroids + (((size_t)b * h + hd) * c_max + j) * kD;
    dst[threadIdx.x] = src[threadIdx.x];
}

// inverse norms of n rows of 128
template <typename T> __global__ __launch_bounds__(256) void inv_norm_kernel(const T *rows, size_t n, float *out)
{
    size_t r = (size_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    int lane16 = threadIdx.x & 15;
    size_t rr = r < n ? r : n - 1;
    float x[8];
    unpack(load_chunk(rows + rr * kD, lane16), x);
    float n2 = group16_sum(lane_partial(x, x));
    if (r < n && lane16 == 0) out[r] = inv_norm_from_sq(n2);
}

// ------------------------------------------------------------------------------
// Algorithm 2 lines 1-2: Cos_kv[b][kv][j] = max over the group of cos(q_h, c_{h,j})
// grid (ceil(c_max/64), batch*g), 256 threads; also clears the step's accumulators.
// ------------------------------------------------------------------------------
struct CosArgs {
    const void *q;            // [batch][h][128]
    const void *centroids;    // [batch][h][c_max][128]
    const float *inv_norm_c;  // [batch][h][c_max]
    const int32_t *n_cent;
    float *cos;               // [batch*g][c_max]
    uint32_t *m_key;          // [batch*g][G]  cleared here
    unsigned long long *S;    // [batch*g][G]  cleared here
    int g, h, c_max;
};

template <typename T, int G> __global__ __launch_bounds__(256) void centroid_cos_kernel(CosArgs a)
{
    const int ul = blockIdx.y;
    const int b = ul / a.g, kv = ul - b * a.g;
    const int C = a.n_cent[b];
    const int tid = threadIdx.x, lane16 = tid & 15, grp = tid >> 4;
    if (blockIdx.x == 0 && tid < G) {
        a.m_key[ul * G + tid] = 0u;
        a.S[ul * G + tid] = 0ull;
    }
    const int tile0 = blockIdx.x * 64;
    if (tile0 >= C) return;
    const T *qb = (const T *)a.q + ((size_t)b * a.h + kv * G) * kD;
    float q[G][8], inv_q[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        unpack(load_chunk(qb + (size_t)hh * kD, lane16), q[hh]);
        inv_q[hh] = inv_norm_from_sq(group16_sum(lane_partial(q[hh], q[hh])));
    }
    const T *cb = (const T *)a.centroids;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        int j = tile0 + r * 16 + grp;
        int jj = j < C ? j : C - 1;
        float best = -__builtin_huge_valf();
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            size_t row = ((size_t)b * a.h + kv * G + hh) * a.c_max + jj;
            float cx[8];
            unpack(load_chunk(cb + row * kD, lane16), cx);
            float dot = group16_sum(lane_partial(q[hh], cx));
            float cs = (dot * a.inv_norm_c[row]) * inv_q[hh];
            best = fmaxf(best, cs);
        }
        if (j < C && lane16 == 0) a.cos[(size_t)ul * a.c_max + j] = best;
    }
}

// ------------------------------------------------------------------------------
// Algorithm 2 lines 3-4: top-C' centroids, then the deduplicated union of their
// lists as an ascending id list.  One block of 1024 threads per (sequence, KV head);
// dynamic shared memory: select scratch (2048 + 32 words) + probe ids (n_probe) +
// bitmap (ceil(s_max/32) words).
// ------------------------------------------------------------------------------
struct RecallArgs {
    const float *cos;         // [batch*g][c_max]
    const int32_t *lists;     // [batch*g][c_max][rho]
    const int32_t *n_cent, *ctx_lens;
    int32_t *probe;           // [batch*g][n_probe]
    int32_t *cand;            // [batch*g][l_stride]
    int32_t *ncand;           // [batch*g]
    int32_t *out_probe, *out_ncand;   // optional copies for the caller
    int g, c_max, rho, n_probe, l_stride;
};

__global__ __launch_bounds__(1024) void recall_kernel(RecallArgs a)
{
    extern __shared__ uint32_t smem[];
    uint32_t *s_sel = smem;                      // 2048 + 32
    int32_t *s_probe = (int32_t *)(smem + 2080);
    uint32_t *s_bits = smem + 2080 + a.n_probe;
    const int ul = blockIdx.x, tid = threadIdx.x;
    const int b = ul / a.g;
    const int C = a.n_cent[b], s = a.ctx_lens[b];
    const float *cosv = a.cos + (size_t)ul * a.c_max;
    // line 3
    block_select_topk<1024>([&](int j) { return ordered_key(cosv[j]); }, C, a.n_probe,
                            [&](int pos, int j) {
                                s_probe[pos] = j;
                                a.probe[(size_t)ul * a.n_probe + pos] = j;
                                if (a.out_probe) a.out_probe[(size_t)ul * a.n_probe + pos] = j;
                            },
                            s_sel);
    const int W = (s + 31) >> 5;
    for (int w = tid; w < W; w += 1024) s_bits[w] = 0u;
    __syncthreads();
    // line 4: mark every key id of the probed lists
    const int32_t *lb = a.lists + (size_t)ul * a.c_max * a.rho;
    const int total = a.n_probe * a.rho;
    for (int idx = tid; idx < total; idx += 1024) {
        int p = idx / a.rho, r = idx - p * a.rho;
        int t = lb[(size_t)s_probe[p] * a.rho + r];
        atomicOr(&s_bits[t >> 5], 1u << (t & 31));
    }
    __syncthreads();
    // ordered expansion of the bitmap: thread t owns words [t*per, (t+1)*per)
    const int per = (W + 1023) >> 10;
    uint32_t cnt = 0;
    for (int q = 0; q < per; ++q) {
        int w = tid * per + q;
        if (w < W) cnt += __popc(s_bits[w]);
    }
    uint32_t tot;
    uint32_t at = block_excl_scan<1024>(cnt, s_sel, &tot);
    int32_t *out = a.cand + (size_t)ul * a.l_stride;
    for (int q = 0; q < per; ++q) {
        int w = tid * per + q;
        if (w < W) {
            uint32_t m = s_bits[w];
            while (m) {
                int bit = __ffs((int)m) - 1;
                m &= m - 1;
                out[at++] = (w << 5) + bit;
            }
        }
    }
    if (tid == 0) {
        a.ncand[ul] = (int32_t)tot;
        if (a.out_ncand) a.out_ncand[ul] = (int32_t)tot;
    }
}

// ------------------------------------------------------------------------------
// Algorithm 2 line 5 / Algorithm 1 line 2, first half: z[h][i] = (q_h . k_i) * scale
// for the G heads of the group over a tile of 256 ids, plus the running maximum
// per head.  grid (ceil(l_stride/256), units), 256 threads.
// ------------------------------------------------------------------------------
struct ScoreArgs {
    Units u;
    const void *q;            // decode: [batch][h][128] (qrows = 1); build: centroids [batch][h][c_max][128] (qrows = c_max)
    int qrows;
    Paged k;
    const int32_t *ctx_lens;
    const int32_t *cand;      // [units][l_stride] or nullptr = all ids 0..s-1
    const int32_t *ncand;     // [units] (with cand)
    int l_stride;
    float *z;                 // [units][l_stride][G]
    uint32_t *m_key;          // [units][G] ordered-key running max (atomicMax)
    float scale;
};

template <typename T, int G> __global__ __launch_bounds__(256) void score_kernel(ScoreArgs a)
{
    int b, kv, j;
    const int ul = blockIdx.y;
    if (!decode_unit(a.u, ul, b, kv, j)) return;
    const int L = a.cand ? a.ncand[ul] : a.ctx_lens[b];
    const int tile0 = blockIdx.x * 256;
    if (tile0 >= L) return;
    __shared__ uint32_t s_row[256];
    __shared__ uint32_t s_max[G];
    const int tid = threadIdx.x, lane16 = tid & 15, grp = tid >> 4;
    {
        int i = min(tile0 + tid, L - 1);
        int t = a.cand ? a.cand[(size_t)ul * a.l_stride + i] : i;
        s_row[tid] = row_of(a.k, a.u.g, b, kv, t);
    }
    if (tid < G) s_max[tid] = 0u;
    float q[G][8];
    const T *qb = (const T *)a.q + (((size_t)b * a.u.h + kv * G) * a.qrows + j) * kD;
#pragma unroll
    for (int hh = 0; hh < G; ++hh) unpack(load_chunk(qb + (size_t)hh * a.qrows * kD, lane16), q[hh]);
    __syncthreads();
    const T *K = (const T *)a.k.pages;
    float mx[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) mx[hh] = -__builtin_huge_valf();
    float *zb = a.z + (size_t)ul * a.l_stride * G;
#pragma unroll 4
    for (int r = 0; r < 16; ++r) {
        const int row = r * 16 + grp;
        float kx[8];
        unpack(load_chunk(K + (size_t)s_row[row] * kD, lane16), kx);
        float zz[G];
#pragma unroll
        for (int hh = 0; hh < G; ++hh) zz[hh] = group16_sum(lane_partial(q[hh], kx)) * a.scale;
        const int i = tile0 + row;
        if (i < L) {
            float mine = zz[0];
#pragma unroll
            for (int hh = 0; hh < G; ++hh) {
                mx[hh] = fmaxf(mx[hh], zz[hh]);
                if (lane16 == hh) mine = zz[hh];
            }
            if (lane16 < G) zb[(size_t)i * G + lane16] = mine;
        }
    }
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        float v = mx[hh];
        v = fmaxf(v, __shfl_xor(v, 16));
        v = fmaxf(v, __shfl_xor(v, 32));
        if (lane_id() == 0) atomicMax(&s_max[hh], ordered_key(v));
    }
    __syncthreads();
    if (tid < G) atomicMax(&a.m_key[ul * G + tid], s_max[tid]);
}

// ------------------------------------------------------------------------------
// softmax denominators: S[h] += sum_i floor(exp(z[h][i] - m[h]) * 2^40)
// grid (ceil(l_stride/1024), units), 256 threads.
// ------------------------------------------------------------------------------
struct DenomArgs {
    Units u;
    const int32_t *ctx_lens, *ncand;   // ncand == nullptr => L = ctx_len
    int l_stride;
    const float *z;
    const uint32_t *m_key;
    unsigned long long *S;
};

template <int G> __global__ __launch_bounds__(256) void denom_kernel(DenomArgs a)
{
    int b, kv, j;
    const int ul = blockIdx.y;
    if (!decode_unit(a.u, ul, b, kv, j)) return;
    const int L = a.ncand ? a.ncand[ul] : a.ctx_lens[b];
    const int tile0 = blockIdx.x * 1024;
    if (tile0 >= L) return;
    const int tid = threadIdx.x;
    __shared__ unsigned long long s_acc[4][G];
    float m[G];
    unsigned long long acc[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        m[hh] = ordered_value(a.m_key[ul * G + hh]);
        acc[hh] = 0ull;
    }
    const float *zb = a.z + (size_t)ul * a.l_stride * G;
    const int end = min(L, tile0 + 1024);
    for (int i = tile0 + tid; i < end; i += 256) {
#pragma unroll
        for (int hh = 0; hh < G; ++hh) acc[hh] += to_fixed40(exp_series(zb[(size_t)i * G + hh] - m[hh]));
    }
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        unsigned long long v = acc[hh];
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
        if (lane_id() == 0) s_acc[tid >> 6][hh] = v;
    }
    __syncthreads();
    if (tid < G) atomicAdd(&a.S[ul * G + tid], s_acc[0][tid] + s_acc[1][tid] + s_acc[2][tid] + s_acc[3][tid]);
}

// ------------------------------------------------------------------------------
// Algorithm 2 lines 5-6 / Algorithm 1 lines 3-4: key_i = max_h log softmax_h(i),
// top-k ids, ascending.  One block of 1024 threads per unit.
//   decode: sel[unit][pos] = cand[i], zsel[unit][pos][G] = z[i][G], nsel[unit]
//   build : lists[(b*g+kv)*c_max + j][pos] = i
// ------------------------------------------------------------------------------
struct SelectArgs {
    Units u;
    const int32_t *ctx_lens, *ncand, *cand;
    int l_stride, top_k;
    const float *z;
    const uint32_t *m_key;
    const unsigned long long *S;
    int32_t *sel;       // decode [units][top_k] ; build: lists base
    float *zsel;        // decode [units][top_k][G]
    int32_t *nsel;      // decode [units]
    int32_t *out_sel;   // optional copy for the caller
};

template <int G> __global__ __launch_bounds__(1024) void rerank_select_kernel(SelectArgs a)
{
    __shared__ uint32_t s_sel[2048 + 32];
    __shared__ float s_m[G], s_ls[G];
    int b, kv, j;
    const int ul = blockIdx.x, tid = threadIdx.x;
    if (!decode_unit(a.u, ul, b, kv, j)) return;
    const int L = a.cand ? a.ncand[ul] : a.ctx_lens[b];
    if (tid < G) {
        s_m[tid] = ordered_value(a.m_key[ul * G + tid]);
        s_ls[tid] = (float)log_fixed40(a.S[ul * G + tid]);
    }
    __syncthreads();
    float m[G], ls[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        m[hh] = s_m[hh];
        ls[hh] = s_ls[hh];
    }
    const float *zb = a.z + (size_t)ul * a.l_stride * G;
    auto key = [&](int i) {
        float best = -__builtin_huge_valf();
#pragma unroll
        for (int hh = 0; hh < G; ++hh) best = fmaxf(best, (zb[(size_t)i * G + hh] - m[hh]) - ls[hh]);
        return ordered_key(best);
    };
    if (a.u.build) {
        int32_t *dst = a.sel + (size_t)(a.u.unit0 + ul) * a.top_k;
        block_select_topk<1024>(key, L, a.top_k, [&](int pos, int i) { dst[pos] = i; }, s_sel);
        return;
    }
    const int32_t *cb = a.cand + (size_t)ul * a.l_stride;
    int32_t *dst = a.sel + (size_t)ul * a.top_k;
    int32_t *dst2 = a.out_sel ? a.out_sel + (size_t)ul * a.top_k : nullptr;
    float *zd = a.zsel + (size_t)ul * a.top_k * G;
    int n = block_select_topk<1024>(key, L, a.top_k,
                                    [&](int pos, int i) {
                                        int t = cb[i];
                                        dst[pos] = t;
                                        if (dst2) dst2[pos] = t;
#pragma unroll
                                        for (int hh = 0; hh < G; ++hh) zd[(size_t)pos * G + hh] = zb[(size_t)i * G + hh];
                                    },
                                    s_sel);
    for (int pos = n + tid; pos < a.top_k; pos += 1024) {
        dst[pos] = -1;
        if (dst2) dst2[pos] = -1;
    }
    if (tid == 0) a.nsel[ul] = n;
}

// ------------------------------------------------------------------------------
// Algorithm 2 lines 7-9: softmax(z_sel) . V_sel, split over chunks of 64 selected
// keys; grid (nsplit, batch*g), 256 threads.  Partials are merged by attn_merge.
// ------------------------------------------------------------------------------
struct AttnArgs {
    Paged v;
    int g, h, top_k, nsplit;
    const int32_t *sel, *nsel;
    const float *zsel;
    float *po;   // [batch*h][nsplit][128] un-normalised partial outputs
    float *pm;   // [batch*h][nsplit] partial maxima
    float *pl;   // [batch*h][nsplit] partial sums
    float *out;  // [batch*h][128]
    float *out_lse;
};

template <typename T, int G> __global__ __launch_bounds__(256) void sparse_attn_kernel(AttnArgs a)
{
    const int ul = blockIdx.y, split = blockIdx.x;
    const int b = ul / a.g, kv = ul - b * a.g;
    const int nsel = a.nsel[ul];
    const int t0 = split * 64;
    if (t0 >= nsel) return;
    __shared__ float s_p[64][G];
    __shared__ uint32_t s_row[64];
    __shared__ float s_o[4][G][kD];
    const int tid = threadIdx.x, lane16 = tid & 15, grp = tid >> 4, wv = tid >> 6, ln = tid & 63;
    if (tid < 64) {
        int tok = t0 + tid;
        bool ok = tok < nsel;
        int t = a.sel[(size_t)ul * a.top_k + (ok ? tok : t0)];
        s_row[tid] = row_of(a.v, a.g, b, kv, t);
#pragma unroll
        for (int hh = 0; hh < G; ++hh)
            s_p[tid][hh] = ok ? a.zsel[((size_t)ul * a.top_k + tok) * G + hh] : -__builtin_huge_valf();
    }
    __syncthreads();
    if (wv == 0) {
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            float v = s_p[ln][hh];
            float m = v;
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
            float p = __expf(v - m);
            float l = p;
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) l += __shfl_xor(l, o);
            s_p[ln][hh] = p;
            if (ln == 0) {
                size_t pi = ((size_t)b * a.h + kv * G + hh) * a.nsplit + split;
                a.pm[pi] = m;
                a.pl[pi] = l;
            }
        }
    }
    __syncthreads();
    float acc[G][8];
#pragma unroll
    for (int hh = 0; hh < G; ++hh)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[hh][e] = 0.0f;
    const T *V = (const T *)a.v.pages;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = r * 16 + grp;
        float vx[8];
        unpack(load_chunk(V + (size_t)s_row[row] * kD, lane16), vx);
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            float p = s_p[row][hh];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[hh][e] = __fmaf_rn(p, vx[e], acc[hh][e]);
        }
    }
#pragma unroll
    for (int hh = 0; hh < G; ++hh)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = acc[hh][e];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            acc[hh][e] = v;
        }
    if (ln < 16) {
#pragma unroll
        for (int hh = 0; hh < G; ++hh)
#pragma unroll
            for (int e = 0; e < 8; ++e) s_o[wv][hh][8 * lane16 + e] = acc[hh][e];
    }
    __syncthreads();
    for (int x = tid; x < G * kD; x += 256) {
        int hh = x / kD, e = x - hh * kD;
        float v = (s_o[0][hh][e] + s_o[1][hh][e]) + (s_o[2][hh][e] + s_o[3][hh][e]);
        a.po[(((size_t)b * a.h + kv * G + hh) * a.nsplit + split) * kD + e] = v;
    }
}

// grid (batch*h), 128 threads
template <int G> __global__ __launch_bounds__(128) void attn_merge_kernel(AttnArgs a)
{
    const int head = blockIdx.x;
    const int b = head / a.h, hq = head - b * a.h;
    const int ul = b * a.g + hq / G;
    const int nsel = a.nsel[ul];
    const int ns = (nsel + 63) >> 6;
    const int e = threadIdx.x;
    if (ns == 0) {
        a.out[(size_t)head * kD + e] = 0.0f;
        if (a.out_lse && e == 0) a.out_lse[head] = -__builtin_huge_valf();
        return;
    }
    const float *pm = a.pm + (size_t)head * a.nsplit;
    const float *pl = a.pl + (size_t)head * a.nsplit;
    float M = pm[0];
    for (int s = 1; s < ns; ++s) M = fmaxf(M, pm[s]);
    float l = 0.0f, o = 0.0f;
    for (int s = 0; s < ns; ++s) {
        float w = __expf(pm[s] - M);
        l = __fmaf_rn(pl[s], w, l);
        o = __fmaf_rn(a.po[((size_t)head * a.nsplit + s) * kD + e], w, o);
    }
    a.out[(size_t)head * kD + e] = o / l;
    if (a.out_lse && e == 0) a.out_lse[head] = M + __logf(l);
}

}  // namespace ctkvr
