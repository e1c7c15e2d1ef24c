// gfx950 kernels of the CTkvr path.
//
// Decode step (Algorithm 2 lines 1-9), seven or eight launches:
//   centroid_cos  lines 1-2   cosine to every centroid, max over the GQA group
//   recall_gather lines 3-4a  top-C' centroids; their lists OR-ed into a bitmap
//   recall_score  lines 4b-5a the bitmap as an ascending id list plus each id's physical
//                             KV row; z = (q . k) * scale for the G heads, running max
//   denom         line 5b     softmax denominators, integer fixed point
//   keyhist       line 5c     max over the group of log-softmax as a ranking key,
//                             and a histogram of the keys
//   classify      line 6a     chip-wide pass over the keys: sure picks as a bitmap, the
//                             deciding bucket as a list
//   rerank_select line 6b     top-rho' ids
//   sparse_attn   lines 7-9   softmax(z_sel) . V_sel, one block per slice of the
//                             head dimension (no cross-block reduction)
//   (select_attn = the last two in one launch, for small batches)
// The exact index build (Algorithm 1 lines 2-4) runs score -> denom -> keyhist -> rerank_select with
// "the recalled set" = all s keys and the centroid in the role of the query,
// which is literally the same formula.
#pragma once
#include "arith.hpp"
#include "common.hpp"

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

// Block -> (unit, block of the unit) for grids (blocks per unit, units).  Workgroups go to the 8 XCDs round-robin by
// linear id, every XCD has an L2 of its own, and what a kernel wrote is still in its XCD's L2 when the next kernel
// runs (a dependent load of such a line: 88 ns on the XCD that wrote it, 220 ns on another).  With by_xcd (the host
// sets it when the units are a multiple of 8) the blocks of unit u are those with linear id congruent u modulo the
// number of units: all on XCD u mod 8, in every kernel of a decode step, so that a unit's intermediate results are read
// where they were written.
__device__ __forceinline__ void unit_block_of(const int by_xcd, int &ul, int &bx)
{
    if (by_xcd) {
        const int lin = (int)(blockIdx.y * gridDim.x + blockIdx.x);
        ul = lin % (int)gridDim.y;
        bx = lin / (int)gridDim.y;
    } else {
        ul = (int)blockIdx.y;
        bx = (int)blockIdx.x;
    }
}

// ------------------------------------------------------------------------------
// small utilities
// ------------------------------------------------------------------------------
__global__ void fill_u32_kernel(uint32_t *p, uint32_t v, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// three ranges cleared by one launch: grid ceil((n0 + n1 + n2) / blockDim.x)
__global__ void zero3_u32_kernel(uint32_t *p0, size_t n0, uint32_t *p1, size_t n1, uint32_t *p2, size_t n2)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n0) {
        p0[i] = 0u;
    } else if (i < n0 + n1) {
        p1[i - n0] = 0u;
    } else if (i < n0 + n1 + n2) {
        p2[i - n0 - n1] = 0u;
    }
}

// Algorithm 1 line 1: centroid j of sequence b, head hd = prompt query at position s_b - C_b + j.
// q_prefill rows [first_row_b + j][h][128] -> centroids [b][h][c_max][128]
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
// grid (ceil(c_max/16), batch*g), 256 threads: one centroid per 16-lane group, its
// G head rows loaded together.  Block x == 0 also clears the step's accumulators.
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
    int by_xcd;               // blocks -> (unit, block of the unit) by unit_block_of
};

template <typename T, int G> __global__ __launch_bounds__(256) void centroid_cos_kernel(CosArgs a)
{
    int ul, bx;
    unit_block_of(a.by_xcd, ul, bx);
    const int b = ul / a.g, kv = ul - b * a.g;
    const int C = a.n_cent[b];
    const int tid = threadIdx.x, lane16 = tid & 15, grp = tid >> 4;
    if (bx == 0 && tid < G) {
        a.m_key[ul * G + tid] = 0u;
        a.S[ul * G + tid] = 0ull;
    }
    CTKVR_STAMP(0);
    const int tile0 = bx * 16;
    if (tile0 >= C) return;
    const int j = tile0 + grp;
    const int jj = j < C ? j : C - 1;
    const T *qb = (const T *)a.q + ((size_t)b * a.h + kv * G) * kD;
    const T *cb = (const T *)a.centroids;
    Chunk<T> cq[G], cc[G];
    float inc[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        size_t row = ((size_t)b * a.h + kv * G + hh) * a.c_max + jj;
        cc[hh] = load_chunk(cb + row * kD, lane16);
        cq[hh] = load_chunk(qb + (size_t)hh * kD, lane16);
        inc[hh] = a.inv_norm_c[row];
    }
    float best = -__builtin_huge_valf();
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        float q[8], cx[8];
        unpack(cq[hh], q);
        unpack(cc[hh], cx);
        float inv_q = inv_norm_from_sq(group16_sum(lane_partial(q, q)));
        float dot = group16_sum(lane_partial(q, cx));
        float cs = (dot * inc[hh]) * inv_q;
        best = fmaxf(best, cs);
    }
    if (j < C && lane16 == 0) a.cos[(size_t)ul * a.c_max + j] = best;
    CTKVR_STAMP(1);
}

// ------------------------------------------------------------------------------
// Algorithm 2 lines 3-4, first part, each (sequence, KV head) spread over several
// blocks so that no single CU has to pull all the probed lists (the bitmap becomes the
// ascending id list in recall_score_kernel).
//
// recall_gather: every block of a unit finds the same top-C' centroids (keys in
// registers, C <= 256*KPT, bisection on the key), takes every gridDim.x-th probed list, ORs its ids into a bitmap in shared memory and then
// ORs the non-empty words into the unit's bitmap in global memory (integer ORs: any
// order gives the same bitmap).  grid (blocks per unit, batch*g), 256 threads; dynamic shared
// memory: kSelLds + n_probe + bitmap words.
// ------------------------------------------------------------------------------
struct GatherArgs {
    const float *cos;         // [batch*g][c_max]
    const int32_t *lists;     // [batch*g][c_max][rho]
    const int32_t *n_cent, *ctx_lens;
    int32_t *probe;           // [batch*g][n_probe]
    int32_t *out_probe;       // optional copy for the caller
    uint32_t *gbits;          // [batch*g][bitmap_words], all zero between steps
    int g, c_max, rho, n_probe, bitmap_words;
    int by_xcd;               // blocks -> (unit, block of the unit) by unit_block_of
};

template <int KPT> __global__ __launch_bounds__(256) void recall_gather_kernel(GatherArgs a)
{
    extern __shared__ uint32_t smem[];
    uint32_t *s_sel = smem;
    int32_t *s_probe = (int32_t *)(smem + kSelLds);
    uint32_t *s_bits = smem + kSelLds + a.n_probe;
    int ul, bx;
    unit_block_of(a.by_xcd, ul, bx);
    const int tid = threadIdx.x, wv = tid >> 6, ln = tid & 63;
    const int b = ul / a.g;
    const int C = a.n_cent[b], s = a.ctx_lens[b];
    const float *cosv = a.cos + (size_t)ul * a.c_max;
    const int W = (s + 31) >> 5;
    CTKVR_STAMP(8);
    CTKVR_STAMP_BLK(0);
    for (int w = tid; w < W; w += 256) s_bits[w] = 0u;
    auto keep = [&](int pos, int j) {
        s_probe[pos] = j;
        if (bx == 0) {
            a.probe[(size_t)ul * a.n_probe + pos] = j;
            if (a.out_probe) a.out_probe[(size_t)ul * a.n_probe + pos] = j;
        }
    };
    // line 3
    // (a handful of probes, the paper's C' = 4: one block-wide maximum per probe; thousands of
    // centroids: 11-bit radix rounds instead of sixteen rounds of 3 x KPT ballots)
    if (a.n_probe <= 8)
        block_extract_topk<256, KPT>([&](int j) { return ordered_key(cosv[j]); }, C, a.n_probe, keep, s_sel);
    else if constexpr (KPT > 8)
        block_select_topk<256, KPT>([&](int j) { return ordered_key(cosv[j]); }, C, a.n_probe, keep, s_sel);
    else
        block_bisect_topk<256, KPT>([&](int j) { return ordered_key(cosv[j]); }, C, a.n_probe, keep, s_sel);
    __syncthreads();
    CTKVR_STAMP(9);
    // line 4: this block's share of the probed lists, one list per wave at a time
    const int32_t *lb = a.lists + (size_t)ul * a.c_max * a.rho;
    // Two lists per round and wave, all of a round's loads requested before the first id is used.
    const int pstride = gridDim.x * 4;
    auto mark = [&](int t) { atomicOr(&s_bits[t >> 5], 1u << (t & 31)); };
    for (int p = bx + gridDim.x * wv; p < a.n_probe; p += 2 * pstride) {
        const bool two = p + pstride < a.n_probe;
        const int32_t *l0 = lb + (size_t)s_probe[p] * a.rho;
        const int32_t *l1 = lb + (size_t)s_probe[two ? p + pstride : p] * a.rho;
        if ((a.rho & 3) == 0) {
            const int4 *s0 = reinterpret_cast<const int4 *>(l0), *s1 = reinterpret_cast<const int4 *>(l1);
            const int rho4 = a.rho >> 2;
            for (int r0 = 0; r0 < rho4; r0 += 64 * 8) {
                // (entries beyond the list's end re-read its last one and are not marked: a load under
                // a per-lane condition is waited for before the next is requested)
                int4 t0[8], t1[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) t0[u] = s0[min(r0 + u * 64 + ln, rho4 - 1)];
                if (two) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) t1[u] = s1[min(r0 + u * 64 + ln, rho4 - 1)];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int r = r0 + u * 64 + ln;
                    if (r < rho4) {
                        mark(t0[u].x); mark(t0[u].y); mark(t0[u].z); mark(t0[u].w);
                        if (two) { mark(t1[u].x); mark(t1[u].y); mark(t1[u].z); mark(t1[u].w); }
                    }
                }
            }
        } else {   // list rows not 16-byte aligned: the same rounds with 4-byte loads
            for (int r0 = 0; r0 < a.rho; r0 += 64 * 8) {
                int32_t t0[8], t1[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) t0[u] = l0[min(r0 + u * 64 + ln, a.rho - 1)];
                if (two) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) t1[u] = l1[min(r0 + u * 64 + ln, a.rho - 1)];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (r0 + u * 64 + ln < a.rho) {
                        mark(t0[u]);
                        if (two) mark(t1[u]);
                    }
                }
            }
        }
    }
    __syncthreads();
    CTKVR_STAMP(10);
    uint32_t *gb = a.gbits + (size_t)ul * a.bitmap_words;
    for (int w = tid; w < W; w += 256) {
        uint32_t v = s_bits[w];
        if (v) atomicOr(&gb[w], v);
    }
    CTKVR_STAMP_BLK(1);
}

// ------------------------------------------------------------------------------
// Algorithm 2 line 5 / Algorithm 1 line 2, first half: z[h][i] = (q_h . k_i) * scale
// for the G heads of the group, plus the running maximum per head.  A block walks
// tiles of 16*R ids (R rows per 16-lane group, all R loads issued before the first
// use) with stride gridDim.x.  grid (nbx, units), 256 threads.
// ------------------------------------------------------------------------------
struct ScoreArgs {
    Units u;
    const void *q;            // decode: [batch][h][128] (qrows = 1); build: centroids [batch][h][c_max][128] (qrows = c_max)
    int qrows;
    Paged k;
    const int32_t *ctx_lens;
    const uint32_t *crow;     // [units][l_stride] physical rows of the recalled ids, or nullptr = all ids 0..s-1
    const int32_t *ncand;     // [units] (with crow)
    int l_stride;
    float *z;                 // [units][l_stride][G]
    uint32_t *m_key;          // [units][G] ordered-key running max (atomicMax)
    uint32_t *ghist;          // decode only: [units][kBuckets] key histogram, cleared here for keyhist
    float scale;
};

template <typename T, int G, int R> __global__ __launch_bounds__(256) void score_kernel(ScoreArgs a)
{
    constexpr int TILE = 16 * R;
    int b, kv, j;
    const int ul = blockIdx.y;
    if (!decode_unit(a.u, ul, b, kv, j)) return;
    const int tid = threadIdx.x, lane16 = tid & 15, grp = tid >> 4;
    // decode: the first tile's row ids are requested together with L, not after it (slots beyond
    // L hold stale words; they are never used as rows, see the clamp below)
    uint32_t pre = 0;
    if (a.crow && tid < TILE) pre = a.crow[(size_t)ul * a.l_stride + min((int)blockIdx.x * TILE + tid, a.l_stride - 1)];
    const int L = a.crow ? a.ncand[ul] : a.ctx_lens[b];
    if (a.ghist)
        for (int w = blockIdx.x * 256 + threadIdx.x; w < kBuckets; w += gridDim.x * 256) a.ghist[(size_t)ul * kBuckets + w] = 0u;
    if ((int)blockIdx.x * TILE >= L) return;
    __shared__ uint32_t s_row[TILE];
    __shared__ uint32_t s_max[G];
    CTKVR_STAMP(20);
    if (tid < G) s_max[tid] = 0u;
    float q[G][8];
    const T *qb = (const T *)a.q + (((size_t)b * a.u.h + kv * G) * a.qrows + j) * kD;
#pragma unroll
    for (int hh = 0; hh < G; ++hh) unpack(load_chunk(qb + (size_t)hh * a.qrows * kD, lane16), q[hh]);
    const T *K = (const T *)a.k.pages;
    float *zb = a.z + (size_t)ul * a.l_stride * G;
    // lane l of a 16-lane group keeps head (l mod G): its score, and that head's running maximum
    float mxl = -__builtin_huge_valf();
    const int myh = lane16 & (G - 1);
    for (int tile0 = blockIdx.x * TILE; tile0 < L; tile0 += gridDim.x * TILE) {
        __syncthreads();   // previous tile's rows are consumed
        if (tid < TILE) {
            int i = min(tile0 + tid, L - 1);
            if (a.crow)
                s_row[tid] = (tile0 == (int)blockIdx.x * TILE) ? pre : a.crow[(size_t)ul * a.l_stride + i];
            else
                s_row[tid] = row_of(a.k.block_table, a.k.max_pages, a.k.page_shift, a.u.g, b, kv, i);
        }
        __syncthreads();
        const int last = L - 1 - tile0;   // slots of the tile beyond it repeat the last valid row
        CTKVR_STAMP(21);
        Chunk<T> ck[R];
#pragma unroll
        for (int r = 0; r < R; ++r) ck[r] = load_chunk(K + (size_t)s_row[min(r * 16 + grp, last)] * kD, lane16);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float kx[8];
            unpack(ck[r], kx);
            float mine = 0.0f;
#pragma unroll
            for (int hh = 0; hh < G; ++hh) {
                float tot = group16_sum(lane_partial(q[hh], kx));
                if (hh == 0 || myh == hh) mine = tot;
            }
            mine = mine * a.scale;
            const int i = tile0 + r * 16 + grp;
            if (i < L) {
                mxl = __builtin_amdgcn_fmed3f(mxl, mine, __builtin_huge_valf());   // max of two non-NaN values
                if (lane16 < G) zb[(size_t)i * G + lane16] = mine;
            }
        }
    }
    {
        float v = mxl;
        v = __builtin_amdgcn_fmed3f(v, __shfl_xor(v, 16), __builtin_huge_valf());
        v = __builtin_amdgcn_fmed3f(v, __shfl_xor(v, 32), __builtin_huge_valf());
        if (lane_id() < G) atomicMax(&s_max[lane_id()], ordered_key(v));
    }
    __syncthreads();
    if (tid < G) atomicMax(&a.m_key[ul * G + tid], s_max[tid]);
    CTKVR_STAMP(22);
}

// ------------------------------------------------------------------------------
// Algorithm 2 lines 10-11: attention over the resident window -- the first n_init keys and the
// keys from s - n_local to the current end of the cache (the tokens decoded since the index was
// built join the local window) -- and its merge with the sparse attention.
// window_attn_kernel: block x of a unit takes every kWinSplit-th run of 64 window rows and leaves
// a partial result relative to its own maximum: m[G], l[G] = sum of exp(z - m), o[G][128] = sum of
// exp(z - m) v.  Online softmax over runs of 64 rows (one row per 16-lane group and pass, four
// passes).  It depends on q, K and V only: as a launch of its own it is the first of a step (grid (kWinSplit,
// units), 256 threads); the step of one launch per stage runs the same blocks as kWinSplit extra blocks per
// unit of recall_score_kernel's launch instead, where they cost no launch and run beside the scoring blocks.
// ------------------------------------------------------------------------------

struct WindowArgs {
    Units u;
    const void *q;            // [batch][h][128]
    Paged k;
    const void *v_pages;
    const int32_t *ctx_lens;  // [batch] s: the prefix the index was built on
    const int32_t *cur_lens;  // optional [batch]: tokens in the cache now (>= s)
    int n_init, n_local;
    int by_xcd;               // blocks -> (unit, block of the unit) by unit_block_of
    float scale;
    float *win;               // [units][kWinSplit][G][2 + 128]
};

// One block's share: bx of kWinSplit, unit ul; 256 threads.
template <typename T, int G> __device__ __forceinline__ void window_attn_block(const WindowArgs &a, const int bx, const int ul)
{
    __shared__ float s_z[64][G];
    __shared__ float s_part[4][G][kD];
    __shared__ float s_ml[G];
    const int b = ul / a.u.g, kv = ul - b * a.u.g;
    const int tid = threadIdx.x, lane16 = tid & 15, grp = tid >> 4;
    const int s = a.ctx_lens[b];
    int cur = a.cur_lens ? a.cur_lens[b] : s;
    cur = max(s, min(cur, a.k.max_pages << a.k.page_shift));
    const int ni = min(a.n_init, s), nl = min(a.n_local, s - ni);
    const int n_w = ni + nl + (cur - s);
    auto id_of = [&](int r) { return r < ni ? r : s - nl + (r - ni); };
    float q[G][8];
    const T *qb = (const T *)a.q + ((size_t)b * a.u.h + kv * G) * kD;
#pragma unroll
    for (int hh = 0; hh < G; ++hh) unpack(load_chunk(qb + (size_t)hh * kD, lane16), q[hh]);
    const T *K = (const T *)a.k.pages;
    const T *V = (const T *)a.v_pages;
    float m_run[G], l_run[G], acc[G][8];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        m_run[hh] = -__builtin_huge_valf();
        l_run[hh] = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[hh][e] = 0.0f;
    }
    for (int r0 = bx * 64; r0 < n_w; r0 += kWinSplit * 64) {
        const int nr = min(64, n_w - r0);
        uint32_t row[4];
        Chunk<T> ck[4], cv[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int r = min(p * 16 + grp, nr - 1);
            row[p] = row_of(a.k.block_table, a.k.max_pages, a.k.page_shift, a.u.g, b, kv, id_of(r0 + r));
        }
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            ck[p] = load_chunk(K + (size_t)row[p] * kD, lane16);
            cv[p] = load_chunk(V + (size_t)row[p] * kD, lane16);
        }
        __syncthreads();   // the previous run's s_z and s_ml have been read
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            float kx[8];
            unpack(ck[p], kx);
#pragma unroll
            for (int hh = 0; hh < G; ++hh) {
                float tot = group16_sum(lane_partial(q[hh], kx)) * a.scale;
                if (lane16 == hh) s_z[p * 16 + grp][hh] = tot;
            }
        }
        __syncthreads();
        if (tid < 64) {   // the run's maximum per head (one row per lane of the first wave)
#pragma unroll
            for (int hh = 0; hh < G; ++hh) {
                float mx = tid < nr ? s_z[tid][hh] : -__builtin_huge_valf();
#pragma unroll
                for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
                if (tid == 0) s_ml[hh] = mx;
            }
        }
        __syncthreads();
        float corr[G];
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            const float m_new = fmaxf(m_run[hh], s_ml[hh]);   // the same in every thread
            corr[hh] = __expf(m_run[hh] - m_new);          // exp(-inf) = 0 on the first run
            m_run[hh] = m_new;
            l_run[hh] *= corr[hh];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[hh][e] *= corr[hh];
        }
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int r = p * 16 + grp;
            if (r < nr) {
                float vx[8];
                unpack(cv[p], vx);
#pragma unroll
                for (int hh = 0; hh < G; ++hh) {
                    const float pr = __expf(s_z[r][hh] - m_run[hh]);
                    if (lane16 == 0) l_run[hh] += pr;   // lane 0 of each group carries the group's share of l
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[hh][e] = __fmaf_rn(pr, vx[e], acc[hh][e]);
                }
            }
        }
    }
    // the 16 groups hold partial sums over their rows, all relative to the same running maximum:
    // first the four groups of a wave (lanes l, l+16, l+32, l+48), then the four waves
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = acc[hh][e];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            acc[hh][e] = v;
        }
        float l = l_run[hh];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        l_run[hh] = l;
    }
    __syncthreads();
    const int wv = tid >> 6;
    if ((tid & 63) < 16) {
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s_part[wv][hh][lane16 * 8 + e] = acc[hh][e];
        }
        if (lane16 == 0) {
#pragma unroll
            for (int hh = 0; hh < G; ++hh) s_z[wv][hh] = l_run[hh];
        }
    }
    __syncthreads();
    float *dst = a.win + ((size_t)ul * kWinSplit + bx) * G * (2 + kD);
    for (int i = tid; i < G * kD; i += 256) {
        const int hh = i >> 7, e = i & 127;
        dst[hh * (2 + kD) + 2 + e] = (s_part[0][hh][e] + s_part[1][hh][e]) + (s_part[2][hh][e] + s_part[3][hh][e]);
    }
    if (tid < G) {
        dst[tid * (2 + kD)] = m_run[tid];
        dst[tid * (2 + kD) + 1] = (s_z[0][tid] + s_z[1][tid]) + (s_z[2][tid] + s_z[3][tid]);
    }
}

template <typename T, int G> __global__ __launch_bounds__(256) void window_attn_kernel(WindowArgs a)
{
    int ul, bx;
    unit_block_of(a.by_xcd, ul, bx);
    window_attn_block<T, G>(a, bx, ul);
}

// ------------------------------------------------------------------------------
// Algorithm 2 lines 4-5 in one launch (decode).  A unit's bitmap of recalled ids is split over the
// unit's blocks; a block turns its part into ascending ids 64 words at a time (one byte per thread,
// positions by a block scan), writes them and their physical rows to their ranks of the recalled
// list, and scores the rows like score_kernel: z[rank][G], running maximum per head.
// Two ways to split, chosen by the host:
//   by id range -- block x owns words [x wpb, (x + 1) wpb), wpb <= 64, and counts the ids in the words
//     before its own (coalesced 4-byte loads, no scan).  The cheapest prologue; recalled keys cluster,
//     so some blocks get several times the rows of others, which does not matter while every CU has
//     many blocks' worth of rows to stream.
//   by rank -- block x takes ranks [x q, (x + 1) q), q = ceil(L / blocks): every block counts the whole
//     bitmap (a contiguous stretch of words per thread, one block scan), which gives L and tells the
//     two threads whose stretches hold the block's first and last rank to name their words.  One more
//     round trip to the cache, but every block then has the same number of rows: for small batches,
//     where a block's rows are one or two round trips to memory and the slowest block is the launch.
// The block that sees the unit's last word (by id) or block 0 (by rank) also writes L.
// grid (nbx [+ kWinSplit], units), 256 threads; by id nbx >= W_max / 64, by rank nbx >= l_stride / kRecallCap.
// ------------------------------------------------------------------------------
constexpr int kRecallWpb = 64;     // by id range: at most 2048 ids per block
constexpr int kRecallCap = 2048;   // ids per block at most

struct RecallScoreArgs {
    Units u;
    const void *q;            // [batch][h][128]
    Paged k;
    const int32_t *ctx_lens;
    const uint32_t *gbits;    // [units][bitmap_words]
    int bitmap_words, l_stride;
    int32_t *cand;            // [units][l_stride] recalled ids, ascending
    uint32_t *crow;           // [units][l_stride] their physical rows
    int32_t *ncand;           // [units] L
    int32_t *out_ncand;       // optional copy for the caller
    float *z;                 // [units][l_stride][G]
    uint32_t *m_key;          // [units][G] ordered-key running max (atomicMax)
    uint32_t *ghist;          // [units][kBuckets] key histogram, cleared here for keyhist
    float scale;
    int stream_k;             // the keys of all sequences exceed what the memory-side cache holds: load them non-temporal
    int by_rank;              // how the bitmap is split over a unit's blocks
    int by_xcd;               // blocks -> (unit, block of the unit) by unit_block_of
    int nbx;                  // blocks per unit that score; with WIN blocks nbx .. nbx + kWinSplit - 1 take the resident window
    WindowArgs win;
};

template <typename T, int G, bool WIN> __global__ __launch_bounds__(256) void recall_score_kernel(RecallScoreArgs a)
{
    constexpr int R = 8, TILE = 16 * R;
    __shared__ uint32_t s_ids[kRecallCap];        // ids of this block's ranks, then their rows
    __shared__ int32_t s_page[256];               // block-table entries of the pages its ids lie in
    __shared__ uint32_t s_tmp[8];
    __shared__ uint32_t s_edge[3];                // first word, ids before it, last word
    __shared__ uint32_t s_max[G];
    int ul, bx;
    unit_block_of(a.by_xcd, ul, bx);
    if constexpr (WIN) {
        if (bx >= a.nbx) {   // Algorithm 2 lines 10-11 beside lines 4-5
            window_attn_block<T, G>(a.win, bx - a.nbx, ul);
            return;
        }
    }
    const int b = ul / a.u.g, kv = ul - b * a.u.g;
    const int tid = threadIdx.x, lane16 = tid & 15, grp = tid >> 4;
    CTKVR_STAMP_BLK(6);
    const int s_len = a.ctx_lens[b];
    const int W = (s_len + 31) >> 5;
    for (int w = bx * 256 + tid; w < kBuckets; w += (uint32_t)a.nbx * 256) a.ghist[(size_t)ul * kBuckets + w] = 0u;
    const uint32_t *gb = a.gbits + (size_t)ul * a.bitmap_words;
    if (tid < G) s_max[tid] = 0u;
    uint32_t r0, r1;   // the block's ranks
    if (a.by_rank) {
        // thread t counts words [t wpt, (t + 1) wpt), wpt a multiple of four: 16-byte loads where the
        // unit's words start on a 16-byte boundary (words from W up to the row's end are zero)
        const int wpt = ((((W + 255) >> 8) + 3) >> 2) << 2;
        const int w0 = tid * wpt;
        const bool wide = ((reinterpret_cast<uintptr_t>(gb) | ((uintptr_t)a.bitmap_words << 2)) & 15u) == 0;
        // up to 16 words per thread (contexts up to 128K) stay in registers, so that the two threads that
        // name the block's edge words below need no further load
        const bool in_regs = wide && wpt <= 16;
        uint4 v[4] = {};
        uint32_t cnt = 0;
        if (in_regs) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int w = w0 + 4 * i;
                const uint4 x = *reinterpret_cast<const uint4 *>(gb + min(w, a.bitmap_words - 4));
                if (i * 4 < wpt && w < a.bitmap_words) v[i] = x;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) cnt += (uint32_t)(__popc(v[i].x) + __popc(v[i].y) + __popc(v[i].z) + __popc(v[i].w));
        } else if (wide) {
#pragma unroll 4
            for (int w = w0; w < min(w0 + wpt, a.bitmap_words); w += 4) {
                const uint4 x = *reinterpret_cast<const uint4 *>(gb + w);
                cnt += (uint32_t)(__popc(x.x) + __popc(x.y) + __popc(x.z) + __popc(x.w));
            }
        } else {
#pragma unroll 4
            for (int w = w0; w < min(w0 + wpt, W); ++w) cnt += (uint32_t)__popc(gb[w]);
        }
        uint32_t L;
        const uint32_t pre = block_excl_scan<256>(cnt, s_tmp, &L);   // barriers inside
        if (bx == 0 && tid == 0) {
            a.ncand[ul] = (int32_t)L;
            if (a.out_ncand) a.out_ncand[ul] = (int32_t)L;
        }
        const uint32_t qn = (L + (uint32_t)a.nbx - 1) / (uint32_t)a.nbx;
        r0 = bx * qn;
        if (r0 >= L) return;
        r1 = min(L, r0 + qn);
        // the threads whose stretches hold ranks r0 and r1 - 1 walk their words to the one that holds it
        const bool own_first = cnt && pre <= r0 && r0 < pre + cnt;
        const bool own_last = cnt && pre < r1 && r1 <= pre + cnt;
        if (in_regs) {
            if (own_first || own_last) {
                const uint32_t wd[16] = {v[0].x, v[0].y, v[0].z, v[0].w, v[1].x, v[1].y, v[1].z, v[1].w,
                                         v[2].x, v[2].y, v[2].z, v[2].w, v[3].x, v[3].y, v[3].z, v[3].w};
                uint32_t p = pre, e0 = 0, e1 = 0, e2 = 0;
                bool f0 = !own_first, f2 = !own_last;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const uint32_t c = (uint32_t)__popc(wd[i]);
                    if (!f0 && r0 < p + c) {
                        e0 = (uint32_t)(w0 + i);
                        e1 = p;
                        f0 = true;
                    }
                    p += c;
                    if (!f2 && r1 <= p) {
                        e2 = (uint32_t)(w0 + i);
                        f2 = true;
                    }
                }
                if (own_first) {
                    s_edge[0] = e0;
                    s_edge[1] = e1;
                }
                if (own_last) s_edge[2] = e2;
            }
        } else {
            if (own_first) {
                uint32_t p = pre;
                for (int w = w0; w < w0 + wpt; ++w) {
                    const uint32_t c = (uint32_t)__popc(gb[w]);
                    if (r0 < p + c) {
                        s_edge[0] = (uint32_t)w;
                        s_edge[1] = p;
                        break;
                    }
                    p += c;
                }
            }
            if (own_last) {
                uint32_t p = pre;
                for (int w = w0; w < w0 + wpt; ++w) {
                    p += (uint32_t)__popc(gb[w]);
                    if (r1 <= p) {
                        s_edge[2] = (uint32_t)w;
                        break;
                    }
                }
            }
        }
    } else {
        // the unit's own words split evenly over the blocks of its row (a short sequence of a ragged
        // batch still uses all of them)
        const int wpb = min(kRecallWpb, (W + a.nbx - 1) / a.nbx);
        const int w_beg = bx * wpb;
        if (w_beg >= W) return;
        uint32_t before = 0;
#pragma unroll 4
        for (int w = tid; w < w_beg; w += 256) before += (uint32_t)__popc(gb[w]);
        before = wave_sum_uniform(before);
        if ((tid & 63) == 0) s_tmp[tid >> 6] = before;
        __syncthreads();
        if (tid == 0) {
            s_edge[0] = (uint32_t)w_beg;
            s_edge[1] = s_tmp[0] + s_tmp[1] + s_tmp[2] + s_tmp[3];
            s_edge[2] = (uint32_t)(min(W, w_beg + wpb) - 1);
        }
        r0 = r1 = 0u;   // known after the (single) pass over the block's words
    }
    __syncthreads();
    const int wa = (int)s_edge[0], wb = (int)s_edge[2];
    uint32_t rank0 = s_edge[1];   // ids before the pass's first word
    if (!a.by_rank) {
        r0 = rank0;
        r1 = 0xffffffffu;
    }
    CTKVR_STAMP_BLK(7);
    // requested together: the first pass's words and the block-table entries of the pages between the two words
    uint32_t myword = (wa + (tid >> 2) <= wb) ? gb[wa + (tid >> 2)] : 0u;
    const int page0 = (wa << 5) >> a.k.page_shift;
    const int npages = ((min((wb << 5) + 31, s_len - 1)) >> a.k.page_shift) - page0 + 1;
    const bool lds_pages = npages <= 256;
    if (lds_pages && tid < npages) s_page[tid] = a.k.block_table[(size_t)b * a.k.max_pages + page0 + tid];
    for (int wp = wa; wp <= wb; wp += 64) {
        if (wp != wa) myword = (wp + (tid >> 2) <= wb) ? gb[wp + (tid >> 2)] : 0u;
        uint32_t m = (myword >> ((tid & 3) << 3)) & 0xffu;
        uint32_t n_pass;
        uint32_t rk = rank0 + block_excl_scan<256>((uint32_t)__popc(m), s_tmp, &n_pass);   // barriers inside
        const uint32_t id0 = ((uint32_t)(wp + (tid >> 2)) << 5) + ((uint32_t)(tid & 3) << 3);
        while (m) {
            const int bit = __ffs((int)m) - 1;
            m &= m - 1u;
            if (rk >= r0 && rk < r1) s_ids[rk - r0] = id0 + (uint32_t)bit;
            ++rk;
        }
        rank0 += n_pass;
    }
    if (!a.by_rank) {   // one pass: the block's ids are all the ids of its words
        r1 = rank0;
        if (wb == W - 1 && tid == 0) {
            a.ncand[ul] = (int32_t)r1;
            if (a.out_ncand) a.out_ncand[ul] = (int32_t)r1;
        }
        if (r1 == r0) return;
    }
    const uint32_t n_blk = r1 - r0;
    __syncthreads();
    const uint32_t base = r0;
    int32_t *cd = a.cand + (size_t)ul * a.l_stride + base;
    uint32_t *rw = a.crow + (size_t)ul * a.l_stride + base;
    const int pmask = (1 << a.k.page_shift) - 1;
    for (uint32_t i = tid; i < n_blk; i += 256) {
        const int t = (int)s_ids[i];
        uint32_t row;
        if (lds_pages)
            row = (uint32_t)((s_page[(t >> a.k.page_shift) - page0] * a.u.g + kv) << a.k.page_shift) + (uint32_t)(t & pmask);
        else
            row = row_of(a.k.block_table, a.k.max_pages, a.k.page_shift, a.u.g, b, kv, t);
        cd[i] = t;
        rw[i] = row;
        s_ids[i] = row;   // each slot is read and rewritten by the same thread
    }
    __syncthreads();
    CTKVR_STAMP_BLK(2);
    const T *K = (const T *)a.k.pages;
    float *zb = a.z + ((size_t)ul * a.l_stride + base) * G;
    // the queries are requested with the first rows (cached, they arrive well before the rows do)
    float q[G][8];
    const T *qb = (const T *)a.q + ((size_t)b * a.u.h + kv * G) * kD;
#pragma unroll
    for (int hh = 0; hh < G; ++hh) unpack(load_chunk(qb + (size_t)hh * kD, lane16), q[hh]);
    // lane l of a 16-lane group keeps head (l mod G): its score, and that head's running maximum
    float mxl = -__builtin_huge_valf();
    const int myh = lane16 & (G - 1);
    const int last = (int)n_blk - 1;
    for (int t0 = 0; t0 < (int)n_blk; t0 += TILE) {
        Chunk<T> ck[R];
        const T *krow[R];
#pragma unroll
        for (int r = 0; r < R; ++r) krow[r] = K + (size_t)s_ids[min(t0 + r * 16 + grp, last)] * kD;
        if (a.stream_k) {
#pragma unroll
            for (int r = 0; r < R; ++r) ck[r] = load_chunk_nt(krow[r], lane16);
        } else {
#pragma unroll
            for (int r = 0; r < R; ++r) ck[r] = load_chunk(krow[r], lane16);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float kx[8];
            unpack(ck[r], kx);
            float mine_z = 0.0f;
#pragma unroll
            for (int hh = 0; hh < G; ++hh) {
                float tot = group16_sum(lane_partial(q[hh], kx));
                if (hh == 0 || myh == hh) mine_z = tot;
            }
            mine_z = mine_z * a.scale;
            const int i = t0 + r * 16 + grp;
            if (i <= last) {
                mxl = __builtin_amdgcn_fmed3f(mxl, mine_z, __builtin_huge_valf());   // max of two non-NaN values
                if (lane16 < G) zb[(size_t)i * G + lane16] = mine_z;
            }
        }
    }
    {
        float v = mxl;
        v = __builtin_amdgcn_fmed3f(v, __shfl_xor(v, 16), __builtin_huge_valf());
        v = __builtin_amdgcn_fmed3f(v, __shfl_xor(v, 32), __builtin_huge_valf());
        if (lane_id() < G) atomicMax(&s_max[lane_id()], ordered_key(v));
    }
    __syncthreads();
    if (tid < G) atomicMax(&a.m_key[ul * G + tid], s_max[tid]);
    CTKVR_STAMP_BLK(3);
}

// ------------------------------------------------------------------------------
// Algorithm 1 line 2 on the matrix cores (bf16 only): the same z = (c_{h,j} . k_t) *
// scale as score_kernel in build mode, but the 128-term dot is a chain of eight
// v_mfma_f32_32x32x16_bf16.  A block owns 8/G sub-tiles of 32 centroids of one
// (sequence, KV head) for all G heads (8 wave work items, two per wave -- two heads of the
// same sub-tile when G >= 2 -- their A fragments resident in registers) and walks a range of
// keys 32 at a time: B fragments are 16-byte pieces of the paged key rows; in the passes that
// form ranking keys the 32x32 results of a head pair are reduced in registers and go through
// shared memory, where the maximum over the pairs is taken.  grid (t_splits, tiles), 256 threads.
// The scores differ from the fixed arithmetic in the accumulation order inside the MFMA and
// the softmax denominators in how they are summed; on inputs whose dot products are exact in
// fp32 only the latter is left.
// ------------------------------------------------------------------------------
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

struct MfmaScoreArgs {
    int g, G, h, c_max;
    int bk0;                   // first (sequence, KV head) pair of this chunk
    int tiles_per_bk;          // ceil(c_max / (32 * 8/G))
    int t_splits;
    const int32_t *n_cent, *ctx_lens;
    const bf16_t *centroids;   // [batch][h][c_max][128]
    Paged k;
    int l_stride;              // s_max
    float2 *part;              // [chunk units][G][t_splits] (maximum of z log2(e), sum of 2^(z log2(e) - maximum)) over a block's keys
    uint32_t *kbuf;            // KEY: [chunk units][l_stride] ranking keys; SAMPLE: [chunk units][sample_stride]
    int n_init, n_local;       // keys of the resident window get the lowest ranking key
    float scale;
    int step_stride;           // SAMPLE: every step_stride-th step of 32 keys is taken (1 in the other passes)
    int sample_stride;         // SAMPLE: keys per unit in kbuf
    const uint32_t *tau;       // PICK: [chunk units] keys at or above it are candidates
    uint2 *cand;               // PICK: [chunk units][t_splits][seg_cap] (key, id): block x of a tile fills segment x of its units
    uint32_t *seg_cnt;         // PICK: [chunk units][t_splits] candidates of the segment (may exceed seg_cap: the excess is not stored)
    int seg_cap;
};

// The scores are never stored: the contraction is repeated in two passes over the same tiles, each
// with its own epilogue -- MFMA_STAT: per (centroid, head) the running maximum m of the scores and the
// running sum of exp(z - m), rescaled whenever the maximum moves, in fp32 with the hardware
// exponential (this route's lists are compared with the fixed arithmetic inside an error band anyway,
// and the band has room for a denominator that is a few 1e-5 off); one (m, sum) pair per block, merged
// in block order by the next pass.  MFMA_KEY: ranking keys max_h ((z - m_h) - log S_h), written as
// ordered uint32 (4 bytes per (centroid, key) instead of 4 G bytes of scores read twice).
// Writing, and twice re-reading, a key for every (centroid, key) pair is most of that route's time, and only
// rho of a unit's s keys are wanted.  MFMA_SAMPLE computes the keys of every step_stride-th step only (a
// systematic sample of the positions) into a small buffer, from which a threshold tau per unit is taken
// (a sample rank chosen so that about 2 rho keys of the unit lie at or above it); MFMA_PICK then computes all
// keys again and keeps the (key, id) pairs at or above tau -- a few thousand per unit -- from which the rho
// largest are selected exactly.  Should a unit end with fewer than rho candidates, or more than fit, the
// chunk is redone by the KEY route: the result never depends on the sample.
enum { MFMA_STAT = 0, MFMA_KEY = 2, MFMA_SAMPLE = 3, MFMA_PICK = 4 };

template <int G, int MODE> __global__ __launch_bounds__(256, 2) void mfma_score_kernel(MfmaScoreArgs a)
{
    constexpr int MT = 8 / G;        // 32-centroid sub-tiles per block
    constexpr int CT = 32 * MT;      // centroids per block
    // The key passes: the result tiles, [head pair][centroid][key] -- a wave's two work items are two heads of
    // the same 32 centroids (G >= 2), so the maximum over that pair is taken in registers and one plane per
    // pair goes through shared memory; a lane's four consecutive keys are one 16-byte write, a reader's four
    // keys one 16-byte read; 36-word rows spread both over the banks
    constexpr int ZS = 36;
    constexpr int NPL = G >= 2 ? G / 2 : 1;    // planes
    constexpr bool KEYS = MODE != MFMA_STAT;   // the passes that form ranking keys
    __shared__ __align__(16) float s_z[KEYS ? 2 * NPL * CT * ZS : 4];   // two buffers: see keys_out
    // PICK: the tile's thresholds and how many candidates this block has found for each of its centroids.  A block
    // owns a segment of every unit's candidate list, so positions are handed out by shared-memory counters: no
    // atomic on device memory (on this part those are served beyond the XCD's cache, a round trip each).
    __shared__ float s_tauf[MODE == MFMA_PICK ? CT : 1];
    __shared__ uint32_t s_cnt[MODE == MFMA_PICK ? CT : 1];
    __shared__ __align__(16) unsigned char s_k[2][32 * 272];
    const int tid = threadIdx.x, wv = tid >> 6, ln = tid & 63;
    const int col = ln & 31, half = ln >> 5;
    const int bkl = blockIdx.y / a.tiles_per_bk, jt = blockIdx.y - bkl * a.tiles_per_bk;
    const int bk = a.bk0 + bkl;
    const int b = bk / a.g, kv = bk - b * a.g;
    const int C = a.n_cent[b], s = a.ctx_lens[b];
    const int j0 = jt * CT;
    if (j0 >= C) return;
    const int tper = (((s + a.t_splits - 1) / a.t_splits) + 31) & ~31;
    const int ST = MODE == MFMA_SAMPLE ? 32 * a.step_stride : 32;   // keys from one step to the next
    // SAMPLE: the steps taken are those that start at a multiple of ST; a block starts at the first one in its range
    const int tbeg = MODE == MFMA_SAMPLE ? ((int)(blockIdx.x * tper) + ST - 1) / ST * ST : (int)(blockIdx.x * tper);
    const int tend = min(s, (int)(blockIdx.x * tper) + tper);
    if (tbeg >= tend) return;
    if constexpr (MODE == MFMA_PICK) {
        if (tid < CT) {
            const uint32_t tk = a.tau[(size_t)bkl * a.c_max + min(j0 + tid, C - 1)];
            s_tauf[tid] = tk ? ordered_value(tk) : -__builtin_huge_valf();   // 0: no threshold, every key is a candidate
            s_cnt[tid] = 0u;
        }
    }
    // The matrix instruction is issued with the keys as its row operand and the centroids as its
    // column operand: a lane then holds ONE centroid (column `col` of its sub-tile) against 16
    // keys (rows 8 (r / 4) + 4 half + r % 4), and that centroid's statistics are single registers.
    int hh[2], mt[2];
    bf16x8_t cfrag[2][8];                  // the centroid fragments, resident
    float mx[2];                           // STAT: running maximum; KEY: the final maximum m
    float lsv[2];                          // STAT: running sum of exp(z - mx); KEY: log S
    size_t stat[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        int it = wv * 2 + q;
        mt[q] = it / G;   // G >= 2: both items of a wave are heads of one sub-tile; G = 1: two sub-tiles
        hh[q] = it - mt[q] * G;
        const int j = min(j0 + mt[q] * 32 + col, C - 1);   // columns beyond C repeat centroid C-1 and are dropped at the end
        const bf16_t *row = a.centroids + (((size_t)b * a.h + kv * G + hh[q]) * a.c_max + j) * kD;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) cfrag[q][ks] = *reinterpret_cast<const bf16x8_t *>(row + ks * 16 + 8 * half);
        stat[q] = ((size_t)bkl * a.c_max + j) * G + hh[q];
        mx[q] = -__builtin_huge_valf();
        lsv[q] = 0.0f;
        if constexpr (KEYS) {
            // the blocks' pairs in block order: the same value in every block that reads them
            const float2 *pp = a.part + stat[q] * a.t_splits;
            float m = -__builtin_huge_valf();
            for (int x = 0; x < a.t_splits && x * tper < s; ++x) m = fmaxf(m, pp[x].x);
            float S = 0.0f;
            for (int x = 0; x < a.t_splits && x * tper < s; ++x) S += pp[x].y * __builtin_amdgcn_exp2f(pp[x].x - m);
            mx[q] = m * 0.693147180559945309f;   // the pairs hold base-two maxima
            lsv[q] = logf(S);
        }
    }
    const float sc2 = a.scale * 1.44269504088896341f;   // scores in base two (statistics pass)
    // key passes: the score's offset -(m + log S), so that a key is one fused multiply-add per score
    const float off[2] = {-(mx[0] + lsv[0]), -(mx[1] + lsv[1])};
    // The 32 key rows of a step (8 KB) go through shared memory once for the four waves, in two
    // buffers; a step's rows are requested two steps ahead and their block-table entries four
    // steps ahead, so that neither latency is waited for.  Rows beyond the sequence are clamped
    // to its last key.
    const bf16_t *K = (const bf16_t *)a.k.pages;
    constexpr int ROWB = 272;   // bytes per staged key row (256 + padding: fragment reads spread over the banks)
    const int srow = tid >> 3, spart = tid & 7;
    // A row's block-table entry is requested four steps ahead and turned into the row only when
    // the row itself is requested: computing it at once would wait for the entry, and with it for
    // every key request still in flight.
    const int32_t *bt_row = a.k.block_table + (size_t)b * a.k.max_pages;
    auto page_at = [&](int t0) { return bt_row[min(t0 + srow, s - 1) >> a.k.page_shift]; };
    auto row_from = [&](int page, int t0) {
        return (uint32_t)((page * a.g + kv) << a.k.page_shift) + (uint32_t)(min(t0 + srow, s - 1) & ((1 << a.k.page_shift) - 1));
    };
    // staging registers as named variables: an array indexed through the helpers would be kept in
    // private memory, and every request would then be waited for at once to be stored there
    uint4 st0a, st0b, st1a, st1b;
    auto fetch = [&](uint4 &x, uint4 &y, uint32_t row) {
        const uint4 *src = reinterpret_cast<const uint4 *>(K + (size_t)row * kD + spart * 16);
        x = src[0];
        y = src[1];
    };
    auto put = [&](const uint4 &x, const uint4 &y, int buf) {
        uint4 *dst = reinterpret_cast<uint4 *>(&s_k[buf][srow * ROWB + spart * 32]);
        dst[0] = x;
        dst[1] = y;
    };
    bool have_prev = false, prev_tail = false;
    int prev_t0 = 0, zb = 0;
    // Second half of a key pass's step: the tile's keys leave shared memory (zsrc: the buffer the step's results
    // were written to).  It runs one step late, after the NEXT step's matrix work, so that one barrier per step serves
    // both the key rows' hand-over and this one (the result tiles are double-buffered).
    auto keys_out = [&](const bool tail, int t0, const float *zsrc) __attribute__((always_inline)) {
        // four consecutive keys of one centroid per thread: maximum over the heads, one 16-byte
        // store where the key rows allow it (whole step in range, row length a multiple of four)
        const bool wide = !tail && ((MODE == MFMA_SAMPLE ? a.sample_stride : a.l_stride) & 3) == 0;
        if constexpr (MODE == MFMA_PICK) {
            // Few keys pass (a few per cent): the verdicts of all of a thread's keys first, then one
            // shared-memory counter bump per (thread, centroid) for the whole group of four, then the stores.
            constexpr int NP = CT * 8 / 256;
            float bv[NP][4];
            uint32_t msk[NP], at[NP];
            const bool inner = !tail && t0 >= a.n_init && t0 + 32 <= s - a.n_local && j0 + CT <= C;
            if (t0 < tend) {
#pragma unroll
                for (int it = 0; it < NP; ++it) {
                    const int p = tid + 256 * it, n4 = (p & 7) * 4, jl = p >> 3;
                    float4 best = *reinterpret_cast<const float4 *>(&zsrc[jl * ZS + n4]);
#pragma unroll
                    for (int c = 1; c < NPL; ++c) {
                        const float4 o = *reinterpret_cast<const float4 *>(&zsrc[(c * CT + jl) * ZS + n4]);
                        best.x = fmaxf(best.x, o.x);
                        best.y = fmaxf(best.y, o.y);
                        best.z = fmaxf(best.z, o.z);
                        best.w = fmaxf(best.w, o.w);
                    }
                    const int t = t0 + n4;
                    bv[it][0] = best.x;
                    bv[it][1] = best.y;
                    bv[it][2] = best.z;
                    bv[it][3] = best.w;
                    // compared as floats: the same verdict as on the ordered images except that -0 passes a
                    // threshold of +0, i.e. at most a candidate too many
                    const float tau = s_tauf[jl];
                    uint32_t m = 0;
                    if (inner) {   // the whole step lies inside the block's range and outside the window, every centroid is real
#pragma unroll
                        for (int e = 0; e < 4; ++e) m |= (uint32_t)(bv[it][e] >= tau) << e;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const bool in = (t + e) < tend && (t + e) >= a.n_init && (t + e) < s - a.n_local && (j0 + jl) < C;
                            m |= (uint32_t)(in && bv[it][e] >= tau) << e;
                        }
                    }
                    msk[it] = m;
                }
#pragma unroll
                for (int it = 0; it < NP; ++it) {
                    at[it] = 0u;
                    if (msk[it]) at[it] = atomicAdd(&s_cnt[(tid + 256 * it) >> 3], (uint32_t)__popc(msk[it]));
                }
#pragma unroll
                for (int it = 0; it < NP; ++it) {
                    if (msk[it]) {
                        const int p = tid + 256 * it, n4 = (p & 7) * 4, jl = p >> 3;
                        uint2 *seg = a.cand + (((size_t)bkl * a.c_max + j0 + jl) * a.t_splits + blockIdx.x) * a.seg_cap;
                        uint32_t w = at[it];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            if ((msk[it] >> e) & 1u) {
                                if (w < (uint32_t)a.seg_cap) seg[w] = make_uint2(ordered_key(bv[it][e]), (uint32_t)(t0 + n4 + e));
                                ++w;
                            }
                        }
                    }
                }
            }
        } else if (t0 < tend) {
            for (int p = tid; p < CT * 8; p += 256) {
                const int n4 = (p & 7) * 4, jl = p >> 3;
                if ((j0 + jl) >= C) continue;
                float4 best = *reinterpret_cast<const float4 *>(&zsrc[jl * ZS + n4]);
#pragma unroll
                for (int c = 1; c < NPL; ++c) {
                    const float4 o = *reinterpret_cast<const float4 *>(&zsrc[(c * CT + jl) * ZS + n4]);
                    best.x = fmaxf(best.x, o.x);
                    best.y = fmaxf(best.y, o.y);
                    best.z = fmaxf(best.z, o.z);
                    best.w = fmaxf(best.w, o.w);
                }
                const int t = t0 + n4;
                uint32_t ok[4] = {ordered_key(best.x), ordered_key(best.y), ordered_key(best.z), ordered_key(best.w)};
                bool win[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    win[e] = (t + e) < a.n_init || (t + e) >= s - a.n_local;
                    if (win[e]) ok[e] = 0x007fffffu;   // the image of -inf
                }
                const size_t unit = (size_t)bkl * a.c_max + j0 + jl;
                {
                    uint32_t *dst = MODE == MFMA_SAMPLE ? a.kbuf + unit * a.sample_stride + (t0 / ST) * 32 + n4
                                                        : a.kbuf + unit * a.l_stride + t;
                    if (wide) {
                        // written once, read much later by other kernels: kept out of the caches that hold the keys
                        u32x4_t v4 = {ok[0], ok[1], ok[2], ok[3]};
                        __builtin_nontemporal_store(v4, reinterpret_cast<u32x4_t *>(dst));
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if ((t + e) < tend) dst[e] = ok[e];
                    }
                }
            }
        }
        };
    // tail: a step whose keys may reach beyond the block's range (a literal at every call).  Such
    // keys are real keys of the sequence, repeated: harmless for a maximum, left out of a sum,
    // not written as ranking keys.
    auto compute = [&](const bool tail, int buf, int t0) __attribute__((always_inline)) {
        bf16x8_t kfrag[8];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            kfrag[ks] = *reinterpret_cast<const bf16x8_t *>(&s_k[buf][col * ROWB + ks * 32 + half * 16]);
        // the two work items' chains interleaved: independent back-to-back matrix instructions
        f32x16_t acc0, acc1;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc0[r] = acc1[r] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfrag[ks], cfrag[0][ks], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfrag[ks], cfrag[1][ks], acc1, 0, 0, 0);
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const f32x16_t &acc = q == 0 ? acc0 : acc1;
            if constexpr (MODE == MFMA_STAT) {
                // the step's maximum first (repeated keys of a tail are real keys: harmless), then its sixteen
                // terms relative to the new running maximum, summed as a tree, and the old sum rescaled
                // (in base two: the scores' maximum as fl(max acc * sc2), monotone since sc2 > 0, and each term
                // 2^(acc * sc2 - m) with one fused multiply-add and the hardware's base-two exponential)
                float am = acc[0];
#pragma unroll
                for (int r = 1; r < 16; r += 2) am = fmaxf(fmaxf(acc[r], r + 1 < 16 ? acc[r + 1] : acc[r]), am);
                const float m = fmaxf(mx[q], am * sc2);
                float e[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    e[r] = __builtin_amdgcn_exp2f(__fmaf_rn(acc[r], sc2, -m));
                    if (tail) e[r] = (t0 + 8 * (r >> 2) + 4 * half + (r & 3)) < tend ? e[r] : 0.0f;
                }
#pragma unroll
                for (int w = 8; w >= 1; w >>= 1)
#pragma unroll
                    for (int r = 0; r < w; ++r) e[r] += e[r + w];
                lsv[q] = __fmaf_rn(lsv[q], __builtin_amdgcn_exp2f(mx[q] - m), e[0]);   // first step: 0 * 2^(-inf) = 0
                mx[q] = m;
            } else if constexpr (G == 1) {   // KEY, SAMPLE, PICK with one head: each item is a sub-tile of its own
                float *zrow = &s_z[zb * (NPL * CT * ZS) + (mt[q] * 32 + col) * ZS + 4 * half];
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    float4 v;
                    v.x = __fmaf_rn(acc[4 * rq + 0], a.scale, off[q]);
                    v.y = __fmaf_rn(acc[4 * rq + 1], a.scale, off[q]);
                    v.z = __fmaf_rn(acc[4 * rq + 2], a.scale, off[q]);
                    v.w = __fmaf_rn(acc[4 * rq + 3], a.scale, off[q]);
                    *reinterpret_cast<float4 *>(zrow + 8 * rq) = v;
                }
            }
        }
        if constexpr (KEYS && G >= 2) {   // the wave's two heads of the same centroids: their maximum, one plane
            float *zrow = &s_z[zb * (NPL * CT * ZS) + ((hh[0] >> 1) * CT + mt[0] * 32 + col) * ZS + 4 * half];
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                float4 v;
                v.x = fmaxf(__fmaf_rn(acc0[4 * rq + 0], a.scale, off[0]), __fmaf_rn(acc1[4 * rq + 0], a.scale, off[1]));
                v.y = fmaxf(__fmaf_rn(acc0[4 * rq + 1], a.scale, off[0]), __fmaf_rn(acc1[4 * rq + 1], a.scale, off[1]));
                v.z = fmaxf(__fmaf_rn(acc0[4 * rq + 2], a.scale, off[0]), __fmaf_rn(acc1[4 * rq + 2], a.scale, off[1]));
                v.w = fmaxf(__fmaf_rn(acc0[4 * rq + 3], a.scale, off[0]), __fmaf_rn(acc1[4 * rq + 3], a.scale, off[1]));
                *reinterpret_cast<float4 *>(zrow + 8 * rq) = v;
            }
        }
        if constexpr (KEYS) {
            if (have_prev) keys_out(prev_tail, prev_t0, s_z + (zb ^ 1) * (NPL * CT * ZS));
            have_prev = true;
            prev_tail = tail;
            prev_t0 = t0;
            zb ^= 1;
        }
    };
    // A step's rows are requested four steps ahead (four register sets).
    {
        uint4 st2a, st2b, st3a, st3b;
        int pg_a = page_at(tbeg + 4 * ST), pg_b = page_at(tbeg + 5 * ST), pg_c = page_at(tbeg + 6 * ST), pg_d = page_at(tbeg + 7 * ST);
        fetch(st0a, st0b, row_from(page_at(tbeg), tbeg));
        fetch(st1a, st1b, row_from(page_at(tbeg + ST), tbeg + ST));
        fetch(st2a, st2b, row_from(page_at(tbeg + 2 * ST), tbeg + 2 * ST));
        fetch(st3a, st3b, row_from(page_at(tbeg + 3 * ST), tbeg + 3 * ST));
        put(st0a, st0b, 0);
        __syncthreads();
        // four steps per trip.  Step i (set i % 4, buffer i % 2): request step i+4 into the set it
        // frees and the entry of step i+8, compute, write step i+1 to the other buffer.
        auto trip = [&](const bool tail, int t0) __attribute__((always_inline)) {
            fetch(st0a, st0b, row_from(pg_a, t0 + 4 * ST));
            pg_a = page_at(t0 + 8 * ST);
            compute(tail, 0, t0);
            put(st1a, st1b, 1);
            __syncthreads();
            fetch(st1a, st1b, row_from(pg_b, t0 + 5 * ST));
            pg_b = page_at(t0 + 9 * ST);
            compute(tail, 1, t0 + ST);
            put(st2a, st2b, 0);
            __syncthreads();
            fetch(st2a, st2b, row_from(pg_c, t0 + 6 * ST));
            pg_c = page_at(t0 + 10 * ST);
            compute(tail, 0, t0 + 2 * ST);
            put(st3a, st3b, 1);
            __syncthreads();
            fetch(st3a, st3b, row_from(pg_d, t0 + 7 * ST));
            pg_d = page_at(t0 + 11 * ST);
            compute(tail, 1, t0 + 3 * ST);
            put(st0a, st0b, 0);
            __syncthreads();
        };
        int t0 = tbeg;
        for (; t0 + 3 * ST + 32 <= tend; t0 += 4 * ST) trip(false, t0);
        if (t0 < tend) trip(true, t0);
    }
    if constexpr (KEYS) {   // the last step's keys (the last trip ended with a barrier)
        if (have_prev) keys_out(prev_tail, prev_t0, s_z + (zb ^ 1) * (NPL * CT * ZS));
    }
    if constexpr (MODE == MFMA_PICK) {
        __syncthreads();
        if (tid < CT && j0 + tid < C) a.seg_cnt[((size_t)bkl * a.c_max + j0 + tid) * a.t_splits + blockIdx.x] = s_cnt[tid];
    }
    if constexpr (KEYS) return;
    // the two halves of a wave hold different keys of the same (centroid, head): merged (the same value
    // on both sides, a sum of two products), then one pair per block
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const bool mine = half == 0 && (j0 + mt[q] * 32 + col) < C;
        const float m_o = __shfl_xor(mx[q], 32), l_o = __shfl_xor(lsv[q], 32);
        const float m = fmaxf(mx[q], m_o);
        const float l = lsv[q] * __builtin_amdgcn_exp2f(mx[q] - m) + l_o * __builtin_amdgcn_exp2f(m_o - m);
        if (mine) a.part[stat[q] * a.t_splits + blockIdx.x] = make_float2(m, l);
    }
}

// ------------------------------------------------------------------------------
// self-check: to_fixed40(exp_series(x)) against exp_fixed40_parts(x) on the fp32 values whose bit
// patterns are first .. first + n - 1; counts the inputs on which they differ.
// ------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void exp_selftest_kernel(uint32_t first, uint32_t n, unsigned long long *bad)
{
    uint32_t mine = 0;
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < n; i += gridDim.x * 256u) {
        const float x = __uint_as_float(first + i);
        uint32_t hi, lo;
        exp_fixed40_parts(x, hi, lo);
        mine += (to_fixed40(exp_series(x)) != (((uint64_t)hi << 24) + lo)) ? 1u : 0u;
    }
    if (mine) atomicAdd(bad, (unsigned long long)mine);
}

// ------------------------------------------------------------------------------
// softmax denominators: S[h] += sum_i floor(exp(z[h][i] - m[h]) * 2^40), integer
// adds, hence the same value in any order.  grid (nbx, units), 256 threads, each
// block walks chunks of 1024 ids with stride gridDim.x.
// ------------------------------------------------------------------------------
struct DenomArgs {
    Units u;
    const int32_t *ctx_lens, *ncand;   // ncand == nullptr => L = ctx_len
    int l_stride;
    const float *z;
    const uint32_t *m_key;
    unsigned long long *S;
    uint32_t *gbits;          // decode only: the recall bitmap, cleared here for the next step
    int bitmap_words;
    int by_xcd;               // blocks -> (unit, block of the unit) by unit_block_of
    uint32_t *gcur;           // optional: [units] list cursors of keyclass_kernel, cleared here
};

template <int G> __global__ __launch_bounds__(256) void denom_kernel(DenomArgs a)
{
    int b, kv, j;
    int ul, bx;
    unit_block_of(a.by_xcd, ul, bx);
    if (!decode_unit(a.u, ul, b, kv, j)) return;
    // everything the block needs to know is requested at once (the maxima before L decides whether
    // the block has work: one round trip instead of three)
    uint32_t mk[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) mk[hh] = a.m_key[ul * G + hh];
    const int s_len = a.ctx_lens[b];
    const int L = a.ncand ? a.ncand[ul] : s_len;
    if (a.gcur && bx == 0 && threadIdx.x == 0) a.gcur[ul] = 0u;
    if (a.gbits) {
        const int W = (s_len + 31) >> 5;
        for (int w = bx * 256 + threadIdx.x; w < W; w += gridDim.x * 256) a.gbits[(size_t)ul * a.bitmap_words + w] = 0u;
    }
    if (bx * 1024 >= L) return;
    const int tid = threadIdx.x;
    __shared__ unsigned long long s_acc[4][G];
    float m[G];
    unsigned long long acc[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        m[hh] = ordered_value(mk[hh]);
        acc[hh] = 0ull;
    }
    const float *zb = a.z + (size_t)ul * a.l_stride * G;
    for (int c0 = bx * 1024; c0 < L; c0 += gridDim.x * 1024) {
        // four terms per head as 32-bit partial sums (hi < 2^17, lo < 2^24 each), then one 64-bit add
        uint32_t shi[G], slo[G];
#pragma unroll
        for (int hh = 0; hh < G; ++hh) shi[hh] = slo[hh] = 0u;
        // the four loads first (ids beyond L read entry L-1 and are left out below): taken one at a
        // time, each would be waited for before the next is requested
        float zv[4][G];
#pragma unroll
        for (int q = 0; q < 4; ++q) load_z<G>(zb, min(c0 + q * 256 + tid, L - 1), zv[q]);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const bool ok = (c0 + q * 256 + tid) < L;
#pragma unroll
            for (int hh = 0; hh < G; ++hh) {
                uint32_t hi, lo;
                exp_fixed40_parts(zv[q][hh] - m[hh], hi, lo);
                shi[hh] += ok ? hi : 0u;
                slo[hh] += ok ? lo : 0u;
            }
        }
#pragma unroll
        for (int hh = 0; hh < G; ++hh) acc[hh] += ((unsigned long long)shi[hh] << 24) + slo[hh];
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
// ranking keys, chip-wide: key_i = max_h ((z[h][i] - m[h]) - log S[h]) as an ordered
// uint32 into kbuf, and the unit's histogram of key_bucket() (shared-memory
// histogram per block, non-empty buckets added to the global one: integer adds).
// grid (nbx, units), 1024 threads, chunks of 4096 ids with stride gridDim.x.
// ------------------------------------------------------------------------------
struct KeyArgs {
    Units u;
    const int32_t *ctx_lens, *ncand;   // ncand == nullptr => L = ctx_len
    int l_stride;
    const float *z;     // nullptr: kbuf holds the keys already, only their histogram is taken
    const uint32_t *m_key;
    const unsigned long long *S;
    uint32_t *kbuf;     // [units][l_stride]
    uint32_t *ghist;    // [units][kBuckets], zero on entry
    uint32_t *gcur;     // decode only: [units] list cursors of classify_kernel, cleared here
    int n_init, n_local;   // build only: ids below n_init or from L - n_local on are never listed
    int by_xcd;              // blocks -> (unit, block of the unit) by unit_block_of
};

template <int G> __global__ __launch_bounds__(1024) void keyhist_kernel(KeyArgs a)
{
    int b, kv, j;
    int ul, bx;
    unit_block_of(a.by_xcd, ul, bx);
    if (!decode_unit(a.u, ul, b, kv, j)) return;
    const int tid = threadIdx.x;
    // the unit's statistics are requested together with L, before L decides whether the block has work
    uint32_t mk[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) mk[hh] = a.z ? a.m_key[ul * G + hh] : 0u;
    const unsigned long long S_mine = (a.z && tid < G) ? a.S[ul * G + tid] : 1ull;
    const int L = a.ncand ? a.ncand[ul] : a.ctx_lens[b];
    if (a.gcur && bx == 0 && threadIdx.x == 0) a.gcur[ul] = 0u;
    if (bx * 4096 >= L) return;
    __shared__ uint32_t s_h[kBuckets];
    __shared__ float s_ls[G];
    for (int w = tid; w < kBuckets; w += 1024) s_h[w] = 0u;
    if (tid < G) s_ls[tid] = a.z ? (float)log_fixed40(S_mine) : 0.0f;
    float m[G], ls[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) m[hh] = a.z ? ordered_value(mk[hh]) : 0.0f;
    __syncthreads();
#pragma unroll
    for (int hh = 0; hh < G; ++hh) ls[hh] = s_ls[hh];
    const float *zb = a.z + (size_t)ul * a.l_stride * G;
    uint32_t *kb = a.kbuf + (size_t)ul * a.l_stride;
    if (!a.z) {   // the keys are there already (matrix-core build): histogram only, four keys per load
        const bool wide = (reinterpret_cast<uintptr_t>(kb) & 15u) == 0;
        // The last bucket takes every key below the histogram's range, often most of them: its
        // count is taken per wave with a ballot (64 lanes adding to one word would be served
        // one after the other); the other buckets are added to directly.
        auto count4 = [&](const uint32_t(&k4)[4], int i) __attribute__((always_inline)) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool valid = i + e < L;
                const uint32_t bk = key_bucket(k4[e]);
                const bool tail = valid && bk == (uint32_t)(kBuckets - 1);
                const uint64_t mt = __ballot(tail);
                if (valid && !tail) atomicAdd(&s_h[bk], 1u);
                if (mt && lane_id() == 0) atomicAdd(&s_h[kBuckets - 1], (uint32_t)__popcll(mt));
            }
        };
        // four chunks of 4096 keys per trip; when all four lie wholly below L their loads are plain
        // and go out together
        const int stride = gridDim.x * 4096;
        for (int c0 = bx * 4096; c0 < L; c0 += 4 * stride) {
            if (wide && c0 + 3 * stride + 4096 <= L) {
                uint4 v[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) v[q] = *reinterpret_cast<const uint4 *>(kb + c0 + q * stride + 4 * tid);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t k4[4] = {v[q].x, v[q].y, v[q].z, v[q].w};
                    count4(k4, c0 + q * stride + 4 * tid);
                }
            } else {
                for (int q = 0; q < 4; ++q) {
                    const int cq = c0 + q * stride;
                    if (cq >= L) break;   // uniform
                    const int i = cq + 4 * tid;
                    uint32_t k4[4] = {0u, 0u, 0u, 0u};
                    if (wide && i + 3 < L) {
                        const uint4 v = *reinterpret_cast<const uint4 *>(kb + i);
                        k4[0] = v.x; k4[1] = v.y; k4[2] = v.z; k4[3] = v.w;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (i + e < L) k4[e] = kb[i + e];
                    }
                    count4(k4, i);
                }
            }
        }
    }
    for (int c0 = bx * 4096; a.z && c0 < L; c0 += gridDim.x * 4096) {
        // the four loads first (ids beyond L read entry L-1 and are dropped): see denom_kernel
        float zv[4][G];
#pragma unroll
        for (int q = 0; q < 4; ++q) load_z<G>(zb, min(c0 + q * 1024 + tid, L - 1), zv[q]);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int i = c0 + q * 1024 + tid;
            const bool valid = i < L;
            float best = -__builtin_huge_valf();
#pragma unroll
            for (int hh = 0; hh < G; ++hh) best = fmaxf(best, (zv[q][hh] - m[hh]) - ls[hh]);
            uint32_t ok = ordered_key(best);
            // keys of the resident window rank below every other key (the image of -inf)
            if (i < a.n_init || i >= L - a.n_local) ok = 0x007fffffu;
            if (valid) kb[i] = ok;
            const uint32_t bk = key_bucket(ok);
            const bool tail = valid && bk == (uint32_t)(kBuckets - 1);   // counted per wave, as above
            const uint64_t mt = __ballot(tail);
            if (valid && !tail) atomicAdd(&s_h[bk], 1u);
            if (mt && lane_id() == 0) atomicAdd(&s_h[kBuckets - 1], (uint32_t)__popcll(mt));
        }
    }
    __syncthreads();
    uint32_t *gh = a.ghist + (size_t)ul * kBuckets;
    for (int w = tid; w < kBuckets; w += 1024) {
        uint32_t v = s_h[w];
        if (v) atomicAdd(&gh[w], v);
    }
}

// ------------------------------------------------------------------------------
// Algorithm 2 line 6, the pass over the ranking keys, spread over the chip (decode).  Every block
// scans its unit's key histogram for the bucket that holds the top_k-th key, then walks its share
// of the ids in groups of 64: ids in higher buckets go into a bitmap (one ballot per group, plain
// stores), the (key, id) pairs of the deciding bucket are appended to the unit's list (one
// cursor bump per wave; the order of the list is arbitrary and nothing depends on it).
// Units with top_k >= L, or with more than kListCap keys in the deciding bucket, are left to the
// select kernel.  grid (nbx, units), 256 threads; keyhist_kernel has cleared the cursors.
// ------------------------------------------------------------------------------
struct ClassifyArgs {
    Units u;
    const int32_t *ctx_lens, *ncand;
    int l_stride, top_k;
    const uint32_t *kbuf;    // [units][l_stride]
    const uint32_t *ghist;   // [units][kBuckets]
    int bits_stride;         // bitmap words per unit
    uint32_t *gbm;           // [units][bits_stride] ids above the deciding bucket
    uint2 *glist;            // [units][kListCap] (key, id) of the deciding bucket
    uint32_t *gcur;          // [units] list cursor, zero on entry
    uint32_t *ginfo;         // [units][4] deciding bucket, keys wanted from it, its population, unused
    int by_xcd;              // blocks -> (unit, block of the unit) by unit_block_of
};

__global__ __launch_bounds__(256) void classify_kernel(ClassifyArgs a)
{
    int b, kv, j;
    int ul, bx;
    unit_block_of(a.by_xcd, ul, bx);
    if (!decode_unit(a.u, ul, b, kv, j)) return;
    const int L = a.ncand ? a.ncand[ul] : a.ctx_lens[b];
    if (a.top_k >= L) return;
    __shared__ uint32_t s_scan[8];
    __shared__ uint32_t s_res[3];
    const int tid = threadIdx.x, ln = lane_id();
    const int nw64 = (L + 63) >> 6;
    const int wg = bx * 4 + (tid >> 6), nwg = gridDim.x * 4;
    const uint32_t *kb = a.kbuf + (size_t)ul * a.l_stride;
    constexpr int UNR = 4;
    // this wave's first groups of keys are requested before the histogram is looked at
    uint32_t kk[UNR];
#pragma unroll
    for (int q = 0; q < UNR; ++q) {
        int i = (wg + q * nwg) * 64 + ln;
        kk[q] = (i < L) ? kb[i] : 0u;
    }
    // thread t owns buckets BPT*t .. BPT*t + BPT-1, in descending key order
    constexpr int BPT = kBuckets / 256;
    static_assert(BPT % 4 == 0, "bucket counts are read as uint4");
    uint32_t c[BPT];
    {
        const uint4 *gh = reinterpret_cast<const uint4 *>(a.ghist + (size_t)ul * kBuckets) + (BPT / 4) * tid;
#pragma unroll
        for (int q = 0; q < BPT / 4; ++q) {
            uint4 v = gh[q];
            c[4 * q] = v.x; c[4 * q + 1] = v.y; c[4 * q + 2] = v.z; c[4 * q + 3] = v.w;
        }
    }
    uint32_t mine = 0;
#pragma unroll
    for (int q = 0; q < BPT; ++q) mine += c[q];
    uint32_t tot;
    uint32_t before = block_excl_scan<256>(mine, s_scan, &tot);
#pragma unroll
    for (int q = 0; q < BPT; ++q) {
        if (before < (uint32_t)a.top_k && (uint32_t)a.top_k <= before + c[q]) {
            s_res[0] = (uint32_t)(BPT * tid + q);
            s_res[1] = (uint32_t)a.top_k - before;
            s_res[2] = c[q];
        }
        before += c[q];
    }
    __syncthreads();
    const uint32_t bkt = s_res[0], nb = s_res[2];
    if (bx == 0 && tid == 0)
        *reinterpret_cast<uint4 *>(a.ginfo + 4 * (size_t)ul) = make_uint4(bkt, s_res[1], nb, 0u);
    if (nb > (uint32_t)kListCap) return;
    uint32_t *bm = a.gbm + (size_t)ul * a.bits_stride;
    uint2 *lst = a.glist + (size_t)ul * kListCap;
    const uint64_t below = (1ull << ln) - 1ull;
    for (int g0 = wg; g0 < nw64; g0 += UNR * nwg) {
        if (g0 != wg) {
#pragma unroll
            for (int q = 0; q < UNR; ++q) {
                int i = (g0 + q * nwg) * 64 + ln;
                kk[q] = (i < L) ? kb[i] : 0u;
            }
        }
#pragma unroll
        for (int q = 0; q < UNR; ++q) {
            const int gq = g0 + q * nwg;
            if (gq < nw64) {
                const int i = gq * 64 + ln;
                const bool valid = i < L;
                const uint32_t bk = key_bucket(kk[q]);
                const bool inb = valid && bk == bkt;
                const uint64_t above = __ballot(valid && bk < bkt);
                const uint64_t listed = __ballot(inb);
                if (ln == 0) *reinterpret_cast<uint2 *>(bm + 2 * gq) = make_uint2((uint32_t)above, (uint32_t)(above >> 32));
                if (listed) {
                    uint32_t at0 = 0;
                    if (ln == 0) at0 = atomicAdd(&a.gcur[ul], (uint32_t)__popcll(listed));
                    at0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)at0);
                    if (inb) lst[at0 + (uint32_t)__popcll(listed & below)] = make_uint2(kk[q], (uint32_t)i);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------
// keyhist_kernel and classify_kernel as ONE launch, for small batches (decode).  The histogram of a unit's
// keys is needed whole before any key can be classified; here every block of the unit takes it itself, over
// ALL the unit's ids (the same few thousand scores read by each of its blocks, from the cache; the histogram
// stays in shared memory), finds the deciding bucket, and then writes and classifies the keys of its own share
// as classify_kernel does.  One launch and one round trip fewer, for work that is repeated per block: only
// where that work is small (the host's choice).  grid (nbx, units), 1024 threads; denom_kernel has cleared the
// list cursors.  No 2048-bucket histogram is left in global memory.
// ------------------------------------------------------------------------------
struct KeyClassArgs {
    Units u;
    const int32_t *ctx_lens, *ncand;
    int l_stride, top_k;
    const float *z;
    const uint32_t *m_key;
    const unsigned long long *S;
    uint32_t *kbuf;          // [units][l_stride]
    int bits_stride;
    uint32_t *gbm;           // [units][bits_stride]
    uint2 *glist;            // [units][kListCap]
    uint32_t *gcur;          // [units], zero on entry
    uint32_t *ginfo;         // [units][4]
    int by_xcd;              // blocks -> (unit, block of the unit) by unit_block_of
};

template <int G> __global__ __launch_bounds__(1024) void keyclass_kernel(KeyClassArgs a)
{
    int b, kv, j;
    int ul, bx;
    unit_block_of(a.by_xcd, ul, bx);
    if (!decode_unit(a.u, ul, b, kv, j)) return;
    const int tid = threadIdx.x, wv = tid >> 6, ln = lane_id();
    uint32_t mk[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) mk[hh] = a.m_key[ul * G + hh];
    const unsigned long long S_mine = tid < G ? a.S[ul * G + tid] : 1ull;
    const int L = a.ncand ? a.ncand[ul] : a.ctx_lens[b];
    __shared__ uint32_t s_h[kBuckets];
    __shared__ float s_ls[G];
    __shared__ uint32_t s_scan[1024 / 64 + 2];
    __shared__ uint32_t s_res[3];
    for (int w = tid; w < kBuckets; w += 1024) s_h[w] = 0u;
    if (tid < G) s_ls[tid] = (float)log_fixed40(S_mine);
    if (tid == 0) s_res[2] = 0xffffffffu;
    float m[G], ls[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) m[hh] = ordered_value(mk[hh]);
    __syncthreads();
#pragma unroll
    for (int hh = 0; hh < G; ++hh) ls[hh] = s_ls[hh];
    const float *zb = a.z + (size_t)ul * a.l_stride * G;
    auto key_of = [&](const float(&zv)[G]) __attribute__((always_inline)) {
        float best = -__builtin_huge_valf();
#pragma unroll
        for (int hh = 0; hh < G; ++hh) best = fmaxf(best, (zv[hh] - m[hh]) - ls[hh]);
        return ordered_key(best);
    };
    const bool rank = a.top_k < L;   // otherwise every recalled key is kept and nothing needs classifying
    // pass 1: the histogram of ALL the unit's keys (the last bucket, which takes every key below the range, counted
    // per wave with a ballot)
    for (int c0 = 0; rank && c0 < L; c0 += 4096) {
        float zv[4][G];
#pragma unroll
        for (int q = 0; q < 4; ++q) load_z<G>(zb, min(c0 + q * 1024 + tid, L - 1), zv[q]);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const bool valid = c0 + q * 1024 + tid < L;
            const uint32_t bk = key_bucket(key_of(zv[q]));
            const bool tail = valid && bk == (uint32_t)(kBuckets - 1);
            const uint64_t mt = __ballot(tail);
            if (valid && !tail) atomicAdd(&s_h[bk], 1u);
            if (mt && ln == 0) atomicAdd(&s_h[kBuckets - 1], (uint32_t)__popcll(mt));
        }
    }
    __syncthreads();
    uint32_t bkt = 0, nb = 0xffffffffu;
    if (rank) {
        // thread t owns buckets 2t, 2t+1, in descending key order
        constexpr int BPT = kBuckets / 1024;
        uint32_t c[BPT], mine = 0;
#pragma unroll
        for (int q = 0; q < BPT; ++q) {
            c[q] = s_h[BPT * tid + q];
            mine += c[q];
        }
        uint32_t tot;
        uint32_t before = block_excl_scan<1024>(mine, s_scan, &tot);
#pragma unroll
        for (int q = 0; q < BPT; ++q) {
            if (before < (uint32_t)a.top_k && (uint32_t)a.top_k <= before + c[q]) {
                s_res[0] = (uint32_t)(BPT * tid + q);
                s_res[1] = (uint32_t)a.top_k - before;
                s_res[2] = c[q];
            }
            before += c[q];
        }
        __syncthreads();
        bkt = s_res[0];
        nb = s_res[2];
        if (bx == 0 && tid == 0) *reinterpret_cast<uint4 *>(a.ginfo + 4 * (size_t)ul) = make_uint4(bkt, s_res[1], nb, 0u);
    }
    const bool classify = rank && nb <= (uint32_t)kListCap;
    // pass 2: this block's share of the ids in groups of 64: keys written, and classified against the deciding bucket
    uint32_t *kb = a.kbuf + (size_t)ul * a.l_stride;
    uint32_t *bm = a.gbm + (size_t)ul * a.bits_stride;
    uint2 *lst = a.glist + (size_t)ul * kListCap;
    const uint64_t below = (1ull << ln) - 1ull;
    const int nw64 = (L + 63) >> 6;
    for (int g0 = bx * 16 + wv; g0 < nw64; g0 += gridDim.x * 16) {
        const int i = g0 * 64 + ln;
        const bool valid = i < L;
        float zv[G];
        load_z<G>(zb, min(i, L - 1), zv);
        const uint32_t ok = key_of(zv);
        if (valid) kb[i] = ok;
        if (classify) {
            const uint32_t bk = key_bucket(ok);
            const bool inb = valid && bk == bkt;
            const uint64_t above = __ballot(valid && bk < bkt);
            const uint64_t listed = __ballot(inb);
            if (ln == 0) *reinterpret_cast<uint2 *>(bm + 2 * g0) = make_uint2((uint32_t)above, (uint32_t)(above >> 32));
            if (listed) {
                uint32_t at0 = 0;
                if (ln == 0) at0 = atomicAdd(&a.gcur[ul], (uint32_t)__popcll(listed));
                at0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)at0);
                if (inb) lst[at0 + (uint32_t)__popcll(listed & below)] = make_uint2(ok, (uint32_t)i);
            }
        }
    }
}

// ------------------------------------------------------------------------------
// Algorithm 2 line 6 / Algorithm 1 line 4.  One block of 1024 threads per unit: the
// top-k ids by ranking key (kbuf), ascending, helped by the key histogram.
//   decode: sel[unit][pos] = cand[i], srow[unit][pos] = crow[i],
//           zsel[unit][pos][G] = z[i][G], nsel[unit]
//   build : lists[(b*g+kv)*c_max + j][pos] = i
// Dynamic shared memory: kSelLds + 2*kListCap + bits_words + top_k words (the last: positions of
// the picked ids, decode only).
// ------------------------------------------------------------------------------
struct SelectArgs {
    Units u;
    const int32_t *ctx_lens, *ncand, *cand;
    const uint32_t *crow;
    int l_stride, top_k;
    int bits_words;          // shared-memory words set aside for the two id bitmaps (0: none)
    const float *z;
    const uint32_t *m_key;
    const uint32_t *kbuf;    // [units][l_stride] ranking keys (keyhist_kernel)
    const uint32_t *ghist;   // [units][kBuckets] their histogram
    const uint32_t *gbm;     // decode: classify_kernel's outputs (nullptr: the block makes the pass itself)
    const uint2 *glist;
    const uint32_t *ginfo;
    int bits_stride;
    int32_t *sel;       // decode [units][top_k] ; build: lists base
    uint32_t *srow;     // decode [units][top_k]
    float *zsel;        // decode [units][top_k][G]
    int32_t *nsel;      // decode [units]
    int32_t *out_sel;   // optional copy for the caller
    int ids_only;       // decode: write sel and nsel only (the dynamic centroid update's second ranking)
};

// writes the decode outputs of one unit from the positions picked into s_idx[0..n)
template <int G>
__device__ __forceinline__ void select_gather(const SelectArgs &a, int ul, int n, const float *zb, const int32_t *s_idx)
{
    const int tid = threadIdx.x;
    const int32_t *cb = a.cand + (size_t)ul * a.l_stride;
    int32_t *dst = a.sel + (size_t)ul * a.top_k;
    if (a.ids_only) {
        for (int pos = tid; pos < a.top_k; pos += 1024) dst[pos] = pos < n ? cb[s_idx[pos]] : -1;
        if (tid == 0) a.nsel[ul] = n;
        return;
    }
    const uint32_t *rb = a.crow + (size_t)ul * a.l_stride;
    uint32_t *dstr = a.srow + (size_t)ul * a.top_k;
    int32_t *dst2 = a.out_sel ? a.out_sel + (size_t)ul * a.top_k : nullptr;
    float *zd = a.zsel + (size_t)ul * a.top_k * G;
#pragma unroll 2
    for (int pos = tid; pos < a.top_k; pos += 1024) {
        if (pos < n) {
            int i = s_idx[pos];
            int t = cb[i];
            uint32_t r = rb[i];
            float zv[G];
            load_z<G>(zb, i, zv);
            dst[pos] = t;
            dstr[pos] = r;
            if (dst2) dst2[pos] = t;
            store_z<G>(zd, pos, zv);
        } else {
            dst[pos] = -1;
            if (dst2) dst2[pos] = -1;
        }
    }
    if (tid == 0) a.nsel[ul] = n;
}

template <int KPT, typename KeyFn, typename EmitFn>
__device__ __forceinline__ int select_generic(KeyFn key, int L, int k, EmitFn emit, uint32_t *s_sel)
{
    return block_select_topk<1024, KPT>(key, L, k, emit, s_sel);
}

// Shared-memory words of the selection: radix scratch, the deciding bucket's list, the two id
// bitmaps, then the positions of the picks (decode).
__device__ __forceinline__ int select_smem_words(int bits_words, int top_k) { return kSelLds + 2 * kListCap + bits_words + top_k; }

// The selection of one unit: positions (decode: into s_idx, ascending; build: ids straight into
// the list) of the top_k ranking keys among L.  Returns their number.  Every thread of the
// 1024-thread block takes part.
template <int G> __device__ __forceinline__ int select_unit(const SelectArgs &a, int ul, int L, uint32_t *smem)
{
    uint32_t *s_sel = smem;                          // kSelLds
    uint32_t *s_list = smem + kSelLds;               // 2 * kListCap
    uint32_t *s_bits = s_list + 2 * kListCap;        // a.bits_words (two bitmaps over the ids)
    int32_t *s_idx = (int32_t *)(s_bits + a.bits_words);   // top_k (decode)
    const uint32_t *kb = a.kbuf + (size_t)ul * a.l_stride;
    auto key = [&](int i) { return kb[i]; };
    int32_t *lst = a.u.build ? a.sel + (size_t)(a.u.unit0 + ul) * a.top_k : nullptr;
    auto emit = [&](int pos, int i) {
        if (lst)
            lst[pos] = i;
        else
            s_idx[pos] = i;
    };
    int n = -1;
    if (a.top_k >= L) {
        for (int i = threadIdx.x; i < L; i += 1024) emit(i, i);
        n = L;
    } else if (4 * ((L + 63) >> 6) <= a.bits_words) {
        if (a.ginfo) {
            const uint4 info = *reinterpret_cast<const uint4 *>(a.ginfo + 4 * (size_t)ul);
            if (info.z <= (uint32_t)kListCap)
                n = block_select_classified<1024>(L, a.top_k, info.y, info.z, a.gbm + (size_t)ul * a.bits_stride,
                                                  a.glist + (size_t)ul * kListCap, emit, s_sel, s_bits, s_list);
        } else {
            n = block_select_hist<1024>(kb, L, a.top_k, emit, s_sel, s_bits, s_list, a.ghist + (size_t)ul * kBuckets);
        }
    }
    if (n < 0) {   // crowded deciding bucket (or no room for the bitmaps): the histogram-free route
        if (L <= 1024 * 8)
            n = select_generic<8>(key, L, a.top_k, emit, s_sel);
        else if (L <= 1024 * 32)
            n = select_generic<32>(key, L, a.top_k, emit, s_sel);
        else
            n = select_generic<0>(key, L, a.top_k, emit, s_sel);
    }
    return n;
}

template <int G> __global__ __launch_bounds__(1024) void rerank_select_kernel(SelectArgs a)
{
    extern __shared__ __align__(16) uint32_t smem[];
    int b, kv, j;
    const int ul = blockIdx.x;
    if (!decode_unit(a.u, ul, b, kv, j)) return;
    const int L = a.cand ? a.ncand[ul] : a.ctx_lens[b];
    CTKVR_STAMP(28);
    CTKVR_STAMP_BLK(2);
    const int n = select_unit<G>(a, ul, L, smem);
    if (!a.u.build) {
        __syncthreads();
        select_gather<G>(a, ul, n, a.z + (size_t)ul * a.l_stride * G,
                         (const int32_t *)(smem + kSelLds + 2 * kListCap + a.bits_words));
    }
    CTKVR_STAMP(31);
    CTKVR_STAMP_BLK(3);
}

// ------------------------------------------------------------------------------
// Matrix-core list build, candidate route (Algorithm 1 line 4 on a few thousand candidates per unit
// instead of all s keys).
// sample_threshold_kernel: tau[unit] = the r-th largest of the unit's sampled keys (slot i of the sample
// row is key id (i / 32) * 32 * step_stride + i % 32; slots of ids beyond s or inside the resident window
// do not count), with r = 2 ceil(rho / step_stride) + 16: about 2 rho + 16 step_stride of the unit's keys
// then lie at or above tau.  Fewer samples than r: tau = 0, every key is a candidate (and the unit
// overflows, see below).
// cand_select_kernel: the rho largest of the unit's candidates (key, id), gathered from the segments the
// blocks of the PICK pass filled, ties to the lowest id, written to the unit's list in ascending id order.
// A unit with fewer than rho candidates, more than cand_cap, or a segment that ran over, raises *fail instead
// (the caller then redoes the chunk by the route that keeps every key).
// Both: grid = chunk units, 1024 threads.  cand_select: dynamic shared memory 2112 + 2 cand_cap + kCandTies +
// ceil(s_max / 32) words (one bitmap over the ids; the candidates that tie with the rho-th key, normally one, are
// sorted out in a short list: more than kCandTies of them also raise *fail); cand_cap <= kCandCap.
// ------------------------------------------------------------------------------
constexpr int kCandCap = 8192;
constexpr int kSampleCap = 8192;   // sampled keys per unit at most

struct CandArgs {
    Units u;
    const int32_t *ctx_lens;
    int rho, step_stride, sample_stride, cand_cap;
    int n_init, n_local;
    const uint32_t *ksamp;    // [chunk units][sample_stride]
    uint32_t *tau;            // [chunk units]
    const uint2 *cand;        // [chunk units][t_splits][seg_cap]
    const uint32_t *seg_cnt;  // [chunk units][t_splits], zero where no block wrote
    int t_splits, seg_cap;
    int32_t *lists;           // [all units][rho]
    uint32_t *fail;           // [1]
};

__global__ __launch_bounds__(1024) void sample_threshold_kernel(CandArgs a)
{
    __shared__ uint32_t s_hist[2048 + 64];
    __shared__ uint32_t s_cnt;
    int b, kv, j;
    const int ul = blockIdx.x, tid = threadIdx.x;
    if (!decode_unit(a.u, ul, b, kv, j)) return;
    const int s = a.ctx_lens[b];
    const int ST = 32 * a.step_stride;
    const int n = ((s + ST - 1) / ST) * 32;   // sample slots of this unit (the last step's may reach beyond s)
    const uint32_t *ks = a.ksamp + (size_t)ul * a.sample_stride;
    if (tid == 0) s_cnt = 0u;
    constexpr int KPT = kSampleCap / 1024;
    uint32_t kreg[KPT];
    uint32_t mine = 0;
#pragma unroll
    for (int q = 0; q < KPT; ++q) {
        const int i = q * 1024 + tid;
        const int t = (i >> 5) * ST + (i & 31);
        const bool valid = i < n && t < s - a.n_local && t >= a.n_init;
        kreg[q] = ks[min(i, n - 1)];
        if (!valid) kreg[q] = 0u;   // below the image of every real key
        mine += valid;
    }
    __syncthreads();
    mine = wave_sum_uniform(mine);
    if ((tid & 63) == 0 && mine) atomicAdd(&s_cnt, mine);
    __syncthreads();
    const uint32_t n_valid = s_cnt;
    const uint32_t r = 2u * (uint32_t)((a.rho + a.step_stride - 1) / a.step_stride) + 16u;
    if (r > n_valid) {   // uniform
        if (tid == 0) a.tau[ul] = 0u;
        return;
    }
    auto for_slots = [&](auto f) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < KPT; ++q) f(q * 1024 + tid, kreg[q] != 0u, kreg[q]);
    };
    uint32_t T, need_eq;
    block_kth_largest<1024>(for_slots, r, s_hist, T, need_eq);
    if (tid == 0) a.tau[ul] = T;
}

constexpr int kCandTies = 256;   // candidates equal to the rho-th key that cand_select_kernel sorts out itself

__global__ __launch_bounds__(1024) void cand_select_kernel(CandArgs a)
{
    extern __shared__ __align__(16) uint32_t smem[];
    int b, kv, j;
    const int ul = blockIdx.x, tid = threadIdx.x;
    if (!decode_unit(a.u, ul, b, kv, j)) return;
    const int s = a.ctx_lens[b];
    // the unit's candidates, segment after segment (every thread walks the few counts itself)
    uint32_t n = 0;
    bool bad = false;
    for (int x = 0; x < a.t_splits; ++x) {
        const uint32_t c = a.seg_cnt[(size_t)ul * a.t_splits + x];
        bad |= c > (uint32_t)a.seg_cap;
        n += c;
    }
    if (bad || n < (uint32_t)a.rho || n > (uint32_t)a.cand_cap) {   // uniform
        if (tid == 0) atomicOr(a.fail, 1u);
        return;
    }
    uint32_t *s_hist = smem;                                   // 2048 + 64
    uint2 *l_ent = reinterpret_cast<uint2 *>(smem + 2112);     // cand_cap entries
    uint32_t *s_ties = smem + 2112 + 2 * a.cand_cap;           // ids of the candidates equal to the rho-th key
    uint32_t *s_bm = s_ties + kCandTies;                       // one bitmap over the ids
    const int nw = (s + 31) >> 5;
    uint32_t *s_x = s_hist + 2048 + 56;                        // [1]: tie cursor (free once the threshold is known)
    {
        uint32_t at = 0;
        for (int x = 0; x < a.t_splits; ++x) {
            const uint32_t c = a.seg_cnt[(size_t)ul * a.t_splits + x];
            const uint2 *src = a.cand + ((size_t)ul * a.t_splits + x) * a.seg_cap;
            for (uint32_t e = tid; e < c; e += 1024) l_ent[at + e] = src[e];
            at += c;
        }
    }
    for (int w = tid; w < nw; w += 1024) s_bm[w] = 0u;
    __syncthreads();
    // T = the rho-th largest key, need_eq = how many of the candidates equal to T belong to the rho largest
    uint32_t T, need_eq;
    block_list_threshold<1024, kCandCap>(n, (uint32_t)a.rho, s_hist, l_ent, T, need_eq);
    __syncthreads();
    if (tid == 0) s_x[1] = 0u;
    __syncthreads();
    for (uint32_t e = tid; e < n; e += 1024) {
        const uint2 en = l_ent[e];
        if (en.x > T) atomicOr(&s_bm[en.y >> 5], 1u << (en.y & 31u));
        if (en.x == T) {
            const uint32_t at = atomicAdd(&s_x[1], 1u);
            if (at < (uint32_t)kCandTies) s_ties[at] = en.y;
        }
    }
    __syncthreads();
    const uint32_t n_eq = s_x[1];
    if (n_eq > (uint32_t)kCandTies) {   // uniform: more exact ties at the threshold than are sorted out here
        if (tid == 0) atomicOr(a.fail, 1u);
        return;
    }
    // the need_eq lowest ids among the ties join the bitmap
    if ((uint32_t)tid < n_eq) {
        const uint32_t mine = s_ties[tid];
        uint32_t lower = 0;
        for (uint32_t e = 0; e < n_eq; ++e) lower += s_ties[e] < mine;
        if (lower < need_eq) atomicOr(&s_bm[mine >> 5], 1u << (mine & 31u));
    }
    __syncthreads();
    // thread t owns words [t wpt, (t + 1) wpt) of the bitmap: count, scan, emit in ascending id order
    uint32_t *s_scan = s_hist + 2048 + 4;
    const int wpt = (nw + 1023) / 1024;
    const int w0 = min(nw, tid * wpt), w1 = min(nw, w0 + wpt);
    uint32_t cnt = 0;
    for (int w = w0; w < w1; ++w) cnt += (uint32_t)__popc(s_bm[w]);
    uint32_t tot;
    uint32_t pos = block_excl_scan<1024>(cnt, s_scan, &tot);
    int32_t *lst = a.lists + (size_t)(a.u.unit0 + ul) * a.rho;
    for (int w = w0; w < w1; ++w) {
        uint32_t m = s_bm[w];
        while (m) {
            const int bpos = __ffs((int)m) - 1;
            m &= m - 1u;
            lst[pos++] = w * 32 + bpos;
        }
    }
}

// ------------------------------------------------------------------------------
// Algorithm 2 lines 7-9: o_h = softmax(z_sel[h]) . V_sel.  grid SL*batch*g, 1024
// threads, SL = 4 or 8 slices: block x owns head dimensions (128/SL) x .. of all G heads of its
// (sequence, KV head), so no partial result crosses a block.  16/SL lanes share a
// row (8 dimensions each; lanes 64 SL/16 apart in a wave), 64 SL rows per pass.  Dynamic shared memory:
// top_k*G floats (softmax weights of the two-pass fallback).
// ------------------------------------------------------------------------------
struct AttnArgs {
    const void *v_pages;
    int g, h, top_k;
    const uint32_t *srow;
    const int32_t *nsel;
    const float *zsel;
    float *out;  // [batch*h][128]
    float *out_lse;
    const float *win;   // optional: window_attn_kernel's partial results, [units][kWinSplit][G][2 + 128]
    const uint32_t *m_key;   // [units][G] ordered-key maxima of the logits over all recalled keys
};


// out element `dim` of head hh of a unit: the sparse part (v = sum of exp(z - m_s) * value, l_s = sum of
// exp(z - m_s); l_s = 0 for an empty part) merged with the window's partial results, if there are any.
template <int G>
__device__ __forceinline__ float merge_window(const float *win, int ul, int hh, int dim, float v, float m_s, float l_s, float &lse)
{
    // all partial results are requested at once (no load depends on another)
    float mx[kWinSplit], lx[kWinSplit], ox[kWinSplit];
#pragma unroll
    for (int x = 0; x < kWinSplit; ++x) {
        mx[x] = -__builtin_huge_valf();
        lx[x] = 0.0f;
        ox[x] = 0.0f;
    }
    if (win) {
        const float *wp = win + (size_t)ul * kWinSplit * G * (2 + kD) + hh * (2 + kD);
#pragma unroll
        for (int x = 0; x < kWinSplit; ++x) {
            mx[x] = wp[x * G * (2 + kD)];
            lx[x] = wp[x * G * (2 + kD) + 1];
            ox[x] = wp[x * G * (2 + kD) + 2 + dim];
        }
    }
    float M = l_s > 0.0f ? m_s : -__builtin_huge_valf();
#pragma unroll
    for (int x = 0; x < kWinSplit; ++x)
        if (lx[x] > 0.0f) M = fmaxf(M, mx[x]);
    if (M == -__builtin_huge_valf()) {   // nothing to attend over at all: defined output
        lse = -__builtin_huge_valf();
        return 0.0f;
    }
    float num = 0.0f, den = 0.0f;
    if (l_s > 0.0f) {
        const float w = __expf(m_s - M);
        num = v * w;
        den = l_s * w;
    }
#pragma unroll
    for (int x = 0; x < kWinSplit; ++x)
        if (lx[x] > 0.0f) {
            const float w = __expf(mx[x] - M);
            num += ox[x] * w;
            den += lx[x] * w;
        }
    lse = M + __logf(den);
    return num / den;
}

// Block id -> (unit, slice).  A slice is 128 / SL head dimensions of all G heads, SL = 4 or 8 (8 while every
// block still has a CU of its own: each block then moves half the bytes and weighs half the rows; beyond that the
// launch is oversubscribed and 4 is faster).  Workgroups go to the 8 XCDs round-robin by linear id; the slices of a
// unit read the same 128-byte lines, so they get ids that are congruent modulo 8: one XCD, one L2.
template <int SL> __device__ __forceinline__ void attn_block_of(int &ul, int &slice)
{
    const int lin = blockIdx.x, nu = gridDim.x / SL;
    if ((nu & 7) == 0) {
        const int xcd = lin & 7, k = lin >> 3;
        ul = (k / SL) * 8 + xcd;
        slice = k % SL;
    } else {
        ul = lin / SL;
        slice = lin % SL;
    }
}

// The attention of one (unit, slice).  row_of(t) = physical row of the t-th selected key (valid for
// every t < top_k), z_of(t, zv) = its G logits, nsel_of() = how many keys were selected; nsel_of is
// asked only after the first value rows have been requested.  s_p: top_k*G floats of shared memory.
template <typename T, int G, int SL, typename RowFn, typename ZFn, typename NFn>
__device__ __forceinline__ void attend_unit(const AttnArgs &a, int ul, int slice, float *s_p, RowFn row_of, ZFn z_of, NFn nsel_of)
{
    constexpr int kSliceDims = kD / SL;            // head dimensions per block
    constexpr int kSliceLanes = kSliceDims / 8;    // lanes that share a value row (8 dimensions each)
    constexpr int kSliceRows = 64 / kSliceLanes;   // rows per wave and pass
    static_assert(kSliceRows % 16 == 0, "the sum over a wave's rows starts with a butterfly inside each 16-lane row");
    // A wave's 64 lanes are kSliceLanes parts of kSliceRows rows: lane l works on row (l mod kSliceRows) of the
    // pass and on the 8 values (l / kSliceRows) of the slice.  Every 16-lane row of a wave thus belongs to one part and
    // is one producer of partial sums; kProd of them per part in the block.
    constexpr int PASS = 16 * kSliceRows, NU = 4, kProd = kSliceRows;   // rows per pass of the block, passes in flight
    __shared__ float s_red[kProd][G];
    __shared__ float s_m[G], s_l[G];
    __shared__ float s_o[kProd][G][kSliceDims];
    const int b = ul / a.g, kv = ul - b * a.g;
    const int tid = threadIdx.x, wv = tid >> 6, ln = tid & 63;
    const int quad = ln / kSliceRows, rin = wv * kSliceRows + (ln % kSliceRows);
    const int prod = wv * (kSliceRows / 16) + ((ln % kSliceRows) >> 4);   // this lane's 16-lane row among its part's producers
    CTKVR_STAMP(44);
    CTKVR_STAMP_BLK(4);
    const T *V = (const T *)a.v_pages + slice * kSliceDims + quad * 8;
    // The first NU * PASS value rows are requested before anything else (rows beyond nsel are valid
    // stale ones whose products get weight 0).
    // The row numbers first, then the rows: taken in turn, each row number would be
    // waited for together with the row requested just before it.
    Chunk<T> cv[NU];
    uint32_t vrow[NU];
#pragma unroll
    for (int u = 0; u < NU; ++u) vrow[u] = row_of(min(u * PASS + rin, a.top_k - 1));
#pragma unroll
    for (int u = 0; u < NU; ++u) cv[u] = load_chunk(V + (size_t)vrow[u] * kD, 0);
    // those keys' logits travel with their value rows
    float zq[NU][G];
#pragma unroll
    for (int u = 0; u < NU; ++u) z_of(min(u * PASS + rin, a.top_k - 1), zq[u]);
    const int nsel = nsel_of();
    if (nsel == 0) {   // nothing recalled: the window alone, or zeros
        if (tid < G * kSliceDims) {
            int hh = tid / kSliceDims, e = tid % kSliceDims;
            float lse;
            const float o = merge_window<G>(a.win, ul, hh, slice * kSliceDims + e, 0.0f, -__builtin_huge_valf(), 0.0f, lse);
            a.out[((size_t)b * a.h + kv * G + hh) * kD + slice * kSliceDims + e] = o;
            if (slice == 0 && e == 0 && a.out_lse) a.out_lse[(size_t)b * a.h + kv * G + hh] = lse;
        }
        return;
    }
    // One pass: weights relative to the unit's maxima over ALL its recalled keys, known since the scoring
    // (every selected logit is at most that maximum), so that no statistics of the selected keys have to be
    // gathered before their value rows can be used.  Lane groups that share a key row compute the same
    // weights; the lanes of a wave's first row carry them into the denominators.
    float acc[G][8], lsum[G], mref[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        mref[hh] = ordered_value(a.m_key[ul * G + hh]);
        lsum[hh] = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[hh][e] = 0.0f;
    }
    for (int r0 = 0; r0 < nsel; r0 += NU * PASS) {
        if (r0 > 0) {
#pragma unroll
            for (int u = 0; u < NU; ++u) vrow[u] = row_of(min(r0 + u * PASS + rin, a.top_k - 1));
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                cv[u] = load_chunk(V + (size_t)vrow[u] * kD, 0);
                z_of(min(r0 + u * PASS + rin, a.top_k - 1), zq[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int t = r0 + u * PASS + rin;
            if (t < nsel) {
                float vx[8];
                unpack(cv[u], vx);
#pragma unroll
                for (int hh = 0; hh < G; ++hh) {
                    const float pw = __expf(zq[u][hh] - mref[hh]);
                    lsum[hh] += quad == 0 ? pw : 0.0f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[hh][e] = __fmaf_rn(pw, vx[e], acc[hh][e]);
                }
            }
        }
    }
    CTKVR_STAMP(48);
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        const float v = group16_sum(lsum[hh]);   // the lanes of the other parts hold zeros
        if ((ln & 15) == 0 && quad == 0) s_red[prod][hh] = v;
    }
    __syncthreads();
    if (tid < G) {
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < kProd; ++w) v += s_red[w][tid];
        s_l[tid] = v;
        s_m[tid] = mref[0];
#pragma unroll
        for (int c = 1; c < G; ++c)
            if (tid == c) s_m[tid] = mref[c];
    }
    __syncthreads();
    CTKVR_STAMP(45);
    bool underflow = false;   // a head whose selected logits all lie far below its maximum: the same for every thread
#pragma unroll
    for (int hh = 0; hh < G; ++hh) underflow |= !(s_l[hh] >= 1e-30f);
    if (underflow) {
        // two passes instead: the selected keys' own maxima first, then weights relative to them
        __syncthreads();
        // softmax statistics over the selected keys, per head
        float mx[G];
#pragma unroll
        for (int hh = 0; hh < G; ++hh) mx[hh] = -__builtin_huge_valf();
        for (int t = tid; t < nsel; t += 1024) {
            float zv[G];
            z_of(t, zv);
#pragma unroll
            for (int hh = 0; hh < G; ++hh) {
                s_p[t * G + hh] = zv[hh];
                mx[hh] = fmaxf(mx[hh], zv[hh]);
            }
        }
        CTKVR_STAMP(48);
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            float v = mx[hh];
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
            if (ln == 0) s_red[wv][hh] = v;
        }
        __syncthreads();
        CTKVR_STAMP(49);
        if (tid < G) {
            float v = s_red[0][tid];
#pragma unroll
            for (int w = 1; w < 16; ++w) v = fmaxf(v, s_red[w][tid]);
            s_m[tid] = v;
        }
        __syncthreads();
        float sm[G];
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            mx[hh] = s_m[hh];
            sm[hh] = 0.0f;
        }
        for (int t = tid; t < nsel; t += 1024) {
#pragma unroll
            for (int hh = 0; hh < G; ++hh) {
                float p = __expf(s_p[t * G + hh] - mx[hh]);
                s_p[t * G + hh] = p;
                sm[hh] += p;
            }
        }
        CTKVR_STAMP(50);
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            float v = sm[hh];
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
            if (ln == 0) s_red[wv][hh] = v;
        }
        __syncthreads();
        if (tid < G) {
            float v = 0.0f;
#pragma unroll
            for (int w = 0; w < 16; ++w) v += s_red[w][tid];
            s_l[tid] = v;
        }
        __syncthreads();
        CTKVR_STAMP(45);
        // weighted sum of the value rows
#pragma unroll
        for (int hh = 0; hh < G; ++hh)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[hh][e] = 0.0f;
        for (int r0 = 0; r0 < nsel; r0 += NU * PASS) {
            {
#pragma unroll
                for (int u = 0; u < NU; ++u) vrow[u] = row_of(min(r0 + u * PASS + rin, a.top_k - 1));
#pragma unroll
                for (int u = 0; u < NU; ++u) cv[u] = load_chunk(V + (size_t)vrow[u] * kD, 0);
            }
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                int t = r0 + u * PASS + rin;
                if (t < nsel) {
                    float vx[8];
                    unpack(cv[u], vx);
                    float pv[G];
                    load_z<G>(s_p, t, pv);
#pragma unroll
                    for (int hh = 0; hh < G; ++hh)
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[hh][e] = __fmaf_rn(pv[hh], vx[e], acc[hh][e]);
                }
            }
        }
    }
    // sum inside each 16-lane row (a DPP butterfly), then over the part's kProd rows of the block in order
#pragma unroll
    for (int hh = 0; hh < G; ++hh)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[hh][e] = group16_sum(acc[hh][e]);
    if ((ln & 15) == 0) {
#pragma unroll
        for (int hh = 0; hh < G; ++hh)
#pragma unroll
            for (int e = 0; e < 8; ++e) s_o[prod][hh][quad * 8 + e] = acc[hh][e];
    }
    __syncthreads();
    CTKVR_STAMP(46);
    if (tid < G * kSliceDims) {
        int hh = tid / kSliceDims, e = tid % kSliceDims;
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < kProd; ++w) v += s_o[w][hh][e];
        float lse;
        const float o = merge_window<G>(a.win, ul, hh, slice * kSliceDims + e, v, s_m[hh], s_l[hh], lse);
        a.out[((size_t)b * a.h + kv * G + hh) * kD + slice * kSliceDims + e] = o;
        if (slice == 0 && e == 0 && a.out_lse) a.out_lse[(size_t)b * a.h + kv * G + hh] = lse;
    }
    CTKVR_STAMP(47);
    CTKVR_STAMP_BLK(5);
}

template <typename T, int G, int SL> __global__ __launch_bounds__(1024) void sparse_attn_kernel(AttnArgs a)
{
    extern __shared__ __align__(16) float s_p[];   // [top_k][G]
    int ul, slice;
    attn_block_of<SL>(ul, slice);
    const uint32_t *rb = a.srow + (size_t)ul * a.top_k;
    const float *zb = a.zsel + (size_t)ul * a.top_k * G;
    attend_unit<T, G, SL>(a, ul, slice, s_p, [&](int t) { return rb[t]; }, [&](int t, float(&zv)[G]) { load_z<G>(zb, t, zv); },
                      [&]() { return a.nsel[ul]; });
}

// ------------------------------------------------------------------------------
// Algorithm 2 lines 6-9 in one launch, for batches small enough that every block has a CU of its
// own: each of the SL slice blocks of a unit makes the unit's selection itself (the same work
// several times over, on as many CUs, instead of a second launch and a round trip of the picks through
// global memory) and then attends over the picks straight from the recalled ids' rows and logits.
// Slice 0 also writes the selected ids and their number.  grid SL*batch*g, 1024 threads; dynamic
// shared memory: the selection's words, then top_k*G floats.
// ------------------------------------------------------------------------------
template <typename T, int G, int SL> __global__ __launch_bounds__(1024) void select_attn_kernel(SelectArgs sa, AttnArgs a)
{
    extern __shared__ __align__(16) uint32_t smem[];
    int ul, slice;
    attn_block_of<SL>(ul, slice);
    const int L = sa.ncand[ul];
    CTKVR_STAMP(28);
    const int n = select_unit<G>(sa, ul, L, smem);
    __syncthreads();
    const int32_t *s_idx = (const int32_t *)(smem + kSelLds + 2 * kListCap + sa.bits_words);
    float *s_p = reinterpret_cast<float *>(smem + select_smem_words(sa.bits_words, sa.top_k));
    const int32_t *cb = sa.cand + (size_t)ul * sa.l_stride;
    const uint32_t *rb = sa.crow + (size_t)ul * sa.l_stride;
    const float *zb = sa.z + (size_t)ul * sa.l_stride * G;
    CTKVR_STAMP(31);
    if (slice == 0) {
        int32_t *dst = sa.sel + (size_t)ul * sa.top_k;
        int32_t *dst2 = sa.out_sel ? sa.out_sel + (size_t)ul * sa.top_k : nullptr;
        for (int pos = threadIdx.x; pos < sa.top_k; pos += 1024) {
            const int t = pos < n ? cb[s_idx[pos]] : -1;
            dst[pos] = t;
            if (dst2) dst2[pos] = t;
        }
        if (threadIdx.x == 0) sa.nsel[ul] = n;
    }
    // positions beyond n repeat the last pick; when nothing was recalled every position reads slot 0 of
    // the row table and then names row 0 of the pool (selects, not a branch: the four row numbers of a
    // pass are then requested together)
    attend_unit<T, G, SL>(a, ul, slice, s_p,
                      [&](int t) {
                          const uint32_t r = rb[n > 0 ? s_idx[min(t, n - 1)] : 0];
                          return n > 0 ? r : 0u;
                      },
                      [&](int t, float(&zv)[G]) { load_z<G>(zb, n > 0 ? s_idx[min(t, n - 1)] : 0, zv); }, [&]() { return n; });
}

// ------------------------------------------------------------------------------
// Algorithm 2 line 12 (dynamic centroid update): the step's query becomes the centroid of the
// FIFO slot (updates so far mod C: the oldest mapping goes first) for the G heads of the group,
// with its inverse norm, and the slot's list becomes src[unit][0..rho): the top-rho ids by rerank
// score, ascending (should fewer have been recalled, the last one is repeated; none: no update).
// grid batch*g, 256 threads; the block that ends last counts the update.
// ------------------------------------------------------------------------------
struct DcuArgs {
    int g, h, G, c_max, rho, src_stride;
    const int32_t *n_cent;
    uint32_t *count;          // [2]: updates so far; blocks of this update that are done (zero between updates)
    const void *q;            // [batch][h][128]
    const int32_t *src;       // [units][src_stride]
    const int32_t *nsrc;      // [units]
    void *centroids;          // [batch][h][c_max][128]
    float *inv_norm_c;        // [batch][h][c_max]
    int32_t *lists;           // [units][c_max][rho]
};

__device__ __forceinline__ void store_chunk(float *row, int lane16, const Chunk<float> &c)
{
    float4 *p = reinterpret_cast<float4 *>(row + 8 * lane16);
    p[0] = c.a;
    p[1] = c.b;
}
__device__ __forceinline__ void store_chunk(bf16_t *row, int lane16, const Chunk<bf16_t> &c)
{
    *reinterpret_cast<uint4 *>(row + 8 * lane16) = c.w;
}

template <typename T> __global__ __launch_bounds__(256) void dcu_write_kernel(DcuArgs a)
{
    const int ul = blockIdx.x, b = ul / a.g, kv = ul - b * a.g, tid = threadIdx.x;
    const int slot = (int)(a.count[0] % (uint32_t)a.n_cent[b]);
    const int n = min(a.nsrc[ul], a.rho);
    if (n > 0) {
        const int32_t *src = a.src + (size_t)ul * a.src_stride;
        int32_t *dst = a.lists + ((size_t)ul * a.c_max + slot) * a.rho;
        for (int r = tid; r < a.rho; r += 256) dst[r] = src[min(r, n - 1)];
        if (tid < 16 * a.G) {
            const int hh = tid >> 4, lane16 = tid & 15;
            const size_t head = (size_t)b * a.h + kv * a.G + hh;
            Chunk<T> c = load_chunk((const T *)a.q + head * kD, lane16);
            store_chunk((T *)a.centroids + (head * a.c_max + slot) * kD, lane16, c);
            float x[8];
            unpack(c, x);
            const float n2 = group16_sum(lane_partial(x, x));
            if (lane16 == 0) a.inv_norm_c[head * a.c_max + slot] = inv_norm_from_sq(n2);
        }
    }
    // The update is counted by the block that ends last: every block has read the count before it reports done.
    __syncthreads();
    if (tid == 0 && atomicAdd(&a.count[1], 1u) == gridDim.x - 1) {
        atomicExch(&a.count[1], 0u);
        atomicAdd(&a.count[0], 1u);
    }
}

}  // namespace ctkvr
