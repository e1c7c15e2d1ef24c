// The decode step (Algorithm 2 lines 1-9) as ONE launch: every (sequence, KV head) unit is worked
// on by a fixed group of co-resident blocks that walk the step's phases together, separated by
// per-unit barriers in global memory instead of kernel boundaries:
//
//   phase 0  cosines of the unit's centroids (lines 1-2), split over the unit's blocks
//   phase 1  every block: top-C' centroids (line 3); its share of the probed lists -> bitmap (line 4)
//   phase 2  every block: prefix popcount of the bitmap, an equal share of the RANKS of the
//            recalled ids -> ids, rows, z = q.k * scale, running maxima (lines 4-5)
//   phase 3  softmax denominators of its share (integer fixed point)
//   phase 4  ranking keys of its share and their histogram
//   phase 5  every block finds the deciding bucket from the histogram, classifies its share
//            (sure picks -> bitmap, deciding bucket -> list) and attends over its own sure picks:
//            a partial (m, l, o) per head relative to its own maximum (lines 6-9, split over keys)
//   final    the unit's first block: threshold inside the deciding bucket, the selected ids in
//            ascending order, attention over the bucket's picks, merge of all partials (and of the
//            resident window's, lines 10-11) -> out, lse
//
// Blocks of different units never wait for each other.  A unit's blocks sit on one XCD when the
// number of units is a multiple of 8 (workgroups go to the XCDs round-robin), so their traffic
// meets in one L2; correctness does not depend on it: every word that another block reads within
// the launch is written with an agent-scope atomic store or read-modify-write (written through to
// memory) and read with an agent-scope atomic load (never served from a stale cache line).
// Every wait is bounded by the wall clock; on expiry the error word is set and the block leaves.
// The grid must be co-resident: units * blocks-per-unit <= CUs, one 1024-thread block per CU.
#pragma once
#include "arith.hpp"
#include "common.hpp"
#include "fused_args.hpp"

namespace ctkvr {


// ---- coherent accesses (see the header comment) -------------------------------------------------
template <typename V> __device__ __forceinline__ V ldc(const V *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
template <typename V> __device__ __forceinline__ void stc(V *p, V v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// All threads of the block call this.  Returns false when the wait expired or another block
// has reported an error: the caller leaves the kernel.
__device__ __forceinline__ bool unit_barrier(uint32_t *ctr, uint32_t members, uint32_t *err, uint32_t *s_flag)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);   // this thread's stores and atomics have been acknowledged
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t ok = 1u;
        if (members > 1u) {
            __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const long long t0 = wall_clock64();
            uint32_t spins = 0;
            while (ldc(ctr) < members) {
                __builtin_amdgcn_s_sleep(1);
                if ((++spins & 63u) == 0u && (ldc(err) != 0u || wall_clock64() - t0 > kFusedWaitTicks)) {
                    stc(err, 1u);
                    ok = 0u;
                    break;
                }
            }
        }
        *s_flag = ok;
    }
    __syncthreads();
    const bool ok = *s_flag != 0u;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    return ok;
}

// Appends, in thread order, `value` of the threads whose `pred` holds to dst[base ...] and returns the
// new fill level to every thread: no atomic decides an order, so the result is the same in every run.
// All threads of the block call it.  s_cnt: NT / 64 words.
template <int NT> __device__ __forceinline__ int block_append_ordered(bool pred, int32_t value, int32_t *dst, int base, uint32_t *s_cnt)
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
    if (pred) dst[base + (int)before + __popcll(m & ((1ull << ln) - 1ull))] = value;
    __syncthreads();
    return base + (int)tot;
}

// Attention of one block over n picks (positions into the unit's recalled list, in s_pick):
// per head the maximum logit (returned in mx[], the same in every thread), and per wave w its
// partial sums relative to that maximum, left in shared memory: s_red[(w * G + hh) * 129 + dim] =
// sum over the wave's picks of exp(z - mx) v[dim], and at dim = 128 the sum of exp(z - mx);
// attend_sum() adds the waves up.  One pick per 16-lane group at a time, four in flight; z and the
// row numbers are read coherently (they may be another block's).  s_red: (NT / 64) * G * 129 words.
// Barriers inside; the caller places one before s_red is written again.
template <typename T, int G, int NT>
__device__ __forceinline__ void attend_picks(int n, const int32_t *s_pick, const float *zb, const uint32_t *rb, const T *V,
                                             float *s_red, float (&mx)[G])
{
    const int tid = threadIdx.x, wv = tid >> 6, ln = tid & 63, lane16 = tid & 15, grp = tid >> 4;
    const int myh = lane16 & (G - 1);
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
    constexpr int NG = NT / 16;   // 16-lane groups
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
    // the four groups of a wave, then the sixteen waves
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

template <typename T, int G, int NT> __global__ __launch_bounds__(NT) void decode_fused_kernel(FusedArgs a)
{
    extern __shared__ __align__(16) uint32_t smem[];
    __shared__ uint32_t s_flag, s_scan[20], s_res[4];
    __shared__ uint32_t s_max[G];
    __shared__ float s_ls[G];
    __shared__ unsigned long long s_acc[NT / 64][G];
    uint32_t *s_sel = smem;                                  // kSelLds
    int32_t *s_probe = (int32_t *)(smem + kSelLds);          // n_probe
    uint32_t *s_reg = smem + kSelLds + a.n_probe;            // the phases' common region
    const size_t sel_bits = 4 * (size_t)((a.l_stride + 63) / 64);
    size_t region = (size_t)a.bitmap_words;
    if (region < (size_t)kFusedChunk) region = kFusedChunk;
    {
        const size_t fin = 2 * (size_t)kListCap + sel_bits + (size_t)a.top_k + (size_t)kListCap;
        if (region < fin) region = fin;
        if (region < (size_t)a.top_k) region = a.top_k;
    }
    float *s_red = reinterpret_cast<float *>(s_reg + region);   // 16 * G * 129

    const int tid = threadIdx.x, wv = tid >> 6, ln = tid & 63, lane16 = tid & 15, grp = tid >> 4;
    // block -> (unit, x): the blocks of a unit get linear ids that agree modulo 8 (one XCD) when the
    // number of units allows it
    int ul, x;
    {
        const int lin = blockIdx.x;
        if ((a.units & 7) == 0) {
            const int xcd = lin & 7, k = lin >> 3;
            ul = (k / a.bpu) * 8 + xcd;
            x = k - (k / a.bpu) * a.bpu;
        } else {
            ul = lin / a.bpu;
            x = lin - ul * a.bpu;
        }
    }
    if (ldc(a.err) != 0u) return;   // an earlier step failed: the workspace is not to be trusted
    const int b = ul / a.g, kv = ul - b * a.g;
    const int C = a.n_cent[b], s_len = a.ctx_lens[b];
    const int W = (s_len + 31) >> 5;
    const uint32_t bpu = (uint32_t)a.bpu;
    uint32_t *bar = a.bar + (size_t)ul * kFusedBarriers;
    const bool stamp = a.prof && ul == 0 && x == 0 && tid == 0;
    if (stamp) a.prof[0] = wall_clock64();
    auto STAMP = [&](int k) {
        if (stamp) a.prof[k] = wall_clock64();
    };

    float *cosv = a.cos + (size_t)ul * a.c_max;
    uint32_t *gb = a.gbits + (size_t)ul * a.bitmap_words;
    uint32_t *gh = a.ghist + (size_t)ul * kBuckets;
    uint32_t *gbm = a.gbm + (size_t)ul * a.bits_stride;
    const T *qb = (const T *)a.q + ((size_t)b * a.h + kv * G) * kD;

    // ---------------------------------------------------------------- phase 0: cosines
    float q[G][8];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) unpack(load_chunk(qb + (size_t)hh * kD, lane16), q[hh]);
    {
        if (x == 0 && tid < G) {
            stc(a.m_key + ul * G + tid, 0u);
            stc(a.S + ul * G + tid, 0ull);
        }
        if (x == 0 && tid == 0) stc(a.gcur + ul, 0u);
        for (int w = x * NT + tid; w < kBuckets; w += a.bpu * NT) stc(gh + w, 0u);
        float inv_q[G];
#pragma unroll
        for (int hh = 0; hh < G; ++hh) inv_q[hh] = inv_norm_from_sq(group16_sum(lane_partial(q[hh], q[hh])));
        const T *cb = (const T *)a.centroids;
        for (int j0 = x * (NT / 16); j0 < C; j0 += a.bpu * (NT / 16)) {
            const int j = j0 + grp;
            const int jj = j < C ? j : C - 1;
            Chunk<T> cc[G];
            float inc[G];
#pragma unroll
            for (int hh = 0; hh < G; ++hh) {
                const size_t row = ((size_t)b * a.h + kv * G + hh) * a.c_max + jj;
                cc[hh] = load_chunk(cb + row * kD, lane16);
                inc[hh] = a.inv_norm_c[row];
            }
            float best = -__builtin_huge_valf();
#pragma unroll
            for (int hh = 0; hh < G; ++hh) {
                float cx[8];
                unpack(cc[hh], cx);
                const float dot = group16_sum(lane_partial(q[hh], cx));
                best = fmaxf(best, (dot * inc[hh]) * inv_q[hh]);
            }
            if (j < C && lane16 == 0) stc(cosv + j, best);
        }
    }
    if (stamp) a.prof[8 + 0] = wall_clock64();   // own work of the phase done
    if (!unit_barrier(bar + 0, bpu, a.err, &s_flag)) return;
    if (stamp) a.prof[1] = wall_clock64();

    // ---------------------------------------------------------------- phase 1: probes, lists -> bitmap
    {
        uint32_t *s_bits = s_reg;
        for (int w = tid; w < W; w += NT) s_bits[w] = 0u;
        auto keep = [&](int pos, int j) {
            s_probe[pos] = j;
            if (x == 0) {
                a.probe[(size_t)ul * a.n_probe + pos] = j;
                if (a.out_probe) a.out_probe[(size_t)ul * a.n_probe + pos] = j;
            }
        };
        auto ckey = [&](int j) { return ordered_key(ldc(cosv + j)); };
        constexpr int K1 = 1024 / NT;   // keys per thread for up to 1024 centroids
        if (a.n_probe <= 8) {
            block_extract_topk<NT, 8 * K1>(ckey, C, a.n_probe, keep, s_sel);
        } else {
            if (a.c_max <= 1024) block_bisect_topk<NT, K1>(ckey, C, a.n_probe, keep, s_sel);
            else if (a.c_max <= 2048) block_bisect_topk<NT, 2 * K1>(ckey, C, a.n_probe, keep, s_sel);
            else block_bisect_topk<NT, 8 * K1>(ckey, C, a.n_probe, keep, s_sel);
        }
        __syncthreads();
        STAMP(16);
        // items of 256 ids (one 16-byte load per lane); item i belongs to wave i mod (waves of the unit)
        const int32_t *lb = a.lists + (size_t)ul * a.c_max * a.rho;
        auto mark = [&](int t) { atomicOr(&s_bits[t >> 5], 1u << (t & 31)); };
        const int wave_u = x * (NT / 64) + wv, nwave_u = a.bpu * (NT / 64);
        if ((a.rho & 3) == 0) {
            const int rho4 = a.rho >> 2;
            const int ipl = (rho4 + 63) >> 6;              // items per list
            const int n_items = a.n_probe * ipl;
            for (int it0 = wave_u; it0 < n_items; it0 += 4 * nwave_u) {
                int4 t[4];
                bool live[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int it = min(it0 + u * nwave_u, n_items - 1);
                    const int p = it / ipl, seg = it - p * ipl;
                    const int r = seg * 64 + ln;
                    live[u] = (it0 + u * nwave_u < n_items) && r < rho4;
                    t[u] = reinterpret_cast<const int4 *>(lb + (size_t)s_probe[p] * a.rho)[min(r, rho4 - 1)];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (live[u]) { mark(t[u].x); mark(t[u].y); mark(t[u].z); mark(t[u].w); }
            }
        } else {
            const int ipl = (a.rho + 63) >> 6;
            const int n_items = a.n_probe * ipl;
            for (int it0 = wave_u; it0 < n_items; it0 += 4 * nwave_u) {
                int32_t t[4];
                bool live[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int it = min(it0 + u * nwave_u, n_items - 1);
                    const int p = it / ipl, seg = it - p * ipl;
                    const int r = seg * 64 + ln;
                    live[u] = (it0 + u * nwave_u < n_items) && r < a.rho;
                    t[u] = lb[(size_t)s_probe[p] * a.rho + min(r, a.rho - 1)];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (live[u]) mark(t[u]);
            }
        }
        __syncthreads();
        STAMP(17);
        for (int w = tid; w < W; w += NT) {
            const uint32_t v = s_bits[w];
            if (v) __hip_atomic_fetch_or(gb + w, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (stamp) a.prof[8 + 1] = wall_clock64();   // own work of the phase done
    if (!unit_barrier(bar + 1, bpu, a.err, &s_flag)) return;
    if (stamp) a.prof[2] = wall_clock64();

    // ---------------------------------------------------------------- phase 2: ids, rows, scores
    int L, r_beg, r_end;
    {
        // thread t owns the words [t*wpt, (t+1)*wpt) of the bitmap
        const int wpt = (W + NT - 1) / NT;
        const int w0 = min(W, tid * wpt), w1 = min(W, w0 + wpt);
        uint32_t cnt = 0;
        uint32_t wreg[4] = {0u, 0u, 0u, 0u};   // the thread's words, kept when there are at most four
        if (wpt <= 4) {
#pragma unroll
            for (int c = 0; c < 4; ++c) wreg[c] = ldc(gb + min(w0 + c, W - 1));
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                wreg[c] = w0 + c < w1 ? wreg[c] : 0u;
                cnt += (uint32_t)__popc(wreg[c]);
            }
        } else {
            for (int w = w0; w < w1; ++w) cnt += (uint32_t)__popc(ldc(gb + w));
        }
        uint32_t tot;
        const uint32_t rank0 = block_excl_scan<NT>(cnt, s_scan, &tot);
        STAMP(18);
        L = (int)tot;
        r_beg = (int)(((unsigned long long)x * tot) / bpu);
        r_end = (int)(((unsigned long long)(x + 1) * tot) / bpu);
        if (x == 0 && tid == 0) {
            a.ncand[ul] = L;
            if (a.out_ncand) a.out_ncand[ul] = L;
        }
        if (tid < G) s_max[tid] = 0u;
        uint32_t *s_ids = s_reg;
        int32_t *cd = a.cand + (size_t)ul * a.l_stride;
        uint32_t *rw = a.crow + (size_t)ul * a.l_stride;
        float *zb = a.z + (size_t)ul * a.l_stride * G;
        const T *K = (const T *)a.k.pages;
        const int pmask = (1 << a.k.page_shift) - 1;
        const int32_t *bt_row = a.k.block_table + (size_t)b * a.k.max_pages;
        constexpr int R = (sizeof(T) == 2 ? 8 : 4) * (NT == 256 ? 2 : 1);   // rows in flight per 16-lane group
        float mxl = -__builtin_huge_valf();
        const int myh = lane16 & (G - 1);
        for (int c_beg = r_beg; c_beg < r_end; c_beg += kFusedChunk) {
            const int c_end = min(r_end, c_beg + kFusedChunk);
            __syncthreads();   // the previous chunk's rows have been consumed
            if ((int)rank0 < c_end && (int)(rank0 + cnt) > c_beg) {
                int rk = (int)rank0;
                for (int w = w0; w < w1; ++w) {
                    uint32_t m;
                    if (wpt <= 4) {
                        const int c = w - w0;
                        m = c == 0 ? wreg[0] : c == 1 ? wreg[1] : c == 2 ? wreg[2] : wreg[3];
                    } else {
                        m = ldc(gb + w);
                    }
                    while (m) {
                        const int bit = __ffs((int)m) - 1;
                        m &= m - 1u;
                        if (rk >= c_beg && rk < c_end) s_ids[rk - c_beg] = ((uint32_t)w << 5) + (uint32_t)bit;
                        ++rk;
                    }
                }
            }
            __syncthreads();
            STAMP(19);
            const int nch = c_end - c_beg;
            for (int i = tid; i < nch; i += NT) {
                const int t = (int)s_ids[i];
                const uint32_t row = (uint32_t)((bt_row[t >> a.k.page_shift] * a.g + kv) << a.k.page_shift) + (uint32_t)(t & pmask);
                stc(cd + c_beg + i, t);
                stc(rw + c_beg + i, row);
                s_ids[i] = row;
            }
            __syncthreads();
            STAMP(20);
            const int last = nch - 1;
            for (int t0 = 0; t0 < nch; t0 += (NT / 16) * R) {
                Chunk<T> ck[R];
                const T *krow[R];
#pragma unroll
                for (int r = 0; r < R; ++r) krow[r] = K + (size_t)s_ids[min(t0 + r * (NT / 16) + grp, last)] * kD;
                if (a.stream_k) {
#pragma unroll
                    for (int r = 0; r < R; ++r) ck[r] = load_chunk_nt(krow[r], lane16);
                } else {
#pragma unroll
                    for (int r = 0; r < R; ++r) ck[r] = load_chunk(krow[r], lane16);
                }
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    if (t0 + r * (NT / 16) + wv * 4 > last) continue;   // nothing for this wave (uniform)
                    float kx[8];
                    unpack(ck[r], kx);
                    float mine_z = 0.0f;
#pragma unroll
                    for (int hh = 0; hh < G; ++hh) {
                        const float tot_d = group16_sum(lane_partial(q[hh], kx));
                        if (hh == 0 || myh == hh) mine_z = tot_d;
                    }
                    mine_z = mine_z * a.scale;
                    const int i = t0 + r * (NT / 16) + grp;
                    if (i <= last) {
                        mxl = __builtin_amdgcn_fmed3f(mxl, mine_z, __builtin_huge_valf());
                        if (lane16 < G) stc(zb + (size_t)(c_beg + i) * G + lane16, mine_z);
                    }
                }
            }
        }
        STAMP(21);
        {
            float v = mxl;
            v = __builtin_amdgcn_fmed3f(v, __shfl_xor(v, 16), __builtin_huge_valf());
            v = __builtin_amdgcn_fmed3f(v, __shfl_xor(v, 32), __builtin_huge_valf());
            if (ln < G && r_end > r_beg) atomicMax(&s_max[ln], ordered_key(v));
        }
        __syncthreads();
        if (tid < G && r_end > r_beg) __hip_atomic_fetch_max(a.m_key + ul * G + tid, s_max[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (stamp) a.prof[8 + 2] = wall_clock64();   // own work of the phase done
    if (!unit_barrier(bar + 2, bpu, a.err, &s_flag)) return;
    if (stamp) a.prof[3] = wall_clock64();
    if (x == 0 && tid == 0) stc(bar + 0, 0u);   // everyone has left barrier 0 (and so on below)

    // ---------------------------------------------------------------- phase 3: denominators
    const float *zb = a.z + (size_t)ul * a.l_stride * G;
    float m[G];
    {
        // the bitmap has been read by every block of the unit: cleared for the next step, and so is
        // the selection's bitmap
        for (int w = x * NT + tid; w < W; w += a.bpu * NT) stc(gb + w, 0u);
        for (int w = x * NT + tid; w < a.bits_stride; w += a.bpu * NT) stc(gbm + w, 0u);
        uint32_t mk[G];
#pragma unroll
        for (int hh = 0; hh < G; ++hh) mk[hh] = ldc(a.m_key + ul * G + hh);
        unsigned long long acc[G];
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            m[hh] = ordered_value(mk[hh]);
            acc[hh] = 0ull;
        }
        for (int c0 = r_beg; c0 < r_end; c0 += 4 * NT) {
            uint32_t shi[G], slo[G];
#pragma unroll
            for (int hh = 0; hh < G; ++hh) shi[hh] = slo[hh] = 0u;
            float zv[4][G];
#pragma unroll
            for (int u = 0; u < 4; ++u) load_z<G>(zb, min(c0 + u * NT + tid, r_end - 1), zv[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (c0 + u * NT + wv * 64 >= r_end) continue;   // nothing for this wave (uniform)
                const bool ok = (c0 + u * NT + tid) < r_end;
#pragma unroll
                for (int hh = 0; hh < G; ++hh) {
                    uint32_t hi, lo;
                    exp_fixed40_parts(zv[u][hh] - m[hh], hi, lo);
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
            if (ln == 0) s_acc[wv][hh] = v;
        }
        __syncthreads();
        if (tid < G) {
            unsigned long long v = 0ull;
#pragma unroll
            for (int w = 0; w < NT / 64; ++w) v += s_acc[w][tid];
            if (v) __hip_atomic_fetch_add(a.S + ul * G + tid, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (stamp) a.prof[8 + 3] = wall_clock64();   // own work of the phase done
    if (!unit_barrier(bar + 3, bpu, a.err, &s_flag)) return;
    if (stamp) a.prof[4] = wall_clock64();
    if (x == 0 && tid == 0) stc(bar + 1, 0u);

    // ---------------------------------------------------------------- phase 4: ranking keys, histogram
    uint32_t *kb = a.kbuf + (size_t)ul * a.l_stride;
    {
        uint32_t *s_h = s_reg;
        for (int w = tid; w < kBuckets; w += NT) s_h[w] = 0u;
        if (tid < G) s_ls[tid] = (float)log_fixed40(ldc(a.S + ul * G + tid));
        __syncthreads();
        float ls[G];
#pragma unroll
        for (int hh = 0; hh < G; ++hh) ls[hh] = s_ls[hh];
        for (int c0 = r_beg; c0 < r_end; c0 += 4 * NT) {
            float zv[4][G];
#pragma unroll
            for (int u = 0; u < 4; ++u) load_z<G>(zb, min(c0 + u * NT + tid, r_end - 1), zv[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (c0 + u * NT + wv * 64 >= r_end) continue;   // nothing for this wave (uniform)
                const int i = c0 + u * NT + tid;
                const bool valid = i < r_end;
                float best = -__builtin_huge_valf();
#pragma unroll
                for (int hh = 0; hh < G; ++hh) best = fmaxf(best, (zv[u][hh] - m[hh]) - ls[hh]);
                const uint32_t ok = ordered_key(best);
                if (valid) stc(kb + i, ok);
                const uint32_t bk = key_bucket(ok);
                const bool tail = valid && bk == (uint32_t)(kBuckets - 1);
                const uint64_t mt = __ballot(tail);
                if (valid && !tail) atomicAdd(&s_h[bk], 1u);
                if (mt && ln == 0) atomicAdd(&s_h[kBuckets - 1], (uint32_t)__popcll(mt));
            }
        }
        __syncthreads();
        for (int w = tid; w < kBuckets; w += NT) {
            const uint32_t v = s_h[w];
            if (v) __hip_atomic_fetch_add(gh + w, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (stamp) a.prof[8 + 4] = wall_clock64();   // own work of the phase done
    if (!unit_barrier(bar + 4, bpu, a.err, &s_flag)) return;
    if (stamp) a.prof[5] = wall_clock64();
    if (x == 0 && tid == 0) stc(bar + 2, 0u);

    // ---------------------------------------------------------------- phase 5: classify, partial attention
    const uint32_t *rb = a.crow + (size_t)ul * a.l_stride;
    const T *V = (const T *)a.v_pages;
    uint32_t bkt = 0, rem = 0, nbk = 0;
    int mode;   // 0: every recalled key is picked; 1: histogram route; 2: the first block selects alone
    {
        int32_t *s_pick = (int32_t *)s_reg;
        if (a.top_k >= L) {
            mode = 0;
        } else {
            constexpr int BPT = kBuckets / NT;
            uint32_t c[BPT], mine = 0;
#pragma unroll
            for (int qq = 0; qq < BPT; ++qq) {
                c[qq] = ldc(gh + BPT * tid + qq);
                mine += c[qq];
            }
            uint32_t tot;
            uint32_t before = block_excl_scan<NT>(mine, s_scan, &tot);
#pragma unroll
            for (int qq = 0; qq < BPT; ++qq) {
                if (before < (uint32_t)a.top_k && (uint32_t)a.top_k <= before + c[qq]) {
                    s_res[0] = (uint32_t)(BPT * tid + qq);
                    s_res[1] = (uint32_t)a.top_k - before;
                    s_res[2] = c[qq];
                }
                before += c[qq];
            }
            __syncthreads();
            STAMP(22);
            bkt = s_res[0];
            rem = s_res[1];
            nbk = s_res[2];
            mode = nbk > (uint32_t)kListCap ? 2 : 1;
        }
        int n_own = 0;
        if (mode == 0) {
            for (int i = r_beg + tid; i < r_end; i += NT) s_pick[i - r_beg] = i;
            n_own = r_end - r_beg;
        } else if (mode == 1) {
            // groups of 64 ranks aligned to 64 in the unit's numbering, so that a ballot is a word pair of the
            // bitmap; a round of one group per wave at a time, its sure picks appended in rank order
            const uint64_t below = (1ull << ln) - 1ull;
            uint2 *lst = a.glist + (size_t)ul * kListCap;
            for (int gr = r_beg >> 6; gr * 64 < r_end; gr += NT / 64) {   // uniform
                const int g0 = gr + wv;
                const int i = g0 * 64 + ln;
                const bool valid = i >= r_beg && i < r_end;
                const uint32_t kk = kb[min(max(i, r_beg), r_end - 1)];
                const uint32_t bk = key_bucket(kk);
                const bool sure = valid && bk < bkt, inb = valid && bk == bkt;
                const uint64_t above = __ballot(sure), listed = __ballot(inb);
                if (ln == 0 && (uint32_t)above) __hip_atomic_fetch_or(gbm + 2 * g0, (uint32_t)above, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (ln == 0 && (uint32_t)(above >> 32)) __hip_atomic_fetch_or(gbm + 2 * g0 + 1, (uint32_t)(above >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (listed) {
                    uint32_t at0 = 0;
                    if (ln == 0) at0 = __hip_atomic_fetch_add(a.gcur + ul, (uint32_t)__popcll(listed), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    at0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)at0);
                    if (inb)
                        stc(reinterpret_cast<unsigned long long *>(lst) + at0 + (uint32_t)__popcll(listed & below),
                            (unsigned long long)kk | ((unsigned long long)(uint32_t)i << 32));
                }
                n_own = block_append_ordered<NT>(sure, i, s_pick, n_own, s_scan);
            }
        }
        __syncthreads();
        STAMP(23);
        float pmx[G];
        attend_picks<T, G, NT>(n_own, s_pick, zb, rb, V, s_red, pmx);
        STAMP(24);
        for (int e = tid; e < G * kD; e += NT) {
            const int hh = e >> 7, dim = e & 127;
            float *dst = a.part + (((size_t)ul * a.bpu + x) * G + hh) * (2 + kD);
            stc(dst + 2 + dim, attend_sum<G, NT>(s_red, hh, dim));
            if (dim == 0) {
                stc(dst, pick_head<G>(pmx, hh));
                stc(dst + 1, attend_sum<G, NT>(s_red, hh, kD));
            }
        }
    }
    // the last barrier: only the unit's first block waits
    if (x != 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (tid == 0) __hip_atomic_fetch_add(bar + 5, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    if (stamp) a.prof[8 + 5] = wall_clock64();   // own work of the phase done
    if (!unit_barrier(bar + 5, bpu, a.err, &s_flag)) return;
    if (stamp) a.prof[6] = wall_clock64();
    if (tid == 0) {
        stc(bar + 3, 0u);
        stc(bar + 4, 0u);
        stc(bar + 5, 0u);
    }

    // ---------------------------------------------------------------- final: selection, merge
    {
        uint32_t *s_list = s_reg;                                  // 2 * kListCap
        uint32_t *s_bits = s_list + 2 * kListCap;                  // sel_bits
        int32_t *s_idx = (int32_t *)(s_bits + sel_bits);           // top_k
        int32_t *s_bpick = s_idx + a.top_k;                        // kListCap: picks from the deciding bucket
        const int32_t *cd = a.cand + (size_t)ul * a.l_stride;
        auto emit = [&](int pos, int i) { s_idx[pos] = i; };
        int n;
        if (mode == 0) {
            n = L;
        } else if (mode == 1) {
            const int nw32 = 2 * ((L + 63) >> 6);
            uint32_t *s_gt = s_bits, *s_eq = s_bits + nw32;
            const unsigned long long *gl = reinterpret_cast<const unsigned long long *>(a.glist + (size_t)ul * kListCap);
            for (uint32_t e = tid; e < nbk; e += NT) {
                const unsigned long long v = ldc(gl + e);
                s_list[2 * e] = (uint32_t)v;
                s_list[2 * e + 1] = (uint32_t)(v >> 32);
            }
            for (int w = tid; w < nw32; w += NT) {
                s_gt[w] = ldc(gbm + w);
                s_eq[w] = 0u;
            }
            __syncthreads();
            STAMP(25);
            block_resolve_emit<NT>(nbk, rem, L, s_sel, s_gt, s_eq, reinterpret_cast<const uint2 *>(s_list), emit);
            STAMP(26);
            n = a.top_k;
        } else {
            auto key = [&](int i) { return ldc(kb + i); };
            n = block_select_topk<NT, 0>(key, L, a.top_k, emit, s_sel);   // rare route: compact code before speed
        }
        __syncthreads();
        // the selected ids, ascending
        {
            int32_t *dst = a.sel + (size_t)ul * a.top_k;
            int32_t *dst2 = a.out_sel ? a.out_sel + (size_t)ul * a.top_k : nullptr;
            for (int pos = tid; pos < a.top_k; pos += NT) {
                int t = -1;
                if (pos < n) t = ldc(cd + (mode == 0 ? pos : s_idx[pos]));
                dst[pos] = t;
                if (dst2) dst2[pos] = t;
            }
            if (tid == 0) a.nsel[ul] = n;
        }
        STAMP(27);
        // picks no block has attended over yet: those of the deciding bucket (mode 1), all of them (mode 2)
        int n_fin = 0;
        if (mode == 1) {
            for (int p0 = 0; p0 < n; p0 += NT) {   // uniform
                const int pos = p0 + tid;
                const int i = s_idx[min(pos, n - 1)];
                const bool fresh = pos < n && !((ldc(gbm + (i >> 5)) >> (i & 31)) & 1u);
                n_fin = block_append_ordered<NT>(fresh, i, s_bpick, n_fin, s_scan);
            }
        } else if (mode == 2) {
            n_fin = n;
        }
        __syncthreads();
        const int32_t *picks = mode == 2 ? s_idx : s_bpick;
        STAMP(28);
        float fmx[G];
        attend_picks<T, G, NT>(n_fin, picks, zb, rb, V, s_red, fmx);
        STAMP(29);
        // merge: the blocks' partial results (not in mode 2: they hold none), this block's, the window's.
        // First the statistics (m, l) of every (partial, head), one per thread, into shared memory, with the
        // window's; then per head the common maximum and each partial's weight; then one pass over the
        // partial outputs, all of a thread's loads in flight together.
        const int np = mode == 2 ? 0 : a.bpu;
        constexpr int NPMAX = 32 + 1 + kWinSplit;                 // blocks, this block, window parts
        float *s_m = reinterpret_cast<float *>(s_reg);            // [NPMAX][G] maxima, then weights
        float *s_l = s_m + NPMAX * G;                             // [NPMAX][G] denominators
        float *s_M = s_l + NPMAX * G;                             // [G] common maximum, [G] total denominator
        const float *pp = a.part + (size_t)ul * a.bpu * G * (2 + kD);
        const float *wp = a.win ? a.win + (size_t)ul * kWinSplit * G * (2 + kD) : nullptr;
        for (int e = tid; e < NPMAX * G; e += NT) {
            const int p = e / G, hh = e - p * G;
            float mv = -__builtin_huge_valf(), lv = 0.0f;
            if (p < np) {
                mv = ldc(pp + ((size_t)p * G + hh) * (2 + kD));
                lv = ldc(pp + ((size_t)p * G + hh) * (2 + kD) + 1);
            } else if (p == 32) {
                mv = pick_head<G>(fmx, hh);
                lv = attend_sum<G, NT>(s_red, hh, kD);
            } else if (p > 32 && wp) {
                mv = wp[((size_t)(p - 33) * G + hh) * (2 + kD)];
                lv = wp[((size_t)(p - 33) * G + hh) * (2 + kD) + 1];
            }
            s_m[e] = mv;
            s_l[e] = lv;
        }
        __syncthreads();
        if (tid < G) {
            float M = -__builtin_huge_valf();
            for (int p = 0; p < NPMAX; ++p)
                if (s_l[p * G + tid] > 0.0f) M = fmaxf(M, s_m[p * G + tid]);
            float den = 0.0f;
            for (int p = 0; p < NPMAX; ++p) {
                const float w = s_l[p * G + tid] > 0.0f ? __expf(s_m[p * G + tid] - M) : 0.0f;
                s_m[p * G + tid] = w;                             // the maximum is no longer needed: its weight
                den += s_l[p * G + tid] * w;
            }
            s_M[tid] = M;
            s_M[G + tid] = den;
        }
        __syncthreads();
        for (int e = tid; e < G * kD; e += NT) {
            const int hh = e >> 7, dim = e & 127;
            const float M = s_M[hh], den = s_M[G + hh];
            float o = 0.0f, lse = -__builtin_huge_valf();
            if (M != -__builtin_huge_valf()) {
                float po[32];
#pragma unroll
                for (int p = 0; p < 32; ++p) po[p] = ldc(pp + ((size_t)min(p, a.bpu - 1) * G + hh) * (2 + kD) + 2 + dim);
                float num = 0.0f;
#pragma unroll
                for (int p = 0; p < 32; ++p) num += p < np ? po[p] * s_m[p * G + hh] : 0.0f;
                num += attend_sum<G, NT>(s_red, hh, dim) * s_m[32 * G + hh];
                if (wp) {
#pragma unroll
                    for (int u = 0; u < kWinSplit; ++u) num += wp[((size_t)u * G + hh) * (2 + kD) + 2 + dim] * s_m[(33 + u) * G + hh];
                }
                o = num / den;
                lse = M + __logf(den);
            }
            a.out[((size_t)b * a.h + kv * G + hh) * kD + dim] = o;
            if (dim == 0 && a.out_lse) a.out_lse[(size_t)b * a.h + kv * G + hh] = lse;
        }
    }
    if (stamp) a.prof[7] = wall_clock64();
}

}  // namespace ctkvr
