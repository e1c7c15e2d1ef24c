// The decode step (Algorithm 2 lines 1-9) as ONE launch: every (sequence, KV head) unit is worked
// on by a fixed group of co-resident blocks that walk the step's phases together, separated by
// per-unit barriers in global memory instead of kernel boundaries.  Block x of a unit owns the key
// ids [x * range, (x + 1) * range) of the sequence from the recall onwards:
//
//   phase 0  cosines of the unit's centroids (lines 1-2), split over the unit's blocks
//   phase 1  every block: top-C' centroids (line 3); the part of every probed list that falls into
//            its own id range -> a bitmap in shared memory (line 4; the lists are ascending, so that
//            part is found from 64 samples per list) -> ids, rows, z = q.k * scale, maxima (line 5)
//   phase 2  ranks of its keys in the unit's recalled list (from all blocks' counts), the unit's
//            maxima; its share of the softmax denominators (integer fixed point)
//   phase 3  ranking keys of its share and their histogram
//   phase 4  every block finds the deciding bin from the summed histograms, classifies its share
//            (sure picks; keys of the deciding bin) and attends over its own sure picks: a
//            partial (m, l, o) per head relative to its own maximum (lines 6-9, split over keys)
//   final    the unit's first block: threshold inside the deciding bin, the selected ids in
//            ascending order, attention over the bin's picks, merge of all partials (and of the
//            resident window's, lines 10-11) -> out, lse
//
// Blocks of different units never wait for each other.  What a block hands to its siblings goes
// through a slot of its own in global memory -- counts, maxima, partial sums, histograms, pick
// lists -- and is combined by every reader: no read-modify-write on a shared word anywhere (such
// atomics are served one after the other).  Every word that another block reads within the launch
// is written with an agent-scope atomic store (written through to memory) and read with an
// agent-scope atomic load (never served from a stale cache line), so correctness does not depend
// on where the blocks run; a unit's blocks sit on one XCD when the number of units is a multiple
// of 8 (workgroups go to the XCDs round-robin), so their traffic meets in one L2.
// Every wait is bounded by the wall clock; on expiry the error word is set and the block leaves.
// The grid must be co-resident: units * blocks-per-unit <= CUs, one block per CU.
#pragma once
#include "arith.hpp"
#include "common.hpp"
#include "fused_args.hpp"
#include "coop.hpp"

namespace ctkvr {

// All threads of the block call this.  wait = false: arrive only (the block has nothing more to
// read from its siblings).  Returns false when the wait expired or another block has reported an
// error: the caller leaves the kernel.
__device__ __forceinline__ bool unit_barrier(uint32_t *ctr, uint32_t members, uint32_t *err, uint32_t *s_flag, bool wait = true)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);   // this thread's stores have been acknowledged
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t ok = 1u;
        if (members > 1u) {
            __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (wait) {
                const long long t0 = wall_clock64();
                uint32_t spins = 0;
                while (ldc(ctr) < members) {
                    if ((++spins & 255u) == 0u && (ldc(err) != 0u || wall_clock64() - t0 > kFusedWaitTicks)) {
                        stc(err, 1u);
                        ok = 0u;
                        break;
                    }
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

// number of entries of the ascending array a[0..n) that are below v
__device__ __forceinline__ int lower_bound_i32(const int32_t *a, int n, int32_t v)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] < v) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// block x' that holds entry e when the blocks' entries are laid end to end: pre[x'] <= e < pre[x' + 1] (pre[0] = 0)
__device__ __forceinline__ int owner_of(const uint32_t *pre, int nblk, uint32_t e)
{
    int xo = 0;
    for (int c = 1; c < nblk; ++c) xo += pre[c] <= e ? 1 : 0;
    return xo;
}

// ranking keys of the single launch fall into kFusedBins bins, 1/8 wide in the log domain (four of
// the 1/32-wide buckets each); bin 0 holds the largest keys
__device__ __forceinline__ uint32_t fused_bin(uint32_t key) { return key_bucket(key) >> 2; }
static_assert(kFusedBins * 4 == kBuckets, "a bin is four buckets");

template <typename T, int G, int NT> __global__ __launch_bounds__(NT) void decode_fused_kernel(FusedArgs a)
{
    constexpr int NW = NT / 64;
    extern __shared__ __align__(16) uint32_t smem[];
    __shared__ uint32_t s_flag, s_scan[24], s_res[4];
    __shared__ uint32_t s_blk[2 * (kFusedMaxBpu + 1) + 2 * kFusedMaxBpu];   // per sibling block: counts, prefixes
    __shared__ uint32_t s_max[G];
    __shared__ float s_ls[G];
    __shared__ unsigned long long s_acc[NW][G];
    uint32_t *s_sel = smem;                                  // kSelLds
    int32_t *s_probe = (int32_t *)(smem + kSelLds);          // n_probe
    uint32_t *s_reg = smem + kSelLds + a.n_probe;            // the phases' common region
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
    const int bpu = a.bpu;
    const int range = fused_range_ids(s_len, bpu);            // key ids per block of THIS unit
    const int lo = min(x * range, s_len), hi = min(lo + range, s_len);
    const int range_words = range >> 5;
    float *s_red;                                             // (NT / 64) * G * 129 words behind the region
    {
        // the region's size as the host computed it (for the longest sequence)
        size_t region = (size_t)((a.stage / bpu) >> 5) + 8 * (size_t)NT + 64;
        const size_t p4 = (size_t)kFusedBins + (size_t)a.top_k + 64;
        const size_t fin = 5 * (size_t)kFusedListCap + 2 * (size_t)a.top_k + 512;
        if (region < p4) region = p4;
        if (region < fin) region = fin;
        s_red = reinterpret_cast<float *>(s_reg + region);
    }
    uint32_t *bar = a.bar + (size_t)ul * kFusedBarriers;
    const bool stamp = a.prof && ul == 0 && x == 0 && tid == 0;
    auto STAMP = [&](int k) {
        if (stamp) a.prof[k] = wall_clock64();
    };
    STAMP(0);

    float *cosv = a.cos + (size_t)ul * a.c_max;
    const size_t st0 = (size_t)ul * a.stage;                  // the unit's staging arrays
    int32_t *sid = a.sid + st0;
    uint32_t *srow = a.srow + st0;
    float *zb = a.z + st0 * G;
    const int own0 = x * range;                               // staging position of this block's first key
    uint32_t *slot_cnt = a.slot_cnt + (size_t)ul * bpu;
    uint32_t *slot_max = a.slot_max + (size_t)ul * bpu * G;
    unsigned long long *slot_S = a.slot_S + (size_t)ul * bpu * G;
    uint32_t *slot_hist = a.slot_hist + (size_t)ul * bpu * kFusedBins;
    uint32_t *slot_npick = a.slot_npick + (size_t)ul * bpu * 2;
    int32_t *slot_sure = a.slot_sure + (size_t)ul * bpu * a.top_k;
    uint4 *slot_bkt = a.slot_bkt + (size_t)ul * bpu * kFusedListCap;
    const T *qb = (const T *)a.q + ((size_t)b * a.h + kv * G) * kD;
    const T *V = (const T *)a.v_pages;

    // ---------------------------------------------------------------- phase 0: cosines
    float q[G][8];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) unpack(load_chunk(qb + (size_t)hh * kD, lane16), q[hh]);
    {
        float inv_q[G];
#pragma unroll
        for (int hh = 0; hh < G; ++hh) inv_q[hh] = inv_norm_from_sq(group16_sum(lane_partial(q[hh], q[hh])));
        const T *cb = (const T *)a.centroids;
        for (int j0 = x * (NT / 16); j0 < C; j0 += bpu * (NT / 16)) {
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
    STAMP(8);
    if (!unit_barrier(bar + 0, (uint32_t)bpu, a.err, &s_flag)) return;
    STAMP(1);

    // ---------------------------------------------------------------- phase 1: probes, own range of the lists, scores
    int cnt_own = 0;
    {
        uint32_t *s_bits = s_reg;                       // range_words
        uint32_t *s_ids = s_reg + range_words;          // 8 * NT: one window of ids, then their rows
        for (int w = tid; w < range_words; w += NT) s_bits[w] = 0u;
        if (tid < G) s_max[tid] = 0u;
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
        // Line 4 for the ids lo .. hi-1.  A list is ascending: lane l of a wave reads its element l * stride,
        // and the 64 samples tell which stretch of the list can hold ids of the range; only that stretch is
        // read.  Four lists per wave at a time, so that their loads travel together.
        if (hi > lo) {
            const int32_t *lb = a.lists + (size_t)ul * a.c_max * a.rho;
            const int stride = (a.rho + 63) >> 6;
            const int sidx = ln * stride;
            for (int p0 = wv; p0 < a.n_probe; p0 += 4 * NW) {
                const int32_t *lp[4];
                int32_t smp[4];
                int first[4], cnt[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    lp[u] = lb + (size_t)s_probe[min(p0 + u * NW, a.n_probe - 1)] * a.rho;
                    smp[u] = lp[u][min(sidx, a.rho - 1)];
                }
                int maxcnt = 0;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int32_t mine = sidx < a.rho ? smp[u] : 0x7fffffff;
                    int32_t nxt = __shfl_down(mine, 1);
                    nxt = ln == 63 ? 0x7fffffff : nxt;
                    const bool need = (p0 + u * NW < a.n_probe) && sidx < a.rho && mine < hi && nxt >= lo;
                    const uint64_t m = __ballot(need);
                    first[u] = 0;
                    cnt[u] = 0;
                    if (m) {
                        const int cf = __ffsll((long long)m) - 1, cl = 63 - __clzll((long long)m);
                        first[u] = cf * stride;
                        cnt[u] = min(a.rho, (cl + 1) * stride) - first[u];
                    }
                    maxcnt = max(maxcnt, cnt[u]);
                }
                for (int off = 0; off < maxcnt; off += 256) {   // uniform
                    int32_t t[4][4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            t[u][k] = lp[u][min(first[u] + min(off + k * 64 + ln, max(cnt[u] - 1, 0)), a.rho - 1)];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const uint32_t rel = (uint32_t)(t[u][k] - lo);
                            if (off + k * 64 + ln < cnt[u] && rel < (uint32_t)(hi - lo)) atomicOr(&s_bits[rel >> 5], 1u << (rel & 31u));
                        }
                }
            }
        }
        __syncthreads();
        STAMP(17);
        // windows of NT bytes of the range's bitmap: a byte per thread -> ids in ascending order -> rows -> scores
        const T *K = (const T *)a.k.pages;
        const int pmask = (1 << a.k.page_shift) - 1;
        const int32_t *bt_row = a.k.block_table + (size_t)b * a.k.max_pages;
        constexpr int R = (sizeof(T) == 2 ? 8 : 4) * (NT == 256 ? 2 : 1);   // rows in flight per 16-lane group
        float mxl = -__builtin_huge_valf();
        const int myh = lane16 & (G - 1);
        for (int w0 = 0; w0 < range_words; w0 += NT / 4) {
            const int wi = w0 + (tid >> 2);
            const uint32_t word = wi < range_words ? s_bits[wi] : 0u;
            uint32_t mine = (word >> ((tid & 3) << 3)) & 0xffu;
            uint32_t nwin;
            uint32_t pos = block_excl_scan<NT>((uint32_t)__popc(mine), s_scan, &nwin);   // barriers inside
            if (nwin == 0u) continue;   // uniform
            const uint32_t id0 = (uint32_t)lo + ((uint32_t)wi << 5) + ((uint32_t)(tid & 3) << 3);
            while (mine) {
                const int bit = __ffs((int)mine) - 1;
                mine &= mine - 1u;
                s_ids[pos++] = id0 + (uint32_t)bit;
            }
            __syncthreads();
            for (int i = tid; i < (int)nwin; i += NT) {
                const int t = (int)s_ids[i];
                const uint32_t row = (uint32_t)((bt_row[t >> a.k.page_shift] * a.g + kv) << a.k.page_shift) + (uint32_t)(t & pmask);
                stc(sid + own0 + cnt_own + i, t);
                stc(srow + own0 + cnt_own + i, row);
                s_ids[i] = row;
            }
            __syncthreads();
            const int last = (int)nwin - 1;
            for (int t0 = 0; t0 <= last; t0 += (NT / 16) * R) {
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
                        if (lane16 < G) stc(zb + (size_t)(own0 + cnt_own + i) * G + lane16, mine_z);
                    }
                }
            }
            cnt_own += (int)nwin;
            __syncthreads();   // the window's rows have been consumed
        }
        STAMP(18);
        {
            float v = mxl;
            v = __builtin_amdgcn_fmed3f(v, __shfl_xor(v, 16), __builtin_huge_valf());
            v = __builtin_amdgcn_fmed3f(v, __shfl_xor(v, 32), __builtin_huge_valf());
            if (ln < G) atomicMax(&s_max[ln], ordered_key(v));
        }
        __syncthreads();
        if (tid < G) stc(slot_max + x * G + tid, s_max[tid]);
        if (tid == 0) stc(slot_cnt + x, (uint32_t)cnt_own);
    }
    STAMP(9);
    if (!unit_barrier(bar + 1, (uint32_t)bpu, a.err, &s_flag)) return;
    STAMP(2);
    if (x == 0 && tid == 0) stc(bar + 0, 0u);   // everyone has left barrier 0 (and so on below)

    // ---------------------------------------------------------------- phase 2: ranks, maxima, denominators
    // s_bcnt[0..bpu): the blocks' counts; s_bpre[0..bpu]: their prefix sums (ranks of their first keys)
    uint32_t *s_bcnt = s_blk, *s_bpre = s_blk + (kFusedMaxBpu + 1);
    int L, base;
    float m[G];
    {
        if (tid < bpu) s_bcnt[tid] = ldc(slot_cnt + tid);
        uint32_t mk[G];
#pragma unroll
        for (int hh = 0; hh < G; ++hh) mk[hh] = ln < bpu ? ldc(slot_max + ln * G + hh) : 0u;
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) mk[hh] = max(mk[hh], (uint32_t)__shfl_xor(mk[hh], o));
            m[hh] = ordered_value(mk[hh]);
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t run = 0;
            for (int c = 0; c < bpu; ++c) {
                s_bpre[c] = run;
                run += s_bcnt[c];
            }
            s_bpre[bpu] = run;
        }
        __syncthreads();
        L = (int)s_bpre[bpu];
        base = (int)s_bpre[x];
        if (x == 0 && tid == 0) {
            a.ncand[ul] = L;
            if (a.out_ncand) a.out_ncand[ul] = L;
        }
        // the recalled list in rank order (inspection, the update, the crowded-bin route)
        int32_t *cd = a.cand + (size_t)ul * a.l_stride;
        for (int i = tid; i < cnt_own; i += NT) stc(cd + base + i, sid[own0 + i]);
        unsigned long long acc[G];
#pragma unroll
        for (int hh = 0; hh < G; ++hh) acc[hh] = 0ull;
        const float *zo = zb + (size_t)own0 * G;
        for (int c0 = 0; c0 < cnt_own; c0 += 4 * NT) {
            uint32_t shi[G], slo[G];
#pragma unroll
            for (int hh = 0; hh < G; ++hh) shi[hh] = slo[hh] = 0u;
            float zv[4][G];
#pragma unroll
            for (int u = 0; u < 4; ++u) load_z<G>(zo, min(c0 + u * NT + tid, cnt_own - 1), zv[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (c0 + u * NT + wv * 64 >= cnt_own) continue;   // nothing for this wave (uniform)
                const bool ok = (c0 + u * NT + tid) < cnt_own;
#pragma unroll
                for (int hh = 0; hh < G; ++hh) {
                    uint32_t hi32, lo32;
                    exp_fixed40_parts(zv[u][hh] - m[hh], hi32, lo32);
                    shi[hh] += ok ? hi32 : 0u;
                    slo[hh] += ok ? lo32 : 0u;
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
            for (int w = 0; w < NW; ++w) v += s_acc[w][tid];
            stc(slot_S + x * G + tid, v);
        }
    }
    STAMP(10);
    if (!unit_barrier(bar + 2, (uint32_t)bpu, a.err, &s_flag)) return;
    STAMP(3);
    if (x == 0 && tid == 0) stc(bar + 1, 0u);

    // ---------------------------------------------------------------- phase 3: ranking keys, histogram
    uint32_t *kb = a.kbuf + (size_t)ul * a.l_stride;
    {
        uint32_t *s_h = s_reg;
        for (int w = tid; w < kFusedBins; w += NT) s_h[w] = 0u;
        if (wv == 0) {   // head hh's denominator: the blocks' shares added by the lanes of the first wave
#pragma unroll
            for (int hh = 0; hh < G; ++hh) {
                unsigned long long v = ln < bpu ? ldc(slot_S + ln * G + hh) : 0ull;
#pragma unroll
                for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
                if (ln == hh) s_ls[hh] = (float)log_fixed40(v);
            }
        }
        __syncthreads();
        float ls[G];
#pragma unroll
        for (int hh = 0; hh < G; ++hh) ls[hh] = s_ls[hh];
        const float *zo = zb + (size_t)own0 * G;
        for (int c0 = 0; c0 < cnt_own; c0 += 4 * NT) {
            float zv[4][G];
#pragma unroll
            for (int u = 0; u < 4; ++u) load_z<G>(zo, min(c0 + u * NT + tid, cnt_own - 1), zv[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (c0 + u * NT + wv * 64 >= cnt_own) continue;   // nothing for this wave (uniform)
                const int i = c0 + u * NT + tid;
                const bool valid = i < cnt_own;
                float best = -__builtin_huge_valf();
#pragma unroll
                for (int hh = 0; hh < G; ++hh) best = fmaxf(best, (zv[u][hh] - m[hh]) - ls[hh]);
                const uint32_t ok = ordered_key(best);
                if (valid) stc(kb + base + i, ok);
                const uint32_t bn = fused_bin(ok);
                const bool tail = valid && bn == (uint32_t)(kFusedBins - 1);
                const uint64_t mt = __ballot(tail);
                if (valid && !tail) atomicAdd(&s_h[bn], 1u);
                if (mt && ln == 0) atomicAdd(&s_h[kFusedBins - 1], (uint32_t)__popcll(mt));
            }
        }
        __syncthreads();
        for (int w = tid; w < kFusedBins; w += NT) stc(slot_hist + (size_t)x * kFusedBins + w, s_h[w]);
    }
    STAMP(11);
    if (!unit_barrier(bar + 3, (uint32_t)bpu, a.err, &s_flag)) return;
    STAMP(4);
    if (x == 0 && tid == 0) stc(bar + 2, 0u);

    // ---------------------------------------------------------------- phase 4: classify, partial attention
    uint32_t bkt = 0, rem = 0, nbk = 0;
    int mode;   // 0: every recalled key is picked; 1: histogram route; 2: the first block selects alone
    {
        uint32_t *s_hs = s_reg;                               // kFusedBins: the unit's histogram
        int32_t *s_pick = (int32_t *)(s_reg + kFusedBins);    // top_k: staging positions of this block's sure picks
        if (a.top_k >= L) {
            mode = 0;
        } else {
            for (int w = tid; w < kFusedBins; w += NT) {
                uint32_t v = 0;
                for (int c0 = 0; c0 < bpu; c0 += 8) {
                    uint32_t t8[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) t8[u] = ldc(slot_hist + (size_t)min(c0 + u, bpu - 1) * kFusedBins + w);
#pragma unroll
                    for (int u = 0; u < 8; ++u) v += c0 + u < bpu ? t8[u] : 0u;
                }
                s_hs[w] = v;
            }
            __syncthreads();
            // thread t owns the bins [t * BPT, (t + 1) * BPT), in descending key order
            constexpr int BPT = (kFusedBins + NT - 1) / NT;
            uint32_t c[BPT], mine = 0;
#pragma unroll
            for (int qq = 0; qq < BPT; ++qq) {
                c[qq] = BPT * tid + qq < kFusedBins ? s_hs[BPT * tid + qq] : 0u;
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
            bkt = s_res[0];
            rem = s_res[1];
            nbk = s_res[2];
            mode = nbk > (uint32_t)kFusedListCap ? 2 : 1;
        }
        STAMP(19);
        int n_sure = 0, n_bkt = 0;
        if (mode == 0) {
            for (int i = tid; i < cnt_own; i += NT) {
                s_pick[i] = own0 + i;
                stc(slot_sure + (size_t)x * a.top_k + i, sid[own0 + i]);
            }
            n_sure = cnt_own;
        } else if (mode == 1) {
            // rounds of NT keys in rank order: the sure picks and the deciding bin's keys keep that order (ascending id)
            for (int c0 = 0; c0 < cnt_own; c0 += NT) {   // uniform
                const int i = c0 + tid;
                const bool valid = i < cnt_own;
                const uint32_t kk = kb[base + min(i, cnt_own - 1)];
                const int32_t id = sid[own0 + min(i, cnt_own - 1)];
                const uint32_t bn = fused_bin(kk);
                const bool sure = valid && bn < bkt, inb = valid && bn == bkt;
                int slot_s, slot_b;
                n_sure = block_ordered_slot<NT>(sure, n_sure, s_scan, slot_s);
                n_bkt = block_ordered_slot<NT>(inb, n_bkt, s_scan, slot_b);
                if (sure) {
                    s_pick[slot_s] = own0 + i;
                    stc(slot_sure + (size_t)x * a.top_k + slot_s, id);
                }
                if (inb) {
                    unsigned long long *dst = reinterpret_cast<unsigned long long *>(slot_bkt + (size_t)x * kFusedListCap + slot_b);
                    stc(dst, (unsigned long long)kk | ((unsigned long long)(uint32_t)(own0 + i) << 32));
                    stc(dst + 1, (unsigned long long)(uint32_t)id);
                }
            }
        }
        if (tid == 0) {
            stc(slot_npick + 2 * x, (uint32_t)n_sure);
            stc(slot_npick + 2 * x + 1, (uint32_t)n_bkt);
        }
        __syncthreads();
        STAMP(20);
        float pmx[G];
        attend_picks<T, G, NT>(n_sure, s_pick, zb, srow, V, s_red, pmx);
        STAMP(21);
        for (int e = tid; e < G * kD; e += NT) {
            const int hh = e >> 7, dim = e & 127;
            float *dst = a.part + (((size_t)ul * bpu + x) * G + hh) * (2 + kD);
            stc(dst + 2 + dim, attend_sum<G, NT>(s_red, hh, dim));
            if (dim == 0) {
                stc(dst, pick_head<G>(pmx, hh));
                stc(dst + 1, attend_sum<G, NT>(s_red, hh, kD));
            }
        }
    }
    STAMP(12);
    // the last barrier: only the unit's first block waits
    if (x != 0) {
        (void)unit_barrier(bar + 4, (uint32_t)bpu, a.err, &s_flag, false);
        return;
    }
    if (!unit_barrier(bar + 4, (uint32_t)bpu, a.err, &s_flag)) return;
    STAMP(5);
    if (tid == 0) {
        stc(bar + 3, 0u);
        stc(bar + 4, 0u);
    }

    // ---------------------------------------------------------------- final: selection, merge
    {
        // the region: the deciding bin's entries as three arrays (keys, staging positions, ids), the winners'
        // places in them, their staging positions, the sure picks' ids, and ids / rank-order positions of picks
        uint32_t *l_key = s_reg;                                       // kFusedListCap
        int32_t *l_st = (int32_t *)(l_key + kFusedListCap);            // kFusedListCap
        int32_t *l_id = l_st + kFusedListCap;                          // kFusedListCap
        int32_t *s_win = l_id + kFusedListCap;                         // kFusedListCap: winners, as places in the arrays above
        int32_t *s_wst = s_win + kFusedListCap;                        // kFusedListCap: their staging positions
        int32_t *s_sure = s_wst + kFusedListCap;                       // top_k: ids of all sure picks, ascending
        int32_t *s_idx = s_sure + a.top_k;                             // top_k: winners' ids; crowded-bin route: positions in rank order
        uint32_t *s_pre_s = s_blk, *s_pre_b = s_blk + (kFusedMaxBpu + 1), *s_tmp = s_blk + 2 * (kFusedMaxBpu + 1);
        int n = 0, n_fin = 0;
        const int32_t *picks = s_wst;
        if (mode != 2) {
            // the blocks' pick counts, laid end to end
            if (tid < 2 * bpu) s_tmp[tid] = ldc(slot_npick + tid);
            __syncthreads();
            if (tid == 0) {
                uint32_t rs = 0, rb2 = 0;
                for (int c = 0; c < bpu; ++c) {
                    s_pre_s[c] = rs;
                    s_pre_b[c] = rb2;
                    rs += s_tmp[2 * c];
                    rb2 += s_tmp[2 * c + 1];
                }
                s_pre_s[bpu] = rs;
                s_pre_b[bpu] = rb2;
            }
            __syncthreads();
            const int ns = (int)s_pre_s[bpu], nb = (int)s_pre_b[bpu];
            for (int e = tid; e < ns; e += NT) {
                const int xo = owner_of(s_pre_s, bpu, (uint32_t)e);
                s_sure[e] = ldc(slot_sure + (size_t)xo * a.top_k + (e - (int)s_pre_s[xo]));
            }
            for (int e = tid; e < nb; e += NT) {
                const int xo = owner_of(s_pre_b, bpu, (uint32_t)e);
                const unsigned long long *src =
                    reinterpret_cast<const unsigned long long *>(slot_bkt + (size_t)xo * kFusedListCap + (e - (int)s_pre_b[xo]));
                const unsigned long long v0 = ldc(src), v1 = ldc(src + 1);
                l_key[e] = (uint32_t)v0;
                l_st[e] = (int32_t)(uint32_t)(v0 >> 32);
                l_id[e] = (int32_t)(uint32_t)v1;
            }
            __syncthreads();
            STAMP(22);
            // the `rem` largest keys of the bin, ties to the lowest id: the entries are in ascending id order, so
            // the selection's own tie rule (lowest place) is the id rule; winners come out in ascending id order
            int nw = 0;
            if (mode == 1) {
                auto key = [&](int i) { return l_key[i]; };
                auto emitw = [&](int pos, int i) { s_win[pos] = i; };
                nw = block_select_topk<NT, kFusedListCap / NT>(key, nb, (int)rem, emitw, s_sel);
                __syncthreads();
            }
            STAMP(23);
            n = ns + nw;
            for (int k = tid; k < nw; k += NT) {
                s_wst[k] = l_st[s_win[k]];
                s_idx[k] = l_id[s_win[k]];
            }
            __syncthreads();
            // merge of the two ascending id sequences: each id's final place is its own place plus the number of
            // ids of the other sequence below it
            int32_t *dst = a.sel + (size_t)ul * a.top_k;
            int32_t *dst2 = a.out_sel ? a.out_sel + (size_t)ul * a.top_k : nullptr;
            for (int j = tid; j < ns; j += NT) {
                const int32_t id = s_sure[j];
                const int pos = j + lower_bound_i32(s_idx, nw, id);
                dst[pos] = id;
                if (dst2) dst2[pos] = id;
            }
            for (int k = tid; k < nw; k += NT) {
                const int32_t id = s_idx[k];
                const int pos = k + lower_bound_i32(s_sure, ns, id);
                dst[pos] = id;
                if (dst2) dst2[pos] = id;
            }
            for (int pos = n + tid; pos < a.top_k; pos += NT) {
                dst[pos] = -1;
                if (dst2) dst2[pos] = -1;
            }
            if (tid == 0) a.nsel[ul] = n;
            n_fin = nw;
        } else {
            // crowded bin (many equal keys, or keys below the histogram's range): this block selects alone, over
            // the unit's keys in rank order, and attends over all the picks itself
            auto key = [&](int i) { return ldc(kb + i); };
            auto emit = [&](int pos, int i) { s_idx[pos] = i; };
            n = block_select_topk<NT, 0>(key, L, a.top_k, emit, s_sel);   // rare route: compact code before speed
            __syncthreads();
            const int32_t *cd = a.cand + (size_t)ul * a.l_stride;
            int32_t *dst = a.sel + (size_t)ul * a.top_k;
            int32_t *dst2 = a.out_sel ? a.out_sel + (size_t)ul * a.top_k : nullptr;
            for (int pos = tid; pos < a.top_k; pos += NT) {
                int32_t t = -1;
                if (pos < n) {
                    const int i = s_idx[pos];
                    t = ldc(cd + i);
                    const int xo = owner_of(s_bpre, bpu, (uint32_t)i);
                    s_sure[pos] = xo * range + (i - (int)s_bpre[xo]);   // its staging position
                }
                dst[pos] = t;
                if (dst2) dst2[pos] = t;
            }
            if (tid == 0) a.nsel[ul] = n;
            picks = s_sure;
            n_fin = n;
        }
        __syncthreads();
        STAMP(24);
        float fmx[G];
        attend_picks<T, G, NT>(n_fin, picks, zb, srow, V, s_red, fmx);
        STAMP(25);
        // merge: the blocks' partial results (not in mode 2: they hold none), this block's, the window's.
        // First the statistics (m, l) of every (partial, head) into shared memory; then per head the common
        // maximum and each partial's weight (one wave per head, a lane per partial); then one pass over the
        // partial outputs, all of a thread's loads in flight together.
        const int np = mode == 2 ? 0 : bpu;
        constexpr int NPMAX = kFusedMaxBpu + 1 + kWinSplit;       // blocks, this block, window parts
        static_assert(NPMAX <= 64, "a lane per partial");
        float *s_m = reinterpret_cast<float *>(s_reg);            // [NPMAX][G] maxima, then weights
        float *s_l = s_m + NPMAX * G;                             // [NPMAX][G] denominators
        float *s_M = s_l + NPMAX * G;                             // [G] common maximum, [G] total denominator
        const float *pp = a.part + (size_t)ul * bpu * G * (2 + kD);
        const float *wp = a.win ? a.win + (size_t)ul * kWinSplit * G * (2 + kD) : nullptr;
        for (int e = tid; e < NPMAX * G; e += NT) {
            const int p = e / G, hh = e - p * G;
            float mv = -__builtin_huge_valf(), lv = 0.0f;
            if (p < np) {
                mv = ldc(pp + ((size_t)p * G + hh) * (2 + kD));
                lv = ldc(pp + ((size_t)p * G + hh) * (2 + kD) + 1);
            } else if (p == kFusedMaxBpu) {
                mv = pick_head<G>(fmx, hh);
                lv = attend_sum<G, NT>(s_red, hh, kD);
            } else if (p > kFusedMaxBpu && wp) {
                mv = wp[((size_t)(p - kFusedMaxBpu - 1) * G + hh) * (2 + kD)];
                lv = wp[((size_t)(p - kFusedMaxBpu - 1) * G + hh) * (2 + kD) + 1];
            }
            s_m[e] = mv;
            s_l[e] = lv;
        }
        __syncthreads();
        for (int hh = wv; hh < G; hh += NW) {   // a wave per head, a lane per partial
            const float mv = ln < NPMAX ? s_m[ln * G + hh] : -__builtin_huge_valf();
            const float lv = ln < NPMAX ? s_l[ln * G + hh] : 0.0f;
            float M = lv > 0.0f ? mv : -__builtin_huge_valf();
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
            const float w = lv > 0.0f ? __expf(mv - M) : 0.0f;
            float den = lv * w;
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) den += __shfl_xor(den, o);
            if (ln < NPMAX) s_m[ln * G + hh] = w;                 // the maximum is no longer needed: its weight
            if (ln == 0) {
                s_M[hh] = M;
                s_M[G + hh] = den;
            }
        }
        __syncthreads();
        for (int e = tid; e < G * kD; e += NT) {
            const int hh = e >> 7, dim = e & 127;
            const float M = s_M[hh], den = s_M[G + hh];
            float o = 0.0f, lse = -__builtin_huge_valf();
            if (M != -__builtin_huge_valf()) {
                float po[kFusedMaxBpu];
#pragma unroll
                for (int p = 0; p < kFusedMaxBpu; ++p) po[p] = ldc(pp + ((size_t)min(p, bpu - 1) * G + hh) * (2 + kD) + 2 + dim);
                float num = 0.0f;
#pragma unroll
                for (int p = 0; p < kFusedMaxBpu; ++p) num += p < np ? po[p] * s_m[p * G + hh] : 0.0f;
                num += attend_sum<G, NT>(s_red, hh, dim) * s_m[kFusedMaxBpu * G + hh];
                if (wp) {
#pragma unroll
                    for (int u = 0; u < kWinSplit; ++u)
                        num += wp[((size_t)u * G + hh) * (2 + kD) + 2 + dim] * s_m[(kFusedMaxBpu + 1 + u) * G + hh];
                }
                o = num / den;
                lse = M + __logf(den);
            }
            a.out[((size_t)b * a.h + kv * G + hh) * kD + dim] = o;
            if (dim == 0 && a.out_lse) a.out_lse[(size_t)b * a.h + kv * G + hh] = lse;
        }
    }
    STAMP(7);
}

}  // namespace ctkvr
