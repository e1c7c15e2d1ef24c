// Fixed arithmetic of every quantity that decides an integer on the CTkvr path
// (which centroids are probed -- Algorithm 2 line 3; which keys enter a list --
// Algorithm 1 line 4; which keys survive the rerank -- Algorithm 2 line 6), and
// the wave/block primitives built on it.  gfx950, wave64.
//
// A 128-element row is owned by 16 adjacent lanes, lane l holding elements
// 8l..8l+7 (one 16-byte load for bf16).  A dot product is 16 lane-partials (a
// sequential fmaf chain over the lane's 8 elements, starting from 0) combined by
// a butterfly over the 16 lanes (xor 1, 2, 4, 8): a fixed balanced tree whose
// value does not depend on which lane looks at it, because a + b == b + a.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ctkvr {

// Development aid (compiled in only with -DCTKVR_TRACE): block (0,0), thread 0 stamps
// the 100 MHz wall clock into g_trace[slot].
#ifdef CTKVR_TRACE
__device__ long long g_trace[128];
#define CTKVR_STAMP(slot)                                                        \
    do {                                                                         \
        if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) g_trace[slot] = wall_clock64(); \
    } while (0)
__device__ long long g_blk[8][2048];
#define CTKVR_STAMP_BLK(slot)                                                    \
    do {                                                                         \
        int bi_ = blockIdx.x + blockIdx.y * gridDim.x;                           \
        if (threadIdx.x == 0 && bi_ < 2048) g_blk[slot][bi_] = wall_clock64();   \
    } while (0)
#else
#define CTKVR_STAMP(slot) do { } while (0)
#define CTKVR_STAMP_BLK(slot) do { } while (0)
#endif

constexpr int kD = 128;          // head dimension
constexpr int kFixShift = 40;    // softmax denominators are summed in 2^-40 fixed point

typedef uint16_t bf16_t;

// ---- raw 8-element chunks ---------------------------------------------------
template <typename T> struct Chunk;
template <> struct Chunk<float> { float4 a, b; };
template <> struct Chunk<bf16_t> { uint4 w; };

__device__ __forceinline__ Chunk<float> load_chunk(const float *row, int lane16)
{
    const float4 *p = reinterpret_cast<const float4 *>(row + 8 * lane16);
    Chunk<float> c;
    c.a = p[0];
    c.b = p[1];
    return c;
}
__device__ __forceinline__ Chunk<bf16_t> load_chunk(const bf16_t *row, int lane16)
{
    Chunk<bf16_t> c;
    c.w = *reinterpret_cast<const uint4 *>(row + 8 * lane16);
    return c;
}
// the same chunks with a non-temporal hint: rows that are read once per step and never again
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ Chunk<float> load_chunk_nt(const float *row, int lane16)
{
    const f32x4_t *p = reinterpret_cast<const f32x4_t *>(row + 8 * lane16);
    const f32x4_t a = __builtin_nontemporal_load(p), b = __builtin_nontemporal_load(p + 1);
    Chunk<float> c;
    c.a = make_float4(a.x, a.y, a.z, a.w);
    c.b = make_float4(b.x, b.y, b.z, b.w);
    return c;
}
__device__ __forceinline__ Chunk<bf16_t> load_chunk_nt(const bf16_t *row, int lane16)
{
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(row + 8 * lane16));
    Chunk<bf16_t> c;
    c.w = make_uint4(v.x, v.y, v.z, v.w);
    return c;
}
__device__ __forceinline__ void unpack(const Chunk<float> &c, float (&x)[8])
{
    x[0] = c.a.x; x[1] = c.a.y; x[2] = c.a.z; x[3] = c.a.w;
    x[4] = c.b.x; x[5] = c.b.y; x[6] = c.b.z; x[7] = c.b.w;
}
__device__ __forceinline__ void unpack(const Chunk<bf16_t> &c, float (&x)[8])
{
    // bf16 -> fp32 is a 16-bit shift: exact
    x[0] = __uint_as_float(c.w.x << 16); x[1] = __uint_as_float(c.w.x & 0xffff0000u);
    x[2] = __uint_as_float(c.w.y << 16); x[3] = __uint_as_float(c.w.y & 0xffff0000u);
    x[4] = __uint_as_float(c.w.z << 16); x[5] = __uint_as_float(c.w.z & 0xffff0000u);
    x[6] = __uint_as_float(c.w.w << 16); x[7] = __uint_as_float(c.w.w & 0xffff0000u);
}

// ---- 16-lane butterfly sum ----------------------------------------------------
// DPP controls: quad_perm[1,0,3,2] = 0xB1, quad_perm[2,3,0,1] = 0x4E,
// row_half_mirror = 0x141, row_mirror = 0x140.  After the two quad steps the four
// lanes of a quad agree, so mirroring within 8 (then 16) lanes pairs each quad
// with the partner the xor-4 (xor-8) step of the butterfly would give it.
template <int CTRL> __device__ __forceinline__ float dpp_f(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float group16_sum(float v)
{
    v = v + dpp_f<0xB1>(v);
    v = v + dpp_f<0x4E>(v);
    v = v + dpp_f<0x141>(v);
    v = v + dpp_f<0x140>(v);
    return v;
}

__device__ __forceinline__ float lane_partial(const float (&a)[8], const float (&b)[8])
{
    float acc = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc = __fmaf_rn(a[e], b[e], acc);
    return acc;
}

// 1/|x| from the squared norm: IEEE sqrt and divide; 0 for the zero vector
__device__ __forceinline__ float inv_norm_from_sq(float n2)
{
    return (n2 > 0.0f) ? (1.0f / sqrtf(n2)) : 0.0f;
}

// ---- exp / fixed point / log ---------------------------------------------------
// exp(x), x <= 0: x = n ln2 + r, degree-7 Taylor polynomial in r, times 2^n.
// Below -30 the term is under 2^-43 and cannot reach the 2^-40 grid: 0.
__device__ __forceinline__ float exp_series(float x)
{
    if (!(x >= -30.0f)) return 0.0f;
    const float kMagic = 12582912.0f;
    float t = __fmaf_rn(x, 1.44269504088896341f, kMagic);
    float n = t - kMagic;
    float r = __fmaf_rn(n, -0.693145751953125f, x);
    r = __fmaf_rn(n, -1.42860682030941723e-6f, r);
    float p = 1.0f / 5040.0f;
    p = __fmaf_rn(p, r, 1.0f / 720.0f);
    p = __fmaf_rn(p, r, 1.0f / 120.0f);
    p = __fmaf_rn(p, r, 1.0f / 24.0f);
    p = __fmaf_rn(p, r, 1.0f / 6.0f);
    p = __fmaf_rn(p, r, 0.5f);
    p = __fmaf_rn(p, r, 1.0f);
    p = __fmaf_rn(p, r, 1.0f);
    float two_n = __uint_as_float((uint32_t)((int)n + 127) << 23);
    return p * two_n;
}

// floor(e * 2^40), 0 <= e < 2, with fp32 and integer operations only
__device__ __forceinline__ uint64_t to_fixed40(float e)
{
    float a = e * 65536.0f;                       // exact
    uint32_t hi = (uint32_t)a;                    // floor
    float rem = a - (float)hi;                    // exact, in [0, 1)
    uint32_t lo = (uint32_t)(rem * 16777216.0f);  // floor(rem * 2^24)
    return ((uint64_t)hi << 24) + lo;
}

// floor(exp_series(x) * 2^40), x <= 0, as hi * 2^24 + lo with lo < 2^24: the value of
// to_fixed40(exp_series(x)) in straight-line code.  x is clamped at -30.5 instead of branching
// (every x below -27.8 gives 0 either way); the power of two enters through the exponent field
// (n is read from the low bits of t, 2^16 added in the same step: exact, as the products it
// replaces are); the fraction is split off with v_fract (exact for a 24-bit value).
__device__ __forceinline__ void exp_fixed40_parts(float x, uint32_t &hi, uint32_t &lo)
{
    const float kMagic = 12582912.0f;
    x = fmaxf(x, -30.5f);
    float t = __fmaf_rn(x, 1.44269504088896341f, kMagic);
    float n = t - kMagic;
    float r = __fmaf_rn(n, -0.693145751953125f, x);
    r = __fmaf_rn(n, -1.42860682030941723e-6f, r);
    float p = 1.0f / 5040.0f;
    p = __fmaf_rn(p, r, 1.0f / 720.0f);
    p = __fmaf_rn(p, r, 1.0f / 120.0f);
    p = __fmaf_rn(p, r, 1.0f / 24.0f);
    p = __fmaf_rn(p, r, 1.0f / 6.0f);
    p = __fmaf_rn(p, r, 0.5f);
    p = __fmaf_rn(p, r, 1.0f);
    p = __fmaf_rn(p, r, 1.0f);
    // a = p * 2^(n + 16): kMagic's low 23 bits are zero, so (bits(t) + 16) << 23 == (n + 16) << 23 mod 2^32
    const float a = __uint_as_float(__float_as_uint(p) + ((__float_as_uint(t) + 16u) << 23));
    hi = (uint32_t)a;
    lo = (uint32_t)(__builtin_amdgcn_fractf(a) * 16777216.0f);
}

// log(S * 2^-40), S >= 1: S = 2^k f, f in [sqrt(1/2), sqrt(2)); log f = 2 atanh((f-1)/(f+1))
__device__ __forceinline__ double log_fixed40(uint64_t S)
{
    if (S == 0) return -__builtin_huge_val();
    int k = 63 - __clzll((long long)S);
    uint64_t mant = (k > 52) ? (S >> (k - 52)) : (S << (52 - k));
    double f = (double)mant * 0x1p-52;
    if (f > 1.4142135623730951) {
        f = f * 0.5;
        k += 1;
    }
    double u = (f - 1.0) / (f + 1.0);
    double u2 = u * u;
    double p = 1.0 / 23.0;
#pragma unroll
    for (int q = 21; q >= 1; q -= 2) p = fma(p, u2, 1.0 / (double)q);
    return fma((double)(k - kFixShift), 0.6931471805599453, 2.0 * u * p);
}

// ---- order-preserving float <-> uint32 ----------------------------------------
// +0.0f first so that -0 and +0 map to one key (they compare equal as floats).
__device__ __forceinline__ uint32_t ordered_key(float x)
{
    uint32_t u = __float_as_uint(x + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ordered_value(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// ---- wave / block helpers -------------------------------------------------------
__device__ __forceinline__ int lane_id() { return __lane_id(); }

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t t = __shfl_up(v, o);
        if (lane_id() >= o) v += t;
    }
    return v;
}

// Exclusive scan of one value per thread over the block; *total gets the sum.
// s_tmp: at least NT/64 + 1 words.  Contains __syncthreads().
template <int NT> __device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t *s_tmp, uint32_t *total)
{
    constexpr int NW = NT / 64;
    uint32_t inc = wave_incl_scan(v);
    int w = threadIdx.x >> 6;
    __syncthreads();
    if (lane_id() == 63) s_tmp[w] = inc;
    __syncthreads();
    if (w == 0) {
        uint32_t t = (lane_id() < NW) ? s_tmp[lane_id()] : 0u;
        uint32_t ti = wave_incl_scan(t);
        if (lane_id() < NW) s_tmp[lane_id()] = ti - t;
        if (lane_id() == NW - 1) s_tmp[NW] = ti;
    }
    __syncthreads();
    uint32_t r = s_tmp[w] + inc - v;
    *total = s_tmp[NW];
    return r;
}

// Two exclusive scans at once (same barriers as one).  s_tmp: 2 * (NT / 64 + 1) words.
template <int NT>
__device__ __forceinline__ void block_excl_scan2(uint32_t va, uint32_t vb, uint32_t *s_tmp, uint32_t &ra, uint32_t &rb)
{
    constexpr int NW = NT / 64;
    const uint32_t ia = wave_incl_scan(va), ib = wave_incl_scan(vb);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if (lane_id() == 63) {
        s_tmp[w] = ia;
        s_tmp[NW + 1 + w] = ib;
    }
    __syncthreads();
    if (w == 0) {
        const uint32_t ta = (lane_id() < NW) ? s_tmp[lane_id()] : 0u, tb = (lane_id() < NW) ? s_tmp[NW + 1 + lane_id()] : 0u;
        const uint32_t sa = wave_incl_scan(ta), sb = wave_incl_scan(tb);
        if (lane_id() < NW) {
            s_tmp[lane_id()] = sa - ta;
            s_tmp[NW + 1 + lane_id()] = sb - tb;
        }
    }
    __syncthreads();
    ra = s_tmp[w] + ia - va;
    rb = s_tmp[NW + 1 + w] + ib - vb;
}

// ---- block-wide top-k selection ---------------------------------------------------
// Shared-memory words the selection routines need at `s_hist`: 2048 histogram bins, then
// [0] lo, [1] hi, [2] bin, [3] remaining, scan scratch, wave counts, and two words at +56.
//
// block_kth_largest: T = the k-th largest of the keys that `for_slots` enumerates (as
// f(id, valid, key), the same sequence in every call, ids distinct), and need_eq = how many of
// the keys equal to T belong to the k largest.  MSB-first radix select on 11-bit digits,
// starting at the highest bit in which the keys differ at all (one min/max pass); when at most
// 128 keys share the deciding digit they are gathered and ranked against each other instead of
// walking the remaining digits.  Every thread of the block takes part; 1 <= k <= number of keys.
template <int NT, typename SlotsFn>
__device__ __forceinline__ void block_kth_largest(SlotsFn for_slots, uint32_t k, uint32_t *s_hist, uint32_t &T,
                                                  uint32_t &need_eq)
{
    const int tid = threadIdx.x;
    const int ln = lane_id();
    uint32_t *s_aux = s_hist + 2048;
    uint32_t *s_scan = s_aux + 4;
    uint32_t *s_x = s_hist + 2048 + 56;   // [0] population of the deciding bin, [1] gather cursor
    // pass 0: range of the keys
    uint32_t lo = 0xffffffffu, hi = 0u;
    for_slots([&](int, bool valid, uint32_t kk) {
        if (valid) {
            lo = min(lo, kk);
            hi = max(hi, kk);
        }
    });
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        lo = min(lo, (uint32_t)__shfl_xor(lo, o));
        hi = max(hi, (uint32_t)__shfl_xor(hi, o));
    }
    __syncthreads();
    if (tid == 0) { s_aux[0] = 0xffffffffu; s_aux[1] = 0u; }
    __syncthreads();
    if (ln == 0) { atomicMin(&s_aux[0], lo); atomicMax(&s_aux[1], hi); }
    __syncthreads();
    lo = s_aux[0];
    hi = s_aux[1];
    uint32_t prefix = hi, pmask = 0xffffffffu;
    uint32_t remaining = k;
    int bit = 0;   // number of still undecided low bits
    if (lo != hi) {
        bit = 32 - __clz((int)(lo ^ hi));
        pmask = (bit >= 32) ? 0u : ~((1u << bit) - 1u);
        prefix = hi & pmask;
    }
    while (bit > 0) {
        const int w = bit < 11 ? bit : 11;
        const int shift = bit - w;
        const uint32_t dmask = (1u << w) - 1u;
        const int nbins = 1 << w;
        __syncthreads();
        for (int i = tid; i < nbins; i += NT) s_hist[i] = 0;
        __syncthreads();
        for_slots([&](int, bool valid, uint32_t kk) {
            if (valid && (kk & pmask) == prefix) atomicAdd(&s_hist[(kk >> shift) & dmask], 1u);
        });
        __syncthreads();
        // walk the bins from the top: thread t owns the BPT bins below nbins - BPT*t
        constexpr int BPT = 2048 / NT;
        uint32_t c[BPT];
        uint32_t mine = 0;
#pragma unroll
        for (int q = 0; q < BPT; ++q) {
            int bq = nbins - 1 - (BPT * tid + q);
            c[q] = (bq >= 0) ? s_hist[bq] : 0u;
            mine += c[q];
        }
        uint32_t tot;
        uint32_t before = block_excl_scan<NT>(mine, s_scan, &tot);
#pragma unroll
        for (int q = 0; q < BPT; ++q) {
            int bq = nbins - 1 - (BPT * tid + q);
            if (bq >= 0 && before < remaining && remaining <= before + c[q]) {
                s_aux[2] = (uint32_t)bq;
                s_aux[3] = remaining - before;
                s_x[0] = c[q];
                s_x[1] = 0u;
            }
            before += c[q];
        }
        __syncthreads();
        prefix |= s_aux[2] << shift;
        pmask |= dmask << shift;
        remaining = s_aux[3];
        bit = shift;
        const uint32_t nb = s_x[0];
        if (bit > 0 && nb <= 128u) {   // ranking is quadratic in nb: only when it is cheaper than another digit
            // The key of rank `remaining` among the gathered ones is T.  Ids only make the ranks
            // distinct here: which of the keys equal to T are picked is decided by the caller.
            uint32_t *l_key = s_hist, *l_idx = s_hist + 1024;
            __syncthreads();   // the histogram has been read by everyone
            for_slots([&](int i, bool valid, uint32_t kk) {
                if (valid && (kk & pmask) == prefix) {
                    uint32_t at = atomicAdd(&s_x[1], 1u);
                    l_key[at] = kk;
                    l_idx[at] = (uint32_t)i;
                }
            });
            __syncthreads();
            for (uint32_t j = tid; j < nb; j += NT) {
                const uint32_t mk = l_key[j], mi = l_idx[j];
                uint32_t rank = 0, gt = 0;
                for (uint32_t e = 0; e < nb; ++e) {
                    const uint32_t ke = l_key[e], ie = l_idx[e];
                    gt += (ke > mk);
                    rank += (ke > mk) || (ke == mk && ie < mi);
                }
                if (rank == remaining - 1u) {
                    s_aux[2] = mk;
                    s_aux[3] = remaining - gt;
                }
            }
            __syncthreads();
            prefix = s_aux[2];
            pmask = 0xffffffffu;
            remaining = s_aux[3];
            bit = 0;
        }
    }
    T = prefix;
    need_eq = remaining;
}

// block_select_topk: among keys key(i), i in [0, n), pick the k largest, ties towards the
// lowest i, and call emit(pos, i) with pos = rank of i among the picked in ascending i.
// One block of NT threads; s_hist needs 2048 + 64 words.  Returns min(n, k) to every thread.
//
// Layout: wave w owns the contiguous ids [w*per, (w+1)*per), lane-strided inside,
// per = a multiple of 64 covering n/NW.  With KPT > 0 each thread keeps its keys
// in KPT registers (needs n <= NT*KPT) and key() is called once per id; with
// KPT == 0 key() is called again in every pass.
//
// After block_kth_largest the picks are compacted in order: each wave counts its range, one scan
// over the wave totals, and every wave writes its picks in place with ballot ranks -- no atomics
// decide an order.
template <int NT, int KPT, typename KeyFn, typename EmitFn>
__device__ int block_select_topk(KeyFn key, int n, int k, EmitFn emit, uint32_t *s_hist)
{
    constexpr int NW = NT / 64;
    const int tid = threadIdx.x;
    const int wv = tid >> 6, ln = lane_id();
    uint32_t *s_scan = s_hist + 2048 + 4;
    if (k >= n) {
        for (int i = tid; i < n; i += NT) emit(i, i);
        return n;
    }
    const int per = ((n + NW - 1) / NW + 63) & ~63;
    const int beg = wv * per;
    const int end = min(n, beg + per);
    uint32_t kreg[KPT > 0 ? KPT : 1];
    if constexpr (KPT > 0) {
#pragma unroll
        for (int it = 0; it < KPT; ++it) kreg[it] = key(min(beg + it * 64 + ln, n - 1));   // clamped, then masked: the loads go out together
#pragma unroll
        for (int it = 0; it < KPT; ++it)
            if (beg + it * 64 + ln >= end) kreg[it] = 0u;
    }
    // f(i, valid, key) for every slot of this thread, wave-uniform trip count
    auto for_slots = [&](auto f) __attribute__((always_inline)) {
        if constexpr (KPT > 0) {
#pragma unroll
            for (int it = 0; it < KPT; ++it) {
                if (beg + it * 64 >= end) break;
                int i = beg + it * 64 + ln;
                f(i, i < end, kreg[it]);
            }
        } else {
            constexpr int CH = 16;   // keys fetched together, so that their loads overlap
            for (int base = beg; base < end; base += 64 * CH) {
                uint32_t kk[CH];
#pragma unroll
                for (int c = 0; c < CH; ++c) kk[c] = key(min(base + c * 64 + ln, n - 1));
#pragma unroll
                for (int c = 0; c < CH; ++c)
                    if (base + c * 64 + ln >= end) kk[c] = 0u;
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    if (base + c * 64 >= end) break;
                    int i = base + c * 64 + ln;
                    f(i, i < end, kk[c]);
                }
            }
        }
    };
    uint32_t T, need_eq;
    block_kth_largest<NT>(for_slots, (uint32_t)k, s_hist, T, need_eq);
    // ordered compaction
    uint32_t cgt = 0, ceq = 0;
    for_slots([&](int, bool valid, uint32_t kk) {
        cgt += (valid && kk > T);
        ceq += (valid && kk == T);
    });
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        cgt += __shfl_xor(cgt, o);
        ceq += __shfl_xor(ceq, o);
    }
    uint32_t *s_cnt = s_scan + NW + 1;
    __syncthreads();
    if (ln == 0) { s_cnt[2 * wv] = cgt; s_cnt[2 * wv + 1] = ceq; }
    __syncthreads();
    uint32_t run_gt = 0, run_eq = 0;
    for (int q = 0; q < wv; ++q) { run_gt += s_cnt[2 * q]; run_eq += s_cnt[2 * q + 1]; }
    const uint64_t below = (1ull << ln) - 1ull;
    for_slots([&](int i, bool valid, uint32_t kk) {
        bool gt = valid && kk > T, eq = valid && kk == T;
        uint64_t mg = __ballot(gt), me = __ballot(eq);
        uint32_t gt_before = run_gt + (uint32_t)__popcll(mg & below);
        uint32_t eq_before = run_eq + (uint32_t)__popcll(me & below);
        if (gt || (eq && eq_before < need_eq)) emit((int)(gt_before + min(eq_before, need_eq)), i);
        run_gt += (uint32_t)__popcll(mg);
        run_eq += (uint32_t)__popcll(me);
    });
    return k;
}

// ---- top-k selection helped by a histogram of the keys ---------------------------------
constexpr int kBuckets = 2048;
constexpr int kListCap = 2048;

// bucket 0 holds the largest keys: buckets are 1/32 wide in the log domain down to -64,
// everything below shares the last one.  Monotone in the key.
__device__ __forceinline__ uint32_t key_bucket(uint32_t kk)
{
    float t = fminf(-ordered_value(kk) * 32.0f, (float)(kBuckets - 1));
    return (uint32_t)fmaxf(t, 0.0f);
}

// T = the rem-th largest of the keys l_ent[0..nb).x (in shared memory), and need_eq = how many of the
// keys equal to T belong to the rem largest.  Every thread of the block takes part; barriers inside.
// s_hist: the 2048 + 64 words of the selection routines.  1 <= rem <= nb <= CAP.
template <int NT, int CAP = kListCap>
__device__ __forceinline__ void block_list_threshold(uint32_t nb, uint32_t rem, uint32_t *s_hist, const uint2 *l_ent, uint32_t &T,
                                                     uint32_t &need_eq)
{
    const int tid = threadIdx.x;
    static_assert(NT <= 1024, "rank counters live in the two halves of the 2048-word histogram");
    if (nb <= (uint32_t)NT / 2) {
        // Few enough to rank every listed key against all the others: the comparisons of one key
        // are split over NT/cap threads (cap = nb rounded up to a power of two, at least a wave, so
        // that the lanes of a wave walk the list together) and their counts meet in shared memory.
        uint32_t *s_aux = s_hist + 2048;
        uint32_t cap = 64;
        while (cap < nb) cap <<= 1;
        const uint32_t parts = (uint32_t)NT / cap, e = (uint32_t)tid & (cap - 1u), part = (uint32_t)tid / cap;
        for (int w = tid; w < 2048; w += NT) s_hist[w] = 0u;
        __syncthreads();
        if (e < nb) {
            const uint32_t mk = l_ent[e].x;
            uint32_t rank = 0, gt = 0;
            for (uint32_t f = part; f < nb; f += parts) {
                const uint32_t ke = l_ent[f].x;
                gt += (ke > mk);
                rank += (ke > mk) || (ke == mk && f < e);
            }
            atomicAdd(&s_hist[e], rank);
            atomicAdd(&s_hist[1024 + e], gt);
        }
        __syncthreads();
        if ((uint32_t)tid < nb && s_hist[tid] == rem - 1u) {
            s_aux[2] = l_ent[tid].x;
            s_aux[3] = rem - s_hist[1024 + tid];
        }
        __syncthreads();
        T = s_aux[2];
        need_eq = s_aux[3];
    } else {
        auto for_list = [&](auto f) __attribute__((always_inline)) {
#pragma unroll
            for (int q = 0; q < CAP / NT; ++q) {
                const uint32_t e = (uint32_t)(q * NT + tid);
                const bool valid = e < nb;
                f((int)e, valid, valid ? l_ent[e].x : 0u);
            }
        };
        block_kth_largest<NT>(for_list, rem, s_hist, T, need_eq);
    }
}

// Second half of the histogram-helped selection, on data already in shared memory: s_gt = bitmap
// of the ids above the deciding bucket, s_eq = zeroed bitmap, l_ent[0..nb) = the (key, id) pairs
// of the deciding bucket, of which the `rem` largest keys are still wanted (ties: lowest ids).
// n ids in all (both bitmaps have 2*ceil(n/64) words).  Starts with the data as written by other
// threads: the caller places a barrier before the call.
template <int NT, int CAP = kListCap, typename EmitFn>
__device__ __forceinline__ void block_resolve_emit(uint32_t nb, uint32_t rem, int n, uint32_t *s_hist, uint32_t *s_gt,
                                                   uint32_t *s_eq, const uint2 *l_ent, EmitFn emit)
{
    const int tid = threadIdx.x;
    uint32_t *s_scan = s_hist + 2048 + 4;
    const int nw64 = (n + 63) >> 6;
    uint32_t T, need_eq;
    block_list_threshold<NT, CAP>(nb, rem, s_hist, l_ent, T, need_eq);
    __syncthreads();
    CTKVR_STAMP(35);
    for (uint32_t e = tid; e < nb; e += NT) {
        const uint2 en = l_ent[e];
        if (en.x > T) atomicOr(&s_gt[en.y >> 5], 1u << (en.y & 31u));
        if (en.x == T) atomicOr(&s_eq[en.y >> 5], 1u << (en.y & 31u));
    }
    __syncthreads();
    CTKVR_STAMP(36);
    // thread t owns the words [t*wpt, (t+1)*wpt) of both bitmaps: count, scan, emit in order
    const int nw32 = 2 * nw64;
    const int wpt = (nw32 + NT - 1) / NT;
    const int w0 = min(nw32, tid * wpt), w1 = min(nw32, w0 + wpt);
    uint32_t cgt = 0, ceq = 0;
    for (int w = w0; w < w1; ++w) {
        cgt += (uint32_t)__popc(s_gt[w]);
        ceq += (uint32_t)__popc(s_eq[w]);
    }
    uint32_t gt_before, eq_before;
    block_excl_scan2<NT>(cgt, ceq, s_scan, gt_before, eq_before);
    uint32_t pos = gt_before + min(eq_before, need_eq);
    CTKVR_STAMP(38);
    for (int w = w0; w < w1; ++w) {
        const uint32_t mg = s_gt[w], me = s_eq[w];
        uint32_t m = mg | me;
        while (m) {
            const int bpos = __ffs((int)m) - 1;
            const uint32_t one = 1u << bpos;
            m &= m - 1u;
            if (mg & one) {
                emit((int)pos++, w * 32 + bpos);
            } else {
                if (eq_before < need_eq) emit((int)pos++, w * 32 + bpos);
                ++eq_before;
            }
        }
    }
}

// Same contract as block_select_topk, for keys keys[0..n) that are images of log-probabilities (<= 0) and
// come with a histogram `ghist` (kBuckets counts) over key_bucket(), built beforehand by a
// chip-wide kernel.  One scan of the histogram names the bucket that holds the k-th key; then ONE
// pass over the keys writes a bitmap of the ids in higher buckets (ballots, no atomics) and
// appends the (key, id) pairs of the deciding bucket to a list in shared memory.  The k-th key T
// is found inside that list (block_kth_largest over at most kListCap entries); list entries above
// T join the bitmap, entries equal to T go to a second bitmap, and a popcount scan over both
// emits the picks in ascending id order, the lowest ids among the keys equal to T first.
//   s_bits : 4 * ceil(n / 64) words (two bitmaps), s_list : 2 * kListCap words.
// Returns -1 to every thread, with nothing emitted, when the deciding bucket holds more than
// kListCap keys (many equal keys, or keys below the histogram's range): the caller then takes
// block_select_topk.
template <int NT, typename EmitFn>
__device__ int block_select_hist(const uint32_t *keys, int n, int k, EmitFn emit, uint32_t *s_hist, uint32_t *s_bits,
                                 uint32_t *s_list, const uint32_t *ghist)
{
    constexpr int NW = NT / 64;
    const int tid = threadIdx.x;
    const int wv = tid >> 6, ln = lane_id();
    uint32_t *s_aux = s_hist + 2048;
    uint32_t *s_scan = s_aux + 4;
    uint32_t *s_x = s_hist + 2048 + 56;
    if (k >= n) {
        for (int i = tid; i < n; i += NT) emit(i, i);
        return n;
    }
    // Wave w owns the contiguous ids [beg, end) in groups of 256: slot c of lane l holds the four
    // ids beg + 256 c + 4 l .. + 3, one 16-byte load (one CU sustains few requests in flight, so
    // they should be wide).  The first CH slots of every thread are requested before the histogram
    // is looked at, so that both latencies overlap.
    const int per = ((n + NW - 1) / NW + 255) & ~255;
    const int beg = wv * per;
    const int end = min(n, beg + per);
    constexpr int CH = 8;
    const bool wide = (reinterpret_cast<uintptr_t>(keys) & 15u) == 0;
    auto load4 = [&](int i) {
        uint4 v;
        if (wide && i + 3 < end) {
            v = *reinterpret_cast<const uint4 *>(keys + i);
        } else {
            v.x = i < end ? keys[i] : 0u;
            v.y = i + 1 < end ? keys[i + 1] : 0u;
            v.z = i + 2 < end ? keys[i + 2] : 0u;
            v.w = i + 3 < end ? keys[i + 3] : 0u;
        }
        return v;
    };
    // A round that lies wholly inside the wave's range takes plain 16-byte loads, all requested
    // together (a load under a per-lane condition is waited for before the next is requested).
    uint4 kv[CH];
    if (wide && beg + 256 * CH <= end) {
#pragma unroll
        for (int c = 0; c < CH; ++c) kv[c] = *reinterpret_cast<const uint4 *>(keys + beg + 256 * c + 4 * ln);
    } else {
#pragma unroll
        for (int c = 0; c < CH; ++c) kv[c] = load4(beg + 256 * c + 4 * ln);
    }
    CTKVR_STAMP(32);
    // the bucket of the k-th key, and how many of its keys are still wanted
    {
        constexpr int BPB = kBuckets / NT;   // buckets per thread, in descending key order
        uint32_t c[BPB];
        uint32_t mine = 0;
#pragma unroll
        for (int q = 0; q < BPB; ++q) {
            c[q] = ghist[BPB * tid + q];
            mine += c[q];
        }
        uint32_t tot;
        uint32_t before = block_excl_scan<NT>(mine, s_scan, &tot);
#pragma unroll
        for (int q = 0; q < BPB; ++q) {
            if (before < (uint32_t)k && (uint32_t)k <= before + c[q]) {
                s_aux[2] = (uint32_t)(BPB * tid + q);
                s_aux[3] = (uint32_t)k - before;
                s_x[0] = c[q];
                s_x[1] = 0u;
            }
            before += c[q];
        }
        __syncthreads();
    }
    const uint32_t bkt = s_aux[2], rem = s_aux[3], nb = s_x[0];
    if (nb > (uint32_t)kListCap) {
        __syncthreads();
        return -1;
    }
    CTKVR_STAMP(33);
    const int nw64 = (n + 63) >> 6;
    uint32_t *s_gt = s_bits, *s_eq = s_bits + 2 * nw64;
    unsigned char *b_gt = reinterpret_cast<unsigned char *>(s_gt), *b_eq = reinterpret_cast<unsigned char *>(s_eq);
    uint2 *l_ent = reinterpret_cast<uint2 *>(s_list);
    // The one pass over the keys.  A lane's four verdicts are a nibble; neighbouring lanes pair
    // theirs into the byte of the bitmap that covers their eight ids (even lanes store it, odd lanes
    // clear the same byte of the second bitmap).
    const uint64_t below = (1ull << ln) - 1ull;
    for (int base = beg; base < end; base += 256 * CH) {
        if (base != beg) {
            if (wide && base + 256 * CH <= end) {
#pragma unroll
                for (int c = 0; c < CH; ++c) kv[c] = *reinterpret_cast<const uint4 *>(keys + base + 256 * c + 4 * ln);
            } else {
#pragma unroll
                for (int c = 0; c < CH; ++c) kv[c] = load4(base + 256 * c + 4 * ln);
            }
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int i0 = base + 256 * c;
            if (i0 < end) {
                const int i = i0 + 4 * ln;
                const uint32_t k4[4] = {kv[c].x, kv[c].y, kv[c].z, kv[c].w};
                uint32_t nib = 0;
                bool inb[4], any_inb = false;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool valid = i + e < end;
                    const uint32_t bk = key_bucket(k4[e]);
                    nib |= (uint32_t)(valid && bk < bkt) << e;
                    inb[e] = valid && bk == bkt;
                    any_inb |= inb[e];
                }
                const uint32_t other = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)nib, 0xB1, 0xF, 0xF, false);   // neighbour's
                const int byte_idx = (i0 >> 3) + (ln >> 1);
                if (byte_idx < nw64 * 8) {
                    if (ln & 1)
                        b_eq[byte_idx] = 0;
                    else
                        b_gt[byte_idx] = (unsigned char)(nib | (other << 4));
                }
                if (__ballot(any_inb)) {   // some key of the deciding bucket: one cursor bump per wave and position
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint64_t listed = __ballot(inb[e]);
                        if (listed) {
                            uint32_t at0 = 0;
                            if (ln == 0) at0 = atomicAdd(&s_x[1], (uint32_t)__popcll(listed));
                            at0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)at0);
                            if (inb[e]) l_ent[at0 + (uint32_t)__popcll(listed & below)] = make_uint2(k4[e], (uint32_t)(i + e));
                        }
                    }
                }
            }
        }
    }
    __syncthreads();
    CTKVR_STAMP(34);
    block_resolve_emit<NT>(nb, rem, n, s_hist, s_gt, s_eq, l_ent, emit);
    CTKVR_STAMP(39);
    return k;
}

// The same selection when a chip-wide kernel has already made the pass over the keys: gbm = its
// bitmap of the ids above the deciding bucket (2*ceil(n/64) words), glist[0..nb) = that bucket's
// (key, id) pairs, both in global memory.  s_bits: 4*ceil(n/64) words, s_list: 2*nb words.
template <int NT, typename EmitFn>
__device__ int block_select_classified(int n, int k, uint32_t rem, uint32_t nb, const uint32_t *gbm, const uint2 *glist,
                                       EmitFn emit, uint32_t *s_hist, uint32_t *s_bits, uint32_t *s_list)
{
    const int tid = threadIdx.x;
    const int nw32 = 2 * ((n + 63) >> 6);
    uint32_t *s_gt = s_bits, *s_eq = s_bits + nw32;
    uint2 *l_ent = reinterpret_cast<uint2 *>(s_list);
    for (uint32_t e = tid; e < nb; e += NT) l_ent[e] = glist[e];
    for (int w = tid; w < nw32; w += NT) {
        s_gt[w] = gbm[w];
        s_eq[w] = 0u;
    }
    __syncthreads();
    CTKVR_STAMP(34);
    block_resolve_emit<NT>(nb, rem, n, s_hist, s_gt, s_eq, l_ent, emit);
    CTKVR_STAMP(39);
    return k;
}

}  // namespace ctkvr

namespace ctkvr {

// Sum of one value per lane over the wave, returned as a wave-uniform value: DPP butterfly inside
// each 16-lane row (full-rate, no LDS), then four scalar lane reads.
__device__ __forceinline__ uint32_t wave_sum_uniform(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, false);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, false);
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 0) + (uint32_t)__builtin_amdgcn_readlane((int)v, 16) +
           (uint32_t)__builtin_amdgcn_readlane((int)v, 32) + (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
}

// ---- small-n top-k selection by bisection ----------------------------------------------
// Same contract as block_select_topk for n <= NT*KPT keys held in registers (slot it of
// thread t is id it*NT + t).  The k-th largest key is found two bits at a time from the top: up to
// 16 rounds of "how many keys are >= candidate" for three candidates (ballot counts per wave, one
// block barrier per round), stopping early at a candidate that exactly k keys reach; then the
// picks are written in ascending id order with ballot ranks.  s_tmp: 6*(NT/64) + 2*KPT*(NT/64) words.  Every thread of the block takes part.
template <int NT, int KPT, typename KeyFn, typename EmitFn>
__device__ __forceinline__ void block_bisect_topk(KeyFn key, int n, int k, EmitFn emit, uint32_t *s_tmp)
{
    constexpr int NW = NT / 64;
    const int tid = threadIdx.x, wv = tid >> 6, ln = lane_id();
    if (k >= n) {
        for (int i = tid; i < n; i += NT) emit(i, i);
        return;
    }
    // slots beyond n hold key 0: below every candidate (candidates are >= 1) and below every real key
    // (loaded at clamped ids and then masked: a load under a per-lane condition would be waited for
    // before the next one is requested)
    uint32_t kreg[KPT];
#pragma unroll
    for (int it = 0; it < KPT; ++it) kreg[it] = key(min(it * NT + tid, n - 1));
#pragma unroll
    for (int it = 0; it < KPT; ++it)
        if (it * NT + tid >= n) kreg[it] = 0u;
    CTKVR_STAMP(13);
    // two bits per round: the counts for the three candidates T|01, T|10, T|11 (times 2^b) are
    // monotone, so the largest candidate still reaching k keys fixes both bits
    uint32_t T = 0;
    for (int b = 30; b >= 0; b -= 2) {
        const uint32_t c1 = T | (1u << b), c2 = T | (2u << b), c3 = T | (3u << b);
        // a compare leaves a 64-bit lane mask; its population count is the wave's count, all scalar
        uint32_t n1 = 0, n2 = 0, n3 = 0;
#pragma unroll
        for (int it = 0; it < KPT; ++it) {
            n1 += (uint32_t)__popcll(__ballot(kreg[it] >= c1));
            n2 += (uint32_t)__popcll(__ballot(kreg[it] >= c2));
            n3 += (uint32_t)__popcll(__ballot(kreg[it] >= c3));
        }
        uint32_t *buf = s_tmp + ((b >> 1) & 1) * 3 * NW;
        if (ln == 0) {
            buf[wv] = n1;
            buf[NW + wv] = n2;
            buf[2 * NW + wv] = n3;
        }
        __syncthreads();
        uint32_t t1 = 0, t2 = 0, t3 = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            t1 += buf[w];
            t2 += buf[NW + w];
            t3 += buf[2 * NW + w];
        }
        if (t3 >= (uint32_t)k) T = c3;
        else if (t2 >= (uint32_t)k) T = c2;
        else if (t1 >= (uint32_t)k) T = c1;
        // A candidate that exactly k keys reach separates the pick from the rest: the keys >= it
        // are the answer and the remaining bits need not be resolved.  (Every thread sees the same
        // totals, so the exit is uniform.)  Never taken while keys tie at the k-th place.
        const uint32_t hit = (t3 == (uint32_t)k) ? c3 : (t2 == (uint32_t)k) ? c2 : (t1 == (uint32_t)k) ? c1 : 0u;
        if (hit) {
            T = hit - 1u;   // "above T" is then "at least hit"; no key equal to T is wanted
            break;
        }
    }
    CTKVR_STAMP(14);
    // T is now the k-th largest key; keys above it are all picked, ties by lowest id.
    // Ordered compaction: ids ascend with (slot, wave, lane).
    uint32_t *s_gt = s_tmp + 6 * NW, *s_eq = s_gt + KPT * NW;
    const uint64_t below = (1ull << ln) - 1ull;
#pragma unroll
    for (int it = 0; it < KPT; ++it) {
        const bool valid = (it * NT + tid) < n;
        const uint64_t mg = __ballot(valid && kreg[it] > T), me = __ballot(valid && kreg[it] == T);
        if (ln == 0) {
            s_gt[it * NW + wv] = (uint32_t)__popcll(mg);
            s_eq[it * NW + wv] = (uint32_t)__popcll(me);
        }
    }
    __syncthreads();
    uint32_t tot_gt = 0;
    for (int q = 0; q < KPT * NW; ++q) tot_gt += s_gt[q];
    const uint32_t need_eq = (uint32_t)k - tot_gt;
    uint32_t run_gt = 0, run_eq = 0;
#pragma unroll
    for (int it = 0; it < KPT; ++it) {
        // counts of everything before (it, wv)
        uint32_t pg = run_gt, pe = run_eq;
        for (int w = 0; w < NW; ++w) {
            if (w < wv) { pg += s_gt[it * NW + w]; pe += s_eq[it * NW + w]; }
            run_gt += s_gt[it * NW + w];
            run_eq += s_eq[it * NW + w];
        }
        const int i = it * NT + tid;
        const bool valid = i < n;
        const bool g = valid && kreg[it] > T, e = valid && kreg[it] == T;
        const uint64_t mg = __ballot(g), me = __ballot(e);
        const uint32_t gb = pg + (uint32_t)__popcll(mg & below);
        const uint32_t eb = pe + (uint32_t)__popcll(me & below);
        if (g || (e && eb < need_eq)) emit((int)(gb + min(eb, need_eq)), i);
    }
}

// ---- top-k for very small k (k <= 8) by repeated extraction ---------------------------------
// Same contract as block_bisect_topk.  Each round takes the block-wide maximum of (key, lowest id)
// (a 64-bit composite: wave reduction, one barrier), records it and retires it in its owner's
// register; k rounds instead of sixteen rounds of ballot counts.  The picks are then written in
// ascending id order.  s_tmp: 4 * (NT / 64) words.  Every thread of the block takes part.
template <int NT, int KPT, typename KeyFn, typename EmitFn>
__device__ __forceinline__ void block_extract_topk(KeyFn key, int n, int k, EmitFn emit, uint32_t *s_tmp)
{
    constexpr int NW = NT / 64, KMAX = 8;
    const int tid = threadIdx.x, wv = tid >> 6, ln = lane_id();
    if (k >= n) {
        for (int i = tid; i < n; i += NT) emit(i, i);
        return;
    }
    uint32_t kreg[KPT];
#pragma unroll
    for (int it = 0; it < KPT; ++it) kreg[it] = key(min(it * NT + tid, n - 1));
#pragma unroll
    for (int it = 0; it < KPT; ++it)
        if (it * NT + tid >= n) kreg[it] = 0u;   // below every real key (their images are >= 1)
    unsigned long long *s_best = reinterpret_cast<unsigned long long *>(s_tmp);
    uint32_t picks[KMAX];
#pragma unroll
    for (int r = 0; r < KMAX; ++r) picks[r] = 0xffffffffu;
#pragma unroll
    for (int r = 0; r < KMAX; ++r) {
        if (r >= k) break;   // uniform
        unsigned long long best = 0ull;
#pragma unroll
        for (int it = 0; it < KPT; ++it) {
            const unsigned long long c = ((unsigned long long)kreg[it] << 32) | (uint32_t)~(uint32_t)(it * NT + tid);
            best = c > best ? c : best;
        }
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) {
            const unsigned long long other = __shfl_xor(best, o);
            best = other > best ? other : best;
        }
        unsigned long long *buf = s_best + (r & 1) * NW;
        if (ln == 0) buf[wv] = best;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < NW; ++w) best = buf[w] > best ? buf[w] : best;
        const uint32_t id = ~(uint32_t)best;
        picks[r] = id;
#pragma unroll
        for (int it = 0; it < KPT; ++it)
            if ((uint32_t)(it * NT + tid) == id) kreg[it] = 0u;
    }
    // thread r < k places pick r: its position is the number of picks with a smaller id
#pragma unroll
    for (int r = 0; r < KMAX; ++r) {
        if (r < k && tid == r) {
            int pos = 0;
#pragma unroll
            for (int q = 0; q < KMAX; ++q) pos += (q < k && picks[q] < picks[r]);
            emit(pos, (int)picks[r]);
        }
    }
}

}  // namespace ctkvr
