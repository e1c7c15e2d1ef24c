// Host side of the C ABI declared in include/ctkvr.h: argument checks, device
// memory of the index and its workspace, kernel launches.  No computation of the
// method happens on the host.
#include "../../include/ctkvr.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <type_traits>
#include <vector>

#include "kernels.hpp"
#include "kmeans.hpp"
#include "fused_args.hpp"

using namespace ctkvr;

namespace {

thread_local std::string g_err;

int fail(int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

#define HIP_TRY(expr)                                                                           \
    do {                                                                                        \
        hipError_t e_ = (expr);                                                                 \
        if (e_ != hipSuccess)                                                                   \
            return fail(e_ == hipErrorOutOfMemory ? CTKVR_ENOMEM : CTKVR_EHIP, "%s: %s", #expr, \
                        hipGetErrorString(e_));                                                 \
    } while (0)

size_t elem_size(int dtype) { return dtype == CTKVR_BF16 ? 2 : 4; }

}  // namespace

// Scratch of the entry point that allocates nothing (ctkvr_decode_step_static): one array per GPU, held
// until the process ends.  Host code never uses the array's name as an address: the device address
// is looked up once per device and kept.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
unsigned char *g_scratch_ptr[kMaxDevices] = {};

// device address of the current device's copy of `scratch`
int static_scratch(unsigned char **out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(CTKVR_EUNSUPPORTED, "device ordinal %d outside 0..%d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        unsigned char *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(CTKVR_EHIP, "hipGetSymbolAddress returned a null address for the scratch array");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return CTKVR_OK;
}

// Scratch of the matrix-core list build's candidate route, kept between builds (an index is built per prompt, and
// freeing a gigabyte costs 0.6 ms of an 8 ms build): one allocation per device, grown when a build needs more, at most
// kBuildCacheMax bytes; a build that finds it taken (another host thread is building) or needs more than that allocates
// its own.  ctkvr_release_scratch() frees it; CTKVR_BUILD_SCRATCH_CACHE=0 switches the cache off.
constexpr size_t kBuildCacheMax = (size_t)2 << 30;
struct BuildCache {
    void *base = nullptr;
    size_t bytes = 0;
    bool busy = false;
};
std::mutex g_build_mu;
BuildCache g_build_cache[kMaxDevices];

// *cached tells build_scratch_put what to do with the pointer afterwards
int build_scratch_get(size_t bytes, void **out, bool *cached)
{
    *out = nullptr;
    *cached = false;
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    const char *env = getenv("CTKVR_BUILD_SCRATCH_CACHE");
    const bool use = dev >= 0 && dev < kMaxDevices && bytes <= kBuildCacheMax && !(env && atoi(env) == 0);
    if (use) {
        std::lock_guard<std::mutex> lock(g_build_mu);
        BuildCache &c = g_build_cache[dev];
        if (!c.busy) {
            if (c.bytes < bytes) {   // (no build is using it: every build ends with a synchronisation of its stream)
                if (c.base) (void)hipFree(c.base);
                c.base = nullptr;
                c.bytes = 0;
                hipError_t e = hipMalloc(&c.base, bytes);
                if (e != hipSuccess) {
                    c.base = nullptr;
                    return fail(e == hipErrorOutOfMemory ? CTKVR_ENOMEM : CTKVR_EHIP, "hipMalloc(%zu): %s", bytes, hipGetErrorString(e));
                }
                c.bytes = bytes;
            }
            c.busy = true;
            *out = c.base;
            *cached = true;
            return CTKVR_OK;
        }
    }
    hipError_t e = hipMalloc(out, bytes ? bytes : 16);
    if (e != hipSuccess) {
        *out = nullptr;
        return fail(e == hipErrorOutOfMemory ? CTKVR_ENOMEM : CTKVR_EHIP, "hipMalloc(%zu): %s", bytes, hipGetErrorString(e));
    }
    return CTKVR_OK;
}

void build_scratch_put(void *ptr, bool cached)
{
    if (!ptr) return;
    if (!cached) {
        (void)hipFree(ptr);
        return;
    }
    std::lock_guard<std::mutex> lock(g_build_mu);
    for (BuildCache &c : g_build_cache)
        if (c.base == ptr) c.busy = false;
}
}  // namespace

// Buffers of one decode step for every (sequence, KV head) unit: everything ctkvr_decode_step
// writes apart from the caller's outputs.  An index owns one set; the entry point that allocates
// nothing lays the same set out in the library's static scratch array.
struct StepWs {
    float *cos = nullptr;
    int32_t *probe = nullptr, *cand = nullptr, *ncand = nullptr, *sel = nullptr, *nsel = nullptr;
    uint32_t *crow = nullptr, *srow = nullptr, *kbuf = nullptr, *gbits = nullptr, *ghist = nullptr;
    uint32_t *gbm = nullptr, *gcur = nullptr, *ginfo = nullptr;   // classify_kernel's outputs
    uint2 *glist = nullptr;
    unsigned long long *S = nullptr;
    float *z = nullptr, *zsel = nullptr;
    float *win = nullptr;   // window_attn_kernel's partial results
    uint32_t *m_key = nullptr;
    // single-launch step only (what its blocks hand to each other; see fused_args.hpp)
    float *part = nullptr;
    uint32_t *bar = nullptr;    // barrier counters, zero between steps
    int32_t *sid = nullptr, *slot_sure = nullptr;
    uint32_t *slot_cnt = nullptr, *slot_max = nullptr, *slot_hist = nullptr, *slot_npick = nullptr;
    unsigned long long *slot_S = nullptr;
    uint4 *slot_bkt = nullptr;
};

struct ctkvr_index {
    ctkvr_params p{};
    int G = 0, c_max = 0, s_max = 0, l_stride = 0, page_shift = 0, units = 0;
    float scale = 0.f;
    std::vector<int32_t> ctx_lens, n_cent;
    std::vector<void *> allocs;
    size_t device_bytes = 0;
    // index proper
    void *centroids = nullptr;
    float *inv_norm_c = nullptr;
    int32_t *lists = nullptr;
    int32_t *d_ctx_lens = nullptr, *d_n_cent = nullptr;
    StepWs ws;   // decode workspace
    // dynamic centroid update
    uint32_t *d_dcu_count = nullptr;   // [2]: updates so far (device side, so that captured graphs replay correctly), blocks of the running update that are done
    int32_t *dsel = nullptr, *dnsel = nullptr;   // top-rho ids of the second ranking (only when rho != rho')
    bool have_step = false;
    size_t recall_lds = 0, select_lds = 0, attn_lds = 0, build_select_lds = 0;
    size_t fused_lds = 0;   // non-zero: selection and attention run as one launch (select_attn_kernel)
    int keyclass = -1;      // key histogram + classification as one launch: -1 chosen per batch, 0 never, 1 always
    int attn_slices = 4;    // blocks per unit of the attention (head-dimension slices): 8 while each has a CU of its own
    int build_redone = 0;   // chunks of the matrix-core list build that the candidate route had to hand back
    int build_by_cand = 0;  // the matrix-core list build took the candidate route
    int xcd_units = -1;       // a unit's blocks on one XCD in every kernel of a step (unit_block_of; the units must be a multiple of 8):
                              // -1 for small batches, 0 never, 1 whenever possible
    int score_by_rank = -1;   // how the scoring kernel splits a unit's recalled ids over its blocks: -1 chosen per batch, 0 by id range, 1 by rank
    int sel_bits = 0, build_bits = 0;   // words for the selection's id bitmaps (0: histogram route off)
    int bitmap_words = 0, recall_split = 1, num_cu = 256;
    // single-launch step (decode_fused_kernel): blocks per unit (0: the geometry does not allow it), its shared memory,
    // the path in use (CTKVR_PATH_*), the sticky error word and the phase stamps
    int fused_bpu = 0, fused_nt = 1024, fused_stage = 0, decode_path = CTKVR_PATH_AUTO;
    bool last_step_fused = false;   // the last step on the index's own workspace left no 2048-bucket key histogram
    size_t fused_smem = 0;
    uint32_t *d_err = nullptr;
    long long *d_prof = nullptr;
    bool prof_phases = false;
    // Groups of sequences whose steps run side by side (fork / join on streams of the library, default priority):
    // the latency-bound selection stages of one group then overlap the key streaming of another.
    int n_groups = 1;
    std::vector<hipStream_t> side;          // n_groups - 1 streams
    hipEvent_t ev_fork = nullptr;
    std::vector<hipEvent_t> ev_join;        // one per side stream
    // per-kernel timing
    std::vector<hipEvent_t> events;
    int prof_max = 0, prof_step = 0;

    template <typename P> int alloc(P **ptr, size_t bytes)
    {
        void *v = nullptr;
        hipError_t e = hipMalloc(&v, bytes ? bytes : 16);
        if (e != hipSuccess)
            return fail(e == hipErrorOutOfMemory ? CTKVR_ENOMEM : CTKVR_EHIP, "hipMalloc(%zu): %s", bytes,
                        hipGetErrorString(e));
        allocs.push_back(v);
        device_bytes += bytes;
        *ptr = (P *)v;
        return CTKVR_OK;
    }
    ~ctkvr_index()
    {
        for (void *v : allocs) (void)hipFree(v);
        for (hipEvent_t e : events) (void)hipEventDestroy(e);
        for (hipEvent_t e : ev_join) (void)hipEventDestroy(e);
        if (ev_fork) (void)hipEventDestroy(ev_fork);
        for (hipStream_t st : side) (void)hipStreamDestroy(st);
    }
    // event slot `stage` (0 = before the first kernel) of the step being recorded
    void mark(int stage, hipStream_t st)
    {
        if (prof_step < prof_max) (void)hipEventRecord(events[(size_t)prof_step * (CTKVR_N_STAGES + 1) + stage], st);
    }
};

namespace {

#define TRY(expr)                    \
    do {                             \
        int rc_ = (expr);            \
        if (rc_ != CTKVR_OK) return rc_; \
    } while (0)

int check_params(const ctkvr_params *p, const int32_t *ctx_lens)
{
    if (!p) return fail(CTKVR_EINVAL, "params is NULL");
    if (!ctx_lens) return fail(CTKVR_EINVAL, "ctx_lens is NULL");
    if (p->batch < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1) return fail(CTKVR_EINVAL, "batch/heads must be >= 1");
    if (p->n_q_heads % p->n_kv_heads) return fail(CTKVR_EINVAL, "n_q_heads %% n_kv_heads != 0");
    if (p->head_dim != 128) return fail(CTKVR_EUNSUPPORTED, "head_dim %d: only 128 is supported", p->head_dim);
    int G = p->n_q_heads / p->n_kv_heads;
    if (G != 1 && G != 2 && G != 4 && G != 8) return fail(CTKVR_EUNSUPPORTED, "group size %d: only 1, 2, 4, 8", G);
    if (p->dtype != CTKVR_F32 && p->dtype != CTKVR_BF16) return fail(CTKVR_EINVAL, "unknown dtype %d", p->dtype);
    if (p->page_size < 1 || p->page_size > 256 || (p->page_size & (p->page_size - 1)))
        return fail(CTKVR_EUNSUPPORTED, "page_size %d: powers of two up to 256", p->page_size);
    if (p->n_centroids < 0 || (p->n_centroids == 0 && p->centroid_div < 1))
        return fail(CTKVR_EINVAL, "n_centroids = 0 needs centroid_div >= 1");
    if (p->list_len < 1 || p->n_probe < 1 || p->top_k < 1) return fail(CTKVR_EINVAL, "list_len, n_probe, top_k must be >= 1");
    if (p->n_probe > 1024) return fail(CTKVR_EUNSUPPORTED, "n_probe %d > 1024", p->n_probe);
    if (p->centroid_mode != CTKVR_CENTROID_LAST_C && p->centroid_mode != CTKVR_CENTROID_KMEANS)
        return fail(CTKVR_EINVAL, "unknown centroid_mode %d", p->centroid_mode);
    if (p->build_algo != CTKVR_BUILD_EXACT && p->build_algo != CTKVR_BUILD_MFMA)
        return fail(CTKVR_EINVAL, "unknown build_algo %d", p->build_algo);
    if (!(p->sm_scale >= 0.0f)) return fail(CTKVR_EINVAL, "sm_scale must be >= 0");
    if (p->n_init < 0 || p->n_local < 0) return fail(CTKVR_EINVAL, "n_init and n_local must be >= 0");
    for (int b = 0; b < p->batch; ++b) {
        int s = ctx_lens[b];
        if (s < 1 || s > (1 << 20)) return fail(s < 1 ? CTKVR_EINVAL : CTKVR_EUNSUPPORTED, "ctx_lens[%d] = %d outside 1..2^20", b, s);
        int C = p->n_centroids ? p->n_centroids : s / p->centroid_div;
        if (C < 1 || C > s) return fail(CTKVR_EINVAL, "sequence %d: %d centroids for %d tokens", b, C, s);
        if (C > 8192) return fail(CTKVR_EUNSUPPORTED, "sequence %d: %d centroids > 8192", b, C);
        if (p->n_probe > C) return fail(CTKVR_EINVAL, "sequence %d: n_probe %d > centroids %d", b, p->n_probe, C);
        if (p->list_len > s - p->n_init - p->n_local)
            return fail(CTKVR_EINVAL, "sequence %d: list_len %d > %d keys outside the resident window", b, p->list_len,
                        s - p->n_init - p->n_local);
    }
    return CTKVR_OK;
}

// Lays the step's buffers out from `base` (each 256-byte aligned) and returns the bytes they take;
// with base == nullptr only the size is computed.  The geometry is the index's.
size_t carve_step_ws(StepWs &w, unsigned char *base, const ctkvr_index *ix)
{
    size_t off = 0;
    auto take = [&](auto **ptr, size_t bytes) {
        using P = std::remove_reference_t<decltype(**ptr)>;
        if (base) *ptr = reinterpret_cast<P *>(base + off);
        off += (std::max<size_t>(bytes, 16) + 255) & ~(size_t)255;
    };
    const ctkvr_params &p = ix->p;
    const size_t U = ix->units, L = ix->l_stride, G = ix->G;
    const size_t bpu = std::max(1, ix->fused_bpu);
    // recalled keys of a unit: rank order (one launch per stage) or one stretch per block range (single launch)
    const size_t LS = std::max<size_t>(L, ix->fused_bpu ? (size_t)ix->fused_stage : 0);
    take(&w.cos, U * ix->c_max * 4);
    take(&w.probe, U * p.n_probe * 4);
    take(&w.cand, U * L * 4);
    take(&w.ncand, U * 4);
    take(&w.z, U * LS * G * 4);
    take(&w.m_key, U * G * 4);
    take(&w.crow, U * LS * 4);
    take(&w.gbits, U * (size_t)((ix->s_max + 31) / 32) * 4);
    take(&w.kbuf, U * L * 4);
    take(&w.ghist, U * (size_t)kBuckets * 4);
    take(&w.gbm, U * (size_t)(2 * ((L + 63) / 64)) * 4);
    take(&w.glist, U * (size_t)kListCap * 8);
    take(&w.gcur, U * 4);
    take(&w.ginfo, U * 16);
    take(&w.win, U * (size_t)kWinSplit * G * (2 + 128) * 4);
    take(&w.srow, U * p.top_k * 4);
    take(&w.S, U * G * 8);
    take(&w.sel, U * p.top_k * 4);
    take(&w.zsel, U * p.top_k * G * 4);
    take(&w.nsel, U * 4);
    take(&w.bar, U * (size_t)kFusedBarriers * 4);
    if (ix->fused_bpu) {
        take(&w.part, U * bpu * G * (2 + 128) * 4);
        take(&w.sid, U * LS * 4);
        take(&w.slot_cnt, U * bpu * 4);
        take(&w.slot_max, U * bpu * G * 4);
        take(&w.slot_S, U * bpu * G * 8);
        take(&w.slot_hist, U * bpu * (size_t)kFusedBins * 4);
        take(&w.slot_npick, U * bpu * 8);
        take(&w.slot_sure, U * bpu * (size_t)p.top_k * 4);
        take(&w.slot_bkt, U * bpu * (size_t)kFusedListCap * 16);
    }
    return off;
}

// allocate everything an index holds; fills the host-side geometry
int create_index(const ctkvr_params *p, const int32_t *ctx_lens, ctkvr_index **out)
{
    ctkvr_index *ix = new (std::nothrow) ctkvr_index();
    if (!ix) return fail(CTKVR_ENOMEM, "host allocation failed");
    ix->p = *p;
    const int B = p->batch, h = p->n_q_heads, g = p->n_kv_heads;
    ix->G = h / g;
    ix->scale = p->sm_scale > 0.0f ? p->sm_scale : (float)(1.0 / sqrt(128.0));
    ix->page_shift = __builtin_ctz(p->page_size);
    ix->units = B * g;
    for (int b = 0; b < B; ++b) {
        int s = ctx_lens[b];
        int C = p->n_centroids ? p->n_centroids : s / p->centroid_div;
        ix->ctx_lens.push_back(s);
        ix->n_cent.push_back(C);
        ix->c_max = std::max(ix->c_max, C);
        ix->s_max = std::max(ix->s_max, s);
        long lm = std::min<long>(s, (long)p->n_probe * p->list_len);
        ix->l_stride = std::max<long>(ix->l_stride, lm);
    }
    const size_t es = elem_size(p->dtype);
    const size_t U = ix->units;
    int rc = CTKVR_OK;
    auto A = [&](auto **ptr, size_t bytes) {
        if (rc == CTKVR_OK) rc = ix->alloc(ptr, bytes);
    };
    A(&ix->centroids, (size_t)B * h * ix->c_max * 128 * es);
    A(&ix->inv_norm_c, (size_t)B * h * ix->c_max * 4);
    A(&ix->lists, U * ix->c_max * p->list_len * 4);
    A(&ix->d_ctx_lens, (size_t)B * 4);
    A(&ix->d_n_cent, (size_t)B * 4);
    A(&ix->d_dcu_count, 8);
    A(&ix->d_err, 4);
    A(&ix->d_prof, 64 * 8);
    {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            ix->num_cu = cus;
    }
    ix->bitmap_words = (ix->s_max + 31) / 32;
    // The single-launch step needs all its blocks resident at once (one 1024-thread block per CU) and
    // its shared-memory plan to fit; up to 32 blocks work on a unit.
    if ((int)U <= ix->num_cu) {
        const int bpu = std::max(1, std::min(kFusedMaxBpu, ix->num_cu / (int)U));
        // Few recalled keys per block: four waves walk the serial parts of every phase (selections, scans,
        // reductions) faster than sixteen; many keys per block: sixteen waves keep more rows in flight.
        int nt = ix->l_stride / bpu <= 2048 ? 256 : 1024;
        if (const char *e = getenv("CTKVR_FUSED_THREADS")) {
            if (!strcmp(e, "256")) nt = 256;
            else if (!strcmp(e, "1024")) nt = 1024;
        }
        const size_t words = fused_smem_words(nt, p->n_probe, ix->s_max, bpu, p->top_k, ix->G);
        if (words * 4 <= (size_t)150 * 1024) {
            ix->fused_bpu = bpu;
            ix->fused_nt = nt;
            ix->fused_smem = words * 4;
            ix->fused_stage = bpu * fused_range_ids(ix->s_max, bpu);
        }
    }
    // Sequences of a batch are independent, and their steps can be issued as groups side by side
    // (CTKVR_DECODE_GROUPS = n at index creation).  One group is the default: on this part the split
    // measured slower on every benchmark batch (128K x 4: 131 us unsplit, 144 us as two groups, 159 us as
    // four; ragged x 16: 154 / 160 / 169 us) -- kernels of different streams take turns rather than share
    // the chip, and every group pays the per-kernel floors again.
    {
        int ng = 1;
        if (const char *e = getenv("CTKVR_DECODE_GROUPS")) ng = std::max(1, std::min(std::min(8, B), atoi(e)));
        if (const char *e = getenv("CTKVR_XCD_UNITS")) ix->xcd_units = atoi(e) != 0;
        if (const char *e = getenv("CTKVR_SCORE_BY_RANK")) ix->score_by_rank = atoi(e) != 0;
        if (const char *e = getenv("CTKVR_KEYCLASS")) ix->keyclass = atoi(e) != 0;
        ix->n_groups = ng;
    }
    if (const char *e = getenv("CTKVR_DECODE_PATH")) {
        if (!strcmp(e, "staged")) ix->decode_path = CTKVR_PATH_STAGED;
        else if (!strcmp(e, "fused") && ix->fused_bpu) ix->decode_path = CTKVR_PATH_FUSED;
    }
    if (p->list_len != p->top_k) {
        A(&ix->dsel, U * (size_t)p->list_len * 4);
        A(&ix->dnsel, U * 4);
    }
    {
        unsigned char *wsmem = nullptr;
        A(&wsmem, carve_step_ws(ix->ws, nullptr, ix));
        if (rc == CTKVR_OK) carve_step_ws(ix->ws, wsmem, ix);
    }
    if (rc != CTKVR_OK) {
        delete ix;
        return rc;
    }
    // shared-memory plan
    ix->bitmap_words = (ix->s_max + 31) / 32;
    ix->recall_lds = ((size_t)kSelLds + p->n_probe + ix->bitmap_words) * 4;
    // selection: radix scratch, the deciding bucket's list, two id bitmaps, the picked positions;
    // where the bitmaps would not fit the histogram route is switched off
    const size_t sel_fixed = (size_t)kSelLds + 2 * kListCap;
    ix->sel_bits = 4 * ((ix->l_stride + 63) / 64);
    const size_t picks = std::max(p->top_k, p->list_len);   // the update ranks once more with budget rho
    if ((sel_fixed + ix->sel_bits + picks) * 4 > 150 * 1024) ix->sel_bits = 0;
    ix->select_lds = (sel_fixed + ix->sel_bits + picks) * 4;
    ix->build_bits = 4 * ((ix->s_max + 63) / 64);
    if ((sel_fixed + ix->build_bits + 1) * 4 > 150 * 1024) ix->build_bits = 0;
    ix->build_select_lds = (sel_fixed + ix->build_bits + 1) * 4;
    ix->attn_lds = (size_t)p->top_k * ix->G * 4;
    {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            ix->num_cu = cus;
    }
    // The selection runs as one 1024-thread block per (sequence, KV head) and is latency-critical:
    // while there are no more such blocks than CUs, ask for over half a CU's shared memory so that
    // two never share a CU.  The recall is spread over recall_split blocks per unit.
    if ((int)U <= ix->num_cu) ix->select_lds = std::max<size_t>(ix->select_lds, 84 * 1024);
    ix->recall_split = std::max(1, std::min(8, ix->num_cu / (int)U));
    // Few enough units for every (unit, slice) block to have a CU of its own: one launch for lines 6-9.
    {
        const size_t fw = ((size_t)kSelLds + 2 * kListCap + ix->sel_bits + p->top_k + (size_t)p->top_k * ix->G) * 4;
        ix->attn_slices = 8 * (int)U <= ix->num_cu ? 8 : 4;
        if (4 * (int)U <= ix->num_cu && fw <= 150 * 1024) ix->fused_lds = fw;
    }
    if (ix->recall_lds > 150 * 1024 || ix->select_lds > 150 * 1024 || ix->attn_lds > 128 * 1024) {
        delete ix;
        return fail(CTKVR_EUNSUPPORTED, "context, top_k or n_probe too large for the shared-memory plan");
    }
    hipError_t e = hipSuccess;
    auto want = [&](const void *fn, size_t bytes) {
        if (e == hipSuccess) e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    };
    want((const void *)recall_gather_kernel<2>, ix->recall_lds);
    want((const void *)recall_gather_kernel<8>, ix->recall_lds);
    want((const void *)recall_gather_kernel<32>, ix->recall_lds);
    const size_t sel_b = std::max(ix->select_lds, ix->build_select_lds);
    want((const void *)rerank_select_kernel<1>, sel_b);
    want((const void *)rerank_select_kernel<2>, sel_b);
    want((const void *)rerank_select_kernel<4>, sel_b);
    want((const void *)rerank_select_kernel<8>, sel_b);
    if (ix->fused_lds) {
        if (p->dtype == CTKVR_BF16) {
            want((const void *)select_attn_kernel<bf16_t, 1, 4>, ix->fused_lds);
            want((const void *)select_attn_kernel<bf16_t, 1, 8>, ix->fused_lds);
            want((const void *)select_attn_kernel<bf16_t, 2, 4>, ix->fused_lds);
            want((const void *)select_attn_kernel<bf16_t, 2, 8>, ix->fused_lds);
            want((const void *)select_attn_kernel<bf16_t, 4, 4>, ix->fused_lds);
            want((const void *)select_attn_kernel<bf16_t, 4, 8>, ix->fused_lds);
            want((const void *)select_attn_kernel<bf16_t, 8, 4>, ix->fused_lds);
            want((const void *)select_attn_kernel<bf16_t, 8, 8>, ix->fused_lds);
        } else {
            want((const void *)select_attn_kernel<float, 1, 4>, ix->fused_lds);
            want((const void *)select_attn_kernel<float, 1, 8>, ix->fused_lds);
            want((const void *)select_attn_kernel<float, 2, 4>, ix->fused_lds);
            want((const void *)select_attn_kernel<float, 2, 8>, ix->fused_lds);
            want((const void *)select_attn_kernel<float, 4, 4>, ix->fused_lds);
            want((const void *)select_attn_kernel<float, 4, 8>, ix->fused_lds);
            want((const void *)select_attn_kernel<float, 8, 4>, ix->fused_lds);
            want((const void *)select_attn_kernel<float, 8, 8>, ix->fused_lds);
        }
    }
    if (ix->fused_bpu && e == hipSuccess) e = fused_set_smem(p->dtype == CTKVR_BF16, ix->G, ix->fused_nt, ix->fused_smem);
    if (p->dtype == CTKVR_BF16) {
        want((const void *)sparse_attn_kernel<bf16_t, 1, 4>, ix->attn_lds);
        want((const void *)sparse_attn_kernel<bf16_t, 1, 8>, ix->attn_lds);
        want((const void *)sparse_attn_kernel<bf16_t, 2, 4>, ix->attn_lds);
        want((const void *)sparse_attn_kernel<bf16_t, 2, 8>, ix->attn_lds);
        want((const void *)sparse_attn_kernel<bf16_t, 4, 4>, ix->attn_lds);
        want((const void *)sparse_attn_kernel<bf16_t, 4, 8>, ix->attn_lds);
        want((const void *)sparse_attn_kernel<bf16_t, 8, 4>, ix->attn_lds);
        want((const void *)sparse_attn_kernel<bf16_t, 8, 8>, ix->attn_lds);
    } else {
        want((const void *)sparse_attn_kernel<float, 1, 4>, ix->attn_lds);
        want((const void *)sparse_attn_kernel<float, 1, 8>, ix->attn_lds);
        want((const void *)sparse_attn_kernel<float, 2, 4>, ix->attn_lds);
        want((const void *)sparse_attn_kernel<float, 2, 8>, ix->attn_lds);
        want((const void *)sparse_attn_kernel<float, 4, 4>, ix->attn_lds);
        want((const void *)sparse_attn_kernel<float, 4, 8>, ix->attn_lds);
        want((const void *)sparse_attn_kernel<float, 8, 4>, ix->attn_lds);
        want((const void *)sparse_attn_kernel<float, 8, 8>, ix->attn_lds);
    }
    {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            ix->num_cu = cus;
    }
    if (e == hipSuccess) e = hipMemset(ix->ws.ghist, 0, U * (size_t)kBuckets * 4);
    if (e == hipSuccess) e = hipMemset(ix->d_dcu_count, 0, 8);
    if (e == hipSuccess) e = hipMemset(ix->d_err, 0, 4);
    if (e == hipSuccess) e = hipMemset(ix->d_prof, 0, 64 * 8);
    if (e == hipSuccess) e = hipMemset(ix->ws.bar, 0, U * (size_t)kFusedBarriers * 4);
    if (e == hipSuccess) e = hipMemset(ix->ws.gbits, 0, U * (size_t)ix->bitmap_words * 4);
    if (e == hipSuccess) e = hipMemset(ix->ws.srow, 0, U * p->top_k * 4);   // always valid rows (see sparse_attn_kernel)
    if (e == hipSuccess) e = hipMemcpy(ix->d_ctx_lens, ix->ctx_lens.data(), (size_t)B * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(ix->d_n_cent, ix->n_cent.data(), (size_t)B * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemset(ix->lists, 0, U * ix->c_max * p->list_len * 4);
    if (e == hipSuccess) e = hipMemset(ix->centroids, 0, (size_t)B * h * ix->c_max * 128 * es);
    if (e == hipSuccess && ix->n_groups > 1) {
        e = hipEventCreateWithFlags(&ix->ev_fork, hipEventDisableTiming);
        for (int i = 1; i < ix->n_groups && e == hipSuccess; ++i) {
            hipStream_t sst = nullptr;
            hipEvent_t ev = nullptr;
            e = hipStreamCreateWithFlags(&sst, hipStreamNonBlocking);
            if (e == hipSuccess) ix->side.push_back(sst);
            if (e == hipSuccess) e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
            if (e == hipSuccess) ix->ev_join.push_back(ev);
        }
    }
    if (e != hipSuccess) {
        delete ix;
        return fail(CTKVR_EHIP, "index set-up: %s", hipGetErrorString(e));
    }
    *out = ix;
    return CTKVR_OK;
}

Units decode_units(const ctkvr_index *ix)
{
    Units u{};
    u.g = ix->p.n_kv_heads;
    u.G = ix->G;
    u.h = ix->p.n_q_heads;
    u.build = 0;
    u.unit0 = 0;
    u.c_max = ix->c_max;
    u.n_cent = ix->d_n_cent;
    return u;
}

template <typename T> int launch_inv_norms(ctkvr_index *ix, hipStream_t st)
{
    size_t n = (size_t)ix->p.batch * ix->p.n_q_heads * ix->c_max;
    inv_norm_kernel<T><<<dim3((unsigned)((n + 15) / 16)), 256, 0, st>>>((const T *)ix->centroids, n, ix->inv_norm_c);
    HIP_TRY(hipGetLastError());
    return CTKVR_OK;
}

// Algorithm 1 lines 2-4 in the decode path's own arithmetic: for chunks of
// (sequence, KV head, centroid) units, score all keys, then per unit sum the
// denominators and select the top-rho.
template <typename T, int G>
int build_lists_exact(ctkvr_index *ix, const void *k_pages, const int32_t *block_table, int max_pages, hipStream_t st)
{
    const bool mfma = ix->p.build_algo == CTKVR_BUILD_MFMA;
    const int total_units = ix->units * ix->c_max;
    const size_t per_unit = (size_t)ix->s_max * G * 4;
    int chunk = (int)std::min<size_t>(total_units, std::max<size_t>(1, ((size_t)2 << 30) / per_unit));
    chunk = std::min(chunk, 16384);
    if (mfma) {   // whole (sequence, KV head) groups per chunk; no scores are stored, only 4-byte keys
        int nbk = (int)std::max<size_t>(1, ((size_t)8 << 30) / ((size_t)ix->s_max * 4 * ix->c_max));
        nbk = std::min(nbk, std::max(1, 16384 / ix->c_max));
        chunk = std::min(ix->units, nbk) * ix->c_max;
    }
    float *z = nullptr;
    uint32_t *m_key = nullptr;
    unsigned long long *S = nullptr;
    uint32_t *kbuf = nullptr, *ghist = nullptr;
    float2 *part = nullptr;   // matrix-core route: one (maximum, sum) pair per unit, head and block of the statistics pass
    constexpr int kMaxSplits = 64;
    // Matrix-core route, candidates only (see mfma_score_kernel): when every sequence is long against rho, so that
    // about 2 rho candidates are a small part of its keys and a 1-in-16 sample of the positions places the threshold
    // well, and the selection's bitmaps and candidate list fit the shared memory.  CTKVR_BUILD_CANDIDATES=0/1 forces
    // the choice where the second condition allows it (1 on short sequences mostly ends in the redo below).
    const int rho = ix->p.list_len;
    const int step_stride = std::max(16, ((ix->s_max + 31) / 32 + 255) / 256);
    const int sample_stride = ((ix->s_max + 32 * step_stride - 1) / (32 * step_stride)) * 32;
    const int cand_cap = std::min(kCandCap, std::max(3 * rho, 2 * rho + 1024));   // about 2 rho + 256 are expected (+-6 % at rho = 2048)
    const size_t cand_lds = ((size_t)2112 + 2 * (size_t)cand_cap + kCandTies + (size_t)((ix->s_max + 31) / 32)) * 4;
    bool by_cand = false;
    if (mfma && cand_lds <= 150 * 1024 && sample_stride <= kSampleCap && cand_cap >= rho) {
        const int s_min = *std::min_element(ix->ctx_lens.begin(), ix->ctx_lens.end());
        by_cand = rho >= 256 && 3 * rho <= kCandCap && (long long)s_min >= 32ll * rho;
        if (const char *e = getenv("CTKVR_BUILD_CANDIDATES")) by_cand = atoi(e) != 0;
    }
    ix->build_by_cand = by_cand;
    if (by_cand) chunk = std::min(chunk, 4 * ix->c_max);   // half the scratch, as fast
    const bool redo_always = by_cand && getenv("CTKVR_BUILD_CANDIDATES_REDO") != nullptr;   // tests: take the redo path
    uint32_t *ksamp = nullptr, *tau = nullptr, *cursor = nullptr, *d_fail = nullptr;
    uint2 *cand = nullptr;
    hipError_t e1 = hipSuccess, e2 = hipSuccess, e3 = hipSuccess, e4 = hipSuccess, e5 = hipSuccess;
    auto alloc_full = [&]() {   // the buffers of the route that keeps every key
        if (!kbuf) e3 = hipMalloc((void **)&kbuf, (size_t)chunk * ix->s_max * 4);
        if (!ghist) e4 = hipMalloc((void **)&ghist, (size_t)chunk * kBuckets * 4);
        return e3 == hipSuccess && e4 == hipSuccess;
    };
    void *block = nullptr;   // candidates route: all of its buffers in one allocation, kept between builds
    bool block_cached = false;
    int rc = CTKVR_OK;
    if (by_cand) {
        // a segment per block of the statistics split: room for twice an even share, at least 256 entries
        const size_t sizes[8] = {(size_t)chunk * G * 4, (size_t)chunk * G * 8, (size_t)chunk * G * kMaxSplits * sizeof(float2),
                                 (size_t)chunk * sample_stride * 4, (size_t)chunk * 4, (size_t)chunk * kMaxSplits * 4, 4,
                                 (size_t)chunk * 2 * std::max(cand_cap, 128 * kMaxSplits) * sizeof(uint2)};
        size_t off[9] = {0};
        for (int i = 0; i < 8; ++i) off[i + 1] = off[i] + ((sizes[i] + 255) & ~(size_t)255);
        rc = build_scratch_get(off[8], &block, &block_cached);
        if (rc == CTKVR_OK) {
            unsigned char *base = (unsigned char *)block;
            m_key = (uint32_t *)(base + off[0]);
            S = (unsigned long long *)(base + off[1]);
            part = (float2 *)(base + off[2]);
            ksamp = (uint32_t *)(base + off[3]);
            tau = (uint32_t *)(base + off[4]);
            cursor = (uint32_t *)(base + off[5]);
            d_fail = (uint32_t *)(base + off[6]);
            cand = (uint2 *)(base + off[7]);
            e5 = hipFuncSetAttribute((const void *)cand_select_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)cand_lds);
        }
    } else {
        if (!mfma) e5 = hipMalloc((void **)&z, (size_t)chunk * per_unit);
        e1 = hipMalloc((void **)&m_key, (size_t)chunk * G * 4);
        e2 = hipMalloc((void **)&S, (size_t)chunk * G * 8);
        if (mfma && e5 == hipSuccess) e5 = hipMalloc((void **)&part, (size_t)chunk * G * kMaxSplits * sizeof(float2));
        alloc_full();
    }
    if (rc == CTKVR_OK && (e1 != hipSuccess || e2 != hipSuccess || e3 != hipSuccess || e4 != hipSuccess || e5 != hipSuccess))
        rc = fail(CTKVR_ENOMEM, "build scratch allocation failed");
    for (int u0 = 0; rc == CTKVR_OK && u0 < total_units; u0 += chunk) {
        const int nu = std::min(chunk, total_units - u0);
        Units u = decode_units(ix);
        u.build = 1;
        u.unit0 = u0;
        fill_u32_kernel<<<dim3((unsigned)((nu * G + 255) / 256)), 256, 0, st>>>(m_key, 0u, (size_t)nu * G);
        fill_u32_kernel<<<dim3((unsigned)((nu * G * 2 + 255) / 256)), 256, 0, st>>>((uint32_t *)S, 0u, (size_t)nu * G * 2);
        if (ghist) fill_u32_kernel<<<dim3((unsigned)(((size_t)nu * kBuckets + 255) / 256)), 256, 0, st>>>(ghist, 0u, (size_t)nu * kBuckets);
        bool keys_written = false;   // kbuf holds this chunk's ranking keys (matrix-core route)
        ScoreArgs sa{};
        sa.u = u;
        sa.q = ix->centroids;
        sa.qrows = ix->c_max;
        sa.k = Paged{k_pages, block_table, max_pages, ix->page_shift};
        sa.ctx_lens = ix->d_ctx_lens;
        sa.crow = nullptr;
        sa.ncand = nullptr;
        sa.l_stride = ix->s_max;
        sa.z = z;
        sa.m_key = m_key;
        sa.scale = ix->scale;
        if constexpr (std::is_same<T, bf16_t>::value) {
            if (mfma) {
                constexpr int CT = 32 * (8 / G);
                MfmaScoreArgs ma{};
                ma.g = ix->p.n_kv_heads;
                ma.G = G;
                ma.h = ix->p.n_q_heads;
                ma.c_max = ix->c_max;
                ma.bk0 = u0 / ix->c_max;
                ma.tiles_per_bk = (ix->c_max + CT - 1) / CT;
                const int tiles = (nu / ix->c_max) * ma.tiles_per_bk;
                ma.t_splits = std::max(1, std::min({(ix->s_max + 1023) / 1024, (4 * ix->num_cu + tiles - 1) / tiles, kMaxSplits}));
                ma.n_cent = ix->d_n_cent;
                ma.ctx_lens = ix->d_ctx_lens;
                ma.centroids = (const bf16_t *)ix->centroids;
                ma.k = sa.k;
                ma.l_stride = ix->s_max;
                ma.part = part;
                ma.kbuf = kbuf;
                ma.n_init = ix->p.n_init;
                ma.n_local = ix->p.n_local;
                ma.scale = ix->scale;
                ma.step_stride = 1;
                // passes over the same tiles: softmax statistics first
                mfma_score_kernel<G, MFMA_STAT><<<dim3(ma.t_splits, tiles), 256, 0, st>>>(ma);
                bool redo = !by_cand;
                if (by_cand) {
                    // keys of a sample of the positions -> a threshold per unit -> all keys again, those at or above
                    // the threshold kept -> the rho largest of them, exactly
                    ma.kbuf = ksamp;
                    ma.step_stride = step_stride;
                    ma.sample_stride = sample_stride;
                    mfma_score_kernel<G, MFMA_SAMPLE><<<dim3(ma.t_splits, tiles), 256, 0, st>>>(ma);
                    CandArgs ca{};
                    ca.u = u;
                    ca.ctx_lens = ix->d_ctx_lens;
                    ca.rho = rho;
                    ca.step_stride = step_stride;
                    ca.sample_stride = sample_stride;
                    ca.cand_cap = cand_cap;
                    ca.n_init = ix->p.n_init;
                    ca.n_local = ix->p.n_local;
                    ca.ksamp = ksamp;
                    ca.tau = tau;
                    const int seg_cap = std::min(cand_cap, std::max(256, 2 * cand_cap / ma.t_splits));   // t_splits * seg_cap <= 2 max(cand_cap, 128 t_splits)
                    ca.cand = cand;
                    ca.seg_cnt = cursor;
                    ca.t_splits = ma.t_splits;
                    ca.seg_cap = seg_cap;
                    ca.lists = ix->lists;
                    ca.fail = d_fail;
                    fill_u32_kernel<<<dim3(1), 64, 0, st>>>(d_fail, 0u, 1);
                    fill_u32_kernel<<<dim3((unsigned)(((size_t)nu * ma.t_splits + 255) / 256)), 256, 0, st>>>(cursor, 0u, (size_t)nu * ma.t_splits);
                    sample_threshold_kernel<<<dim3(nu), 1024, 0, st>>>(ca);
                    ma.step_stride = 1;
                    ma.tau = tau;
                    ma.cand = cand;
                    ma.seg_cnt = cursor;
                    ma.seg_cap = seg_cap;
                    mfma_score_kernel<G, MFMA_PICK><<<dim3(ma.t_splits, tiles), 256, 0, st>>>(ma);
                    cand_select_kernel<<<dim3(nu), 1024, cand_lds, st>>>(ca);
                    uint32_t failed = 0;
                    hipError_t ec = hipMemcpyAsync(&failed, d_fail, 4, hipMemcpyDeviceToHost, st);
                    if (ec == hipSuccess) ec = hipStreamSynchronize(st);
                    if (ec != hipSuccess) {
                        rc = fail(CTKVR_EHIP, "build: %s", hipGetErrorString(ec));
                        break;
                    }
                    redo = failed != 0 || redo_always;
                    if (redo) {
                        ix->build_redone++;
                        if (!alloc_full()) {
                            rc = fail(CTKVR_ENOMEM, "build scratch allocation failed");
                            break;
                        }
                        fill_u32_kernel<<<dim3((unsigned)(((size_t)nu * kBuckets + 255) / 256)), 256, 0, st>>>(ghist, 0u, (size_t)nu * kBuckets);
                    }
                }
                if (redo) {   // every key stored, then histogram and selection over all of them
                    ma.kbuf = kbuf;
                    mfma_score_kernel<G, MFMA_KEY><<<dim3(ma.t_splits, tiles), 256, 0, st>>>(ma);
                    keys_written = true;
                }
            } else {
                score_kernel<T, G, 16><<<dim3((ix->s_max + 255) / 256, nu), 256, 0, st>>>(sa);
            }
        } else {
            score_kernel<T, G, 16><<<dim3((ix->s_max + 255) / 256, nu), 256, 0, st>>>(sa);
        }
        if (!mfma) {
            DenomArgs da{};
            da.u = u;
            da.ctx_lens = ix->d_ctx_lens;
            da.ncand = nullptr;
            da.l_stride = ix->s_max;
            da.z = z;
            da.m_key = m_key;
            da.S = S;
            denom_kernel<G><<<dim3(std::min((ix->s_max + 1023) / 1024, 64), nu), 256, 0, st>>>(da);
        }
        if (mfma && !keys_written) {   // the candidate route has written this chunk's lists
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) rc = fail(CTKVR_EHIP, "build launch: %s", hipGetErrorString(e));
            continue;
        }
        KeyArgs ka{};
        ka.u = u;
        ka.ctx_lens = ix->d_ctx_lens;
        ka.ncand = nullptr;
        ka.l_stride = ix->s_max;
        ka.z = mfma ? nullptr : z;   // the matrix-core passes have written the keys: histogram only
        ka.m_key = m_key;
        ka.S = S;
        ka.kbuf = kbuf;
        ka.ghist = ghist;
        ka.n_init = ix->p.n_init;
        ka.n_local = ix->p.n_local;
        keyhist_kernel<G><<<dim3(std::min((ix->s_max + 4095) / 4096, 8), nu), 1024, 0, st>>>(ka);
        SelectArgs se{};
        se.u = u;
        se.ctx_lens = ix->d_ctx_lens;
        se.ncand = nullptr;
        se.cand = nullptr;
        se.crow = nullptr;
        se.l_stride = ix->s_max;
        se.top_k = ix->p.list_len;
        se.z = z;
        se.m_key = m_key;
        se.kbuf = kbuf;
        se.ghist = ghist;
        se.bits_words = ix->build_bits;
        se.sel = ix->lists;
        rerank_select_kernel<G><<<dim3(nu), 1024, ix->build_select_lds, st>>>(se);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) rc = fail(CTKVR_EHIP, "build launch: %s", hipGetErrorString(e));
    }
    hipError_t es = hipStreamSynchronize(st);
    if (rc == CTKVR_OK && es != hipSuccess) rc = fail(CTKVR_EHIP, "build: %s", hipGetErrorString(es));
    if (by_cand) {
        build_scratch_put(block, block_cached);
    } else {
        (void)hipFree(z);
        (void)hipFree(m_key);
        (void)hipFree(S);
        (void)hipFree(part);
    }
    (void)hipFree(kbuf);
    (void)hipFree(ghist);
    return rc;
}

template <typename T>
int build_lists_dispatch(ctkvr_index *ix, const void *k_pages, const int32_t *bt, int max_pages, hipStream_t st)
{
    switch (ix->G) {
        case 1: return build_lists_exact<T, 1>(ix, k_pages, bt, max_pages, st);
        case 2: return build_lists_exact<T, 2>(ix, k_pages, bt, max_pages, st);
        case 4: return build_lists_exact<T, 4>(ix, k_pages, bt, max_pages, st);
        default: return build_lists_exact<T, 8>(ix, k_pages, bt, max_pages, st);
    }
}

template <typename T, int G>
int decode_launch_group(ctkvr_index *ix, const StepWs &w_all, int b0, int nb, bool whole, const void *q, const void *k_pages,
                        const void *v_pages, const int32_t *bt, int max_pages, const int32_t *cur_lens, float *out, float *out_lse,
                        int32_t *out_sel, int32_t *out_ncand, int32_t *out_probe, hipStream_t st)
{
    // The step for the sequences b0 .. b0 + nb - 1 of the batch: every per-sequence and per-unit array is entered
    // at that group's first element, and the kernels see a batch of nb sequences.  whole: the group is the batch
    // (per-kernel timing marks and the single-launch form apply to whole batches only).
    const ctkvr_params &p = ix->p;
    const int U = nb * p.n_kv_heads, u0 = b0 * p.n_kv_heads;
    const size_t es = elem_size(p.dtype);
    auto adv = [](auto *ptr, size_t n) { return ptr ? ptr + n : ptr; };
    q = (const char *)q + (size_t)b0 * p.n_q_heads * 128 * es;
    bt = bt + (size_t)b0 * max_pages;
    cur_lens = adv(cur_lens, b0);
    out = out + (size_t)b0 * p.n_q_heads * 128;
    out_lse = adv(out_lse, (size_t)b0 * p.n_q_heads);
    out_sel = adv(out_sel, (size_t)u0 * p.top_k);
    out_ncand = adv(out_ncand, u0);
    out_probe = adv(out_probe, (size_t)u0 * p.n_probe);
    const void *cen = (const char *)ix->centroids + (size_t)b0 * p.n_q_heads * ix->c_max * 128 * es;
    const float *inv_c = ix->inv_norm_c + (size_t)b0 * p.n_q_heads * ix->c_max;
    const int32_t *lists = ix->lists + (size_t)u0 * ix->c_max * p.list_len;
    const int32_t *d_n_cent = ix->d_n_cent + b0, *d_ctx_lens = ix->d_ctx_lens + b0;
    StepWs w = w_all;
    if (u0) {
        const size_t L = ix->l_stride, Gs = ix->G;
        w.cos += (size_t)u0 * ix->c_max;
        w.probe += (size_t)u0 * p.n_probe;
        w.cand += u0 * L;
        w.ncand += u0;
        w.z += u0 * L * Gs;
        w.m_key += u0 * Gs;
        w.crow += u0 * L;
        w.gbits += (size_t)u0 * ix->bitmap_words;
        w.kbuf += u0 * L;
        w.ghist += (size_t)u0 * kBuckets;
        w.gbm += (size_t)u0 * (2 * ((L + 63) / 64));
        w.glist += (size_t)u0 * kListCap;
        w.gcur += u0;
        w.ginfo += (size_t)u0 * 4;
        w.win += (size_t)u0 * kWinSplit * Gs * (2 + 128);
        w.srow += (size_t)u0 * p.top_k;
        w.S += u0 * Gs;
        w.sel += (size_t)u0 * p.top_k;
        w.zsel += (size_t)u0 * p.top_k * Gs;
        w.nsel += u0;
    }
    Units units = decode_units(ix);
    units.n_cent = d_n_cent;
    // A unit's blocks on one XCD (unit_block_of; needs a multiple of 8 units): in every kernel for small batches
    // (latency-bound: a step is a chain of dependent loads of what the previous kernel wrote); for large ones in all but
    // the two bandwidth-bound launches -- the cosines, and the scoring, whose blocks are better handed to whichever XCD is free.
    const bool xcd_small = ix->xcd_units < 0 ? (long long)ix->l_stride * U <= 2048ll * ix->num_cu : ix->xcd_units != 0;
    const int by_xcd = U % 8 == 0 && ix->xcd_units != 0;
    const int by_xcd_all = by_xcd && xcd_small;
    // lines 10-11 first: the window's share depends on q, K and V only
    const bool window = p.n_init + p.n_local > 0 || cur_lens;
    WindowArgs wa{};
    const bool one_launch = whole && ix->fused_bpu && ix->decode_path == CTKVR_PATH_FUSED;
    if (window) {
        wa.u = units;
        wa.q = q;
        wa.k = Paged{k_pages, bt, max_pages, ix->page_shift};
        wa.v_pages = v_pages;
        wa.ctx_lens = d_ctx_lens;
        wa.cur_lens = cur_lens;
        wa.n_init = p.n_init;
        wa.n_local = p.n_local;
        wa.scale = ix->scale;
        wa.win = w.win;
        wa.by_xcd = by_xcd;
        // a launch of its own before the single-launch step, and for groups of eight heads (where the window's
        // registers would cost the scoring blocks a wave per SIMD); otherwise its blocks ride in the scoring launch below
        if (one_launch || G > 4) window_attn_kernel<T, G><<<dim3(kWinSplit, U), 256, 0, st>>>(wa);
    }
    const bool stream_k = [&] {
        // key bytes the batch can touch per step: above 128 MiB (half of the 256 MB memory-side cache) few rows
        // survive to the next step, and a non-temporal hint keeps the centroid table, the lists and the step's
        // own buffers cached instead
        size_t kbytes = 0;
        for (int sl : ix->ctx_lens) kbytes += (size_t)sl * p.n_kv_heads * 128 * elem_size(p.dtype);
        return kbytes > ((size_t)128 << 20);
    }();
    if (one_launch) {
        FusedArgs fa{};
        fa.g = p.n_kv_heads;
        fa.h = p.n_q_heads;
        fa.c_max = ix->c_max;
        fa.rho = p.list_len;
        fa.n_probe = p.n_probe;
        fa.top_k = p.top_k;
        fa.l_stride = ix->l_stride;
        fa.bpu = ix->fused_bpu;
        fa.units = U;
        fa.stage = ix->fused_stage;
        fa.stream_k = stream_k;
        fa.scale = ix->scale;
        fa.n_cent = d_n_cent;
        fa.ctx_lens = d_ctx_lens;
        fa.q = q;
        fa.centroids = cen;
        fa.inv_norm_c = inv_c;
        fa.lists = lists;
        fa.k = Paged{k_pages, bt, max_pages, ix->page_shift};
        fa.v_pages = v_pages;
        fa.cos = w.cos;
        fa.probe = w.probe;
        fa.out_probe = out_probe;
        fa.sid = w.sid;
        fa.srow = w.crow;
        fa.z = w.z;
        fa.cand = w.cand;
        fa.kbuf = w.kbuf;
        fa.ncand = w.ncand;
        fa.out_ncand = out_ncand;
        fa.slot_cnt = w.slot_cnt;
        fa.slot_max = w.slot_max;
        fa.slot_S = w.slot_S;
        fa.slot_hist = w.slot_hist;
        fa.slot_npick = w.slot_npick;
        fa.slot_sure = w.slot_sure;
        fa.slot_bkt = w.slot_bkt;
        fa.part = w.part;
        fa.sel = w.sel;
        fa.nsel = w.nsel;
        fa.out_sel = out_sel;
        fa.out = out;
        fa.out_lse = out_lse;
        fa.win = window ? w.win : nullptr;
        fa.bar = w.bar;
        fa.err = ix->d_err;
        fa.prof = ix->prof_phases ? ix->d_prof : nullptr;
        if (whole) ix->mark(0, st);
        HIP_TRY(fused_launch(p.dtype == CTKVR_BF16, G, ix->fused_nt, (unsigned)(U * ix->fused_bpu), ix->fused_smem, st, fa));
        for (int k = 1; k <= 8; ++k) ix->mark(k, st);   // the whole step reads as stage 0
        if (ix->prof_step < ix->prof_max) {
            fill_u32_kernel<<<dim3(1), 64, 0, st>>>((uint32_t *)w.nsel, 0u, 0);
            if (whole) ix->mark(9, st);
            ix->prof_step++;
        }
        HIP_TRY(hipGetLastError());
        ix->have_step = &w_all == &ix->ws;
        ix->last_step_fused = true;
        return CTKVR_OK;
    }
    ix->last_step_fused = false;
    CosArgs ca{};
    ca.q = q;
    ca.centroids = cen;
    ca.inv_norm_c = inv_c;
    ca.n_cent = d_n_cent;
    ca.cos = w.cos;
    ca.m_key = w.m_key;
    ca.S = w.S;
    ca.g = p.n_kv_heads;
    ca.h = p.n_q_heads;
    ca.c_max = ix->c_max;
    ca.by_xcd = by_xcd_all;
    if (whole) ix->mark(0, st);
    centroid_cos_kernel<T, G><<<dim3((ix->c_max + 15) / 16, U), 256, 0, st>>>(ca);
    if (whole) ix->mark(1, st);

    GatherArgs ga{};
    ga.cos = w.cos;
    ga.lists = lists;
    ga.n_cent = d_n_cent;
    ga.ctx_lens = d_ctx_lens;
    ga.probe = w.probe;
    ga.out_probe = out_probe;
    ga.gbits = w.gbits;
    ga.g = p.n_kv_heads;
    ga.c_max = ix->c_max;
    ga.rho = p.list_len;
    ga.n_probe = p.n_probe;
    ga.bitmap_words = ix->bitmap_words;
    ga.by_xcd = by_xcd;
    const dim3 rgrid(ix->recall_split, U);
    if (ix->c_max <= 512)
        recall_gather_kernel<2><<<rgrid, 256, ix->recall_lds, st>>>(ga);
    else if (ix->c_max <= 2048)
        recall_gather_kernel<8><<<rgrid, 256, ix->recall_lds, st>>>(ga);
    else
        recall_gather_kernel<32><<<rgrid, 256, ix->recall_lds, st>>>(ga);
    if (whole) ix->mark(2, st);

    // lines 4-5: bitmap -> recalled ids, their rows and their scores in one launch
    Units u = units;
    RecallScoreArgs sa{};
    sa.u = u;
    sa.stream_k = stream_k;
    sa.q = q;
    sa.k = Paged{k_pages, bt, max_pages, ix->page_shift};
    sa.ctx_lens = d_ctx_lens;
    sa.gbits = w.gbits;
    sa.bitmap_words = ix->bitmap_words;
    sa.l_stride = ix->l_stride;
    sa.cand = w.cand;
    sa.crow = w.crow;
    sa.ncand = w.ncand;
    sa.out_ncand = out_ncand;
    sa.z = w.z;
    sa.m_key = w.m_key;
    sa.ghist = w.ghist;
    sa.scale = ix->scale;
    sa.by_xcd = by_xcd_all;
    {
        // Few rows per CU (a small batch): a block's rows are one round trip to memory and the slowest block
        // is the launch, so the ids are split by rank -- two blocks per CU, at least 32 per unit and 64 ranks
        // per block.  Otherwise by id range: enough blocks to fill the chip a few times over, each owning
        // 8..64 words of the bitmap.
        const bool by_rank = ix->score_by_rank < 0 ? (long long)ix->l_stride * U <= 2048ll * ix->num_cu : ix->score_by_rank != 0;
        sa.by_rank = by_rank;
        int nbx;
        if (by_rank) {
            nbx = std::min(std::max(32, (2 * ix->num_cu + U - 1) / U), (ix->l_stride + 63) / 64);
            nbx = std::max({1, nbx, (ix->l_stride + kRecallCap - 1) / kRecallCap});
        } else {
            const int target = std::max(32, (8 * ix->num_cu + U - 1) / U);
            const int wpb = std::max(8, std::min(kRecallWpb, (ix->bitmap_words + target - 1) / target));
            nbx = (ix->bitmap_words + wpb - 1) / wpb;
        }
        sa.nbx = nbx;
        bool launched = false;
        if constexpr (G <= 4) {
            if (window) {
                sa.win = wa;
                recall_score_kernel<T, G, true><<<dim3(nbx + kWinSplit, U), 256, 0, st>>>(sa);
                launched = true;
            }
        }
        if (!launched) recall_score_kernel<T, G, false><<<dim3(nbx, U), 256, 0, st>>>(sa);
    }
    if (whole) ix->mark(3, st);

    DenomArgs da{};
    da.u = u;
    da.ctx_lens = d_ctx_lens;
    da.ncand = w.ncand;
    da.l_stride = ix->l_stride;
    da.z = w.z;
    da.m_key = w.m_key;
    da.S = w.S;
    da.gbits = w.gbits;
    da.bitmap_words = ix->bitmap_words;
    da.gcur = w.gcur;
    da.by_xcd = by_xcd;
    const int chunks = (ix->l_stride + 1023) / 1024;
    denom_kernel<G><<<dim3(std::max(1, std::min(chunks, (4 * ix->num_cu + U - 1) / U)), U), 256, 0, st>>>(da);
    if (whole) ix->mark(4, st);

    // Small batches: the key histogram and the classification pass as one launch, every block taking the unit's
    // whole histogram itself (keyclass_kernel); otherwise two chip-wide launches.
    const bool keyclass = ix->sel_bits && (ix->keyclass < 0 ? (long long)ix->l_stride * U <= 2048ll * ix->num_cu : ix->keyclass != 0);
    if (keyclass) {
        KeyClassArgs kc{};
        kc.u = u;
        kc.ctx_lens = d_ctx_lens;
        kc.ncand = w.ncand;
        kc.l_stride = ix->l_stride;
        kc.top_k = p.top_k;
        kc.z = w.z;
        kc.m_key = w.m_key;
        kc.S = w.S;
        kc.kbuf = w.kbuf;
        kc.bits_stride = 2 * ((ix->l_stride + 63) / 64);
        kc.gbm = w.gbm;
        kc.glist = w.glist;
        kc.gcur = w.gcur;
        kc.ginfo = w.ginfo;
        kc.by_xcd = by_xcd;
        keyclass_kernel<G><<<dim3(std::max(1, std::min((ix->l_stride + 4095) / 4096, (2 * ix->num_cu + U - 1) / U)), U), 1024, 0, st>>>(kc);
        if (whole) ix->mark(5, st);
        if (&w_all == &ix->ws) ix->last_step_fused = true;   // no 2048-bucket histogram is left for a second ranking
    } else {
    KeyArgs ka{};
    ka.u = u;
    ka.ctx_lens = d_ctx_lens;
    ka.ncand = w.ncand;
    ka.l_stride = ix->l_stride;
    ka.z = w.z;
    ka.m_key = w.m_key;
    ka.S = w.S;
    ka.kbuf = w.kbuf;
    ka.ghist = w.ghist;
    ka.gcur = w.gcur;
    ka.by_xcd = by_xcd;
    keyhist_kernel<G><<<dim3(std::max(1, std::min((ix->l_stride + 4095) / 4096, (2 * ix->num_cu + U - 1) / U)), U), 1024, 0, st>>>(ka);
    if (whole) ix->mark(5, st);
    }

    if (ix->sel_bits && !keyclass) {
        ClassifyArgs ca{};
        ca.u = u;
        ca.ctx_lens = d_ctx_lens;
        ca.ncand = w.ncand;
        ca.l_stride = ix->l_stride;
        ca.top_k = p.top_k;
        ca.kbuf = w.kbuf;
        ca.ghist = w.ghist;
        ca.bits_stride = 2 * ((ix->l_stride + 63) / 64);
        ca.gbm = w.gbm;
        ca.glist = w.glist;
        ca.gcur = w.gcur;
        ca.ginfo = w.ginfo;
        ca.by_xcd = by_xcd;
        classify_kernel<<<dim3(std::max(1, std::min(chunks, (4 * ix->num_cu + U - 1) / U)), U), 256, 0, st>>>(ca);
    }
    if (whole) ix->mark(6, st);

    SelectArgs se{};
    se.u = u;
    se.ctx_lens = d_ctx_lens;
    se.ncand = w.ncand;
    se.cand = w.cand;
    se.crow = w.crow;
    se.l_stride = ix->l_stride;
    se.top_k = p.top_k;
    se.z = w.z;
    se.m_key = w.m_key;
    se.kbuf = w.kbuf;
    se.ghist = w.ghist;
    se.bits_words = ix->sel_bits;
    if (ix->sel_bits) {
        se.gbm = w.gbm;
        se.glist = w.glist;
        se.ginfo = w.ginfo;
        se.bits_stride = 2 * ((ix->l_stride + 63) / 64);
    }
    se.sel = w.sel;
    se.srow = w.srow;
    se.zsel = w.zsel;
    se.nsel = w.nsel;
    se.out_sel = out_sel;
    AttnArgs aa{};
    aa.v_pages = v_pages;
    aa.g = p.n_kv_heads;
    aa.h = p.n_q_heads;
    aa.top_k = p.top_k;
    aa.srow = w.srow;
    aa.nsel = w.nsel;
    aa.zsel = w.zsel;
    aa.out = out;
    aa.out_lse = out_lse;
    aa.win = window ? w.win : nullptr;
    aa.m_key = w.m_key;
    if (ix->fused_lds) {
        if (whole) ix->mark(7, st);   // no separate selection launch: its stage reads as the cost of an event pair
        if (ix->attn_slices == 8)
            select_attn_kernel<T, G, 8><<<dim3(8 * U), 1024, ix->fused_lds, st>>>(se, aa);
        else
            select_attn_kernel<T, G, 4><<<dim3(4 * U), 1024, ix->fused_lds, st>>>(se, aa);
    } else {
        rerank_select_kernel<G><<<dim3(U), 1024, ix->select_lds, st>>>(se);
        if (whole) ix->mark(7, st);
        if (ix->attn_slices == 8)
            sparse_attn_kernel<T, G, 8><<<dim3(8 * U), 1024, ix->attn_lds, st>>>(aa);
        else
            sparse_attn_kernel<T, G, 4><<<dim3(4 * U), 1024, ix->attn_lds, st>>>(aa);
    }
    if (whole) ix->mark(8, st);
    if (whole && ix->prof_step < ix->prof_max) {   // a null kernel between two events: what the bracketing itself costs
        fill_u32_kernel<<<dim3(1), 64, 0, st>>>((uint32_t *)w.nsel, 0u, 0);
        if (whole) ix->mark(9, st);
    }
    if (whole && ix->prof_step < ix->prof_max) ix->prof_step++;
    HIP_TRY(hipGetLastError());
    ix->have_step = &w_all == &ix->ws;   // the update reads the index's own workspace
    return CTKVR_OK;
}

// One step for the whole batch: a single group on the caller's stream, or (several sequences, no per-kernel
// timing, staged launches) the groups side by side -- the first on the caller's stream, the others on the
// library's streams, forked from and joined back into the caller's stream with events, so that the step is
// still one unit of work on that stream and can be captured into a graph.
template <typename T, int G>
int decode_launch(ctkvr_index *ix, const StepWs &w, const void *q, const void *k_pages, const void *v_pages, const int32_t *bt,
                  int max_pages, const int32_t *cur_lens, float *out, float *out_lse, int32_t *out_sel, int32_t *out_ncand,
                  int32_t *out_probe, hipStream_t st)
{
    const int B = ix->p.batch;
    const bool fused = ix->fused_bpu && ix->decode_path == CTKVR_PATH_FUSED;
    const int ng = (fused || ix->prof_step < ix->prof_max) ? 1 : std::min(ix->n_groups, B);
    if (ng <= 1)
        return decode_launch_group<T, G>(ix, w, 0, B, true, q, k_pages, v_pages, bt, max_pages, cur_lens, out, out_lse, out_sel,
                                         out_ncand, out_probe, st);
    HIP_TRY(hipEventRecord(ix->ev_fork, st));
    int rc = CTKVR_OK;
    for (int gi = 0; gi < ng && rc == CTKVR_OK; ++gi) {
        const int b0 = (int)((long long)B * gi / ng), b1 = (int)((long long)B * (gi + 1) / ng);
        hipStream_t gs = gi == 0 ? st : ix->side[gi - 1];
        if (gi > 0) HIP_TRY(hipStreamWaitEvent(gs, ix->ev_fork, 0));
        rc = decode_launch_group<T, G>(ix, w, b0, b1 - b0, false, q, k_pages, v_pages, bt, max_pages, cur_lens, out, out_lse,
                                       out_sel, out_ncand, out_probe, gs);
        if (gi > 0 && rc == CTKVR_OK) {
            HIP_TRY(hipEventRecord(ix->ev_join[gi - 1], gs));
            HIP_TRY(hipStreamWaitEvent(st, ix->ev_join[gi - 1], 0));
        }
    }
    return rc;
}

template <typename T>
int decode_dispatch(ctkvr_index *ix, const StepWs &w, const void *q, const void *k, const void *v, const int32_t *bt, int mp,
                    const int32_t *cur, float *out, float *lse, int32_t *sel, int32_t *ncand, int32_t *probe, hipStream_t st)
{
    switch (ix->G) {
        case 1: return decode_launch<T, 1>(ix, w, q, k, v, bt, mp, cur, out, lse, sel, ncand, probe, st);
        case 2: return decode_launch<T, 2>(ix, w, q, k, v, bt, mp, cur, out, lse, sel, ncand, probe, st);
        case 4: return decode_launch<T, 4>(ix, w, q, k, v, bt, mp, cur, out, lse, sel, ncand, probe, st);
        default: return decode_launch<T, 8>(ix, w, q, k, v, bt, mp, cur, out, lse, sel, ncand, probe, st);
    }
}

// Lloyd iterations on the centroid table (k-means centroid mode)
template <int G> int run_kmeans_g(ctkvr_index *ix, KmeansArgs ka, hipStream_t st)
{
    const int U = ix->units;
    const size_t hn_lds = (size_t)((ix->c_max + 127) & ~127) * 4;
    hipError_t e = hipFuncSetAttribute((const void *)kmeans_assign_kernel<G>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)hn_lds);
    if (e != hipSuccess) return fail(CTKVR_EHIP, "k-means set-up: %s", hipGetErrorString(e));
    kmeans_init_kernel<<<dim3(ix->c_max, ix->p.n_q_heads, ix->p.batch), 128, 0, st>>>(ka, G);
    for (int it = 0; it < ix->p.kmeans_iters; ++it) {
        kmeans_halfnorm_kernel<G><<<dim3((ix->c_max + 15) / 16, U), 256, 0, st>>>(ka);
        kmeans_assign_kernel<G><<<dim3((ix->s_max + 255) / 256, U), 512, hn_lds, st>>>(ka);
        kmeans_offsets_kernel<<<dim3(U), 1024, 0, st>>>(ka);
        kmeans_scatter_kernel<<<dim3((ix->s_max + 255) / 256, U), 256, 0, st>>>(ka);
        kmeans_reduce_kernel<G><<<dim3(ix->c_max, U), 512, 0, st>>>(ka);
    }
    HIP_TRY(hipGetLastError());
    return CTKVR_OK;
}

int run_kmeans(ctkvr_index *ix, const bf16_t *q_prefill, const int32_t *d_first, const int32_t *init_pos, hipStream_t st)
{
    const size_t U = ix->units;
    KmeansArgs ka{};
    ka.g = ix->p.n_kv_heads;
    ka.h = ix->p.n_q_heads;
    ka.c_max = ix->c_max;
    ka.s_max = ix->s_max;
    ka.n_cent = ix->d_n_cent;
    ka.ctx_lens = ix->d_ctx_lens;
    ka.first_row = d_first;
    ka.q = q_prefill;
    ka.centroids = (bf16_t *)ix->centroids;
    ka.init_pos = init_pos;
    void *bufs[6] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    const size_t sz[6] = {U * ix->c_max * 4, U * ix->s_max * 4, U * ix->c_max * 4,
                          U * ix->c_max * 4, U * ix->c_max * 4, U * ix->s_max * 4};
    int rc = CTKVR_OK;
    for (int i = 0; i < 6 && rc == CTKVR_OK; ++i) {
        hipError_t e = hipMalloc(&bufs[i], sz[i]);
        if (e == hipSuccess && i == 2) e = hipMemsetAsync(bufs[i], 0, sz[i], st);
        if (e != hipSuccess) rc = fail(CTKVR_ENOMEM, "k-means scratch: %s", hipGetErrorString(e));
    }
    if (rc == CTKVR_OK) {
        ka.half_norm = (float *)bufs[0];
        ka.assign = (int32_t *)bufs[1];
        ka.counts = (uint32_t *)bufs[2];
        ka.start = (uint32_t *)bufs[3];
        ka.cursor = (uint32_t *)bufs[4];
        ka.order = (int32_t *)bufs[5];
        switch (ix->G) {
            case 1: rc = run_kmeans_g<1>(ix, ka, st); break;
            case 2: rc = run_kmeans_g<2>(ix, ka, st); break;
            case 4: rc = run_kmeans_g<4>(ix, ka, st); break;
            default: rc = run_kmeans_g<8>(ix, ka, st); break;
        }
    }
    hipError_t es = hipStreamSynchronize(st);
    if (rc == CTKVR_OK && es != hipSuccess) rc = fail(CTKVR_EHIP, "k-means: %s", hipGetErrorString(es));
    for (void *b : bufs)
        if (b) (void)hipFree(b);
    return rc;
}

// Algorithm 2 line 12 after a decode step: the step's ranking keys, their histogram and the
// recalled ids are still in the workspace.
template <typename T, int G> int update_launch(ctkvr_index *ix, const void *q, hipStream_t st)
{
    const ctkvr_params &p = ix->p;
    const int U = ix->units;
    DcuArgs da{};
    da.g = p.n_kv_heads;
    da.h = p.n_q_heads;
    da.G = G;
    da.c_max = ix->c_max;
    da.rho = p.list_len;
    da.n_cent = ix->d_n_cent;
    da.count = ix->d_dcu_count;
    da.q = q;
    da.centroids = ix->centroids;
    da.inv_norm_c = ix->inv_norm_c;
    da.lists = ix->lists;
    if (p.list_len == p.top_k) {   // the list is the selection of line 6
        da.src = ix->ws.sel;
        da.nsrc = ix->ws.nsel;
        da.src_stride = p.top_k;
    } else {                       // the same ranking once more, with budget rho
        Units u = decode_units(ix);
        const int chunks = (ix->l_stride + 1023) / 1024;
        SelectArgs se{};
        se.u = u;
        se.ctx_lens = ix->d_ctx_lens;
        se.ncand = ix->ws.ncand;
        se.cand = ix->ws.cand;
        se.l_stride = ix->l_stride;
        se.top_k = p.list_len;
        se.z = ix->ws.z;
        se.m_key = ix->ws.m_key;
        se.kbuf = ix->ws.kbuf;
        se.ghist = ix->ws.ghist;
        se.bits_words = ix->sel_bits;
        se.sel = ix->dsel;
        se.nsel = ix->dnsel;
        se.ids_only = 1;
        if (ix->sel_bits && ix->last_step_fused) {
            // the single launch leaves the ranking keys but not their 2048-bucket histogram: taken here
            fill_u32_kernel<<<dim3((unsigned)(((size_t)U * kBuckets + 255) / 256)), 256, 0, st>>>(ix->ws.ghist, 0u, (size_t)U * kBuckets);
            KeyArgs ka{};
            ka.u = u;
            ka.ctx_lens = ix->d_ctx_lens;
            ka.ncand = ix->ws.ncand;
            ka.l_stride = ix->l_stride;
            ka.z = nullptr;
            ka.m_key = ix->ws.m_key;
            ka.S = ix->ws.S;
            ka.kbuf = ix->ws.kbuf;
            ka.ghist = ix->ws.ghist;
            ka.gcur = ix->ws.gcur;
            keyhist_kernel<G><<<dim3(std::max(1, std::min((ix->l_stride + 4095) / 4096, (2 * ix->num_cu + U - 1) / U)), U), 1024, 0, st>>>(ka);
        }
        if (ix->sel_bits) {
            fill_u32_kernel<<<dim3((U + 255) / 256), 256, 0, st>>>(ix->ws.gcur, 0u, (size_t)U);
            ClassifyArgs ca{};
            ca.u = u;
            ca.ctx_lens = ix->d_ctx_lens;
            ca.ncand = ix->ws.ncand;
            ca.l_stride = ix->l_stride;
            ca.top_k = p.list_len;
            ca.kbuf = ix->ws.kbuf;
            ca.ghist = ix->ws.ghist;
            ca.bits_stride = 2 * ((ix->l_stride + 63) / 64);
            ca.gbm = ix->ws.gbm;
            ca.glist = ix->ws.glist;
            ca.gcur = ix->ws.gcur;
            ca.ginfo = ix->ws.ginfo;
            classify_kernel<<<dim3(std::max(1, std::min(chunks, (4 * ix->num_cu + U - 1) / U)), U), 256, 0, st>>>(ca);
            se.gbm = ix->ws.gbm;
            se.glist = ix->ws.glist;
            se.ginfo = ix->ws.ginfo;
            se.bits_stride = ca.bits_stride;
        }
        rerank_select_kernel<G><<<dim3(U), 1024, ix->select_lds, st>>>(se);
        da.src = ix->dsel;
        da.nsrc = ix->dnsel;
        da.src_stride = p.list_len;
    }
    dcu_write_kernel<T><<<dim3(U), 256, 0, st>>>(da);
    HIP_TRY(hipGetLastError());
    ix->have_step = false;
    return CTKVR_OK;
}

template <typename T> int update_dispatch(ctkvr_index *ix, const void *q, hipStream_t st)
{
    switch (ix->G) {
        case 1: return update_launch<T, 1>(ix, q, st);
        case 2: return update_launch<T, 2>(ix, q, st);
        case 4: return update_launch<T, 4>(ix, q, st);
        default: return update_launch<T, 8>(ix, q, st);
    }
}

int min_pages_needed(const ctkvr_index *ix)
{
    return (ix->s_max + ix->p.page_size - 1) / ix->p.page_size;
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

const char *ctkvr_last_error(void) { return g_err.c_str(); }

int ctkvr_build_index(const ctkvr_params *p, const void *q_prefill, const int32_t *cu_seqlens, int32_t q_is_tail,
                      const void *k_pages, const int32_t *block_table, int32_t max_pages, const int32_t *ctx_lens,
                      const int32_t *init_pos, void *hip_stream, ctkvr_index **out_index)
{
    if (!out_index) return fail(CTKVR_EINVAL, "out_index is NULL");
    *out_index = nullptr;
    TRY(check_params(p, ctx_lens));
    if (!q_prefill || !cu_seqlens || !k_pages || !block_table) return fail(CTKVR_EINVAL, "a required pointer is NULL");
    const bool kmeans = p->centroid_mode == CTKVR_CENTROID_KMEANS;
    if (kmeans) {
        if (p->dtype != CTKVR_BF16) return fail(CTKVR_EUNSUPPORTED, "the k-means centroid mode needs bf16 data");
        if (q_is_tail) return fail(CTKVR_EINVAL, "the k-means centroid mode needs all prompt queries (q_is_tail = 0)");
        if (!init_pos) return fail(CTKVR_EINVAL, "the k-means centroid mode needs init_pos");
        if (p->kmeans_iters < 0 || p->kmeans_iters > 1000) return fail(CTKVR_EINVAL, "kmeans_iters %d outside 0..1000", p->kmeans_iters);
    }
    if (p->build_algo == CTKVR_BUILD_MFMA && p->dtype != CTKVR_BF16)
        return fail(CTKVR_EUNSUPPORTED, "the matrix-core list build needs bf16 data");
    std::vector<int32_t> first_row(p->batch);
    for (int b = 0; b < p->batch; ++b) {
        int s = ctx_lens[b];
        int C = p->n_centroids ? p->n_centroids : s / p->centroid_div;
        int rows = cu_seqlens[b + 1] - cu_seqlens[b];
        int need = q_is_tail ? C : s;
        if (rows != need)
            return fail(CTKVR_EINVAL, "sequence %d: cu_seqlens gives %d query rows, expected %d", b, rows, need);
        if (max_pages * p->page_size < s) return fail(CTKVR_EINVAL, "max_pages %d too small for ctx_len %d", max_pages, s);
        first_row[b] = kmeans ? cu_seqlens[b] : cu_seqlens[b] + rows - C;
    }
    ctkvr_index *ix = nullptr;
    TRY(create_index(p, ctx_lens, &ix));
    hipStream_t st = (hipStream_t)hip_stream;
    int rc = CTKVR_OK;
    int32_t *d_first = nullptr;
    hipError_t e = hipMalloc((void **)&d_first, (size_t)p->batch * 4);
    if (e == hipSuccess) e = hipMemcpy(d_first, first_row.data(), (size_t)p->batch * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) rc = fail(CTKVR_EHIP, "build set-up: %s", hipGetErrorString(e));
    if (rc == CTKVR_OK) {
        dim3 grid(ix->c_max, p->n_q_heads, p->batch);
        if (kmeans) {
            rc = run_kmeans(ix, (const bf16_t *)q_prefill, d_first, init_pos, st);
            if (rc == CTKVR_OK) rc = launch_inv_norms<bf16_t>(ix, st);
            if (rc == CTKVR_OK) rc = build_lists_dispatch<bf16_t>(ix, k_pages, block_table, max_pages, st);
        } else if (p->dtype == CTKVR_BF16) {
            copy_centroids_kernel<bf16_t><<<grid, 128, 0, st>>>((const bf16_t *)q_prefill, d_first, ix->d_n_cent,
                                                                 p->n_q_heads, ix->c_max, (bf16_t *)ix->centroids);
            rc = launch_inv_norms<bf16_t>(ix, st);
            if (rc == CTKVR_OK) rc = build_lists_dispatch<bf16_t>(ix, k_pages, block_table, max_pages, st);
        } else {
            copy_centroids_kernel<float><<<grid, 128, 0, st>>>((const float *)q_prefill, d_first, ix->d_n_cent,
                                                                p->n_q_heads, ix->c_max, (float *)ix->centroids);
            rc = launch_inv_norms<float>(ix, st);
            if (rc == CTKVR_OK) rc = build_lists_dispatch<float>(ix, k_pages, block_table, max_pages, st);
        }
    }
    if (rc == CTKVR_OK) {
        e = hipStreamSynchronize(st);
        if (e != hipSuccess) rc = fail(CTKVR_EHIP, "build: %s", hipGetErrorString(e));
    }
    if (d_first) (void)hipFree(d_first);
    if (rc != CTKVR_OK) {
        delete ix;
        return rc;
    }
    *out_index = ix;
    return CTKVR_OK;
}

int ctkvr_index_load(const ctkvr_params *p, const int32_t *ctx_lens, const void *centroids, const int32_t *lists,
                     void *hip_stream, ctkvr_index **out_index)
{
    if (!out_index) return fail(CTKVR_EINVAL, "out_index is NULL");
    *out_index = nullptr;
    TRY(check_params(p, ctx_lens));
    if (!centroids || !lists) return fail(CTKVR_EINVAL, "a required pointer is NULL");
    ctkvr_index *ix = nullptr;
    TRY(create_index(p, ctx_lens, &ix));
    // every id a decode step may touch must be a valid key id of its sequence
    const int g = p->n_kv_heads;
    for (int b = 0; b < p->batch; ++b)
        for (int kv = 0; kv < g; ++kv)
            for (int j = 0; j < ix->n_cent[b]; ++j) {
                const int32_t *l = lists + (((size_t)b * g + kv) * ix->c_max + j) * p->list_len;
                for (int r = 0; r < p->list_len; ++r)
                    if (l[r] < 0 || l[r] >= ix->ctx_lens[b]) {
                        delete ix;
                        return fail(CTKVR_EINVAL, "list (%d,%d,%d)[%d] = %d is not a key id of the sequence", b, kv, j, r, l[r]);
                    }
            }
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t es = elem_size(p->dtype);
    hipError_t e = hipMemcpy(ix->centroids, centroids, (size_t)p->batch * p->n_q_heads * ix->c_max * 128 * es,
                             hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(ix->lists, lists, (size_t)ix->units * ix->c_max * p->list_len * 4, hipMemcpyHostToDevice);
    int rc = CTKVR_OK;
    if (e != hipSuccess) rc = fail(CTKVR_EHIP, "index upload: %s", hipGetErrorString(e));
    if (rc == CTKVR_OK) rc = p->dtype == CTKVR_BF16 ? launch_inv_norms<bf16_t>(ix, st) : launch_inv_norms<float>(ix, st);
    if (rc == CTKVR_OK) {
        e = hipStreamSynchronize(st);
        if (e != hipSuccess) rc = fail(CTKVR_EHIP, "index upload: %s", hipGetErrorString(e));
    }
    if (rc != CTKVR_OK) {
        delete ix;
        return rc;
    }
    *out_index = ix;
    return CTKVR_OK;
}

int ctkvr_decode_step_window(ctkvr_index *idx, const void *q, const void *k_pages, const void *v_pages,
                             const int32_t *block_table, int32_t max_pages, const int32_t *cur_lens, float *out,
                             float *out_lse, int32_t *out_sel, int32_t *out_ncand, int32_t *out_probe, void *hip_stream)
{
    if (!idx) return fail(CTKVR_EINVAL, "index is NULL");
    if (!q || !k_pages || !v_pages || !block_table || !out) return fail(CTKVR_EINVAL, "a required pointer is NULL");
    if (max_pages < min_pages_needed(idx))
        return fail(CTKVR_EINVAL, "max_pages %d < %d pages of the longest sequence", max_pages, min_pages_needed(idx));
    hipStream_t st = (hipStream_t)hip_stream;
    if (idx->p.dtype == CTKVR_BF16)
        return decode_dispatch<bf16_t>(idx, idx->ws, q, k_pages, v_pages, block_table, max_pages, cur_lens, out, out_lse,
                                       out_sel, out_ncand, out_probe, st);
    return decode_dispatch<float>(idx, idx->ws, q, k_pages, v_pages, block_table, max_pages, cur_lens, out, out_lse, out_sel,
                                  out_ncand, out_probe, st);
}

int ctkvr_decode_step(ctkvr_index *idx, const void *q, const void *k_pages, const void *v_pages,
                      const int32_t *block_table, int32_t max_pages, float *out, float *out_lse, int32_t *out_sel,
                      int32_t *out_ncand, int32_t *out_probe, void *hip_stream)
{
    return ctkvr_decode_step_window(idx, q, k_pages, v_pages, block_table, max_pages, nullptr, out, out_lse, out_sel,
                                    out_ncand, out_probe, hip_stream);
}

int ctkvr_decode_step_static(ctkvr_index *idx, const void *q, const void *k_pages, const void *v_pages,
                             const int32_t *block_table, int32_t max_pages, float *out, float *out_lse, int32_t *out_sel,
                             int32_t *out_ncand, int32_t *out_probe, void *hip_stream)
{
    if (!idx) return fail(CTKVR_EINVAL, "index is NULL");
    if (!q || !k_pages || !v_pages || !block_table || !out) return fail(CTKVR_EINVAL, "a required pointer is NULL");
    if (max_pages < min_pages_needed(idx))
        return fail(CTKVR_EINVAL, "max_pages %d < %d pages of the longest sequence", max_pages, min_pages_needed(idx));
    StepWs w;
    const size_t need = carve_step_ws(w, nullptr, idx);
    if (need > kStaticScratchBytes)
        return fail(CTKVR_EUNSUPPORTED, "the step's workspace (%zu bytes) exceeds the static scratch of %zu bytes", need,
                    kStaticScratchBytes);
    unsigned char *base = nullptr;
    TRY(static_scratch(&base));
    carve_step_ws(w, base, idx);
    hipStream_t st = (hipStream_t)hip_stream;
    // The array keeps the last call's contents, possibly of another index: what a step expects to find
    // zero is cleared here (fill kernels, so that a captured call replays correctly): the recall bitmap, and
    // the selected rows (slots beyond the selection are read as valid row numbers).
    const size_t nbits = (size_t)idx->units * idx->bitmap_words, nrow = (size_t)idx->units * idx->p.top_k;
    const size_t nbar = (size_t)idx->units * kFusedBarriers;
    zero3_u32_kernel<<<dim3((unsigned)((nbits + nrow + nbar + 255) / 256)), 256, 0, st>>>(w.gbits, nbits, w.srow, nrow, w.bar, nbar);
    if (idx->p.dtype == CTKVR_BF16)
        return decode_dispatch<bf16_t>(idx, w, q, k_pages, v_pages, block_table, max_pages, nullptr, out, out_lse, out_sel,
                                       out_ncand, out_probe, st);
    return decode_dispatch<float>(idx, w, q, k_pages, v_pages, block_table, max_pages, nullptr, out, out_lse, out_sel,
                                  out_ncand, out_probe, st);
}

int ctkvr_centroid_update(ctkvr_index *idx, const void *q, void *hip_stream)
{
    if (!idx) return fail(CTKVR_EINVAL, "index is NULL");
    if (!q) return fail(CTKVR_EINVAL, "q is NULL");
    if (!idx->have_step) return fail(CTKVR_EINVAL, "no decode step since the index was built or last updated");
    hipStream_t st = (hipStream_t)hip_stream;
    if (idx->p.dtype == CTKVR_BF16) return update_dispatch<bf16_t>(idx, q, st);
    return update_dispatch<float>(idx, q, st);
}

void ctkvr_free(ctkvr_index *idx)
{
    if (!idx) return;
    (void)hipDeviceSynchronize();
    delete idx;
}

int ctkvr_profile_enable(ctkvr_index *idx, int32_t max_steps)
{
    if (!idx || max_steps < 0) return fail(CTKVR_EINVAL, "bad argument");
    HIP_TRY(hipDeviceSynchronize());
    for (hipEvent_t e : idx->events) (void)hipEventDestroy(e);
    idx->events.clear();
    idx->prof_max = idx->prof_step = 0;
    for (size_t i = 0; i < (size_t)max_steps * (CTKVR_N_STAGES + 1); ++i) {
        hipEvent_t e;
        HIP_TRY(hipEventCreate(&e));
        idx->events.push_back(e);
    }
    idx->prof_max = max_steps;
    return CTKVR_OK;
}

int ctkvr_profile_collect(ctkvr_index *idx, float *ms_host, int32_t capacity_steps, int32_t *n_steps)
{
    if (!idx || !ms_host || !n_steps) return fail(CTKVR_EINVAL, "NULL argument");
    HIP_TRY(hipDeviceSynchronize());
    int n = std::min<int>(idx->prof_step, capacity_steps);
    for (int s = 0; s < n; ++s)
        for (int k = 0; k < CTKVR_N_STAGES; ++k) {
            const hipEvent_t *ev = &idx->events[(size_t)s * (CTKVR_N_STAGES + 1)];
            HIP_TRY(hipEventElapsedTime(&ms_host[(size_t)s * CTKVR_N_STAGES + k], ev[k], ev[k + 1]));
        }
    *n_steps = n;
    idx->prof_step = 0;
    return CTKVR_OK;
}

int ctkvr_index_set_decode_path(ctkvr_index *idx, int32_t path)
{
    if (!idx) return fail(CTKVR_EINVAL, "index is NULL");
    if (path != CTKVR_PATH_AUTO && path != CTKVR_PATH_STAGED && path != CTKVR_PATH_FUSED)
        return fail(CTKVR_EINVAL, "unknown decode path %d", path);
    if (path == CTKVR_PATH_FUSED && !idx->fused_bpu)
        return fail(CTKVR_EUNSUPPORTED, "the single-launch step does not fit this geometry (%d units on %d CUs, or its shared memory)",
                    idx->units, idx->num_cu);
    idx->decode_path = path;
    return CTKVR_OK;
}

int ctkvr_release_scratch(void)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return CTKVR_OK;
    std::lock_guard<std::mutex> lock(g_build_mu);
    BuildCache &c = g_build_cache[dev];
    if (c.busy) return fail(CTKVR_EINVAL, "an index build is using the scratch");
    if (c.base) HIP_TRY(hipFree(c.base));
    c.base = nullptr;
    c.bytes = 0;
    return CTKVR_OK;
}

int ctkvr_index_build_route(const ctkvr_index *idx, int32_t *by_candidates_host, int32_t *chunks_redone_host)
{
    if (!idx) return fail(CTKVR_EINVAL, "null index");
    if (by_candidates_host) *by_candidates_host = idx->build_by_cand;
    if (chunks_redone_host) *chunks_redone_host = idx->build_redone;
    return CTKVR_OK;
}

int ctkvr_index_decode_path(const ctkvr_index *idx)
{
    if (!idx) return fail(CTKVR_EINVAL, "index is NULL");
    return (idx->fused_bpu && idx->decode_path == CTKVR_PATH_FUSED) ? CTKVR_PATH_FUSED : CTKVR_PATH_STAGED;
}

int ctkvr_index_check(ctkvr_index *idx)
{
    if (!idx) return fail(CTKVR_EINVAL, "index is NULL");
    HIP_TRY(hipDeviceSynchronize());
    uint32_t e = 0;
    HIP_TRY(hipMemcpy(&e, idx->d_err, 4, hipMemcpyDeviceToHost));
    if (e)
        return fail(CTKVR_EHIP, "a single-launch decode step gave up waiting for its sibling blocks (were two such steps "
                                "running on this GPU at once?); results since then are invalid");
    return CTKVR_OK;
}

int ctkvr_profile_phases(ctkvr_index *idx, int32_t enable, long long *ticks_host)
{
    if (!idx) return fail(CTKVR_EINVAL, "index is NULL");
    HIP_TRY(hipDeviceSynchronize());
    if (ticks_host) HIP_TRY(hipMemcpy(ticks_host, idx->d_prof, 64 * sizeof(long long), hipMemcpyDeviceToHost));
    idx->prof_phases = enable != 0;
    return CTKVR_OK;
}

int ctkvr_measure_dispatch_floor(int32_t n_launches, float *us_per_launch_host, void *hip_stream)
{
    if (n_launches < 1 || n_launches > 100000 || !us_per_launch_host) return fail(CTKVR_EINVAL, "bad argument");
    hipStream_t st = nullptr;
    (void)hip_stream;
    HIP_TRY(hipStreamCreate(&st));   // capture needs a stream of its own (not the legacy default stream)
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = CTKVR_OK;
    auto step = [&](hipError_t e, const char *what) {
        if (rc == CTKVR_OK && e != hipSuccess) rc = fail(CTKVR_EHIP, "%s: %s", what, hipGetErrorString(e));
        return rc == CTKVR_OK;
    };
    if (step(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal), "begin capture")) {
        for (int i = 0; i < n_launches; ++i) fill_u32_kernel<<<dim3(1), 64, 0, st>>>(nullptr, 0u, 0);
        step(hipStreamEndCapture(st, &graph), "end capture");
    }
    if (rc == CTKVR_OK) step(hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0), "instantiate");
    if (rc == CTKVR_OK) step(hipEventCreate(&e0), "event");
    if (rc == CTKVR_OK) step(hipEventCreate(&e1), "event");
    if (rc == CTKVR_OK) step(hipGraphLaunch(exec, st), "warm-up launch");
    if (rc == CTKVR_OK) step(hipStreamSynchronize(st), "sync");
    if (rc == CTKVR_OK) step(hipEventRecord(e0, st), "record");
    if (rc == CTKVR_OK) step(hipGraphLaunch(exec, st), "launch");
    if (rc == CTKVR_OK) step(hipEventRecord(e1, st), "record");
    if (rc == CTKVR_OK) step(hipEventSynchronize(e1), "sync");
    float ms = 0.0f;
    if (rc == CTKVR_OK) step(hipEventElapsedTime(&ms, e0, e1), "elapsed");
    if (rc == CTKVR_OK) *us_per_launch_host = ms * 1e3f / (float)n_launches;
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (exec) (void)hipGraphExecDestroy(exec);
    if (graph) (void)hipGraphDestroy(graph);
    (void)hipStreamDestroy(st);
    return rc;
}

int ctkvr_selftest_exp(uint64_t *mismatches_host, void *stream)
{
    if (!mismatches_host) return fail(CTKVR_EINVAL, "NULL argument");
    hipStream_t st = (hipStream_t)stream;
    unsigned long long *bad = nullptr;
    HIP_TRY(hipMalloc(&bad, sizeof(*bad)));
    fill_u32_kernel<<<1, 64, 0, st>>>((uint32_t *)bad, 0u, 2);
    // the negative values from -0 down to -32 have the bit patterns 0x80000000 .. 0xC2000000; then +0
    exp_selftest_kernel<<<4096, 256, 0, st>>>(0x80000000u, 0x42000001u, bad);
    exp_selftest_kernel<<<1, 256, 0, st>>>(0u, 1u, bad);
    unsigned long long h = ~0ull;
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(&h, bad, sizeof(h), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipFree(bad);
    if (e != hipSuccess) return fail(CTKVR_EHIP, "exp self-check: %s", hipGetErrorString(e));
    *mismatches_host = h;
    return CTKVR_OK;
}

int ctkvr_index_info(const ctkvr_index *idx, ctkvr_index_info_t *out)
{
    if (!idx || !out) return fail(CTKVR_EINVAL, "NULL argument");
    out->batch = idx->p.batch;
    out->n_q_heads = idx->p.n_q_heads;
    out->n_kv_heads = idx->p.n_kv_heads;
    out->head_dim = idx->p.head_dim;
    out->dtype = idx->p.dtype;
    out->c_max = idx->c_max;
    out->list_len = idx->p.list_len;
    out->n_probe = idx->p.n_probe;
    out->top_k = idx->p.top_k;
    out->l_stride = idx->l_stride;
    out->index_bytes = (int64_t)idx->units * idx->c_max * idx->p.list_len * 4;
    out->device_bytes = (int64_t)idx->device_bytes;
    return CTKVR_OK;
}

int ctkvr_index_lists(const ctkvr_index *idx, int32_t *dst_host)
{
    if (!idx || !dst_host) return fail(CTKVR_EINVAL, "NULL argument");
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(dst_host, idx->lists, (size_t)idx->units * idx->c_max * idx->p.list_len * 4, hipMemcpyDeviceToHost));
    return CTKVR_OK;
}

int ctkvr_index_centroids(const ctkvr_index *idx, void *dst_host)
{
    if (!idx || !dst_host) return fail(CTKVR_EINVAL, "NULL argument");
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(dst_host, idx->centroids,
                      (size_t)idx->p.batch * idx->p.n_q_heads * idx->c_max * 128 * elem_size(idx->p.dtype),
                      hipMemcpyDeviceToHost));
    return CTKVR_OK;
}

int ctkvr_index_last_candidates(const ctkvr_index *idx, int32_t *dst_host)
{
    if (!idx || !dst_host) return fail(CTKVR_EINVAL, "NULL argument");
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(dst_host, idx->ws.cand, (size_t)idx->units * idx->l_stride * 4, hipMemcpyDeviceToHost));
    return CTKVR_OK;
}

#ifdef CTKVR_TRACE
int ctkvr_debug_trace_read(long long *dst_host)
{
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpyFromSymbol(dst_host, HIP_SYMBOL(ctkvr::g_trace), sizeof(long long) * 128));
    return CTKVR_OK;
}
int ctkvr_debug_blk_read(long long *dst_host)
{
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpyFromSymbol(dst_host, HIP_SYMBOL(ctkvr::g_blk), sizeof(long long) * 8 * 2048));
    return CTKVR_OK;
}
#endif

}  // extern "C"
#pragma GCC visibility pop
