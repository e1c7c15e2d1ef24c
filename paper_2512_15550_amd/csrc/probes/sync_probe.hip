// Measurement aid, not part of the library: what synchronising inside one launch costs on gfx950.
//   1. the launch floor: dependent empty kernels replayed from a graph;
//   2. which XCD a block lands on (the hardware's XCC id against blockIdx % 8);
//   3. a barrier among the blocks of a launch (agent-scope atomic counter), whole grid and per XCD group;
//   4. which store kind x load kind makes one block's data visible to another block after such a barrier,
//      on the same XCD and on another one (a stale read is counted, nothing else happens).
// Every wait is bounded: on expiry a flag is set and the kernel runs to its end.
// Build:  hipcc --offload-arch=gfx950 -O3 -o sync_probe sync_probe.hip   (python -m paper_2512_15550_amd.build --probes)
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <algorithm>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); exit(1);} } while (0)

__global__ void empty_kernel(int *p) { if (p && threadIdx.x == 1234567) p[0] = 1; }

__device__ __forceinline__ unsigned xcc_id() { return __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 15u; }

constexpr unsigned kSpinMax = 1u << 22;

// Only agent scope is instantiated for the barrier: counters kept at workgroup scope are served by each CU's own
// cache and a wait on them among blocks of different CUs need not end.
enum { SC_WG = 0, SC_AGENT = 1 };

template <int SCOPE> __device__ __forceinline__ unsigned ld_ctr(const unsigned *p)
{
    if constexpr (SCOPE == SC_WG) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    else return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <int SCOPE> __device__ __forceinline__ void add_ctr(unsigned *p)
{
    if constexpr (SCOPE == SC_WG) __hip_atomic_fetch_add(p, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    else __hip_atomic_fetch_add(p, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// barrier of `members` blocks on counter ctr: arrival number `round` (1-based) is complete when ctr >= round * members
template <int SCOPE> __device__ __forceinline__ void group_barrier(unsigned *ctr, unsigned target, unsigned *abort_flag)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x == 0) {
        add_ctr<SCOPE>(ctr);
        unsigned spins = 0;
        while (ld_ctr<SCOPE>(ctr) < target) {
            if (++spins > kSpinMax || __hip_atomic_load(abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
                __hip_atomic_store(abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// ---- barrier cost -----------------------------------------------------------------------------
// GROUPED: blocks with equal blockIdx % 8 form a group (one XCD when dispatch is round-robin)
template <int SCOPE, bool GROUPED> __global__ void barrier_kernel(unsigned *ctrs, unsigned *abort_flag, int rounds, unsigned *xcc_out)
{
    const unsigned nb = gridDim.x;
    unsigned *ctr = GROUPED ? ctrs + 64 * (blockIdx.x & 7) : ctrs;
    const unsigned members = GROUPED ? (nb + 7 - (blockIdx.x & 7)) / 8 : nb;
    if (threadIdx.x == 0 && xcc_out) xcc_out[blockIdx.x] = xcc_id();
    for (int r = 1; r <= rounds; ++r) group_barrier<SCOPE>(ctr, (unsigned)r * members, abort_flag);
}

// ---- visibility -------------------------------------------------------------------------------
enum { ST_PLAIN = 0, ST_ATOMIC = 1, ST_NT = 2, ST_WG = 3 };
enum { LD_PLAIN = 0, LD_ATOMIC = 1, LD_WG = 2, LD_NT = 3 };

template <int ST> __device__ __forceinline__ void st(unsigned *p, unsigned v)
{
    if constexpr (ST == ST_PLAIN) *p = v;
    else if constexpr (ST == ST_ATOMIC) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else if constexpr (ST == ST_WG) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    else __builtin_nontemporal_store(v, p);
}
template <int LD> __device__ __forceinline__ unsigned ld(const unsigned *p)
{
    if constexpr (LD == LD_PLAIN) return *(const volatile unsigned *)p;
    else if constexpr (LD == LD_ATOMIC) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else if constexpr (LD == LD_WG) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    else return __builtin_nontemporal_load(p);
}

// each round: block b writes payload[b][tid] = f(round, b, tid); barrier (agent scope, whole grid); reads the payload
// of its partner (same group: b + 8, other group: b + 1) and counts wrong words; barrier again (so that the next
// round's writes do not race with this round's reads)
template <int ST, int LD, bool SAME> __global__ void visib_kernel(unsigned *payload, unsigned *ctrs, unsigned *abort_flag, int rounds,
                                                                  unsigned long long *bad)
{
    const unsigned nb = gridDim.x, b = blockIdx.x, tid = threadIdx.x;
    const unsigned partner = SAME ? (b + 8) % nb : (b + 1) % nb;
    unsigned wrong = 0;
    for (int r = 1; r <= rounds; ++r) {
        st<ST>(payload + (size_t)b * blockDim.x + tid, (unsigned)r * 1000003u + b * 1024u + tid);
        group_barrier<SC_AGENT>(ctrs, (unsigned)(2 * r - 1) * nb, abort_flag);
        const unsigned v = ld<LD>(payload + (size_t)partner * blockDim.x + tid);
        wrong += v != (unsigned)r * 1000003u + partner * 1024u + tid;
        group_barrier<SC_AGENT>(ctrs, (unsigned)(2 * r) * nb, abort_flag);
    }
    if (wrong) atomicAdd(bad, (unsigned long long)wrong);
}

struct Dev {
    unsigned *ctrs, *abort_flag, *payload, *xcc;
    unsigned long long *bad;
};

template <typename F> float time_ms(F f)
{
    hipEvent_t a, b;
    CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    CK(hipEventRecord(a, 0));
    f();
    CK(hipEventRecord(b, 0));
    CK(hipEventSynchronize(b));
    float ms = 0;
    CK(hipEventElapsedTime(&ms, a, b));
    CK(hipGetLastError());
    return ms;
}

void reset(Dev &d)
{
    CK(hipMemset(d.ctrs, 0, 4096));
    CK(hipMemset(d.abort_flag, 0, 4));
    CK(hipMemset(d.bad, 0, 8));
}
unsigned aborted(Dev &d)
{
    unsigned h = 0;
    CK(hipMemcpy(&h, d.abort_flag, 4, hipMemcpyDeviceToHost));
    return h;
}

template <int SCOPE, bool GROUPED> void run_barrier(Dev &d, int nb, int nt, int rounds, const char *name)
{
    reset(d);
    barrier_kernel<SCOPE, GROUPED><<<nb, nt>>>(d.ctrs, d.abort_flag, 4, d.xcc);   // warm
    CK(hipDeviceSynchronize());
    if (aborted(d)) { printf("barrier %-28s grid %4d x %4d: TIMED OUT in warm-up\n", name, nb, nt); return; }
    reset(d);
    float ms = time_ms([&] { barrier_kernel<SCOPE, GROUPED><<<nb, nt>>>(d.ctrs, d.abort_flag, rounds, nullptr); });
    printf("barrier %-28s grid %4d x %4d: %8.3f us/round%s\n", name, nb, nt, ms * 1e3 / rounds, aborted(d) ? "  (TIMED OUT)" : "");
    fflush(stdout);
}

template <int ST, int LD, bool SAME> void run_visib(Dev &d, int nb, int nt, int rounds, const char *name)
{
    reset(d);
    float ms = time_ms([&] { visib_kernel<ST, LD, SAME><<<nb, nt>>>(d.payload, d.ctrs, d.abort_flag, rounds, d.bad); });
    unsigned long long bad = 0;
    CK(hipMemcpy(&bad, d.bad, 8, hipMemcpyDeviceToHost));
    printf("visib %-44s %s: wrong words %llu of %llu, %7.3f us/round%s\n", name, SAME ? "same group " : "other group", bad,
           (unsigned long long)nb * nt * rounds, ms * 1e3 / rounds, aborted(d) ? "  (TIMED OUT)" : "");
    fflush(stdout);
}

int main()
{
    Dev d;
    CK(hipMalloc(&d.ctrs, 4096));
    CK(hipMalloc(&d.abort_flag, 4));
    CK(hipMalloc(&d.payload, 4 << 20));
    CK(hipMalloc(&d.xcc, 4096 * 4));
    CK(hipMalloc(&d.bad, 8));
    hipDeviceProp_t pr;
    CK(hipGetDeviceProperties(&pr, 0));
    printf("device %s, %d CUs, L2 %d KB\n", pr.name, pr.multiProcessorCount, pr.l2CacheSize >> 10);

    // ---- 1. launch floor: N dependent empty kernels in one graph ------------------------------------
    for (int nt : {64, 1024}) {
        for (int nb : {1, 256}) {
            hipStream_t s;
            CK(hipStreamCreate(&s));
            hipGraph_t g;
            hipGraphExec_t ge;
            const int N = 200;
            CK(hipStreamBeginCapture(s, hipStreamCaptureModeGlobal));
            for (int i = 0; i < N; ++i) empty_kernel<<<nb, nt, 0, s>>>(nullptr);
            CK(hipStreamEndCapture(s, &g));
            CK(hipGraphInstantiate(&ge, g, nullptr, nullptr, 0));
            CK(hipGraphLaunch(ge, s));
            CK(hipStreamSynchronize(s));
            hipEvent_t a, b;
            CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
            CK(hipEventRecord(a, s));
            CK(hipGraphLaunch(ge, s));
            CK(hipEventRecord(b, s));
            CK(hipEventSynchronize(b));
            float ms;
            CK(hipEventElapsedTime(&ms, a, b));
            printf("graph of %d empty kernels %4d x %4d: %.3f us per kernel\n", N, nb, nt, ms * 1e3 / N);
            CK(hipGraphExecDestroy(ge)); CK(hipGraphDestroy(g)); CK(hipStreamDestroy(s));
        }
    }
    fflush(stdout);

    // ---- 2. XCC ids ------------------------------------------------------------------------------
    {
        reset(d);
        barrier_kernel<SC_AGENT, false><<<256, 256>>>(d.ctrs, d.abort_flag, 2, d.xcc);
        CK(hipDeviceSynchronize());
        std::vector<unsigned> x(256);
        CK(hipMemcpy(x.data(), d.xcc, 256 * 4, hipMemcpyDeviceToHost));
        int rr = 0;
        for (int i = 0; i < 256; ++i) rr += (x[i] == (unsigned)(i & 7));
        printf("xcc_id == blockIdx %% 8 for %d of 256 blocks; first 16:", rr);
        for (int i = 0; i < 16; ++i) printf(" %u", x[i]);
        printf("\n");
        reset(d);
        barrier_kernel<SC_AGENT, false><<<512, 512>>>(d.ctrs, d.abort_flag, 2, d.xcc);
        CK(hipDeviceSynchronize());
        x.resize(512);
        CK(hipMemcpy(x.data(), d.xcc, 512 * 4, hipMemcpyDeviceToHost));
        rr = 0;
        for (int i = 0; i < 512; ++i) rr += (x[i] == (unsigned)(i & 7));
        printf("grid 512 x 512: xcc_id == blockIdx %% 8 for %d of 512 blocks%s\n", rr, aborted(d) ? " (TIMED OUT)" : "");
        fflush(stdout);
    }

    // ---- 3. barrier cost ---------------------------------------------------------------------------
    const int R = 2000;
    run_barrier<SC_AGENT, false>(d, 256, 256, R, "agent scope, whole grid");
    run_barrier<SC_AGENT, false>(d, 256, 1024, R, "agent scope, whole grid");
    run_barrier<SC_AGENT, false>(d, 512, 512, R, "agent scope, whole grid");
    run_barrier<SC_AGENT, false>(d, 1024, 256, R, "agent scope, whole grid");
    run_barrier<SC_AGENT, true>(d, 256, 256, R, "agent scope, per XCD group");
    run_barrier<SC_AGENT, true>(d, 256, 1024, R, "agent scope, per XCD group");
    run_barrier<SC_AGENT, true>(d, 512, 512, R, "agent scope, per XCD group");
    run_barrier<SC_AGENT, true>(d, 64, 256, R, "agent scope, per XCD group");

    // ---- 4. visibility -----------------------------------------------------------------------------
    const int RV = 500;
#define VIS(ST, LD) run_visib<ST, LD, true>(d, 256, 256, RV, #ST " -> " #LD); run_visib<ST, LD, false>(d, 256, 256, RV, #ST " -> " #LD);
    VIS(ST_PLAIN, LD_PLAIN)
    VIS(ST_PLAIN, LD_WG)
    VIS(ST_PLAIN, LD_ATOMIC)
    VIS(ST_PLAIN, LD_NT)
    VIS(ST_WG, LD_WG)
    VIS(ST_WG, LD_PLAIN)
    VIS(ST_ATOMIC, LD_PLAIN)
    VIS(ST_ATOMIC, LD_WG)
    VIS(ST_ATOMIC, LD_ATOMIC)
    VIS(ST_NT, LD_ATOMIC)
    VIS(ST_NT, LD_NT)
    printf("done\n");
    return 0;
}
