// Measurement aid, not part of the library: what bandwidth a gather of 256-byte rows at ascending, scattered positions
// reaches on gfx950, against the same loop over every row.  The launch has the shape of the decode step's scoring
// kernel at a 128K context: 32 units of 131072 rows each (1 GiB of rows in all), 64 blocks of 256 threads per unit,
// a block owns an equal share of its unit's chosen rows and walks it in tiles of 16 R rows, a 16-lane group per row
// (16 bytes per lane), R loads requested before the first is used.  Printed: GB/s of the chosen rows' bytes for
//   pattern  all (every row), bernoulli (each row with probability p), runs (runs of chosen rows of mean length 8,
//            the gaps sized to give the same p); with "paged" the rows of a unit lie in 16-row pages scattered over
//            the whole pool by a permutation, 8 units interleaved inside a page (the library's key layout)
//   loads    cached or non-temporal
//   R        4, 8, 16
//   work     fused multiply-adds per row and lane on the loaded words (four dependent chains), 0 or 80: the scoring
//            kernel spends about 80-90 vector instructions per row
//   blocks per CU  8, or 4 (forced by 40 KB of unused shared memory per block): the scoring kernel holds 4
// Build:  hipcc --offload-arch=gfx950 -O3 -o gather_probe gather_probe.hip   (python -m paper_2512_15550_amd.build --probes)
// Run:    gather_probe [p = 0.46]
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <utility>
#include <vector>
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); exit(1);} } while (0)

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
constexpr int kUnits = 32, kRowsPerUnit = 131072, kBlocksPerUnit = 64, kRowBytes = 256, kPage = 16, kUnitsPerPage = 8;

template <int V> __device__ __forceinline__ float work(uint4 v, float q0, float q1, float q2, float q3)
{
    float a0 = __uint_as_float(v.x), a1 = __uint_as_float(v.y), a2 = __uint_as_float(v.z), a3 = __uint_as_float(v.w);
#pragma unroll
    for (int i = 0; i < V / 4; ++i) {
        a0 = __fmaf_rn(a0, q0, q1); a1 = __fmaf_rn(a1, q1, q2); a2 = __fmaf_rn(a2, q2, q3); a3 = __fmaf_rn(a3, q3, q0);
    }
    return (a0 + a1) + (a2 + a3);
}

// ids: the chosen rows of every unit as row numbers in the pool, ascending by the unit's own order
template <int R, int V, bool NT> __global__ __launch_bounds__(256) void gather_kernel(const uint4 *rows, const uint32_t *ids, const int *n_ids, float *out, float q0)
{
    extern __shared__ uint32_t unused_lds[];
    const int ul = blockIdx.y, tid = threadIdx.x, lane16 = tid & 15, grp = tid >> 4;
    const int n = n_ids[ul];
    const int q = (n + gridDim.x - 1) / gridDim.x;
    const int r0 = blockIdx.x * q, r1 = min(n, r0 + q);
    const uint32_t *my = ids + (size_t)ul * kRowsPerUnit;
    const float q1 = q0 + 1.f, q2 = q0 + 2.f, q3 = q0 + 3.f;
    float acc = 0.f;
    for (int t0 = r0; t0 < r1; t0 += 16 * R) {
        uint4 v[R];
        uint32_t id[R];
#pragma unroll
        for (int r = 0; r < R; ++r) id[r] = my[min(t0 + r * 16 + grp, r1 - 1)];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint4 *p = rows + (size_t)id[r] * (kRowBytes / 16) + lane16;
            if (NT) {
                const u32x4_t x = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));   // one 16-byte load
                v[r] = make_uint4(x.x, x.y, x.z, x.w);
            } else {
                v[r] = *p;
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) acc += work<V>(v[r], q0, q1, q2, q3);
    }
    if (acc == 123.456f) out[blockIdx.y * gridDim.x + blockIdx.x] = acc + (float)unused_lds[0];   // never true for the zero-filled rows
}

static uint64_t rng_state = 0x243f6a8885a308d3ull;
static double uniform()
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) * (1.0 / 9007199254740992.0);
}

template <int R, int V, bool NT> static double time_one(const uint4 *rows, const uint32_t *ids, const int *n_ids, float *out, size_t chosen, int lds)
{
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const dim3 grid(kBlocksPerUnit, kUnits);
    CK(hipFuncSetAttribute((const void *)gather_kernel<R, V, NT>, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    for (int i = 0; i < 3; ++i) gather_kernel<R, V, NT><<<grid, 256, lds>>>(rows, ids, n_ids, out, 0.5f);
    CK(hipDeviceSynchronize());
    const int reps = 20;
    CK(hipEventRecord(e0));
    for (int i = 0; i < reps; ++i) gather_kernel<R, V, NT><<<grid, 256, lds>>>(rows, ids, n_ids, out, 0.5f);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms = 0;
    CK(hipEventElapsedTime(&ms, e0, e1));
    CK(hipEventDestroy(e0)); CK(hipEventDestroy(e1));
    return (double)chosen * kRowBytes * reps / (ms * 1e-3) * 1e-9;
}

int main(int argc, char **argv)
{
    const double p = argc > 1 ? atof(argv[1]) : 0.46;
    if (!(p > 0.0 && p <= 1.0)) { printf("p must lie in (0, 1]\n"); return 1; }
    uint4 *rows; uint32_t *ids; float *out; int *n_ids;
    const size_t total = (size_t)kUnits * kRowsPerUnit;
    CK(hipMalloc(&rows, total * kRowBytes));
    CK(hipMemset(rows, 0, total * kRowBytes));
    CK(hipMalloc(&ids, total * 4));
    CK(hipMalloc(&n_ids, kUnits * 4));
    CK(hipMalloc(&out, kUnits * kBlocksPerUnit * 4));
    std::vector<uint32_t> h(total);
    std::vector<int> hn(kUnits);
    // page table: unit u belongs to sequence u / 8 and is slot u % 8 of that sequence's pages
    const size_t pages_per_seq = kRowsPerUnit / kPage, n_pages = pages_per_seq * (kUnits / kUnitsPerPage);
    std::vector<uint32_t> perm(n_pages);
    for (size_t i = 0; i < n_pages; ++i) perm[i] = (uint32_t)i;
    for (size_t i = n_pages - 1; i > 0; --i) std::swap(perm[i], perm[(size_t)(uniform() * (double)(i + 1))]);
    const char *names[4] = {"all", "bernoulli", "runs", "runs, paged"};
    for (int pattern = 0; pattern < 4; ++pattern) {
        size_t chosen = 0;
        for (int u = 0; u < kUnits; ++u) {
            uint32_t *d = h.data() + (size_t)u * kRowsPerUnit;
            int n = 0;
            auto row_of = [&](int t) {
                if (pattern < 3) return (uint32_t)((size_t)u * kRowsPerUnit + t);
                const size_t page = perm[(size_t)(u / kUnitsPerPage) * pages_per_seq + t / kPage];
                return (uint32_t)((page * kUnitsPerPage + u % kUnitsPerPage) * kPage + t % kPage);
            };
            if (pattern == 0) {
                for (int t = 0; t < kRowsPerUnit; ++t) d[n++] = row_of(t);
            } else if (pattern == 1) {
                for (int t = 0; t < kRowsPerUnit; ++t) if (uniform() < p) d[n++] = row_of(t);
            } else {
                // a chosen run ends after each row with probability 1/8; a gap ends with the probability that gives density p
                const double end_run = 1.0 / 8.0, end_gap = p < 1.0 ? end_run * p / (1.0 - p) : 1.0;
                bool in_run = uniform() < p;
                for (int t = 0; t < kRowsPerUnit; ++t) {
                    if (in_run) d[n++] = row_of(t);
                    if (uniform() < (in_run ? end_run : end_gap)) in_run = !in_run;
                }
            }
            if (n == 0) d[n++] = row_of(0);
            hn[u] = n;
            chosen += (size_t)n;
        }
        CK(hipMemcpy(ids, h.data(), total * 4, hipMemcpyHostToDevice));
        CK(hipMemcpy(n_ids, hn.data(), kUnits * 4, hipMemcpyHostToDevice));
        printf("%-11s %.1f MB of rows per launch (density %.3f)\n", names[pattern], (double)chosen * kRowBytes * 1e-6, (double)chosen / (double)total);
        printf("  cached,       no work, 8 blocks/CU   R=4 %5.0f GB/s   R=8 %5.0f GB/s   R=16 %5.0f GB/s\n",
               time_one<4, 0, false>(rows, ids, n_ids, out, chosen, 0), time_one<8, 0, false>(rows, ids, n_ids, out, chosen, 0), time_one<16, 0, false>(rows, ids, n_ids, out, chosen, 0));
        printf("  non-temporal, no work, 8 blocks/CU   R=4 %5.0f GB/s   R=8 %5.0f GB/s   R=16 %5.0f GB/s\n",
               time_one<4, 0, true>(rows, ids, n_ids, out, chosen, 0), time_one<8, 0, true>(rows, ids, n_ids, out, chosen, 0), time_one<16, 0, true>(rows, ids, n_ids, out, chosen, 0));
        printf("  non-temporal, 80 FMAs, 8 blocks/CU   R=4 %5.0f GB/s   R=8 %5.0f GB/s\n",
               time_one<4, 80, true>(rows, ids, n_ids, out, chosen, 0), time_one<8, 80, true>(rows, ids, n_ids, out, chosen, 0));
        printf("  non-temporal, 80 FMAs, 4 blocks/CU   R=4 %5.0f GB/s   R=8 %5.0f GB/s\n",
               time_one<4, 80, true>(rows, ids, n_ids, out, chosen, 40 << 10), time_one<8, 80, true>(rows, ids, n_ids, out, chosen, 40 << 10));
        fflush(stdout);
    }
    CK(hipFree(rows)); CK(hipFree(ids)); CK(hipFree(n_ids)); CK(hipFree(out));
    return 0;
}
