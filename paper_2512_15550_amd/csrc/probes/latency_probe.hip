// Measurement aid, not part of the library: one lane per block measures, with the 100 MHz wall clock, chains of
// dependent memory operations of several kinds on gfx950 (loads, stores, atomics, fences; and atomics of many blocks on
// one address), and the XCC id that blocks of 256 / 512 / 1024 threads land on.
// Build:  hipcc --offload-arch=gfx950 -O3 -o latency_probe latency_probe.hip   (python -m paper_2512_15550_amd.build --probes)
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); exit(1);} } while (0)

__device__ __forceinline__ unsigned xcc_id() { return __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 15u; }

__global__ void xcc_kernel(unsigned *out) { if (threadIdx.x == 0) out[blockIdx.x] = xcc_id(); }

// mode: 0 plain load chain (pointer chase through a table another kernel wrote), 1 agent-scope atomic load chain,
// 2 plain store + wait, 3 agent atomic store + wait, 4 agent atomic add no return + wait, 5 agent atomic add with return,
// 6 fence acquire agent, 7 fence release agent (after 64 plain stores), 8 fence acq_rel agent with nothing pending,
// 9 agent atomic add with return, every block on the same word
__global__ void lat_kernel(unsigned *tab, unsigned *scratch, int mode, int iters, long long *out)
{
    if (threadIdx.x != 0) return;
    unsigned idx = blockIdx.x * 977u % 65536u;
    long long t0 = wall_clock64();
    unsigned acc = 0;
    for (int i = 0; i < iters; ++i) {
        switch (mode) {
            case 0: idx = tab[idx]; break;
            case 1: idx = __hip_atomic_load(tab + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); break;
            case 2: scratch[(idx + i * 64) & 0xffff] = i; __builtin_amdgcn_s_waitcnt(0); break;
            case 3: __hip_atomic_store(scratch + ((idx + i * 64) & 0xffff), (unsigned)i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); __builtin_amdgcn_s_waitcnt(0); break;
            case 4: __hip_atomic_fetch_add(scratch + ((idx + i * 64) & 0xffff), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); __builtin_amdgcn_s_waitcnt(0); break;
            case 5: acc += __hip_atomic_fetch_add(scratch + ((idx + i * 64 + acc) & 0xffff), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); break;
            case 6: __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent"); break;
            case 7: for (int j = 0; j < 64; ++j) scratch[(idx + (i * 64 + j) * 16) & 0xffff] = j; __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent"); break;
            case 8: __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "agent"); break;
            case 9: acc += __hip_atomic_fetch_add(scratch + (acc & 0u), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); break;
        }
    }
    long long t1 = wall_clock64();
    out[blockIdx.x] = t1 - t0;
    if (acc == 0x12345678u || idx == 0x87654321u) out[1000] = 1;
}

__global__ void fill_tab(unsigned *tab) { unsigned i = blockIdx.x * 256 + threadIdx.x; tab[i] = (i * 40503u + 12345u) & 0xffffu; }

int main()
{
    unsigned *tab, *scratch, *xo;
    long long *out;
    CK(hipMalloc(&tab, 65536 * 4)); CK(hipMalloc(&scratch, 65536 * 4)); CK(hipMalloc(&out, 2048 * 8)); CK(hipMalloc(&xo, 4096 * 4));
    CK(hipMemset(scratch, 0, 65536 * 4));
    fill_tab<<<256, 256>>>(tab);
    CK(hipDeviceSynchronize());
    for (int nt : {256, 512, 1024}) {
        xcc_kernel<<<256, nt>>>(xo);
        CK(hipDeviceSynchronize());
        std::vector<unsigned> x(256);
        CK(hipMemcpy(x.data(), xo, 256 * 4, hipMemcpyDeviceToHost));
        int rr = 0;
        for (int i = 0; i < 256; ++i) rr += x[i] == (unsigned)(i & 7);
        printf("blocks of %4d threads: xcc_id == blockIdx %% 8 for %d of 256; first 24:", nt, rr);
        for (int i = 0; i < 24; ++i) printf(" %u", x[i]);
        printf("\n");
    }
    // with a large dynamic LDS request (one block per CU)
    {
        hipLaunchKernelGGL(xcc_kernel, dim3(256), dim3(1024), 100 * 1024, 0, xo);
        hipError_t e = hipDeviceSynchronize();
        printf("1024 threads + 100 KB LDS launch: %s\n", hipGetErrorString(e));
    }
    const char *names[] = {"plain load chain (L2/HBM)", "agent atomic load chain", "plain store + wait", "agent atomic store + wait",
                           "agent atomic add (no return) + wait", "agent atomic add with return chain", "fence acquire agent",
                           "64 plain stores + fence release agent", "fence acq_rel agent, nothing pending",
                           "agent atomic add, all blocks on one word"};
    for (int mode = 0; mode < 10; ++mode) {
        const int iters = 200;
        for (int nb : {1, 64, 256}) {
            if (nb == 256 && mode != 9) continue;
            lat_kernel<<<nb, 64>>>(tab, scratch, mode, iters, out);   // warm
            lat_kernel<<<nb, 64>>>(tab, scratch, mode, iters, out);
            CK(hipDeviceSynchronize());
            std::vector<long long> h(nb);
            CK(hipMemcpy(h.data(), out, nb * 8, hipMemcpyDeviceToHost));
            double s = 0;
            for (auto v : h) s += v;
            printf("%-44s %3d blocks: %7.1f ns per op", names[mode], nb, s / nb / iters * 10.0);
            if (mode == 9 && nb > 1) printf("  = %5.1f ns between operations on the word", s / nb / iters * 10.0 / nb);
            printf("\n");
        }
    }
    return 0;
}
