// Measurement aid, not part of the library: is what a kernel wrote still in its XCD's L2 when the next kernel runs?
// Kernel 1: block i (i = 0..7; workgroups go to the XCDs round-robin by linear id, so block i runs on XCD i, which the
// program prints) writes a pointer-chase table of its own, one entry per 128-byte line, 2 MB.  Kernel 2: one lane of block i
// follows the table of block (i + shift) mod 8 through dependent loads of distinct lines and times them with the 100 MHz
// wall clock: shift 0 reads on the XCD that wrote, any other shift on another XCD.
// Build:  hipcc --offload-arch=gfx950 -O3 -o xcd_probe xcd_probe.hip   (python -m paper_2512_15550_amd.build --probes)
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); exit(1);} } while (0)

__device__ __forceinline__ unsigned xcc_id() { return __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 15u; }
constexpr int kEntries = 16384;   // per table, one per 128-byte line
constexpr int kStride = 32;       // uint32 per line

__global__ void write_kernel(unsigned *tabs, unsigned *xcc)
{
    unsigned *t = tabs + (size_t)blockIdx.x * kEntries * kStride;
    for (int i = threadIdx.x; i < kEntries; i += blockDim.x) t[(size_t)i * kStride] = (unsigned)((i * 4099 + 17) % kEntries);
    if (threadIdx.x == 0) xcc[blockIdx.x] = xcc_id();
}

__global__ void read_kernel(const unsigned *tabs, int shift, int iters, long long *out, unsigned *xcc)
{
    if (threadIdx.x != 0) return;
    const unsigned *t = tabs + (size_t)((blockIdx.x + shift) % gridDim.x) * kEntries * kStride;
    unsigned idx = 1;
    const long long t0 = wall_clock64();
    for (int i = 0; i < iters; ++i) idx = t[(size_t)idx * kStride];   // (4099 is coprime to 16384: no short cycle)
    const long long t1 = wall_clock64();
    out[blockIdx.x] = t1 - t0;
    xcc[8 + blockIdx.x] = xcc_id();
    if (idx == 0xffffffffu) out[100] = 1;
}

int main()
{
    unsigned *tabs, *xcc;
    long long *out;
    CK(hipMalloc(&tabs, (size_t)8 * kEntries * kStride * 4));
    CK(hipMalloc(&xcc, 64 * 4));
    CK(hipMalloc(&out, 128 * 8));
    for (int shift : {0, 0, 1, 0, 3, 0, 7}) {   // (the first pair of launches also pays for loading the code)
        for (int iters : {64, 1024}) {
            write_kernel<<<8, 256>>>(tabs, xcc);
            read_kernel<<<8, 64>>>(tabs, shift, iters, out, xcc);
            CK(hipDeviceSynchronize());
            std::vector<long long> h(8);
            std::vector<unsigned> x(16);
            CK(hipMemcpy(h.data(), out, 64, hipMemcpyDeviceToHost));
            CK(hipMemcpy(x.data(), xcc, 64, hipMemcpyDeviceToHost));
            double ns = 0;
            for (int i = 0; i < 8; ++i) ns += (double)h[i] * 10.0 / iters;
            printf("table of block i+%d, %4d dependent loads: %4.0f ns per load   (writers on XCC %u %u %u %u %u %u %u %u, readers on %u %u %u %u %u %u %u %u)\n",
                   shift, iters, ns / 8, x[0], x[1], x[2], x[3], x[4], x[5], x[6], x[7], x[8], x[9], x[10], x[11], x[12], x[13], x[14], x[15]);
        }
    }
    CK(hipFree(tabs)); CK(hipFree(xcc)); CK(hipFree(out));
    return 0;
}
