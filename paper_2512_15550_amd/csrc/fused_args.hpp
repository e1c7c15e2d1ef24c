// Arguments and sizes of the single-launch decode step (decode_fused_kernel); plain data, shared by
// the host side of the library and the translation unit that holds the kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "common.hpp"

namespace ctkvr {

constexpr int kFusedChunk = 4096;        // ranks a block expands and scores per round
constexpr int kFusedBarriers = 8;        // counters per unit (6 used)
constexpr long long kFusedWaitTicks = 20000000;   // 0.2 s of the 100 MHz wall clock

struct FusedArgs {
    int g, h, c_max, rho, n_probe, top_k, bitmap_words, l_stride, bits_stride;
    int bpu;                        // blocks per unit
    int units;
    int stream_k;
    float scale;
    const int32_t *n_cent, *ctx_lens;
    const void *q;                  // [batch][h][128]
    const void *centroids;          // [batch][h][c_max][128]
    const float *inv_norm_c;        // [batch][h][c_max]
    const int32_t *lists;           // [units][c_max][rho]
    Paged k;
    const void *v_pages;
    // workspace (per unit)
    float *cos;                     // [c_max]
    int32_t *probe, *out_probe;     // [n_probe]
    uint32_t *gbits;                // [bitmap_words], zero between steps
    int32_t *cand;                  // [l_stride]
    uint32_t *crow;                 // [l_stride]
    int32_t *ncand, *out_ncand;
    float *z;                       // [l_stride][G]
    uint32_t *m_key;                // [G]
    unsigned long long *S;          // [G]
    uint32_t *kbuf;                 // [l_stride]
    uint32_t *ghist;                // [kBuckets]
    uint32_t *gbm;                  // [bits_stride] sure picks, zero between steps
    uint2 *glist;                   // [kListCap]
    uint32_t *gcur;                 // list cursor
    float *part;                    // [bpu][G][2 + 128] partial attention results
    int32_t *sel, *nsel, *out_sel;  // [top_k]
    float *out, *out_lse;
    const float *win;               // optional window partials
    uint32_t *bar;                  // [units][kFusedBarriers], zero between steps
    uint32_t *err;                  // sticky error word
    long long *prof;                // optional [64] wall-clock stamps of unit 0's first block
};

// Dynamic shared memory of the fused kernel, in words.
__host__ __device__ inline size_t fused_smem_words(int n_probe, int bitmap_words, int l_stride, int top_k, int G)
{
    const size_t sel_bits = 4 * (size_t)((l_stride + 63) / 64);
    size_t region = (size_t)bitmap_words;
    if (region < (size_t)kFusedChunk) region = kFusedChunk;
    const size_t fin = 2 * (size_t)kListCap + sel_bits + (size_t)top_k + (size_t)kListCap;
    if (region < fin) region = fin;
    if (region < (size_t)top_k) region = top_k;
    return (size_t)kSelLds + (size_t)n_probe + region + (size_t)16 * G * (kD + 1) + 64;
}


// Host entry points of that translation unit.  nt = threads per block (256 or 1024).
hipError_t fused_set_smem(int dtype_is_bf16, int G, int nt, size_t smem_bytes);
hipError_t fused_launch(int dtype_is_bf16, int G, int nt, unsigned grid, size_t smem_bytes, hipStream_t st, const FusedArgs &a);

}  // namespace ctkvr
