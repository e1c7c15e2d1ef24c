// Arguments and sizes of the single-launch decode step (decode_fused_kernel); plain data, shared by
// the host side of the library and the translation unit that holds the kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "common.hpp"

namespace ctkvr {

constexpr int kFusedBarriers = 8;        // counters per unit (5 used)
constexpr int kFusedBins = 512;          // ranking-key histogram of the single launch: 1/8 wide in the log domain
constexpr int kFusedListCap = 1024;      // keys of the deciding bin the unit's first block resolves
constexpr int kFusedMaxBpu = 32;         // blocks per unit at most
constexpr long long kFusedWaitTicks = 20000000;   // 0.2 s of the 100 MHz wall clock

// Everything a block hands to the other blocks of its unit goes through a slot of its own (written
// with plain-address stores, never a read-modify-write on a shared word: atomics on one address are
// served one after the other, about 25 ns each on this part).
struct FusedArgs {
    int g, h, c_max, rho, n_probe, top_k, l_stride;
    int bpu;                        // blocks per unit
    int units;
    int stage;                      // staging slots per unit: bpu * (ids per block range at the longest sequence)
    int stream_k;
    float scale;
    const int32_t *n_cent, *ctx_lens;
    const void *q;                  // [batch][h][128]
    const void *centroids;          // [batch][h][c_max][128]
    const float *inv_norm_c;        // [batch][h][c_max]
    const int32_t *lists;           // [units][c_max][rho]
    Paged k;
    const void *v_pages;
    float *cos;                     // [units][c_max]
    int32_t *probe, *out_probe;     // [units][n_probe]
    // staging: block x of a unit owns the key ids [x * range, (x + 1) * range); its j-th recalled key sits at x * range + j
    int32_t *sid;                   // [units][stage] key ids
    uint32_t *srow;                 // [units][stage] physical rows
    float *z;                       // [units][stage][G] logits
    // dense, in rank order (inspection, the dynamic centroid update, the crowded-bin route)
    int32_t *cand;                  // [units][l_stride]
    uint32_t *kbuf;                 // [units][l_stride] ranking keys
    int32_t *ncand, *out_ncand;     // [units]
    // slots, one per (unit, block)
    uint32_t *slot_cnt;             // [units][bpu] recalled keys of the block's range
    uint32_t *slot_max;             // [units][bpu][G] ordered-key maxima of its logits
    unsigned long long *slot_S;     // [units][bpu][G] its share of the softmax denominators
    uint32_t *slot_hist;            // [units][bpu][kFusedBins] histogram of its ranking keys
    uint32_t *slot_npick;           // [units][bpu][2] its sure picks, its keys in the deciding bin
    int32_t *slot_sure;             // [units][bpu][top_k] ids of its sure picks, ascending
    uint4 *slot_bkt;                // [units][bpu][kFusedListCap] (key, staging position, id, 0) of its keys in the deciding bin, ascending id
    float *part;                    // [units][bpu][G][2 + 128] partial attention results
    int32_t *sel, *nsel, *out_sel;  // [units][top_k], [units]
    float *out, *out_lse;
    const float *win;               // optional window partials
    uint32_t *bar;                  // [units][kFusedBarriers], zero between steps
    uint32_t *err;                  // sticky error word
    long long *prof;                // optional [64] wall-clock stamps of unit 0's first block
};

// ids per block range for a sequence of s keys split over bpu blocks (whole bitmap words)
__host__ __device__ inline int fused_range_ids(int s, int bpu) { return (((s + bpu - 1) / bpu) + 31) & ~31; }

// Dynamic shared memory of the fused kernel, in words (nt threads per block).
__host__ __device__ inline size_t fused_smem_words(int nt, int n_probe, int s_max, int bpu, int top_k, int G)
{
    const size_t range_words = (size_t)fused_range_ids(s_max, bpu) / 32;
    size_t region = range_words + 8 * (size_t)nt + 64;                       // range bitmap + one window of ids
    const size_t p4 = (size_t)kFusedBins + (size_t)top_k + 64;               // summed histogram + sure picks
    const size_t fin = 5 * (size_t)kFusedListCap + 2 * (size_t)top_k + 512;  // bin entries (3 arrays) + winners (2) + sure and winner ids
    if (region < p4) region = p4;
    if (region < fin) region = fin;
    return (size_t)kSelLds + (size_t)n_probe + region + (size_t)16 * G * (kD + 1) + 64;
}

// Host entry points of that translation unit.  nt = threads per block (256 or 1024).
hipError_t fused_set_smem(int dtype_is_bf16, int G, int nt, size_t smem_bytes);
hipError_t fused_launch(int dtype_is_bf16, int G, int nt, unsigned grid, size_t smem_bytes, hipStream_t st, const FusedArgs &a);

}  // namespace ctkvr
