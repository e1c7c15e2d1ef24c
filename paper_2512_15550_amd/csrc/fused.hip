// Translation unit of the single-launch decode step: the kernel's instantiations (storage type x
// group size x threads per block) and their host-side launch, compiled apart from the rest of the
// library so that the two halves build in parallel.
#include "fused.hpp"

namespace ctkvr {

namespace {

template <typename T, int G, int NT> hipError_t set_one(size_t smem)
{
    return hipFuncSetAttribute((const void *)decode_fused_kernel<T, G, NT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
}
template <typename T, int G, int NT> hipError_t launch_one(unsigned grid, size_t smem, hipStream_t st, const FusedArgs &a)
{
    decode_fused_kernel<T, G, NT><<<dim3(grid), NT, smem, st>>>(a);
    return hipGetLastError();
}

// calls f.template operator()<T, G, NT>() for the runtime triple
template <typename F> hipError_t dispatch(int bf16, int G, int nt, F f)
{
#define CTKVR_CASE(TT, GG)                                        \
    if (G == GG) return nt == 256 ? f.template operator()<TT, GG, 256>() : f.template operator()<TT, GG, 1024>();
    if (nt != 256 && nt != 1024) return hipErrorInvalidValue;
    if (bf16) {
        CTKVR_CASE(bf16_t, 1) CTKVR_CASE(bf16_t, 2) CTKVR_CASE(bf16_t, 4) CTKVR_CASE(bf16_t, 8)
    } else {
        CTKVR_CASE(float, 1) CTKVR_CASE(float, 2) CTKVR_CASE(float, 4) CTKVR_CASE(float, 8)
    }
#undef CTKVR_CASE
    return hipErrorInvalidValue;
}

struct SetSmem {
    size_t smem;
    template <typename T, int G, int NT> hipError_t operator()() const { return set_one<T, G, NT>(smem); }
};
struct Launch {
    unsigned grid;
    size_t smem;
    hipStream_t st;
    const FusedArgs &a;
    template <typename T, int G, int NT> hipError_t operator()() const { return launch_one<T, G, NT>(grid, smem, st, a); }
};

}  // namespace

hipError_t fused_set_smem(int dtype_is_bf16, int G, int nt, size_t smem_bytes)
{
    return dispatch(dtype_is_bf16, G, nt, SetSmem{smem_bytes});
}

hipError_t fused_launch(int dtype_is_bf16, int G, int nt, unsigned grid, size_t smem_bytes, hipStream_t st, const FusedArgs &a)
{
    return dispatch(dtype_is_bf16, G, nt, Launch{grid, smem_bytes, st, a});
}

}  // namespace ctkvr
