"""MI355X-native CTkvr hot path: thin Python binding over the C ABI of
``include/ctkvr.h`` (``libctkvr.so``, hand-written HIP for gfx950).

The binding only marshals arguments: torch tensors provide device memory and
the current HIP stream; every step of the method runs in the library's kernels.
There is no CPU or PyTorch fallback -- if the library is missing or fails to
load, importing the entry points raises.
"""
from .binding import (CtkvrError, Index, Params, ctkvr_build_index, ctkvr_decode_step, ctkvr_free,  # noqa: F401
                      ctkvr_index_info, ctkvr_index_last_candidates, ctkvr_index_lists, ctkvr_index_centroids,
                      ctkvr_index_load, ctkvr_last_error, library_path, load_library, BF16, F32, LAST_C, KMEANS,
                      BUILD_EXACT, BUILD_MFMA, ctkvr_profile_enable, ctkvr_profile_collect, ctkvr_selftest_exp, STAGE_NAMES,
                      ctkvr_centroid_update, ctkvr_decode_step_window, ctkvr_decode_step_static,
                      ctkvr_index_set_decode_path, ctkvr_index_decode_path, ctkvr_index_check, ctkvr_index_build_route, ctkvr_profile_phases,
                      ctkvr_measure_dispatch_floor, ctkvr_release_scratch, PATH_AUTO, PATH_STAGED, PATH_FUSED)
