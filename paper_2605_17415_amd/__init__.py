"""IVF-TQ hot path for AMD MI355X: HIP kernels behind a C ABI, plus a thin ctypes binding."""
from .binding import (ALLOC_FN, FREE_FN, Index, IvftqError, declared_symbols, ivftq_build_codebook,  # noqa: F401
                      ivftq_build_refined_codebook, ivftq_build_coarsened_codebook,
                      ivftq_haar_from_gaussian, ivftq_haar_rotation, ivftq_measure_mfma_rate, ivftq_quantiser_grid, ivftq_rerank, ivftq_version,
                      load_library)
