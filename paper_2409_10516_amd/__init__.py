"""RetrievalAttention decode hot path and index build for AMD MI355X.

`binding` wraps the C ABI of libra.so (include/ra.h); `synth` holds the seeded input
generators. The library is loaded on first use, not at import.
"""
from .binding import (Index, RaError, lib, ra_attend, ra_build_index, ra_decode_step,  # noqa: F401
                      ra_flat_topk, ra_full_attention, ra_hbm_gather_probe, ra_hbm_read_probe, ra_index_export, ra_index_import, ra_knn,
                      ra_project, ra_quantize_keys, ra_rerank, ra_search, ra_test_configure)
