"""Relative NN-Descent graph construction on AMD MI355X (gfx950).

Thin binding over the C ABI of ``include/rnnd.h`` (``librnnd.so``, built in-tree by
``paper_2310_20419_amd.build``).  Every step runs in the library's HIP kernels; this module only
marshals arguments.  PyTorch is used for device memory and streams, nothing else.  There is no
CPU fallback: if the library is missing or no GPU is usable, calls raise.
"""
from ._binding import (  # noqa: F401
    RnndError, Stats, lib_path, load_library, exported_symbols,
    rnnd_build, rnnd_build_ex, rnnd_build_static, rnnd_release_workspace, rnnd_set_workspace_poison, rnnd_build_wide, rnnd_build_blocks, rnnd_update_neighbors_blocks, rnnd_workspace_bytes, rnnd_random_graph, rnnd_update_neighbors,
    rnnd_add_reverse_edges, rnnd_add_reverse_edges_wide, rnnd_export_graph, rnnd_search, rnnd_probe_gather, rnnd_probe_gather_map, rnnd_set_kernel_variant, rnnd_set_transpose_path, rnnd_set_scan_launches, rnnd_set_event_timing, rnnd_strerror, rnnd_version,
    pack_keys, unpack_keys, RNND_U8, RNND_F32, RNND_F16, RNND_BF16, RNND_L2SQ, RNND_MAX_R, RNND_STATIC_SCRATCH_BYTES,
)
