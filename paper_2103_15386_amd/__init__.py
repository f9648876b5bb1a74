"""MI355X-native GPU NN-Descent (GNND) and graph merge (GGM), arxiv 2103.15386.

Thin Python binding over the C ABI of libgnnd_hip.so (include/gnnd.h): argument
marshalling only.  PyTorch provides device memory and streams; every step of
the method runs in the library's HIP kernels.  There is no CPU fallback: without
the built library (or without a GPU) the calls raise.
"""
from .binding import (  # noqa: F401
    ANGULAR_F32, CHI2_F32, COSINE_F32, JOIN_AUTO, JOIN_GRAM, JOIN_MFMA, JOIN_MFMA_DIRECT, JOIN_VALU, LISTS_PLAIN, LISTS_SEGMENTED, L2SQ_F32, L2SQ_U8, UPDATE_ALL_PAIRS,
    UPDATE_SELECTIVE, GnndError, Gnnd, IterStats,
    exact_knn, gnnd_append, gnnd_build, gnnd_build_sharded, gnnd_build_static, gnnd_build_sharded_files,
    gnnd_init_random, gnnd_iterate, gnnd_merge, library_path, load_library, recall_at,
    workspace_bytes,
)
