"""MI355X-native hot path of split-parallel mini-batch GNN training (GSplit, arXiv 2303.13775).

The package is a thin binding over libgsplit.so (hand-written HIP for gfx950).  Importing it does
not load the library; constructing a Context does, and fails loudly if the library is missing.
"""
from .binding import (Context, SageParams, GatParams, GsplitError, load_library, LIB_PATH, EXPORTS,  # noqa: F401
                      GSPLIT_F32, GSPLIT_BF16, gsplit_sample_split_noalloc, noalloc_output_sizes,
                      gsplit_sample_split_multi, gsplit_gather_features_multi)
