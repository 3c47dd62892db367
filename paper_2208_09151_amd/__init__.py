"""MI355X-native hot path of the Ginex inspector-executor pipeline (arXiv 2208.09151).

Thin Python binding over ``libginex.so`` (hand-written HIP kernels for gfx950 behind the C
ABI of ``include/ginex.h``).  The functions here only marshal arguments: every step of the
path runs in the library's kernels.  PyTorch supplies device memory and streams.
There is no CPU fallback: without the built library, or without a GPU, calls raise.
"""
from .api import (GinexError, FeatureCache, SampleResult, ChangesetResult,  # noqa: F401
                  NeighborCache, neighbor_cache_build, sample_superbatch, changeset,
                  changeset_resume, static_select,
                  library_path, version)
from .pipeline import Executor, InspectorPipeline  # noqa: F401
