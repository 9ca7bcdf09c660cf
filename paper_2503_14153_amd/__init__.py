"""MI355X-native speculative-decoding step (HIP kernels behind a C ABI) -- Python binding.

The package is a thin ctypes wrapper over `libspecdec.so` (see include/specdec.h): argument
marshalling only, every step of the path runs in the library's HIP kernels. PyTorch is used
for device memory and streams. Importing the package does not load the library; the first
call does, and fails loudly if it has not been built (`python -m paper_2503_14153_amd.build`).
"""
from .binding import (  # noqa: F401
    KVCache, Model, build_labels, kv_commit_rows, SpecDecError, StepOutput, Tree, greedy_step, lib, lib_path, prefill, sample_tokens, spec_step,
    spec_step_typical, verify_tree, verify_tree_typical, verify_tree_typical_static, EXPORTED_SYMBOLS,
)
