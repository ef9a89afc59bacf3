"""MI355X-native hashed sparse embedding hot path (forward, backward+SGD, embedding hash,
inference cache) behind the C ABI of include/hctr.h.  This package only marshals arguments:
every step runs in the HIP kernels of libhctr.so; PyTorch supplies device memory and streams."""
from .binding import (  # noqa: F401
    F32, F16, SUM, MEAN, HctrError, EmbeddingLayer, EmbeddingGroup, EmbeddingTrainingCache, HashTable, EmbeddingCache, check_offsets, allocate_table, behind_spacer, lib, lib_path,
)
