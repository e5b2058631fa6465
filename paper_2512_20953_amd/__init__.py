"""MI355X-native pipeline-stage compute (forward + backward of a run of decoder
layers on one tensor-parallel shard).  Thin ctypes binding over libahstage.so;
every step runs in the HIP kernels of that library."""
from .binding import (AH_ARCH_GPT, AH_ARCH_LLAMA, PARAM_INDEX, AhError, Stage, StageConfig, attention_bwd, attention_fwd,
                      gemm_nn, gemm_nt, gemm_tn, lib, library_path)

__all__ = ["AH_ARCH_GPT", "AH_ARCH_LLAMA", "PARAM_INDEX", "AhError", "Stage", "StageConfig", "attention_bwd",
           "attention_fwd", "gemm_nn", "gemm_nt", "gemm_tn", "lib", "library_path"]
