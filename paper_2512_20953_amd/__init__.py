"""MI355X-native pipeline-stage compute (forward + backward of a run of decoder
layers on one tensor-parallel shard).  Thin ctypes binding over libahstage.so;
every step runs in the HIP kernels of that library."""
import importlib

_LAZY = ("AH_ARCH_GPT", "AH_ARCH_LLAMA", "AH_ARCH_BERT", "PARAM_INDEX", "AhError", "Stage", "StageConfig", "attention_bwd",
         "attention_fwd", "attention_bwd_static", "ATTENTION_STATIC_MAX_ROWS", "gemm_nn", "gemm_nn_swiglu", "gemm_nt", "gemm_tn", "gemm_tn_segmented", "lib", "library_path", "query_sizes", "cost_layers_time",
         "cost_pipeline_time", "cost_iteration_time", "cost_idle_fractions", "cost_partition_layers")


def __getattr__(name):
    # the binding loads libahstage.so on first use, so that importing the package
    # (to reach paper_2512_20953_amd.build) works before the library is built
    if name in _LAZY:
        return getattr(importlib.import_module(__name__ + ".binding"), name)
    raise AttributeError(name)
