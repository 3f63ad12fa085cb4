"""MI355X-native virtual-node training step (VirtualFlow, arxiv 2009.09523, Sections 3.2
and 5.2): thin ctypes binding over the C ABI of libvf.so.  All computation happens in the
HIP kernels of the library; this package only marshals arguments."""
from .binding import (VF_ADAM, VF_BF16, VF_CONV, VF_ENCODER, VF_F32, VF_FLAG_FUSED_ACCUMULATE,
                      VF_FLAG_NO_GRAPH, VF_FLAG_ORDERED_FOLD, VF_FLAG_OVERLAP, VF_MLP, VF_SGDM, VfConfig, VfError, VirtualNodeStep,
                      exported_symbols, lib, lib_path, vf_accumulate, vf_adam_update,
                      vf_gemm, vf_gemm_noalloc, vf_partition, vf_solve_split, vf_sgdm_update, parse_state,
                      VF_NOALLOC_SCRATCH_BYTES)

__all__ = ["VF_ADAM", "VF_BF16", "VF_CONV", "VF_ENCODER", "VF_F32", "VF_FLAG_FUSED_ACCUMULATE",
           "VF_FLAG_NO_GRAPH", "VF_FLAG_ORDERED_FOLD", "VF_FLAG_OVERLAP", "VF_MLP", "VF_SGDM", "VfConfig", "VfError", "VirtualNodeStep",
           "exported_symbols", "lib", "lib_path", "vf_accumulate", "vf_adam_update",
           "vf_gemm", "vf_gemm_noalloc", "vf_partition", "vf_solve_split", "vf_sgdm_update", "parse_state",
           "VF_NOALLOC_SCRATCH_BYTES"]
