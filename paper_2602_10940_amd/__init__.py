"""MI355X (gfx950) hot path of Unified Sequence Parallel attention: ring attention with
log-sum-exp merging and FP8 (E4M3) payload pack/unpack, as a C-ABI HIP library
(include/usp.h, built into libusp.so) with a thin ctypes binding.

    from paper_2602_10940_amd import usp_ring_attn_fwd, usp_lse_merge, usp_fp8_quant, usp_fp8_dequant

`workloads` (numpy only) holds the seeded synthetic input generators.
"""
_BINDING_NAMES = (
    "usp_ring_attn_fwd", "usp_ring_attn_fwd_noalloc", "USP_NOALLOC_SCRATCH_BYTES", "usp_ring_attn_workspace_bytes", "usp_lse_merge", "usp_fp8_quant",
    "usp_fp8_dequant", "usp_fp8_quant_mapped", "usp_fp8_dequant_mapped", "make_row_map", "usp_version", "make_attn_desc", "load_library", "UspError", "AttnDesc",
    "USP_F32", "USP_BF16", "USP_FP8_E4M3FN", "USP_ATTN_DOUBLE_BUFFER", "USP_ATTN_UNFUSED_MERGE",
    "USP_ATTN_KERNEL_WIDE", "USP_ATTN_KERNEL_SPLIT", "USP_ATTN_FUSED_PREFETCH", "USP_ATTN_KERNEL_MIXED", "USP_ATTN_STEPWISE",
)


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
