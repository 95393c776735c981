"""libentro for MI355X: Huffman-coded LLM weights decoded on the GPU.

The Python layer only marshals arguments into the C ABI declared in
include/entro.h; every step of the hot path runs in the HIP kernels of
libentro.so.  Importing the package does not need a GPU; calling a device entry
point without the built library raises.
"""
from .binding import (  # noqa: F401
    EntroError, Codebook, QParams, EncodedTensor, DeviceTensor, Plan,
    lib, library_path,
    entro_quantize, entro_build_codebook, entro_codebook_from_counts, entro_codebook_from_lengths,
    entro_codebook_from_counts_limited, entro_build_codebook_limited,
    entro_num_chunks, entro_encode_bound, entro_encode, entro_check_offsets, entro_sub_index,
    entro_bits_saved, entro_theoretical_speedup, entro_status_string,
    entro_decode, entro_decode_dequant, entro_decode_gemv, entro_decode_gemv_static, entro_gemv_workspace_bytes,
    entro_workspace_bytes, entro_plan_init, entro_plan_staging_bytes, entro_plan_init_staged, entro_plan_run,
    entro_decode_batch, entro_decode_dequant_batch, entro_decode_gemv_batch,
    entro_last_device_error, encode_tensor, to_device,
    entro_range_device, entro_qparams_from_range, entro_scheme_for_range, entro_quantize_device, entro_encoded_bytes,
    entro_encode_device, entro_encode_device_status, compress_on_device,
    ENTRO_UNSIGNED, ENTRO_ASYMMETRIC, ENTRO_U8, ENTRO_U4_PACKED, ENTRO_F32, ENTRO_BF16,
    ENTRO_OP_DECODE, ENTRO_OP_DEQUANT, ENTRO_OP_GEMV,
)
