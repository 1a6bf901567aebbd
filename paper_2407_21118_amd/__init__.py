"""MI355X-native decode attention over a low-rank latent KV-cache (Palu).

The package is a thin ctypes binding over the C-ABI library built from
``csrc/`` (see ``include/palu.h``); every step of the path runs in the HIP
kernels.  PyTorch is used only for device memory and streams.
"""

from .binding import (  # noqa: F401
    PALU_BF16, PALU_DECODE_STAGES, PALU_F16, PALU_I2, PALU_I3, PALU_I4, LayerDesc, PaluError, lib_path, load_library,
    palu_attn_decode, palu_attn_decode_noalloc, palu_attn_decode_latent, palu_attn_decode_multi, palu_decode_step, palu_decode_step_t, palu_encode_kv_t, palu_attn_decode_workspace_bytes, palu_encode, palu_encode_kv, palu_encode_workspace_bytes,
    palu_encode_quant, palu_probe_mfma, palu_probe_read, palu_quant_latent, palu_rope_table_bytes, palu_set_option, palu_rope_table_init, palu_status_string, palu_version,
)
