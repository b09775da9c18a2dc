"""MI355X-native masked-layer hot path of DarKnight (matrix masking).

The product is the C-ABI library ``libdarknight.so`` (hand-written HIP for
gfx950, declared in ``include/darknight.h`` and, for the finite-field
variant, ``include/darknight_field.h``).  This package is the thin
Python binding over it: same entry-point names, argument marshalling only.
PyTorch is used for device memory and streams, nothing else.
"""
from .binding import (DkError, DkLayer, lib_path, load, dk_version, dk_status_str,
                      dk_workspace_bytes, dk_layer_in_len, dk_layer_out_len, dk_coeffs,
                      dk_encode, dk_linear_fwd, dk_conv_fwd, dk_wgrad, dk_decode, dk_verify,
                      dk_decode_verify, dk_decode_verify_static, dk_static_scratch_bytes, dk_profile_enable, dk_profile_read,
                      dk_probe_mfma_rate,
                      dk_conv_fwd_decode_verify, dk_conv_fwd_decode_verify_workspace_bytes, dk_set_option, dk_get_option,
                      DK_OPT_FUSE_FWD, DK_OPT_FUSE_WGRAD, DK_FUSE_NEVER, DK_FUSE_ALWAYS, DK_FUSE_AUTO,
                      dk_coeffs_m, dk_encode_m, dk_decode_verify_m, dk_wgrad_m, dk_noise_rng, dk_encode_rng, dk_dgrad,
                      DK_OP_FWD, DK_OP_WGRAD, DK_OP_VERIFY, DK_MAX_K)

from .field import (DKF_P, DKF_L, dkf_coeffs, dkf_quantize, dkf_dequantize, dkf_encode, dkf_linear_fwd, dkf_linear_fwd_w,
                    dkf_decode_verify, dkf_wgrad, dkf_fwd_workspace_bytes, dkf_wgrad_workspace_bytes,
                    dkf_conv_fwd, dkf_conv_fwd_workspace_bytes, dkf_noise_rng, dkf_encode_rng, dkf_norm_scales,
                    dkf_coeffs_m, dkf_encode_m, dkf_decode_verify_m, dkf_wgrad_m, dkf_wgrad_workspace_bytes_m,
                    dkf_add_bias, dkf_probe_mfma_rate)

__all__ = ["DKF_P", "DKF_L", "dkf_coeffs", "dkf_quantize", "dkf_dequantize", "dkf_encode",
           "dkf_linear_fwd", "dkf_linear_fwd_w", "dkf_decode_verify", "dkf_wgrad", "dkf_fwd_workspace_bytes",
           "dkf_wgrad_workspace_bytes", "dkf_conv_fwd", "dkf_conv_fwd_workspace_bytes",
           "DkError", "DkLayer", "lib_path", "load", "dk_version", "dk_status_str",
           "dk_workspace_bytes", "dk_layer_in_len", "dk_layer_out_len", "dk_coeffs",
           "dk_encode", "dk_linear_fwd", "dk_conv_fwd", "dk_wgrad", "dk_decode", "dk_verify",
           "dk_decode_verify", "dk_decode_verify_static", "dk_static_scratch_bytes", "dk_profile_enable", "dk_profile_read",
           "dk_probe_mfma_rate",
           "dk_conv_fwd_decode_verify", "dk_conv_fwd_decode_verify_workspace_bytes", "dk_set_option", "dk_get_option",
           "DK_OPT_FUSE_FWD", "DK_OPT_FUSE_WGRAD", "DK_FUSE_NEVER", "DK_FUSE_ALWAYS", "DK_FUSE_AUTO",
           "dk_coeffs_m", "dk_encode_m", "dk_decode_verify_m", "dk_wgrad_m", "dk_noise_rng", "dk_encode_rng", "dk_dgrad",
           "dkf_noise_rng", "dkf_encode_rng", "dkf_norm_scales",
           "dkf_add_bias", "dkf_probe_mfma_rate", "dkf_coeffs_m", "dkf_encode_m", "dkf_decode_verify_m", "dkf_wgrad_m", "dkf_wgrad_workspace_bytes_m",
           "DK_OP_FWD", "DK_OP_WGRAD", "DK_OP_VERIFY", "DK_MAX_K"]
