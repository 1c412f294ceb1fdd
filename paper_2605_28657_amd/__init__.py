"""MI355X-native windowed VAE decode (paper section 3.6): ctypes binding over libdemon_vae.so."""
from .binding import (DemonVAE, DemonVAEEncoder, DemonError, demon_vae_create_encoder, demon_vae_encode, demon_vae_encode_windowed,
                      demon_vae_encoder_weight_count, demon_vae_encoder_rf_from_config, load_library, demon_vae_create, demon_vae_destroy,  # noqa: F401
                      demon_vae_decode, demon_vae_decode_windowed, demon_vae_decode_windowed_pcm16, demon_vae_decode_windowed_gated,
                      demon_vae_decode_windowed_static,
                      demon_vae_receptive_field,
                      demon_vae_rf_from_config, demon_vae_forward_support, demon_vae_plan_windows,
                      demon_vae_weight_count, demon_vae_debug_tap, demon_vae_last_error,
                      demon_vae_set_timing, demon_vae_get_timing, demon_vae_latent_similarity, demon_vae_crossfade,
                      latent_similarity, crossfade,
                      DEMON_OK, DEMON_ERR_INVALID_ARG, DEMON_ERR_UNSUPPORTED, DEMON_ERR_WORKSPACE, DEMON_ERR_HIP,
                      DEMON_F32, DEMON_BF16, DEMON_VAE_FLAG_NO_FUSED, DEMON_VAE_FLAG_ONE_STREAM, DEMON_VAE_FLAG_NO_WIDE_TILE, DEMON_VAE_FLAG_NO_HEAD_FUSION)
