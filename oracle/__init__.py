"""CPU oracle of the windowed VAE decode.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; it shares no code with the HIP library and never calls it.
"""
from .oracle import (conv1d, convT1d, snake, decode, decode_windowed, window_grid,  # noqa: F401
                     receptive_field, backward_interval, forward_interval, omp_threads, pcm16,
                     latent_mse, latent_unchanged, crossfade, decode_gated,
                     conv1d_strided, encode_moments, encode_moments_windowed, sample_latent,
                     encoder_backward_interval, encoder_forward_interval, encoder_receptive_field)
