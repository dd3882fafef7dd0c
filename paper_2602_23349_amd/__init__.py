"""MI355X-native FlashOptim optimizer-step library: thin Python binding over the C ABI.

Importing the package does not load the HIP library; the first call does, and it fails
loudly if the library has not been built (python paper_2602_23349_amd/build.py).
"""
from .binding import (  # noqa: F401
    FlashOptimError, TensorList, ParamBuffers, library_path, load_library,
    adamw_step, adamw_step_exact, adamw_step_noalloc, shard_range, sgd_step, lion_step, adamw_step_ex, sgd_step_ex, lion_step_ex, TensorListEx,
    SPLIT_WEIGHTS, QUANTIZE_STATES,
    split_weights, reconstruct_weights, split_weights_i16, reconstruct_weights_i16, reconstruction_sweep, reconstruction_sweep_ex,
    quantize_momentum, dequantize_momentum, quantize_variance, dequantize_variance,
    quantize_state, dequantize_state, quantization_nmse, compress_state, decompress_state, stream_probe, step_launch_count,
    checkpoint_size, checkpoint_pack, checkpoint_unpack,
    strerror, release_cache, version, selftest, faithful_rounding_stats, short_sqrt_state, ClockMonitor, EXPORTED_SYMBOLS, KIND,
)
