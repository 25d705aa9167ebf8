"""MI355X-native hot path of Quantized Evolution Strategies (QES): thin Python binding of libqes.

Argument marshalling only: every step of the path runs in the HIP kernels of libqes.so. PyTorch is
used for device memory and streams, nothing else. There is no CPU fallback: importing the binding
without a built library raises.
"""
from .binding import (QesError, Tensor, abi_version, bench_copy, bench_mfma, bench_noise, gemm_batch_workspace_bytes,
                      gemm_workspace_bytes, perturbed_qgemm_batch,
                      library_path, noise_delta, noise_from_words, noise_gauss, noise_words, normalize_fitness,
                      perturbed_qgemm, replay_residual, status_string, update, update_batch, update_full_residual,
                      update_stochastic_rounding)

__all__ = ["QesError", "Tensor", "abi_version", "bench_copy", "bench_mfma", "bench_noise", "gemm_batch_workspace_bytes",
           "gemm_workspace_bytes", "perturbed_qgemm_batch",
           "library_path", "noise_delta", "noise_from_words", "noise_gauss", "noise_words", "normalize_fitness",
           "perturbed_qgemm", "replay_residual", "status_string", "update", "update_batch", "update_full_residual",
           "update_stochastic_rounding"]
