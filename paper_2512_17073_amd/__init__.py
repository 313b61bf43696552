"""MI355X-native MoE layer with router-guided low-rank compensation: HIP kernels behind a C ABI
(libmoe_lrc.so) and a thin ctypes binding.  Importing the package does not load the library;
the first call does, and raises if it has not been built."""
from .binding import (RESIDENT, STAGED, POOLED, Stack, StackStats, Config, Layer, MoeLrcError, Stats, bf16_tensor, lib,  # noqa: F401
                      pack_codes, unpack_codes, offline_quantize, offline_factors, offline_kurtosis, allocate_ranks, f64_to_f16_bits, calibrate, selftest_decode_index, selftest_factor_pair, CAL_HBM_READ, CAL_H2D, CAL_MFMA_F16, CAL_MFMA_F16_32, CAL_MFMA_VALU, CAL_SUBSTEP)
