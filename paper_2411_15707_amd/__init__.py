"""MI355X (gfx950) library for the client side of the Nimbus COP linear layer.

Thin ctypes binding over libnimbus_cop.so (C ABI in include/nimbus_cop.h, and
include/nimbus_rlwe.h for the server side: encryption of the weights, decryption): argument
marshalling only, every step of the computation runs in the HIP kernels.
"""
from .binding import (  # noqa: F401
    NimbusCopError,
    lib_path,
    load_library,
    nimbus_cop_matmul,
    nimbus_cop_matmul_valu,
    nimbus_cop_matmul_prepared,
    nimbus_cop_matmul_prepared_static,
    nimbus_cop_matmul_staged,
    nimbus_cop_pack,
    nimbus_cop_check_inputs,
    nimbus_cop_packed_count,
    nimbus_cop_stage_shares,
    nimbus_cop_prepare,
    nimbus_cop_prepared_bytes,
    nimbus_cop_strerror,
    nimbus_cop_version,
    nimbus_cop_workspace_bytes,
    EXPORTED_SYMBOLS,
    CALIBRATION_SYMBOLS,
    nimbus_calib_butterflies,
    nimbus_calib_mfma_i8,
    nimbus_calib_stream_read,
    LOADER_SYMBOLS,
    nimbus_loader_create,
    nimbus_loader_destroy,
    nimbus_loader_load,
    nimbus_loader_acquire,
    nimbus_loader_release,
    RLWE_SYMBOLS,
    nimbus_rlwe_tables_bytes,
    nimbus_rlwe_setup,
    nimbus_rlwe_phase,
    nimbus_rlwe_decode,
    nimbus_rlwe_decrypt,
    nimbus_rlwe_encrypt,
)
