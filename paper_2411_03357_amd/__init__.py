"""Batched AES-GCM (AES-256 first of all) for one MI355X: a thin ctypes binding over libpgcm.so.

The binding marshals arguments only; every step of the cipher runs in the library's HIP
kernels.  Importing the package does not load the library; the first call does, and fails
loudly when libpgcm.so has not been built (python -m paper_2411_03357_amd.build).
"""
from .binding import (PgcmError, Key, expand_key, expand_key_bytes, encrypt_batch, decrypt_verify_batch,  # noqa: F401
                      encrypt_batch_keys, decrypt_verify_batch_keys, encrypt_batch_static, reserve,
                      describe_schedule, STATIC_WORKSPACE_BYTES, STATIC_MAX_CHUNKS,
                      plan_units, unit_bytes, batch_unit_bytes, library_path, load_library, set_timing, set_unit_bytes, set_one_launch, set_matrix_hash, bitsliced_keystream, copy_key_tables,
                      last_bulk_kernel_ms, bulk_kernel_ms_history, measure_passes, EXPORTS, Sequencer, seq_iv_bytes, SEQ_EXPORTS, BouncePool,
                      BOUNCE_EXPORTS, Pipe, Receiver, PIPE_EXPORTS)
