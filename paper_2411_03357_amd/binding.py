"""ctypes binding for the C ABI in include/pgcm.h: same names, argument marshalling only."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpgcm.so")
_lib = None

EXPORTS = ("pgcm_expand_key", "pgcm_expand_key_bytes", "pgcm_free_key", "pgcm_encrypt_batch",
           "pgcm_decrypt_verify_batch", "pgcm_encrypt_batch_iv", "pgcm_decrypt_verify_batch_iv",
           "pgcm_encrypt_batch_static", "pgcm_reserve", "pgcm_describe_schedule",
           "pgcm_encrypt_batch_keys", "pgcm_decrypt_verify_batch_keys",
           "pgcm_strerror", "pgcm_last_hip_error", "pgcm_plan_units", "pgcm_unit_bytes",
           "pgcm_batch_unit_bytes", "pgcm_set_unit_bytes", "pgcm_key_tables_bytes",
           "pgcm_copy_key_tables",
           "pgcm_set_timing", "pgcm_last_bulk_kernel_ms", "pgcm_bulk_kernel_ms_history",
           "pgcm_measure_passes", "pgcm_set_one_launch", "pgcm_set_matrix_hash",
           "pgcm_bitsliced_keystream")


class PgcmError(RuntimeError):
    def __init__(self, status, hip_error=0):
        self.status, self.hip_error = status, hip_error
        text = load_library().pgcm_strerror(status).decode()
        super().__init__("pgcm status %d (%s)%s" % (
            status, text, ", hipError %d" % hip_error if hip_error else ""))


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libpgcm.so; there is no fallback when it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libpgcm.so is not built: run `python -m paper_2411_03357_amd.build` "
                          "(needs hipcc); there is no CPU fallback")
    lib = C.CDLL(_LIB_PATH)
    vp, sz = C.c_void_p, C.c_size_t
    lib.pgcm_expand_key.argtypes = [vp, vp, C.POINTER(vp)]
    lib.pgcm_expand_key.restype = C.c_int
    lib.pgcm_expand_key_bytes.argtypes = [vp, C.c_uint32, vp, C.POINTER(vp)]
    lib.pgcm_expand_key_bytes.restype = C.c_int
    lib.pgcm_free_key.argtypes = [vp]
    lib.pgcm_free_key.restype = None
    lib.pgcm_encrypt_batch.argtypes = [vp, sz, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.pgcm_encrypt_batch.restype = C.c_int
    lib.pgcm_encrypt_batch_static.argtypes = [vp, sz, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.pgcm_encrypt_batch_static.restype = C.c_int
    lib.pgcm_reserve.argtypes = [vp, vp, sz, C.c_uint64]
    lib.pgcm_reserve.restype = C.c_int
    lib.pgcm_describe_schedule.argtypes = [sz, vp, C.c_uint32, C.c_uint32, vp, vp, sz]
    lib.pgcm_describe_schedule.restype = C.c_int
    lib.pgcm_decrypt_verify_batch.argtypes = [vp, sz, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.pgcm_decrypt_verify_batch.restype = C.c_int
    lib.pgcm_encrypt_batch_iv.argtypes = [vp, sz, vp, C.c_uint32, vp, vp, vp, vp, vp, vp, vp]
    lib.pgcm_encrypt_batch_iv.restype = C.c_int
    lib.pgcm_decrypt_verify_batch_iv.argtypes = [vp, sz, vp, C.c_uint32, vp, vp, vp, vp, vp, vp,
                                                 vp, vp]
    lib.pgcm_decrypt_verify_batch_iv.restype = C.c_int
    lib.pgcm_encrypt_batch_keys.argtypes = [vp, sz, vp, sz, vp, C.c_uint32, vp, vp, vp, vp, vp, vp,
                                            vp]
    lib.pgcm_encrypt_batch_keys.restype = C.c_int
    lib.pgcm_decrypt_verify_batch_keys.argtypes = [vp, sz, vp, sz, vp, C.c_uint32, vp, vp, vp, vp,
                                                   vp, vp, vp, vp]
    lib.pgcm_decrypt_verify_batch_keys.restype = C.c_int
    lib.pgcm_strerror.argtypes = [C.c_int]
    lib.pgcm_strerror.restype = C.c_char_p
    lib.pgcm_last_hip_error.argtypes = []
    lib.pgcm_last_hip_error.restype = C.c_int
    lib.pgcm_plan_units.argtypes = [sz, vp, vp, vp, vp, vp, vp]
    lib.pgcm_plan_units.restype = C.c_int64
    lib.pgcm_unit_bytes.argtypes = []
    lib.pgcm_unit_bytes.restype = C.c_uint32
    lib.pgcm_batch_unit_bytes.argtypes = [sz, vp]
    lib.pgcm_batch_unit_bytes.restype = C.c_uint32
    lib.pgcm_key_tables_bytes.argtypes = []
    lib.pgcm_key_tables_bytes.restype = sz
    lib.pgcm_copy_key_tables.argtypes = [vp, vp, sz]
    lib.pgcm_copy_key_tables.restype = C.c_int
    lib.pgcm_set_unit_bytes.argtypes = [vp, C.c_uint32]
    lib.pgcm_set_unit_bytes.restype = C.c_int
    lib.pgcm_bitsliced_keystream.argtypes = [vp, vp, C.c_uint32, C.c_uint64, vp, vp]
    lib.pgcm_bitsliced_keystream.restype = C.c_int
    lib.pgcm_set_one_launch.argtypes = [vp, C.c_int]
    lib.pgcm_set_one_launch.restype = C.c_int
    lib.pgcm_set_matrix_hash.argtypes = [vp, C.c_int]
    lib.pgcm_set_matrix_hash.restype = C.c_int
    lib.pgcm_set_timing.argtypes = [vp, C.c_int]
    lib.pgcm_set_timing.restype = C.c_int
    lib.pgcm_last_bulk_kernel_ms.argtypes = [vp, C.POINTER(C.c_float)]
    lib.pgcm_last_bulk_kernel_ms.restype = C.c_int
    lib.pgcm_measure_passes.argtypes = [vp, sz, vp, C.c_uint32, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                        C.c_uint32, C.c_int, C.POINTER(C.c_double)]
    lib.pgcm_measure_passes.restype = C.c_int
    lib.pgcm_bulk_kernel_ms_history.argtypes = [vp, vp, sz]
    lib.pgcm_bulk_kernel_ms_history.restype = C.c_int64
    _lib = lib
    return lib


def _check(status):
    if status != 0:
        raise PgcmError(status, load_library().pgcm_last_hip_error() if status == -5 else 0)


def _stream_handle(stream):
    """None -> torch's current stream; an int is taken as a hipStream_t; a torch stream -> its
    handle"""
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _dev_ptr(t):
    """device address of a torch CUDA tensor, or an int taken as is; None -> NULL"""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous CUDA tensor")
    return t.data_ptr()


def _host_array(a, dtype, n, what):
    """host descriptor array: numpy array of `dtype` with n entries (None stays None)"""
    if a is None:
        return None
    arr = np.ascontiguousarray(a, dtype=dtype)
    if arr.shape != (n,):
        raise ValueError("%s must have %d entries" % (what, n))
    return arr


def _addr(arr):
    return None if arr is None else arr.ctypes.data


class Key:
    """Owns a pgcm_key_t; free() (or garbage collection) wipes and releases it."""

    def __init__(self, handle):
        self._h = handle

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("key already freed")
        return self._h

    def free(self):
        if self._h is not None:
            load_library().pgcm_free_key(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def _key_bytes(key):
    return np.frombuffer(bytes(key), dtype=np.uint8) if not isinstance(key, np.ndarray) else \
        np.ascontiguousarray(key, dtype=np.uint8)


def expand_key(key, stream=None) -> Key:
    """pgcm_expand_key: `key` is 32 bytes (bytes or uint8 array)."""
    kb = _key_bytes(key)
    if kb.size != 32:
        raise ValueError("AES-256 keys are 32 bytes")
    out = C.c_void_p()
    _check(load_library().pgcm_expand_key(kb.ctypes.data, _stream_handle(stream), C.byref(out)))
    return Key(out.value)


def expand_key_bytes(key, stream=None) -> Key:
    """pgcm_expand_key_bytes: `key` is 16, 24 or 32 bytes; the library checks the length."""
    kb = _key_bytes(key)
    out = C.c_void_p()
    _check(load_library().pgcm_expand_key_bytes(kb.ctypes.data, kb.size, _stream_handle(stream),
                                                C.byref(out)))
    return Key(out.value)


def encrypt_batch(key: Key, ivs, aad, aad_len, src, length, dst, tags, stream=None, iv_bytes=None):
    """pgcm_encrypt_batch, or pgcm_encrypt_batch_iv when iv_bytes is given.  ivs, tags: CUDA uint8
    tensors (n*12 or n*iv_bytes, n*16 bytes) or device addresses; src, dst, aad: sequences / uint64
    arrays of n device addresses; length: n byte counts; aad and aad_len are both None when no
    chunk has AAD."""
    n = len(length)
    src_a = _host_array(src, np.uint64, n, "src")
    dst_a = _host_array(dst, np.uint64, n, "dst")
    len_a = _host_array(length, np.uint64, n, "length")
    aad_a = _host_array(aad, np.uint64, n, "aad")
    alen_a = _host_array(aad_len, np.uint32, n, "aad_len")
    if iv_bytes is not None:
        _check(load_library().pgcm_encrypt_batch_iv(
            key.handle, n, _dev_ptr(ivs), iv_bytes, _addr(aad_a), _addr(alen_a), _addr(src_a),
            _addr(len_a), _addr(dst_a), _dev_ptr(tags), _stream_handle(stream)))
        return
    _check(load_library().pgcm_encrypt_batch(
        key.handle, n, _dev_ptr(ivs), _addr(aad_a), _addr(alen_a), _addr(src_a), _addr(len_a),
        _addr(dst_a), _dev_ptr(tags), _stream_handle(stream)))


STATIC_WORKSPACE_BYTES = 8 << 20   # PGCM_STATIC_WORKSPACE_BYTES
STATIC_MAX_CHUNKS = 1024           # PGCM_STATIC_MAX_CHUNKS


def encrypt_batch_static(key: Key, ivs, aad, aad_len, src, length, dst, tags, stream=None):
    """pgcm_encrypt_batch_static: pgcm_encrypt_batch that allocates nothing; arguments as for
    encrypt_batch.  (The arrays this wrapper builds are the caller's side of the call.)"""
    n = len(length)
    src_a = _host_array(src, np.uint64, n, "src")
    dst_a = _host_array(dst, np.uint64, n, "dst")
    len_a = _host_array(length, np.uint64, n, "length")
    aad_a = _host_array(aad, np.uint64, n, "aad")
    alen_a = _host_array(aad_len, np.uint32, n, "aad_len")
    _check(load_library().pgcm_encrypt_batch_static(
        key.handle, n, _dev_ptr(ivs), _addr(aad_a), _addr(alen_a), _addr(src_a), _addr(len_a),
        _addr(dst_a), _dev_ptr(tags), _stream_handle(stream)))


def reserve(key: Key, n_max: int, payload_bytes_max: int, stream=None):
    """pgcm_reserve"""
    _check(load_library().pgcm_reserve(key.handle, _stream_handle(stream), n_max,
                                       payload_bytes_max))


class _ScheduleInfo(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("desc_offset", "unit_base_offset", "coarse_map_offset",
                                          "fold_items_offset", "image_bytes", "workspace_bytes")] + \
               [(n, C.c_uint32) for n in ("unit_power", "nunits", "nslots", "ncoarse", "nfold")] + \
               [("fold_count", C.c_uint32 * 4), ("fold_first", C.c_uint32 * 4),
                ("path", C.c_uint32)]


CHUNK_DESC_DTYPE = np.dtype([("src", "<u8"), ("dst", "<u8"), ("aad", "<u8"), ("len", "<u8"),
                             ("aad_len", "<u4"), ("unit_base", "<u4"), ("nunits", "<u4"),
                             ("first_blocks", "<u4"), ("final_base", "<u4"),
                             ("final_count", "<u4"), ("final_power", "<u4"), ("index", "<u4")])
FOLD_ITEM_DTYPE = np.dtype([("in_base", "<u4"), ("in_count", "<u4"), ("out_slot", "<u4"),
                            ("pad", "<u4")])


def describe_schedule(length, unit_bytes=0, wave_slots=0) -> dict:
    """pgcm_describe_schedule, taken apart; host only.  -> dict with the info fields and the
    arrays `desc` (CHUNK_DESC_DTYPE), `unit_base`, `coarse_map`, `fold_items` (FOLD_ITEM_DTYPE)."""
    len_a = np.ascontiguousarray(length, dtype=np.uint64)
    n = len_a.size
    info = _ScheduleInfo()
    lib = load_library()
    _check(lib.pgcm_describe_schedule(n, _addr(len_a) if n else None, unit_bytes, wave_slots,
                                      C.addressof(info), None, 0))
    image = np.zeros(max(1, int(info.image_bytes)), np.uint8)
    _check(lib.pgcm_describe_schedule(n, _addr(len_a) if n else None, unit_bytes, wave_slots,
                                      C.addressof(info), image.ctypes.data, image.size))
    out = {k: int(getattr(info, k)) for k, _ in _ScheduleInfo._fields_
           if k not in ("fold_count", "fold_first")}
    out["fold_count"] = [int(v) for v in info.fold_count]
    out["fold_first"] = [int(v) for v in info.fold_first]
    out["desc"] = image[out["desc_offset"]:out["desc_offset"] + 64 * n].view(CHUNK_DESC_DTYPE)
    ub = out["unit_base_offset"]
    out["unit_base"] = image[ub:ub + 4 * (n + 1)].view(np.uint32) if n else np.zeros(1, np.uint32)
    cm = out["coarse_map_offset"]
    out["coarse_map"] = image[cm:cm + 4 * out["ncoarse"]].view(np.uint32)
    fi = out["fold_items_offset"]
    out["fold_items"] = image[fi:fi + 16 * out["nfold"]].view(FOLD_ITEM_DTYPE)
    return out


def decrypt_verify_batch(key: Key, ivs, aad, aad_len, src, length, dst, tags, ok, stream=None,
                         iv_bytes=None):
    """pgcm_decrypt_verify_batch (pgcm_decrypt_verify_batch_iv when iv_bytes is given).  As
    encrypt_batch; tags is read, ok (CUDA uint8 tensor of n
    bytes) receives 1 per authentic chunk and 0 per rejected one."""
    n = len(length)
    src_a = _host_array(src, np.uint64, n, "src")
    dst_a = _host_array(dst, np.uint64, n, "dst")
    len_a = _host_array(length, np.uint64, n, "length")
    aad_a = _host_array(aad, np.uint64, n, "aad")
    alen_a = _host_array(aad_len, np.uint32, n, "aad_len")
    if iv_bytes is not None:
        _check(load_library().pgcm_decrypt_verify_batch_iv(
            key.handle, n, _dev_ptr(ivs), iv_bytes, _addr(aad_a), _addr(alen_a), _addr(src_a),
            _addr(len_a), _addr(dst_a), _dev_ptr(tags), _dev_ptr(ok), _stream_handle(stream)))
        return
    _check(load_library().pgcm_decrypt_verify_batch(
        key.handle, n, _dev_ptr(ivs), _addr(aad_a), _addr(alen_a), _addr(src_a), _addr(len_a),
        _addr(dst_a), _dev_ptr(tags), _dev_ptr(ok), _stream_handle(stream)))


def _key_handles(keys):
    return np.array([k.handle for k in keys], np.uint64)


def encrypt_batch_keys(keys, key_index, ivs, iv_bytes, aad, aad_len, src, length, dst, tags,
                       stream=None):
    """pgcm_encrypt_batch_keys: keys is a sequence of Key objects, key_index n indices into it."""
    n = len(length)
    handles = _key_handles(keys)
    idx_a = _host_array(key_index, np.uint32, n, "key_index")
    src_a = _host_array(src, np.uint64, n, "src")
    dst_a = _host_array(dst, np.uint64, n, "dst")
    len_a = _host_array(length, np.uint64, n, "length")
    aad_a = _host_array(aad, np.uint64, n, "aad")
    alen_a = _host_array(aad_len, np.uint32, n, "aad_len")
    _check(load_library().pgcm_encrypt_batch_keys(
        _addr(handles) if handles.size else None, handles.size, _addr(idx_a), n, _dev_ptr(ivs),
        iv_bytes, _addr(aad_a), _addr(alen_a), _addr(src_a), _addr(len_a), _addr(dst_a),
        _dev_ptr(tags), _stream_handle(stream)))


def decrypt_verify_batch_keys(keys, key_index, ivs, iv_bytes, aad, aad_len, src, length, dst, tags,
                              ok, stream=None):
    """pgcm_decrypt_verify_batch_keys"""
    n = len(length)
    handles = _key_handles(keys)
    idx_a = _host_array(key_index, np.uint32, n, "key_index")
    src_a = _host_array(src, np.uint64, n, "src")
    dst_a = _host_array(dst, np.uint64, n, "dst")
    len_a = _host_array(length, np.uint64, n, "length")
    aad_a = _host_array(aad, np.uint64, n, "aad")
    alen_a = _host_array(aad_len, np.uint32, n, "aad_len")
    _check(load_library().pgcm_decrypt_verify_batch_keys(
        _addr(handles) if handles.size else None, handles.size, _addr(idx_a), n, _dev_ptr(ivs),
        iv_bytes, _addr(aad_a), _addr(alen_a), _addr(src_a), _addr(len_a), _addr(dst_a),
        _dev_ptr(tags), _dev_ptr(ok), _stream_handle(stream)))


def plan_units(length):
    """pgcm_plan_units -> dict(total, nunits, first_blocks, unit_base, final_count, final_power);
    host only."""
    len_a = np.ascontiguousarray(length, dtype=np.uint64)
    n = len_a.size
    out = {k: np.zeros(n, np.uint32) for k in ("nunits", "first_blocks", "unit_base",
                                                "final_count", "final_power")}
    total = load_library().pgcm_plan_units(n, _addr(len_a) if n else None,
                                           *[out[k].ctypes.data for k in
                                             ("nunits", "first_blocks", "unit_base", "final_count",
                                              "final_power")])
    if total < 0:
        raise PgcmError(int(total))
    out["total"] = int(total)
    return out


def copy_key_tables(key: Key) -> dict:
    """pgcm_copy_key_tables, taken apart: rk (60 uint32), rounds, te (4, 256) uint32, h (16 uint8),
    ghash (31, 512, 16) uint8, row_matrix (4, 2, 64, 4) uint32: [product tile][depth slice][lane]
    [register] of the matrix-core operands of the multiplication by H^64, ghash_lane (3, 512, 16)
    uint8: nibble tables of H^3, H^12, H^48"""
    n = int(load_library().pgcm_key_tables_bytes())
    raw = np.zeros(n, np.uint8)
    _check(load_library().pgcm_copy_key_tables(key.handle, raw.ctypes.data, n))
    words = raw[:256].view(np.uint32)
    out = {"rk": words[:60].copy(), "rounds": int(words[60]),
           "te": raw[256:256 + 4096].view(np.uint32).reshape(4, 256).copy(),
           "h": raw[4352:4368].copy(),
           "ghash": raw[4368:4368 + 31 * 8192].reshape(31, 512, 16).copy(),
           "row_matrix": raw[4368 + 31 * 8192:4368 + 32 * 8192].view(np.uint32)
                         .reshape(4, 2, 64, 4).copy(),
           "ghash_lane": raw[4368 + 32 * 8192:].reshape(3, 512, 16).copy()}
    raw[:] = 0
    return out


def set_unit_bytes(key: Key, unit_bytes: int):
    """pgcm_set_unit_bytes (0: chosen per batch)"""
    _check(load_library().pgcm_set_unit_bytes(key.handle, unit_bytes))


def bitsliced_keystream(key: Key, iv, ctr_base: int, nblocks: int, out, stream=None):
    """pgcm_bitsliced_keystream: iv is 12 bytes (host), out a CUDA uint8 tensor of 16 * nblocks
    bytes or a device address"""
    v = np.frombuffer(bytes(iv), dtype=np.uint8)
    if v.size != 12:
        raise ValueError("IVs are 12 bytes")
    _check(load_library().pgcm_bitsliced_keystream(key.handle, v.ctypes.data, ctr_base, nblocks,
                                                   _dev_ptr(out), _stream_handle(stream)))


def set_matrix_hash(key: Key, enable: bool):
    """pgcm_set_matrix_hash"""
    _check(load_library().pgcm_set_matrix_hash(key.handle, 1 if enable else 0))


def set_one_launch(key: Key, enable: bool):
    """pgcm_set_one_launch"""
    _check(load_library().pgcm_set_one_launch(key.handle, 1 if enable else 0))


def set_timing(key: Key, enable: bool):
    """pgcm_set_timing"""
    _check(load_library().pgcm_set_timing(key.handle, 1 if enable else 0))


def last_bulk_kernel_ms(key: Key) -> float:
    """pgcm_last_bulk_kernel_ms"""
    ms = C.c_float(0.0)
    _check(load_library().pgcm_last_bulk_kernel_ms(key.handle, C.byref(ms)))
    return float(ms.value)


def bulk_kernel_ms_history(key: Key, max_launches: int = 256):
    """pgcm_bulk_kernel_ms_history -> list of durations in ms, oldest first"""
    out = np.zeros(max(1, max_launches), np.float32)
    n = load_library().pgcm_bulk_kernel_ms_history(key.handle, out.ctypes.data, max_launches)
    if n < 0:
        raise PgcmError(int(n), load_library().pgcm_last_hip_error() if n == -5 else 0)
    return [float(v) for v in out[:n]]


def measure_passes(key: Key, ivs, aad, aad_len, src, length, cipher, back, tags, ok, steps,
                   direction=0, stream=None, iv_bytes=12) -> float:
    """pgcm_measure_passes -> host milliseconds for `steps` passes (direction 0: encrypt then
    decrypt-verify, 1: encrypt only, 2: decrypt-verify only)"""
    n = len(length)
    src_a = _host_array(src, np.uint64, n, "src")
    ct_a = _host_array(cipher, np.uint64, n, "cipher")
    back_a = _host_array(back, np.uint64, n, "back")
    len_a = _host_array(length, np.uint64, n, "length")
    aad_a = _host_array(aad, np.uint64, n, "aad")
    alen_a = _host_array(aad_len, np.uint32, n, "aad_len")
    ms = C.c_double(0.0)
    _check(load_library().pgcm_measure_passes(
        key.handle, n, _dev_ptr(ivs), iv_bytes, _addr(aad_a), _addr(alen_a), _addr(src_a),
        _addr(len_a), _addr(ct_a), _addr(back_a), _dev_ptr(tags), _dev_ptr(ok), _stream_handle(stream), steps,
        direction, C.byref(ms)))
    return float(ms.value)


def unit_bytes() -> int:
    return int(load_library().pgcm_unit_bytes())


def batch_unit_bytes(length) -> int:
    """pgcm_batch_unit_bytes; host only."""
    len_a = np.ascontiguousarray(length, dtype=np.uint64)
    return int(load_library().pgcm_batch_unit_bytes(len_a.size, _addr(len_a) if len_a.size else None))


# ---------------------------------------------------------------------------------------------
# include/pgcm_seq.h: the speculative-pipeline state machine (host only)

SEQ_EXPORTS = ("pgcm_seq_create", "pgcm_seq_destroy", "pgcm_seq_swap_out", "pgcm_seq_notify_write",
               "pgcm_seq_request", "pgcm_seq_sync", "pgcm_seq_take_actions", "pgcm_seq_current_iv",
               "pgcm_seq_iv_bytes")
SEQ_KINDS = {1: "pre", 2: "send", 3: "now", 4: "nop", 5: "drop"}


class _SeqAction(C.Structure):
    _fields_ = [("kind", C.c_uint32), ("reserved", C.c_uint32), ("addr", C.c_uint64),
                ("len", C.c_uint64), ("iv", C.c_uint64)]


def _seq_lib(lib=None):
    """declares the pgcm_seq_* entry points on the library (or on another build of the host-only
    sequencer handed in as a ctypes.CDLL)"""
    lib = load_library() if lib is None else lib
    if not getattr(lib, "_seq_bound", False):
        vp = C.c_void_p
        lib.pgcm_seq_create.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64, C.c_uint32,
                                        C.POINTER(vp)]
        lib.pgcm_seq_create.restype = C.c_int
        lib.pgcm_seq_destroy.argtypes = [vp]
        lib.pgcm_seq_destroy.restype = None
        for name in ("pgcm_seq_swap_out", "pgcm_seq_notify_write", "pgcm_seq_request"):
            getattr(lib, name).argtypes = [vp, C.c_uint64, C.c_uint64]
            getattr(lib, name).restype = C.c_int
        lib.pgcm_seq_sync.argtypes = [vp]
        lib.pgcm_seq_sync.restype = C.c_int
        lib.pgcm_seq_take_actions.argtypes = [vp, C.POINTER(_SeqAction), C.c_size_t]
        lib.pgcm_seq_take_actions.restype = C.c_size_t
        lib.pgcm_seq_current_iv.argtypes = [vp]
        lib.pgcm_seq_current_iv.restype = C.c_uint64
        lib.pgcm_seq_iv_bytes.argtypes = [vp, C.c_uint64, vp]
        lib.pgcm_seq_iv_bytes.restype = None
        lib._seq_bound = True
    return lib


class Sequencer:
    """pgcm_seq_t: events in, actions out (tuples (kind, (addr, len), iv); NOPs are (kind, iv))"""

    def __init__(self, iv_start=0, depth=4, leeway=0, threshold=128 * 1024, history_limit=512,
                 lib=None):
        self._h = None
        self._lib = _seq_lib(lib)
        h = C.c_void_p()
        _check(self._lib.pgcm_seq_create(iv_start, depth, leeway, threshold, history_limit,
                                         C.byref(h)))
        self._h = h.value

    def close(self):
        if self._h is not None:
            self._lib.pgcm_seq_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def swap_out(self, chunk):
        _check(self._lib.pgcm_seq_swap_out(self._h, chunk[0], chunk[1]))

    def notify_write(self, chunk):
        _check(self._lib.pgcm_seq_notify_write(self._h, chunk[0], chunk[1]))

    def request(self, chunk):
        _check(self._lib.pgcm_seq_request(self._h, chunk[0], chunk[1]))

    def sync(self):
        _check(self._lib.pgcm_seq_sync(self._h))

    @property
    def iv_cur(self):
        return int(self._lib.pgcm_seq_current_iv(self._h))

    def take_actions(self):
        out = []
        buf = (_SeqAction * 64)()
        while True:
            n = self._lib.pgcm_seq_take_actions(self._h, buf, 64)
            for a in buf[:n]:
                kind = SEQ_KINDS[a.kind]
                out.append((kind, a.iv) if kind == "nop" else (kind, (a.addr, a.len), a.iv))
            if n < 64:
                return out


def seq_iv_bytes(iv0, n) -> bytes:
    """pgcm_seq_iv_bytes: iv0 + n as 12 big-endian bytes"""
    a = np.frombuffer(bytes(iv0), dtype=np.uint8).copy()
    if a.size != 12:
        raise ValueError("IVs are 12 bytes")
    out = np.zeros(12, np.uint8)
    _seq_lib().pgcm_seq_iv_bytes(a.ctypes.data, n, out.ctypes.data)
    return out.tobytes()


# ---------------------------------------------------------------------------------------------
# include/pgcm_bounce.h: the pool of pinned bounce buffers
BOUNCE_EXPORTS = ("pgcm_bounce_create", "pgcm_bounce_destroy", "pgcm_bounce_acquire",
                  "pgcm_bounce_release", "pgcm_bounce_buffer_bytes", "pgcm_bounce_count")


def _bounce_lib():
    lib = load_library()
    if not getattr(lib, "_bounce_bound", False):
        vp = C.c_void_p
        lib.pgcm_bounce_create.argtypes = [C.c_size_t, C.c_uint32, C.POINTER(vp)]
        lib.pgcm_bounce_create.restype = C.c_int
        lib.pgcm_bounce_destroy.argtypes = [vp]
        lib.pgcm_bounce_destroy.restype = None
        lib.pgcm_bounce_acquire.argtypes = [vp, C.POINTER(vp), C.POINTER(C.c_uint32)]
        lib.pgcm_bounce_acquire.restype = C.c_int
        lib.pgcm_bounce_release.argtypes = [vp, C.c_uint32, vp]
        lib.pgcm_bounce_release.restype = C.c_int
        lib.pgcm_bounce_buffer_bytes.argtypes = [vp]
        lib.pgcm_bounce_buffer_bytes.restype = C.c_size_t
        lib.pgcm_bounce_count.argtypes = [vp]
        lib.pgcm_bounce_count.restype = C.c_uint32
        lib._bounce_bound = True
    return lib


class BouncePool:
    """Owns a pgcm_bounce_t.  acquire() -> (address, slot); release(slot, stream)."""

    def __init__(self, buffer_bytes: int, count: int):
        self._h = None
        out = C.c_void_p()
        _check(_bounce_lib().pgcm_bounce_create(buffer_bytes, count, C.byref(out)))
        self._h = out.value

    @property
    def buffer_bytes(self) -> int:
        return int(_bounce_lib().pgcm_bounce_buffer_bytes(self._h))

    @property
    def count(self) -> int:
        return int(_bounce_lib().pgcm_bounce_count(self._h))

    def acquire(self):
        buf, slot = C.c_void_p(), C.c_uint32()
        _check(_bounce_lib().pgcm_bounce_acquire(self._h, C.byref(buf), C.byref(slot)))
        return int(buf.value), int(slot.value)

    def release(self, slot: int, stream=None):
        _check(_bounce_lib().pgcm_bounce_release(self._h, slot, _stream_handle(stream)))

    def view(self, address: int, nbytes: int) -> np.ndarray:
        """host view of nbytes at an address inside the pool (no copy)"""
        return np.ctypeslib.as_array((C.c_uint8 * nbytes).from_address(address))

    def destroy(self):
        if self._h is not None:
            _bounce_lib().pgcm_bounce_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


# ---------------------------------------------------------------------------------------------
# include/pgcm_pipe.h: the pipeline driver
PIPE_EXPORTS = ("pgcm_pipe_create", "pgcm_pipe_destroy", "pgcm_pipe_swap_out",
                "pgcm_pipe_notify_write", "pgcm_pipe_request", "pgcm_pipe_sync",
                "pgcm_pipe_get_stats", "pgcm_recv_create", "pgcm_recv_destroy", "pgcm_recv_accept",
                "pgcm_recv_next_iv")


class _PipeConfig(C.Structure):
    _fields_ = [("iv0", C.c_uint8 * 12), ("depth", C.c_uint32), ("iv_start", C.c_uint64),
                ("leeway", C.c_uint32), ("history_limit", C.c_uint32),
                ("swap_threshold", C.c_uint64), ("max_chunk_bytes", C.c_uint64)]


class _PipeStats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("transfers", "nops", "ahead_bytes", "critical_bytes",
                                          "pre_bytes", "dropped_bytes")]


_DELIVER_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_uint32, C.c_uint64, C.c_uint64, C.c_uint64,
                          C.c_void_p, C.c_void_p, C.c_void_p)


def _pipe_lib():
    lib = load_library()
    if not getattr(lib, "_pipe_bound", False):
        vp = C.c_void_p
        lib.pgcm_pipe_create.argtypes = [vp, C.POINTER(_PipeConfig), _DELIVER_FN, vp, C.POINTER(vp)]
        lib.pgcm_pipe_create.restype = C.c_int
        lib.pgcm_pipe_destroy.argtypes = [vp]
        lib.pgcm_pipe_destroy.restype = None
        for name in ("pgcm_pipe_swap_out", "pgcm_pipe_notify_write", "pgcm_pipe_request"):
            getattr(lib, name).argtypes = [vp, vp, C.c_uint64, vp]
            getattr(lib, name).restype = C.c_int
        lib.pgcm_pipe_sync.argtypes = [vp, vp]
        lib.pgcm_pipe_sync.restype = C.c_int
        lib.pgcm_pipe_get_stats.argtypes = [vp, C.POINTER(_PipeStats)]
        lib.pgcm_pipe_get_stats.restype = C.c_int
        lib.pgcm_recv_create.argtypes = [vp, vp, C.c_uint64, C.POINTER(vp)]
        lib.pgcm_recv_create.restype = C.c_int
        lib.pgcm_recv_destroy.argtypes = [vp]
        lib.pgcm_recv_destroy.restype = None
        lib.pgcm_recv_accept.argtypes = [vp, vp, C.c_uint64, vp, vp, vp, vp]
        lib.pgcm_recv_accept.restype = C.c_int
        lib.pgcm_recv_next_iv.argtypes = [vp]
        lib.pgcm_recv_next_iv.restype = C.c_uint64
        lib._pipe_bound = True
    return lib


class Pipe:
    """Owns a pgcm_pipe_t.  deliver(kind, addr, length, iv, ciphertext_address, tag_address,
    stream_handle) is called once per transfer, in wire order; kind is "send", "now" or "nop"."""

    def __init__(self, key: Key, iv0: bytes, deliver, depth=4, iv_start=0, leeway=0,
                 history_limit=512, swap_threshold=128 * 1024, max_chunk_bytes=8 << 20):
        self._h = None
        self._key = key                      # keeps the key alive as long as the pipe

        def _trampoline(_user, kind, addr, length, iv, ct, tag, stream):
            deliver(SEQ_KINDS[kind], addr, length, iv, ct, tag, stream or 0)

        self._cb = _DELIVER_FN(_trampoline)  # must outlive the pipe
        cfg = _PipeConfig()
        iv0 = bytes(iv0)
        if len(iv0) != 12:
            raise ValueError("iv0 is 12 bytes")
        for i in range(12):
            cfg.iv0[i] = iv0[i]
        cfg.depth, cfg.iv_start, cfg.leeway = depth, iv_start, leeway
        cfg.history_limit, cfg.swap_threshold = history_limit, swap_threshold
        cfg.max_chunk_bytes = max_chunk_bytes
        out = C.c_void_p()
        _check(_pipe_lib().pgcm_pipe_create(key.handle, C.byref(cfg), self._cb, None,
                                            C.byref(out)))
        self._h = out.value

    def swap_out(self, addr: int, length: int, stream=None):
        _check(_pipe_lib().pgcm_pipe_swap_out(self._h, addr, length, _stream_handle(stream)))

    def notify_write(self, addr: int, length: int, stream=None):
        _check(_pipe_lib().pgcm_pipe_notify_write(self._h, addr, length, _stream_handle(stream)))

    def request(self, addr: int, length: int, stream=None):
        _check(_pipe_lib().pgcm_pipe_request(self._h, addr, length, _stream_handle(stream)))

    def sync(self, stream=None):
        _check(_pipe_lib().pgcm_pipe_sync(self._h, _stream_handle(stream)))

    def stats(self) -> dict:
        st = _PipeStats()
        _check(_pipe_lib().pgcm_pipe_get_stats(self._h, C.byref(st)))
        return {n: int(getattr(st, n)) for n, _ in _PipeStats._fields_}

    def destroy(self):
        if self._h is not None:
            _pipe_lib().pgcm_pipe_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class Receiver:
    """Owns a pgcm_recv_t: the peer that accepts transfer k under IV_0 + k only."""

    def __init__(self, key: Key, iv0: bytes, iv_start=0):
        self._h = None
        self._key = key
        iv0 = bytes(iv0)
        if len(iv0) != 12:
            raise ValueError("iv0 is 12 bytes")
        buf = (C.c_uint8 * 12)(*iv0)
        out = C.c_void_p()
        _check(_pipe_lib().pgcm_recv_create(key.handle, buf, iv_start, C.byref(out)))
        self._h = out.value

    def accept(self, ciphertext, length, tag, dst, ok, stream=None):
        """ciphertext, tag: device addresses (or CUDA tensors); dst, ok: CUDA tensors"""
        _check(_pipe_lib().pgcm_recv_accept(self._h, _dev_ptr(ciphertext), length, _dev_ptr(tag),
                                            _dev_ptr(dst), _dev_ptr(ok), _stream_handle(stream)))

    @property
    def next_iv(self) -> int:
        return int(_pipe_lib().pgcm_recv_next_iv(self._h))

    def destroy(self):
        if self._h is not None:
            _pipe_lib().pgcm_recv_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
