"""AES-GCM (128-, 192-, 256-bit keys, any IV length) from the host's libcrypto (EVP interface) through ctypes.

An implementation independent of both the oracle and the GPU library, used by tests as a
second opinion.  The paper's own CPU side calls this same library (section 6).
"""
import ctypes as C
import ctypes.util

_name = ctypes.util.find_library("crypto")
if _name is None:
    raise ImportError("libcrypto not found")
_lc = C.CDLL(_name)

_lc.EVP_CIPHER_CTX_new.restype = C.c_void_p
_lc.EVP_CIPHER_CTX_free.argtypes = [C.c_void_p]
for _bits in (128, 192, 256):
    getattr(_lc, "EVP_aes_%d_gcm" % _bits).restype = C.c_void_p
    getattr(_lc, "EVP_aes_%d_ecb" % _bits).restype = C.c_void_p
for _f in ("EVP_EncryptInit_ex", "EVP_DecryptInit_ex"):
    getattr(_lc, _f).argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_char_p, C.c_char_p]
for _f in ("EVP_EncryptUpdate", "EVP_DecryptUpdate"):
    getattr(_lc, _f).argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int), C.c_void_p, C.c_int]
for _f in ("EVP_EncryptFinal_ex", "EVP_DecryptFinal_ex"):
    getattr(_lc, _f).argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int)]
_lc.EVP_CIPHER_CTX_ctrl.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p]
_lc.EVP_CIPHER_CTX_set_padding.argtypes = [C.c_void_p, C.c_int]

_SET_IVLEN, _GET_TAG, _SET_TAG = 0x9, 0x10, 0x11
_STEP = 1 << 30  # EVP lengths are ints


def _cipher(key, mode):
    return getattr(_lc, "EVP_aes_%d_%s" % (8 * len(key), mode))()


def _check(rc, what):
    if rc != 1:
        raise RuntimeError("libcrypto: %s failed" % what)


def _update(fn, ctx, out_addr, data):
    """feeds `data` (bytes-like) in pieces; out_addr None means AAD"""
    n = C.c_int(0)
    mv = memoryview(data).cast("B")
    total = 0
    for off in range(0, len(mv), _STEP):
        piece = bytes(mv[off:off + _STEP]) if not isinstance(data, bytes) else data[off:off + _STEP]
        dst = None if out_addr is None else out_addr + off
        _check(fn(ctx, dst, C.byref(n), piece, len(piece)), "update")
        total += n.value
    return total


def encrypt(key: bytes, iv: bytes, aad: bytes, pt: bytes):
    ctx = _lc.EVP_CIPHER_CTX_new()
    try:
        _check(_lc.EVP_EncryptInit_ex(ctx, _cipher(key, "gcm"), None, None, None), "init")
        _check(_lc.EVP_CIPHER_CTX_ctrl(ctx, _SET_IVLEN, len(iv), None), "ivlen")
        _check(_lc.EVP_EncryptInit_ex(ctx, None, None, bytes(key), bytes(iv)), "key")
        if len(aad):
            _update(_lc.EVP_EncryptUpdate, ctx, None, bytes(aad))
        out = C.create_string_buffer(max(len(pt), 1))
        if len(pt):
            _update(_lc.EVP_EncryptUpdate, ctx, C.addressof(out), bytes(pt))
        n = C.c_int(0)
        fin = C.create_string_buffer(16)
        _check(_lc.EVP_EncryptFinal_ex(ctx, fin, C.byref(n)), "final")
        tag = C.create_string_buffer(16)
        _check(_lc.EVP_CIPHER_CTX_ctrl(ctx, _GET_TAG, 16, tag), "get tag")
        return out.raw[:len(pt)], tag.raw
    finally:
        _lc.EVP_CIPHER_CTX_free(ctx)


def decrypt_verify(key: bytes, iv: bytes, aad: bytes, ct: bytes, tag: bytes):
    """-> (ok, plaintext or None)"""
    ctx = _lc.EVP_CIPHER_CTX_new()
    try:
        _check(_lc.EVP_DecryptInit_ex(ctx, _cipher(key, "gcm"), None, None, None), "init")
        _check(_lc.EVP_CIPHER_CTX_ctrl(ctx, _SET_IVLEN, len(iv), None), "ivlen")
        _check(_lc.EVP_DecryptInit_ex(ctx, None, None, bytes(key), bytes(iv)), "key")
        if len(aad):
            _update(_lc.EVP_DecryptUpdate, ctx, None, bytes(aad))
        out = C.create_string_buffer(max(len(ct), 1))
        if len(ct):
            _update(_lc.EVP_DecryptUpdate, ctx, C.addressof(out), bytes(ct))
        t = C.create_string_buffer(bytes(tag), 16)
        _check(_lc.EVP_CIPHER_CTX_ctrl(ctx, _SET_TAG, 16, t), "set tag")
        n = C.c_int(0)
        fin = C.create_string_buffer(16)
        ok = _lc.EVP_DecryptFinal_ex(ctx, fin, C.byref(n)) == 1
        return ok, (out.raw[:len(ct)] if ok else None)
    finally:
        _lc.EVP_CIPHER_CTX_free(ctx)


def aes_ecb_block(key: bytes, block: bytes) -> bytes:
    ctx = _lc.EVP_CIPHER_CTX_new()
    try:
        _check(_lc.EVP_EncryptInit_ex(ctx, _cipher(key, "ecb"), None, bytes(key), None), "init")
        _lc.EVP_CIPHER_CTX_set_padding(ctx, 0)
        out = C.create_string_buffer(32)
        n = C.c_int(0)
        _check(_lc.EVP_EncryptUpdate(ctx, out, C.byref(n), bytes(block), 16), "update")
        return out.raw[:16]
    finally:
        _lc.EVP_CIPHER_CTX_free(ctx)


aes256_ecb_block = aes_ecb_block


class GcmEncryptStream:
    """libcrypto's GCM encryption fed piece by piece (for messages too long to hold twice in host
    memory): update(numpy uint8 array) -> ciphertext array of the same length; tag() at the end"""

    def __init__(self, key: bytes, iv: bytes, aad: bytes = b""):
        self._ctx = _lc.EVP_CIPHER_CTX_new()
        _check(_lc.EVP_EncryptInit_ex(self._ctx, _cipher(key, "gcm"), None, None, None), "init")
        _check(_lc.EVP_CIPHER_CTX_ctrl(self._ctx, _SET_IVLEN, len(iv), None), "ivlen")
        _check(_lc.EVP_EncryptInit_ex(self._ctx, None, None, bytes(key), bytes(iv)), "key")
        if len(aad):
            _update(_lc.EVP_EncryptUpdate, self._ctx, None, bytes(aad))

    def update(self, piece, out=None):
        import numpy as np
        assert piece.dtype == np.uint8 and piece.flags["C_CONTIGUOUS"]
        if out is None:
            out = np.empty(piece.size, np.uint8)
        n = C.c_int(0)
        for off in range(0, piece.size, _STEP):
            m = min(_STEP, piece.size - off)
            _check(_lc.EVP_EncryptUpdate(self._ctx, C.c_void_p(out.ctypes.data + off), C.byref(n),
                                         C.c_void_p(piece.ctypes.data + off), m), "update")
            assert n.value == m
        return out[:piece.size]

    def tag(self) -> bytes:
        n = C.c_int(0)
        fin = C.create_string_buffer(16)
        _check(_lc.EVP_EncryptFinal_ex(self._ctx, fin, C.byref(n)), "final")
        t = C.create_string_buffer(16)
        _check(_lc.EVP_CIPHER_CTX_ctrl(self._ctx, _GET_TAG, 16, t), "get tag")
        _lc.EVP_CIPHER_CTX_free(self._ctx)
        self._ctx = None
        return t.raw
