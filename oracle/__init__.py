"""ctypes face of the C oracle in gcm_oracle.c: test infrastructure, not product code.

A plain CPU AES-GCM written from FIPS-197 and NIST SP 800-38D (the key length follows from
len(key): 16, 24 or 32 bytes; the IV length from len(iv)), standing for what the paper's
transport, AES-256 with 96-bit IVs, computes per transfer (section 2.2, "A closer look at NVIDIA CC"; section 4.1,
"Swapping sequence and IVs").  Only tests, the smoke check and the benchmark's CPU-baseline leg
may import this module; it shares nothing with the GPU library and never imports it.
"""
import ctypes as C

import numpy as np

from . import build as _build

def _bind(lib):
    """declares the argument types of the oracle's C entry points on a loaded library"""
    lib.orc_sbox.argtypes = [C.c_void_p]
    lib.orc_aes256_key_expand.argtypes = [C.c_void_p, C.c_void_p]
    lib.orc_aes256_encrypt_block.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    lib.orc_aes_key_expand.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
    lib.orc_aes_key_expand.restype = C.c_int
    lib.orc_aes_encrypt_block.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
    lib.orc_gf128_mul.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    lib.orc_ghash_update.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.orc_gctr.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
    one = [C.c_void_p, C.c_int, C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64, C.c_void_p,
           C.c_uint64, C.c_void_p, C.c_void_p]
    lib.orc_gcm_encrypt_ex.argtypes = one
    lib.orc_gcm_encrypt_ex.restype = C.c_int
    lib.orc_gcm_decrypt_verify_ex.argtypes = one
    lib.orc_gcm_decrypt_verify_ex.restype = C.c_int
    common = [C.c_void_p, C.c_int, C.c_uint64, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p,
              C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.orc_gcm_encrypt_batch_ex.argtypes = common + [C.c_int]
    lib.orc_gcm_encrypt_batch_ex.restype = C.c_int
    lib.orc_gcm_decrypt_verify_batch_ex.argtypes = common + [C.c_void_p, C.c_int]
    lib.orc_gcm_decrypt_verify_batch_ex.restype = C.c_int
    return lib


_lib = _bind(C.CDLL(_build.build()))


def _in(b, n=None):
    a = np.frombuffer(bytes(b), dtype=np.uint8) if not isinstance(b, np.ndarray) else \
        np.ascontiguousarray(b, dtype=np.uint8)
    if n is not None and a.size != n:
        raise ValueError("expected %d bytes, got %d" % (n, a.size))
    return a


def _ptr(a):
    return a.ctypes.data if a.size else None


def sbox() -> bytes:
    out = np.zeros(256, np.uint8)
    _lib.orc_sbox(out.ctypes.data)
    return out.tobytes()


def aes256_key_expand(key) -> bytes:
    k = _in(key, 32)
    rk = np.zeros(240, np.uint8)
    _lib.orc_aes256_key_expand(k.ctypes.data, rk.ctypes.data)
    return rk.tobytes()


def aes256_encrypt_block(key, block) -> bytes:
    rk = _in(aes256_key_expand(key))
    b = _in(block, 16)
    out = np.zeros(16, np.uint8)
    _lib.orc_aes256_encrypt_block(rk.ctypes.data, b.ctypes.data, out.ctypes.data)
    return out.tobytes()


def _key(key):
    k = _in(key)
    if k.size not in (16, 24, 32):
        raise ValueError("AES keys are 16, 24 or 32 bytes")
    return k


def aes_key_expand(key) -> bytes:
    """round keys 0..Nr, 16 bytes each (Nr = 10, 12, 14 for 16-, 24-, 32-byte keys)"""
    k = _key(key)
    rk = np.zeros(240, np.uint8)
    nr = _lib.orc_aes_key_expand(k.ctypes.data, k.size, rk.ctypes.data)
    return rk[:16 * (nr + 1)].tobytes()


def aes_encrypt_block(key, block) -> bytes:
    k = _key(key)
    rk = np.zeros(240, np.uint8)
    nr = _lib.orc_aes_key_expand(k.ctypes.data, k.size, rk.ctypes.data)
    b = _in(block, 16)
    out = np.zeros(16, np.uint8)
    _lib.orc_aes_encrypt_block(rk.ctypes.data, nr, b.ctypes.data, out.ctypes.data)
    return out.tobytes()


def gf128_mul(x, y) -> bytes:
    a, b = _in(x, 16), _in(y, 16)
    out = np.zeros(16, np.uint8)
    _lib.orc_gf128_mul(a.ctypes.data, b.ctypes.data, out.ctypes.data)
    return out.tobytes()


def ghash(h, data, y0=bytes(16)) -> bytes:
    """GHASH_H over whole blocks (len(data) % 16 == 0), continuing from state y0."""
    hh, d = _in(h, 16), _in(data)
    if d.size % 16:
        raise ValueError("ghash takes whole blocks")
    y = _in(y0, 16).copy()
    _lib.orc_ghash_update(hh.ctypes.data, _ptr(d), d.size // 16, y.ctypes.data)
    return y.tobytes()


def gctr(key, iv, data) -> bytes:
    rk, v, d = _in(aes256_key_expand(key)), _in(iv, 12), _in(data)
    out = np.zeros(d.size, np.uint8)
    _lib.orc_gctr(rk.ctypes.data, v.ctypes.data, _ptr(d), d.size, _ptr(out))
    return out.tobytes()


def encrypt(key, iv, aad, pt):
    """-> (ciphertext bytes, 16-byte tag)"""
    k, v, a, p = _key(key), _in(iv), _in(aad), _in(pt)
    if v.size == 0:
        raise ValueError("GCM takes no empty IV")
    ct = np.zeros(p.size, np.uint8)
    tag = np.zeros(16, np.uint8)
    done = _lib.orc_gcm_encrypt_ex(k.ctypes.data, k.size, v.ctypes.data, v.size, _ptr(a), a.size,
                                   _ptr(p), p.size, _ptr(ct), tag.ctypes.data)
    assert done == 1
    return ct.tobytes(), tag.tobytes()


def decrypt_verify(key, iv, aad, ct, tag):
    """-> (ok flag, plaintext bytes; all zero when ok is False)"""
    k, v, a, c, t = _key(key), _in(iv), _in(aad), _in(ct), _in(tag, 16)
    if v.size == 0:
        raise ValueError("GCM takes no empty IV")
    pt = np.full(c.size, 0xAA, np.uint8)
    ok = _lib.orc_gcm_decrypt_verify_ex(k.ctypes.data, k.size, v.ctypes.data, v.size, _ptr(a),
                                        a.size, _ptr(c), c.size, t.ctypes.data, _ptr(pt))
    return bool(ok), pt.tobytes()


def _batch_args(key, ivs, aads, srcs):
    n = len(srcs)
    k = _key(key)
    v = _in(np.asarray(ivs, dtype=np.uint8).reshape(-1))
    if n == 0 or v.size == 0 or v.size % n:
        raise ValueError("ivs: n IVs of one length (12 bytes in the paper's transport)")
    src = [np.ascontiguousarray(s, dtype=np.uint8) for s in srcs]
    lens = np.array([s.size for s in src], np.uint64)
    src_p = np.array([s.ctypes.data for s in src], np.uint64)
    dst = [np.zeros(s.size, np.uint8) for s in src]
    dst_p = np.array([d.ctypes.data for d in dst], np.uint64)
    if aads is None:
        aad, aad_p, aad_l = None, None, None
    else:
        aad = [np.ascontiguousarray(a, dtype=np.uint8) for a in aads]
        aad_p = np.array([a.ctypes.data for a in aad], np.uint64)
        aad_l = np.array([a.size for a in aad], np.uint32)
    keep = (k, v, src, aad, lens, src_p, dst_p, aad_p, aad_l)
    return n, k, v, aad_p, aad_l, src_p, lens, dst, dst_p, keep


def encrypt_batch(key, ivs, aads, srcs, nthreads=1):
    """srcs: list of uint8 arrays; aads: list of uint8 arrays or None; ivs: n IVs of one length.
    -> (list of ciphertext arrays, tags array (n,16), threads used)"""
    n, k, v, aad_p, aad_l, src_p, lens, dst, dst_p, keep = _batch_args(key, ivs, aads, srcs)
    tags = np.zeros((n, 16), np.uint8)
    used = _lib.orc_gcm_encrypt_batch_ex(
        k.ctypes.data, k.size, v.size // n, n, _ptr(v), None if aad_p is None else aad_p.ctypes.data,
        None if aad_l is None else aad_l.ctypes.data, src_p.ctypes.data, lens.ctypes.data,
        dst_p.ctypes.data, tags.ctypes.data, nthreads)
    del keep
    return dst, tags, used


def decrypt_verify_batch(key, ivs, aads, srcs, tags, nthreads=1):
    """-> (list of plaintext arrays, ok array (n,) uint8, threads used)"""
    n, k, v, aad_p, aad_l, src_p, lens, dst, dst_p, keep = _batch_args(key, ivs, aads, srcs)
    t = _in(np.asarray(tags, dtype=np.uint8).reshape(-1), 16 * n)
    ok = np.zeros(n, np.uint8)
    used = _lib.orc_gcm_decrypt_verify_batch_ex(
        k.ctypes.data, k.size, v.size // n, n, _ptr(v), None if aad_p is None else aad_p.ctypes.data,
        None if aad_l is None else aad_l.ctypes.data, src_p.ctypes.data, lens.ctypes.data,
        dst_p.ctypes.data, _ptr(t), ok.ctypes.data, nthreads)
    del keep
    return dst, ok, used
