"""The published GCM worked examples (tests/golden/aes_gcm_vectors.txt: all eighteen cases of the
GCM specification's appendix B, three key lengths, 64-, 96- and 480-bit IVs) run on the GPU
straight through the C ABI.  No torch here: device memory comes from the HIP runtime through
ctypes, so this is also the check that the boundary needs nothing but plain pointers and sizes.
The expected values are the specification's, not the oracle's."""
import ctypes as C
import os

import pytest

import paper_2411_03357_amd as pgcm
from paper_2411_03357_amd import binding

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "aes_gcm_vectors.txt")


def _records():
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                name, *fields = [p.strip() for p in line.split("|")]
                yield (name,) + tuple(b"" if v == "-" else bytes.fromhex(v) for v in fields)


class _Hip:
    def __init__(self):
        # the HIP runtime the library itself is linked to: its symbols resolve through the
        # library's handle
        self.lib = C.CDLL(pgcm.library_path())
        self.lib.hipMalloc.argtypes = [C.POINTER(C.c_void_p), C.c_size_t]
        self.lib.hipFree.argtypes = [C.c_void_p]
        self.lib.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        self.held = []

    def _ok(self, rc):
        assert rc == 0, "HIP error %d" % rc

    def alloc(self, nbytes):
        p = C.c_void_p()
        self._ok(self.lib.hipMalloc(C.byref(p), max(nbytes, 16)))
        self.held.append(p)
        return p.value

    def put(self, data: bytes):
        p = self.alloc(len(data))
        if data:
            self._ok(self.lib.hipMemcpy(p, data, len(data), 1))   # host to device
        return p

    def get(self, p, nbytes):
        out = C.create_string_buffer(max(nbytes, 1))
        self._ok(self.lib.hipDeviceSynchronize())
        if nbytes:
            self._ok(self.lib.hipMemcpy(out, p, nbytes, 2))       # device to host
        return out.raw[:nbytes]

    def free_all(self):
        self._ok(self.lib.hipDeviceSynchronize())
        for p in self.held:
            self._ok(self.lib.hipFree(p))
        self.held = []


def _arr(values, ctype):
    return (ctype * len(values))(*values)


def test_published_vectors_one_call_each():
    lib = binding.load_library()
    hip = _Hip()
    n = 0
    for name, key, iv, aad, pt, ct, tag in _records():
        handle = C.c_void_p()
        assert lib.pgcm_expand_key_bytes(key, len(key), None, C.byref(handle)) == 0, name
        d_iv, d_aad, d_pt = hip.put(iv), hip.put(aad), hip.put(pt)
        d_ct, d_back, d_tag, d_ok = (hip.alloc(len(pt)), hip.alloc(len(pt)), hip.alloc(16),
                                     hip.put(b"\xee"))
        aads, alens = _arr([d_aad], C.c_void_p), _arr([len(aad)], C.c_uint32)
        lens = _arr([len(pt)], C.c_uint64)
        rc = lib.pgcm_encrypt_batch_iv(handle, 1, d_iv, len(iv), aads, alens,
                                       _arr([d_pt], C.c_void_p), lens, _arr([d_ct], C.c_void_p),
                                       d_tag, None)
        assert rc == 0, name
        assert hip.get(d_ct, len(pt)) == ct, name
        assert hip.get(d_tag, 16) == tag, name
        rc = lib.pgcm_decrypt_verify_batch_iv(handle, 1, d_iv, len(iv), aads, alens,
                                              _arr([d_ct], C.c_void_p), lens,
                                              _arr([d_back], C.c_void_p), d_tag, d_ok, None)
        assert rc == 0, name
        assert hip.get(d_ok, 1) == b"\x01" and hip.get(d_back, len(pt)) == pt, name
        # the published tag with one bit flipped is refused and nothing of the plaintext stays
        d_bad = hip.put(bytes([tag[0] ^ 0x80]) + tag[1:])
        rc = lib.pgcm_decrypt_verify_batch_iv(handle, 1, d_iv, len(iv), aads, alens,
                                              _arr([d_ct], C.c_void_p), lens,
                                              _arr([d_back], C.c_void_p), d_bad, d_ok, None)
        assert rc == 0, name
        assert hip.get(d_ok, 1) == b"\x00" and hip.get(d_back, len(pt)) == bytes(len(pt)), name
        hip.free_all()
        lib.pgcm_free_key(handle)
        n += 1
    assert n == 18


def test_published_vectors_as_one_batch_of_several_keys():
    """the twelve cases with 96-bit IVs in one call: six keys of three lengths, a key per chunk"""
    lib = binding.load_library()
    hip = _Hip()
    cases = [r for r in _records() if len(r[2]) == 12]
    assert len(cases) == 12
    keys = sorted({r[1] for r in cases})
    assert sorted({len(k) for k in keys}) == [16, 24, 32] and len(keys) == 6
    handles = []
    for k in keys:
        h = C.c_void_p()
        assert lib.pgcm_expand_key_bytes(k, len(k), None, C.byref(h)) == 0
        handles.append(h)
    n = len(cases)
    d_ivs = hip.put(b"".join(r[2] for r in cases))
    d_tags, d_ok = hip.alloc(16 * n), hip.put(b"\xee" * n)
    srcs = [hip.put(r[4]) for r in cases]
    dsts = [hip.alloc(len(r[4])) for r in cases]
    aads = [hip.put(r[3]) for r in cases]
    index = _arr([keys.index(r[1]) for r in cases], C.c_uint32)
    alens = _arr([len(r[3]) for r in cases], C.c_uint32)
    lens = _arr([len(r[4]) for r in cases], C.c_uint64)
    hs = _arr([h.value for h in handles], C.c_void_p)
    rc = lib.pgcm_encrypt_batch_keys(hs, len(keys), index, n, d_ivs, 12, _arr(aads, C.c_void_p),
                                     alens, _arr(srcs, C.c_void_p), lens, _arr(dsts, C.c_void_p),
                                     d_tags, None)
    assert rc == 0
    tags = hip.get(d_tags, 16 * n)
    for i, r in enumerate(cases):
        assert hip.get(dsts[i], len(r[4])) == r[5], r[0]
        assert tags[16 * i:16 * i + 16] == r[6], r[0]
    # decrypt in place, one tag damaged (a case with 64 bytes of plaintext)
    damaged = 10
    assert len(cases[damaged][4]) == 64
    bad = bytearray(tags)
    bad[16 * damaged + 15] ^= 1
    d_bad = hip.put(bytes(bad))
    rc = lib.pgcm_decrypt_verify_batch_keys(hs, len(keys), index, n, d_ivs, 12,
                                            _arr(aads, C.c_void_p), alens, _arr(dsts, C.c_void_p),
                                            lens, _arr(dsts, C.c_void_p), d_bad, d_ok, None)
    assert rc == 0
    ok = hip.get(d_ok, n)
    assert ok == bytes(0 if i == damaged else 1 for i in range(n))
    for i, r in enumerate(cases):
        assert hip.get(dsts[i], len(r[4])) == (bytes(len(r[4])) if i == damaged else r[4]), r[0]
    hip.free_all()
    for h in handles:
        lib.pgcm_free_key(h)
