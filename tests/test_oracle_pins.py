"""Pins the CPU oracle to things other than itself: published worked examples, closed forms,
field axioms, an independent textbook formulation of each field, and the host's libcrypto.
Runs without a GPU."""
import os

import numpy as np
import pytest

import openssl_ref
import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _records(name):
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                yield [p.strip() for p in line.split("|")]


def _hex(s):
    return b"" if s == "-" else bytes.fromhex(s.replace(" ", ""))


# ---------------------------------------------------------------- GF(2^8) and the S-box
def _gf8_tables():
    """log / antilog tables of GF(2^8) with generator 0x03: a formulation of the field that
    does not share the oracle's shift-and-add multiply"""
    exp, log = [0] * 255, [0] * 256
    x = 1
    for i in range(255):
        exp[i], log[x] = x, i
        x2 = (x << 1) ^ (0x11B if x & 0x80 else 0)
        x = x2 ^ x          # times 3 = times 2 plus itself
    return exp, log


def test_sbox_against_log_tables_and_printed_entries():
    S = oracle.sbox()
    exp, log = _gf8_tables()
    for x in range(256):
        inv = 0 if x == 0 else exp[(255 - log[x]) % 255]
        b = inv
        # affine map written as rotations: b ^ rotl(b,1) ^ rotl(b,2) ^ rotl(b,3) ^ rotl(b,4) ^ 63
        rot = lambda v, k: ((v << k) | (v >> (8 - k))) & 0xFF
        assert S[x] == b ^ rot(b, 1) ^ rot(b, 2) ^ rot(b, 3) ^ rot(b, 4) ^ 0x63
    # entries FIPS-197 prints (figure 7 and the worked S-box example for 0x53)
    assert (S[0x00], S[0x01], S[0x53], S[0xFF]) == (0x63, 0x7C, 0xED, 0x16)
    assert sorted(S) == list(range(256))
    assert all(S[x] != x and S[x] != x ^ 0xFF for x in range(256))


def test_block_cipher_and_key_schedule_worked_examples():
    seen = set()
    for rec in _records("aes_block_vectors.txt"):
        key = _hex(rec[1])
        seen.add((rec[0], len(key)))
        if rec[0] == "block":
            assert oracle.aes_encrypt_block(key, _hex(rec[2])) == _hex(rec[3])
        elif rec[0] == "hzero":
            assert oracle.aes_encrypt_block(key, bytes(16)) == _hex(rec[2])
        elif rec[0] == "rkeys":
            rk = oracle.aes_key_expand(key)
            assert len(rk) == 16 * (len(key) // 4 + 7)
            first = int(rec[2])
            words = _hex(rec[3])
            assert rk[4 * first:4 * first + len(words)] == words
            assert rk[:len(key)] == key
        if len(key) == 32 and rec[0] == "block":
            assert oracle.aes256_encrypt_block(key, _hex(rec[2])) == _hex(rec[3])
            assert oracle.aes256_key_expand(key) == oracle.aes_key_expand(key)
    assert {("block", 16), ("block", 24), ("block", 32), ("rkeys", 16), ("rkeys", 24),
            ("rkeys", 32)} <= seen


def test_block_cipher_against_libcrypto_ecb():
    rng = np.random.default_rng(11)
    for i in range(450):
        k = rng.integers(0, 256, (16, 24, 32)[i % 3], dtype=np.uint8).tobytes()
        b = rng.integers(0, 256, 16, dtype=np.uint8).tobytes()
        assert oracle.aes_encrypt_block(k, b) == openssl_ref.aes_ecb_block(k, b)


# ---------------------------------------------------------------- GF(2^128)
_R = (1 << 128) | (1 << 7) | (1 << 2) | (1 << 1) | 1   # x^128 + x^7 + x^2 + x + 1


def _to_poly(block: bytes) -> int:
    """GCM's bit i (bit 0 = most significant bit of byte 0) is the coefficient of x^i"""
    v = int.from_bytes(block, "big")
    return sum(((v >> (127 - i)) & 1) << i for i in range(128))


def _from_poly(p: int) -> bytes:
    v = sum(((p >> i) & 1) << (127 - i) for i in range(128))
    return v.to_bytes(16, "big")


def _poly_mul(a: int, b: int) -> int:
    """schoolbook carry-less product followed by long division by the field polynomial"""
    prod = 0
    for i in range(128):
        if (b >> i) & 1:
            prod ^= a << i
    for d in range(prod.bit_length() - 1, 127, -1):
        if (prod >> d) & 1:
            prod ^= _R << (d - 128)
    return prod


def _rand_blocks(rng, n):
    return [rng.integers(0, 256, 16, dtype=np.uint8).tobytes() for _ in range(n)]


def test_gf128_mul_against_polynomial_arithmetic():
    rng = np.random.default_rng(12)
    for x, y in zip(_rand_blocks(rng, 200), _rand_blocks(rng, 200)):
        assert oracle.gf128_mul(x, y) == _from_poly(_poly_mul(_to_poly(x), _to_poly(y)))


def test_gf128_closed_forms_and_axioms():
    rng = np.random.default_rng(13)
    one = bytes([0x80]) + bytes(15)            # the field's 1: only bit 0 set
    x1 = bytes([0x40]) + bytes(15)             # the element x
    x127 = bytes(15) + bytes([0x01])           # x^127
    zero = bytes(16)
    # x^127 * x = x^128 = x^7 + x^2 + x + 1 -> bits 0,1,2,7 -> byte 0 = 0xE1
    assert oracle.gf128_mul(x127, x1) == bytes([0xE1]) + bytes(15)
    assert oracle.gf128_mul(x1, x127) == bytes([0xE1]) + bytes(15)
    xor = lambda a, b: bytes(p ^ q for p, q in zip(a, b))
    for a, b, c in zip(*(_rand_blocks(rng, 60) for _ in range(3))):
        assert oracle.gf128_mul(a, one) == a and oracle.gf128_mul(one, a) == a
        assert oracle.gf128_mul(a, zero) == zero
        assert oracle.gf128_mul(a, b) == oracle.gf128_mul(b, a)
        assert oracle.gf128_mul(a, xor(b, c)) == xor(oracle.gf128_mul(a, b), oracle.gf128_mul(a, c))
        assert oracle.gf128_mul(oracle.gf128_mul(a, b), c) == \
            oracle.gf128_mul(a, oracle.gf128_mul(b, c))
    # multiplying by x shifts toward bit 127 when the top coefficient is clear
    a = bytes([0x12, 0x34]) + bytes(13) + bytes([0x10])
    shifted = (int.from_bytes(a, "big") >> 1).to_bytes(16, "big")
    assert oracle.gf128_mul(a, x1) == shifted


def test_ghash_is_the_polynomial_in_h():
    rng = np.random.default_rng(14)
    h = _rand_blocks(rng, 1)[0]
    xor = lambda a, b: bytes(p ^ q for p, q in zip(a, b))
    for m in (0, 1, 2, 3, 7, 20):
        xs = _rand_blocks(rng, m)
        # sum_i X_i * H^(m - i + 1), powers by repeated polynomial multiplication
        acc, hp = 0, _to_poly(h)
        powers = [hp]
        for _ in range(m):
            powers.append(_poly_mul(powers[-1], hp))
        for i, x in enumerate(xs, start=1):
            acc ^= _poly_mul(_to_poly(x), powers[m - i])
        assert oracle.ghash(h, b"".join(xs)) == _from_poly(acc)
        # linearity in the input and invariance under a zero prefix
        ys = _rand_blocks(rng, m)
        both = b"".join(xor(a, b) for a, b in zip(xs, ys))
        assert oracle.ghash(h, both) == xor(oracle.ghash(h, b"".join(xs)),
                                            oracle.ghash(h, b"".join(ys)))
        assert oracle.ghash(h, bytes(48) + b"".join(xs)) == oracle.ghash(h, b"".join(xs))
        # continuing from a state equals hashing with that state as a leading block
        if m:
            y0 = _rand_blocks(rng, 1)[0]
            lead = xor(y0, xs[0]) + b"".join(xs[1:])
            assert oracle.ghash(h, b"".join(xs), y0) == oracle.ghash(h, lead)


# ---------------------------------------------------------------- GCM
def test_gcm_published_vectors():
    n = 0
    for name, key, iv, aad, pt, ct, tag in _records("aes_gcm_vectors.txt"):
        c, t = oracle.encrypt(_hex(key), _hex(iv), _hex(aad), _hex(pt))
        assert (c, t) == (_hex(ct), _hex(tag)), name
        ok, p = oracle.decrypt_verify(_hex(key), _hex(iv), _hex(aad), _hex(ct), _hex(tag))
        assert ok and p == _hex(pt), name
        n += 1
    assert n == 18


def test_gcm_closed_forms_from_the_block_cipher():
    """counter blocks: J0 = IV || 00000001 masks the tag, data block b uses IV || be32(b + 2);
    checked with libcrypto's plain ECB, a different routine from its GCM"""
    rng = np.random.default_rng(15)
    for _ in range(20):
        k = rng.integers(0, 256, 32, dtype=np.uint8).tobytes()
        iv = rng.integers(0, 256, 12, dtype=np.uint8).tobytes()
        ecb = lambda ctr: openssl_ref.aes256_ecb_block(k, iv + ctr.to_bytes(4, "big"))
        # empty A and P: GHASH input is the single all-zero length block, so S = 0
        assert oracle.encrypt(k, iv, b"", b"") == (b"", ecb(1))
        # zero plaintext exposes the keystream
        ct, tag = oracle.encrypt(k, iv, b"", bytes(16 * 5 + 3))
        assert ct == b"".join(ecb(2 + b) for b in range(6))[:83]
        assert oracle.gctr(k, iv, bytes(40)) == (ecb(2) + ecb(3) + ecb(4))[:40]
        # tag = GHASH(A pad || C pad || [8|A|]_64 [8|C|]_64) xor E_K(J0), assembled by hand
        h = openssl_ref.aes256_ecb_block(k, bytes(16))
        aad = rng.integers(0, 256, 21, dtype=np.uint8).tobytes()
        ct, tag = oracle.encrypt(k, iv, aad, bytes(83))
        blocks = aad + bytes(11) + ct + bytes(13) + (8 * 21).to_bytes(8, "big") + \
            (8 * 83).to_bytes(8, "big")
        s = _to_poly(bytes(16))
        hp = _to_poly(h)
        for i in range(0, len(blocks), 16):
            s = _poly_mul(s ^ _to_poly(blocks[i:i + 16]), hp)
        assert tag == bytes(a ^ b for a, b in zip(_from_poly(s), ecb(1)))


def test_pre_counter_block_of_other_iv_lengths_and_counter_wrap():
    """an IV that is not 96 bits long is hashed into J0 = GHASH_H(IV pad || 0^64 || [8|IV|]_64)
    (SP 800-38D 7.1 step 2) and the counter is the last 32 bits of J0 alone, wrapping modulo
    2^32 (6.2).  J0 is assembled here from polynomial arithmetic and libcrypto's ECB; a 16-byte
    IV is then solved for (J0 is linear in it) so that the counter wraps inside the message."""
    import iv_craft
    rng = np.random.default_rng(21)
    for trial in range(12):
        k = rng.integers(0, 256, (16, 24, 32)[trial % 3], dtype=np.uint8).tobytes()
        h = openssl_ref.aes_ecb_block(k, bytes(16))
        for ivlen in (1, 8, 11, 13, 16, 17, 60, 128):
            iv = rng.integers(0, 256, ivlen, dtype=np.uint8).tobytes()
            j0 = iv_craft.j0_of(h, iv)
            ctr = int.from_bytes(j0[12:], "big")
            ecb = lambda n: openssl_ref.aes_ecb_block(
                k, j0[:12] + ((ctr + n) % (1 << 32)).to_bytes(4, "big"))
            assert oracle.encrypt(k, iv, b"", b"") == (b"", ecb(0))
            ct, _ = oracle.encrypt(k, iv, b"", bytes(50))
            assert ct == b"".join(ecb(1 + b) for b in range(4))[:50]
        # counter field of J0 set to 2^32 - 3: data blocks use 2^32-2, 2^32-1, 0, 1, ...
        want = rng.integers(0, 256, 12, dtype=np.uint8).tobytes() + (2 ** 32 - 3).to_bytes(4, "big")
        iv = iv_craft.iv_for_j0(h, want)
        assert len(iv) == 16 and iv_craft.j0_of(h, iv) == want
        ecb = lambda c: openssl_ref.aes_ecb_block(k, want[:12] + (c % (1 << 32)).to_bytes(4, "big"))
        a = rng.integers(0, 256, 5, dtype=np.uint8).tobytes()
        p = rng.integers(0, 256, 16 * 6 + 9, dtype=np.uint8).tobytes()
        ct, tag = oracle.encrypt(k, iv, a, p)
        ks = b"".join(ecb(2 ** 32 - 2 + b) for b in range(7))
        assert ct == bytes(x ^ y for x, y in zip(p, ks))
        assert (ct, tag) == openssl_ref.encrypt(k, iv, a, p)
        assert oracle.decrypt_verify(k, iv, a, ct, tag) == (True, p)


def test_gcm_against_libcrypto_other_key_and_iv_lengths():
    rng = np.random.default_rng(22)
    for i in range(600):
        k = rng.integers(0, 256, (16, 24, 32)[i % 3], dtype=np.uint8).tobytes()
        ivlen = int(rng.integers(1, 129)) if i % 5 else 12    # libcrypto takes IVs up to 128 bytes
        iv = rng.integers(0, 256, ivlen, dtype=np.uint8).tobytes()
        a = rng.integers(0, 256, int(rng.integers(0, 65)), dtype=np.uint8).tobytes()
        p = rng.integers(0, 256, int(rng.integers(0, 1500)), dtype=np.uint8).tobytes()
        c, t = oracle.encrypt(k, iv, a, p)
        assert (c, t) == openssl_ref.encrypt(k, iv, a, p), (len(k), ivlen, len(p))
        assert oracle.decrypt_verify(k, iv, a, c, t) == (True, p)
        if len(p):
            bad = bytearray(c)
            bad[int(rng.integers(0, len(p)))] ^= 1 << int(rng.integers(0, 8))
            assert oracle.decrypt_verify(k, iv, a, bytes(bad), t) == (False, bytes(len(p)))


def test_gcm_against_libcrypto_random():
    rng = np.random.default_rng(16)
    lens = list(range(0, 70)) + [int(v) for v in rng.integers(0, 4097, 900)] + \
        [1023, 1024, 1025, 4095, 4096, 65536 + 17]
    keys, ivs, aads, pts = [], [], [], []
    for ln in lens:
        keys.append(rng.integers(0, 256, 32, dtype=np.uint8).tobytes())
        ivs.append(rng.integers(0, 256, 12, dtype=np.uint8).tobytes())
        aads.append(rng.integers(0, 256, int(rng.integers(0, 65)), dtype=np.uint8).tobytes())
        pts.append(rng.integers(0, 256, ln, dtype=np.uint8).tobytes())
    for k, iv, a, p in zip(keys, ivs, aads, pts):
        c, t = oracle.encrypt(k, iv, a, p)
        assert (c, t) == openssl_ref.encrypt(k, iv, a, p)
        ok, back = oracle.decrypt_verify(k, iv, a, c, t)
        assert ok and back == p


def test_gcm_invariants():
    rng = np.random.default_rng(17)
    xor = lambda a, b: bytes(p ^ q for p, q in zip(a, b))
    for ln in (0, 1, 16, 33, 100, 1000):
        k = rng.integers(0, 256, 32, dtype=np.uint8).tobytes()
        iv = rng.integers(0, 256, 12, dtype=np.uint8).tobytes()
        a = rng.integers(0, 256, 20, dtype=np.uint8).tobytes()
        p = rng.integers(0, 256, ln, dtype=np.uint8).tobytes()
        d = rng.integers(0, 256, ln, dtype=np.uint8).tobytes()
        c1, t1 = oracle.encrypt(k, iv, a, p)
        c2, t2 = oracle.encrypt(k, iv, a, xor(p, d))
        # CTR: the keystream does not depend on the data
        assert c2 == xor(c1, d)
        # tags of two equal-length messages differ by the GHASH of the ciphertext difference
        h = oracle.aes256_encrypt_block(k, bytes(16))
        pad = (-ln) % 16
        expect = oracle.ghash(h, bytes(32) + xor(c1, c2) + bytes(pad) + bytes(16))
        assert xor(t1, t2) == expect
        assert oracle.decrypt_verify(k, iv, a, c1, t1) == (True, p)


def test_every_single_bit_flip_is_rejected_and_output_is_wiped():
    rng = np.random.default_rng(18)
    k = rng.integers(0, 256, 32, dtype=np.uint8).tobytes()
    iv = rng.integers(0, 256, 12, dtype=np.uint8).tobytes()
    a = rng.integers(0, 256, 16, dtype=np.uint8).tobytes()
    p = rng.integers(0, 256, 64, dtype=np.uint8).tobytes()
    c, t = oracle.encrypt(k, iv, a, p)

    def flips(b):
        for i in range(8 * len(b)):
            m = bytearray(b)
            m[i // 8] ^= 1 << (i % 8)
            yield bytes(m)

    bad = (False, bytes(64))
    for m in flips(c):
        assert oracle.decrypt_verify(k, iv, a, m, t) == bad
    for m in flips(a):
        assert oracle.decrypt_verify(k, iv, m, c, t) == bad
    for m in flips(iv):
        assert oracle.decrypt_verify(k, m, a, c, t) == bad
    for m in flips(t):
        assert oracle.decrypt_verify(k, iv, a, c, m) == bad
    # a wrong key, a truncated and an extended message are rejected too
    assert oracle.decrypt_verify(bytes(32), iv, a, c, t) == bad
    assert oracle.decrypt_verify(k, iv, a, c[:-1], t)[0] is False
    assert oracle.decrypt_verify(k, iv, a, c + b"\0", t)[0] is False


def test_batch_entry_points_equal_the_single_calls():
    import workloads
    w = workloads.ragged_small()
    buf = w.payload_host()
    srcs = [w.chunk(buf, i) for i in range(w.n)]
    aads = [np.frombuffer(w.aad_of(i), np.uint8) for i in range(w.n)]
    cts, tags, used = oracle.encrypt_batch(w.key, w.ivs, aads, srcs, nthreads=4)
    assert 1 <= used <= 4
    for i in range(w.n):
        c, t = oracle.encrypt(w.key, w.ivs[i], aads[i], srcs[i])
        assert cts[i].tobytes() == c and tags[i].tobytes() == t
        assert (c, t) == openssl_ref.encrypt(w.key.tobytes(), w.ivs[i].tobytes(), w.aad_of(i),
                                             srcs[i].tobytes())
    bad_tags = tags.copy()
    bad_tags[3, 5] ^= 0x10
    pts, ok, _ = oracle.decrypt_verify_batch(w.key, w.ivs, aads, cts, bad_tags, nthreads=4)
    for i in range(w.n):
        assert ok[i] == (0 if i == 3 else 1)
        assert pts[i].tobytes() == (bytes(srcs[i].size) if i == 3 else srcs[i].tobytes())
    # "no AAD at all" form
    cts2, tags2, _ = oracle.encrypt_batch(w.key, w.ivs[:5], None, srcs[:5], nthreads=2)
    for i in range(5):
        assert (cts2[i].tobytes(), tags2[i].tobytes()) == oracle.encrypt(w.key, w.ivs[i], b"",
                                                                         srcs[i])
    # other key and IV lengths go through the same batch entry points
    rng = np.random.default_rng(23)
    for klen, ivlen in ((16, 8), (24, 16), (32, 60), (16, 12)):
        key = rng.integers(0, 256, klen, dtype=np.uint8)
        ivs = rng.integers(0, 256, (8, ivlen), dtype=np.uint8)
        cts3, tags3, _ = oracle.encrypt_batch(key, ivs, aads[:8], srcs[:8], nthreads=3)
        pts3, ok3, _ = oracle.decrypt_verify_batch(key, ivs, aads[:8], cts3, tags3, nthreads=3)
        for i in range(8):
            assert (cts3[i].tobytes(), tags3[i].tobytes()) == oracle.encrypt(key, ivs[i], aads[i],
                                                                             srcs[i])
            assert ok3[i] == 1 and pts3[i].tobytes() == srcs[i].tobytes()
