"""The tables the key set-up kernel leaves on the device, piece by piece against the oracle: key
schedule (FIPS-197 5.2), round tables (S-box and MixColumns coefficients), H = E_K(0), and the
nibble tables of H^(2^k), each entry being one GF(2^128) product (SP 800-38D 6.3), and the
multiplication by H^64 written out as a 128 x 128 matrix over GF(2) for the matrix cores, and the
nibble tables of H^3, H^12, H^48 the lane tree uses."""
import numpy as np
import pytest

import oracle

import paper_2411_03357_amd as pgcm

pytestmark = pytest.mark.gpu


def _xtime(v):
    return ((v << 1) ^ (0x1B if v & 0x80 else 0)) & 0xFF


@pytest.mark.parametrize("key_bytes", [16, 24, 32])
def test_device_tables_entry_by_entry(key_bytes):
    rng = np.random.default_rng(1000 + key_bytes)
    keyb = rng.integers(0, 256, key_bytes, dtype=np.uint8).tobytes()
    key = pgcm.expand_key_bytes(keyb)
    t = pgcm.copy_key_tables(key)
    key.free()
    assert pgcm.load_library().pgcm_key_tables_bytes() == 256 + 4096 + 16 + 31 * 512 * 16 + 8192 + 3 * 512 * 16

    # key schedule
    rk = oracle.aes_key_expand(keyb)
    nr = key_bytes // 4 + 6
    assert t["rounds"] == nr and len(rk) == 16 * (nr + 1)
    assert t["rk"][:4 * (nr + 1)].tobytes() == rk          # little-endian words = the bytes
    assert not t["rk"][4 * (nr + 1):].any()

    # round tables: te[0][x] = (2 S(x), S(x), S(x), 3 S(x)) in bytes 0..3, te[r] rotated by r bytes
    S = oracle.sbox()
    for x in range(256):
        s = S[x]
        col = bytes([_xtime(s), s, s, _xtime(s) ^ s])
        for r in range(4):
            want = bytes(col[(b - r) % 4] for b in range(4))
            assert int(t["te"][r][x]).to_bytes(4, "little") == want, (r, x)

    # H and the nibble tables of its powers
    h = oracle.aes_encrypt_block(keyb, bytes(16))
    assert t["h"].tobytes() == h
    assert t["ghash"].shape == (31, 512, 16)
    power = h
    for k in range(31):
        tab = t["ghash"][k]
        for pos in range(32):
            for val in (1, 2, 4, 8, 15, int(rng.integers(0, 16))):
                x = bytearray(16)
                x[pos // 2] = val << 4 if pos % 2 == 0 else val
                want = oracle.gf128_mul(bytes(x), power)
                assert tab[pos * 16 + val].tobytes() == want, (k, pos, val)
            assert not tab[pos * 16].any()                  # value 0 -> the zero block
        # the table is linear in the nibble: entry[a ^ b] = entry[a] ^ entry[b], all of it
        rows = tab.reshape(32, 16, 16)
        for a in (1, 2, 4, 8):
            for b in range(16):
                assert np.array_equal(rows[:, a ^ b], rows[:, a] ^ rows[:, b])
        power = oracle.gf128_mul(power, power)               # H^(2^(k+1))


    # the three constants of the lane tree that are not H^(2^k)
    def power(e):
        r, base = None, h
        while e:
            if e & 1:
                r = base if r is None else oracle.gf128_mul(r, base)
            base = oracle.gf128_mul(base, base)
            e >>= 1
        return r
    assert t["ghash_lane"].shape == (3, 512, 16)
    for k, e in enumerate((3, 12, 48)):
        c = power(e)
        tab = t["ghash_lane"][k]
        for pos in range(32):
            for val in range(16):
                x = bytearray(16)
                x[pos // 2] = val << 4 if pos % 2 == 0 else val
                assert tab[pos * 16 + val].tobytes() == oracle.gf128_mul(bytes(x), c), (e, pos, val)

    # Multiplication by H^64 as matrix-core operands.  Bit b of a block, as the kernels hold it, is
    # bit b % 32 of the little-endian word b // 32.  Lane l of tile mt holds the matrix row whose
    # sum lands in result register reg = 4 * (l % 32 // 8) + l % 4 and makes bit
    # 16 * (reg // 8) + 8 * (mt % 2) + reg % 8 of product word 2 * ((l % 32 // 4) % 2) + mt // 2;
    # nibble j of register r in depth slice ks is the entry for multiplicand bit
    # 32 r + 4 j + 2 ks + l // 32: 2 (1.0 as a 4-bit float) where x^bit * H^64 has the product bit.
    h64 = h
    for _ in range(6):
        h64 = oracle.gf128_mul(h64, h64)
    cols = []
    for b in range(128):
        x = bytearray(16)
        x[b // 8] = 1 << (b % 8)
        cols.append(int.from_bytes(oracle.gf128_mul(bytes(x), h64), "little"))
    m = t["row_matrix"]
    for mt in range(4):
        for ks in range(2):
            for lane in range(64):
                ml, half = lane % 32, lane // 32
                reg = 4 * (ml // 8) + ml % 4
                out_bit = 32 * (2 * ((ml // 4) % 2) + mt // 2) + 16 * (reg // 8) + 8 * (mt % 2) + reg % 8
                for r in range(4):
                    want = 0
                    for j in range(8):
                        if (cols[32 * r + 4 * j + 2 * ks + half] >> out_bit) & 1:
                            want |= 2 << (4 * j)
                    assert int(m[mt, ks, lane, r]) == want, (mt, ks, lane, r)
