"""The tables the key set-up kernel leaves on the device, piece by piece against the oracle: key
schedule (FIPS-197 5.2), round tables (S-box and MixColumns coefficients), H = E_K(0), and the
nibble tables of H^(2^k), each entry being one GF(2^128) product (SP 800-38D 6.3)."""
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
    assert pgcm.load_library().pgcm_key_tables_bytes() == 256 + 4096 + 16 + 31 * 512 * 16

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
