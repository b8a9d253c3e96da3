"""Do the pins bite?  Plausible mistakes are planted in copies of the oracle's C source (on the
CPU, never in GPU code); each mutant must fail at least one of the oracle's pin tests."""
import ctypes
import os
import subprocess
import sys
import tempfile

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "gcm_oracle.c")

# (name, text to find, replacement); every "find" occurs exactly once in the source
MUTANTS = [
    ("sbox affine constant", "((0x63 >> i) & 1)", "((0x62 >> i) & 1)"),
    ("sbox affine tap", "((b >> ((i + 4) % 8)) & 1)", "((b >> ((i + 3) % 8)) & 1)"),
    ("gf8 reduction polynomial", "a ^= 0x1B;", "a ^= 0x1D;"),
    ("rcon start", "uint8_t rcon = 0x01;", "uint8_t rcon = 0x02;"),
    ("key schedule: SubWord at i%Nk==4 dropped", "} else if (nk > 6 && i % nk == 4) {",
     "} else if (nk > 6 && i % nk == 9) {"),
    ("key schedule: SubWord at i%Nk==4 for 192-bit keys too", "} else if (nk > 6 && i % nk == 4) {",
     "} else if (nk >= 6 && i % nk == 4) {"),
    ("key schedule: one round too few", "nr = nk + 6;", "nr = nk + 5;"),
    ("RotWord direction", "t[0] = S[t[1]] ^ rcon;\n            t[1] = S[t[2]];\n            t[2] = S[t[3]];\n            t[3] = S[t0];",
     "t[0] = S[t[3]] ^ rcon;\n            t[3] = S[t[2]];\n            t[2] = S[t[1]];\n            t[1] = S[t0];"),
    ("state is row-major", "s[r][c] = in[r + 4 * c] ^ rk[r + 4 * c];", "s[r][c] = in[4 * r + c] ^ rk[4 * r + c];"),
    ("ShiftRows rotates right", "row[c] = s[r][(c + r) % 4];", "row[c] = s[r][(c + 4 - r) % 4];"),
    ("MixColumns coefficients swapped", "s[0][c] = gf8_mul(a0, 2) ^ gf8_mul(a1, 3) ^ a2 ^ a3;",
     "s[0][c] = gf8_mul(a0, 3) ^ gf8_mul(a1, 2) ^ a2 ^ a3;"),
    ("MixColumns in the last round too", "if (round != nr) {", "if (round != nr + 1) {"),
    ("last round missing", "for (int round = 1; round <= nr; round++) {", "for (int round = 1; round < nr; round++) {"),
    ("gf128 bit order", "return (b[i / 8] >> (7 - (i % 8))) & 1;", "return (b[i / 8] >> (i % 8)) & 1;"),
    ("gf128 reduction constant", "v[0] ^= 0xE1;", "v[0] ^= 0x87;"),
    ("gf128 shift loses the carry between bytes", "v[k] = (uint8_t)((v[k] >> 1) | ((v[k - 1] & 1) << 7));",
     "v[k] = (uint8_t)(v[k] >> 1);"),
    ("ghash multiplies before adding", "t[k] = y[k] ^ x[16 * i + k];\n        orc_gf128_mul(t, h, y);",
     "t[k] = y[k];\n        orc_gf128_mul(t, h, y);\n        for (int k = 0; k < 16; k++) y[k] ^= x[16 * i + k];"),
    ("first data block uses J0 itself", "uint32_t n = 1;", "uint32_t n = 0;"),
    ("counter little endian", "cb[12] = (uint8_t)(c >> 24);\n    cb[13] = (uint8_t)(c >> 16);\n    cb[14] = (uint8_t)(c >> 8);\n    cb[15] = (uint8_t)c;",
     "cb[15] = (uint8_t)(c >> 24);\n    cb[14] = (uint8_t)(c >> 16);\n    cb[13] = (uint8_t)(c >> 8);\n    cb[12] = (uint8_t)c;"),
    ("counter wrap carries into the rest of the block", "memcpy(cb, j0, 12);\n    cb[12]",
     "memcpy(cb, j0, 12);\n    if (c < n) cb[11]++;\n    cb[12]"),
    ("counter saturates instead of wrapping", "c += n; /* wraps modulo 2^32 */",
     "c = (c + n < c) ? 0xFFFFFFFFu : c + n;"),
    ("J0 of a 96-bit IV ends in 0", "j0[12] = 0, j0[13] = 0, j0[14] = 0, j0[15] = 1;\n        return;",
     "j0[12] = 0, j0[13] = 0, j0[14] = 0, j0[15] = 0;\n        return;"),
    ("J0: IV length in the wrong half of its block", "be64(8 * iv_bytes, lens + 8);", "be64(8 * iv_bytes, lens);"),
    ("J0: IV length in bytes", "be64(8 * iv_bytes, lens + 8);", "be64(iv_bytes, lens + 8);"),
    ("J0: length block left out", "orc_ghash_update(k->h, lens, 1, j0);", ";"),
    ("J0: IV not padded to a block", "ghash_padded(k->h, iv, iv_bytes, j0);",
     "orc_ghash_update(k->h, iv, (size_t)(iv_bytes / 16), j0);"),
    ("length block order", "be64(8 * alen, lens);\n    be64(8 * len, lens + 8);", "be64(8 * len, lens);\n    be64(8 * alen, lens + 8);"),
    ("lengths in bytes not bits", "be64(8 * len, lens + 8);", "be64(len, lens + 8);"),
    ("lengths little endian", "out[i] = (uint8_t)(v >> (56 - 8 * i));", "out[i] = (uint8_t)(v >> (8 * i));"),
    ("AAD hashed after the ciphertext", "ghash_padded(k->h, aad, alen, y);\n    ghash_padded(k->h, ct, len, y);",
     "ghash_padded(k->h, ct, len, y);\n    ghash_padded(k->h, aad, alen, y);"),
    ("partial block not hashed", "if (len % 16) {\n        uint8_t last[16] = {0};", "if (len % 16 > 16) {\n        uint8_t last[16] = {0};"),
    ("tag hashes the plaintext", "gcm_tag(&k, j0, aad, alen, ct, len, tag);\n    return 1;", "gcm_tag(&k, j0, aad, alen, pt, len, tag);\n    return 1;"),
    ("tag not masked", "tag[i] = y[i] ^ ekj0[i];", "tag[i] = y[i];"),
    ("compare skips the last byte", "for (int i = 0; i < 16; i++) /* all 16 bytes, no early exit */", "for (int i = 0; i < 15; i++) /* mutated */"),
    ("rejected output not wiped", "if (diff != 0) {\n        memset(pt, 0, (size_t)len);\n        return 0;",
     "if (diff != 0) {\n        gctr(&k, j0, ct, len, pt);\n        return 0;"),
    ("H is E_K of ones", "uint8_t zero[16] = {0};\n    k->nr", "uint8_t zero[16] = {1};\n    k->nr"),
]

PIN_TESTS = [
    pins.test_sbox_against_log_tables_and_printed_entries,
    pins.test_block_cipher_and_key_schedule_worked_examples,
    pins.test_gf128_closed_forms_and_axioms,
    pins.test_gf128_mul_against_polynomial_arithmetic,
    pins.test_ghash_is_the_polynomial_in_h,
    pins.test_gcm_published_vectors,
    pins.test_gcm_closed_forms_from_the_block_cipher,
    pins.test_pre_counter_block_of_other_iv_lengths_and_counter_wrap,
    pins.test_every_single_bit_flip_is_rejected_and_output_is_wiped,
    pins.test_gcm_invariants,
]


def _first_failing_pin():
    for t in PIN_TESTS:
        try:
            t()
        except AssertionError:
            return t.__name__
    return None


def test_the_unmutated_oracle_passes_the_pins_used_here():
    assert _first_failing_pin() is None


@pytest.mark.parametrize("name,find,repl", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(name, find, repl):
    text = open(SRC).read()
    assert text.count(find) == 1, "mutation site not unique: %r" % find
    with tempfile.TemporaryDirectory() as d:
        c = os.path.join(d, "mutant.c")
        so = os.path.join(d, "mutant.so")
        open(c, "w").write(text.replace(find, repl))
        subprocess.check_call(["gcc", "-O1", "-std=c11", "-shared", "-fPIC", "-pthread", c, "-o", so])
        good = oracle._lib
        oracle._lib = oracle._bind(ctypes.CDLL(so))
        try:
            caught = _first_failing_pin()
        finally:
            oracle._lib = good
    assert caught is not None, "no pin notices: " + name
