"""The generator of the bitsliced round pieces: the committed header is what the generator
writes (its own checks compare the S-box circuit with the definition for all 256 inputs and the
MixColumns circuit with the definition on random columns before anything is written)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GEN = os.path.join(ROOT, "paper_2411_03357_amd", "csrc", "gen_bitsliced_aes.py")


def test_committed_header_is_what_the_generator_writes():
    assert subprocess.call([sys.executable, GEN, "--check"]) == 0


def test_generated_sbox_circuit_equals_the_definition_and_a_planted_fault_is_seen():
    sys.path.insert(0, os.path.dirname(GEN))
    import gen_bitsliced_aes as g
    cost, tower, gates, packed, out_names, nands = g.best_sbox()
    assert nands == 36 and cost == len(packed) <= 120
    # FIPS-197's own examples of the S-box
    for x, y in ((0x00, 0x63), (0x01, 0x7c), (0x53, 0xed), (0xff, 0x16)):
        assert g.sbox_value(x) == y and g.evaluate_packed(packed, out_names, 8, x) == y
    # one truth-table bit flipped somewhere must show
    nid, tt, ins = packed[len(packed) // 2]
    broken = list(packed)
    broken[len(packed) // 2] = (nid, tt ^ 2, ins)
    assert any(g.evaluate_packed(broken, out_names, 8, x) != g.sbox_value(x) for x in range(256))
