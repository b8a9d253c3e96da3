"""The bitsliced counter-mode kernel (a measurement aid, not the batch path) against the oracle's
block cipher: every block of a launch that spans several workgroups, all three key lengths, a
counter that wraps; bit-exact."""
import numpy as np
import pytest
import torch

import oracle

import paper_2411_03357_amd as pgcm

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("key_bytes", [32, 16, 24])
def test_bitsliced_keystream_equals_the_oracles_block_cipher(key_bytes):
    rng = np.random.default_rng(31 + key_bytes)
    keyb = rng.integers(0, 256, key_bytes, dtype=np.uint8)
    iv = rng.integers(0, 256, 12, dtype=np.uint8).tobytes()
    key = pgcm.expand_key_bytes(keyb)
    for ctr_base, nblocks in ((0, 2048), (32 * 12345, 3 * 2048), (2 ** 32 - 2048, 2 * 2048)):
        out = torch.full((16 * nblocks,), 0xEE, dtype=torch.uint8, device="cuda")
        pgcm.bitsliced_keystream(key, iv, ctr_base, nblocks, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy().reshape(nblocks, 16)
        step = 1 if nblocks <= 2048 else 7
        for b in list(range(0, nblocks, step)) + [nblocks - 1]:
            ctr = (ctr_base + b) % 2 ** 32
            want = oracle.aes_encrypt_block(keyb, iv + ctr.to_bytes(4, "big"))
            assert got[b].tobytes() == want, (key_bytes, ctr_base, b)
    # argument checks
    out = torch.zeros(16 * 2048, dtype=torch.uint8, device="cuda")
    for bad in (dict(ctr_base=5, nblocks=2048), dict(ctr_base=0, nblocks=100)):
        with pytest.raises(pgcm.PgcmError) as e:
            pgcm.bitsliced_keystream(key, iv, bad["ctr_base"], bad["nblocks"], out)
        assert e.value.status == -1
    key.free()
