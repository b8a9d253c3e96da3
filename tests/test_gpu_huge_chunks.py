"""Single chunks beyond 4 GiB and at the GCM length limit (2^36 - 32 bytes): 64-bit offsets, four
fold levels, counters up to 2^32 - 1.  The CPU oracle is far too slow for these sizes (it is
pinned to libcrypto on small inputs, tests/test_oracle_pins.py), so the whole ciphertext and the
tag are compared against libcrypto fed piece by piece, and sampled blocks against the keystream
the oracle's block cipher gives one counter block at a time."""
import time

import numpy as np
import pytest
import torch

import openssl_ref
import oracle
import workloads

import paper_2411_03357_amd as pgcm

pytestmark = pytest.mark.gpu

GIB = 1 << 30
PIECE = 1 << 30


def _random_fill(t, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    step = 1 << 30
    for off in range(0, t.numel(), step):
        n = min(step, t.numel() - off)
        words = (n + 7) // 8
        r = torch.randint(-(1 << 62), 1 << 62, (words,), dtype=torch.int64, device="cuda",
                          generator=g).view(torch.uint8)
        t[off:off + n] = r[:n]
        del r


def _run(length, seed, aad_len):
    free, _ = torch.cuda.mem_get_info()
    if free < 2 * length + 6 * GIB:
        pytest.skip("needs %.0f GiB of device memory" % ((2 * length + 6 * GIB) / GIB))
    rng = np.random.default_rng(workloads.BASE_SEED + seed)
    keyb = rng.integers(0, 256, 32, dtype=np.uint8)
    iv = rng.integers(0, 256, 12, dtype=np.uint8)
    aad = rng.integers(0, 256, aad_len, dtype=np.uint8)
    key = pgcm.expand_key(keyb)
    plain = torch.empty(length, dtype=torch.uint8, device="cuda")
    _random_fill(plain, seed)
    cipher = torch.empty(length, dtype=torch.uint8, device="cuda")
    ivs = torch.from_numpy(iv.copy()).cuda()
    aad_d = torch.from_numpy(aad.copy()).cuda()
    tags = torch.zeros(16, dtype=torch.uint8, device="cuda")
    ok = torch.zeros(1, dtype=torch.uint8, device="cuda")
    lens = np.array([length], np.uint64)
    t0 = time.perf_counter()
    pgcm.encrypt_batch(key, ivs, [aad_d.data_ptr()], [aad_len], [plain.data_ptr()], lens,
                       [cipher.data_ptr()], tags)
    torch.cuda.synchronize()
    print("encrypt of %.1f GiB: %.1f ms" % (length / GIB, (time.perf_counter() - t0) * 1e3), flush=True)

    # sampled blocks, one counter block at a time: C_b = P_b xor E_K(IV || be32(b + 2))
    nblk = (length + 15) // 16
    picks = sorted({0, 1, 63, 64, 1023, 1024, (1 << 28) - 1, 1 << 28, (1 << 28) + 1,
                    nblk // 2, nblk - 65, nblk - 2, nblk - 1} | {int(v) for v in
                                                                 rng.integers(0, nblk, 40)})
    for b in picks:
        if not 0 <= b < nblk:
            continue
        m = min(16, length - 16 * b)
        p = plain[16 * b:16 * b + m].cpu().numpy()
        c = cipher[16 * b:16 * b + m].cpu().numpy()
        ks = oracle.aes_encrypt_block(keyb, iv.tobytes() + (b + 2).to_bytes(4, "big"))
        assert (p ^ np.frombuffer(ks, np.uint8)[:m]).tobytes() == c.tobytes(), b

    # every byte and the tag against libcrypto, piece by piece through pinned memory
    stream = openssl_ref.GcmEncryptStream(keyb.tobytes(), iv.tobytes(), aad.tobytes())
    hp = torch.empty(PIECE, dtype=torch.uint8, pin_memory=True)
    hc = torch.empty(PIECE, dtype=torch.uint8, pin_memory=True)
    out = np.empty(PIECE, np.uint8)
    t0 = time.perf_counter()
    for off in range(0, length, PIECE):
        n = min(PIECE, length - off)
        hp[:n].copy_(plain[off:off + n])
        hc[:n].copy_(cipher[off:off + n])
        torch.cuda.synchronize()
        ref = stream.update(hp.numpy()[:n], out)
        assert np.array_equal(ref, hc.numpy()[:n]), "ciphertext differs in the piece at %d" % off
        if (off // PIECE) % 8 == 7:
            print("compared %d GiB, %.0f s" % (off // GIB + 1, time.perf_counter() - t0), flush=True)
    assert tags.cpu().numpy().tobytes() == stream.tag()

    # decrypt in place: authentic, and the plaintext is back
    pgcm.decrypt_verify_batch(key, ivs, [aad_d.data_ptr()], [aad_len], [cipher.data_ptr()], lens,
                              [cipher.data_ptr()], tags, ok)
    torch.cuda.synchronize()
    assert int(ok.item()) == 1
    for off in range(0, length, 8 * PIECE):
        n = min(8 * PIECE, length - off)
        assert torch.equal(cipher[off:off + n], plain[off:off + n]), off
    # one flipped bit far beyond 4 GiB: rejected, all of the output wiped
    pgcm.encrypt_batch(key, ivs, [aad_d.data_ptr()], [aad_len], [plain.data_ptr()], lens,
                       [cipher.data_ptr()], tags)
    cipher[length - 5 * GIB // 8 - 3] ^= 0x04
    pgcm.decrypt_verify_batch(key, ivs, [aad_d.data_ptr()], [aad_len], [cipher.data_ptr()], lens,
                              [cipher.data_ptr()], tags, ok)
    torch.cuda.synchronize()
    assert int(ok.item()) == 0
    for off in range(0, length, 8 * PIECE):
        n = min(8 * PIECE, length - off)
        assert int(torch.count_nonzero(cipher[off:off + n]).item()) == 0, off
    key.free()
    return plain, cipher


def _same_with_one_unit_per_wavefront(plain, cipher, length):
    """the chunk once more in 4096 forced units of 16 MiB, a wavefront each (4096 sets -> 128
    -> 4, again 2^30 blocks apart): same tag (which covers every ciphertext byte) and the same
    bytes where sampled as with the 2^22 units of 16 KiB taken from the counter, which _run has
    compared with libcrypto"""
    rng = np.random.default_rng(workloads.BASE_SEED + 99)
    key = pgcm.expand_key(rng.integers(0, 256, 32, dtype=np.uint8))
    ivs = torch.from_numpy(rng.integers(0, 256, 12, dtype=np.uint8)).cuda()
    lens = np.array([length], np.uint64)
    span = 1 << 22
    spots = [0, span + 16, length // 2 - 5, length - span]
    got = []
    for unit in (0, 16 << 20):
        pgcm.set_unit_bytes(key, unit)
        tags = torch.zeros(16, dtype=torch.uint8, device="cuda")
        pgcm.encrypt_batch(key, ivs, None, None, [plain.data_ptr()], lens, [cipher.data_ptr()],
                           tags)
        torch.cuda.synchronize()
        got.append((tags.cpu(), [cipher[o:o + span].clone() for o in spots]))
    assert torch.equal(got[0][0], got[1][0])
    for a, b in zip(got[0][1], got[1][1]):
        assert torch.equal(a, b)
    # ... and what the large units wrote decrypts and verifies under the chosen unit
    pgcm.set_unit_bytes(key, 0)
    ok = torch.zeros(1, dtype=torch.uint8, device="cuda")
    pgcm.decrypt_verify_batch(key, ivs, None, None, [cipher.data_ptr()], lens,
                              [cipher.data_ptr()], got[1][0].cuda(), ok)
    torch.cuda.synchronize()
    assert int(ok.item()) == 1
    for off in range(0, length, 8 * PIECE):
        n = min(8 * PIECE, length - off)
        assert torch.equal(cipher[off:off + n], plain[off:off + n]), off
    key.free()


def test_chunk_that_crosses_4_gib():
    plan = pgcm.plan_units([5 * GIB + 16 * 7 + 3])
    assert int(plan["nunits"][0]) == 327681 and int(plan["final_power"][0]) == 25
    _run(5 * GIB + 16 * 7 + 3, 31, 20)


def test_chunk_of_the_maximum_length():
    """2^36 - 32 bytes: the last counter block is IV || 0xFFFFFFFF; one byte more is refused"""
    length = (1 << 36) - 32
    plan = pgcm.plan_units([length])
    assert int(plan["nunits"][0]) == 1 << 22 and int(plan["final_power"][0]) == 30
    assert int(plan["final_count"][0]) == 4
    plain, cipher = _run(length, 32, 0)
    _same_with_one_unit_per_wavefront(plain, cipher, length)
    key = pgcm.expand_key(np.zeros(32, np.uint8))
    ivs = torch.zeros(12, dtype=torch.uint8, device="cuda")
    tags = torch.zeros(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(pgcm.PgcmError) as e:
        pgcm.encrypt_batch(key, ivs, None, None, [plain.data_ptr()], [length + 1],
                           [cipher.data_ptr()], tags)
    assert e.value.status == -3
    key.free()
