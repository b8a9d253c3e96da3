"""The cipher beyond the paper's AES-256 / 96-bit-IV transport: 128- and 192-bit keys, IVs of other
lengths (SP 800-38D 7.1 step 2) and the 32-bit counter's wrap (6.2), GPU library against the CPU
oracle through the C ABI.  Tolerance: none, byte work."""
import numpy as np
import pytest
import torch

import iv_craft
import openssl_ref
import oracle
import workloads
from device_batch import DeviceBatch, expand
from test_gpu_parity import _full_parity

import paper_2411_03357_amd as pgcm

pytestmark = pytest.mark.gpu

FLIPS_RAGGED = [(13, 4094, 7, "ct"), (25, 0, 0, "ct"), (2, 15, 3, "tag"), (0, 0, 0, "tag")]
FLIPS_SMALL = [(0, 0, 0, "ct"), (12, 1023, 7, "ct"), (27, 8191, 0, "ct"), (1, 5, 1, "tag")]


@pytest.mark.parametrize("key_bytes,iv_bytes", [(16, 12), (24, 12), (16, 8), (24, 16), (32, 60),
                                                (32, 1), (16, 13), (24, 128)])
def test_key_and_iv_lengths_both_paths(key_bytes, iv_bytes):
    _full_parity(workloads.with_cipher(workloads.ragged_small(), key_bytes, iv_bytes),
                 flip=FLIPS_RAGGED)
    _full_parity(workloads.with_cipher(workloads.small_transfers(), key_bytes, iv_bytes),
                 flip=FLIPS_SMALL)


def test_iv_entry_points_with_96_bit_ivs_equal_the_plain_ones():
    for w in (workloads.ragged_small(), workloads.small_transfers()):
        _full_parity(w, iv_entry=True)


@pytest.mark.parametrize("key_bytes", [16, 24])
def test_shorter_keys_on_a_kv_swap_batch(key_bytes):
    """multi-unit chunks with a fold level, as in the headline workload, under the other keys"""
    _full_parity(workloads.with_cipher(workloads.mini(2), key_bytes, 12))


def test_counter_wrap_inside_chunks():
    """16-byte IVs solved for so that J0's counter field sits just below 2^32: the counter then
    wraps at a chosen block of the chunk (first block, inside a row of 64, across a row and across
    a 16 KiB unit) while the other 96 bits of the counter block stay put"""
    rng = np.random.default_rng(workloads.BASE_SEED + 77)
    for key_bytes in (32, 16):
        key = rng.integers(0, 256, key_bytes, dtype=np.uint8)
        h = openssl_ref.aes_ecb_block(key.tobytes(), bytes(16))
        # (blocks before the wrap, chunk length)
        cases = [(0, 100), (1, 64), (5, 5000), (63, 8192), (64, 8192), (70, 200 * 1024 + 3),
                 (1023, 64 * 1024), (1024, 64 * 1024 + 16), (3000, 300 * 1024 + 5), (2, 16),
                 (10, 170)]
        ivs = np.zeros((len(cases), 16), np.uint8)
        for i, (before, _) in enumerate(cases):
            # data block b uses counter field J0.ctr + 1 + b: it is 0 for b == before
            ctr = (2 ** 32 - 1 - before) % (2 ** 32)
            j0 = rng.integers(0, 256, 12, dtype=np.uint8).tobytes() + ctr.to_bytes(4, "big")
            ivs[i] = np.frombuffer(iv_craft.iv_for_j0(h, j0), np.uint8)
        lens = np.array([c[1] for c in cases], np.uint64)
        for pick, name in ((lens > 0, "bulk"), (lens <= 8192, "small")):
            sel = np.flatnonzero(pick)
            sub = lens[sel]
            offsets, total = workloads._layout(sub)
            w = workloads.Workload("wrap_%s_k%d" % (name, key_bytes), 5, key, ivs[sel], sub,
                                   offsets, total, "u8")
            _full_parity(w, flip=[(0, 0, 0, "ct")])
            # and against libcrypto, which the oracle's wrap is pinned to as well
            host = w.payload_host()
            k = expand(w)
            b = DeviceBatch(w, torch.from_numpy(host).cuda())
            b.encrypt(k)
            torch.cuda.synchronize()
            for i in range(w.n):
                ct, tag = openssl_ref.encrypt(key.tobytes(), w.ivs[i].tobytes(), b"",
                                              w.chunk(host, i).tobytes())
                assert b.chunk_host(b.cipher, i).tobytes() == ct, (w.name, i)
                assert b.tags[16 * i:16 * i + 16].cpu().numpy().tobytes() == tag, (w.name, i)
            k.free()


def test_lengths_the_cipher_does_not_have_are_errors():
    for n in (0, 15, 17, 31, 33, 64):
        with pytest.raises(pgcm.PgcmError) as e:
            pgcm.expand_key_bytes(bytes(n))
        assert e.value.status == -1
    w = workloads.config1(n=2, size=64)
    key = pgcm.expand_key(w.key)
    b = DeviceBatch(w, torch.from_numpy(w.payload_host()).cuda())
    b.iv_bytes = 0
    with pytest.raises(pgcm.PgcmError) as e:
        b.encrypt(key)
    assert e.value.status == -1
    with pytest.raises(pgcm.PgcmError) as e:
        b.decrypt(key)
    assert e.value.status == -1
    key.free()


@pytest.mark.parametrize("iv_bytes", [12, 16])
def test_several_keys_in_one_batch(iv_bytes):
    """every chunk names its key; groups of one key take the bulk or the small-transfer path on
    their own (key 3 only gets chunks of at most 8 KiB), ivs / tags / ok stay indexed by chunk"""
    w = workloads.with_cipher(workloads.ragged_small(), 32, iv_bytes)
    rng = np.random.default_rng(workloads.BASE_SEED + 99 + iv_bytes)
    raw_keys = [rng.integers(0, 256, kb, dtype=np.uint8) for kb in (32, 16, 24, 32, 16)]
    key_index = rng.integers(0, 3, w.n).astype(np.uint32)
    key_index[w.lens <= 8192] = rng.integers(0, 4, int((w.lens <= 8192).sum()))   # key 4: unused
    assert set(key_index.tolist()) == {0, 1, 2, 3}
    keys = [pgcm.expand_key_bytes(k) for k in raw_keys]
    host = w.payload_host()
    b = DeviceBatch(w, torch.from_numpy(host).cuda())
    b.cipher.fill_(0xEE)
    pgcm.encrypt_batch_keys(keys, key_index, b.ivs, iv_bytes, b.aad_ptrs, b.aad_lens,
                            b.ptrs(b.plain), b.lens, b.ptrs(b.cipher), b.tags)
    torch.cuda.synchronize()
    cipher = b.cipher.cpu().numpy()
    tags = b.tags.cpu().numpy().reshape(-1, 16)
    expect = np.full(w.total_bytes, 0xEE, np.uint8)
    for i in range(w.n):
        ct, tag = oracle.encrypt(raw_keys[key_index[i]], w.ivs[i], w.aad_of(i), w.chunk(host, i))
        off = int(w.offsets[i])
        expect[off:off + len(ct)] = np.frombuffer(ct, np.uint8)
        assert tags[i].tobytes() == tag, i
    assert np.array_equal(cipher, expect)

    # decrypt: one chunk tampered, one chunk given to the wrong key
    bad_ct, wrong_key = 14, 20
    cipher_t = b.cipher.clone()
    cipher_t[int(w.offsets[bad_ct]) + 7] ^= 0x20
    idx2 = key_index.copy()
    idx2[wrong_key] = (idx2[wrong_key] + 1) % 3
    b.back.fill_(0xDD)
    pgcm.decrypt_verify_batch_keys(keys, idx2, b.ivs, iv_bytes, b.aad_ptrs, b.aad_lens,
                                   b.ptrs(cipher_t), b.lens, b.ptrs(b.back), b.tags, b.ok)
    torch.cuda.synchronize()
    ok = b.ok.cpu().numpy()
    back = b.back.cpu().numpy()
    expect = np.full(w.total_bytes, 0xDD, np.uint8)
    for i in range(w.n):
        off, ln = int(w.offsets[i]), int(w.lens[i])
        good = i not in (bad_ct, wrong_key)
        assert ok[i] == (1 if good else 0), i
        expect[off:off + ln] = host[off:off + ln] if good else 0
    assert np.array_equal(back, expect)

    # argument errors: nothing may be enqueued, outputs stay as they are
    before = b.tags.clone()
    idx3 = key_index.copy()
    idx3[5] = len(keys)
    with pytest.raises(pgcm.PgcmError) as e:
        pgcm.encrypt_batch_keys(keys, idx3, b.ivs, iv_bytes, b.aad_ptrs, b.aad_lens,
                                b.ptrs(b.plain), b.lens, b.ptrs(b.cipher), b.tags)
    assert e.value.status == -1
    with pytest.raises(pgcm.PgcmError) as e:
        pgcm.encrypt_batch_keys([], key_index, b.ivs, iv_bytes, b.aad_ptrs, b.aad_lens,
                                b.ptrs(b.plain), b.lens, b.ptrs(b.cipher), b.tags)
    assert e.value.status == -1
    misaligned = b.ptrs(b.plain).copy()
    misaligned[w.n - 1] += 4     # the last chunk, in the last group: still nothing is enqueued
    b.tags.zero_()
    with pytest.raises(pgcm.PgcmError) as e:
        pgcm.encrypt_batch_keys(keys, key_index, b.ivs, iv_bytes, b.aad_ptrs, b.aad_lens,
                                misaligned, b.lens, b.ptrs(b.cipher), b.tags)
    assert e.value.status == -2
    torch.cuda.synchronize()
    assert not bool(b.tags.any())
    b.tags.copy_(before)
    for k in keys:
        k.free()
