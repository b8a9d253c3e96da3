"""Seeded random batches against libcrypto (which the oracle is pinned to): chunk counts, lengths
clustered around every boundary the scheduler has (blocks, 1 KiB rows, 1..16 KiB units, the 8 KiB
small-transfer limit), AAD lengths, key lengths and IV lengths are all drawn at random, so that
combinations nobody wrote down get compared byte for byte as well."""
import numpy as np
import pytest
import torch

import openssl_ref
import workloads
from device_batch import DeviceBatch, expand

import paper_2411_03357_amd as pgcm

pytestmark = pytest.mark.gpu


def _draw_length(rng):
    kind = rng.integers(0, 6)
    if kind == 0:
        return int(rng.integers(0, 70))
    if kind == 1:                       # around a multiple of a row
        return max(0, int(rng.integers(1, 40)) * 1024 + int(rng.integers(-17, 18)))
    if kind == 2:                       # around a multiple of some unit size
        unit = 1024 << int(rng.integers(0, 5))
        return max(0, int(rng.integers(1, 70)) * unit + int(rng.integers(-17, 18)))
    if kind == 3:                       # around the small-transfer limit
        return 8192 + int(rng.integers(-40, 41))
    if kind == 4:
        return int(np.exp(rng.uniform(np.log(16), np.log(4 << 20))))
    return int(rng.integers(0, 4)) * 16 + int(rng.integers(0, 3)) * 1024 * 16


def _random_workload(seed):
    rng = np.random.default_rng([workloads.BASE_SEED, 4242, seed])
    n = int(rng.integers(1, 48))
    if seed % 5 == 0:
        lens = [min(_draw_length(rng), 8192) for _ in range(n)]     # small-transfer path
    else:
        lens = [_draw_length(rng) for _ in range(n)]
    lens = np.array(lens, np.uint64)
    alens = [int(rng.integers(0, 81)) if rng.random() < 0.6 else 0 for _ in range(n)]
    offsets, total = workloads._layout(lens)
    aad_off = np.zeros(n + 1, np.uint64)
    aad_off[1:] = np.cumsum(alens)
    aad = rng.integers(0, 256, int(sum(alens)), dtype=np.uint8)
    key_bytes = int(rng.choice([16, 24, 32, 32]))
    iv_bytes = int(rng.choice([12, 12, 12, 8, 16, 1, 60]))
    w = workloads.Workload("random_%d" % seed, 900 + seed, np.zeros(32, np.uint8),
                           np.zeros((n, 12), np.uint8), lens, offsets, total, "u8", aad, aad_off)
    return workloads.with_cipher(w, key_bytes, iv_bytes), rng


@pytest.mark.parametrize("first_seed", [0, 12, 24, 36])
def test_random_batches_against_libcrypto(first_seed):
    for seed in range(first_seed, first_seed + 12):
        w, rng = _random_workload(seed)
        what = "seed %d: %d chunks, %d bytes, key %d, iv %d" % (
            seed, w.n, w.payload_bytes, w.key.size, w.ivs.shape[1])
        host = w.payload_host()
        key = expand(w)
        b = DeviceBatch(w, torch.from_numpy(host).cuda())
        b.cipher.fill_(0xEE)
        b.encrypt(key)
        torch.cuda.synchronize()
        cipher = b.cipher.cpu().numpy()
        tags = b.tags.cpu().numpy().reshape(-1, 16)
        expect = np.full(w.total_bytes, 0xEE, np.uint8)
        kb = w.key.tobytes()
        for i in range(w.n):
            ct, tag = openssl_ref.encrypt(kb, w.ivs[i].tobytes(), w.aad_of(i),
                                          w.chunk(host, i).tobytes())
            off = int(w.offsets[i])
            expect[off:off + len(ct)] = np.frombuffer(ct, np.uint8)
            assert tags[i].tobytes() == tag, "%s: tag of chunk %d (len %d)" % (what, i, w.lens[i])
        bad = np.flatnonzero(cipher != expect)
        assert bad.size == 0, "%s: ciphertext byte %d" % (what, bad[0])
        # tamper with one non-empty chunk (if there is one) and with one tag
        victims = set()
        nonempty = np.flatnonzero(w.lens > 0)
        cipher_t, tags_t = b.cipher.clone(), b.tags.clone()
        if nonempty.size:
            v = int(rng.choice(nonempty))
            cipher_t[int(w.offsets[v]) + int(rng.integers(0, int(w.lens[v])))] ^= 1 << int(
                rng.integers(0, 8))
            victims.add(v)
        v2 = int(rng.integers(0, w.n))
        tags_t[16 * v2 + int(rng.integers(0, 16))] ^= 1 << int(rng.integers(0, 8))
        victims.add(v2)
        b.back.fill_(0xDD)
        b.decrypt(key, src=cipher_t, tags=tags_t)
        torch.cuda.synchronize()
        ok = b.ok.cpu().numpy()
        back = b.back.cpu().numpy()
        expect = np.full(w.total_bytes, 0xDD, np.uint8)
        for i in range(w.n):
            off, ln = int(w.offsets[i]), int(w.lens[i])
            assert ok[i] == (0 if i in victims else 1), "%s: verdict of chunk %d" % (what, i)
            expect[off:off + ln] = 0 if i in victims else host[off:off + ln]
        bad = np.flatnonzero(back != expect)
        assert bad.size == 0, "%s: plaintext byte %d" % (what, bad[0])
        key.free()


def test_many_short_chunks():
    """more short multi-row chunks than the workgroup-per-chunk kernel is used for: the batch goes
    through the unit schedule, most chunks being a single short unit; and as many one-row chunks,
    which stay on the wavefront-per-chunk kernel"""
    for hi, seed in ((8192, 1), (1008, 2)):
        rng = np.random.default_rng([workloads.BASE_SEED, 777, seed])
        n = 700
        lens = rng.integers(0, hi + 1, n).astype(np.uint64)
        lens[:4] = [hi, 0, 1, hi - 1]
        alens = rng.integers(0, 30, n)
        offsets, total = workloads._layout(lens)
        aad_off = np.zeros(n + 1, np.uint64)
        aad_off[1:] = np.cumsum(alens)
        w = workloads.Workload("many_short_%d" % hi, 950 + seed,
                               rng.integers(0, 256, 32, dtype=np.uint8),
                               workloads.iv_sequence(int(rng.integers(1, 1 << 62)), n), lens,
                               offsets, total, "u8",
                               rng.integers(0, 256, int(alens.sum()), dtype=np.uint8), aad_off)
        host = w.payload_host()
        key = expand(w)
        b = DeviceBatch(w, torch.from_numpy(host).cuda())
        b.encrypt(key)
        bad_chunk = 123
        torch.cuda.synchronize()
        cipher = b.cipher.cpu().numpy()
        tags = b.tags.cpu().numpy().reshape(-1, 16)
        kb = w.key.tobytes()
        for i in range(n):
            ct, tag = openssl_ref.encrypt(kb, w.ivs[i].tobytes(), w.aad_of(i),
                                          w.chunk(host, i).tobytes())
            assert w.chunk(cipher, i).tobytes() == ct and tags[i].tobytes() == tag, (hi, i)
        b.tags[16 * bad_chunk + 3] ^= 0x40
        b.decrypt(key)
        torch.cuda.synchronize()
        ok = b.ok.cpu().numpy()
        assert [int(i) for i in np.flatnonzero(ok == 0)] == [bad_chunk]
        back = b.back.cpu().numpy()
        for i in range(n):
            expect = np.zeros(int(lens[i]), np.uint8) if i == bad_chunk else w.chunk(host, i)
            assert np.array_equal(w.chunk(back, i), expect), (hi, i)
        key.free()
