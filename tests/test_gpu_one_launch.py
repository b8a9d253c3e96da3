"""Batches of few chunks that do not fill the chip are done by one kernel launch (the paper's
swaps come a few chunks at a time, section 5.1).  Every shape that path has — a chunk of one
unit, of one workgroup, of several workgroups whose sets the last one to arrive folds, runs of
1, 2, 4, 8 and 16 sets per wavefront, empty chunks, ragged ends, AAD, in place, each forced unit
size, decryption with rejected chunks — against the CPU oracle, bit for bit; and against the
sequence of kernels that larger batches take, which must give the same bytes."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from device_batch import DeviceBatch

import paper_2411_03357_amd as pgcm

pytestmark = pytest.mark.gpu

KIB, MIB = 1024, 1 << 20


def _workload(seed, lens, alens=None):
    rng = np.random.default_rng([workloads.BASE_SEED, 2718, seed])
    lens = np.array(lens, np.uint64)
    n = lens.size
    if alens is None:
        alens = [int(v) for v in rng.integers(0, 40, n)]
    offsets, total = workloads._layout(lens)
    aad_off = np.zeros(n + 1, np.uint64)
    aad_off[1:] = np.cumsum(alens)
    return workloads.Workload("one_launch_%d" % seed, 800 + seed,
                              rng.integers(0, 256, 32, dtype=np.uint8),
                              workloads.iv_sequence(int(rng.integers(1, 1 << 62)), n), lens,
                              offsets, total, "u8",
                              rng.integers(0, 256, int(np.sum(alens)), dtype=np.uint8), aad_off)


def _check_against_oracle(w, unit_bytes=0, tamper=()):
    host = w.payload_host()
    srcs = [w.chunk(host, i) for i in range(w.n)]
    aads = [np.frombuffer(w.aad_of(i), np.uint8) for i in range(w.n)]
    cts, tags, _ = oracle.encrypt_batch(w.key, w.ivs, aads, srcs, nthreads=16)
    results = {}
    for one_launch in (True, False):
        key = pgcm.expand_key(w.key)
        pgcm.set_one_launch(key, one_launch)
        pgcm.set_unit_bytes(key, unit_bytes)
        b = DeviceBatch(w, torch.from_numpy(host).cuda())
        b.cipher.fill_(0xEE)
        for _ in range(2):               # twice: the arrival words must be left clean
            b.tags.zero_()
            b.encrypt(key)
        torch.cuda.synchronize()
        cipher = b.cipher.cpu().numpy()
        expect = np.full(w.total_bytes, 0xEE, np.uint8)
        for i in range(w.n):
            off = int(w.offsets[i])
            expect[off:off + cts[i].size] = cts[i]
        bad = np.flatnonzero(cipher != expect)
        assert bad.size == 0, "%s one_launch=%s: ciphertext byte %d" % (w.name, one_launch, bad[0])
        got_tags = b.tags.cpu().numpy().reshape(-1, 16)
        for i in range(w.n):
            assert np.array_equal(got_tags[i], tags[i]), \
                "%s one_launch=%s: tag of chunk %d (len %d)" % (w.name, one_launch, i, w.lens[i])
        # decrypt-verify, some chunks damaged
        cipher_t, tags_t = b.cipher.clone(), b.tags.clone()
        for i in tamper:
            if int(w.lens[i]):
                cipher_t[int(w.offsets[i]) + int(w.lens[i]) // 2] ^= 0x04
            else:
                tags_t[16 * i + 7] ^= 0x80
        b.back.fill_(0xDD)
        b.decrypt(key, src=cipher_t, tags=tags_t)
        torch.cuda.synchronize()
        ok = b.ok.cpu().numpy()
        back = b.back.cpu().numpy()
        expect = np.full(w.total_bytes, 0xDD, np.uint8)
        for i in range(w.n):
            off, ln = int(w.offsets[i]), int(w.lens[i])
            assert ok[i] == (0 if i in tamper else 1), (w.name, one_launch, i)
            expect[off:off + ln] = 0 if i in tamper else host[off:off + ln]
        bad = np.flatnonzero(back != expect)
        assert bad.size == 0, "%s one_launch=%s: plaintext byte %d" % (w.name, one_launch, bad[0])
        # in place
        b.plain.copy_(torch.from_numpy(host).cuda())
        b.encrypt(key, dst=b.plain)
        torch.cuda.synchronize()
        inplace = b.plain.cpu().numpy()
        for i in range(w.n):
            assert np.array_equal(w.chunk(inplace, i), cts[i]), (w.name, one_launch, "in place", i)
        results[one_launch] = (cipher, got_tags)
        key.free()
    assert np.array_equal(results[True][0], results[False][0])
    assert np.array_equal(results[True][1], results[False][1])


def test_one_chunk_of_each_shape():
    # one unit (more than the 8 KiB of the short-transfer path); a few units in one workgroup;
    # exactly 16, 17, 32, 33 units; several workgroups; runs of 1 .. 16 sets per wavefront
    # (1 KiB units up to 4096 of them: 16 workgroups -> run 1, 256 -> run 16)
    for seed, ln in enumerate([8193, 9 * KIB, 16 * KIB, 16 * KIB + 1, 17 * KIB - 5, 32 * KIB,
                               33 * KIB + 7, 100 * KIB + 3, 320 * KIB, 512 * KIB + 9, MIB,
                               2 * MIB, 4 * MIB - 11, 4 * MIB]):
        _check_against_oracle(_workload(seed, [ln]))


def test_several_chunks_mixed():
    _check_against_oracle(_workload(30, [320 * KIB] * 4, [16] * 4), tamper=(2,))
    _check_against_oracle(_workload(31, [0, 2 * MIB, 1, 0, 9000, 320 * KIB + 5, 17, 100000],
                                    [5, 0, 0, 33, 64, 1, 0, 70]), tamper=(0, 1, 4))
    rng = np.random.default_rng(99)
    lens = [int(v) for v in np.exp(rng.uniform(np.log(1), np.log(300 * KIB), 24))]
    lens[3], lens[11] = 0, 150 * KIB
    _check_against_oracle(_workload(32, lens), tamper=(3, 11, 23))
    # 25 chunks: one more than the arguments hold, so the other kernels serve it
    _check_against_oracle(_workload(33, [40 * KIB] * 25))


@pytest.mark.parametrize("unit", [1024, 2048, 4096, 8192, 16384])
def test_forced_unit_sizes(unit):
    _check_against_oracle(_workload(40 + unit // 1024, [3 * MIB + 100, 0, 50 * KIB, 9 * KIB - 1]),
                          unit_bytes=unit, tamper=(1,))


def test_two_keys_alternate_on_one_stream_and_other_batches_in_between():
    """the arrival words live at the start of the context's workspace, where a batch of the
    other kind puts its descriptors: alternating the two kinds must keep both right"""
    small = _workload(50, [300 * KIB, 2 * MIB, 0, 11 * KIB])
    big = _workload(51, [64 * KIB] * 600)          # 600 chunks: the sequence of kernels
    hs, hb = small.payload_host(), big.payload_host()
    key = pgcm.expand_key(small.key)
    big.key = small.key.copy()
    bs = DeviceBatch(small, torch.from_numpy(hs).cuda())
    bb = DeviceBatch(big, torch.from_numpy(hb).cuda())
    for _ in range(3):
        bs.encrypt(key)
        bb.encrypt(key)
        bs.decrypt(key)
        bb.decrypt(key)
    torch.cuda.synchronize()
    assert bool((bs.ok == 1).all()) and torch.equal(bs.back, bs.plain)
    assert bool((bb.ok == 1).all()) and torch.equal(bb.back, bb.plain)
    for w, b, h in ((small, bs, hs), (big, bb, hb)):
        srcs = [w.chunk(h, i) for i in range(w.n)]
        aads = [np.frombuffer(w.aad_of(i), np.uint8) for i in range(w.n)]
        cts, tags, _ = oracle.encrypt_batch(w.key, w.ivs, aads, srcs, nthreads=16)
        cipher = b.cipher.cpu().numpy()
        for i in range(w.n):
            assert np.array_equal(w.chunk(cipher, i), cts[i]), (w.name, i)
        assert np.array_equal(b.tags.cpu().numpy().reshape(-1, 16), tags)
    key.free()
