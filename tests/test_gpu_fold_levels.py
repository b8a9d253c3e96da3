"""Chunks long enough to need two and three fold levels (more than 32^2 and 32^3 units of
16 KiB), with ragged ends so that every level has a short first group.

The 16 MiB+ chunk is checked against the oracle on every byte.  The oracle would need minutes for
the 512 MiB+ chunk, so that one is checked against libcrypto (an independent implementation the
oracle itself is pinned to) plus the round-trip identity."""
import numpy as np
import pytest
import torch

import openssl_ref
import oracle
import workloads
from device_batch import DeviceBatch

import paper_2411_03357_amd as pgcm

pytestmark = pytest.mark.gpu


def _workload(lens, seed_shift, aad_len):
    seed, rng, key, iv0 = workloads._base(7, seed_shift)
    lens = np.array(lens, np.uint64)
    offsets, total = workloads._layout(lens)
    aad = rng.integers(0, 256, aad_len * lens.size, dtype=np.uint8)
    aad_off = np.arange(lens.size + 1, dtype=np.uint64) * aad_len
    return workloads.Workload("fold_levels", seed, key, workloads.iv_sequence(iv0, lens.size),
                              lens, offsets, total, "u8", aad, aad_off)


def _levels(nunits):
    levels = 0
    while nunits > 32:
        nunits, levels = (nunits + 31) // 32, levels + 1
    return levels


@pytest.mark.parametrize("forced_unit,levels", [(None, 2), (16384, 2), (1024, 2), (32768, 1),
                                                (512 * 1024, 1), (16 << 20, 0)])
def test_fold_levels_against_the_oracle(forced_unit, levels):
    """a 16 MiB chunk: two fold levels with 16 KiB units (1025 sets -> 33, the first group short,
    -> 2), with the 8 KiB units a batch of this size gets by itself (2049 -> 65 -> 3) and with
    1 KiB units (16385 -> 513 -> 17); one with 32 KiB units (513 -> 17) and 512 KiB units
    (33 -> 2, the first group a single short unit); none with 16 MiB units (2 sets)"""
    unit = pgcm.unit_bytes()
    big = 1024 * unit + 3 * 16 + 5
    w = _workload([big, 33 * unit + 1, 40], 0, 20)
    auto = pgcm.batch_unit_bytes(w.lens)
    assert auto == 8192
    plan = pgcm.plan_units(w.lens)
    up = auto.bit_length() - 5                  # log2(blocks per unit)
    for i in range(2):
        nunits = -(-int(w.lens[i]) // auto)
        assert int(plan["nunits"][i]) == nunits
        assert int(plan["final_power"][i]) == up + 5 * _levels(nunits)
    use = forced_unit or auto
    assert _levels(-(-big // use)) == levels
    key = pgcm.expand_key(w.key)
    if forced_unit:
        pgcm.set_unit_bytes(key, forced_unit)
    b = DeviceBatch(w, w.payload_device())
    b.encrypt(key)
    b.decrypt(key)
    torch.cuda.synchronize()
    srcs = [b.chunk_host(b.plain, i) for i in range(w.n)]
    aads = [np.frombuffer(w.aad_of(i), np.uint8) for i in range(w.n)]
    cts, tags, _ = oracle.encrypt_batch(w.key, w.ivs, aads, srcs, nthreads=3)
    got = b.tags.cpu().numpy().reshape(-1, 16)
    for i in range(w.n):
        assert np.array_equal(b.chunk_host(b.cipher, i), cts[i]), i
        assert np.array_equal(got[i], tags[i]), i
    assert bool((b.ok == 1).all()) and torch.equal(b.back, b.plain)
    # a flipped bit deep inside the long chunk is noticed and the chunk wiped
    bad = b.cipher.clone()
    bad[int(w.offsets[0]) + 7 * 1024 * 1024 + 3] ^= 0x20
    b.decrypt(key, src=bad)
    torch.cuda.synchronize()
    assert b.ok.cpu().tolist() == [0, 1, 1]
    assert int(b.chunk_host(b.back, 0).max()) == 0
    assert np.array_equal(b.chunk_host(b.back, 1), srcs[1])
    key.free()


def test_one_forced_large_unit_per_wavefront_against_libcrypto():
    """4096 equal chunks of 20 KiB + 5 B are 8192 units of 16 KiB; with 32 KiB units forced
    every chunk is one short unit, every wavefront takes exactly one and nothing is handed out.
    Every chunk against libcrypto, a few against the oracle."""
    n, ln = 4096, 20 * 1024 + 5
    w = _workload([ln] * n, 2, 9)
    assert pgcm.batch_unit_bytes(w.lens) == 16384 and pgcm.plan_units(w.lens)["total"] == 2 * n
    key = pgcm.expand_key(w.key)
    pgcm.set_unit_bytes(key, 32768)
    b = DeviceBatch(w, w.payload_device())
    b.encrypt(key)
    b.decrypt(key)
    torch.cuda.synchronize()
    assert bool((b.ok == 1).all()) and torch.equal(b.back, b.plain)
    got = b.tags.cpu().numpy().reshape(-1, 16)
    kb = w.key.tobytes()
    for i in range(n):
        c, t = openssl_ref.encrypt(kb, w.ivs[i].tobytes(), w.aad_of(i),
                                   b.chunk_host(b.plain, i).tobytes())
        assert got[i].tobytes() == t, i
        assert b.chunk_host(b.cipher, i).tobytes() == c, i
    for i in (0, 1, 2047, n - 1):
        c, t = oracle.encrypt(w.key, w.ivs[i], np.frombuffer(w.aad_of(i), np.uint8),
                              b.chunk_host(b.plain, i))
        assert got[i].tobytes() == t and b.chunk_host(b.cipher, i).tobytes() == c, i
    # one flipped bit: that chunk alone is rejected and wiped
    bad = b.cipher.clone()
    bad[int(w.offsets[77]) + ln - 1] ^= 1
    b.decrypt(key, src=bad)
    torch.cuda.synchronize()
    ok = b.ok.cpu().numpy()
    assert int(ok[77]) == 0 and int(ok.sum()) == n - 1
    assert int(b.chunk_host(b.back, 77).max()) == 0
    assert np.array_equal(b.chunk_host(b.back, 78), b.chunk_host(b.plain, 78))
    key.free()


def test_three_fold_levels_against_libcrypto():
    unit = pgcm.unit_bytes()
    big = (32 * 32 * 32 + 40) * unit + 16 * 9 + 11      # 512 MiB + 640 KiB + ...
    w = _workload([big], 1, 13)
    assert pgcm.batch_unit_bytes(w.lens) == unit      # 512 MiB fills the chip with full units
    plan = pgcm.plan_units(w.lens)
    assert int(plan["final_power"][0]) == 25
    key = pgcm.expand_key(w.key)
    b = DeviceBatch(w, w.payload_device())
    b.encrypt(key)
    b.decrypt(key)
    torch.cuda.synchronize()
    assert bool((b.ok == 1).all()) and torch.equal(b.back, b.plain)
    pt = b.chunk_host(b.plain, 0).tobytes()
    c, t = openssl_ref.encrypt(w.key.tobytes(), w.ivs[0].tobytes(), w.aad_of(0), pt)
    assert b.tags.cpu().numpy().tobytes() == t
    assert b.chunk_host(b.cipher, 0).tobytes() == c
    key.free()
