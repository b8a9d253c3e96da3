"""Ciphertext kept in pinned host memory: encrypt straight into a host bounce buffer, decrypt
straight out of it, so that a swap crosses PCIe once, as ciphertext (the placement the paper's
transport uses, section 6).  Same bit-exact bar as device-resident ciphertext."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from device_batch import DeviceBatch

import paper_2411_03357_amd as pgcm

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("which", ["ragged", "kv"])
def test_ciphertext_in_pinned_host_memory(which):
    w = workloads.ragged_small(seed_shift=3) if which == "ragged" else workloads.mini(2)
    host = w.payload_host()
    key = pgcm.expand_key(w.key)
    b = DeviceBatch(w, torch.from_numpy(host).cuda())
    bounce = torch.zeros(w.total_bytes, dtype=torch.uint8, pin_memory=True)
    b.encrypt(key, dst=bounce)
    torch.cuda.synchronize()
    srcs = [w.chunk(host, i) for i in range(w.n)]
    aads = [np.frombuffer(w.aad_of(i), np.uint8) for i in range(w.n)]
    cts, tags, _ = oracle.encrypt_batch(w.key, w.ivs, aads, srcs, nthreads=8)
    bn = bounce.numpy()
    for i in range(w.n):
        assert np.array_equal(w.chunk(bn, i), cts[i]), i
    assert np.array_equal(b.tags.cpu().numpy().reshape(-1, 16), tags)
    # tamper on the host side, then decrypt out of the bounce buffer
    victim = 5 if which == "ragged" else 3
    bn[int(w.offsets[victim])] ^= 1
    b.decrypt(key, src=bounce)
    torch.cuda.synchronize()
    ok = b.ok.cpu().numpy()
    assert [int(i) for i in np.flatnonzero(ok == 0)] == [victim]
    back = b.back.cpu().numpy()
    for i in range(w.n):
        expect = np.zeros_like(srcs[i]) if i == victim else srcs[i]
        assert np.array_equal(w.chunk(back, i), expect), i
    key.free()


def test_bounce_pool_streams_chunks_through_three_buffers():
    """ciphertext of ten chunks goes through a pool of three fixed-size pinned buffers: the
    encrypt kernel writes straight into the buffer, the host takes the ciphertext out when the
    pool hands the buffer out again (which waits for that kernel), and a second key object
    decrypts straight out of the buffers on the way back"""
    w = workloads.config1(n=10, size=300 * 1024 + 7)
    host = w.payload_host()
    key = pgcm.expand_key(w.key)
    plain = torch.from_numpy(host).cuda()
    b = DeviceBatch(w, plain)
    pool = pgcm.BouncePool(300 * 1024 + 7, 3)
    assert pool.count == 3 and pool.buffer_bytes == 300 * 1024 + 256
    in_flight = {}            # slot -> chunk whose ciphertext the buffer will hold
    wire = [None] * w.n       # ciphertext as taken off the buffers, by chunk

    def collect(slot, address):
        if slot in in_flight:
            i = in_flight.pop(slot)
            wire[i] = pool.view(address, int(w.lens[i])).copy()

    for i in range(w.n):
        address, slot = pool.acquire()          # waits for the kernel that last wrote this buffer
        collect(slot, address)
        one = np.array([i])
        pgcm.encrypt_batch(key, b.ivs[12 * i:12 * i + 12], None, None, b.ptrs(plain)[one],
                           b.lens[one], np.array([address], np.uint64), b.tags[16 * i:16 * i + 16])
        in_flight[slot] = i
        pool.release(slot)                      # free again once the stream has passed this point
    for _ in range(3):
        address, slot = pool.acquire()
        collect(slot, address)
        pool.release(slot)
    assert not in_flight and all(c is not None for c in wire)
    srcs = [w.chunk(host, i) for i in range(w.n)]
    cts, tags, _ = oracle.encrypt_batch(w.key, w.ivs, None, srcs, nthreads=8)
    for i in range(w.n):
        assert np.array_equal(wire[i], cts[i]), i
    assert np.array_equal(b.tags.cpu().numpy().reshape(-1, 16), tags)

    # the way back: ciphertext lands in a pool buffer, is decrypted straight out of it
    for i in range(w.n):
        address, slot = pool.acquire()
        pool.view(address, int(w.lens[i]))[:] = wire[i]
        if i == 6:
            pool.view(address, 1)[0] ^= 0x80    # damaged in transit
        one = np.array([i])
        pgcm.decrypt_verify_batch(key, b.ivs[12 * i:12 * i + 12], None, None,
                                  np.array([address], np.uint64), b.lens[one],
                                  b.ptrs(b.back)[one], b.tags[16 * i:16 * i + 16],
                                  b.ok[i:i + 1])
        pool.release(slot)
    torch.cuda.synchronize()
    assert b.ok.cpu().tolist() == [1] * 6 + [0] + [1] * 3
    back = b.back.cpu().numpy()
    for i in range(w.n):
        expect = np.zeros_like(srcs[i]) if i == 6 else srcs[i]
        assert np.array_equal(w.chunk(back, i), expect), i

    # holding every buffer is reported, not waited for; a slot is released once
    held = [pool.acquire() for _ in range(3)]
    with pytest.raises(pgcm.PgcmError) as e:
        pool.acquire()
    assert e.value.status == -6
    pool.release(held[0][1])
    with pytest.raises(pgcm.PgcmError) as e:
        pool.release(held[0][1])
    assert e.value.status == -1
    with pytest.raises(pgcm.PgcmError) as e:
        pool.release(99)
    assert e.value.status == -1
    address, slot = pool.acquire()
    assert slot == held[0][1]
    for _, s in held[1:] + [(address, slot)]:
        pool.release(s)
    pool.destroy()
    key.free()
