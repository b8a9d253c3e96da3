"""One key object used by several host threads on several streams at once (the paper's transport
has one session key serving both directions, section 2.2): every thread's results are
bit-identical to the CPU oracle's; and pgcm_reserve, after which batches within the reserved
sizes leave the amount of free device memory unchanged."""
import threading

import numpy as np
import pytest
import torch

import oracle
import workloads
from device_batch import DeviceBatch

import paper_2411_03357_amd as pgcm

pytestmark = pytest.mark.gpu


def _oracle_results(w, host):
    srcs = [w.chunk(host, i) for i in range(w.n)]
    aads = None if w.aad is None else [np.frombuffer(w.aad_of(i), np.uint8) for i in range(w.n)]
    cts, tags, _ = oracle.encrypt_batch(w.key, w.ivs, aads, srcs, nthreads=8)
    return cts, tags


def test_two_threads_encrypt_and_decrypt_under_one_key_on_two_streams():
    # both directions of one session: thread A encrypts batch after batch (swap-out), thread B
    # decrypt-verifies other batches (swap-in), same key, a stream each, no lock around the calls
    wa, wb = workloads.mini(2), workloads.mini(4)
    wb.key = wa.key.copy()
    key = pgcm.expand_key(wa.key)
    ha, hb = wa.payload_host(), wb.payload_host()
    ba = DeviceBatch(wa, torch.from_numpy(ha).cuda())
    bb = DeviceBatch(wb, torch.from_numpy(hb).cuda())
    cts_a, tags_a = _oracle_results(wa, ha)
    cts_b, tags_b = _oracle_results(wb, hb)
    # thread B's input: the oracle's ciphertext and tags, one chunk damaged
    for i in range(wb.n):
        off = int(wb.offsets[i])
        bb.cipher[off:off + cts_b[i].size] = torch.from_numpy(cts_b[i]).cuda()
    bb.tags.copy_(torch.from_numpy(tags_b.reshape(-1)).cuda())
    victim = 5
    bb.cipher[int(wb.offsets[victim]) + 3] ^= 0x10
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    rounds, errors = 40, []
    barrier = threading.Barrier(2)

    def run_a():
        try:
            barrier.wait()
            for r in range(rounds):
                ba.encrypt(key, stream=streams[0])
                if r % 8 == 7:
                    streams[0].synchronize()
                    cipher = ba.cipher.cpu().numpy()
                    tags = ba.tags.cpu().numpy().reshape(-1, 16)
                    for i in range(wa.n):
                        assert np.array_equal(wa.chunk(cipher, i), cts_a[i]), ("A ct", r, i)
                    assert np.array_equal(tags, tags_a), ("A tags", r)
                    ba.cipher.zero_()
                    ba.tags.zero_()
                    torch.cuda.current_stream().synchronize()
        except Exception as e:   # noqa: BLE001 - handed to the main thread
            errors.append(e)

    def run_b():
        try:
            barrier.wait()
            for r in range(rounds):
                bb.decrypt(key, stream=streams[1])
                if r % 8 == 7:
                    streams[1].synchronize()
                    ok = bb.ok.cpu().numpy()
                    back = bb.back.cpu().numpy()
                    for i in range(wb.n):
                        assert ok[i] == (0 if i == victim else 1), ("B ok", r, i)
                        expect = np.zeros(int(wb.lens[i]), np.uint8) if i == victim \
                            else wb.chunk(hb, i)
                        assert np.array_equal(wb.chunk(back, i), expect), ("B pt", r, i)
                    bb.back.fill_(0x77)
                    bb.ok.fill_(0x55)
                    torch.cuda.current_stream().synchronize()
        except Exception as e:   # noqa: BLE001
            errors.append(e)

    ta, tb = threading.Thread(target=run_a), threading.Thread(target=run_b)
    ta.start(), tb.start()
    ta.join(), tb.join()
    torch.cuda.synchronize()
    if errors:
        raise errors[0]
    key.free()


def test_many_streams_share_and_rebind_contexts():
    """more streams than the key keeps contexts: a context whose last batch has ended is bound to
    the next stream that asks, and results stay exact"""
    w = workloads.mini(2)
    host = w.payload_host()
    key = pgcm.expand_key(w.key)
    cts, tags = _oracle_results(w, host)
    streams = [torch.cuda.Stream() for _ in range(24)]
    batches = [DeviceBatch(w, torch.from_numpy(host).cuda()) for _ in range(4)]
    for r, st in enumerate(streams * 2):
        b = batches[r % 4]
        b.encrypt(key, stream=st)
        if r % 4 == 3:
            torch.cuda.synchronize()
            for bb in batches:
                cipher = bb.cipher.cpu().numpy()
                for i in range(w.n):
                    assert np.array_equal(w.chunk(cipher, i), cts[i]), (r, i)
                assert np.array_equal(bb.tags.cpu().numpy().reshape(-1, 16), tags), r
                bb.cipher.zero_()
                bb.tags.zero_()
            torch.cuda.synchronize()
    key.free()


def test_reserve_then_batches_do_not_allocate():
    w = workloads.mini(3)                      # three 2 MiB chunks
    host = w.payload_host()
    key = pgcm.expand_key(w.key)
    b = DeviceBatch(w, torch.from_numpy(host).cuda())
    stream = torch.cuda.Stream()
    pgcm.reserve(key, w.n, w.payload_bytes, stream)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    for _ in range(6):
        b.encrypt(key, stream=stream)
        b.decrypt(key, stream=stream)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before
    cts, tags = _oracle_results(w, host)
    cipher = b.cipher.cpu().numpy()
    for i in range(w.n):
        assert np.array_equal(w.chunk(cipher, i), cts[i])
    assert np.array_equal(b.tags.cpu().numpy().reshape(-1, 16), tags)
    assert bool((b.ok == 1).all()) and torch.equal(b.back, b.plain)
    with pytest.raises(pgcm.PgcmError):
        pgcm.reserve(key, 1 << 40, 0, stream)
    key.free()
