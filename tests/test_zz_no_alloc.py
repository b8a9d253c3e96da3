"""pgcm_encrypt_batch_static, the entry point for callers that cannot allocate, against
pgcm_encrypt_batch on the same inputs: bit-identical ciphertext and tags (the bar every GPU
result here is held to), on calls in a row that share the static device workspace, the later
ones smaller than the first, with no host wait in between; and the limits it refuses."""
import numpy as np
import pytest
import torch

import workloads
from device_batch import DeviceBatch

import paper_2411_03357_amd as pgcm

pytestmark = pytest.mark.gpu

KIB, MIB = 1024, 1 << 20


def _workload(name, seed, lens, alens):
    rng = np.random.default_rng([workloads.BASE_SEED, 31337, seed])
    lens = np.array(lens, np.uint64)
    n = lens.size
    offsets, total = workloads._layout(lens)
    aad_off = np.zeros(n + 1, np.uint64)
    aad_off[1:] = np.cumsum(alens)
    return workloads.Workload(name, 700 + seed, rng.integers(0, 256, 32, dtype=np.uint8),
                              workloads.iv_sequence(int(rng.integers(1, 1 << 62)), n), lens,
                              offsets, total, "u8",
                              rng.integers(0, 256, int(np.sum(alens)), dtype=np.uint8), aad_off)


def _batches():
    rng = np.random.default_rng([workloads.BASE_SEED, 31337])
    # about 21 MB in 24 chunks: 8 KiB units, some 2600 partial sets and a fold level
    big = [0, 1, 3 * MIB + 5, 2 * MIB, 320 * KIB, 16 * KIB - 1, 8 * KIB + 1, 33 * 16 * KIB] + \
          [int(v) for v in rng.integers(1, 1400 * KIB, 16)]
    big_aad = [int(v) for v in rng.integers(0, 70, len(big))]
    # a smaller one right after it: 1 KiB units
    mid = [320 * KIB, 100 * KIB + 3, 0, 17, 64 * KIB]
    mid_aad = [16, 0, 5, 0, 33]
    # ... and one that takes the one-kernel path for short transfers (no device workspace)
    small = [1, 4096, 8192, 0, 1000]
    small_aad = [0, 0, 12, 7, 0]
    return [_workload("static_big", 1, big, big_aad), _workload("static_mid", 2, mid, mid_aad),
            _workload("static_small", 3, small, small_aad)]


def test_static_entry_point_equals_encrypt_batch_on_calls_in_a_row():
    ws = _batches()
    key = pgcm.expand_key(ws[0].key)
    stream = torch.cuda.current_stream()
    bs = [DeviceBatch(w, torch.from_numpy(w.payload_host()).cuda()) for w in ws]
    # what the existing entry point gives
    want = []
    for b in bs:
        b.cipher.fill_(0xEE)
        b.encrypt(key)
        torch.cuda.synchronize()
        want.append((b.cipher.clone(), b.tags.clone()))
        b.cipher.fill_(0xEE)
        b.tags.zero_()
    first_cipher, first_tags = torch.empty_like(bs[0].cipher), torch.empty_like(bs[0].tags)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    # the static entry point: three calls back to back on one stream, sharing its one workspace,
    # then the first (largest) once more over what the smaller ones left there
    order = [0, 1, 2, 0]
    got = []
    for k, i in enumerate(order):
        b = bs[i]
        if k == 3:
            torch.cuda.synchronize()
            first_cipher.copy_(b.cipher)                     # result of the first call
            first_tags.copy_(b.tags)
            got.append((first_cipher, first_tags))
            b.cipher.fill_(0xEE)
            b.tags.zero_()
        pgcm.encrypt_batch_static(key, b.ivs, b.aad_ptrs, b.aad_lens, b.ptrs(b.plain), b.lens,
                                  b.ptrs(b.cipher), b.tags, stream)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before, "device memory was allocated or freed"
    got += [(bs[1].cipher, bs[1].tags), (bs[2].cipher, bs[2].tags), (bs[0].cipher, bs[0].tags)]
    for k, i in enumerate(order):
        assert torch.equal(got[k][0], want[i][0]), "ciphertext of call %d (%s)" % (k, ws[i].name)
        assert torch.equal(got[k][1], want[i][1]), "tags of call %d (%s)" % (k, ws[i].name)
    # the receiver's side: the ordinary decrypt-verify accepts what the static call produced
    for b in bs:
        b.decrypt(key)
    torch.cuda.synchronize()
    for b in bs:
        assert bool((b.ok == 1).all()) and torch.equal(b.back, b.plain)
    key.free()


def test_static_entry_point_refuses_what_does_not_fit():
    key = pgcm.expand_key(bytes(range(32)))
    # more chunks than its descriptor staging holds
    n = pgcm.STATIC_MAX_CHUNKS + 1
    w = _workload("too_many", 4, [16] * n, [0] * n)
    b = DeviceBatch(w, torch.from_numpy(w.payload_host()).cuda())
    with pytest.raises(pgcm.PgcmError) as e:
        pgcm.encrypt_batch_static(key, b.ivs, None, None, b.ptrs(b.plain), b.lens,
                                  b.ptrs(b.cipher), b.tags)
    assert e.value.status == -7
    # more partial hash sums than its workspace holds: 160 MiB is 10240 units of 16 KiB, 10 MiB
    # of sets.  The lengths are all the host looks at before it refuses, so the pointers need not
    # be backed by that much memory.
    lens = np.array([160 * MIB], np.uint64)
    one = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    ptr = np.array([one.data_ptr()], np.uint64)
    with pytest.raises(pgcm.PgcmError) as e:
        pgcm.encrypt_batch_static(key, b.ivs, None, None, ptr, lens, ptr, b.tags)
    assert e.value.status == -7
    torch.cuda.synchronize()
    # nothing was enqueued or written
    assert bool((b.cipher == 0).all()) and bool((b.tags == 0).all())
    # ... and the ordinary call still serves the first batch
    b.encrypt(key)
    b.decrypt(key)
    torch.cuda.synchronize()
    assert bool((b.ok == 1).all()) and torch.equal(b.back, b.plain)
    key.free()
