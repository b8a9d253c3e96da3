"""GPU library against the CPU oracle, element by element, through the C ABI.

Tolerance: none.  AES-GCM is exact integer/byte work, so ciphertext, tags, recovered plaintext
and verdicts must be bit-identical to the oracle's."""
import numpy as np
import pytest
import torch

import openssl_ref
import oracle
import workloads
from device_batch import DeviceBatch, apply_tampers, expand

import paper_2411_03357_amd as pgcm

pytestmark = pytest.mark.gpu

NTHREADS = 16


def _oracle_encrypt(w, host_buf, idx=None):
    idx = list(range(w.n)) if idx is None else idx
    srcs = [w.chunk(host_buf, i) for i in idx]
    aads = None if w.aad is None else [np.frombuffer(w.aad_of(i), np.uint8) for i in idx]
    cts, tags, _ = oracle.encrypt_batch(w.key, w.ivs[idx], aads, srcs, nthreads=NTHREADS)
    return cts, tags


def _full_parity(w, flip=None, iv_entry=None, unit_bytes=0, matrix_hash=False):
    """encrypt + decrypt-verify of the whole workload compared with the oracle on every byte;
    unit_bytes forces the scheduler's unit size (0: its own choice for the batch); matrix_hash
    sends the batch through the unit kernel with its row hash on the matrix cores"""
    host = w.payload_host()
    key = expand(w)
    pgcm.set_unit_bytes(key, unit_bytes)
    if matrix_hash:
        pgcm.set_matrix_hash(key, True)
        pgcm.set_one_launch(key, False)     # few chunks would otherwise skip the unit kernel
    b = DeviceBatch(w, torch.from_numpy(host).cuda(), iv_entry=iv_entry)
    b.cipher.fill_(0xEE)            # gaps between chunks must stay untouched
    b.encrypt(key)
    torch.cuda.synchronize()
    cts, tags = _oracle_encrypt(w, host)
    got_tags = b.tags.cpu().numpy().reshape(-1, 16)
    cipher_host = b.cipher.cpu().numpy()
    expect_buf = np.full(w.total_bytes, 0xEE, np.uint8)
    for i in range(w.n):
        off = int(w.offsets[i])
        expect_buf[off:off + cts[i].size] = cts[i]
    bad = np.flatnonzero(cipher_host != expect_buf)
    assert bad.size == 0, "%s: first ciphertext mismatch at byte %d" % (w.name, bad[0])
    assert np.array_equal(got_tags, tags), "%s: tag mismatch in chunks %s" % (
        w.name, np.flatnonzero((got_tags != tags).any(axis=1))[:8])

    # decrypt-verify, with the workload's tampering (and optional extra flips) applied
    cipher_t, tags_t = b.cipher.clone(), b.tags.clone()
    apply_tampers(w, cipher_t, tags_t)
    for (chunk, byte, bit, where) in (flip or []):
        if where == "ct":
            cipher_t[int(w.offsets[chunk]) + byte] ^= (1 << bit)
        else:
            tags_t[16 * chunk + byte] ^= (1 << bit)
    b.back.fill_(0xDD)
    b.decrypt(key, src=cipher_t, tags=tags_t)
    torch.cuda.synchronize()
    ct_host = cipher_t.cpu().numpy()
    srcs = [w.chunk(ct_host, i) for i in range(w.n)]
    aads = None if w.aad is None else [np.frombuffer(w.aad_of(i), np.uint8) for i in range(w.n)]
    pts, ok, _ = oracle.decrypt_verify_batch(w.key, w.ivs, aads, srcs,
                                             tags_t.cpu().numpy().reshape(-1, 16), NTHREADS)
    assert np.array_equal(b.ok.cpu().numpy(), ok), w.name
    back = b.back.cpu().numpy()
    expect_buf = np.full(w.total_bytes, 0xDD, np.uint8)
    for i in range(w.n):
        off = int(w.offsets[i])
        expect_buf[off:off + pts[i].size] = pts[i]
    bad = np.flatnonzero(back != expect_buf)
    assert bad.size == 0, "%s: first plaintext mismatch at byte %d" % (w.name, bad[0])
    tampered = {t.chunk for t in w.tampers} | {f[0] for f in (flip or [])}
    assert set(np.flatnonzero(ok == 0).tolist()) == tampered
    key.free()
    return b


def test_config1_full_parity():
    _full_parity(workloads.config1())


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_reduced_configs_full_parity(cfg):
    _full_parity(workloads.mini(cfg))


def test_ragged_edge_cases_full_parity():
    w = workloads.ragged_small()
    # reject a ragged chunk via its last byte, a multi-segment one via its first, one via its tag
    last = int(w.lens[13]) - 1
    _full_parity(w, flip=[(13, last, 7, "ct"), (25, 0, 0, "ct"), (2, 15, 3, "tag"),
                          (0, 0, 0, "tag")])


@pytest.mark.parametrize("unit_bytes", [1024, 2048, 4096, 8192, 16384, 32768, 128 * 1024,
                                        16 << 20])
def test_every_unit_size_full_parity(unit_bytes):
    """small batches get small units by themselves; here every unit size is forced on the
    edge-case batch and on a ragged mixed-size batch, so that unit boundaries, short first units
    and fold levels of each size are compared byte for byte"""
    w = workloads.ragged_small()
    last = int(w.lens[13]) - 1
    _full_parity(w, flip=[(13, last, 7, "ct"), (25, 0, 0, "ct"), (2, 15, 3, "tag")],
                 unit_bytes=unit_bytes)
    _full_parity(workloads.mini(4), unit_bytes=unit_bytes)
    key = pgcm.expand_key(w.key)
    for bad in (1, 512, 1000, 3000, 3 << 14, 1 << 25):
        with pytest.raises(pgcm.PgcmError) as e:
            pgcm.set_unit_bytes(key, bad)
        assert e.value.status == -1
    key.free()


@pytest.mark.parametrize("unit_bytes", [0, 1024, 16384, 128 * 1024])
def test_row_hash_on_matrix_cores_full_parity(unit_bytes):
    """The unit kernel's other engine for Y * H^64 (a GF(2) matrix product on the matrix cores
    instead of table lookups) on the same batches, byte for byte against the oracle: every length
    class, tampered chunks, the four KV / weight / mixed batch shapes, forced unit sizes, and the
    two shorter key lengths (other round counts are other kernels)."""
    w = workloads.ragged_small()
    last = int(w.lens[13]) - 1
    _full_parity(w, flip=[(13, last, 7, "ct"), (25, 0, 0, "ct"), (2, 15, 3, "tag")],
                 unit_bytes=unit_bytes or 2048, matrix_hash=True)
    for cfg in (2, 3, 4, 5):
        _full_parity(workloads.mini(cfg), unit_bytes=unit_bytes, matrix_hash=True)
    for key_bytes in (16, 24):
        _full_parity(workloads.with_cipher(workloads.mini(4), key_bytes, 12),
                     unit_bytes=unit_bytes, matrix_hash=True)


def test_small_transfer_path_full_parity():
    """batches made only of chunks of at most 8 KiB take the one-kernel path"""
    w = workloads.small_transfers()
    assert int(w.lens.max()) <= 8192
    _full_parity(w, flip=[(0, 0, 0, "ct"), (12, 1023, 7, "ct"), (27, 8191, 0, "ct"),
                          (1, 5, 1, "tag"), (20, 3, 2, "tag")])
    # a single 1-byte transfer (the paper's NOP) and a single empty one
    for n_bytes in (1, 0):
        w1 = workloads.config1(n=1, size=n_bytes)
        _full_parity(w1)


def test_small_transfer_path_in_place():
    w = workloads.small_transfers(seed_shift=2)
    host = w.payload_host()
    key = pgcm.expand_key(w.key)
    b = DeviceBatch(w, torch.from_numpy(host).cuda())
    work = b.plain.clone()
    b.encrypt(key, src=work, dst=work)
    b.decrypt(key, src=work, dst=work)
    torch.cuda.synchronize()
    assert torch.equal(work, b.plain) and bool((b.ok == 1).all())
    cts, tags = _oracle_encrypt(w, host)
    assert np.array_equal(b.tags.cpu().numpy().reshape(-1, 16), tags)
    key.free()


def test_no_aad_form_and_in_place():
    w = workloads.ragged_small(seed_shift=1)
    w.aad, w.aad_off = None, None
    host = w.payload_host()
    key = pgcm.expand_key(w.key)
    b = DeviceBatch(w, torch.from_numpy(host).cuda())
    work = b.plain.clone()
    b.encrypt(key, src=work, dst=work)          # in place
    torch.cuda.synchronize()
    cts, tags = _oracle_encrypt(w, host)
    wh = work.cpu().numpy()
    for i in range(w.n):
        assert np.array_equal(w.chunk(wh, i), cts[i]), i
    assert np.array_equal(b.tags.cpu().numpy().reshape(-1, 16), tags)
    b.decrypt(key, src=work, dst=work)
    torch.cuda.synchronize()
    assert torch.equal(work, b.plain)
    assert bool((b.ok == 1).all())
    key.free()


def test_against_libcrypto_on_device_generated_payload():
    w = workloads.mini(4)
    key = pgcm.expand_key(w.key)
    b = DeviceBatch(w, w.payload_device())
    b.encrypt(key)
    torch.cuda.synchronize()
    tags = b.tags.cpu().numpy().reshape(-1, 16)
    for i in range(w.n):
        c, t = openssl_ref.encrypt(w.key.tobytes(), w.ivs[i].tobytes(), w.aad_of(i),
                                   b.chunk_host(b.plain, i).tobytes())
        assert b.chunk_host(b.cipher, i).tobytes() == c and tags[i].tobytes() == t, i
    key.free()


def test_two_keys_and_back_to_back_batches_on_one_stream():
    """the descriptor staging buffers are reused from call to call; results must not mix"""
    w1, w2 = workloads.mini(1), workloads.config1(n=37, size=5000)
    h1, h2 = w1.payload_host(), w2.payload_host()
    k1 = pgcm.expand_key(w1.key)
    b1 = DeviceBatch(w1, torch.from_numpy(h1).cuda())
    b2 = DeviceBatch(w2, torch.from_numpy(h2).cuda())
    # same key object, different batches queued without synchronising in between
    w2.key = w1.key
    for _ in range(3):
        b1.encrypt(k1)
        b2.encrypt(k1)
        b1.decrypt(k1)
        b2.decrypt(k1)
    torch.cuda.synchronize()
    for w, h, b in ((w1, h1, b1), (w2, h2, b2)):
        cts, tags = _oracle_encrypt(w, h)
        ch = b.cipher.cpu().numpy()
        for i in range(w.n):
            assert np.array_equal(w.chunk(ch, i), cts[i])
        assert np.array_equal(b.tags.cpu().numpy().reshape(-1, 16), tags)
        assert bool((b.ok == 1).all())
        bh = b.back.cpu().numpy()
        for i in range(w.n):
            assert np.array_equal(w.chunk(bh, i), w.chunk(h, i))
    k1.free()


def test_two_keys_on_two_streams_at_once():
    """a key object belongs to one stream at a time, but two keys may run on two streams
    concurrently; the streams are ordinary torch streams of default priority"""
    wa, wb = workloads.mini(3), workloads.mini(4)
    wb.key = np.random.default_rng(3).integers(0, 256, 32, dtype=np.uint8)
    ha, hb = wa.payload_host(), wb.payload_host()
    ka, kb = pgcm.expand_key(wa.key), pgcm.expand_key(wb.key)
    ba = DeviceBatch(wa, torch.from_numpy(ha).cuda())
    bb = DeviceBatch(wb, torch.from_numpy(hb).cuda())
    torch.cuda.synchronize()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    for _ in range(4):
        ba.encrypt(ka, stream=sa)
        bb.encrypt(kb, stream=sb)
        ba.decrypt(ka, stream=sa)
        bb.decrypt(kb, stream=sb)
    sa.synchronize()
    sb.synchronize()
    for w, h, b in ((wa, ha, ba), (wb, hb, bb)):
        cts, tags = _oracle_encrypt(w, h)
        ch = b.cipher.cpu().numpy()
        for i in range(w.n):
            assert np.array_equal(w.chunk(ch, i), cts[i])
        assert np.array_equal(b.tags.cpu().numpy().reshape(-1, 16), tags)
        assert bool((b.ok == 1).all()) and torch.equal(b.back, b.plain)
    ka.free()
    kb.free()


@pytest.mark.parametrize("lens", [[0, 40, 1000], [0, 3000, 8192], [0, 5, 70000, 1 << 20]])
def test_long_aad_on_every_path(lens):
    """AAD of thousands of bytes (ragged, block-aligned, and 70 001 bytes) with chunks that take
    the one-row kernel, the workgroup-per-chunk kernel and the unit schedule; the empty chunk's
    AAD is hashed by the final step"""
    seed, rng, key, iv0 = workloads._base(11, len(lens))
    alens = [4099, 4096, 70001, 17][:len(lens)]
    la = np.array(lens, np.uint64)
    offsets, total = workloads._layout(la)
    aad_off = np.zeros(len(alens) + 1, np.uint64)
    aad_off[1:] = np.cumsum(alens)
    aad = rng.integers(0, 256, int(sum(alens)), dtype=np.uint8)
    w = workloads.Workload("long_aad", seed, key, workloads.iv_sequence(iv0, la.size), la, offsets,
                           total, "u8", aad, aad_off)
    last = len(lens) - 1
    _full_parity(w, flip=[(last, int(lens[last]) - 1, 0, "ct")])


def test_two_host_threads_each_with_its_key_and_stream():
    """the library keeps no state outside its key objects (the last HIP error is per thread):
    two host threads submit batches at the same time, each under its own key on its own stream"""
    import threading
    ws = [workloads.mini(3), workloads.mini(4)]
    ws[1].key = np.random.default_rng(5).integers(0, 256, 32, dtype=np.uint8)
    hosts = [w.payload_host() for w in ws]
    keys = [pgcm.expand_key(w.key) for w in ws]
    batches = [DeviceBatch(w, torch.from_numpy(h).cuda()) for w, h in zip(ws, hosts)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    errors = []
    start = threading.Barrier(2)

    def run(k):
        try:
            start.wait()
            for _ in range(25):
                batches[k].encrypt(keys[k], stream=streams[k])
                batches[k].decrypt(keys[k], stream=streams[k])
            streams[k].synchronize()
        except Exception as e:      # noqa: BLE001 - reported by the main thread
            errors.append((k, e))

    threads = [threading.Thread(target=run, args=(k,)) for k in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for w, h, b in zip(ws, hosts, batches):
        cts, tags = _oracle_encrypt(w, h)
        ch = b.cipher.cpu().numpy()
        for i in range(w.n):
            assert np.array_equal(w.chunk(ch, i), cts[i])
        assert np.array_equal(b.tags.cpu().numpy().reshape(-1, 16), tags)
        assert bool((b.ok == 1).all()) and torch.equal(b.back, b.plain)
    for k in keys:
        k.free()


def test_error_codes_and_empty_batch():
    w = workloads.config1(n=4, size=64)
    key = pgcm.expand_key(w.key)
    b = DeviceBatch(w, torch.from_numpy(w.payload_host()).cuda())
    before = b.cipher.clone()
    # empty batch: nothing happens
    pgcm.encrypt_batch(key, b.ivs, None, None, np.zeros(0, np.uint64), np.zeros(0, np.uint64),
                       np.zeros(0, np.uint64), b.tags)
    src, dst = b.ptrs(b.plain), b.ptrs(b.cipher)
    with pytest.raises(pgcm.PgcmError) as e:
        pgcm.encrypt_batch(key, b.ivs, None, None, src + np.uint64(4), b.lens, dst, b.tags)
    assert e.value.status == -2
    with pytest.raises(pgcm.PgcmError) as e:
        big = b.lens.copy()
        big[1] = (1 << 36) - 31
        pgcm.encrypt_batch(key, b.ivs, None, None, src, big, dst, b.tags)
    assert e.value.status == -3
    with pytest.raises(pgcm.PgcmError) as e:
        pgcm.encrypt_batch(key, b.ivs, None, np.zeros(4, np.uint32), src, b.lens, dst, b.tags)
    assert e.value.status == -1
    with pytest.raises(pgcm.PgcmError) as e:
        pgcm.encrypt_batch(key, None, None, None, src, b.lens, dst, b.tags)
    assert e.value.status == -1
    with pytest.raises(pgcm.PgcmError) as e:
        pgcm.decrypt_verify_batch(key, b.ivs, None, None, src, b.lens, dst, b.tags, None)
    assert e.value.status == -1
    torch.cuda.synchronize()
    assert torch.equal(b.cipher, before)        # failed calls enqueue nothing
    key.free()


def test_bulk_kernel_timing_history():
    w = workloads.mini(2)
    key = pgcm.expand_key(w.key)
    b = DeviceBatch(w, torch.from_numpy(w.payload_host()).cuda())
    with pytest.raises(pgcm.PgcmError):
        pgcm.last_bulk_kernel_ms(key)          # nothing timed yet
    assert pgcm.bulk_kernel_ms_history(key) == []
    pgcm.set_timing(key, True)
    for _ in range(5):
        b.encrypt(key)
        b.decrypt(key)
    hist = pgcm.bulk_kernel_ms_history(key)
    assert len(hist) == 10 and all(0.0 < t < 50.0 for t in hist)
    assert pgcm.bulk_kernel_ms_history(key, 3) == hist[-3:]
    assert pgcm.last_bulk_kernel_ms(key) == hist[-1]
    for _ in range(130):                       # more launches than the ring holds
        b.encrypt(key)
        b.decrypt(key)
    assert len(pgcm.bulk_kernel_ms_history(key, 1000)) == 256
    pgcm.set_timing(key, True)                 # switching on again forgets
    assert pgcm.bulk_kernel_ms_history(key) == []
    pgcm.set_timing(key, False)
    b.encrypt(key)
    assert pgcm.bulk_kernel_ms_history(key) == []
    torch.cuda.synchronize()
    assert bool((b.ok == 1).all()) and torch.equal(b.back, b.plain)
    key.free()
