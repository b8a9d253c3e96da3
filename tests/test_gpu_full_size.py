"""The four large configurations at full size, in the launch configuration bench.py times,
compared with the CPU oracle on EVERY chunk, in both directions.

Encryption: every ciphertext byte and every tag of every chunk equals the oracle's; the bytes
between chunks keep their fill value.  Decryption with verification (with the configuration's
tampering applied to the ciphertext and tags): every verdict equals the oracle's, every output
byte of every chunk equals the oracle's (plaintext where authentic, zeros where rejected), and
the bytes between chunks keep their fill value.  Beside the oracle, libcrypto (an independent
implementation the oracle itself is pinned to) checks every ciphertext and tag once more.

The oracle is bit-serial by design (about 5 MB/s per core), so a direction of a configuration
takes between twenty seconds and a minute on sixteen host cores; it is fed in slices of a few
hundred megabytes and every slice reports on the terminal, so that a slow host shows progress
instead of silence."""
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import openssl_ref
import oracle
import workloads
from device_batch import DeviceBatch, apply_tampers

import paper_2411_03357_amd as pgcm

pytestmark = pytest.mark.gpu

ORACLE_THREADS = 16
SLICE_BYTES = 192 << 20
CIPHER_FILL, BACK_FILL = 0xEE, 0xDD


def _slices(w):
    """runs of consecutive chunks of about SLICE_BYTES of payload each"""
    out, lo, acc = [], 0, 0
    for i in range(w.n):
        acc += int(w.lens[i])
        if acc >= SLICE_BYTES or i + 1 == w.n:
            out.append((lo, i + 1))
            lo, acc = i + 1, 0
    return out


def _say(capsys, text):
    with capsys.disabled():
        print(text, flush=True)


def _aads(w, lo, hi):
    if w.aad is None:
        return None
    return [np.frombuffer(w.aad_of(i), np.uint8) for i in range(lo, hi)]


def _gaps_hold(w, host, fill):
    """every byte between chunks (alignment padding) still has the fill value"""
    ends = (w.offsets + w.lens).astype(np.int64)
    nxt = np.append(w.offsets[1:].astype(np.int64), w.total_bytes)
    for i in np.flatnonzero(nxt > ends):
        if not (host[int(ends[i]):int(nxt[i])] == fill).all():
            return int(i)
    return None


def _first_chunk_libcrypto_disagrees_with(w, plain, cipher, tags):
    """plain, cipher: host copies of the whole buffers; -> index of the first chunk whose
    ciphertext or tag differs from libcrypto's, or None"""
    kb = w.key.tobytes()

    def check(lo, hi):
        out = np.empty(int(w.lens[lo:hi].max()) if hi > lo else 0, np.uint8)
        for i in range(lo, hi):
            off, ln = int(w.offsets[i]), int(w.lens[i])
            st = openssl_ref.GcmEncryptStream(kb, w.ivs[i].tobytes(), w.aad_of(i))
            ref = st.update(plain[off:off + ln], out)
            if not np.array_equal(ref, cipher[off:off + ln]) or st.tag() != tags[i].tobytes():
                return i
        return None

    nthreads = 8   # libcrypto releases the interpreter lock inside its calls
    cuts = np.linspace(0, w.n, nthreads + 1).astype(int)
    with ThreadPoolExecutor(nthreads) as pool:
        found = list(pool.map(lambda k: check(int(cuts[k]), int(cuts[k + 1])), range(nthreads)))
    found = [i for i in found if i is not None]
    return min(found) if found else None


def _encrypt_on_gpu(w):
    key = pgcm.expand_key(w.key)
    b = DeviceBatch(w, w.payload_device())
    b.cipher.fill_(CIPHER_FILL)
    b.encrypt(key)
    torch.cuda.synchronize()
    return key, b


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_full_size_encrypt_every_chunk_against_the_oracle(cfg, capsys):
    w = workloads.FULL[cfg]()
    key, b = _encrypt_on_gpu(w)
    plain, cipher = b.plain.cpu().numpy(), b.cipher.cpu().numpy()
    tags = b.tags.cpu().numpy().reshape(-1, 16)
    key.free()
    t0 = time.time()
    for lo, hi in _slices(w):
        srcs = [w.chunk(plain, i) for i in range(lo, hi)]
        cts, otags, _ = oracle.encrypt_batch(w.key, w.ivs[lo:hi], _aads(w, lo, hi), srcs,
                                             nthreads=ORACLE_THREADS)
        for j, i in enumerate(range(lo, hi)):
            assert np.array_equal(w.chunk(cipher, i), cts[j]), "ciphertext, chunk %d" % i
            assert np.array_equal(tags[i], otags[j]), "tag, chunk %d" % i
        _say(capsys, "  config %d encrypt: chunks %d..%d of %d equal the oracle's (%.0f s)"
             % (cfg, lo, hi - 1, w.n, time.time() - t0))
    bad_gap = _gaps_hold(w, cipher, CIPHER_FILL)
    assert bad_gap is None, "bytes after chunk %d were written" % bad_gap
    differs = _first_chunk_libcrypto_disagrees_with(w, plain, cipher, tags)
    assert differs is None, "chunk %d: ciphertext or tag differs from libcrypto's" % differs


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_full_size_decrypt_verify_every_chunk_against_the_oracle(cfg, capsys):
    w = workloads.FULL[cfg]()
    key, b = _encrypt_on_gpu(w)   # its output is checked by the test above
    cipher_t, tags_t = b.cipher, b.tags.clone()
    apply_tampers(w, cipher_t, tags_t)
    b.back.fill_(BACK_FILL)
    b.decrypt(key, src=cipher_t, tags=tags_t)
    torch.cuda.synchronize()
    key.free()
    ok = b.ok.cpu().numpy()
    bad = sorted({t.chunk for t in w.tampers})
    assert sorted(np.flatnonzero(ok == 0).tolist()) == bad
    assert int((ok == 1).sum()) == w.n - len(bad)

    # the whole output buffer, exactly: plaintext where authentic, zeros where rejected, the
    # fill value between chunks
    expect = b.plain.clone()
    ends = (w.offsets + w.lens).astype(np.int64)
    nxt = np.append(w.offsets[1:].astype(np.int64), w.total_bytes)
    for i in np.flatnonzero(nxt > ends):
        expect[int(ends[i]):int(nxt[i])] = BACK_FILL
    for i in bad:
        off, ln = int(w.offsets[i]), int(w.lens[i])
        expect[off:off + ln] = 0
    mism = int((b.back != expect).sum())
    assert mism == 0, "%d output bytes differ from plaintext / zeros / fill" % mism
    del expect

    # ... and every chunk and verdict against the oracle's decryption of the same ciphertext
    cipher, back = cipher_t.cpu().numpy(), b.back.cpu().numpy()
    tags = tags_t.cpu().numpy().reshape(-1, 16)
    t0 = time.time()
    for lo, hi in _slices(w):
        srcs = [w.chunk(cipher, i) for i in range(lo, hi)]
        pts, ook, _ = oracle.decrypt_verify_batch(w.key, w.ivs[lo:hi], _aads(w, lo, hi), srcs,
                                                  tags[lo:hi], ORACLE_THREADS)
        for j, i in enumerate(range(lo, hi)):
            assert ok[i] == ook[j], "verdict, chunk %d" % i
            assert np.array_equal(w.chunk(back, i), pts[j]), "output, chunk %d" % i
        _say(capsys, "  config %d decrypt-verify: chunks %d..%d of %d equal the oracle's (%.0f s)"
             % (cfg, lo, hi - 1, w.n, time.time() - t0))
    bad_gap = _gaps_hold(w, back, BACK_FILL)
    assert bad_gap is None, "bytes after chunk %d were written" % bad_gap


@pytest.mark.parametrize("cfg", [2, 4])
def test_full_size_matrix_hash_engine(cfg):
    """The unit kernel's second engine for the row hash (GF(2) matrix product on the matrix cores)
    at full size.  It shares everything but the multiplication Y * H^64 with the table engine,
    whose output the tests above compare with the oracle chunk by chunk; here every ciphertext
    byte, tag, verdict and output byte must equal the table engine's on the same inputs, with
    the configuration's tampering (config 4 has none: three chunks are tampered with here), and
    every ciphertext and tag is checked against libcrypto as well."""
    w = workloads.FULL[cfg]()
    key, b = _encrypt_on_gpu(w)                       # table engine
    ref_cipher, ref_tags = b.cipher.clone(), b.tags.clone()
    pgcm.set_matrix_hash(key, True)
    b.cipher.fill_(CIPHER_FILL)
    b.tags.zero_()
    b.encrypt(key)
    torch.cuda.synchronize()
    assert torch.equal(b.cipher, ref_cipher) and torch.equal(b.tags, ref_tags)
    differs = _first_chunk_libcrypto_disagrees_with(
        w, b.plain.cpu().numpy(), b.cipher.cpu().numpy(), b.tags.cpu().numpy().reshape(-1, 16))
    assert differs is None, "chunk %d: ciphertext or tag differs from libcrypto's" % differs

    cipher_t, tags_t = ref_cipher, ref_tags.clone()
    rejected = [7, w.n // 2, w.n - 1]
    cipher_t[int(w.offsets[rejected[0]])] ^= 0x01                                   # first byte
    cipher_t[int(w.offsets[rejected[1]]) + int(w.lens[rejected[1]]) - 1] ^= 0x80    # last byte
    tags_t[16 * rejected[2] + 5] ^= 0x10
    outs = []
    for matrix in (False, True):
        pgcm.set_matrix_hash(key, matrix)
        b.back.fill_(BACK_FILL)
        b.ok.fill_(9)
        b.decrypt(key, src=cipher_t, tags=tags_t)
        torch.cuda.synchronize()
        outs.append((b.back.clone(), b.ok.clone()))
    key.free()
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    ok = outs[1][1].cpu().numpy()
    assert sorted(np.flatnonzero(ok == 0).tolist()) == rejected and int((ok == 1).sum()) == w.n - 3
    for i in rejected:
        off, ln = int(w.offsets[i]), int(w.lens[i])
        assert not bool(outs[1][0][off:off + ln].any())
    good = np.setdiff1d(np.arange(w.n), rejected)[:: max(1, w.n // 64)]
    for i in good:
        off, ln = int(w.offsets[i]), int(w.lens[i])
        assert torch.equal(outs[1][0][off:off + ln], b.plain[off:off + ln])
