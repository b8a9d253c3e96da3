"""The five configurations at full size, in the launch configuration bench.py times.

The oracle cannot hash gigabytes in a test, so each run is checked (a) bit for bit against the
oracle on sampled chunks (first, last, extremes of length, ragged, tampered), (b) on every chunk,
every ciphertext byte and every tag, against libcrypto (an independent implementation that the
oracle itself is pinned to), and (c) through properties that hold at any size: decryption of
the encryption is the identity, exactly the tampered chunks are rejected and wiped, bytes
between chunks are never touched."""
from concurrent.futures import ThreadPoolExecutor


import numpy as np
import pytest
import torch

import openssl_ref
import oracle
import workloads
from gpu_harness import DeviceBatch, apply_tampers

import paper_2411_03357_amd as pgcm

pytestmark = pytest.mark.gpu


def _sample(w, k_oracle=6):
    rng = np.random.default_rng(w.seed + 99)
    must = {0, w.n - 1, int(np.argmin(w.lens)), int(np.argmax(w.lens))}
    ragged = np.flatnonzero(w.lens % 16 != 0)
    if ragged.size:
        must |= {int(ragged[0]), int(ragged[-1])}
    must |= {t.chunk for t in w.tampers[:2]}
    extra = [int(i) for i in rng.permutation(w.n)[:k_oracle]]
    return sorted(must | set(extra[:max(0, k_oracle - len(must))]))


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


def _run_full(cfg):
    w = workloads.FULL[cfg]()
    key = pgcm.expand_key(w.key)
    b = DeviceBatch(w, w.payload_device())
    b.cipher.fill_(0xEE)
    b.encrypt(key)
    torch.cuda.synchronize()
    ora = _sample(w)
    tags = b.tags.cpu().numpy().reshape(-1, 16)

    # (a) oracle on sampled chunks
    srcs = [b.chunk_host(b.plain, i) for i in ora]
    aads = None if w.aad is None else [np.frombuffer(w.aad_of(i), np.uint8) for i in ora]
    cts, otags, _ = oracle.encrypt_batch(w.key, w.ivs[ora], aads, srcs, nthreads=16)
    for j, i in enumerate(ora):
        assert np.array_equal(b.chunk_host(b.cipher, i), cts[j]), "ciphertext, chunk %d" % i
        assert np.array_equal(tags[i], otags[j]), "tag, chunk %d" % i
    # (b) libcrypto on every chunk
    differs = _first_chunk_libcrypto_disagrees_with(w, b.plain.cpu().numpy(),
                                                    b.cipher.cpu().numpy(), tags)
    assert differs is None, "chunk %d: ciphertext or tag differs from libcrypto's" % differs
    # gaps between chunks untouched
    for i in ora:
        end = int(w.offsets[i] + w.lens[i])
        nxt = int(w.offsets[i + 1]) if i + 1 < w.n else w.total_bytes
        assert bool((b.cipher[end:nxt] == 0xEE).all())

    # (c) decrypt-verify with the configuration's tampering
    cipher_t, tags_t = b.cipher, b.tags.clone()
    apply_tampers(w, cipher_t, tags_t)
    b.back.fill_(0xDD)
    b.decrypt(key, src=cipher_t, tags=tags_t)
    torch.cuda.synchronize()
    ok = b.ok.cpu().numpy()
    bad = sorted({t.chunk for t in w.tampers})
    assert sorted(np.flatnonzero(ok == 0).tolist()) == bad
    assert int((ok == 1).sum()) == w.n - len(bad)
    expect = b.plain.clone()
    for i in bad:
        off, ln = int(w.offsets[i]), int(w.lens[i])
        expect[off:off + ln] = 0
    # compare chunk payloads only (gaps hold the fill value)
    same = (b.back == expect) | (b.back == 0xDD)
    mism = int((~same).sum())
    assert mism == 0, "%d plaintext bytes differ" % mism
    for i in ora:
        got = b.chunk_host(b.back, i)
        assert np.array_equal(got, b.chunk_host(expect, i)), i
        end = int(w.offsets[i] + w.lens[i])
        nxt = int(w.offsets[i + 1]) if i + 1 < w.n else w.total_bytes
        assert bool((b.back[end:nxt] == 0xDD).all())
    # oracle's verdict and output on the sampled chunks, tampered ones included
    srcs = [b.chunk_host(cipher_t, i) for i in ora]
    pts, ook, _ = oracle.decrypt_verify_batch(w.key, w.ivs[ora], aads, srcs,
                                              tags_t.cpu().numpy().reshape(-1, 16)[ora], 16)
    for j, i in enumerate(ora):
        assert ok[i] == ook[j], i
        assert np.array_equal(b.chunk_host(b.back, i), pts[j]), i
    key.free()


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_full_size_configuration(cfg):
    _run_full(cfg)
