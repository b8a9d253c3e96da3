/*
 * AES-256-GCM oracle: test infrastructure, not product code.
 *
 * A plain, slow, byte-at-a-time AES-256 and bit-at-a-time GHASH written from
 * the public definitions (FIPS-197 for the block cipher, NIST SP 800-38D for
 * GCM).  It is what the paper's transport computes per transfer: one AES-GCM
 * invocation with a key and a unique IV (paper section 2.2, "A closer look at
 * NVIDIA CC"; section 4.1, "Swapping sequence and IVs"), with the receiver
 * rejecting anything that fails the integrity check (section 8.3).
 *
 * No tables beyond the S-box (which is computed from its definition at first
 * use), no blocking, no SIMD.  Only tests, the smoke check and the CPU-baseline
 * leg of the benchmark may call this; it shares nothing with the GPU library.
 */
#include <pthread.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* GF(2^8), reduction polynomial x^8 + x^4 + x^3 + x + 1 (FIPS-197 4.2) */

static uint8_t gf8_mul(uint8_t a, uint8_t b)
{
    uint8_t p = 0;
    for (int i = 0; i < 8; i++) {
        if (b & 1)
            p ^= a;
        uint8_t carry = a & 0x80;
        a = (uint8_t)(a << 1);
        if (carry)
            a ^= 0x1B;
        b >>= 1;
    }
    return p;
}

/* multiplicative inverse by exhaustive search; 0 maps to 0 (FIPS-197 5.1.1) */
static uint8_t gf8_inv(uint8_t a)
{
    if (a == 0)
        return 0;
    for (int c = 1; c < 256; c++)
        if (gf8_mul(a, (uint8_t)c) == 1)
            return (uint8_t)c;
    return 0; /* unreachable: every non-zero element has an inverse */
}

static uint8_t g_sbox[256];
static pthread_once_t g_sbox_once = PTHREAD_ONCE_INIT;

/* S(x) = affine(x^-1): b'_i = b_i ^ b_(i+4) ^ b_(i+5) ^ b_(i+6) ^ b_(i+7) ^ c_i,
 * indices mod 8, c = 0x63 (FIPS-197 5.1.1, eq. 5.1) */
static void sbox_build(void)
{
    for (int x = 0; x < 256; x++) {
        uint8_t b = gf8_inv((uint8_t)x);
        uint8_t out = 0;
        for (int i = 0; i < 8; i++) {
            int bit = ((b >> i) & 1) ^ ((b >> ((i + 4) % 8)) & 1) ^
                      ((b >> ((i + 5) % 8)) & 1) ^ ((b >> ((i + 6) % 8)) & 1) ^
                      ((b >> ((i + 7) % 8)) & 1) ^ ((0x63 >> i) & 1);
            out |= (uint8_t)(bit << i);
        }
        g_sbox[x] = out;
    }
}

static const uint8_t *sbox(void)
{
    pthread_once(&g_sbox_once, sbox_build);
    return g_sbox;
}

void orc_sbox(uint8_t out[256])
{
    memcpy(out, sbox(), 256);
}

/* ------------------------------------------------------------------ */
/* AES-256: Nk = 8 words, Nr = 14 rounds, 15 round keys (FIPS-197 5.2)  */

/* rk receives 60 words as 240 bytes, word i at rk[4i..4i+3] in key byte order */
void orc_aes256_key_expand(const uint8_t key[32], uint8_t rk[240])
{
    const uint8_t *S = sbox();
    memcpy(rk, key, 32);
    uint8_t rcon = 0x01;
    for (int i = 8; i < 60; i++) {
        uint8_t t[4];
        memcpy(t, rk + 4 * (i - 1), 4);
        if (i % 8 == 0) {
            /* RotWord then SubWord then Rcon on the first byte */
            uint8_t t0 = t[0];
            t[0] = S[t[1]] ^ rcon;
            t[1] = S[t[2]];
            t[2] = S[t[3]];
            t[3] = S[t0];
            rcon = gf8_mul(rcon, 2);
        } else if (i % 8 == 4) {
            for (int k = 0; k < 4; k++)
                t[k] = S[t[k]];
        }
        for (int k = 0; k < 4; k++)
            rk[4 * i + k] = rk[4 * (i - 8) + k] ^ t[k];
    }
}

/* state s[r][c] = in[r + 4c] (FIPS-197 3.4) */
void orc_aes256_encrypt_block(const uint8_t rk[240], const uint8_t in[16], uint8_t out[16])
{
    const uint8_t *S = sbox();
    uint8_t s[4][4];
    for (int c = 0; c < 4; c++)
        for (int r = 0; r < 4; r++)
            s[r][c] = in[r + 4 * c] ^ rk[r + 4 * c];

    for (int round = 1; round <= 14; round++) {
        /* SubBytes */
        for (int r = 0; r < 4; r++)
            for (int c = 0; c < 4; c++)
                s[r][c] = S[s[r][c]];
        /* ShiftRows: row r rotates left by r positions */
        for (int r = 1; r < 4; r++) {
            uint8_t row[4];
            for (int c = 0; c < 4; c++)
                row[c] = s[r][(c + r) % 4];
            for (int c = 0; c < 4; c++)
                s[r][c] = row[c];
        }
        /* MixColumns, skipped in the last round */
        if (round != 14) {
            for (int c = 0; c < 4; c++) {
                uint8_t a0 = s[0][c], a1 = s[1][c], a2 = s[2][c], a3 = s[3][c];
                s[0][c] = gf8_mul(a0, 2) ^ gf8_mul(a1, 3) ^ a2 ^ a3;
                s[1][c] = a0 ^ gf8_mul(a1, 2) ^ gf8_mul(a2, 3) ^ a3;
                s[2][c] = a0 ^ a1 ^ gf8_mul(a2, 2) ^ gf8_mul(a3, 3);
                s[3][c] = gf8_mul(a0, 3) ^ a1 ^ a2 ^ gf8_mul(a3, 2);
            }
        }
        /* AddRoundKey */
        for (int c = 0; c < 4; c++)
            for (int r = 0; r < 4; r++)
                s[r][c] ^= rk[16 * round + r + 4 * c];
    }
    for (int c = 0; c < 4; c++)
        for (int r = 0; r < 4; r++)
            out[r + 4 * c] = s[r][c];
}

/* ------------------------------------------------------------------ */
/* GF(2^128) as GCM defines it (SP 800-38D 6.3): a block is a bit string
 * whose bit 0 is the most significant bit of byte 0; the reduction constant
 * R is 11100001 followed by 120 zero bits.                              */

static int block_bit(const uint8_t b[16], int i)
{
    return (b[i / 8] >> (7 - (i % 8))) & 1;
}

void orc_gf128_mul(const uint8_t x[16], const uint8_t y[16], uint8_t z_out[16])
{
    uint8_t z[16] = {0};
    uint8_t v[16];
    memcpy(v, y, 16);
    for (int i = 0; i < 128; i++) {
        if (block_bit(x, i))
            for (int k = 0; k < 16; k++)
                z[k] ^= v[k];
        int lsb = v[15] & 1;
        /* shift the whole string one position toward bit 127 */
        for (int k = 15; k > 0; k--)
            v[k] = (uint8_t)((v[k] >> 1) | ((v[k - 1] & 1) << 7));
        v[0] >>= 1;
        if (lsb)
            v[0] ^= 0xE1;
    }
    memcpy(z_out, z, 16);
}

/* GHASH_H over nblocks complete blocks, continuing from y (SP 800-38D 6.4):
 * Y_i = (Y_{i-1} xor X_i) . H */
void orc_ghash_update(const uint8_t h[16], const uint8_t *x, size_t nblocks, uint8_t y[16])
{
    for (size_t i = 0; i < nblocks; i++) {
        uint8_t t[16];
        for (int k = 0; k < 16; k++)
            t[k] = y[k] ^ x[16 * i + k];
        orc_gf128_mul(t, h, y);
    }
}

/* absorbs a byte string, right-padding its last block with zeros */
static void ghash_padded(const uint8_t h[16], const uint8_t *data, uint64_t len, uint8_t y[16])
{
    uint64_t full = len / 16;
    orc_ghash_update(h, data, (size_t)full, y);
    if (len % 16) {
        uint8_t last[16] = {0};
        memcpy(last, data + 16 * full, (size_t)(len % 16));
        orc_ghash_update(h, last, 1, y);
    }
}

static void be64(uint64_t v, uint8_t out[8])
{
    for (int i = 0; i < 8; i++)
        out[i] = (uint8_t)(v >> (56 - 8 * i));
}

/* ------------------------------------------------------------------ */
/* GCM with a 96-bit IV (SP 800-38D 7.1, 7.2)                           */

/* counter block number j of the invocation: IV || [j]_32, big endian */
static void counter_block(const uint8_t iv[12], uint32_t j, uint8_t cb[16])
{
    memcpy(cb, iv, 12);
    cb[12] = (uint8_t)(j >> 24);
    cb[13] = (uint8_t)(j >> 16);
    cb[14] = (uint8_t)(j >> 8);
    cb[15] = (uint8_t)j;
}

/* out = in xor keystream, keystream block b (0-based) = E_K(IV || [b+2]_32) */
void orc_gctr(const uint8_t rk[240], const uint8_t iv[12], const uint8_t *in, uint64_t len,
              uint8_t *out)
{
    uint32_t ctr = 2;
    for (uint64_t off = 0; off < len; off += 16) {
        uint8_t cb[16], ks[16];
        counter_block(iv, ctr, cb);
        orc_aes256_encrypt_block(rk, cb, ks);
        uint64_t n = len - off < 16 ? len - off : 16;
        for (uint64_t k = 0; k < n; k++)
            out[off + k] = in[off + k] ^ ks[k];
        ctr++; /* inc32: wraps modulo 2^32 */
    }
}

/* T = GHASH_H(A || pad || C || pad || [8|A|]_64 || [8|C|]_64) xor E_K(IV || 0^31 1) */
static void gcm_tag(const uint8_t rk[240], const uint8_t iv[12], const uint8_t *aad, uint64_t alen,
                    const uint8_t *ct, uint64_t len, uint8_t tag[16])
{
    uint8_t zero[16] = {0}, h[16], y[16] = {0}, lens[16], j0[16], ekj0[16];
    orc_aes256_encrypt_block(rk, zero, h);
    ghash_padded(h, aad, alen, y);
    ghash_padded(h, ct, len, y);
    be64(8 * alen, lens);
    be64(8 * len, lens + 8);
    orc_ghash_update(h, lens, 1, y);
    counter_block(iv, 1, j0);
    orc_aes256_encrypt_block(rk, j0, ekj0);
    for (int k = 0; k < 16; k++)
        tag[k] = y[k] ^ ekj0[k];
}

void orc_gcm_encrypt(const uint8_t key[32], const uint8_t iv[12], const uint8_t *aad,
                     uint64_t alen, const uint8_t *pt, uint64_t len, uint8_t *ct, uint8_t tag[16])
{
    uint8_t rk[240];
    orc_aes256_key_expand(key, rk);
    orc_gctr(rk, iv, pt, len, ct);
    gcm_tag(rk, iv, aad, alen, ct, len, tag);
}

/* returns 1 and the plaintext when the tag matches; otherwise returns 0 and
 * writes len zero bytes: unauthenticated plaintext is never released */
int orc_gcm_decrypt_verify(const uint8_t key[32], const uint8_t iv[12], const uint8_t *aad,
                           uint64_t alen, const uint8_t *ct, uint64_t len, const uint8_t tag[16],
                           uint8_t *pt)
{
    uint8_t rk[240], expect[16];
    orc_aes256_key_expand(key, rk);
    gcm_tag(rk, iv, aad, alen, ct, len, expect);
    uint8_t diff = 0;
    for (int k = 0; k < 16; k++) /* all 16 bytes, no early exit */
        diff |= (uint8_t)(expect[k] ^ tag[k]);
    if (diff != 0) {
        memset(pt, 0, (size_t)len);
        return 0;
    }
    orc_gctr(rk, iv, ct, len, pt);
    return 1;
}

/* ------------------------------------------------------------------ */
/* Batches: chunks are independent invocations, handed to threads whole. */

typedef struct {
    int decrypt;
    const uint8_t *key;
    size_t n;
    const uint8_t *ivs;           /* n * 12 bytes */
    const uint8_t *const *aad;    /* may be NULL */
    const uint32_t *aad_len;      /* may be NULL */
    const uint8_t *const *src;
    const uint64_t *len;
    uint8_t *const *dst;
    uint8_t *tags;                /* n * 16 bytes: written (encrypt) or read (decrypt) */
    uint8_t *ok;                  /* decrypt only */
    size_t next;
    pthread_mutex_t lock;
} batch_job;

static void *batch_worker(void *arg)
{
    batch_job *job = (batch_job *)arg;
    for (;;) {
        pthread_mutex_lock(&job->lock);
        size_t i = job->next++;
        pthread_mutex_unlock(&job->lock);
        if (i >= job->n)
            return NULL;
        const uint8_t *a = job->aad_len ? job->aad[i] : NULL;
        uint64_t alen = job->aad_len ? job->aad_len[i] : 0;
        if (job->decrypt)
            job->ok[i] = (uint8_t)orc_gcm_decrypt_verify(job->key, job->ivs + 12 * i, a, alen,
                                                         job->src[i], job->len[i],
                                                         job->tags + 16 * i, job->dst[i]);
        else
            orc_gcm_encrypt(job->key, job->ivs + 12 * i, a, alen, job->src[i], job->len[i],
                            job->dst[i], job->tags + 16 * i);
    }
}

static int run_batch(batch_job *job, int nthreads)
{
    if (nthreads < 1)
        nthreads = 1;
    if ((size_t)nthreads > job->n)
        nthreads = job->n ? (int)job->n : 1;
    if (nthreads > 256)
        nthreads = 256;
    pthread_t tid[256];
    job->next = 0;
    pthread_mutex_init(&job->lock, NULL);
    int started = 0;
    for (int t = 1; t < nthreads; t++) {
        if (pthread_create(&tid[started], NULL, batch_worker, job) != 0)
            break;
        started++;
    }
    batch_worker(job);
    for (int t = 0; t < started; t++)
        pthread_join(tid[t], NULL);
    pthread_mutex_destroy(&job->lock);
    return started + 1; /* threads that actually worked */
}

int orc_gcm_encrypt_batch(const uint8_t key[32], size_t n, const uint8_t *ivs,
                          const uint8_t *const *aad, const uint32_t *aad_len,
                          const uint8_t *const *src, const uint64_t *len, uint8_t *const *dst,
                          uint8_t *tags, int nthreads)
{
    batch_job job = {0, key, n, ivs, aad, aad_len, src, len, dst, tags, NULL, 0,
                     PTHREAD_MUTEX_INITIALIZER};
    return run_batch(&job, nthreads);
}

int orc_gcm_decrypt_verify_batch(const uint8_t key[32], size_t n, const uint8_t *ivs,
                                 const uint8_t *const *aad, const uint32_t *aad_len,
                                 const uint8_t *const *src, const uint64_t *len,
                                 uint8_t *const *dst, const uint8_t *tags, uint8_t *ok,
                                 int nthreads)
{
    batch_job job = {1, key, n, ivs, aad, aad_len, src, len, dst, (uint8_t *)tags, ok, 0,
                     PTHREAD_MUTEX_INITIALIZER};
    return run_batch(&job, nthreads);
}
