/*
 * AES-GCM oracle (AES-128/192/256, any IV length): test infrastructure, not product code.
 *
 * A plain, slow, byte-at-a-time AES and bit-at-a-time GHASH written from
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
/* AES key expansion for Nk = 4, 6, 8 words: Nr = Nk + 6 rounds, Nr + 1 round keys
 * (FIPS-197 5.2).  The paper's transport uses Nk = 8.                     */

/* rk receives 4 (Nr + 1) words, word i at rk[4i..4i+3] in key byte order; returns Nr, or 0 when
 * key_bytes is not 16, 24 or 32 */
int orc_aes_key_expand(const uint8_t *key, int key_bytes, uint8_t rk[240])
{
    const uint8_t *S = sbox();
    if (key_bytes != 16 && key_bytes != 24 && key_bytes != 32)
        return 0;
    int nk = key_bytes / 4, nr = nk + 6;
    memcpy(rk, key, (size_t)key_bytes);
    uint8_t rcon = 0x01;
    for (int i = nk; i < 4 * (nr + 1); i++) {
        uint8_t t[4];
        memcpy(t, rk + 4 * (i - 1), 4);
        if (i % nk == 0) {
            /* RotWord then SubWord then Rcon on the first byte */
            uint8_t t0 = t[0];
            t[0] = S[t[1]] ^ rcon;
            t[1] = S[t[2]];
            t[2] = S[t[3]];
            t[3] = S[t0];
            rcon = gf8_mul(rcon, 2);
        } else if (nk > 6 && i % nk == 4) {
            for (int k = 0; k < 4; k++)
                t[k] = S[t[k]];
        }
        for (int k = 0; k < 4; k++)
            rk[4 * i + k] = rk[4 * (i - nk) + k] ^ t[k];
    }
    return nr;
}

void orc_aes256_key_expand(const uint8_t key[32], uint8_t rk[240])
{
    (void)orc_aes_key_expand(key, 32, rk);
}

/* state s[r][c] = in[r + 4c] (FIPS-197 3.4) */
void orc_aes_encrypt_block(const uint8_t rk[240], int nr, const uint8_t in[16], uint8_t out[16])
{
    const uint8_t *S = sbox();
    uint8_t s[4][4];
    for (int c = 0; c < 4; c++)
        for (int r = 0; r < 4; r++)
            s[r][c] = in[r + 4 * c] ^ rk[r + 4 * c];

    for (int round = 1; round <= nr; round++) {
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
        if (round != nr) {
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

void orc_aes256_encrypt_block(const uint8_t rk[240], const uint8_t in[16], uint8_t out[16])
{
    orc_aes_encrypt_block(rk, 14, in, out);
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
/* GCM (SP 800-38D 7.1, 7.2)                                             */

typedef struct {
    uint8_t rk[240];
    int nr;
    uint8_t h[16];
} gcm_key;

static int gcm_key_init(gcm_key *k, const uint8_t *key, int key_bytes)
{
    uint8_t zero[16] = {0};
    k->nr = orc_aes_key_expand(key, key_bytes, k->rk);
    if (k->nr == 0)
        return 0;
    orc_aes_encrypt_block(k->rk, k->nr, zero, k->h);
    return 1;
}

/* pre-counter block J0 (7.1 step 2): IV || 0^31 1 for a 96-bit IV, otherwise
 * GHASH_H(IV || 0-pad || 0^64 || [8 |IV|]_64) */
static void gcm_j0(const gcm_key *k, const uint8_t *iv, uint64_t iv_bytes, uint8_t j0[16])
{
    if (iv_bytes == 12) {
        memcpy(j0, iv, 12);
        j0[12] = 0, j0[13] = 0, j0[14] = 0, j0[15] = 1;
        return;
    }
    uint8_t lens[16] = {0};
    memset(j0, 0, 16);
    ghash_padded(k->h, iv, iv_bytes, j0);
    be64(8 * iv_bytes, lens + 8);
    orc_ghash_update(k->h, lens, 1, j0);
}

/* inc32^n: the last 32 bits of the block, as a big-endian integer, plus n modulo 2^32 */
static void counter_block(const uint8_t j0[16], uint32_t n, uint8_t cb[16])
{
    uint32_t c = ((uint32_t)j0[12] << 24) | ((uint32_t)j0[13] << 16) | ((uint32_t)j0[14] << 8) |
                 (uint32_t)j0[15];
    c += n; /* wraps modulo 2^32 */
    memcpy(cb, j0, 12);
    cb[12] = (uint8_t)(c >> 24);
    cb[13] = (uint8_t)(c >> 16);
    cb[14] = (uint8_t)(c >> 8);
    cb[15] = (uint8_t)c;
}

/* GCTR from inc32(J0): out = in xor keystream, keystream block b (0-based) = E_K(inc32^(b+1)(J0)) */
static void gctr(const gcm_key *k, const uint8_t j0[16], const uint8_t *in, uint64_t len,
                 uint8_t *out)
{
    uint32_t n = 1;
    for (uint64_t off = 0; off < len; off += 16) {
        uint8_t cb[16], ks[16];
        counter_block(j0, n, cb);
        orc_aes_encrypt_block(k->rk, k->nr, cb, ks);
        uint64_t m = len - off < 16 ? len - off : 16;
        for (uint64_t i = 0; i < m; i++)
            out[off + i] = in[off + i] ^ ks[i];
        n++;
    }
}

/* 96-bit IV form kept for the tests that exercise the keystream alone */
void orc_gctr(const uint8_t rk[240], const uint8_t iv[12], const uint8_t *in, uint64_t len,
              uint8_t *out)
{
    gcm_key k;
    uint8_t j0[16];
    memcpy(k.rk, rk, 240);
    k.nr = 14;
    memcpy(j0, iv, 12);
    j0[12] = 0, j0[13] = 0, j0[14] = 0, j0[15] = 1;
    gctr(&k, j0, in, len, out);
}

/* T = GHASH_H(A || pad || C || pad || [8|A|]_64 || [8|C|]_64) xor E_K(J0) */
static void gcm_tag(const gcm_key *k, const uint8_t j0[16], const uint8_t *aad, uint64_t alen,
                    const uint8_t *ct, uint64_t len, uint8_t tag[16])
{
    uint8_t y[16] = {0}, lens[16], ekj0[16];
    ghash_padded(k->h, aad, alen, y);
    ghash_padded(k->h, ct, len, y);
    be64(8 * alen, lens);
    be64(8 * len, lens + 8);
    orc_ghash_update(k->h, lens, 1, y);
    orc_aes_encrypt_block(k->rk, k->nr, j0, ekj0);
    for (int i = 0; i < 16; i++)
        tag[i] = y[i] ^ ekj0[i];
}

/* returns 0 for an unsupported key length or an empty IV, else 1 */
int orc_gcm_encrypt_ex(const uint8_t *key, int key_bytes, const uint8_t *iv, uint64_t iv_bytes,
                       const uint8_t *aad, uint64_t alen, const uint8_t *pt, uint64_t len,
                       uint8_t *ct, uint8_t tag[16])
{
    gcm_key k;
    uint8_t j0[16];
    if (!gcm_key_init(&k, key, key_bytes) || iv_bytes == 0)
        return 0;
    gcm_j0(&k, iv, iv_bytes, j0);
    gctr(&k, j0, pt, len, ct);
    gcm_tag(&k, j0, aad, alen, ct, len, tag);
    return 1;
}

/* returns 1 and the plaintext when the tag matches; otherwise returns 0 and
 * writes len zero bytes: unauthenticated plaintext is never released */
int orc_gcm_decrypt_verify_ex(const uint8_t *key, int key_bytes, const uint8_t *iv,
                              uint64_t iv_bytes, const uint8_t *aad, uint64_t alen,
                              const uint8_t *ct, uint64_t len, const uint8_t tag[16], uint8_t *pt)
{
    gcm_key k;
    uint8_t j0[16], expect[16];
    if (!gcm_key_init(&k, key, key_bytes) || iv_bytes == 0) {
        memset(pt, 0, (size_t)len);
        return 0;
    }
    gcm_j0(&k, iv, iv_bytes, j0);
    gcm_tag(&k, j0, aad, alen, ct, len, expect);
    uint8_t diff = 0;
    for (int i = 0; i < 16; i++) /* all 16 bytes, no early exit */
        diff |= (uint8_t)(expect[i] ^ tag[i]);
    if (diff != 0) {
        memset(pt, 0, (size_t)len);
        return 0;
    }
    gctr(&k, j0, ct, len, pt);
    return 1;
}

void orc_gcm_encrypt(const uint8_t key[32], const uint8_t iv[12], const uint8_t *aad,
                     uint64_t alen, const uint8_t *pt, uint64_t len, uint8_t *ct, uint8_t tag[16])
{
    (void)orc_gcm_encrypt_ex(key, 32, iv, 12, aad, alen, pt, len, ct, tag);
}

int orc_gcm_decrypt_verify(const uint8_t key[32], const uint8_t iv[12], const uint8_t *aad,
                           uint64_t alen, const uint8_t *ct, uint64_t len, const uint8_t tag[16],
                           uint8_t *pt)
{
    return orc_gcm_decrypt_verify_ex(key, 32, iv, 12, aad, alen, ct, len, tag, pt);
}

/* ------------------------------------------------------------------ */
/* Batches: chunks are independent invocations, handed to threads whole. */

typedef struct {
    int decrypt;
    const uint8_t *key;
    int key_bytes;
    uint64_t iv_bytes;
    size_t n;
    const uint8_t *ivs;           /* n * iv_bytes bytes */
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
        const uint8_t *iv = job->ivs + job->iv_bytes * i;
        if (job->decrypt)
            job->ok[i] = (uint8_t)orc_gcm_decrypt_verify_ex(job->key, job->key_bytes, iv,
                                                            job->iv_bytes, a, alen, job->src[i],
                                                            job->len[i], job->tags + 16 * i,
                                                            job->dst[i]);
        else
            (void)orc_gcm_encrypt_ex(job->key, job->key_bytes, iv, job->iv_bytes, a, alen,
                                     job->src[i], job->len[i], job->dst[i], job->tags + 16 * i);
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

int orc_gcm_encrypt_batch_ex(const uint8_t *key, int key_bytes, uint64_t iv_bytes, size_t n,
                             const uint8_t *ivs, const uint8_t *const *aad,
                             const uint32_t *aad_len, const uint8_t *const *src,
                             const uint64_t *len, uint8_t *const *dst, uint8_t *tags, int nthreads)
{
    batch_job job = {0, key, key_bytes, iv_bytes, n, ivs, aad, aad_len, src, len, dst, tags, NULL,
                     0, PTHREAD_MUTEX_INITIALIZER};
    return run_batch(&job, nthreads);
}

int orc_gcm_decrypt_verify_batch_ex(const uint8_t *key, int key_bytes, uint64_t iv_bytes, size_t n,
                                    const uint8_t *ivs, const uint8_t *const *aad,
                                    const uint32_t *aad_len, const uint8_t *const *src,
                                    const uint64_t *len, uint8_t *const *dst, const uint8_t *tags,
                                    uint8_t *ok, int nthreads)
{
    batch_job job = {1, key, key_bytes, iv_bytes, n, ivs, aad, aad_len, src, len, dst,
                     (uint8_t *)tags, ok, 0, PTHREAD_MUTEX_INITIALIZER};
    return run_batch(&job, nthreads);
}

int orc_gcm_encrypt_batch(const uint8_t key[32], size_t n, const uint8_t *ivs,
                          const uint8_t *const *aad, const uint32_t *aad_len,
                          const uint8_t *const *src, const uint64_t *len, uint8_t *const *dst,
                          uint8_t *tags, int nthreads)
{
    return orc_gcm_encrypt_batch_ex(key, 32, 12, n, ivs, aad, aad_len, src, len, dst, tags,
                                    nthreads);
}

int orc_gcm_decrypt_verify_batch(const uint8_t key[32], size_t n, const uint8_t *ivs,
                                 const uint8_t *const *aad, const uint32_t *aad_len,
                                 const uint8_t *const *src, const uint64_t *len,
                                 uint8_t *const *dst, const uint8_t *tags, uint8_t *ok,
                                 int nthreads)
{
    return orc_gcm_decrypt_verify_batch_ex(key, 32, 12, n, ivs, aad, aad_len, src, len, dst, tags,
                                           ok, nthreads);
}
