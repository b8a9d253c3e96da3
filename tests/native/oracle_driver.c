/* Drives the C oracle under sanitizers: encrypts and decrypts messages of many lengths with all
 * three key lengths and several IV lengths, prints the tags for comparison with the normal
 * build, and checks round trips and rejection itself.  Test infrastructure. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int orc_gcm_encrypt_ex(const uint8_t *key, int key_bytes, const uint8_t *iv, uint64_t iv_bytes,
                       const uint8_t *aad, uint64_t alen, const uint8_t *pt, uint64_t len,
                       uint8_t *ct, uint8_t tag[16]);
int orc_gcm_decrypt_verify_ex(const uint8_t *key, int key_bytes, const uint8_t *iv,
                              uint64_t iv_bytes, const uint8_t *aad, uint64_t alen,
                              const uint8_t *ct, uint64_t len, const uint8_t tag[16], uint8_t *pt);

static uint32_t state = 2463534242u;
static uint8_t next_byte(void)
{
    state ^= state << 13;
    state ^= state >> 17;
    state ^= state << 5;
    return (uint8_t)(state >> 11);
}

int main(void)
{
    static const int key_lens[3] = {16, 24, 32};
    static const int iv_lens[5] = {12, 1, 8, 16, 60};
    static const int lens[12] = {0, 1, 15, 16, 17, 31, 32, 33, 100, 1023, 1024, 1025};
    for (int k = 0; k < 3; k++)
        for (int v = 0; v < 5; v++)
            for (int l = 0; l < 12; l++) {
                int len = lens[l], alen = (l * 7 + v) % 40;
                /* exact-size heap buffers, so that any access past an end is reported */
                uint8_t *key = malloc((size_t)key_lens[k]), *iv = malloc((size_t)iv_lens[v]);
                uint8_t *aad = malloc((size_t)alen + 1), *pt = malloc((size_t)len + 1);
                uint8_t *ct = malloc((size_t)len + 1), *back = malloc((size_t)len + 1);
                uint8_t tag[16];
                for (int i = 0; i < key_lens[k]; i++) key[i] = next_byte();
                for (int i = 0; i < iv_lens[v]; i++) iv[i] = next_byte();
                for (int i = 0; i < alen; i++) aad[i] = next_byte();
                for (int i = 0; i < len; i++) pt[i] = next_byte();
                /* the +1 bytes above only avoid zero-size allocations; shrink to exact sizes */
                aad = realloc(aad, alen ? (size_t)alen : 1);
                pt = realloc(pt, len ? (size_t)len : 1);
                ct = realloc(ct, len ? (size_t)len : 1);
                back = realloc(back, len ? (size_t)len : 1);
                if (!orc_gcm_encrypt_ex(key, key_lens[k], iv, (uint64_t)iv_lens[v], aad,
                                        (uint64_t)alen, pt, (uint64_t)len, ct, tag))
                    return 2;
                if (!orc_gcm_decrypt_verify_ex(key, key_lens[k], iv, (uint64_t)iv_lens[v], aad,
                                               (uint64_t)alen, ct, (uint64_t)len, tag, back) ||
                    memcmp(back, pt, (size_t)len) != 0)
                    return 3;
                tag[5] ^= 0x08;
                if (orc_gcm_decrypt_verify_ex(key, key_lens[k], iv, (uint64_t)iv_lens[v], aad,
                                              (uint64_t)alen, ct, (uint64_t)len, tag, back))
                    return 4;
                for (int i = 0; i < len; i++)
                    if (back[i] != 0) return 5;
                tag[5] ^= 0x08;
                printf("%d %d %d ", key_lens[k], iv_lens[v], len);
                for (int i = 0; i < 16; i++) printf("%02x", tag[i]);
                printf("\n");
                free(key), free(iv), free(aad), free(pt), free(ct), free(back);
            }
    return 0;
}
