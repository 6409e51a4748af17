/* Runs the C oracle's entry points once on a small parameter set; built with -fsanitize=address,undefined by
 * tests/test_sanitizers.py (CPU only).  Exit code 0 when every decrypted result is the plain gate; the sanitizers
 * abort the run on any out-of-bounds access, misaligned or overflowing signed arithmetic. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct { uint32_t n, N, k, bg_bit, l, ks_t, ks_basebit; double lwe_std, bk_std; } orc_params;
size_t orc_bk_words(const orc_params *P);
size_t orc_ks_words(const orc_params *P);
int orc_keygen(const orc_params *P, uint64_t seed, uint8_t *lwe_key, uint8_t *ring_key, uint32_t *bk, uint32_t *ks);
int orc_encrypt_bits(const orc_params *P, const uint8_t *lwe_key, const uint8_t *bits, size_t nbits, uint64_t enc_seed,
                     uint32_t *out);
int orc_decrypt_bits(const orc_params *P, const uint8_t *lwe_key, const uint32_t *cts, size_t count, uint8_t *bits);
int orc_gate(const orc_params *P, const uint32_t *bk, const uint32_t *ks, int type, const uint32_t *ca, const uint32_t *cb,
             uint32_t *out);
int orc_gate3(const orc_params *P, const uint32_t *bk, const uint32_t *ks, int type, const uint32_t *ca, const uint32_t *cb,
              const uint32_t *cc, uint32_t *out);
int orc_mux(const orc_params *P, const uint32_t *bk, const uint32_t *ks, int code1, int code0, const uint32_t *sel,
            const uint32_t *c1, const uint32_t *c0, uint32_t *out);
int orc_eval_gates(const orc_params *P, const uint32_t *bk, const uint32_t *ks, uint32_t *pool, const uint8_t *type,
                   const uint32_t *in0, const uint32_t *in1, const uint32_t *outid, size_t ngates, int threads);
int orc_trgsw_encrypt_bits(const orc_params *P, const uint8_t *ring_key, const uint8_t *bits, size_t count, uint64_t seed,
                           double sigma, uint32_t *out);
int orc_trlwe_encrypt(const orc_params *P, const uint8_t *ring_key, const uint32_t *mu, size_t count, uint64_t seed,
                      double sigma, uint32_t *out);
void orc_cmux(const orc_params *P, const uint32_t *C, const uint32_t *d1, const uint32_t *d0, uint32_t *out);
void orc_trlwe_phase(uint32_t N, const uint8_t *ring_key, const uint32_t *acc, uint32_t *phase);

static int plain2(int code, int a, int b)
{
    switch (code) {
    case 0: return !(a && b); case 1: return a && b; case 2: return a || b; case 3: return a ^ b; case 4: return !(a ^ b);
    case 5: return !(a || b); case 6: return !a && b; case 7: return a && !b; case 8: return !a || b; default: return a || !b;
    }
}

int main(void)
{
    const orc_params P = {24, 64, 1, 7, 3, 8, 2, 1.0 / 1048576.0, 1.0 / 1073741824.0};
    const size_t w = P.n + 1;
    uint8_t *lwe = malloc(P.n), *ring = malloc(P.N);
    uint32_t *bk = malloc(orc_bk_words(&P) * 4), *ks = malloc(orc_ks_words(&P) * 4);
    if (orc_keygen(&P, 99, lwe, ring, bk, ks)) return 2;
    const uint8_t bits[4] = {0, 1, 1, 0};
    uint32_t *cts = malloc(4 * w * 4), *out = malloc(w * 4);
    orc_encrypt_bits(&P, lwe, bits, 4, 5, cts);
    int bad = 0;
    uint8_t d;
    for (int code = 0; code < 10; code++)
        for (int a = 0; a < 2; a++)
            for (int b = 1; b < 3; b++) {
                if (orc_gate(&P, bk, ks, code, cts + (size_t)(a ? 1 : 0) * w, cts + (size_t)b * w, out)) return 2;
                orc_decrypt_bits(&P, lwe, out, 1, &d);
                bad += d != plain2(code, bits[a ? 1 : 0], bits[b]);
            }
    for (int mask = 0; mask < 8; mask++) {                      /* majority and parity, every complement mask */
        const int x = bits[0] ^ (mask & 1), y = bits[1] ^ ((mask >> 1) & 1), z = bits[2] ^ ((mask >> 2) & 1);
        orc_gate3(&P, bk, ks, 176 + mask, cts, cts + w, cts + 2 * w, out);
        orc_decrypt_bits(&P, lwe, out, 1, &d);
        bad += d != (x + y + z >= 2);
        orc_gate3(&P, bk, ks, 184 + mask, cts, cts + w, cts + 2 * w, out);
        orc_decrypt_bits(&P, lwe, out, 1, &d);
        bad += d != (x ^ y ^ z);
    }
    for (int s = 0; s < 2; s++) {                               /* native MUX: sel ? c1 : c0 */
        orc_mux(&P, bk, ks, 1, 6, cts + (size_t)s * w, cts + 2 * w, cts + 3 * w, out);
        orc_decrypt_bits(&P, lwe, out, 1, &d);
        bad += d != (bits[s] ? bits[2] : bits[3]);
    }
    /* a level through the pool interface, two threads */
    uint32_t *pool = calloc(8 * w, 4);
    memcpy(pool, cts, 4 * w * 4);
    const uint8_t ty[3] = {3, 1, 2};
    const uint32_t i0[3] = {0, 1, 2}, i1[3] = {1, 2, 3}, io[3] = {4, 5, 6};
    if (orc_eval_gates(&P, bk, ks, pool, ty, i0, i1, io, 3, 2)) return 2;
    uint8_t lev[3];
    orc_decrypt_bits(&P, lwe, pool + 4 * w, 3, lev);
    bad += lev[0] != 1 || lev[1] != 1 || lev[2] != 1;
    /* leveled mode: one CMux each way */
    uint32_t *sel = malloc((size_t)2 * 2 * P.l * 2 * P.N * 4), *mu = malloc((size_t)2 * P.N * 4);
    uint32_t *dat = malloc((size_t)2 * 2 * P.N * 4), *res = malloc((size_t)2 * P.N * 4), *ph = malloc((size_t)P.N * 4);
    const uint8_t sb[2] = {0, 1};
    orc_trgsw_encrypt_bits(&P, ring, sb, 2, 7, P.bk_std, sel);
    for (uint32_t j = 0; j < P.N; j++) { mu[j] = 1u << 29; mu[P.N + j] = 0u - (1u << 29); }
    orc_trlwe_encrypt(&P, ring, mu, 2, 8, P.bk_std, dat);
    for (int s = 0; s < 2; s++) {
        orc_cmux(&P, sel + (size_t)s * 2 * P.l * 2 * P.N, dat, dat + 2 * P.N, res);      /* sel ? d1 = +1/8 : d0 = -1/8 */
        orc_trlwe_phase(P.N, ring, res, ph);
        for (uint32_t j = 0; j < P.N; j++) bad += ((int32_t)ph[j] > 0) != (s == 1);
    }
    free(lwe); free(ring); free(bk); free(ks); free(cts); free(out); free(pool); free(sel); free(mu); free(dat); free(res); free(ph);
    printf("oracle under sanitizers: wrong results %d\n", bad);
    return bad ? 1 : 0;
}
