/*
 * CPU oracle for bootstrapped TFHE binary gates (TEST INFRASTRUCTURE ONLY).
 *
 * This file is the slow, exact-integer statement of what the GPU library must
 * compute.  It exists so that tests, the smoke check and the benchmark's
 * cpu_baseline leg can compare against it; no product code path may call it,
 * link it or fall back to it.  It shares no source with the HIP library.
 *
 * What the paper fixes (SHE, arXiv 1906.00148): ciphertexts live on the torus
 * modulo 1 and the scheme is Ring-LWE based (Section 2, "TFHE"); every Boolean
 * operator of the network is a 2-input homomorphic gate (Section 3.1); a gate
 * in fully homomorphic mode needs a bootstrapping (Section 2, "Homomorphic
 * Encryption"); three sample levels TLWE / TRLWE / TRGSW exist (Section 4,
 * "TFHE setting").  The paper does not restate the gate bootstrapping itself;
 * it is the public construction it cites: TLWE linear combination, blind
 * rotation made of n CMux external products, sample extraction, key switch.
 * Every constant the paper leaves open (message encoding, rounding rules,
 * gadget offsets, key layouts, the random streams) is fixed here and must be
 * implemented identically, but independently, by the library.
 *
 * Arithmetic: Torus32 = uint32_t t standing for t / 2^32 in R/Z; everything is
 * exact arithmetic modulo 2^32.  The polynomial product is the schoolbook
 * negacyclic convolution, written out from its definition.
 *
 * Parity status: the ciphertext words themselves are "parity unpinned" by the
 * paper (it prints no ciphertext values).  Everything else is pinned by the
 * CPU tests: X^N = -1, brute-force products, gadget reconstruction, phase
 * identities, gate truth tables and the analytic noise bound.
 *
 * Leveled mode (Section 4, "TFHE setting": all three sample levels are used
 * without bootstrapping): fresh TRGSW samples of bits, TRLWE samples of torus
 * polynomials and the CMux  d0 + C [.] (d1 - d0)  built on the same external
 * product as the blind rotation.  Pinned by: selection of the right message,
 * the exact phase identity for a noiseless selector, and the noise bound.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    uint32_t n;          /* TLWE dimension */
    uint32_t N;          /* ring degree, power of two */
    uint32_t k;          /* TRLWE mask polynomials, must be 1 */
    uint32_t bg_bit;     /* log2 of gadget base Bg */
    uint32_t l;          /* gadget length */
    uint32_t ks_t;       /* key-switch digits */
    uint32_t ks_basebit; /* log2 of key-switch base */
    double lwe_std;      /* TLWE / key-switch noise, as a fraction of the torus */
    double bk_std;       /* bootstrapping-key noise */
} orc_params;

enum { ORC_NAND, ORC_AND, ORC_OR, ORC_XOR, ORC_XNOR, ORC_NOR, ORC_ANDNY, ORC_ANDYN, ORC_ORNY, ORC_ORYN,
       ORC_NGATES };
/* Three-input gates bootstrapped once: type = ORC_GATE3_BASE + 8*kind + negmask, kind 0 = majority,
 * kind 1 = parity (XOR of the three); bit i of negmask complements input i. */
enum { ORC_GATE3_BASE = 176, ORC_MAJ3 = 176, ORC_XOR3 = 184, ORC_GATE3_END = 192 };

enum { TAG_LWE_KEY = 1, TAG_RING_KEY = 2, TAG_BK_ROW = 3, TAG_KS_ROW = 4, TAG_FRESH = 5, TAG_TRGSW_ROW = 6,
       TAG_TRLWE = 7 };

/* ------------------------------------------------------------------------- */
/* Random streams.  One stream per object, addressed by (seed, tag, index);   */
/* word `ctr` of a stream is a pure function of those four numbers, so the    */
/* order in which objects are generated does not matter.                      */
/* ------------------------------------------------------------------------- */

static uint64_t mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

uint64_t orc_stream_key(uint64_t seed, uint64_t tag, uint64_t index)
{
    return mix64(mix64(mix64(seed) + tag) + index);
}

uint64_t orc_stream_word(uint64_t key, uint64_t ctr)
{
    return mix64(key + (ctr + 1) * 0x9E3779B97F4A7C15ull);
}

/* uniform Torus32 = top half of a stream word */
static uint32_t stream_torus(uint64_t key, uint64_t ctr) { return (uint32_t)(orc_stream_word(key, ctr) >> 32); }

/* key bit = top bit of a stream word */
static uint32_t stream_bit(uint64_t key, uint64_t ctr) { return (uint32_t)(orc_stream_word(key, ctr) >> 63); }

/* Gaussian torus error: Box-Muller (cosine branch) on two 53-bit uniforms taken
 * from words ctr and ctr+1, u1 in (0,1], u2 in [0,1); scaled by sigma*2^32 and
 * rounded to the nearest integer, reduced mod 2^32. */
uint32_t orc_gaussian32(uint64_t key, uint64_t ctr, double sigma)
{
    const double two_m53 = 1.0 / 9007199254740992.0;
    double u1 = (double)((orc_stream_word(key, ctr) >> 11) + 1) * two_m53;
    double u2 = (double)(orc_stream_word(key, ctr + 1) >> 11) * two_m53;
    double r = sqrt(-2.0 * log(u1));
    double z = r * cos(6.283185307179586476925286766559 * u2);
    double scaled = z * sigma;
    scaled = scaled * 4294967296.0;
    return (uint32_t)(int64_t)llround(scaled);
}

/* ------------------------------------------------------------------------- */
/* Ring arithmetic in Z_{2^32}[X]/(X^N+1)                                      */
/* ------------------------------------------------------------------------- */

/* c = a (*) b, negacyclic: c_m = sum_{i+j=m} a_i b_j - sum_{i+j=m+N} a_i b_j */
void orc_negacyclic_mul(uint32_t N, const uint32_t *a, const uint32_t *b, uint32_t *c)
{
    for (uint32_t m = 0; m < N; m++) c[m] = 0;
    for (size_t i = 0; i < N; i++) {
        const uint32_t ai = a[i];
        const uint32_t *bw = b + (N - i);     /* the b_j with i+j >= N                 */
        uint32_t *lo = c + i;
        for (size_t j = 0; j < N - i; j++) lo[j] += ai * b[j];     /* X^(i+j), i+j < N         */
        for (size_t m = 0; m < i; m++) c[m] -= ai * bw[m];         /* X^(i+j) = -X^(i+j-N)     */
    }
}

/* out = X^a * p for 0 <= a < 2N, using X^N = -1 */
void orc_mul_by_xpow(uint32_t N, uint32_t a, const uint32_t *p, uint32_t *out)
{
    for (uint32_t j = 0; j < N; j++) {
        uint32_t src = (j + 2 * N - a) % (2 * N);    /* exponent that lands on j, in [0,2N) */
        out[j] = (src < N) ? p[src] : (uint32_t)(0u - p[src - N]);
    }
}

/* ------------------------------------------------------------------------- */
/* Keys                                                                        */
/* ------------------------------------------------------------------------- */

static int params_ok(const orc_params *P)
{
    if (!P || P->k != 1) return 0;
    if (P->N < 2 || (P->N & (P->N - 1))) return 0;
    if (P->n < 1 || P->l < 1 || P->bg_bit < 1 || P->l * P->bg_bit > 31) return 0;
    if (P->ks_t < 1 || P->ks_basebit < 1 || P->ks_t * P->ks_basebit > 31) return 0;
    return 1;
}

size_t orc_bk_words(const orc_params *P) { return (size_t)P->n * 2 * P->l * 2 * P->N; }
size_t orc_ks_words(const orc_params *P)
{
    return (size_t)P->N * P->ks_t * ((1u << P->ks_basebit) - 1) * (P->n + 1);
}

/* TLWE sample of message mu under key s (n bits): a uniform, b = <a,s> + mu + e.
 * Stream layout: words 0..n-1 -> a_i, words n, n+1 -> the Gaussian. */
static void lwe_sample(uint32_t n, const uint8_t *s, uint32_t mu, double sigma, uint64_t key, uint32_t *out)
{
    uint32_t b = mu + orc_gaussian32(key, n, sigma);
    for (uint32_t i = 0; i < n; i++) {
        out[i] = stream_torus(key, i);
        if (s[i]) b += out[i];
    }
    out[n] = b;
}

/* Generates all key material.
 *  lwe_key[n], ring_key[N]: bits.
 *  bk: [i<n][c<2][p<l][comp<2][N]; row (c,p) of BK_i is a fresh TRLWE encryption
 *      of zero (comp 0 = mask A, comp 1 = body B = A (*) s' + E) to which
 *      s_i * 2^(32 - (p+1)*bg_bit) is added at coefficient 0 of component c.
 *  ks: [i<N][j<t][v-1<base-1][n+1]; TLWE under the LWE key of
 *      v * s'_i * 2^(32 - (j+1)*basebit), independent noise per row.           */
int orc_keygen(const orc_params *P, uint64_t seed, uint8_t *lwe_key, uint8_t *ring_key, uint32_t *bk, uint32_t *ks)
{
    if (!params_ok(P)) return -1;
    const uint32_t n = P->n, N = P->N, l = P->l;
    uint64_t kk = orc_stream_key(seed, TAG_LWE_KEY, 0);
    for (uint32_t i = 0; i < n; i++) lwe_key[i] = (uint8_t)stream_bit(kk, i);
    kk = orc_stream_key(seed, TAG_RING_KEY, 0);
    for (uint32_t j = 0; j < N; j++) ring_key[j] = (uint8_t)stream_bit(kk, j);

    uint32_t *sp = (uint32_t *)malloc(sizeof(uint32_t) * N);
    if (!sp) return -2;
    for (uint32_t j = 0; j < N; j++) sp[j] = ring_key[j];

    for (uint32_t i = 0; i < n; i++)
        for (uint32_t c = 0; c < 2; c++)
            for (uint32_t p = 0; p < l; p++) {
                uint64_t row = ((uint64_t)i * 2 + c) * l + p;
                uint64_t key = orc_stream_key(seed, TAG_BK_ROW, row);
                uint32_t *A = bk + row * 2 * N, *B = A + N;
                for (uint32_t j = 0; j < N; j++) A[j] = stream_torus(key, j);
                orc_negacyclic_mul(N, A, sp, B);
                for (uint32_t j = 0; j < N; j++) B[j] += orc_gaussian32(key, N + 2 * (uint64_t)j, P->bk_std);
                if (lwe_key[i]) (c == 0 ? A : B)[0] += 1u << (32 - (p + 1) * P->bg_bit);
            }
    free(sp);

    const uint32_t base = 1u << P->ks_basebit;
    for (uint32_t i = 0; i < N; i++)
        for (uint32_t j = 0; j < P->ks_t; j++)
            for (uint32_t v = 1; v < base; v++) {
                uint64_t row = ((uint64_t)i * P->ks_t + j) * (base - 1) + (v - 1);
                uint32_t mu = ring_key[i] ? v << (32 - (j + 1) * P->ks_basebit) : 0u;
                lwe_sample(n, lwe_key, mu, P->lwe_std, orc_stream_key(seed, TAG_KS_ROW, row), ks + row * (n + 1));
            }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Client side: bit k of a call is mu = +2^29 (bit 1) or -2^29 (bit 0),        */
/* noise stream (enc_seed, TAG_FRESH, k).                                      */
/* ------------------------------------------------------------------------- */

int orc_encrypt_bits(const orc_params *P, const uint8_t *lwe_key, const uint8_t *bits, size_t nbits,
                     uint64_t enc_seed, uint32_t *out /* [nbits][n+1] */)
{
    if (!params_ok(P)) return -1;
    for (size_t k = 0; k < nbits; k++) {
        uint32_t mu = bits[k] ? (1u << 29) : (uint32_t)(0u - (1u << 29));
        lwe_sample(P->n, lwe_key, mu, P->lwe_std, orc_stream_key(enc_seed, TAG_FRESH, k), out + k * (P->n + 1));
    }
    return 0;
}

/* phase = b - <a,s>, as a torus element */
uint32_t orc_lwe_phase(uint32_t n, const uint8_t *key, const uint32_t *ct)
{
    uint32_t ph = ct[n];
    for (uint32_t i = 0; i < n; i++) if (key[i]) ph -= ct[i];
    return ph;
}

int orc_decrypt_bits(const orc_params *P, const uint8_t *lwe_key, const uint32_t *cts, size_t count, uint8_t *bits)
{
    if (!params_ok(P)) return -1;
    for (size_t k = 0; k < count; k++)
        bits[k] = (int32_t)orc_lwe_phase(P->n, lwe_key, cts + k * (P->n + 1)) > 0;
    return 0;
}

/* phase polynomial of a TRLWE sample: B - A (*) s' */
void orc_trlwe_phase(uint32_t N, const uint8_t *ring_key, const uint32_t *acc /* [2][N] */, uint32_t *phase)
{
    uint32_t *sp = (uint32_t *)malloc(sizeof(uint32_t) * N);
    for (uint32_t j = 0; j < N; j++) sp[j] = ring_key[j];
    orc_negacyclic_mul(N, acc, sp, phase);
    for (uint32_t j = 0; j < N; j++) phase[j] = acc[N + j] - phase[j];
    free(sp);
}

/* ------------------------------------------------------------------------- */
/* Leveled mode: TRGSW selectors, TRLWE data, CMux                             */
/* ------------------------------------------------------------------------- */

/* Fresh TRGSW samples of bits under the ring key.  Sample k has the layout of
 * one BK_i, [c<2][p<l][comp<2][N]: row (c,p) is a TRLWE encryption of zero with
 * noise sigma, stream (seed, TAG_TRGSW_ROW, (k*2+c)*l+p) (words 0..N-1 the mask,
 * word N+2j the Gaussian of body coefficient j), plus bit*2^(32-(p+1)*bg_bit)
 * on coefficient 0 of component c. */
int orc_trgsw_encrypt_bits(const orc_params *P, const uint8_t *ring_key, const uint8_t *bits, size_t count,
                           uint64_t seed, double sigma, uint32_t *out /* [count][2][l][2][N] */)
{
    if (!params_ok(P)) return -1;
    const uint32_t N = P->N, l = P->l;
    uint32_t *sp = (uint32_t *)malloc(sizeof(uint32_t) * N);
    if (!sp) return -2;
    for (uint32_t j = 0; j < N; j++) sp[j] = ring_key[j];
    for (size_t k = 0; k < count; k++)
        for (uint32_t c = 0; c < 2; c++)
            for (uint32_t p = 0; p < l; p++) {
                uint64_t row = ((uint64_t)k * 2 + c) * l + p;
                uint64_t key = orc_stream_key(seed, TAG_TRGSW_ROW, row);
                uint32_t *A = out + row * 2 * N, *B = A + N;
                for (uint32_t j = 0; j < N; j++) A[j] = stream_torus(key, j);
                orc_negacyclic_mul(N, A, sp, B);
                for (uint32_t j = 0; j < N; j++) B[j] += orc_gaussian32(key, N + 2 * (uint64_t)j, sigma);
                if (bits[k]) (c == 0 ? A : B)[0] += 1u << (32 - (p + 1) * P->bg_bit);
            }
    free(sp);
    return 0;
}

/* Fresh TRLWE samples of torus polynomials mu_k: A uniform from stream
 * (seed, TAG_TRLWE, k) words 0..N-1, B = A (*) s' + mu + E with E_j from word N+2j. */
int orc_trlwe_encrypt(const orc_params *P, const uint8_t *ring_key, const uint32_t *mu /* [count][N] */, size_t count,
                      uint64_t seed, double sigma, uint32_t *out /* [count][2][N] */)
{
    if (!params_ok(P)) return -1;
    const uint32_t N = P->N;
    uint32_t *sp = (uint32_t *)malloc(sizeof(uint32_t) * N);
    if (!sp) return -2;
    for (uint32_t j = 0; j < N; j++) sp[j] = ring_key[j];
    for (size_t k = 0; k < count; k++) {
        uint64_t key = orc_stream_key(seed, TAG_TRLWE, k);
        uint32_t *A = out + k * 2 * N, *B = A + N;
        for (uint32_t j = 0; j < N; j++) A[j] = stream_torus(key, j);
        orc_negacyclic_mul(N, A, sp, B);
        for (uint32_t j = 0; j < N; j++) B[j] += mu[k * N + j] + orc_gaussian32(key, N + 2 * (uint64_t)j, sigma);
    }
    free(sp);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Gate = linear combination + bootstrap                                       */
/* ------------------------------------------------------------------------- */

/* Pre-bootstrap sample of each gate: (0, offset) + sa*ca + sb*cb, all of it
 * doubled for XOR/XNOR.  Offsets in units of 1/8 of the torus. */
int orc_gate_lincomb(uint32_t n, int type, const uint32_t *ca, const uint32_t *cb, uint32_t *out)
{
    const uint32_t e = 1u << 29; /* one eighth */
    uint32_t off; int sa, sb, dbl = 0;
    switch (type) {
    case ORC_AND:   off = 0u - e; sa = +1; sb = +1; break;
    case ORC_NAND:  off = e;      sa = -1; sb = -1; break;
    case ORC_OR:    off = e;      sa = +1; sb = +1; break;
    case ORC_NOR:   off = 0u - e; sa = -1; sb = -1; break;
    case ORC_XOR:   off = 2 * e;      sa = +1; sb = +1; dbl = 1; break;
    case ORC_XNOR:  off = 0u - 2 * e; sa = -1; sb = -1; dbl = 1; break;
    case ORC_ANDNY: off = 0u - e; sa = -1; sb = +1; break;   /* (not a) and b */
    case ORC_ANDYN: off = 0u - e; sa = +1; sb = -1; break;   /* a and (not b) */
    case ORC_ORNY:  off = e;      sa = -1; sb = +1; break;   /* (not a) or b */
    case ORC_ORYN:  off = e;      sa = +1; sb = -1; break;   /* a or (not b) */
    default: return -1;
    }
    for (uint32_t i = 0; i <= n; i++) {
        uint32_t x = (sa > 0 ? ca[i] : 0u - ca[i]) + (sb > 0 ? cb[i] : 0u - cb[i]);
        if (dbl) x *= 2u;
        out[i] = x;
    }
    out[n] += off;
    return 0;
}

/* Pre-bootstrap sample of a three-input gate (Section 3.1: the operators are built from homomorphic
 * gates; a gate is any linear combination whose phase has the wanted sign, followed by one bootstrap).
 * With inputs of phase +-1/8, s = sum_i (+-c_i) has phase (2k-3)/8 for k true (possibly complemented)
 * inputs: majority is the sign of s itself (margin 1/8), parity is the sign of -2s, whose phase is
 * +1/4 for odd k and -1/4 for even k modulo 1 (margin 1/4).  No offset is added. */
int orc_gate3_lincomb(uint32_t n, int type, const uint32_t *ca, const uint32_t *cb, const uint32_t *cc, uint32_t *out)
{
    if (type < ORC_GATE3_BASE || type >= ORC_GATE3_END) return -1;
    const int kind = (type - ORC_GATE3_BASE) >> 3, neg = (type - ORC_GATE3_BASE) & 7;
    for (uint32_t i = 0; i <= n; i++) {
        uint32_t x = ((neg & 1) ? 0u - ca[i] : ca[i]) + ((neg & 2) ? 0u - cb[i] : cb[i]) + ((neg & 4) ? 0u - cc[i] : cc[i]);
        out[i] = kind == 0 ? x : 0u - 2u * x;
    }
    return 0;
}

/* round a torus element to the nearest multiple of 1/(2N); result in [0,2N) */
uint32_t orc_modswitch(uint32_t N, uint32_t x)
{
    uint32_t L = 1; while ((1u << L) < 2 * N) L++;         /* 2N = 2^L */
    return (uint32_t)(x + (1u << (31 - L))) >> (32 - L);
}

/* Signed gadget digits of x: x is rounded to the nearest multiple of
 * 2^(32 - l*bg_bit) and written as sum_p d_p * 2^(32 - p*bg_bit), p=1..l,
 * with every d_p in [-Bg/2, Bg/2).  digits[p-1] = d_p. */
void orc_gadget_decompose(const orc_params *P, uint32_t x, int32_t *digits)
{
    const uint32_t Bg = 1u << P->bg_bit, half = Bg >> 1;
    uint32_t offset = 1u << (31 - P->l * P->bg_bit);       /* rounding of the dropped bits */
    for (uint32_t p = 1; p <= P->l; p++) offset += half << (32 - p * P->bg_bit);
    uint32_t y = x + offset;
    for (uint32_t p = 1; p <= P->l; p++)
        digits[p - 1] = (int32_t)((y >> (32 - p * P->bg_bit)) & (Bg - 1)) - (int32_t)half;
}

/* out = G [.] D where G = BK_i (2l rows x 2 comps x N) and D = (D_0, D_1):
 * out_comp = sum_{c<2} sum_{p<l} digit_{c,p}(X) (*) G[c][p][comp]             */
void orc_external_product(const orc_params *P, const uint32_t *G, const uint32_t *D, uint32_t *out /* [2][N] */)
{
    const uint32_t N = P->N, l = P->l;
    uint32_t *dig = (uint32_t *)malloc(sizeof(uint32_t) * N * l);
    uint32_t *prod = (uint32_t *)malloc(sizeof(uint32_t) * N);
    int32_t d[32];
    memset(out, 0, sizeof(uint32_t) * 2 * N);
    for (uint32_t c = 0; c < 2; c++) {
        for (uint32_t j = 0; j < N; j++) {
            orc_gadget_decompose(P, D[c * N + j], d);
            for (uint32_t p = 0; p < l; p++) dig[p * N + j] = (uint32_t)d[p];
        }
        for (uint32_t p = 0; p < l; p++)
            for (uint32_t comp = 0; comp < 2; comp++) {
                const uint32_t *row = G + (((size_t)c * l + p) * 2 + comp) * N;
                orc_negacyclic_mul(N, dig + p * N, row, prod);
                for (uint32_t j = 0; j < N; j++) out[comp * N + j] += prod[j];
            }
    }
    free(dig); free(prod);
}

/* CMux: out = d0 + C [.] (d1 - d0); encrypts the message of d1 if C encrypts 1, of d0 if 0.
 * C is one TRGSW sample [2][l][2][N], d1 / d0 / out are TRLWE samples [2][N] (out may alias neither). */
void orc_cmux(const orc_params *P, const uint32_t *C, const uint32_t *d1, const uint32_t *d0, uint32_t *out)
{
    const uint32_t N = P->N;
    uint32_t *D = (uint32_t *)malloc(sizeof(uint32_t) * 2 * N);
    for (uint32_t j = 0; j < 2 * N; j++) D[j] = d1[j] - d0[j];
    orc_external_product(P, C, D, out);
    for (uint32_t j = 0; j < 2 * N; j++) out[j] += d0[j];
    free(D);
}

/* ACC <- (0, X^(-bbar) * testv), testv = mu on every coefficient;
 * then for each i: ACC <- ACC + BK_i [.] ((X^abar_i - 1) * ACC).              */
void orc_blind_rotate(const orc_params *P, const uint32_t *bk, const uint32_t *abar, uint32_t bbar, uint32_t mu,
                      uint32_t *acc /* [2][N] */)
{
    const uint32_t N = P->N;
    uint32_t *tv = (uint32_t *)malloc(sizeof(uint32_t) * N);
    uint32_t *D = (uint32_t *)malloc(sizeof(uint32_t) * 2 * N);
    uint32_t *E = (uint32_t *)malloc(sizeof(uint32_t) * 2 * N);
    for (uint32_t j = 0; j < N; j++) { tv[j] = mu; acc[j] = 0; }
    orc_mul_by_xpow(N, (2 * N - bbar) % (2 * N), tv, acc + N);
    for (uint32_t i = 0; i < P->n; i++) {
        if (abar[i] == 0) continue;                         /* X^0 - 1 = 0: nothing to add */
        for (uint32_t c = 0; c < 2; c++) {
            orc_mul_by_xpow(N, abar[i], acc + c * N, D + c * N);
            for (uint32_t j = 0; j < N; j++) D[c * N + j] -= acc[c * N + j];
        }
        orc_external_product(P, bk + (size_t)i * 2 * P->l * 2 * N, D, E);
        for (uint32_t j = 0; j < 2 * N; j++) acc[j] += E[j];
    }
    free(tv); free(D); free(E);
}

/* TLWE of dimension N under the coefficients of s' whose phase is coefficient 0
 * of the TRLWE phase: a''_0 = A_0, a''_j = -A_{N-j}, b'' = B_0.               */
void orc_sample_extract(uint32_t N, const uint32_t *acc, uint32_t *ext /* [N+1] */)
{
    ext[0] = acc[0];
    for (uint32_t j = 1; j < N; j++) ext[j] = 0u - acc[N - j];
    ext[N] = acc[N];
}

/* out = (0, b'') - sum_{i<N} sum_{j<t} KS[i][j][d_ij], d_ij the base-2^basebit
 * digits (most significant first) of a''_i rounded to t*basebit bits.         */
void orc_key_switch(const orc_params *P, const uint32_t *ks, const uint32_t *ext, uint32_t *out /* [n+1] */)
{
    const uint32_t n = P->n, t = P->ks_t, bb = P->ks_basebit, base = 1u << bb;
    for (uint32_t c = 0; c < n; c++) out[c] = 0;
    out[n] = ext[P->N];
    for (uint32_t i = 0; i < P->N; i++) {
        uint32_t y = ext[i] + (1u << (31 - t * bb));
        for (uint32_t j = 0; j < t; j++) {
            uint32_t d = (y >> (32 - (j + 1) * bb)) & (base - 1);
            if (!d) continue;
            const uint32_t *row = ks + (((size_t)i * t + j) * (base - 1) + (d - 1)) * (n + 1);
            for (uint32_t c = 0; c <= n; c++) out[c] -= row[c];
        }
    }
}

/* Bootstrap of a TLWE sample to a fresh one of message +-2^29 (sign of phase). */
int orc_bootstrap(const orc_params *P, const uint32_t *bk, const uint32_t *ks, const uint32_t *in, uint32_t *out)
{
    if (!params_ok(P)) return -1;
    const uint32_t n = P->n, N = P->N;
    uint32_t *abar = (uint32_t *)malloc(sizeof(uint32_t) * n);
    uint32_t *acc = (uint32_t *)malloc(sizeof(uint32_t) * 2 * N);
    uint32_t *ext = (uint32_t *)malloc(sizeof(uint32_t) * (N + 1));
    for (uint32_t i = 0; i < n; i++) abar[i] = orc_modswitch(N, in[i]);
    orc_blind_rotate(P, bk, abar, orc_modswitch(N, in[n]), 1u << 29, acc);
    orc_sample_extract(N, acc, ext);
    orc_key_switch(P, ks, ext, out);
    free(abar); free(acc); free(ext);
    return 0;
}

int orc_gate(const orc_params *P, const uint32_t *bk, const uint32_t *ks, int type, const uint32_t *ca,
             const uint32_t *cb, uint32_t *out)
{
    if (!params_ok(P)) return -1;
    uint32_t *tmp = (uint32_t *)malloc(sizeof(uint32_t) * (P->n + 1));
    int rc = orc_gate_lincomb(P->n, type, ca, cb, tmp);
    if (rc == 0) rc = orc_bootstrap(P, bk, ks, tmp, out);
    free(tmp);
    return rc;
}

int orc_gate3(const orc_params *P, const uint32_t *bk, const uint32_t *ks, int type, const uint32_t *ca,
              const uint32_t *cb, const uint32_t *cc, uint32_t *out)
{
    if (!params_ok(P)) return -1;
    uint32_t *tmp = (uint32_t *)malloc(sizeof(uint32_t) * (P->n + 1));
    int rc = orc_gate3_lincomb(P->n, type, ca, cb, cc, tmp);
    if (rc == 0) rc = orc_bootstrap(P, bk, ks, tmp, out);
    free(tmp);
    return rc;
}

/* Blind rotation and extraction only: TLWE of dimension N under the ring key's coefficients. */
static void bootstrap_wo_keyswitch(const orc_params *P, const uint32_t *bk, const uint32_t *in, uint32_t *ext /* [N+1] */)
{
    const uint32_t n = P->n, N = P->N;
    uint32_t *abar = (uint32_t *)malloc(sizeof(uint32_t) * n);
    uint32_t *acc = (uint32_t *)malloc(sizeof(uint32_t) * 2 * N);
    for (uint32_t i = 0; i < n; i++) abar[i] = orc_modswitch(N, in[i]);
    orc_blind_rotate(P, bk, abar, orc_modswitch(N, in[n]), 1u << 29, acc);
    orc_sample_extract(N, acc, ext);
    free(abar); free(acc);
}

/* Native three-input MUX (Section 3.1 names MUX among the gates): out = sel ? c1 : c0 as
 * two blind rotations and ONE key switch.  The first rotation bootstraps code1(sel, c1), the
 * second code0(sel, c0), where for plain operands code1 = AND and code0 = ANDNY (not sel and c0);
 * a caller that wants a complemented operand passes the matching gate code instead (ANDYN, NOR,
 * ...).  At most one of the two is +1/8, so their sum plus 1/8 is +-1/8; it is key-switched once. */
int orc_mux(const orc_params *P, const uint32_t *bk, const uint32_t *ks, int code1, int code0, const uint32_t *sel,
            const uint32_t *c1, const uint32_t *c0, uint32_t *out)
{
    if (!params_ok(P)) return -1;
    const uint32_t n = P->n, N = P->N;
    uint32_t *t = (uint32_t *)malloc(sizeof(uint32_t) * (n + 1));
    uint32_t *e1 = (uint32_t *)malloc(sizeof(uint32_t) * (N + 1));
    uint32_t *e0 = (uint32_t *)malloc(sizeof(uint32_t) * (N + 1));
    int rc = orc_gate_lincomb(n, code1, sel, c1, t);
    if (rc == 0) {
        bootstrap_wo_keyswitch(P, bk, t, e1);
        rc = orc_gate_lincomb(n, code0, sel, c0, t);
    }
    if (rc == 0) {
        bootstrap_wo_keyswitch(P, bk, t, e0);
        for (uint32_t j = 0; j <= N; j++) e1[j] += e0[j];
        e1[N] += 1u << 29;
        orc_key_switch(P, ks, e1, out);
    }
    free(t); free(e1); free(e0);
    return rc;
}

/* A list of gates over a ciphertext pool pool[slot][n+1], evaluated in the
 * order given (so a netlist in topological order may be passed whole).  With
 * threads > 1 the gates must be mutually independent (one circuit level).
 * type[g] < ORC_NGATES: out = type(in0, in1).  type[g] = ORC_NGATES + 16*code1 + code0 (< ORC_GATE3_BASE):
 * native MUX with selector in0, operands in1 (taken when sel = 1) and in2.
 * type[g] >= ORC_GATE3_BASE: three-input gate of in0, in1, in2.                */
static int eval_one(const orc_params *P, const uint32_t *bk, const uint32_t *ks, uint32_t *pool, size_t w, uint32_t type,
                    uint32_t a, uint32_t b, uint32_t c, uint32_t o)
{
    if (type < ORC_NGATES) return orc_gate(P, bk, ks, (int)type, pool + a * w, pool + b * w, pool + o * w);
    if (type >= ORC_GATE3_BASE) return orc_gate3(P, bk, ks, (int)type, pool + a * w, pool + b * w, pool + c * w, pool + o * w);
    const uint32_t m = type - ORC_NGATES;
    return orc_mux(P, bk, ks, (int)(m >> 4), (int)(m & 15), pool + a * w, pool + b * w, pool + c * w, pool + o * w);
}

int orc_eval_netlist(const orc_params *P, const uint32_t *bk, const uint32_t *ks, uint32_t *pool, const uint32_t *type,
                     const uint32_t *in0, const uint32_t *in1, const uint32_t *in2, const uint32_t *outid,
                     size_t ngates, int threads)
{
    if (!params_ok(P)) return -1;
    const size_t w = P->n + 1;
    int bad = 0;
    if (threads <= 1) {
        for (size_t g = 0; g < ngates; g++)
            if (eval_one(P, bk, ks, pool, w, type[g], in0[g], in1[g], in2[g], outid[g])) bad = 1;
    } else {
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
        for (size_t g = 0; g < ngates; g++)
            if (eval_one(P, bk, ks, pool, w, type[g], in0[g], in1[g], in2[g], outid[g])) bad = 1;
    }
    return bad ? -1 : 0;
}

int orc_eval_gates(const orc_params *P, const uint32_t *bk, const uint32_t *ks, uint32_t *pool, const uint8_t *type,
                   const uint32_t *in0, const uint32_t *in1, const uint32_t *outid, size_t ngates, int threads)
{
    if (!params_ok(P)) return -1;
    const size_t w = P->n + 1;
    int bad = 0;
    if (threads <= 1) {
        for (size_t g = 0; g < ngates; g++)
            if (orc_gate(P, bk, ks, type[g], pool + in0[g] * w, pool + in1[g] * w, pool + outid[g] * w)) bad = 1;
    } else {
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
        for (size_t g = 0; g < ngates; g++)
            if (orc_gate(P, bk, ks, type[g], pool + in0[g] * w, pool + in1[g] * w, pool + outid[g] * w)) bad = 1;
    }
    return bad ? -1 : 0;
}
