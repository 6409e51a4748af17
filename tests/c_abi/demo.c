/* A client of the C ABI in plain C (no Python, no torch): key generation, bit-by-bit encryption of two
 * 4-bit numbers, one level of gates, a shift-accumulation, ReLU, decryption.  Exit code 0 when every
 * decrypted result equals the plain computation.  Built and run by tests/test_gpu_c_abi.py. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "she.h"

#define CHECK(call)                                                                                  \
    do {                                                                                             \
        int rc_ = (call);                                                                            \
        if (rc_ != SHE_OK) {                                                                         \
            fprintf(stderr, "%s failed: %d (%s)\n", #call, rc_, she_last_error(ctx));                \
            return 2;                                                                                \
        }                                                                                            \
    } while (0)

int main(void)
{
    const she_params toy = {128, 256, 1, 7, 3, 8, 2, 1.0 / 32768.0, 1.0 / 33554432.0};
    she_ctx *ctx = NULL;
    if (she_keygen(&toy, 42u, 256, &ctx) != SHE_OK) {
        fprintf(stderr, "she_keygen: %s\n", she_last_error(NULL));
        return 2;
    }
    /* x = 11, y = 6 as 4-bit unsigned numbers in slots 0..3 and 4..7 (least significant bit first) */
    const unsigned x = 11, y = 6;
    uint8_t bits[8];
    uint32_t ids[8];
    for (int i = 0; i < 4; i++) { bits[i] = (x >> i) & 1; bits[4 + i] = (y >> i) & 1; }
    for (uint32_t i = 0; i < 8; i++) ids[i] = i;
    CHECK(she_encrypt_bits(ctx, bits, 8, 7u, ids));

    /* one level: bitwise AND, XOR, NAND and (not x) and y */
    uint8_t type[16];
    uint32_t in0[16], in1[16], out[16];
    const uint8_t codes[4] = {SHE_AND, SHE_XOR, SHE_NAND, SHE_ANDNY};
    for (int g = 0; g < 16; g++) { type[g] = codes[g / 4]; in0[g] = g % 4; in1[g] = 4 + g % 4; out[g] = 16 + g; }
    CHECK(she_eval_gates(ctx, type, in0, in1, out, 16));
    uint8_t got[16];
    CHECK(she_decrypt(ctx, out, 16, got));
    int bad = 0;
    for (int g = 0; g < 16; g++) {
        const unsigned a = (x >> (g % 4)) & 1, b = (y >> (g % 4)) & 1;
        const unsigned want = g / 4 == 0 ? (a & b) : g / 4 == 1 ? (a ^ b) : g / 4 == 2 ? 1u - (a & b) : ((1u - a) & b);
        if (got[g] != want) bad++;
    }

    /* x - (y >> 1) into an 8-bit accumulator, then ReLU of it and of its negative */
    const int8_t sign[2] = {1, -1}, expo[2] = {0, -1};
    uint32_t acc_ids[8], neg_ids[8], relu_ids[16], both[16];
    for (uint32_t i = 0; i < 8; i++) { acc_ids[i] = 40 + i; neg_ids[i] = 50 + i; }
    uint64_t gates = 0;
    CHECK(she_shift_acc(ctx, ids, 1, 2, 4, sign, expo, 8, acc_ids, &gates));
    const int8_t sign_neg[2] = {-1, 1};
    CHECK(she_shift_acc(ctx, ids, 1, 2, 4, sign_neg, expo, 8, neg_ids, NULL));
    memcpy(both, acc_ids, sizeof acc_ids);
    memcpy(both + 8, neg_ids, sizeof neg_ids);
    for (uint32_t i = 0; i < 16; i++) relu_ids[i] = 60 + i;
    CHECK(she_relu(ctx, both, 2, 8, relu_ids, NULL));
    uint8_t rb[16];
    CHECK(she_decrypt(ctx, relu_ids, 16, rb));
    int v0 = 0, v1 = 0;
    for (int i = 0; i < 8; i++) { v0 |= rb[i] << i; v1 |= rb[8 + i] << i; }
    const int want0 = (int)x - (int)(y >> 1);             /* 11 - 3 = 8 */
    if (v0 != want0 || v1 != 0) bad++;
    printf("gates evaluated by she_shift_acc: %llu, relu(x - y/2) = %d, relu(y/2 - x) = %d, wrong results: %d\n",
           (unsigned long long)gates, v0, v1, bad);
    she_free(ctx);
    return bad ? 1 : 0;
}
