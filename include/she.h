/*
 * she.h - C ABI of the MI355X library for SHE's encrypted-inference hot path:
 * batched bootstrapped TFHE binary gates and the layer operators that lower to them.
 *
 * Citations are to "SHE: A Fast and Accurate Deep Neural Network for Encrypted
 * Data" (arXiv 1906.00148).  The paper states the problem (client encrypts bit by
 * bit, server evaluates 2-input homomorphic gates, shifts, accumulations, ReLU and
 * max pooling on ciphertexts, client decrypts) and cites the TFHE gate
 * bootstrapping without restating it; the encodings and rounding rules this library
 * fixes where the paper is silent are stated with the calls below.
 *
 * Conventions that hold for every call:
 *  - All pointer arguments are HOST pointers unless a comment says "device".  They
 *    are caller-owned and not retained after the call returns.
 *  - Ciphertexts live in a device-resident pool of `pool_capacity` TLWE slots owned
 *    by the context and addressed by a 32-bit id in [0, pool_capacity).  The caller
 *    decides which id holds what.  A slot is n+1 Torus32 words (a_0..a_{n-1}, b).
 *    Temporaries of the layer operators live in a separate internal buffer.
 *  - Torus32: a uint32_t t stands for t / 2^32 in R/Z; arithmetic is modulo 2^32.
 *    Bit 1 is encoded as +2^29 (+1/8), bit 0 as -2^29; decryption takes the sign of
 *    the phase.  Integers are vectors of bit ids, least significant bit first,
 *    two's complement where signed (Section 3.2: data are encrypted bit by bit and
 *    keep the order of the plaintext bits).
 *  - Return value: SHE_OK (0) or a negative code; she_last_error() gives the text.
 *    Nothing is thrown across this boundary.  On error the pool contents that the
 *    failing call was going to write are unspecified; inputs are untouched.
 *  - Calls run on the context's HIP stream and return after the work has finished
 *    (they synchronise that stream), unless stated otherwise.  A context is not
 *    thread-safe.  One GPU: the context uses the HIP device current at she_keygen.
 *  - There is no CPU fallback: without a usable GPU every call that computes
 *    returns SHE_EDEVICE.
 */
#ifndef SHE_H
#define SHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct she_ctx she_ctx; /* opaque: keys (secret ones too), device buffers, stream */

/* TFHE parameter set (Section 4, "TFHE setting", names the three sample levels; the
 * gate-bootstrapping values used by the benchmarks are n=630, N=1024, k=1, bg_bit=7,
 * l=3, ks_t=8, ks_basebit=2, lwe_std=2^-15, bk_std=2^-25).  Supported: k = 1;
 * N in {256, 512, 1024, 2048} (2048, the N-bar of Section 4's leveled setting, for the leveled calls only: the gate and
 * layer-operator calls return SHE_EINVAL there); 1 <= n <= 4096; l*bg_bit <= 31 with l <= 8, 2*l*N*Bg^2 <= 2^32 and l*N*Bg <= 2^20; ks_t*ks_basebit
 * <= 16 with ks_basebit <= 4.  The two gadget bounds belong to the FP64 polynomial products: the second keeps every sum
 * of products below 2^51 whatever the digits and key words are, which the rounding step needs; under the first the
 * transforms' rounding errors stay far below 1/2 for digits and key words as they occur (measured, largest distance
 * from an integer 0.012 at the benchmark's parameters, 0.07 on the bound; she_set_round_tracking records it), so the
 * rounded results are the exact integers with overwhelming probability rather than by proof. */
typedef struct {
    uint32_t n;          /* TLWE dimension */
    uint32_t N;          /* ring degree of TRLWE / TRGSW samples */
    uint32_t k;          /* number of TRLWE mask polynomials */
    uint32_t bg_bit;     /* log2 of the gadget base Bg */
    uint32_t l;          /* gadget length */
    uint32_t ks_t;       /* key-switch digits per coefficient */
    uint32_t ks_basebit; /* log2 of the key-switch base */
    double lwe_std;      /* noise of fresh TLWE samples and key-switch rows (fraction of the torus) */
    double bk_std;       /* noise of bootstrapping-key rows */
} she_params;

enum { SHE_OK = 0, SHE_EINVAL = -1, SHE_ENOMEM = -2, SHE_EDEVICE = -3, SHE_ERANGE = -4 };

/* Gate codes of she_eval_gates (Section 3.1: any 2-input binary homomorphic operation).
 * ANDNY = (not a) and b, ANDYN = a and (not b), ORNY = (not a) or b, ORYN = a or (not b).
 * NOT, copies and constants are not gates: the layer operators realise them as
 * re-wiring or as noiseless trivial ciphertexts (Section 3.2: a shift costs no gate). */
enum { SHE_NAND = 0, SHE_AND, SHE_OR, SHE_XOR, SHE_XNOR, SHE_NOR, SHE_ANDNY, SHE_ANDYN, SHE_ORNY, SHE_ORYN,
       SHE_NUM_GATES };

/* Codes of she_eval_gates3: SHE_MAJ3 + mask (at least two of the three inputs true) and SHE_XOR3 + mask (an odd
 * number true); bit i of mask (0..7) complements input i first. */
enum { SHE_MAJ3 = 176, SHE_XOR3 = 184 };

/* Section 2 ("Homomorphic Encryption": key pair of the client).  Generates the TLWE key,
 * the ring key, the bootstrapping key BK_i = TRGSW(s_i) and the key-switching key from
 * `seed`, uploads them, transforms BK to the kernels' spectral layout and allocates the
 * pool.  *out receives a new context; release it with she_free.  Errors: SHE_EINVAL
 * (unsupported parameters, null pointers), SHE_ENOMEM (host or device allocation),
 * SHE_EDEVICE (no GPU / HIP failure). */
int she_keygen(const she_params *params, uint64_t seed, uint32_t pool_capacity, she_ctx **out);

/* Frees every host and device resource of the context.  NULL is allowed. */
void she_free(she_ctx *ctx);

/* Section 2 (encryption function) / Section 3.2 (bit-by-bit encryption).  Encrypts
 * bits[0..nbits) (each 0 or 1) as fresh TLWE samples; sample k uses the noise stream
 * (enc_seed, k) and is stored in slot dst_ids[k].  Errors: SHE_ERANGE for an id outside
 * the pool, SHE_EINVAL for a bit other than 0/1 or null pointers. */
int she_encrypt_bits(she_ctx *ctx, const uint8_t *bits, size_t nbits, uint64_t enc_seed, const uint32_t *dst_ids);

/* Section 2 (decryption function).  bits_out[k] = 1 iff the phase of slot ids[k] is
 * positive.  Uses the secret key held by the context. */
int she_decrypt(she_ctx *ctx, const uint32_t *ids, size_t count, uint8_t *bits_out);

/* Section 3.1 (2-input homomorphic gates), Section 2 (bootstrapping keeps the noise in
 * check).  Evaluates ONE circuit level: ngates mutually independent bootstrapped gates,
 * slot out[g] <- type[g](slot in0[g], slot in1[g]).  Per gate: TLWE linear combination,
 * modulus switch, blind rotation (n CMux external products), sample extraction, key
 * switch.  All four arrays have ngates entries.  No out id may equal an in id of the
 * same call or another out id (SHE_EINVAL); ids outside the pool give SHE_ERANGE; a
 * type >= SHE_NUM_GATES gives SHE_EINVAL.  ngates = 0 is a no-op. */
int she_eval_gates(she_ctx *ctx, const uint8_t *type, const uint32_t *in0, const uint32_t *in1,
                   const uint32_t *out, size_t ngates);

/* Section 3.1 (the units are built from homomorphic gates; a bootstrapped gate is a linear combination of
 * its inputs whose phase has the wanted sign, then one bootstrap) and Section 3.3 (the accumulator's adders).
 * ONE level of ngates three-input gates, each with a single bootstrap like a 2-input gate:
 *   SHE_MAJ3: pre-bootstrap sample +-c0 +- c1 +- c2, phase (2k-3)/8 for k true inputs, sign = majority;
 *   SHE_XOR3: -2 times that sample, phase +1/4 for odd k and -1/4 for even k.
 * A full-adder cell is sum = XOR3(a, b, carry), next carry = MAJ3(a, b, carry): two bootstraps instead of
 * five (see SHE_OPT_GATE3_CELLS).  Decision margins against the output noise of earlier bootstraps stay above
 * 20 standard deviations at the supported parameter sets.  Same id rules and error codes as she_eval_gates. */
int she_eval_gates3(she_ctx *ctx, const uint8_t *type, const uint32_t *in0, const uint32_t *in1, const uint32_t *in2,
                    const uint32_t *out, size_t ngates);

/* Section 3.2 (logarithmic quantization: sum_i binaryshift(input_i, weightQ_i)) and
 * Section 3.3 (mixed-bitwidth accumulator).  For each of `units` output neurons:
 *   out = sum_t w_sign[t] * (x_t >> -w_exp[t])   modulo 2^acc_bits (two's complement),
 * x_t unsigned in_bits-bit inputs.  Shifts re-wire ids (dropped low bits, trivial zeros on
 * top); positive and negative terms are summed by separate adder trees whose level j uses
 * min(in_bits+j, acc_bits)-bit ripple-carry adders, followed by one subtraction.
 *   x_ids   [units][terms][in_bits]  pool ids, LSB first
 *   w_sign  [units][terms]           +1 or -1
 *   w_exp   [units][terms]           in [-(in_bits-1), 0]
 *   out_ids [units][acc_bits]        pool ids that receive the result bits
 * Requires 1 <= in_bits <= acc_bits <= 32.  All units are levelized together and each
 * level is one batched gate evaluation.  *gates_out (may be NULL) receives the number of
 * bootstrapped gates evaluated.  out ids must not overlap x ids. */
int she_shift_acc(she_ctx *ctx, const uint32_t *x_ids, uint32_t units, uint32_t terms, uint32_t in_bits,
                  const int8_t *w_sign, const int8_t *w_exp, uint32_t acc_bits, const uint32_t *out_ids,
                  uint64_t *gates_out);

/* Section 5 / Table 3 (the layer sequences C-B-A-P: a batch normalisation sits between the linear layer and the
 * activation; with plaintext weights its scale folds into the weights and its shift is a constant per unit).
 * she_shift_acc with a plaintext constant per unit:
 *   out = bias[u] + sum_t w_sign[t] * (x_t >> -w_exp[t])   modulo 2^acc_bits,
 * bias [units] (NULL = all zero; any int32 value, it wraps like the sum).  The constant enters as noiseless trivial
 * ciphertexts: with the adder trees a constant that is not 0 modulo 2^acc_bits costs one more acc_bits-wide adder
 * on the positive tree's sum (most of its gates fold away under SHE_OPT_FOLD_CONSTANTS); under
 * SHE_OPT_COLUMN_ADDER it joins the negative terms' constants in plain arithmetic and costs no adder.
 * Everything else as she_shift_acc, which is this call with bias = NULL. */
int she_shift_acc_bias(she_ctx *ctx, const uint32_t *x_ids, uint32_t units, uint32_t terms, uint32_t in_bits,
                       const int8_t *w_sign, const int8_t *w_exp, const int32_t *bias, uint32_t acc_bits,
                       const uint32_t *out_ids, uint64_t *gates_out);

/* Section 3.1 (ReLU(x) = max(x, 0) from Boolean gates).  x_ids [count][bits] two's
 * complement, out_ids [count][bits]; every lower bit is masked by the sign bit, the
 * result's sign bit is a trivial zero.  bits >= 2.  One level of count*(bits-1) gates. */
int she_relu(she_ctx *ctx, const uint32_t *x_ids, uint32_t count, uint32_t bits, const uint32_t *out_ids,
             uint64_t *gates_out);

/* Section 3.1 (max pooling unit).  2x2 window, stride 2 over x_ids [H][W][C][bits]
 * (two's complement); out_ids [H/2][W/2][C][bits].  A ragged last row or column is
 * dropped.  Each max is a ripple comparator plus one MUX per bit; MUX(s,u,v) is lowered
 * to OR(AND(s,u), ANDNY(s,v)). */
int she_maxpool(she_ctx *ctx, const uint32_t *x_ids, uint32_t H, uint32_t W, uint32_t C, uint32_t bits,
                const uint32_t *out_ids, uint64_t *gates_out);

/* Section 3.1 (activation followed by pooling, the A-P pair of the layer sequences in Section 5): ReLU then 2x2
 * stride-2 max pooling in one call, same shapes as she_maxpool.  max(x, 0) is monotone, so the result equals the
 * ReLU of the window's maximum: the window is pooled on the signed values and one sign mask is applied to the pooled
 * value, a quarter of the masking gates of she_relu on every input.  Decrypts to the same values as she_relu followed
 * by she_maxpool. */
int she_relu_maxpool(she_ctx *ctx, const uint32_t *x_ids, uint32_t H, uint32_t W, uint32_t C, uint32_t bits,
                     const uint32_t *out_ids, uint64_t *gates_out);

/* Section 5 / Table 3 (a network is a sequence of layers C-B-A-P-...; Section 3.1-3.3 lower each layer to gates) and
 * Section 3.1 (gates that do not depend on each other can be evaluated together).  Between she_defer_begin and
 * she_defer_run the layer operators (she_shift_acc, she_shift_acc_bias, she_relu, she_maxpool, she_relu_maxpool) only
 * record their netlists: an operator that reads a slot which a recorded operator writes is wired to that operator's
 * result.  she_defer_run then schedules ALL recorded entries at their earliest depth level and evaluates each level as
 * one batch, so the last carries of a layer's adders run beside the first comparator stages of the pooling that
 * follows, instead of one operator after the other; every recorded output still lands in its pool slot.  The results
 * are the ciphertexts that the same calls give one by one (identical words without SHE_OPT_FOLD_CONSTANTS; with it
 * the folding also sees constants across operator boundaries, e.g. the zero sign bit after a ReLU, and may spend
 * fewer gates).  Rules while recording: an operator's out ids must not be read by an earlier recorded operator as an
 * input of the circuit, nor be written twice (SHE_EINVAL; the scheduler may reorder such accesses); the options
 * cannot change; every other call that touches the pool returns SHE_EINVAL.  An operator's *gates_out is the number
 * of entries it recorded; *entries_out (may be NULL) of she_defer_run the number evaluated; she_last_timing then
 * covers the whole circuit.  A failed she_defer_run, and an operator that fails with SHE_ENOMEM / SHE_ERANGE while
 * recording, drop the recorded circuit. */
int she_defer_begin(she_ctx *ctx);
int she_defer_run(she_ctx *ctx, uint64_t *entries_out);

/* Section 3.1 (every operator of the network is a circuit of homomorphic gates; "Homomorphic Operations" names the
 * 2-input operations and the MUX).  A whole circuit in one call: ngates entries in topological order, entry g of
 * code type[g] reading the references in0[g], in1[g] (and in2[g] for three-input codes and SHE_CIRCUIT_MUX).  A
 * reference is a pool id, SHE_WIRE_GATE | h for the result of entry h < g of the same call, SHE_WIRE_ZERO /
 * SHE_WIRE_ONE for the noiseless trivial ciphertexts, each optionally with SHE_WIRE_NOT (the complement, a free
 * word-wise negation; accepted only under SHE_OPT_FOLD_CONSTANTS, which absorbs it into the gate codes).
 * Codes: the ten 2-input codes, SHE_MAJ3 + mask, SHE_XOR3 + mask, and SHE_CIRCUIT_MUX (in0 ? in1 : in2, three gates
 * or one native entry under SHE_OPT_NATIVE_MUX).  The library schedules every entry at its earliest depth level,
 * evaluates each level as one batch (as she_eval_gates / she_eval_gates3 / she_eval_mux do), keeps intermediate
 * results in its own temporaries, and leaves the results named by out_refs[0..nout) in the pool slots out_ids;
 * the options fold entries exactly as they do inside the layer operators.  out_ids must be distinct and disjoint
 * from every pool id the circuit reads.  *entries_out (may be NULL) receives the number of entries evaluated.
 * Errors: SHE_EINVAL (unknown code, forward reference, SHE_WIRE_NOT without folding, null pointers, clashing ids),
 * SHE_ERANGE (id outside the pool). */
#define SHE_WIRE_GATE 0x40000000u
#define SHE_WIRE_NOT 0x80000000u
#define SHE_WIRE_ZERO 0x3FFFFFFEu
#define SHE_WIRE_ONE 0x3FFFFFFFu
#define SHE_CIRCUIT_MUX 255
int she_eval_circuit(she_ctx *ctx, const uint8_t *type, const uint32_t *in0, const uint32_t *in1, const uint32_t *in2,
                     size_t ngates, const uint32_t *out_refs, const uint32_t *out_ids, size_t nout, uint64_t *entries_out);
/* The same circuit without a GPU: entries left after folding under `options` (bitwise OR of the netlist options SHE_OPT_FOLD_CONSTANTS,
 * SHE_OPT_NATIVE_MUX, SHE_OPT_GATE3_CELLS, SHE_OPT_COLUMN_ADDER: 1, 2, 4, 8), depth levels and blind rotations; pool ids in the references must be below `capacity`. */
int she_plan_circuit(uint32_t capacity, const uint8_t *type, const uint32_t *in0, const uint32_t *in1, const uint32_t *in2,
                     size_t ngates, int options, uint64_t *gates, uint32_t *levels, uint64_t *rotations);

/* Options.  SHE_OPT_FOLD_CONSTANTS (default 0): the layer operators stop spending a bootstrap on
 * gates whose result is fixed by a trivial-constant or repeated operand (the zeros that a shift
 * leaves on top of a term, the carry-in of the subtraction, the comparator's first stage): such a
 * gate becomes a constant, its other operand, or that operand's complement, and complements are
 * absorbed into the next gate's code or applied as a free word-wise negation (Section 3.2: what
 * only re-wires ciphertexts costs no gate).  Results decrypt identically; gate counts drop. */
enum { SHE_OPT_FOLD_CONSTANTS = 1, SHE_OPT_NATIVE_MUX = 2, SHE_OPT_SPLIT_BELOW = 3, SHE_OPT_GATE3_CELLS = 4,
       SHE_OPT_COLUMN_ADDER = 8 };
int she_set_option(she_ctx *ctx, int option, int value);
int she_get_option(she_ctx *ctx, int option, int *value);   /* SHE_EINVAL for an unknown option or a null pointer */
/* SHE_OPT_SPLIT_BELOW (default: 6 x the device's compute units, 1536 on MI355X): a kernel launch of at
 * most this many blind rotations spreads each one over two wavefronts (one per accumulator component),
 * which shortens the serial chain per CMux when the level is too small to fill the chip; larger launches
 * keep one wavefront per rotation.  0 never splits.  Every ciphertext comes out the same word for word
 * either way (both kernels round exact integers). */
/* SHE_OPT_COLUMN_ADDER (default 0; needs SHE_OPT_FOLD_CONSTANTS and SHE_OPT_GATE3_CELLS, else she_shift_acc returns
 * SHE_EINVAL): she_shift_acc sums by column compression instead of adder trees and a subtraction (Section 3.3: adders
 * only as wide as the bits they receive).  Every bit of every shifted term sits in the column of its weight; a
 * negative term enters as the complements of its w wires plus the plaintext constant 1 - 2^w; stages of full-adder
 * cells (parity stays, majority moves one column up) leave at most two wires per column, and one ripple adder of
 * cells finishes.  About a third fewer gates than the trees for a 3x3 kernel, 39 % fewer for 576 terms. */
/* SHE_OPT_GATE3_CELLS (default 0): the operators use three-input gates (she_eval_gates3).  The adders and the
 * subtraction of she_shift_acc become full-adder cells of two gates above the lowest bit: a w-bit adder costs 2w gates
 * in w levels instead of 5w-3 gates in 2w-1 levels (a 576-term 8-bit tree: 10,332 gates instead of 24,104).  The
 * comparator of she_maxpool becomes one majority gate per bit, majority(x_i, not y_i, greater-so-far), instead of an
 * equality gate and a MUX per bit.  Results decrypt identically. */
/* SHE_OPT_NATIVE_MUX (default 0): she_maxpool evaluates every MUX of its comparators and selectors
 * with she_eval_mux's three-input gate instead of three 2-input gates (7w gates per max become
 * w gates + 2w MUX entries = 5w blind rotations and 3w key switches, and half the levels). */

/* Section 3.1 (MUX is named among the homomorphic gates).  One level of nmux independent native
 * MUX gates: slot out[m] <- slot sel[m] ? slot in1[m] : slot in0[m].  Each is two blind rotations
 * (of sel AND in1 and of (NOT sel) AND in0), whose extracted samples are added with 1/8 on the body,
 * and ONE key switch.  Same id rules and error codes as she_eval_gates. */
int she_eval_mux(she_ctx *ctx, const uint32_t *sel, const uint32_t *in1, const uint32_t *in0, const uint32_t *out,
                 size_t nmux);

/* Host-only planning (no GPU, no context): what she_shift_acc / she_relu / she_maxpool would evaluate
 * for these shapes and weights under `options` (bitwise OR of the netlist options SHE_OPT_FOLD_CONSTANTS, SHE_OPT_NATIVE_MUX,
 * SHE_OPT_GATE3_CELLS, SHE_OPT_COLUMN_ADDER, which are 1, 2, 4, 8; SHE_OPT_SPLIT_BELOW is not one): number of netlist
 * entries (gates + MUX entries), of circuit levels, and of blind rotations (one per gate, two per
 * MUX entry).  Any output pointer may be NULL.  Same argument checks as the operators. */
int she_plan_shift_acc(uint32_t units, uint32_t terms, uint32_t in_bits, const int8_t *w_sign, const int8_t *w_exp,
                       uint32_t acc_bits, int options, uint64_t *gates, uint32_t *levels, uint64_t *rotations);
int she_plan_shift_acc_bias(uint32_t units, uint32_t terms, uint32_t in_bits, const int8_t *w_sign, const int8_t *w_exp,
                            const int32_t *bias, uint32_t acc_bits, int options, uint64_t *gates, uint32_t *levels,
                            uint64_t *rotations);
/* Section 3.3 (the accumulator's adders are sized by the bits they can receive; the weights and constants are
 * plaintext, so the server knows the range).  *bits_out = the smallest two's-complement width that holds
 * bias[u] + sum_t w_sign[t] * (x_t >> -w_exp[t]) for every unit u and all unsigned in_bits-bit inputs, at least
 * in_bits; a layer run at this acc_bits gives the same integers as at any larger one.  bias may be NULL.  Host only. */
int she_plan_accumulator_bits(uint32_t units, uint32_t terms, uint32_t in_bits, const int8_t *w_sign, const int8_t *w_exp,
                              const int32_t *bias, uint32_t *bits_out);
int she_plan_relu(uint32_t count, uint32_t bits, int options, uint64_t *gates, uint32_t *levels, uint64_t *rotations);
int she_plan_maxpool(uint32_t H, uint32_t W, uint32_t C, uint32_t bits, int options, uint64_t *gates, uint32_t *levels,
                     uint64_t *rotations);
int she_plan_relu_maxpool(uint32_t H, uint32_t W, uint32_t C, uint32_t bits, int options, uint64_t *gates, uint32_t *levels,
                          uint64_t *rotations);

/* ---- leveled mode (Section 4, "TFHE setting": the three sample levels TLWE / TRLWE / TRGSW used
 * without bootstrapping) ----
 * Ring degrees: every supported N, including Section 4's N-bar = 2048 (with that section's n = 500 or any other n;
 * the leveled calls use the ring key only).
 * Selector bits are TRGSW samples, data are TRLWE samples of torus polynomials, and the one
 * homomorphic operation is the CMux  out = d0 + C [.] (d1 - d0)  (the external product of the
 * blind rotation's inner step): out carries d1's message if C encrypts 1 and d0's if 0, and the
 * noise grows additively per CMux instead of being reset.  Lookup tables and decision trees
 * evaluate as levels of CMuxes.  Both kinds of sample live in device pools of their own, addressed
 * by 32-bit ids: TRGSW samples in the kernels' spectral form (2l x 2 spectra of N/2 complex
 * doubles), TRLWE samples as [2][N] Torus32 words (mask polynomial, body polynomial). */

/* Allocates (or re-allocates, dropping the contents) the two pools.  SHE_EINVAL for a zero capacity. */
int she_leveled_init(she_ctx *ctx, uint32_t trgsw_capacity, uint32_t trlwe_capacity);

/* Fresh TRGSW samples of bits[0..count) under the ring key with noise bk_std; sample k has the
 * layout of one bootstrapping-key entry, rows (c, p) = TRLWE samples of zero from noise stream
 * (seed, (k*2+c)*l+p) plus bits[k] * 2^(32-(p+1)*bg_bit) on coefficient 0 of component c, and is
 * stored, transformed, in selector slot dst_ids[k].  SHE_EINVAL before she_leveled_init or for a
 * bit other than 0/1, SHE_ERANGE for an id outside the selector pool. */
int she_trgsw_encrypt_bits(she_ctx *ctx, const uint8_t *bits, size_t count, uint64_t seed, const uint32_t *dst_ids);

/* Fresh TRLWE samples of the torus polynomials mu[count][N] (noise bk_std, stream (seed, k)) into
 * data slots dst_ids[k]. */
int she_trlwe_encrypt(she_ctx *ctx, const uint32_t *mu, size_t count, uint64_t seed, const uint32_t *dst_ids);

/* Copies samples[count][2][N] into / out of data slots (a noiseless constant is the sample (0, mu)). */
int she_trlwe_write(she_ctx *ctx, const uint32_t *samples, size_t count, const uint32_t *dst_ids);
int she_trlwe_read(she_ctx *ctx, const uint32_t *ids, size_t count, uint32_t *samples);

/* Decryption side: phases[k][N] = B - A (*) s' of data slot ids[k], with the ring key of the context. */
int she_trlwe_phase(she_ctx *ctx, const uint32_t *ids, size_t count, uint32_t *phases);

/* ONE level of `count` mutually independent CMuxes: data slot out[m] <- selector sel[m] ? data slot
 * in1[m] : data slot in0[m].  Per entry: gadget decomposition of in1 - in0 (signed digits, rounded
 * to nearest), 2l forward transforms, 2l x 2 pointwise products with the selector's spectra, two
 * inverse transforms, addition of in0.  Results are exact integers (the same rounding argument as
 * the blind rotation).  No out id may equal an in1 / in0 id of the same call or another out id
 * (SHE_EINVAL); ids outside their pools give SHE_ERANGE.  The entries are evaluated in an order of the
 * library's choosing (grouped by selector, so that entries which share a selector's spectra run
 * together).  she_last_timing then reports the kernel's time in ms[1]. */
int she_eval_cmux(she_ctx *ctx, const uint32_t *sel, const uint32_t *in1, const uint32_t *in0, const uint32_t *out,
                  size_t count);

/* ---- diagnostics and plumbing (not part of the paper's problem statement) ---- */

/* Copies slot `id` to dst[0..n] (a_0..a_{n-1}, b) / overwrites it from src. */
int she_read_ct(she_ctx *ctx, uint32_t id, uint32_t *dst);
int she_write_ct(she_ctx *ctx, uint32_t id, const uint32_t *src);

/* Copies the generated keys to caller buffers (any may be NULL): lwe_key[n] and
 * ring_key[N] bits, bk[n][2][l][2][N] and ks[N][ks_t][2^ks_basebit-1][n+1] Torus32
 * words in the logical layout used for generation (not the device layout). */
int she_export_keys(she_ctx *ctx, uint8_t *lwe_key, uint8_t *ring_key, uint32_t *bk, uint32_t *ks);

/* Work of later calls is enqueued on `hip_stream` (a hipStream_t; NULL = default stream). */
int she_set_stream(she_ctx *ctx, void *hip_stream);

/* Replaces the pool by caller-owned DEVICE memory of at least she_pool_bytes(ctx) bytes
 * (256-byte aligned); the old pool's contents are not copied.  The caller keeps ownership
 * and must keep it alive until she_free or the next she_bind_pool. */
int she_bind_pool(she_ctx *ctx, void *dev_ptr, size_t bytes);
size_t she_pool_bytes(const she_ctx *ctx);

/* Enqueues one level like she_eval_gates but takes DEVICE arrays, validates nothing but
 * ngates, and does not synchronise: for timing loops and callers that keep netlists on
 * the device.  The arrays must stay valid until the stream has finished. */
int she_eval_gates_device(she_ctx *ctx, const uint8_t *d_type, const uint32_t *d_in0, const uint32_t *d_in1,
                          const uint32_t *d_out, size_t ngates);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): she_eval_gates_device with the level's scratch (rounded samples,
 * extracted bodies, key-switch digits) in a static 16 MiB device buffer of the library instead of
 * allocated buffers.  It calls no hipMalloc / hipFree and creates no events (it is never timed:
 * she_last_timing does not see it); inputs, outputs, the pool and the keys are the caller's and the
 * context's as before.  Same arguments, same results word for word, same lack of validation and of
 * synchronisation as she_eval_gates_device.  Limit: bar + bodies + digits of one call must fit the
 * buffer, i.e. ngates * (2*(n+1 rounded up to 2) + 4 + 2*N) bytes (+ alignment) <= 16 MiB: 5056 gates at
 * n=630, N=1024; more gives SHE_ERANGE and she_last_error names the limit.  Every context on one GPU
 * shares that GPU's buffer, which keeps the previous call's contents (nothing in it has to start at
 * zero): calls that overlap on one GPU (two streams, two contexts) race; calls on one stream are safe. */
int she_eval_gates_device_noalloc(she_ctx *ctx, const uint8_t *d_type, const uint32_t *d_in0, const uint32_t *d_in1,
                                  const uint32_t *d_out, size_t ngates);

/* Largest distance from an integer seen by the blind rotation's rounding of inverse
 * transform outputs since the last reset (0 <= value <= 0.5); only recorded while
 * tracking is on (slower kernel).  Exact integer results need this to stay well below 0.5. */
int she_set_round_tracking(she_ctx *ctx, int on);
int she_get_round_error(she_ctx *ctx, double *max_abs_frac, int reset);

/* Kernel timing with HIP events on the context's stream (on by default; she_set_timing(ctx, 0)
 * removes the events).  she_last_timing gives the milliseconds spent in each kernel family by
 * the last she_eval_gates / layer-operator call, or summed over all she_eval_gates_device
 * calls since the previous she_last_timing (it then waits for the stream): ms[0] linear
 * combination, ms[1] blind rotation + extraction, ms[2] key switch, ms[3] levels launched. */
int she_set_timing(she_ctx *ctx, int on);
int she_last_timing(she_ctx *ctx, double ms[4]);

/* The schedule of the last circuit that the context ran (a layer operator, she_eval_circuit, she_defer_run): level v
 * (0-based, in the order the levels ran) held gates[v] gate entries and muxes[v] native MUX entries (two blind
 * rotations each).  *levels_out (may be NULL) is the number of levels; at most `capacity` entries of each array are
 * written (the arrays may be NULL with capacity 0 to ask for the count only). */
int she_last_level_sizes(const she_ctx *ctx, uint64_t *gates, uint64_t *muxes, size_t capacity, size_t *levels_out);

/* Text of the last error of this context ("" if none).  ctx may be NULL: then the text
 * of the last failed she_keygen of the calling thread. */
const char *she_last_error(const she_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* SHE_H */
