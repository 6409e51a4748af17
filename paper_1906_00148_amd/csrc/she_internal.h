// Internal declarations shared by the host files and the kernel file of the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "../../include/she.h"

namespace she {

constexpr int KS_GROUP = 32;        // gates whose key-switch digits are stored together / share one key-switch block
constexpr int MAX_LEVEL_CHUNK = 32768;  // gates per kernel launch; larger levels are cut into chunks

inline uint32_t round_up(uint32_t v, uint32_t m) { return (v + m - 1) / m * m; }

// Everything a kernel needs to find ciphertexts: ids below `cap` are pool slots, ids from
// `cap` on are slots of the internal temporary buffer (slot 0 = trivial 0, slot 1 = trivial 1).
struct CtSpace {
    uint32_t *pool;
    uint32_t *temp;
    uint32_t cap;
    uint32_t stride;   // words per slot (n+1 rounded up to 32)
};

struct DeviceKeys {
    double2 *bk_hat = nullptr;    // [n][2l][2][P][L] spectra of the bootstrapping key
    uint32_t *ks = nullptr;       // [N][t][base-1][ks_stride]; only for key-switch shapes without an MFMA kernel
    int8_t *ks_bytes = nullptr;   // [N][4 byte planes][ks_cols][32 = 8 digits x 4 values] signed bytes (base 4, t = 8)
    uint32_t ks_cols = 0;         // n+1 rounded up to 32
    double2 *twiddles = nullptr;  // [K-1][P][L]
    uint32_t ks_stride = 0;
    uint32_t cus = 1;             // compute units of the device (launch shaping)
};

struct LevelWork {                // scratch of one level launch, sized for `gates` gates
    uint16_t *bar = nullptr;      // [gates][bar_stride]: abar_0..abar_{n-1}, bbar
    uint32_t *ext_b = nullptr;    // [gates] body of the extracted sample
    uint16_t *ksd = nullptr;      // [gates/KS_GROUP][N][KS_GROUP] rounded top bits of the extracted mask
    uint32_t bar_stride = 0;
    size_t gates = 0;
    uint32_t *raw_ext = nullptr;  // [jobs][N+1] extracted samples of MUX rotations (not yet key-switched)
    size_t raw_jobs = 0;
};

// ---- kernel launchers (she_kernels.hip); each returns a hipError_t and never synchronises ----
bool plan_supported(uint32_t N);
size_t twiddle_doubles(uint32_t N);
void fill_twiddles(uint32_t N, double *host_out);
size_t bk_hat_elems(const she_params &P);   // number of double2 in DeviceKeys::bk_hat

hipError_t launch_bk_transform(const she_params &P, const uint32_t *d_bk_int, const DeviceKeys &K, hipStream_t st);
// leveled mode: spectra of `samples` TRGSW samples d_int[s][2l][2][N] into slots d_ids[s] of trgsw_hat; CMux batch
hipError_t launch_trgsw_transform(const she_params &P, const DeviceKeys &K, const uint32_t *d_int, double2 *trgsw_hat,
                                  const uint32_t *d_ids, size_t samples, hipStream_t st);
hipError_t launch_cmux(const she_params &P, const DeviceKeys &K, const double2 *trgsw_hat, uint32_t *trlwe,
                       const uint32_t *d_sel, const uint32_t *d_in1, const uint32_t *d_in0, const uint32_t *d_out,
                       size_t count, unsigned *d_round_err, hipStream_t st);
// d_in2 may be null when no type is a three-input gate
hipError_t launch_lincomb(const she_params &P, const CtSpace &cs, const uint8_t *d_type, const uint32_t *d_in0,
                          const uint32_t *d_in1, const uint32_t *d_in2, size_t gates, const LevelWork &W, hipStream_t st);
hipError_t launch_blind_rotate(const she_params &P, const DeviceKeys &K, const CtSpace &cs, const uint32_t *d_out,
                               size_t gates, const LevelWork &W, unsigned *d_round_err /* nullptr = no tracking */,
                               hipStream_t st, bool raw = false /* write W.raw_ext instead of digits and slots */,
                               bool split = false /* two wavefronts per gate: for levels that leave the chip underfilled */);
// MUX m: sample = raw_ext[2m] + raw_ext[2m+1] + (0, 1/8) -> key-switch digits, body and slot initialisation of gate m
hipError_t launch_mux_combine(const she_params &P, const DeviceKeys &K, const CtSpace &cs, const uint32_t *d_out,
                              size_t muxes, const LevelWork &W, hipStream_t st);
hipError_t launch_key_switch(const she_params &P, const DeviceKeys &K, const CtSpace &cs, const uint32_t *d_out,
                             size_t gates, const LevelWork &W, hipStream_t st);
hipError_t launch_scatter(const CtSpace &cs, const uint32_t *d_src /* [count][n+1] */, const uint32_t *d_ids,
                          size_t count, uint32_t n, hipStream_t st);
hipError_t launch_gather(const CtSpace &cs, uint32_t *d_dst /* [count][n+1] */, const uint32_t *d_ids, size_t count,
                         uint32_t n, hipStream_t st);
// diagnostic: `blocks` workgroups of 256 threads, each thread 64*iters dependent-free FP64 instructions of one form
hipError_t launch_fp64_probe(int form, double *d_out, uint32_t blocks, int iters, const double2 *src, uint32_t src_rows,
                             hipStream_t st);
hipError_t launch_lds_probe(int form, uint32_t *d_out, uint32_t blocks, int iters, hipStream_t st);
hipError_t launch_copy_ct(const CtSpace &cs, const uint32_t *d_src_ids, const uint32_t *d_dst_ids, size_t count,
                          uint32_t n, hipStream_t st);

// Device address and size of the static scratch buffer on `device` (which must be the current device); looked up
// once per device and kept.  The buffer belongs to the loaded code object: it is never freed.
hipError_t noalloc_scratch(int device, void **ptr, size_t *bytes);

// ---- host-side key material and samples (she_host.cpp) ----
struct HostKeys {
    std::vector<uint8_t> lwe_key, ring_key;
    std::vector<uint32_t> bk;    // [n][2][l][2][N]
    std::vector<uint32_t> ks;    // [N][t][base-1][n+1]
};
void generate_keys(const she_params &P, uint64_t seed, HostKeys &out);
void fresh_samples(const she_params &P, const std::vector<uint8_t> &lwe_key, const uint8_t *bits, size_t nbits,
                   uint64_t enc_seed, uint32_t *out /* [nbits][n+1] */);
// key-switching key as signed byte planes for the MFMA kernel: out[i][plane][col][j*4+v]
void pack_ks_bytes(const she_params &P, const std::vector<uint32_t> &ks, uint32_t cols_p, std::vector<int8_t> &out);
// leveled mode: fresh TRGSW samples of bits [count][2][l][2][N], fresh TRLWE samples of mu[count][N] as [count][2][N]
// (noise bk_std, or none), phases B - A*s' of TRLWE samples
void fresh_trgsw(const she_params &P, const std::vector<uint8_t> &ring_key, const uint8_t *bits, size_t count,
                 uint64_t seed, uint32_t *out);
void fresh_trlwe(const she_params &P, const std::vector<uint8_t> &ring_key, const uint32_t *mu, size_t count,
                 uint64_t seed, uint32_t *out);
void trlwe_phases(const she_params &P, const std::vector<uint8_t> &ring_key, const uint32_t *cts, size_t count,
                  uint32_t *phases);
void phases_to_bits(const she_params &P, const std::vector<uint8_t> &lwe_key, const uint32_t *cts, size_t count,
                    uint8_t *bits);

// ---- netlists of the layer operators (she_circuits.cpp) ----
constexpr uint32_t WIRE_NEG = 0x80000000u;   // flag on a wire reference: the complement of that wire
constexpr int MUX_BASE = SHE_NUM_GATES;       // netlist type of a native MUX entry: MUX_BASE + 16*code1 + code0 (< SHE_MAJ3)
inline bool is_mux_type(uint8_t t) { return t >= MUX_BASE && t < SHE_MAJ3; }
inline bool has_third_operand(uint8_t t) { return t >= MUX_BASE; }     // MUX entries and three-input gates

struct Netlist {
    // wire ids: [0, cap) pool slots, cap = trivial 0, cap+1 = trivial 1, cap+2.. temporaries.
    // With `fold` set, a gate fixed by constant or repeated operands is not emitted: gate()
    // returns a constant, an operand, or an operand with WIRE_NEG (complementing a ciphertext
    // is a free negation of its words), and complemented operands of a real gate are absorbed
    // into the gate code.
    uint32_t cap = 0;
    uint32_t next_temp = 0;
    bool fold = false;
    bool native_mux = false;                    // mux() emits one three-input entry instead of three gates
    bool cells3 = false;                        // adders use cells of two three-input gates (parity, majority)
    bool columns = false;                       // shift-accumulate sums by column compression (nl_columns)
    bool overflow = false;                      // more wires than 31-bit ids can name
    std::vector<uint8_t> type;
    std::vector<uint32_t> in0, in1, in2, out;   // in2: third operand of MUX entries and three-input gates (0 otherwise)
    std::vector<uint32_t> copy_src, copy_dst;   // executed after all gates; copy_src may carry WIRE_NEG

    explicit Netlist(uint32_t capacity, bool fold_constants = false, bool mux_native = false, bool cells3 = false,
                     bool columns = false)
        : cap(capacity), next_temp(capacity + 2), fold(fold_constants), native_mux(mux_native), cells3(cells3),
          columns(columns) {}
    uint64_t rotations() const;                 // blind rotations: one per gate, two per MUX entry
    uint32_t zero() const { return cap; }
    uint32_t one() const { return cap + 1; }
    uint32_t gate(int code, uint32_t a, uint32_t b);
    uint32_t mux(uint32_t s, uint32_t u, uint32_t v);
    // majority (base SHE_MAJ3) or parity (base SHE_XOR3) of three wires with one bootstrap
    uint32_t gate3(int base, uint32_t a, uint32_t b, uint32_t c);
    // route the wires in `wires` to the caller's ids `dst`: gate outputs are renamed,
    // anything else (inputs, constants, a wire used twice) is copied at the end
    void bind_outputs(const std::vector<uint32_t> &wires, const uint32_t *dst);
    // stable sort of the entries by (depth, gates before MUX entries); returns the first index of each
    // level (+ end); mux_start[lv] receives the index of level lv's first MUX entry
    std::vector<size_t> levelize(std::vector<size_t> *mux_start = nullptr);
    // after levelize and bind_outputs: re-numbers the remaining temporaries so that slots are reused once their last
    // reader's level has run; `bounds` are levelize's.  Returns the slots needed (constants included), 0 on an
    // internal inconsistency.
    size_t compact_temporaries(const std::vector<size_t> &bounds);
};
std::vector<uint32_t> nl_add(Netlist &nl, const std::vector<uint32_t> &a, const std::vector<uint32_t> &b, uint32_t cap_bits);
std::vector<uint32_t> nl_sub(Netlist &nl, const std::vector<uint32_t> &p, const std::vector<uint32_t> &q);
std::vector<uint32_t> nl_tree(Netlist &nl, std::vector<std::vector<uint32_t>> terms, uint32_t in_bits, uint32_t acc_bits);
std::vector<uint32_t> nl_max(Netlist &nl, const std::vector<uint32_t> &x, const std::vector<uint32_t> &y);
// signed sum of unsigned terms (wires LSB first, no padding; sign +1 / -1) mod 2^acc_bits by column compression;
// the netlist must fold constants and use three-input cells
struct SignedTerm { std::vector<uint32_t> bits; int sign; };
std::vector<uint32_t> nl_columns(Netlist &nl, const std::vector<SignedTerm> &terms, uint32_t acc_bits, int64_t bias = 0);
std::vector<uint32_t> nl_constant(Netlist &nl, int64_t value, uint32_t bits);   // trivial wires of a plaintext integer

}  // namespace she
