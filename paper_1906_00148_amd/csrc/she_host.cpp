// Client-side pieces: random streams, key generation, fresh encryptions, decryption.
// (SHE, arXiv 1906.00148, Section 2: the client owns the private key, encrypts its data
// and decrypts the result.)  Host code only; none of it is on the timed path.
//
// Random streams.  Every generated object has its own stream addressed by
// (seed, tag, index); word c of a stream is mix(key + (c+1)*GOLDEN) with
// key = mix(mix(mix(seed) + tag) + index) and mix the SplitMix64 finaliser.  A uniform
// Torus32 is the top half of a word, a key bit its top bit.  A Gaussian error uses two
// consecutive words as 53-bit uniforms u1 in (0,1], u2 in [0,1):
// e = round(sqrt(-2 ln u1) * cos(2 pi u2) * sigma * 2^32), reduced modulo 2^32.
#include <algorithm>
#include <cmath>
#include <thread>

#include "she_internal.h"

namespace she {
namespace {

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;
enum : uint64_t { kTagLweKey = 1, kTagRingKey = 2, kTagBkRow = 3, kTagKsRow = 4, kTagFresh = 5, kTagTrgswRow = 6,
                  kTagTrlwe = 7 };

inline uint64_t finalise(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

struct Stream {
    uint64_t key;
    Stream(uint64_t seed, uint64_t tag, uint64_t index) : key(finalise(finalise(finalise(seed) + tag) + index)) {}
    uint64_t word(uint64_t c) const { return finalise(key + (c + 1) * kGolden); }
    uint32_t torus(uint64_t c) const { return (uint32_t)(word(c) >> 32); }
    uint8_t bit(uint64_t c) const { return (uint8_t)(word(c) >> 63); }
    uint32_t gaussian(uint64_t c, double sigma) const
    {
        const double unit = 1.0 / 9007199254740992.0;   // 2^-53
        const double u1 = (double)((word(c) >> 11) + 1) * unit;
        const double u2 = (double)(word(c + 1) >> 11) * unit;
        const double radius = std::sqrt(-2.0 * std::log(u1));
        const double normal = radius * std::cos(6.283185307179586476925286766559 * u2);
        double scaled = normal * sigma;
        scaled *= 4294967296.0;
        return (uint32_t)(int64_t)std::llround(scaled);
    }
};

template <class F> void parallel_for(size_t count, F &&body)
{
    unsigned hw = std::thread::hardware_concurrency();
    size_t workers = std::min<size_t>(std::max(1u, std::min(hw, 16u)), count ? count : 1);
    if (workers <= 1) {
        for (size_t i = 0; i < count; i++) body(i);
        return;
    }
    std::vector<std::thread> pool;
    for (size_t w = 0; w < workers; w++)
        pool.emplace_back([&, w] {
            for (size_t i = w; i < count; i += workers) body(i);
        });
    for (auto &th : pool) th.join();
}

// TLWE sample under `key`: words 0..n-1 of the stream are the mask, words n, n+1 feed the error.
void tlwe_sample(uint32_t n, const uint8_t *key, uint32_t message, double sigma, const Stream &st, uint32_t *out)
{
    uint32_t body = message + st.gaussian(n, sigma);
    for (uint32_t i = 0; i < n; i++) {
        const uint32_t a = st.torus(i);
        out[i] = a;
        body += key[i] ? a : 0u;
    }
    out[n] = body;
}

// TRLWE sample of zero under the ring key whose set bits are listed in `ones`: words 0..N-1 of the
// stream are the mask A, word N+2j feeds the error of body coefficient j; B = A*s' + E.
void trlwe_of_zero(uint32_t N, const std::vector<uint32_t> &ones, const Stream &st, double sigma, uint32_t *A, uint32_t *B)
{
    for (uint32_t j = 0; j < N; j++) {
        A[j] = st.torus(j);
        B[j] = st.gaussian(N + 2 * (uint64_t)j, sigma);
    }
    // B += A * s' in Z[X]/(X^N+1): each set key bit adds a negacyclic rotation of A
    for (uint32_t s : ones) {
        for (uint32_t j = 0; j < N - s; j++) B[j + s] += A[j];
        for (uint32_t j = N - s; j < N; j++) B[j + s - N] -= A[j];
    }
}

std::vector<uint32_t> set_bits(const std::vector<uint8_t> &key)
{
    std::vector<uint32_t> ones;
    for (uint32_t j = 0; j < key.size(); j++)
        if (key[j]) ones.push_back(j);
    return ones;
}

}  // namespace

void generate_keys(const she_params &P, uint64_t seed, HostKeys &K)
{
    const uint32_t n = P.n, N = P.N, l = P.l;
    K.lwe_key.resize(n);
    K.ring_key.resize(N);
    {
        Stream s(seed, kTagLweKey, 0);
        for (uint32_t i = 0; i < n; i++) K.lwe_key[i] = s.bit(i);
        Stream r(seed, kTagRingKey, 0);
        for (uint32_t j = 0; j < N; j++) K.ring_key[j] = r.bit(j);
    }
    const std::vector<uint32_t> ones = set_bits(K.ring_key);

    // Bootstrapping key: BK_i = TRGSW(s_i) as 2l TRLWE rows.  Row (c, p) is (A, A*s' + E) with
    // s_i * Bg^-(p+1) added to the constant coefficient of component c.
    K.bk.assign((size_t)n * 2 * l * 2 * N, 0u);
    parallel_for((size_t)n * 2 * l, [&](size_t row) {
        const uint32_t i = (uint32_t)(row / (2 * l)), c = (uint32_t)(row / l) & 1u, p = (uint32_t)(row % l);
        uint32_t *A = K.bk.data() + row * 2 * N, *B = A + N;
        trlwe_of_zero(N, ones, Stream(seed, kTagBkRow, row), P.bk_std, A, B);
        if (K.lwe_key[i]) (c ? B : A)[0] += 1u << (32 - (p + 1) * P.bg_bit);
    });

    // Key-switching key: for ring-key bit i, digit position j and digit value v a TLWE
    // encryption of v * s'_i / base^(j+1), every row with its own noise.
    const uint32_t base = 1u << P.ks_basebit, rows_per = base - 1;
    K.ks.assign((size_t)N * P.ks_t * rows_per * (n + 1), 0u);
    parallel_for((size_t)N * P.ks_t * rows_per, [&](size_t row) {
        const uint32_t v = (uint32_t)(row % rows_per) + 1;
        const uint32_t j = (uint32_t)(row / rows_per) % P.ks_t;
        const uint32_t i = (uint32_t)(row / rows_per / P.ks_t);
        const uint32_t msg = K.ring_key[i] ? v << (32 - (j + 1) * P.ks_basebit) : 0u;
        tlwe_sample(n, K.lwe_key.data(), msg, P.lwe_std, Stream(seed, kTagKsRow, row), K.ks.data() + row * (n + 1));
    });
}

void fresh_samples(const she_params &P, const std::vector<uint8_t> &lwe_key, const uint8_t *bits, size_t nbits,
                   uint64_t enc_seed, uint32_t *out)
{
    parallel_for(nbits, [&](size_t k) {
        const uint32_t msg = bits[k] ? (1u << 29) : 0u - (1u << 29);
        tlwe_sample(P.n, lwe_key.data(), msg, P.lwe_std, Stream(enc_seed, kTagFresh, k), out + k * (P.n + 1));
    });
}

void fresh_trgsw(const she_params &P, const std::vector<uint8_t> &ring_key, const uint8_t *bits, size_t count,
                 uint64_t seed, uint32_t *out)
{
    const uint32_t N = P.N, l = P.l;
    const std::vector<uint32_t> ones = set_bits(ring_key);
    parallel_for(count * 2 * l, [&](size_t row) {
        const size_t k = row / (2 * l);
        const uint32_t c = (uint32_t)(row / l) & 1u, p = (uint32_t)(row % l);
        uint32_t *A = out + row * 2 * N, *B = A + N;
        trlwe_of_zero(N, ones, Stream(seed, kTagTrgswRow, row), P.bk_std, A, B);
        if (bits[k]) (c ? B : A)[0] += 1u << (32 - (p + 1) * P.bg_bit);
    });
}

void fresh_trlwe(const she_params &P, const std::vector<uint8_t> &ring_key, const uint32_t *mu, size_t count,
                 uint64_t seed, uint32_t *out)
{
    const uint32_t N = P.N;
    const std::vector<uint32_t> ones = set_bits(ring_key);
    parallel_for(count, [&](size_t k) {
        uint32_t *A = out + k * 2 * N, *B = A + N;
        trlwe_of_zero(N, ones, Stream(seed, kTagTrlwe, k), P.bk_std, A, B);
        for (uint32_t j = 0; j < N; j++) B[j] += mu[k * N + j];
    });
}

void trlwe_phases(const she_params &P, const std::vector<uint8_t> &ring_key, const uint32_t *cts, size_t count,
                  uint32_t *phases)
{
    const uint32_t N = P.N;
    const std::vector<uint32_t> ones = set_bits(ring_key);
    parallel_for(count, [&](size_t k) {
        const uint32_t *A = cts + k * 2 * N, *B = A + N;
        uint32_t *ph = phases + k * N;
        for (uint32_t j = 0; j < N; j++) ph[j] = B[j];
        for (uint32_t s : ones) {
            for (uint32_t j = 0; j < N - s; j++) ph[j + s] -= A[j];
            for (uint32_t j = N - s; j < N; j++) ph[j + s - N] += A[j];
        }
    });
}

void pack_ks_bytes(const she_params &P, const std::vector<uint32_t> &ks, uint32_t cols_p, std::vector<int8_t> &out)
{
    // word = s0 + 256*s1 + 256^2*s2 + 256^3*s3 (mod 2^32) with every s in [-128, 127]
    const uint32_t n = P.n, t = P.ks_t, rows_per = (1u << P.ks_basebit) - 1, kk = t * (rows_per + 1);
    out.assign((size_t)P.N * 4 * cols_p * kk, 0);
    parallel_for(P.N, [&](size_t i) {
        for (uint32_t j = 0; j < t; j++)
            for (uint32_t v = 1; v <= rows_per; v++) {
                const uint32_t *row = ks.data() + (((size_t)i * t + j) * rows_per + (v - 1)) * (n + 1);
                for (uint32_t c = 0; c <= n; c++) {
                    uint32_t w = row[c];
                    for (uint32_t plane = 0; plane < 4; plane++) {
                        const int8_t s = (int8_t)(w & 0xffu);
                        w = (w - (uint32_t)(int32_t)s) >> 8;
                        out[(((size_t)i * 4 + plane) * cols_p + c) * kk + j * (rows_per + 1) + v] = s;
                    }
                }
            }
    });
}

void phases_to_bits(const she_params &P, const std::vector<uint8_t> &lwe_key, const uint32_t *cts, size_t count,
                    uint8_t *bits)
{
    parallel_for(count, [&](size_t k) {
        const uint32_t *ct = cts + k * (P.n + 1);
        uint32_t phase = ct[P.n];
        for (uint32_t i = 0; i < P.n; i++) phase -= lwe_key[i] ? ct[i] : 0u;
        bits[k] = (int32_t)phase > 0;
    });
}

}  // namespace she
