// Host emulation of the ring-degree-2048 transforms of negacyclic_fft.h: the 64 lanes are looped over, the LDS
// exchange is an array, and the stages, table rows and index rules are the header's own (node_pass,
// node_pass_inverse, make_twiddles, first_pass_entries16, the exchange's store row and load slot).  Checks:
//   1. the forward transform against its definition X_k = sum_j u_j exp(2 pi i j (4k+1) / (4M)) in long double, in
//      the layout the kernels use (lane 8 k0 + k1, register 8 h + k2 <-> k = h + 2 k0 + 16 k1 + 128 k2);
//   2. inverse(forward(u)) = u;
//   3. a product in Z[X]/(X^2048 + 1) of a digit-sized polynomial and a Torus32-sized one through the transforms
//      against the schoolbook negacyclic product in 128-bit integers: every coefficient rounds to the exact integer.
// Built and run by tests/test_host_fft.py.
#include <cmath>
#include <complex>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "negacyclic_fft.h"

using namespace she;
using PL = Plan2048;
constexpr int P = PL::P, L = PL::L, M = PL::M, N = PL::N, H = PL::XP, LOGH = PL::LOGXP;

static std::vector<double> g_tw;

struct Lanes { double r[L][P], i[L][P]; };

static int rd_base(int t, int s)
{
    const int Ts = ipow(H, PL::K - 1 - s), Tn = Ts / H;
    const int q = t / Tn, tn = t % Tn, ks = q % H, kap = q / H;
    return ks * PL::xrow(s) + tn + Ts * kap;
}

static void entries(int t, int pass, int h, CosTan (&e)[4])
{
    const int R = pass == 1 ? h + 2 * (t >> 3) : h + 2 * (t >> 3) + 16 * (t & 7);
    const double *row = g_tw.data() + 2 * ((size_t)TwTable<PL>::node_offset(pass) + 4 * (size_t)R);
    for (int q = 0; q < 4; q++) { e[q].c = row[2 * q]; e[q].t = row[2 * q + 1]; }
}

static void forward_emulated(Lanes &x)
{
    CosTan e0[8];
    first_pass_entries16(e0);
    for (int t = 0; t < L; t++) node_pass<16>(x.r[t], x.i[t], e0);
    static double br[PL::XSLOTS], bi[PL::XSLOTS];
    for (int pass = 1; pass < 3; pass++) {
        const int Tn = ipow(H, 2 - pass);
        for (int h = 0; h < 2; h++) {
            for (int t = 0; t < L; t++)
                for (int m = 0; m < H; m++) { br[brev(m, LOGH) * PL::xrow(pass - 1) + t] = x.r[t][H * h + m]; bi[brev(m, LOGH) * PL::xrow(pass - 1) + t] = x.i[t][H * h + m]; }
            for (int t = 0; t < L; t++) {
                for (int m = 0; m < H; m++) { x.r[t][H * h + m] = br[rd_base(t, pass - 1) + m * Tn]; x.i[t][H * h + m] = bi[rd_base(t, pass - 1) + m * Tn]; }
                CosTan e[4];
                entries(t, pass, h, e);
                node_pass<H>(*reinterpret_cast<double(*)[H]>(&x.r[t][H * h]), *reinterpret_cast<double(*)[H]>(&x.i[t][H * h]), e);
            }
        }
    }
    for (int t = 0; t < L; t++)
        for (int h = 0; h < 2; h++) {
            double yr[H], yi[H];
            for (int m = 0; m < H; m++) { yr[brev(m, LOGH)] = x.r[t][H * h + m]; yi[brev(m, LOGH)] = x.i[t][H * h + m]; }
            for (int m = 0; m < H; m++) { x.r[t][H * h + m] = yr[m]; x.i[t][H * h + m] = yi[m]; }
        }
}

static void inverse_emulated(Lanes &x)
{
    for (int t = 0; t < L; t++)
        for (int h = 0; h < 2; h++) {
            double yr[H], yi[H];
            for (int m = 0; m < H; m++) { yr[m] = x.r[t][H * h + brev(m, LOGH)]; yi[m] = x.i[t][H * h + brev(m, LOGH)]; }
            for (int m = 0; m < H; m++) { x.r[t][H * h + m] = yr[m]; x.i[t][H * h + m] = yi[m]; }
        }
    static double br[PL::XSLOTS], bi[PL::XSLOTS];
    for (int pass = 2; pass >= 1; pass--) {
        const int Tn = ipow(H, 2 - pass);
        for (int h = 0; h < 2; h++) {
            for (int t = 0; t < L; t++) {
                CosTan e[4];
                entries(t, pass, h, e);
                node_pass_inverse<H>(*reinterpret_cast<double(*)[H]>(&x.r[t][H * h]), *reinterpret_cast<double(*)[H]>(&x.i[t][H * h]), e);
                for (int m = 0; m < H; m++) { br[rd_base(t, pass - 1) + m * Tn] = x.r[t][H * h + m]; bi[rd_base(t, pass - 1) + m * Tn] = x.i[t][H * h + m]; }
            }
            for (int t = 0; t < L; t++)
                for (int m = 0; m < H; m++) { x.r[t][H * h + m] = br[brev(m, LOGH) * PL::xrow(pass - 1) + t]; x.i[t][H * h + m] = bi[brev(m, LOGH) * PL::xrow(pass - 1) + t]; }
        }
    }
    CosTan e0[8];
    first_pass_entries16(e0);
    for (int t = 0; t < L; t++) {
        node_pass_inverse<16>(x.r[t], x.i[t], e0);
        for (int m = 0; m < P; m++) { x.r[t][m] /= M; x.i[t][m] /= M; }
    }
}

// folded polynomial: u_j = a_j + i a_{j+M} at lane j % 64, register j / 64
static void fold(const std::vector<long long> &a, Lanes &x)
{
    for (int j = 0; j < M; j++) { x.r[j % L][j / L] = (double)a[j]; x.i[j % L][j / L] = (double)a[j + M]; }
}

int main()
{
    g_tw.resize(2 * (size_t)TwTable<PL>::COUNT);
    make_twiddles<PL>(g_tw.data());
    const long double pi = 3.14159265358979323846264338327950288L;
    int bad = 0;
    for (int e = 0; e < 4; e++)
        for (int i = 0; i < (e == 0 ? 1 : 1 << (e - 1)); i++) {
            const long double a = pi * node_angle(e, i);
            const CosTan v = first_pass_entry(e, i);
            if (v.c != (double)cosl(a) || std::fabs(v.t - (double)tanl(a)) > 4e-16 * std::fabs(v.t)) {
                std::printf("first-pass constant (%d, %d) is off: %.20g %.20g\n", e, i, v.c, v.t);
                bad++;
            }
        }
    unsigned long long st = 88172645463325252ull;
    auto rnd = [&]() { st ^= st << 13; st ^= st >> 7; st ^= st << 17; return st; };
    // 1 + 2: forward against the definition, and the round trip
    static Lanes x, x0;
    std::vector<long long> a(N);
    for (int j = 0; j < N; j++) a[j] = (long long)(rnd() % 128) - 64;
    fold(a, x);
    x0 = x;
    forward_emulated(x);
    double worst = 0;
    for (int t = 0; t < L; t++)
        for (int m = 0; m < P; m++) {
            const int h = m / H, k2 = m % H, k = h + 2 * (t / 8) + 16 * (t % 8) + 128 * k2;
            std::complex<long double> want = 0;
            for (int j = 0; j < M; j++) {
                const long double ang = 2 * pi * (long double)((long long)j * (4 * k + 1) % (4 * M)) / (long double)(4 * M);
                want += std::complex<long double>((long double)a[j], (long double)a[j + M]) * std::complex<long double>(cosl(ang), sinl(ang));
            }
            worst = std::fmax(worst, (double)std::abs(std::complex<long double>(x.r[t][m], x.i[t][m]) - want));
        }
    std::printf("forward transform, N = 2048: largest error against the definition %.3g\n", worst);
    if (worst > 1e-8) bad++;
    inverse_emulated(x);
    worst = 0;
    for (int t = 0; t < L; t++)
        for (int m = 0; m < P; m++) worst = std::fmax(worst, std::fmax(std::fabs(x.r[t][m] - x0.r[t][m]), std::fabs(x.i[t][m] - x0.i[t][m])));
    std::printf("inverse of forward: largest deviation %.3g\n", worst);
    if (worst > 1e-9) bad++;
    // 3: products with every digit at full magnitude and Torus32-sized key words: 6 rows summed like an external product
    static Lanes acc, d, k;
    for (int t = 0; t < L; t++) for (int m = 0; m < P; m++) acc.r[t][m] = acc.i[t][m] = 0;
    std::vector<std::vector<long long>> dig(6, std::vector<long long>(N)), key(6, std::vector<long long>(N));
    for (int r = 0; r < 6; r++) {
        for (int j = 0; j < N; j++) { dig[r][j] = (rnd() & 1) ? 63 : -64; key[r][j] = (long long)(int32_t)(uint32_t)rnd(); }
        fold(dig[r], d); fold(key[r], k);
        forward_emulated(d); forward_emulated(k);
        for (int t = 0; t < L; t++)
            for (int m = 0; m < P; m++) {
                acc.r[t][m] += d.r[t][m] * k.r[t][m] - d.i[t][m] * k.i[t][m];
                acc.i[t][m] += d.r[t][m] * k.i[t][m] + d.i[t][m] * k.r[t][m];
            }
    }
    inverse_emulated(acc);
    double off = 0;
    int wrong = 0;
    for (int j = 0; j < N; j += 1) {
        if (j % 37 && j != N - 1) continue;                               // a spread of coefficients, both halves
        __int128 exact = 0;
        for (int r = 0; r < 6; r++)
            for (int i = 0; i < N; i++) {
                const int jj = j - i;
                exact += (jj >= 0) ? (__int128)dig[r][i] * key[r][jj] : -(__int128)dig[r][i] * key[r][jj + N];
            }
        const double got = j < M ? acc.r[j % L][j / L] : acc.i[(j - M) % L][(j - M) / L];
        off = std::fmax(off, std::fabs(got - std::rint(got)));
        if ((__int128)std::llrint(got) != exact) wrong++;
    }
    std::printf("sum of 6 products, worst-case digits: largest distance from an integer %.4f, wrong coefficients %d\n", off, wrong);
    if (wrong || off > 0.2) bad++;
    std::printf("failures %d\n", bad);
    return bad ? 1 : 0;
}
