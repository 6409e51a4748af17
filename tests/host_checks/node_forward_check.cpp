// Host emulation of the node-ordered forward transform of negacyclic_fft.h for N = 1024: the 64 lanes of a transform
// are looped over, the LDS exchange is an array, and the passes, table rows and index rules are the header's own
// (node_pass, make_twiddles, first_pass_entry, the exchange's store row and load slot).  Checked against the
// definition X_k = sum_j u_j exp(2 pi i j (4k+1) / (4M)) in long double, in the layout that the inverse transform and
// the key spectra use: lane 8*k0 + k1, register k2 <-> k = k0 + 8 k1 + 64 k2.  Built and run by tests/test_host_fft.py.
#include <cmath>
#include <complex>
#include <cstdio>
#include <vector>

#include "negacyclic_fft.h"

using namespace she;
using PL = Plan<3, 3>;

int main()
{
    constexpr int P = PL::P, L = PL::L, M = PL::M, K = PL::K, LOGP = PL::LOGP, ROW = P / 2;
    static_assert(TwTable<PL>::NODE_FORWARD, "this plan uses the node-ordered forward transform");
    std::vector<double> tw(2 * (size_t)TwTable<PL>::COUNT);
    make_twiddles<PL>(tw.data());
    // the compile-time constants of the first pass against libm
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
    // input: small signed integers like gadget digits, and one run with large values like key words
    double worst = 0;
    for (int trial = 0; trial < 3; trial++) {
        std::vector<std::complex<long double>> u(M);
        unsigned long long st = 88172645463325252ull + trial;
        auto rnd = [&]() { st ^= st << 13; st ^= st >> 7; st ^= st << 17; return st; };
        for (int j = 0; j < M; j++) {
            const long double scale = trial == 2 ? 33554432.0L : 1.0L;
            u[j] = {(long double)((long long)(rnd() % 128) - 64) * scale, (long double)((long long)(rnd() % 128) - 64) * scale};
        }
        static double xr[L][P], xi[L][P];
        for (int t = 0; t < L; t++)
            for (int m = 0; m < P; m++) { xr[t][m] = (double)u[t + L * m].real(); xi[t][m] = (double)u[t + L * m].imag(); }
        static double bufr[PL::XSLOTS], bufi[PL::XSLOTS];
        for (int pass = 0; pass < K; pass++) {
            for (int t = 0; t < L; t++) {
                CosTan e[ROW];
                if (pass == 0) {
                    for (int stg = 0; stg < LOGP; stg++)
                        for (int i = 0; i < (stg == 0 ? 1 : 1 << (stg - 1)); i++)
                            e[stg == 0 ? 0 : (1 << (stg - 1)) + i] = first_pass_entry(stg, i);
                } else {
                    const int lane_part = t / ipow(P, K - 1 - pass);
                    const double *row = tw.data() + 2 * ((size_t)TwTable<PL>::node_offset(pass) + (size_t)ROW * lane_part);
                    for (int i = 0; i < ROW; i++) { e[i].c = row[2 * i]; e[i].t = row[2 * i + 1]; }
                }
                node_pass<P>(xr[t], xi[t], e);
            }
            if (pass == K - 1) break;
            for (int t = 0; t < L; t++)
                for (int m = 0; m < P; m++) { bufr[brev(m, LOGP) * PL::XROW + t] = xr[t][m]; bufi[brev(m, LOGP) * PL::XROW + t] = xi[t][m]; }
            const int Ts = ipow(P, K - 1 - pass), Tn = Ts / P;
            for (int t = 0; t < L; t++) {
                const int q = t / Tn, tn = t % Tn, ks = q % P, kap = q / P;
                const int rd_base = ks * PL::XROW + tn + Ts * kap;
                for (int m = 0; m < P; m++) { xr[t][m] = bufr[rd_base + m * Tn]; xi[t][m] = bufi[rd_base + m * Tn]; }
            }
        }
        // register m holds frequency digit brev(m)
        long double scale = trial == 2 ? 33554432.0L : 1.0L;
        for (int t = 0; t < L; t++)
            for (int m = 0; m < P; m++) {
                const int k0 = t / 8, k1 = t % 8, k2 = brev(m, LOGP), k = k0 + 8 * k1 + 64 * k2;
                std::complex<long double> want = 0;
                for (int j = 0; j < M; j++) {
                    const long double ang = 2 * pi * (long double)((long long)j * (4 * k + 1) % (4 * M)) / (long double)(4 * M);
                    want += u[j] * std::complex<long double>(cosl(ang), sinl(ang));
                }
                const double err = (double)(std::abs(std::complex<long double>(xr[t][m], xi[t][m]) - want) / scale);
                if (err > worst) worst = err;
            }
    }
    std::printf("node-ordered forward transform, N = 1024: largest error %.3g (digit-sized inputs, relative to the input scale)\n", worst);
    if (worst > 1e-9) bad++;
    std::printf("failures %d\n", bad);
    return bad ? 1 : 0;
}
