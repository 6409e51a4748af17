// In-register negacyclic transform for gfx950 wavefronts.
//
// A real polynomial a(X) of degree < N in R[X]/(X^N+1) is folded to M = N/2 complex
// numbers u_j = a_j + i*a_{j+M}, twisted by psi^j (psi = exp(i*pi/N)) and sent through an
// M-point complex DFT with kernel exp(+2*pi*i*jk/M).  The result is a(X) evaluated at the
// M roots psi^(4k+1) of X^N+1 (the other M roots are their conjugates), so a product in
// the ring is a pointwise complex product there.
//
// Mapping: M = P^K.  One transform is spread over L = M/P lanes of a wavefront, each lane
// holding P complex points in registers; 64/L transforms run side by side in one
// wavefront.  The forward transform is K decimation-in-frequency passes of radix P with
// K-1 transpositions through a wave-private LDS buffer; its output order is digit-reversed
// and is never undone: the inverse transform is the exact mirror (decimation in time), so
// it takes that order as input and returns coefficients to the lane and register they
// were read from.  The twist and the first pass share one per-lane twiddle.
#pragma once
#include <hip/hip_runtime.h>
// device arithmetic may fuse multiply-adds (the host's key generation is compiled without fusion)
#pragma clang fp contract(fast)
#include <stdint.h>
#include <cmath>

namespace she {

// cos(pi*k/64), k = 0..32
__host__ __device__ constexpr double cos_pi64_q(int k)
{
    constexpr double t[33] = {
        1.0, 0.9987954562051724, 0.9951847266721969, 0.989176509964781, 0.9807852804032304, 0.970031253194544,
        0.9569403357322088, 0.9415440651830208, 0.9238795325112867, 0.9039892931234433, 0.881921264348355,
        0.8577286100002721, 0.8314696123025452, 0.8032075314806449, 0.773010453362737, 0.7409511253549591,
        0.7071067811865476, 0.6715589548470183, 0.6343932841636455, 0.5956993044924335, 0.5555702330196023,
        0.5141027441932217, 0.4713967368259978, 0.4275550934302822, 0.38268343236508984, 0.33688985339222005,
        0.29028467725446233, 0.24298017990326398, 0.19509032201612833, 0.14673047445536175, 0.09801714032956077,
        0.049067674327418126, 0.0};
    return t[k];
}
// cos / sin of pi*a/64 for any integer a
__host__ __device__ constexpr double cos_pi64(int a)
{
    a = ((a % 128) + 128) % 128;
    if (a > 64) a = 128 - a;                     // cos is even about pi
    return a <= 32 ? cos_pi64_q(a) : -cos_pi64_q(64 - a);
}
__host__ __device__ constexpr double sin_pi64(int a) { return cos_pi64(a - 32); }

constexpr int ipow(int b, int e) { return e == 0 ? 1 : b * ipow(b, e - 1); }
constexpr int brev(int v, int bits) { int r = 0; for (int i = 0; i < bits; i++) r |= ((v >> i) & 1) << (bits - 1 - i); return r; }

template <int LOGP_, int K_> struct Plan {
    static constexpr int LOGP = LOGP_;
    static constexpr int K = K_;                      // passes
    static constexpr int P = 1 << LOGP;               // points per lane, radix of every pass
    static constexpr int M = ipow(P, K);              // complex length
    static constexpr int N = 2 * M;                   // ring degree
    static constexpr int L = M / P;                   // lanes per transform
    static constexpr int GPW = 64 / L;                // transforms (gates) per wavefront
    static constexpr int XROW = L + 1;                // padded row of the exchange buffer, 16-byte slots
                                                      // (measured: +0 costs 18 %, +8 17 %, +2 +3 +4 +5 +9 are no better than +1)
    // Row length of the exchange that follows pass s.  LDS serves sixteen lanes' 16-byte reads per clock when they fall
    // into sixteen different slots modulo 16.  With eight points per lane and three passes, lane 8a + b reads slots
    // a*row + b + 8m after the first pass (row = 8 mod 16 keeps neighbouring a apart: measured 575 against 203 B/ns per
    // compute unit with row = 65) and b*row + 8a + m after the second (any odd row: 550 B/ns, 76 with row = 72), so
    // the two exchanges want different rows.  Writes (about 183 B/ns whatever the row) do not care.
    static constexpr int xrow(int s) { return (P == 8 && K == 3 && s == 0) ? L + 8 : L + 1; }
    static constexpr int XSLOTS = P * ((P == 8 && K == 3) ? L + 8 : L + 1);   // exchange slots per transform
    static constexpr int XP = P;                      // points that one exchange moves per lane
    static constexpr bool NODES = false;              // radix-P passes below; true: node-ordered stages (Plan2048)
    static_assert(L >= 1 && L <= 64 && 64 % L == 0, "one transform must fit a wavefront");
};

// Ring degree 2048: M = 1024 complex points, 16 per lane on 64 lanes, which is not a power of the radix.  The top
// position bit stays in the register index for the whole transform: the first pass couples the two halves and then
// each half of 512 points (8 registers) goes through the two exchanges of the 512-point plan on its own, through the
// same buffer one after the other.  All stages are the node-ordered butterflies described below.
struct Plan2048 {
    static constexpr int LOGP = 4, P = 16, K = 3, M = 1024, N = 2048, L = 64, GPW = 1;
    static constexpr int XP = 8, LOGXP = 3;           // one half
    static constexpr int XROW = L + 1;
    static constexpr int xrow(int s) { return s == 0 ? L + 8 : L + 1; }   // as in the 512-point plan, whose exchanges these are
    static constexpr int XSLOTS = XP * (L + 8);
    static constexpr bool NODES = true;
};

// ---- radix-P DFT on registers ------------------------------------------------------------
// y_k = sum_m x_m exp(SIGN*2*pi*i*k*m/P), decimation in frequency; y_k is left at position
// brev(k) and handed back in natural order by a compile-time register renaming.
template <int P, int SIGN> __host__ __device__ __forceinline__ void dft_regs(double (&xr)[P], double (&xi)[P])
{
    if constexpr (P == 8) {
        // Radix 8 written out.  The two outputs of the first stage that carry a factor 1/sqrt2 keep it pending
        // through the second stage (they only meet each other there) and it is applied inside the last stage's
        // additions as fused multiply-adds: 4 multiplications fewer than scaling them straight away.
        constexpr double h = 0.7071067811865476;
        constexpr double S = SIGN;
        // first stage: a_j = x_j + x_{j+4}, t_j = x_j - x_{j+4}
        const double a0r = xr[0] + xr[4], a0i = xi[0] + xi[4], t0r = xr[0] - xr[4], t0i = xi[0] - xi[4];
        const double a1r = xr[1] + xr[5], a1i = xi[1] + xi[5], t1r = xr[1] - xr[5], t1i = xi[1] - xi[5];
        const double a2r = xr[2] + xr[6], a2i = xi[2] + xi[6], t2r = xr[2] - xr[6], t2i = xi[2] - xi[6];
        const double a3r = xr[3] + xr[7], a3i = xi[3] + xi[7], t3r = xr[3] - xr[7], t3i = xi[3] - xi[7];
        // b_1 = h q_1, q_1 = (1 + S i) t_1;  b_3 = h q_3, q_3 = (-1 + S i) t_3;  b_2 = S i t_2
        const double q1r = t1r - S * t1i, q1i = t1i + S * t1r;
        const double q3r = -t3r - S * t3i, q3i = S * t3r - t3i;
        const double b2r = -S * t2i, b2i = S * t2r;
        // second stage, upper half
        const double c0r = a0r + a2r, c0i = a0i + a2i, c2r = a0r - a2r, c2i = a0i - a2i;
        const double c1r = a1r + a3r, c1i = a1i + a3i;
        const double u3r = a1r - a3r, u3i = a1i - a3i;             // times S i below
        const double c3r = -S * u3i, c3i = S * u3r;
        // second stage, lower half: d_1 = h e_1, d_3 = h e_3
        const double d0r = t0r + b2r, d0i = t0i + b2i, d2r = t0r - b2r, d2i = t0i - b2i;
        const double e1r = q1r + q3r, e1i = q1i + q3i;
        const double v3r = q1r - q3r, v3i = q1i - q3i;
        const double e3r = -S * v3i, e3i = S * v3r;
        // last stage; y_k in natural order
        xr[0] = c0r + c1r; xi[0] = c0i + c1i;
        xr[4] = c0r - c1r; xi[4] = c0i - c1i;
        xr[2] = c2r + c3r; xi[2] = c2i + c3i;
        xr[6] = c2r - c3r; xi[6] = c2i - c3i;
        xr[1] = __builtin_fma(h, e1r, d0r);  xi[1] = __builtin_fma(h, e1i, d0i);
        xr[5] = __builtin_fma(-h, e1r, d0r); xi[5] = __builtin_fma(-h, e1i, d0i);
        xr[3] = __builtin_fma(h, e3r, d2r);  xi[3] = __builtin_fma(h, e3i, d2i);
        xr[7] = __builtin_fma(-h, e3r, d2r); xi[7] = __builtin_fma(-h, e3i, d2i);
        return;
    }
    constexpr int LOGP = __builtin_ctz(P);
#pragma unroll
    for (int len = P; len >= 2; len >>= 1) {
        const int half = len >> 1;
#pragma unroll
        for (int base = 0; base < P; base += len) {
#pragma unroll
            for (int j = 0; j < half; j++) {
                const int a = base + j, b = a + half;
                const double tr = xr[a] - xr[b], ti = xi[a] - xi[b];
                xr[a] += xr[b];
                xi[a] += xi[b];
                if (j == 0) {
                    xr[b] = tr; xi[b] = ti;
                } else if (4 * j == len) {                       // multiply by SIGN*i
                    xr[b] = -SIGN * ti; xi[b] = SIGN * tr;
                } else if (8 * j == len) {                       // (1 + SIGN*i)/sqrt2
                    const double h = 0.7071067811865476;
                    xr[b] = (tr - SIGN * ti) * h; xi[b] = (ti + SIGN * tr) * h;
                } else if (8 * j == 3 * len) {                   // (-1 + SIGN*i)/sqrt2
                    const double h = 0.7071067811865476;
                    xr[b] = (-tr - SIGN * ti) * h; xi[b] = (SIGN * tr - ti) * h;
                } else {
                    const double wr = cos_pi64(128 * j / len), wi = SIGN * sin_pi64(128 * j / len);
                    xr[b] = tr * wr - ti * wi; xi[b] = tr * wi + ti * wr;
                }
            }
        }
    }
    double yr[P], yi[P];
#pragma unroll
    for (int k = 0; k < P; k++) { yr[k] = xr[brev(k, LOGP)]; yi[k] = xi[brev(k, LOGP)]; }
#pragma unroll
    for (int k = 0; k < P; k++) { xr[k] = yr[k]; xi[k] = yi[k]; }
}

// Orders LDS traffic of one wavefront: a wave's LDS operations complete in issue order,
// so only the compiler has to be kept from moving them across this point.  It is required:
// without it the compiler does reorder the exchange's stores and loads (other lanes' slots
// look independent to it) and results are wrong.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Twiddle table, shared by every transform of a workgroup (kept in LDS by the kernels).
// Pass s (0-based, s < K-1) multiplies output k of lane t by
//   s = 0: exp(i*pi*t*(1+4k)/N)                    (twist psi^t merged with the first pass)
//   s > 0: exp(2*pi*i*k*(t mod T)/(P*T)), T = P^(K-1-s)
// which depends on t only through t mod T, so pass s stores P*T entries: [k][t mod T].
template <class PL> struct TwTable {
    static constexpr int period(int s) { return ipow(PL::P, PL::K - 1 - s); }              // T of pass s
    static constexpr int offset(int s) { return s == 0 ? 0 : offset(s - 1) + PL::P * period(s - 1); }
    static constexpr int COUNT = PL::K > 1 ? offset(PL::K - 1) : 1;                          // complex entries
};

// Plan2048: rows of four entries (cos, tan) per value R of the node index that lane and half contribute:
// 16 rows for the second pass (stages 4-6), 128 rows for the third (stages 7-9).
template <> struct TwTable<Plan2048> {
    static constexpr int ROW = 4;
    static constexpr int node_offset(int pass) { return pass == 1 ? 0 : 16 * ROW; }
    static constexpr int COUNT = 16 * ROW + 128 * ROW;
};

// ---- node-ordered transform (used by Plan2048) -----------------------------------------------------------------
// The same transform X_k = sum_j u_j exp(2*pi*i*j*(4k+1)/(4M)) computed as m = log2(M) stages of radix-2 butterflies
// (a, b) -> (a + w b, a - w b) on positions j, j + M/2^(s+1) (stage s = 0..m-1), in place.  Splitting the sum by the
// top bit of j shows that the two halves are again sums of this form, of half the length, with the shift 1/4 replaced
// by (1/4 + r)/2^s, r = the s low bits of k that the earlier stages fixed: the butterflies of one such sub-sum (a
// "node") share ONE twiddle
//     w(s, r) = exp(i*pi*(1 + 4r) / 2^(s+2)),
// the twist needs no multiplication of its own, and no twiddle is trivial, so every butterfly is six fused
// multiply-adds with w = c*(1 + i*t):  p = b + i*t*b (2), a +- c*p (4).  Further w(s, r + 2^(s-1)) = i*w(s, r): a node
// whose most recently fixed bit is 1 uses its sibling's entry on i*b, which only renames and negates operands.
// Position q ends up holding X_k with k = the bits of q reversed.  With P points of a lane covering the top log2(P)
// position bits in the first pass and the exchanges of forward_n(), pass p's node index is r = R + (bits fixed inside
// the pass) * 2^(p*log2 P), R given by the lane; a lane needs P/2 entries per pass: for stage e of the pass, entry
// w(p*log2 P + e, R + 2^(p*log2 P) * (index of the node among those of the stage, most recent bit dropped)).
// The first pass has R = 0: compile-time constants.  The inverse transform undoes the stages in reverse order:
// (y0, y1) -> (y0 + y1, conj(w) (y0 - y1)), eight instructions, the factor 1/2 per stage collected into one 1/M.
// (For N = 1024 the forward half of this was built into the radix-8 plan and measured: 216 instead of 243 FP64
// instructions per transform, bit-exact, but 0.5-1 % slower, because its fused multiply-adds take three vector
// registers each, which issue about 17 % slower than the additions that dominate the radix-8 passes.)
struct CosTan { double c, t; };
__host__ __device__ inline long double node_angle(int s, int r)       // of w(s, r), in units of pi
{
    return (long double)(1 + 4 * r) / (long double)(1ll << (s + 2));
}
// constants of the first pass (R = 0): stage e entry i is w(e, i), i < max(1, 2^(e-1)); up to 16 points per lane
__host__ __device__ constexpr CosTan first_pass_entry(int e, int i)
{
    // cos and tan of pi*(1+4i)/2^(e+2): e=0: pi/4; e=1: pi/8; e=2: pi/16, 5pi/16; e=3: pi/32, 5pi/32, 9pi/32, 13pi/32
    constexpr CosTan v[8] = {
        {0.70710678118654752440, 1.0},
        {0.92387953251128675613, 0.41421356237309504880},
        {0.98078528040323044913, 0.19891236737965800691},
        {0.55557023301960222474, 1.49660576266548901760},
        {0.99518472667219688624, 0.09849140335716425308},
        {0.88192126434835502971, 0.53451113595079164641},
        {0.63439328416364549822, 1.21850352558797634479},
        {0.29028467725446236764, 3.29655820893832042688},
    };
    return v[e == 0 ? 0 : (1 << (e - 1)) + i];
}

// y0 = a + w*b -> a, y1 = a - w*b -> b, with w = c*(1 + i*t), or i times that when ROT
template <bool ROT>
__host__ __device__ __forceinline__ void node_butterfly(double &ar, double &ai, double &br, double &bi, double c, double t)
{
    double pr, pi;
    if (!ROT) { pr = __builtin_fma(-t, bi, br); pi = __builtin_fma(t, br, bi); }
    else      { pr = __builtin_fma(-t, br, -bi); pi = __builtin_fma(-t, bi, br); }       // (1 + i*t) * (i*b)
    const double sr = __builtin_fma(c, pr, ar), si = __builtin_fma(c, pi, ai);
    br = __builtin_fma(-c, pr, ar); bi = __builtin_fma(-c, pi, ai);
    ar = sr; ai = si;
}

// One pass: log2(P) stages on the P points of a lane; register index = the pass's position bits, top bit first fixed.
// e[] = the lane's P/2 entries in stage order (1, 1, 2, 4, ... per stage).
struct NoEmit { __host__ __device__ void operator()(int) const {} };
// `done(m)` is called for each register as soon as the last stage has produced it (the exchange stores go there, so that
// they overlap the remaining butterflies).
template <int P, class EMIT = NoEmit>
__host__ __device__ __forceinline__ void node_pass(double (&xr)[P], double (&xi)[P], const CosTan (&e)[P / 2], EMIT done = EMIT())
{
    constexpr int LOGP = __builtin_ctz(P);
#pragma unroll
    for (int st = 0; st < LOGP; st++) {
        const int half = P >> (st + 1);                  // distance of the pair
#pragma unroll
        for (int base = 0; base < P; base += 2 * half) {
            const int fixed = base / (2 * half);         // the st bits fixed so far, first fixed = highest
            // node index inside the pass = those bits reversed; its top (most recent) bit selects the rotated form
            int rev = 0;
            for (int i = 0; i < st; i++) rev |= ((fixed >> (st - 1 - i)) & 1) << i;
            const bool rot = st > 0 && ((rev >> (st - 1)) & 1);
            const int idx = st > 0 ? (rev & ((1 << (st - 1)) - 1)) : 0;
            const CosTan w = e[st == 0 ? 0 : (1 << (st - 1)) + idx];
#pragma unroll
            for (int j = 0; j < half; j++) {
                if (rot) node_butterfly<true>(xr[base + j], xi[base + j], xr[base + j + half], xi[base + j + half], w.c, w.t);
                else node_butterfly<false>(xr[base + j], xi[base + j], xr[base + j + half], xi[base + j + half], w.c, w.t);
                if (st == LOGP - 1) { done(base + j); done(base + j + half); }
            }
        }
    }
}

// a = y0 + y1, b = conj(w) * (y0 - y1) (twice the forward pass's inputs), w as in node_butterfly
template <bool ROT>
__host__ __device__ __forceinline__ void node_butterfly_inverse(double &ar, double &ai, double &br, double &bi, double c, double t)
{
    const double dr = ar - br, di = ai - bi;
    ar += br; ai += bi;
    const double gr = __builtin_fma(t, di, dr), gi = __builtin_fma(-t, dr, di);          // (1 - i*t) * d
    if (!ROT) { br = c * gr; bi = c * gi; }
    else      { br = c * gi; bi = -c * gr; }                                             // conj(i*w) = -i * conj(w)
}

// The mirror of node_pass: last stage first.
template <int P>
__host__ __device__ __forceinline__ void node_pass_inverse(double (&xr)[P], double (&xi)[P], const CosTan (&e)[P / 2])
{
    constexpr int LOGP = __builtin_ctz(P);
#pragma unroll
    for (int st = LOGP - 1; st >= 0; st--) {
        const int half = P >> (st + 1);
#pragma unroll
        for (int base = 0; base < P; base += 2 * half) {
            const int fixed = base / (2 * half);
            int rev = 0;
            for (int i = 0; i < st; i++) rev |= ((fixed >> (st - 1 - i)) & 1) << i;
            const bool rot = st > 0 && ((rev >> (st - 1)) & 1);
            const int idx = st > 0 ? (rev & ((1 << (st - 1)) - 1)) : 0;
            const CosTan w = e[st == 0 ? 0 : (1 << (st - 1)) + idx];
#pragma unroll
            for (int j = 0; j < half; j++) {
                if (rot) node_butterfly_inverse<true>(xr[base + j], xi[base + j], xr[base + j + half], xi[base + j + half], w.c, w.t);
                else node_butterfly_inverse<false>(xr[base + j], xi[base + j], xr[base + j + half], xi[base + j + half], w.c, w.t);
            }
        }
    }
}

template <class PL> inline void make_twiddles(double *out /* [TwTable::COUNT][2] */)
{
    if constexpr (PL::NODES) {
        // pass p = 1, 2 (stages s0 = 3p+1 ...): row R holds w(s0, R), w(s0+1, R), w(s0+2, R), w(s0+2, R + 2^s0)
        const long double pi = 3.14159265358979323846264338327950288L;
        for (int pass = 1; pass <= 2; pass++) {
            const int s0 = 3 * pass + 1, rows = 1 << s0;
            for (int R = 0; R < rows; R++) {
                double *row = out + 2 * ((size_t)TwTable<PL>::node_offset(pass) + (size_t)R * TwTable<PL>::ROW);
                const int st[4] = {s0, s0 + 1, s0 + 2, s0 + 2}, rr[4] = {R, R, R, R + rows};
                for (int q = 0; q < 4; q++) {
                    const long double ang = pi * node_angle(st[q], rr[q]);
                    row[2 * q] = (double)cosl(ang);
                    row[2 * q + 1] = (double)tanl(ang);
                }
            }
        }
        return;
    } else {
    const long double pi = 3.14159265358979323846264338327950288L;
    for (int s = 0; s + 1 < PL::K; s++) {
        const int T = TwTable<PL>::period(s);
        for (int k = 0; k < PL::P; k++)
            for (int t = 0; t < T; t++) {
                const long double ang = s == 0 ? pi * (long double)t * (1 + 4 * k) / (long double)PL::N
                                               : 2.0L * pi * (long double)k * t / (long double)(PL::P * T);
                double *o = out + 2 * ((size_t)TwTable<PL>::offset(s) + (size_t)k * T + t);
                o[0] = (double)cosl(ang);
                o[1] = (double)sinl(ang);
            }
    }
    }
}

// Per-lane view of a transform: exchange addresses and where this lane's twiddles start.
template <class PL> struct LaneCtx {
    static constexpr int NP = PL::K > 1 ? PL::K - 1 : 1;
    int rd_base[NP];        // slot read by this lane after pass s (register m adds m*T_{s+1})
    int t;                  // lane within the transform
    double2 *xch;           // this transform's exchange buffer (XSLOTS slots)
    const double2 *tw;      // the workgroup's twiddle table in LDS

    __device__ __forceinline__ void init(int lane_in_transform, double2 *xbuf, const double2 *tw_lds)
    {
        t = lane_in_transform;
        xch = xbuf;
        tw = tw_lds;
#pragma unroll
        for (int s = 0; s < PL::K - 1; s++) {
            const int Ts = ipow(PL::XP, PL::K - 1 - s);      // sub-transform length after pass s
            const int Tn = Ts / PL::XP;
            const int q = t / Tn, tn = t % Tn, ks = q % PL::XP, kap = q / PL::XP;
            rd_base[s] = ks * PL::xrow(s) + tn + Ts * kap;
        }
    }
    // twiddle of pass s, output k
    __device__ __forceinline__ double2 twiddle(int s, int k) const
    {
        const int T = TwTable<PL>::period(s);
        return tw[TwTable<PL>::offset(s) + k * T + (t & (T - 1))];
    }
};

// Copies the twiddle table from device memory to the workgroup's LDS copy (all threads, then a barrier).
template <class PL> __device__ __forceinline__ void load_twiddles(double2 *lds, const double2 *__restrict__ global_table)
{
    for (int e = threadIdx.x; e < TwTable<PL>::COUNT; e += blockDim.x) lds[e] = global_table[e];
    __syncthreads();
}

// ---- Plan2048: node-ordered transforms on two halves -------------------------------------------------------------
// Register m = 8h + m8 holds position t + 64 m: h is the top position bit (the lowest frequency bit once the first
// stage has run), m8 the next three.  After the transform lane t = 8 k0 + k1, register 8h + k2 holds the frequency
// k = h + 2 k0 + 16 k1 + 128 k2.
template <class PL> __device__ __forceinline__ void half_entries(const LaneCtx<PL> &lc, int pass, int h, CosTan (&e)[4])
{
    // node index that the lane and the half contribute: pass 1: h + 2 k0; pass 2: h + 2 k0 + 16 k1
    const int R = pass == 1 ? h + 2 * (lc.t >> 3) : h + 2 * (lc.t >> 3) + 16 * (lc.t & 7);
    const double2 *row = lc.tw + TwTable<PL>::node_offset(pass) + 4 * R;
#pragma unroll
    for (int i = 0; i < 4; i++) { const double2 v = row[i]; e[i].c = v.x; e[i].t = v.y; }
}

__host__ __device__ __forceinline__ void first_pass_entries16(CosTan (&e)[8])
{
#pragma unroll
    for (int st = 0; st < 4; st++)
#pragma unroll
        for (int i = 0; i < (st == 0 ? 1 : 1 << (st - 1)); i++) e[st == 0 ? 0 : (1 << (st - 1)) + i] = first_pass_entry(st, i);
}

template <class PL, int NB>
__device__ __forceinline__ void forward_halves(const LaneCtx<PL> &lc, double2 *const (&xch)[NB], double (&xr)[NB][PL::P],
                                               double (&xi)[NB][PL::P])
{
    constexpr int H = PL::XP, LOGH = PL::LOGXP;
    static_assert(PL::P == 2 * H && PL::K == 3, "two halves, three passes");
    {
        CosTan e0[8];
        first_pass_entries16(e0);
#pragma unroll
        for (int b = 0; b < NB; b++) node_pass<16>(xr[b], xi[b], e0);
    }
#pragma unroll
    for (int pass = 1; pass < 3; pass++) {
        const int Tn = ipow(H, 2 - pass);                    // 8 after the first pass, 1 after the second
#pragma unroll
        for (int h = 0; h < 2; h++) {
            CosTan e[4];
            half_entries<PL>(lc, pass, h, e);                // requested before the exchange: they arrive with it
#pragma unroll
            for (int b = 0; b < NB; b++) {
                double(&r)[H] = *reinterpret_cast<double(*)[H]>(&xr[b][H * h]);
                double(&i)[H] = *reinterpret_cast<double(*)[H]>(&xi[b][H * h]);
                wave_lds_fence();
#pragma unroll
                for (int m = 0; m < H; m++) xch[b][brev(m, LOGH) * PL::xrow(pass - 1) + lc.t] = make_double2(r[m], i[m]);
                wave_lds_fence();
#pragma unroll
                for (int m = 0; m < H; m++) {
                    const double2 v = xch[b][lc.rd_base[pass - 1] + m * Tn];
                    r[m] = v.x; i[m] = v.y;
                }
                node_pass<H>(r, i, e);
            }
        }
    }
    // register m8 of a half holds the frequency whose top digit is brev(m8): hand them back in frequency order
#pragma unroll
    for (int b = 0; b < NB; b++)
#pragma unroll
        for (int h = 0; h < 2; h++) {
            double yr[H], yi[H];
#pragma unroll
            for (int m = 0; m < H; m++) { yr[brev(m, LOGH)] = xr[b][H * h + m]; yi[brev(m, LOGH)] = xi[b][H * h + m]; }
#pragma unroll
            for (int m = 0; m < H; m++) { xr[b][H * h + m] = yr[m]; xi[b][H * h + m] = yi[m]; }
        }
}

// The exact mirror; out: xr/xi[b][m] = u_{t + 64 m} (the factor 1/M applied at the end, a power of two).
template <class PL, int NB>
__device__ __forceinline__ void inverse_halves(const LaneCtx<PL> &lc, double2 *const (&xch)[NB], double (&xr)[NB][PL::P],
                                               double (&xi)[NB][PL::P])
{
    constexpr int H = PL::XP, LOGH = PL::LOGXP;
#pragma unroll
    for (int b = 0; b < NB; b++)
#pragma unroll
        for (int h = 0; h < 2; h++) {
            double yr[H], yi[H];
#pragma unroll
            for (int m = 0; m < H; m++) { yr[m] = xr[b][H * h + brev(m, LOGH)]; yi[m] = xi[b][H * h + brev(m, LOGH)]; }
#pragma unroll
            for (int m = 0; m < H; m++) { xr[b][H * h + m] = yr[m]; xi[b][H * h + m] = yi[m]; }
        }
#pragma unroll
    for (int pass = 2; pass >= 1; pass--) {
        const int Tn = ipow(H, 2 - pass);
#pragma unroll
        for (int h = 0; h < 2; h++) {
            CosTan e[4];
            half_entries<PL>(lc, pass, h, e);
#pragma unroll
            for (int b = 0; b < NB; b++) {
                double(&r)[H] = *reinterpret_cast<double(*)[H]>(&xr[b][H * h]);
                double(&i)[H] = *reinterpret_cast<double(*)[H]>(&xi[b][H * h]);
                node_pass_inverse<H>(r, i, e);
                wave_lds_fence();                            // undo the transposition that preceded this pass
#pragma unroll
                for (int m = 0; m < H; m++) xch[b][lc.rd_base[pass - 1] + m * Tn] = make_double2(r[m], i[m]);
                wave_lds_fence();
#pragma unroll
                for (int m = 0; m < H; m++) {
                    const double2 v = xch[b][brev(m, LOGH) * PL::xrow(pass - 1) + lc.t];
                    r[m] = v.x; i[m] = v.y;
                }
            }
        }
    }
    CosTan e0[8];
    first_pass_entries16(e0);
    constexpr double scale = 1.0 / (double)PL::M;
#pragma unroll
    for (int b = 0; b < NB; b++) {
        node_pass_inverse<16>(xr[b], xi[b], e0);
#pragma unroll
        for (int m = 0; m < PL::P; m++) { xr[b][m] *= scale; xi[b][m] *= scale; }
    }
}

// Forward transform of NB independent polynomials held by the same lanes (NB register sets, NB
// exchange buffers); their passes are written side by side so that one set's arithmetic can fill the
// other's LDS round trips.  In: xr/xi[b][m] = u_{t + L*m} (folded, not yet twisted).  Out: spectra in
// the lane/register order that inverse_n() and the pointwise products share.
template <class PL, int NB>
__device__ __forceinline__ void forward_radix(const LaneCtx<PL> &lc, double2 *const (&xch)[NB], double (&xr)[NB][PL::P],
                                              double (&xi)[NB][PL::P])
{
    constexpr int P = PL::P, K = PL::K;
    // register-dependent part of the twist: psi^(L*m) = exp(i*pi*m/(2P))
#pragma unroll
    for (int b = 0; b < NB; b++)
#pragma unroll
        for (int m = 1; m < P; m++) {
            const double cr = cos_pi64(32 * m / P), ci = sin_pi64(32 * m / P);
            const double r = xr[b][m], i = xi[b][m];
            xr[b][m] = r * cr - i * ci;
            xi[b][m] = r * ci + i * cr;
        }
#pragma unroll
    for (int s = 0; s < K; s++) {
        // the pass's twiddles are requested ahead of its butterflies (the table is read-only, so the reads may
        // sit before the fence): they arrive while the butterflies run instead of one round trip per product
        double2 w[P];
        if (s < K - 1) {
#pragma unroll
            for (int k = (s == 0 ? 0 : 1); k < P; k++) w[k] = lc.twiddle(s, k);
        }
#pragma unroll
        for (int b = 0; b < NB; b++) dft_regs<P, +1>(xr[b], xi[b]);
        if (s == K - 1) break;
        wave_lds_fence();
#pragma unroll
        for (int k = 0; k < P; k++) {
#pragma unroll
            for (int b = 0; b < NB; b++) {
                if (k >= (s == 0 ? 0 : 1)) {
                    const double r = xr[b][k], i = xi[b][k];
                    xr[b][k] = r * w[k].x - i * w[k].y;
                    xi[b][k] = r * w[k].y + i * w[k].x;
                }
                xch[b][k * PL::xrow(s) + lc.t] = make_double2(xr[b][k], xi[b][k]);   // stores overlap the remaining products
            }
        }
        wave_lds_fence();
        const int Tn = ipow(P, K - 2 - s);
#pragma unroll
        for (int b = 0; b < NB; b++)
#pragma unroll
            for (int m = 0; m < P; m++) {
                const double2 v = xch[b][lc.rd_base[s] + m * Tn];
                xr[b][m] = v.x; xi[b][m] = v.y;
            }
    }
}

template <class PL, int NB>
__device__ __forceinline__ void forward_n(const LaneCtx<PL> &lc, double2 *const (&xch)[NB], double (&xr)[NB][PL::P],
                                          double (&xi)[NB][PL::P])
{
    if constexpr (PL::NODES) forward_halves<PL, NB>(lc, xch, xr, xi);
    else forward_radix<PL, NB>(lc, xch, xr, xi);
}

// Forward transforms of NB polynomials through ONE exchange buffer, software-pipelined: within a pass, set b's
// butterflies are followed at once by its exchange (twiddle products, stores, loads), then set b+1's butterflies
// and exchange, and so on.  A wavefront's LDS operations execute in issue order, so a set's stores cannot overtake
// the previous set's loads, and the values a set loaded are first needed one round later, in the next pass, after
// the other sets' arithmetic: no round trip is waited for with nothing to do.  It pays where a wavefront has a
// SIMD to itself (nothing else covers its round trips) and costs NB register sets.
template <class PL, int NB>
__device__ __forceinline__ void forward_pipelined(const LaneCtx<PL> &lc, double (&xr)[NB][PL::P], double (&xi)[NB][PL::P])
{
    constexpr int P = PL::P, K = PL::K;
#pragma unroll
    for (int b = 0; b < NB; b++)
#pragma unroll
        for (int m = 1; m < P; m++) {                               // register-dependent part of the twist
            const double cr = cos_pi64(32 * m / P), ci = sin_pi64(32 * m / P);
            const double r = xr[b][m], i = xi[b][m];
            xr[b][m] = r * cr - i * ci;
            xi[b][m] = r * ci + i * cr;
        }
#pragma unroll
    for (int s = 0; s < K; s++) {
        double2 w[P];
        if (s < K - 1) {
#pragma unroll
            for (int k = (s == 0 ? 0 : 1); k < P; k++) w[k] = lc.twiddle(s, k);
        }
        const int Tn = s < K - 1 ? ipow(P, K - 2 - s) : 1;
#pragma unroll
        for (int b = 0; b < NB; b++) {
            dft_regs<P, +1>(xr[b], xi[b]);
            if (s < K - 1) {
                wave_lds_fence();
#pragma unroll
                for (int k = 0; k < P; k++) {
                    if (k >= (s == 0 ? 0 : 1)) {
                        const double r = xr[b][k], i = xi[b][k];
                        xr[b][k] = r * w[k].x - i * w[k].y;
                        xi[b][k] = r * w[k].y + i * w[k].x;
                    }
                    lc.xch[k * PL::xrow(s) + lc.t] = make_double2(xr[b][k], xi[b][k]);
                }
                wave_lds_fence();
#pragma unroll
                for (int m = 0; m < P; m++) {
                    const double2 v = lc.xch[lc.rd_base[s] + m * Tn];
                    xr[b][m] = v.x; xi[b][m] = v.y;
                }
            }
        }
    }
}

// Inverse transforms, the mirror of forward_n(); the 1/M normalisation is folded into the last
// constant multiplication.  Out: xr/xi[b][m] = u_{t + L*m}.
// SHARED: every set goes through the same exchange buffer, one after the other (store, load, next set's store,
// ...); a wavefront's LDS operations execute in issue order, so a set's stores cannot overtake the previous
// set's loads, and a set's round trip overlaps the arithmetic of the sets before it.
template <class PL, int NB, bool SHARED = false>
__device__ __forceinline__ void inverse_radix(const LaneCtx<PL> &lc, double2 *const (&xch)[NB], double (&xr)[NB][PL::P],
                                              double (&xi)[NB][PL::P])
{
    constexpr int P = PL::P, K = PL::K;
#pragma unroll
    for (int s = K - 1; s >= 0; s--) {
        if (s < K - 1) {
            // undo the transposition that followed pass s+1; the twiddles are requested first
            const int Tn = ipow(P, K - 2 - s);
            double2 w[P];
#pragma unroll
            for (int k = (s == 0 ? 0 : 1); k < P; k++) w[k] = lc.twiddle(s, k);
            if (SHARED) {
#pragma unroll
                for (int b = 0; b < NB; b++) {
                    wave_lds_fence();
#pragma unroll
                    for (int m = 0; m < P; m++) xch[b][lc.rd_base[s] + m * Tn] = make_double2(xr[b][m], xi[b][m]);
                    wave_lds_fence();
#pragma unroll
                    for (int k = 0; k < P; k++) {
                        const double2 v = xch[b][k * PL::xrow(s) + lc.t];
                        xr[b][k] = v.x; xi[b][k] = v.y;
                    }
                }
            } else {
            wave_lds_fence();
#pragma unroll
            for (int b = 0; b < NB; b++)
#pragma unroll
                for (int m = 0; m < P; m++) xch[b][lc.rd_base[s] + m * Tn] = make_double2(xr[b][m], xi[b][m]);
            wave_lds_fence();
#pragma unroll
            for (int b = 0; b < NB; b++)
#pragma unroll
                for (int k = 0; k < P; k++) {
                    const double2 v = xch[b][k * PL::xrow(s) + lc.t];
                    xr[b][k] = v.x; xi[b][k] = v.y;
                }
            }
#pragma unroll
            for (int k = (s == 0 ? 0 : 1); k < P; k++) {            // conjugate twiddle
#pragma unroll
                for (int b = 0; b < NB; b++) {
                    const double r = xr[b][k], i = xi[b][k];
                    xr[b][k] = r * w[k].x + i * w[k].y;
                    xi[b][k] = i * w[k].x - r * w[k].y;
                }
            }
        }
#pragma unroll
        for (int b = 0; b < NB; b++) dft_regs<P, -1>(xr[b], xi[b]);
    }
    constexpr double scale = 1.0 / (double)PL::M;                    // a power of two: products stay exact
#pragma unroll
    for (int b = 0; b < NB; b++) {
        xr[b][0] *= scale;
        xi[b][0] *= scale;
#pragma unroll
        for (int m = 1; m < P; m++) {                                // conjugate of psi^(L*m), times 1/M
            const double cr = cos_pi64(32 * m / P) * scale, ci = sin_pi64(32 * m / P) * scale;
            const double r = xr[b][m], i = xi[b][m];
            xr[b][m] = r * cr + i * ci;
            xi[b][m] = i * cr - r * ci;
        }
    }
}

template <class PL, int NB, bool SHARED = false>
__device__ __forceinline__ void inverse_n(const LaneCtx<PL> &lc, double2 *const (&xch)[NB], double (&xr)[NB][PL::P],
                                          double (&xi)[NB][PL::P])
{
    if constexpr (PL::NODES) inverse_halves<PL, NB>(lc, xch, xr, xi);
    else inverse_radix<PL, NB, SHARED>(lc, xch, xr, xi);
}

// One polynomial at a time.
template <class PL> __device__ __forceinline__ void forward(const LaneCtx<PL> &lc, double (&xr)[PL::P], double (&xi)[PL::P])
{
    double2 *const xch[1] = {lc.xch};
    forward_n<PL, 1>(lc, xch, reinterpret_cast<double (&)[1][PL::P]>(xr), reinterpret_cast<double (&)[1][PL::P]>(xi));
}
template <class PL> __device__ __forceinline__ void inverse(const LaneCtx<PL> &lc, double (&xr)[PL::P], double (&xi)[PL::P])
{
    double2 *const xch[1] = {lc.xch};
    inverse_n<PL, 1>(lc, xch, reinterpret_cast<double (&)[1][PL::P]>(xr), reinterpret_cast<double (&)[1][PL::P]>(xi));
}

}  // namespace she
