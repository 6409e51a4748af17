// HIP kernels of the bootstrapped-gate path for gfx950 (MI355X).
//
// One circuit level of G independent gates runs as three launches:
//   k_lincomb       gate-specific TLWE linear combination + modulus switch to Z_2N
//   k_blind_rotate  n CMux steps per gate (decompose, forward transforms, pointwise
//                   products with the streamed spectral bootstrapping key, inverse
//                   transforms), then sample extraction and key-switch digit rounding
//   k_key_switch    subtraction of the selected key-switching rows
// (SHE, arXiv 1906.00148: Section 3.1 for the gates, Section 2 for bootstrapping; the
// construction itself is the cited TFHE gate bootstrapping.)
#include "negacyclic_fft.h"
#include "she_internal.h"
#include <mutex>
#pragma clang fp contract(fast)

namespace she {

__device__ __forceinline__ uint32_t *ct_ptr(const CtSpace &cs, uint32_t id)
{
    return id < cs.cap ? cs.pool + (size_t)id * cs.stride : cs.temp + (size_t)(id - cs.cap) * cs.stride;
}

// ------------------------------------------------------------------------------------------
// Linear combination and modulus switch.  One block per gate.
// Pre-bootstrap sample = (0, off) + sa*ca + sb*cb, doubled for XOR/XNOR; every word is then
// rounded to the nearest multiple of 1/2N.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(128) void k_lincomb(CtSpace cs, const uint8_t *__restrict__ type,
                                                 const uint32_t *__restrict__ in0, const uint32_t *__restrict__ in1,
                                                 const uint32_t *__restrict__ in2, uint32_t n, uint32_t log2_2N,
                                                 uint16_t *__restrict__ bar, uint32_t bar_stride)
{
    const uint32_t g = blockIdx.x;
    const uint32_t ty = type[g];
    const uint32_t e = 1u << 29;
    const uint32_t rnd = 1u << (31 - log2_2N), sh = 32 - log2_2N;
    uint16_t *dst = bar + (size_t)g * bar_stride;
    if (ty >= SHE_MAJ3) {
        // three-input gate: s = +-ca +- cb +- cc has phase (2k-3)/8 for k true inputs; majority is the sign of s,
        // parity the sign of -2s (phase +1/4 for odd k, -1/4 for even k); no offset (in2 is non-null for these)
        const uint32_t m = ty - SHE_MAJ3;
        const bool parity = (m >> 3) != 0;
        const uint32_t *ca = ct_ptr(cs, in0[g]), *cb = ct_ptr(cs, in1[g]), *cc = ct_ptr(cs, in2[g]);
        for (uint32_t i = threadIdx.x; i <= n; i += blockDim.x) {
            const uint32_t a = ca[i], b = cb[i], c = cc[i];
            uint32_t x = ((m & 1) ? 0u - a : a) + ((m & 2) ? 0u - b : b) + ((m & 4) ? 0u - c : c);
            if (parity) x = 0u - 2u * x;
            dst[i] = (uint16_t)((x + rnd) >> sh);
        }
        return;
    }
    // sign of ca, sign of cb, offset, doubling
    uint32_t off = e; bool na = false, nb = false, dbl = false;
    switch (ty) {
    case SHE_AND:   off = 0u - e; break;
    case SHE_NAND:  off = e; na = nb = true; break;
    case SHE_OR:    off = e; break;
    case SHE_NOR:   off = 0u - e; na = nb = true; break;
    case SHE_XOR:   off = 2 * e; dbl = true; break;
    case SHE_XNOR:  off = 0u - 2 * e; na = nb = true; dbl = true; break;
    case SHE_ANDNY: off = 0u - e; na = true; break;
    case SHE_ANDYN: off = 0u - e; nb = true; break;
    case SHE_ORNY:  off = e; na = true; break;
    default:        off = e; nb = true; break;     // SHE_ORYN
    }
    const uint32_t *ca = ct_ptr(cs, in0[g]);
    const uint32_t *cb = ct_ptr(cs, in1[g]);
    for (uint32_t i = threadIdx.x; i <= n; i += blockDim.x) {
        uint32_t a = ca[i], b = cb[i];
        uint32_t x = (na ? 0u - a : a) + (nb ? 0u - b : b);
        if (dbl) x += x;
        if (i == n) x += off;
        dst[i] = (uint16_t)((x + rnd) >> sh);
    }
}

// ------------------------------------------------------------------------------------------
// Blind rotation.  One gate per L lanes; a wavefront never talks to another one.
// ------------------------------------------------------------------------------------------
constexpr int BR_WAVES = 4;     // measured: 2 and 8 wavefronts per workgroup are slower

// LC: the gadget length when it is known at compile time (the loops over the 2 LC rows of a step are then unrolled:
// shifts and row offsets become constants, measured 1.2 % faster at l = 3 on alternating runs), 0 for any length.
template <class PL, bool TRACK, int LC>
__global__ __launch_bounds__(64 * BR_WAVES, 2) void k_blind_rotate(
    const uint16_t *__restrict__ bar, uint32_t bar_stride, uint32_t n, uint32_t l_arg, uint32_t bg_bit,
    const double2 *__restrict__ bk_hat, const double2 *__restrict__ tw_table, uint32_t ks_bits,
    uint32_t *__restrict__ ext_b, uint16_t *__restrict__ ksd, uint32_t gates, unsigned *round_err, CtSpace cs,
    const uint32_t *__restrict__ out_ids, uint32_t *__restrict__ raw_ext)
{
    constexpr int P = PL::P, L = PL::L, M = PL::M, N = PL::N, GPW = PL::GPW;
    const uint32_t l = LC ? (uint32_t)LC : l_arg;
    __shared__ uint32_t s_acc[BR_WAVES * GPW][2][N];
    __shared__ double2 s_xch[BR_WAVES * GPW][PL::XSLOTS];
    __shared__ double2 s_tw[TwTable<PL>::COUNT];

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int sub = lane / L, t = lane % L;
    const int slot = wave * GPW + sub;
    const uint32_t g_raw = (blockIdx.x * BR_WAVES + wave) * GPW + sub;
    load_twiddles<PL>(s_tw, tw_table);                                    // the only workgroup barrier
    if ((blockIdx.x * BR_WAVES + wave) * GPW >= gates) return;          // whole wavefront idle
    const bool live = g_raw < gates;
    const uint32_t g = live ? g_raw : gates - 1;                          // idle lanes shadow the last gate

    LaneCtx<PL> lc;
    lc.init(t, s_xch[slot], s_tw);
    uint32_t(*acc)[N] = s_acc[slot];
    const uint16_t *mybar = bar + (size_t)g * bar_stride;

    // ACC = (0, X^(-bbar) * testv), testv = 1/8 on every coefficient
    {
        const uint32_t bbar = mybar[n];
        for (int j = t; j < N; j += L) {
            acc[0][j] = 0;
            acc[1][j] = (((uint32_t)j + bbar) & N) ? 0u - (1u << 29) : (1u << 29);
        }
    }
    wave_lds_fence();

    const uint32_t Bg = 1u << bg_bit, half_bg = Bg >> 1;
    uint32_t dec_off = 1u << (31 - l * bg_bit);
    uint32_t flip = 0;      // top bit of every digit field: field ^ top, read as signed, is field - Bg/2
    for (uint32_t p = 1; p <= l; p++) { dec_off += half_bg << (32 - p * bg_bit); flip |= half_bg << (32 - p * bg_bit); }
    float worst = 0.f;

    uint32_t abar_next = mybar[0];
    // spectra of the key row in use; row 0 of the next step is requested before the inverse transforms
    double2 bv[2][P];
    {
        const double2 *row = bk_hat + t;
#pragma unroll
        for (int o = 0; o < 2; o++)
#pragma unroll
            for (int k = 0; k < P; k++) bv[o][k] = row[(o * P + k) * L];
    }
    for (uint32_t i = 0; i < n; i++) {
        const uint32_t abar = abar_next;
        abar_next = mybar[i + 1];                                          // i+1 == n reads bbar: harmless

        double sr[2][P], si[2][P];                                         // spectra of the two output components
#pragma unroll
        for (int k = 0; k < P; k++) { sr[0][k] = si[0][k] = sr[1][k] = si[1][k] = 0.0; }

#pragma unroll(LC ? 2 : 1)
        for (int c = 0; c < 2; c++) {
            // D_c = X^abar * ACC_c - ACC_c at this lane's 2P coefficients
            uint32_t dlo[P], dhi[P];
#pragma unroll
            for (int m = 0; m < P; m++) {
                const uint32_t j0 = t + L * m, j1 = j0 + M;
                const uint32_t s0 = (j0 - abar) & (2 * N - 1), s1 = (j1 - abar) & (2 * N - 1);
                uint32_t v0 = acc[c][s0 & (N - 1)], v1 = acc[c][s1 & (N - 1)];
                v0 = (s0 & N) ? 0u - v0 : v0;
                v1 = (s1 & N) ? 0u - v1 : v1;
                // + dec_off: rounding and digit centring; ^ flip: turns each field into its signed digit
                dlo[m] = (v0 - acc[c][j0] + dec_off) ^ flip;
                dhi[m] = (v1 - acc[c][j1] + dec_off) ^ flip;
            }
#pragma unroll(LC ? LC : 1)
            for (uint32_t p = 0; p < l; p++) {
                const uint32_t sh = 32 - (p + 1) * bg_bit;
                const uint32_t r = c * l + p;
                double xr[P], xi[P];
#pragma unroll
                for (int m = 0; m < P; m++) {
                    // the builtin returns unsigned: go through int so that the conversion is signed
                    xr[m] = (double)(int)__builtin_amdgcn_sbfe(dlo[m], sh, bg_bit);
                    xi[m] = (double)(int)__builtin_amdgcn_sbfe(dhi[m], sh, bg_bit);
                }
                // a wavefront inside a transform issues ahead of one in the products or the decomposition: its LDS
                // round trips start sooner and the other wavefront's arithmetic fills them (measured: 1-2 %)
                __builtin_amdgcn_s_setprio(3);
                forward<PL>(lc, xr, xi);
                __builtin_amdgcn_s_setprio(0);
                __builtin_amdgcn_sched_barrier(0);     // keeps the products out of the transform's schedule (measured: +4%)
                // request the next row (of this step, or row 0 of the next one) register by register as the products
                // free them; after the last step this reads the last row once more, which is harmless
                const size_t nxt = std::min<size_t>((size_t)i * 2 * l + r + 1, (size_t)n * 2 * l - 1);
                const double2 *row = bk_hat + nxt * 2 * P * L + t;
#pragma unroll
                for (int o = 0; o < 2; o++) {
#pragma unroll
                    for (int k = 0; k < P; k++) {
                        const double2 b = bv[o][k];
                        // two fused multiply-adds per part (a += x*y - z*w would cost a multiply, an fma and an add)
                        sr[o][k] = __builtin_fma(-xi[k], b.y, __builtin_fma(xr[k], b.x, sr[o][k]));
                        si[o][k] = __builtin_fma(xi[k], b.x, __builtin_fma(xr[k], b.y, si[o][k]));
                        bv[o][k] = row[(o * P + k) * L];
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        {
            // both inverse transforms side by side through the one exchange buffer (measured: 21.0 -> 20.7 ms)
            double2 *const xch2[2] = {lc.xch, lc.xch};
            inverse_n<PL, 2, true>(lc, xch2, sr, si);
        }
#pragma unroll
        for (int o = 0; o < 2; o++) {
#pragma unroll
            for (int m = 0; m < P; m++) {
                const double vr = sr[o][m], vi = si[o][m];
                if (TRACK) {
                    worst = fmaxf(worst, (float)fabs(vr - rint(vr)));
                    worst = fmaxf(worst, (float)fabs(vi - rint(vi)));
                }
                // |v| < 2^51: adding 1.5*2^52 leaves round(v) mod 2^32 in the low word
                const uint32_t ir = (uint32_t)__double2loint(vr + 6755399441055744.0);
                const uint32_t ii = (uint32_t)__double2loint(vi + 6755399441055744.0);
                acc[o][t + L * m] += ir;
                acc[o][t + L * m + M] += ii;
            }
        }
        wave_lds_fence();
    }

    if (TRACK && round_err) atomicMax(round_err, __float_as_uint(worst));

    // sample extraction: a''_0 = A_0, a''_j = -A_{N-j}, b'' = B_0
    if (live && raw_ext) {
        // a rotation of a MUX: the sample itself is kept, two of them are summed before the key switch
        uint32_t *dst = raw_ext + (size_t)g * (N + 1);
        for (int j = t; j < N; j += L) dst[j] = (j == 0) ? acc[0][0] : 0u - acc[0][N - j];
        if (t == 0) dst[N] = acc[1][0];
    } else if (live) {
        // keep the top ks_bits of each a'' rounded
        const uint32_t rnd = 1u << (31 - ks_bits), sh = 32 - ks_bits;
        uint16_t *dst = ksd + ((size_t)(g / KS_GROUP) * N) * KS_GROUP + (g % KS_GROUP);
        for (int j = t; j < N; j += L) {
            const uint32_t a = (j == 0) ? acc[0][0] : 0u - acc[0][N - j];
            dst[(size_t)j * KS_GROUP] = (uint16_t)((a + rnd) >> sh);
        }
        if (t == 0) ext_b[g] = acc[1][0];
        // the key switch subtracts its rows from (0, b''): leave that in the output slot
        if (out_ids) {
            uint32_t *o = ct_ptr(cs, out_ids[g]);
            const uint32_t body = acc[1][0];
            for (uint32_t c = t; c <= n; c += L) o[c] = (c == n) ? body : 0u;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Blind rotation of a small level: one gate per workgroup of two wavefronts.
// A level of a few hundred gates leaves most SIMDs with one wavefront or none, and the time of
// the kernel above is then the latency of one wavefront's serial chain of 6 forward and 2
// inverse transforms per CMux.  Here wavefront c of a gate owns accumulator component c: it
// decomposes ACC_c, transforms its l digit polynomials, multiplies them with rows c*l..c*l+l-1
// of the key for both output components, hands the partial spectrum of the other component to
// its partner through LDS, and inverse-transforms its own component.  The chain per CMux is
// l forward transforms, one exchange and one inverse transform.  Results are bit-identical to
// k_blind_rotate's only up to FP64 summation order; both are exact after rounding.
// ------------------------------------------------------------------------------------------
// Workgroup barrier for LDS traffic only: earlier LDS operations of this wavefront are complete
// (they finish in issue order, the counter reaches zero when the last one has), global loads
// stay in flight.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

constexpr int largest_divisor_up_to(int v, int cap) { int d = cap < v ? cap : v; while (d > 1 && v % d) d--; return d < 1 ? 1 : d; }
constexpr int SPLIT_KD = 16;       // key values in flight per wavefront of the split kernel (measured: 8 is slower)
// LR > 0: the gadget has LR levels (l == LR) and a wavefront transforms its LR digit polynomials side by side
// (forward_pipelined), streaming the key rows through SPLIT_KD values in flight; LR == 0: any l, one at a time.
template <class PL, bool TRACK, int GB, int LR>
__global__ __launch_bounds__(128 * GB, 2) void k_blind_rotate_split(
    const uint16_t *__restrict__ bar, uint32_t bar_stride, uint32_t n, uint32_t l, uint32_t bg_bit,
    const double2 *__restrict__ bk_hat, const double2 *__restrict__ tw_table, uint32_t ks_bits,
    uint32_t *__restrict__ ext_b, uint16_t *__restrict__ ksd, uint32_t gates, unsigned *round_err, CtSpace cs,
    const uint32_t *__restrict__ out_ids, uint32_t *__restrict__ raw_ext)
{
    constexpr int P = PL::P, L = PL::L, M = PL::M, N = PL::N;
    static_assert(PL::GPW == 1, "one transform per wavefront");
    __shared__ uint32_t s_acc[2 * GB][N];
    __shared__ double2 s_xch[2 * GB][PL::XSLOTS];
    __shared__ double2 s_tw[TwTable<PL>::COUNT];

    const int wave = threadIdx.x >> 6, t = threadIdx.x & 63;
    const int c = wave & 1;                                               // component owned
    // a wavefront pair past the end shadows the last gate and stores nothing: it still meets every barrier
    const uint32_t g_raw = blockIdx.x * GB + (wave >> 1);
    const bool live = g_raw < gates;
    const uint32_t g = live ? g_raw : gates - 1;
    load_twiddles<PL>(s_tw, tw_table);

    LaneCtx<PL> lc;
    lc.init(t, s_xch[wave], s_tw);
    uint32_t *acc = s_acc[wave];
    const double2 *theirs = s_xch[wave ^ 1];
    const uint16_t *mybar = bar + (size_t)g * bar_stride;

    // ACC = (0, X^(-bbar) * testv), testv = 1/8 on every coefficient
    {
        const uint32_t bbar = mybar[n];
        for (int j = t; j < N; j += L) acc[j] = c == 0 ? 0u : ((((uint32_t)j + bbar) & N) ? 0u - (1u << 29) : (1u << 29));
    }
    wave_lds_fence();

    const uint32_t Bg = 1u << bg_bit, half_bg = Bg >> 1;
    uint32_t dec_off = 1u << (31 - l * bg_bit);
    uint32_t flip = 0;
    for (uint32_t p = 1; p <= l; p++) { dec_off += half_bg << (32 - p * bg_bit); flip |= half_bg << (32 - p * bg_bit); }
    float worst = 0.f;

    // spectra of the key row in use, own output component first
    const size_t row_elems = (size_t)2 * P * L;
    const int mine_off = c * P * L + t, other_off = (c ^ 1) * P * L + t;
    double2 bm[P], bo[P];
    if constexpr (LR == 0) {
        const double2 *row = bk_hat + (size_t)(c * l) * row_elems;
#pragma unroll
        for (int k = 0; k < P; k++) { bm[k] = row[mine_off + k * L]; bo[k] = row[other_off + k * L]; }
    }
    // LR > 0: key value j = (p*2 + o)*P + k of this component's LR rows sits at rows[j*L]
    // (KD divides NV, so that a value keeps its place in the ring from one step to the next)
    constexpr int NV = LR * 2 * P, KD = LR > 0 ? largest_divisor_up_to(NV, SPLIT_KD) : 1;
    double2 kv[KD];
    if constexpr (LR > 0) {
        const double2 *rows = bk_hat + (size_t)(c * LR) * row_elems + t;
#pragma unroll
        for (int j = 0; j < KD; j++) kv[j] = rows[j * L];
    }
    uint32_t abar_next = mybar[0];
    for (uint32_t i = 0; i < n; i++) {
        const uint32_t abar = abar_next;
        abar_next = mybar[i + 1];                                          // i+1 == n reads bbar: harmless

        double mr[P], mi[P], orr[P], oi[P];                                // partial spectra: own component, the other one
        if constexpr (LR == 0) {
#pragma unroll
            for (int k = 0; k < P; k++) { mr[k] = mi[k] = orr[k] = oi[k] = 0.0; }
        }

        // D_c = X^abar * ACC_c - ACC_c at this lane's 2P coefficients
        uint32_t dlo[P], dhi[P];
#pragma unroll
        for (int m = 0; m < P; m++) {
            const uint32_t j0 = t + L * m, j1 = j0 + M;
            const uint32_t s0 = (j0 - abar) & (2 * N - 1), s1 = (j1 - abar) & (2 * N - 1);
            uint32_t v0 = acc[s0 & (N - 1)], v1 = acc[s1 & (N - 1)];
            v0 = (s0 & N) ? 0u - v0 : v0;
            v1 = (s1 & N) ? 0u - v1 : v1;
            dlo[m] = (v0 - acc[j0] + dec_off) ^ flip;
            dhi[m] = (v1 - acc[j1] + dec_off) ^ flip;
        }
        if constexpr (LR > 0) {
            double xr[LR][P], xi[LR][P];
#pragma unroll
            for (int p = 0; p < LR; p++)
#pragma unroll
                for (int m = 0; m < P; m++) {
                    xr[p][m] = (double)(int)__builtin_amdgcn_sbfe(dlo[m], 32 - (p + 1) * bg_bit, bg_bit);
                    xi[p][m] = (double)(int)__builtin_amdgcn_sbfe(dhi[m], 32 - (p + 1) * bg_bit, bg_bit);
                }
            forward_pipelined<PL, LR>(lc, xr, xi);
            __builtin_amdgcn_sched_barrier(0);
            // this step's remaining key values, then the first KD of the next step (the last step's again at the end)
            const double2 *rows = bk_hat + ((size_t)i * 2 * LR + c * LR) * row_elems + t;
            const double2 *rows_next = bk_hat + ((size_t)std::min(i + 1, n - 1) * 2 * LR + c * LR) * row_elems + t;
#pragma unroll
            for (int j = 0; j < NV; j++) {
                const int p = j / (2 * P), o = (j / P) % 2, k = j % P;
                const double2 b = kv[j % KD];
                // output component o of the key row; o == c is this wavefront's own
                double &ar = (o == c) ? mr[k] : orr[k];
                double &ai = (o == c) ? mi[k] : oi[k];
                if (p == 0) {
                    ar = __builtin_fma(-xi[p][k], b.y, xr[p][k] * b.x);
                    ai = __builtin_fma(xi[p][k], b.x, xr[p][k] * b.y);
                } else {
                    ar = __builtin_fma(-xi[p][k], b.y, __builtin_fma(xr[p][k], b.x, ar));
                    ai = __builtin_fma(xi[p][k], b.x, __builtin_fma(xr[p][k], b.y, ai));
                }
                kv[j % KD] = (j + KD < NV) ? rows[(j + KD) * L] : rows_next[(j + KD - NV) * L];
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        for (uint32_t p = 0; LR == 0 && p < l; p++) {
            const uint32_t sh = 32 - (p + 1) * bg_bit;
            double xr[P], xi[P];
#pragma unroll
            for (int m = 0; m < P; m++) {
                xr[m] = (double)(int)__builtin_amdgcn_sbfe(dlo[m], sh, bg_bit);
                xi[m] = (double)(int)__builtin_amdgcn_sbfe(dhi[m], sh, bg_bit);
            }
            forward<PL>(lc, xr, xi);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < P; k++) {
                mr[k] = __builtin_fma(-xi[k], bm[k].y, __builtin_fma(xr[k], bm[k].x, mr[k]));
                mi[k] = __builtin_fma(xi[k], bm[k].x, __builtin_fma(xr[k], bm[k].y, mi[k]));
                orr[k] = __builtin_fma(-xi[k], bo[k].y, __builtin_fma(xr[k], bo[k].x, orr[k]));
                oi[k] = __builtin_fma(xi[k], bo[k].x, __builtin_fma(xr[k], bo[k].y, oi[k]));
            }
            // next row of this component: same step, or the first of the next step (the last row again at the end)
            {
                const uint32_t ni = (p + 1 < l) ? i : std::min(i + 1, n - 1), np = (p + 1 < l) ? p + 1 : 0;
                const double2 *row = bk_hat + ((size_t)ni * 2 * l + c * l + np) * row_elems;
#pragma unroll
                for (int k = 0; k < P; k++) { bm[k] = row[mine_off + k * L]; bo[k] = row[other_off + k * L]; }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // hand the other component's partial spectrum to the partner, take the partner's for this one
        wave_lds_fence();
#pragma unroll
        for (int k = 0; k < P; k++) lc.xch[k * PL::XROW + t] = make_double2(orr[k], oi[k]);
        lds_barrier();
#pragma unroll
        for (int k = 0; k < P; k++) {
            const double2 v = theirs[k * PL::XROW + t];
            mr[k] += v.x; mi[k] += v.y;
        }
        lds_barrier();                                                      // the partner has read this buffer: free for the inverse
        inverse<PL>(lc, mr, mi);
#pragma unroll
        for (int m = 0; m < P; m++) {
            const double vr = mr[m], vi = mi[m];
            if (TRACK) {
                worst = fmaxf(worst, (float)fabs(vr - rint(vr)));
                worst = fmaxf(worst, (float)fabs(vi - rint(vi)));
            }
            acc[t + L * m] += (uint32_t)__double2loint(vr + 6755399441055744.0);
            acc[t + L * m + M] += (uint32_t)__double2loint(vi + 6755399441055744.0);
        }
        wave_lds_fence();
    }

    if (TRACK && round_err) atomicMax(round_err, __float_as_uint(worst));

    // sample extraction: wavefront 0 holds A (mask a''_0 = A_0, a''_j = -A_{N-j}), wavefront 1 holds B (body b'' = B_0)
    if (!live) return;
    if (raw_ext) {
        uint32_t *dst = raw_ext + (size_t)g * (N + 1);
        if (c == 0) {
            for (int j = t; j < N; j += L) dst[j] = (j == 0) ? acc[0] : 0u - acc[N - j];
        } else if (t == 0) {
            dst[N] = acc[0];
        }
    } else if (c == 0) {
        const uint32_t rnd = 1u << (31 - ks_bits), sh = 32 - ks_bits;
        uint16_t *dst = ksd + ((size_t)(g / KS_GROUP) * N) * KS_GROUP + (g % KS_GROUP);
        for (int j = t; j < N; j += L) {
            const uint32_t a = (j == 0) ? acc[0] : 0u - acc[N - j];
            dst[(size_t)j * KS_GROUP] = (uint16_t)((a + rnd) >> sh);
        }
    } else {
        const uint32_t body = acc[0];
        if (t == 0) ext_b[g] = body;
        if (out_ids) {                       // the key switch subtracts its rows from (0, b'')
            uint32_t *o = ct_ptr(cs, out_ids[g]);
            for (uint32_t w = t; w <= n; w += L) o[w] = (w == n) ? body : 0u;
        }
    }
}

// Second half of a native MUX: the two rotations' samples are added, 1/8 goes on the body, and the
// sum is prepared for the key switch exactly as the blind rotation's epilogue prepares a gate.
__global__ __launch_bounds__(256) void k_mux_combine(const uint32_t *__restrict__ raw_ext, uint32_t N, uint32_t n,
                                                     uint32_t ks_bits, uint32_t *__restrict__ ext_b,
                                                     uint16_t *__restrict__ ksd, CtSpace cs,
                                                     const uint32_t *__restrict__ out_ids)
{
    const uint32_t g = blockIdx.x;
    const uint32_t *e1 = raw_ext + (size_t)(2 * g) * (N + 1), *e0 = e1 + (N + 1);
    const uint32_t rnd = 1u << (31 - ks_bits), sh = 32 - ks_bits;
    uint16_t *dst = ksd + ((size_t)(g / KS_GROUP) * N) * KS_GROUP + (g % KS_GROUP);
    for (uint32_t j = threadIdx.x; j < N; j += blockDim.x)
        dst[(size_t)j * KS_GROUP] = (uint16_t)((e1[j] + e0[j] + rnd) >> sh);
    const uint32_t body = e1[N] + e0[N] + (1u << 29);
    if (threadIdx.x == 0) ext_b[g] = body;
    if (out_ids) {
        uint32_t *o = ct_ptr(cs, out_ids[g]);
        for (uint32_t c = threadIdx.x; c <= n; c += blockDim.x) o[c] = (c == n) ? body : 0u;
    }
}

// Spectra of the bootstrapping key: one transform per (i, row, component) polynomial.
template <class PL>
__global__ __launch_bounds__(64 * BR_WAVES) void k_bk_transform(const uint32_t *__restrict__ bk_int,
                                                                const double2 *__restrict__ tw_table,
                                                                double2 *__restrict__ bk_hat, uint32_t polys,
                                                                const uint32_t *__restrict__ dst_ids,
                                                                uint32_t polys_per_sample)
{
    constexpr int P = PL::P, L = PL::L, M = PL::M, N = PL::N, GPW = PL::GPW;
    __shared__ double2 s_xch[BR_WAVES * GPW][PL::XSLOTS];
    __shared__ double2 s_tw[TwTable<PL>::COUNT];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int sub = lane / L, t = lane % L;
    const uint32_t first = (blockIdx.x * BR_WAVES + wave) * GPW;
    load_twiddles<PL>(s_tw, tw_table);
    if (first >= polys) return;
    const bool live = first + sub < polys;
    const uint32_t q = live ? first + sub : polys - 1;
    LaneCtx<PL> lc;
    lc.init(t, s_xch[wave * GPW + sub], s_tw);
    const uint32_t *src = bk_int + (size_t)q * N;
    double xr[P], xi[P];
#pragma unroll
    for (int m = 0; m < P; m++) {
        xr[m] = (double)(int)src[t + L * m];                 // torus words taken as signed: centred, |x| <= 2^31
        xi[m] = (double)(int)src[t + L * m + M];
    }
    forward<PL>(lc, xr, xi);
    if (live) {
        // sample s of the source goes to sample dst_ids[s] of the destination (in place when there is no list)
        const size_t qo = dst_ids ? (size_t)dst_ids[q / polys_per_sample] * polys_per_sample + q % polys_per_sample : q;
        double2 *dst = bk_hat + qo * P * L + t;
#pragma unroll
        for (int k = 0; k < P; k++) dst[k * L] = make_double2(xr[k], xi[k]);
    }
}

// ------------------------------------------------------------------------------------------
// Leveled CMux: out = d0 + C [.] (d1 - d0) for a TRGSW selector C in spectral form and TRLWE
// samples in HBM.  One CMux per wavefront; the same decomposition, transforms and products as
// one step of the blind rotation, with the operands streamed from memory instead of LDS.
// ------------------------------------------------------------------------------------------
// With 16 points per lane (N = 2048) the two output spectra and one transform fill the register file (192 of 256), so
// no selector row and no operand is requested ahead there.  What keeps that version at two wavefronts per SIMD and off
// the scratch memory: the words that the digits are cut from wait in LDS between the rows (32 registers), and the
// selector's values run through a ring of four points' worth of loads inside the products.  Per 4096 CMuxes: one
// wavefront per SIMD 282 us; two, every selector value loaded and waited for singly 162 us; the ring 149 us (45
// registers spilled); the words in LDS as well 101 us (12 spilled).
// (Both halves of a transform through one LDS round trip, in a buffer of twice the size, spills 31 registers: 214 us.)

// Sixteen bytes per lane from global memory straight into LDS (lane t's word lands at dst_wave + t): no register is
// held while the load is in flight.  dst_wave is the same for the whole wavefront.
__device__ __forceinline__ void load_to_lds16(const uint4 *src_lane, uint4 *dst_wave)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src_lane,
                                     (__attribute__((address_space(3))) void *)dst_wave, 16, 0, 0);
}

// LC: the gadget length when it is known at compile time (both loops over the rows are then unrolled, and a wait for
// memory sits at the first use of what was loaded instead of at a loop's entry), 0 for a length read at run time.
template <class PL, bool TRACK, int LC>
__global__ __launch_bounds__(64 * BR_WAVES, 2) void k_cmux(const double2 *__restrict__ trgsw_hat,
                                                           uint32_t *trlwe, const uint32_t *__restrict__ sel,
                                                           const uint32_t *__restrict__ in1, const uint32_t *__restrict__ in0,
                                                           const uint32_t *__restrict__ out, uint32_t count, uint32_t l_arg,
                                                           uint32_t bg_bit, const double2 *__restrict__ tw_table,
                                                           unsigned *round_err)
{
    constexpr int P = PL::P, L = PL::L, N = PL::N;
    const uint32_t l = LC ? (uint32_t)LC : l_arg;
    static_assert(PL::GPW == 1, "one transform per wavefront");
    __shared__ double2 s_xch[BR_WAVES][PL::XSLOTS];
    __shared__ double2 s_tw[TwTable<PL>::COUNT];
    constexpr bool STAGE = P <= 8;                                        // component 1's operands wait in LDS
    __shared__ uint4 s_stage[STAGE ? BR_WAVES : 1][STAGE ? P * L : 1];    // [d1 | d0] x P/2 words x 64 lanes
    // With 16 points per lane the words that the digits are cut from wait in LDS between the rows (each lane reads
    // back what it wrote): 32 registers that the transform and the products need.
    constexpr bool WORDS_IN_LDS = P > 8;
    __shared__ uint4 s_words[WORDS_IN_LDS ? BR_WAVES : 1][WORDS_IN_LDS ? (P / 2) * L : 1];
    const int wave = threadIdx.x >> 6, t = threadIdx.x & 63;
    load_twiddles<PL>(s_tw, tw_table);                                    // once per workgroup: the grid is persistent

    LaneCtx<PL> lc;
    lc.init(t, s_xch[wave], s_tw);
    const uint32_t Bg = 1u << bg_bit, half_bg = Bg >> 1;
    uint32_t dec_off = 1u << (31 - l * bg_bit);
    uint32_t flip = 0;
    for (uint32_t p = 1; p <= l; p++) { dec_off += half_bg << (32 - p * bg_bit); flip |= half_bg << (32 - p * bg_bit); }
    float worst = 0.f;

    // a wavefront takes CMux g, g + (wavefronts in the grid), ...; g is uniform, so the four ids are scalar loads.
    // Operands are requested ahead, before the inverse transforms: the words of d0 that the result is added to and
    // component 0 of the NEXT CMux into registers (the selector row's are idle then), component 1 of the next CMux
    // into LDS, which costs no register.  (Component 1 requested into registers during component 0's last transform
    // spills 86 of them: 73 us per 4096 CMuxes against 55 with nothing ahead, 53 without component 1, 47 with LDS.)
    const uint32_t stride = gridDim.x * BR_WAVES;
    constexpr int Q = P / 2;
    constexpr bool AHEAD = P <= 8;                                         // 16 points per lane leave no idle registers
    uint4 pu[Q], pv[Q];                                                    // requested TRLWE words of d1 and d0
    uint32_t g = __builtin_amdgcn_readfirstlane(blockIdx.x * BR_WAVES + wave);
    if (AHEAD && g < count) {
        const uint4 *a1 = reinterpret_cast<const uint4 *>(trlwe + (size_t)in1[g] * 2 * N) + t;
        const uint4 *a0 = reinterpret_cast<const uint4 *>(trlwe + (size_t)in0[g] * 2 * N) + t;
        if constexpr (STAGE) {
#pragma unroll
            for (int q = 0; q < Q; q++) {
                load_to_lds16(a1 + N / 4 + q * L, &s_stage[wave][q * L]);
                load_to_lds16(a0 + N / 4 + q * L, &s_stage[wave][(Q + q) * L]);
            }
        }
#pragma unroll
        for (int q = 0; q < Q; q++) { pu[q] = a1[q * L]; pv[q] = a0[q * L]; }
    }
    for (; g < count; g += stride) {
    const uint32_t *d1 = trlwe + (size_t)in1[g] * 2 * N, *d0 = trlwe + (size_t)in0[g] * 2 * N;
    uint32_t *dst = trlwe + (size_t)out[g] * 2 * N;
    const double2 *rows = trgsw_hat + (size_t)sel[g] * 2 * l * 2 * P * L + t;

    constexpr bool ROW_AHEAD = P <= 8;
    double2 bv[2][ROW_AHEAD ? P : 1];
    if constexpr (ROW_AHEAD) {
#pragma unroll
        for (int o = 0; o < 2; o++)
#pragma unroll
            for (int k = 0; k < P; k++) bv[o][k] = rows[(o * P + k) * L];
    }

    double sr[2][P], si[2][P];
#pragma unroll
    for (int k = 0; k < P; k++) { sr[0][k] = si[0][k] = sr[1][k] = si[1][k] = 0.0; }

#pragma unroll(LC ? 2 : 1)
    for (int c = 0; c < 2; c++) {
        // TRLWE samples are stored in transform order: the 16-byte word (q, t) of a component holds the coefficients
        // t + L*2q, t + L*2q + M, t + L*(2q+1), t + L*(2q+1) + M, the ones lane t works on
        uint32_t dlo[WORDS_IN_LDS ? 1 : P], dhi[WORDS_IN_LDS ? 1 : P];
        if (STAGE && c == 1) {
#pragma unroll
            for (int q = 0; q < Q; q++) { pu[q] = s_stage[wave][q * L + t]; pv[q] = s_stage[wave][(Q + q) * L + t]; }
        } else if (c == 1 || !AHEAD) {
            const uint4 *a1 = reinterpret_cast<const uint4 *>(d1 + c * N) + t, *a0 = reinterpret_cast<const uint4 *>(d0 + c * N) + t;
#pragma unroll
            for (int q = 0; q < Q; q++) { pu[q] = a1[q * L]; pv[q] = a0[q * L]; }
        }
#pragma unroll
        for (int q = 0; q < Q; q++) {
            const uint4 u = pu[q], v = pv[q];
            const uint4 w = make_uint4((u.x - v.x + dec_off) ^ flip, (u.y - v.y + dec_off) ^ flip,
                                       (u.z - v.z + dec_off) ^ flip, (u.w - v.w + dec_off) ^ flip);
            if constexpr (WORDS_IN_LDS) {
                s_words[wave][q * L + t] = w;
            } else {
                dlo[2 * q] = w.x; dhi[2 * q] = w.y; dlo[2 * q + 1] = w.z; dhi[2 * q + 1] = w.w;
            }
        }
#pragma unroll(LC ? LC : 1)
        for (uint32_t p = 0; p < l; p++) {
            const uint32_t sh = 32 - (p + 1) * bg_bit;
            const uint32_t r = c * l + p;
            double xr[P], xi[P];
            if constexpr (WORDS_IN_LDS) {
#pragma unroll
                for (int q = 0; q < Q; q++) {
                    const uint4 w = s_words[wave][q * L + t];
                    xr[2 * q] = (double)(int)__builtin_amdgcn_sbfe(w.x, sh, bg_bit);
                    xi[2 * q] = (double)(int)__builtin_amdgcn_sbfe(w.y, sh, bg_bit);
                    xr[2 * q + 1] = (double)(int)__builtin_amdgcn_sbfe(w.z, sh, bg_bit);
                    xi[2 * q + 1] = (double)(int)__builtin_amdgcn_sbfe(w.w, sh, bg_bit);
                }
            } else {
#pragma unroll
                for (int m = 0; m < P; m++) {
                    xr[m] = (double)(int)__builtin_amdgcn_sbfe(dlo[m], sh, bg_bit);
                    xi[m] = (double)(int)__builtin_amdgcn_sbfe(dhi[m], sh, bg_bit);
                }
            }
            forward<PL>(lc, xr, xi);
            if constexpr (ROW_AHEAD) {
#pragma unroll
                for (int o = 0; o < 2; o++)
#pragma unroll
                    for (int k = 0; k < P; k++) {
                        const double2 b = bv[o][k];
                        sr[o][k] = __builtin_fma(-xi[k], b.y, __builtin_fma(xr[k], b.x, sr[o][k]));
                        si[o][k] = __builtin_fma(xi[k], b.x, __builtin_fma(xr[k], b.y, si[o][k]));
                    }
            } else {
                // no room for a row: the selector's values for RING points are in flight while the products of the
                // points before them run (a transformed value's registers are free once both outputs have used it)
                constexpr int RING = 4;
                const double2 *row = rows + (size_t)r * 2 * P * L;
                double2 ring[RING][2];
                __builtin_amdgcn_sched_barrier(0);                        // not into the transform: no register is free there
#pragma unroll
                for (int k = 0; k < RING; k++) { ring[k][0] = row[k * L]; ring[k][1] = row[(P + k) * L]; }
#pragma unroll
                for (int k = 0; k < P; k++) {
                    const double2 b0 = ring[k % RING][0], b1 = ring[k % RING][1];
                    if (k + RING < P) { ring[k % RING][0] = row[(k + RING) * L]; ring[k % RING][1] = row[(P + k + RING) * L]; }
                    sr[0][k] = __builtin_fma(-xi[k], b0.y, __builtin_fma(xr[k], b0.x, sr[0][k]));
                    si[0][k] = __builtin_fma(xi[k], b0.x, __builtin_fma(xr[k], b0.y, si[0][k]));
                    sr[1][k] = __builtin_fma(-xi[k], b1.y, __builtin_fma(xr[k], b1.x, sr[1][k]));
                    si[1][k] = __builtin_fma(xi[k], b1.x, __builtin_fma(xr[k], b1.y, si[1][k]));
                }
            }
            if (ROW_AHEAD && r + 1 < 2 * l) {
                const double2 *row = rows + (size_t)(r + 1) * 2 * P * L;
#pragma unroll
                for (int o = 0; o < 2; o++)
#pragma unroll
                    for (int k = 0; k < (ROW_AHEAD ? P : 0); k++) bv[o][k] = row[(o * P + k) * L];
            }
        }
    }
    // the words of d0 that the products are added to, and the next CMux's first component (this one's again after the
    // last: harmless), requested ahead of the inverse transforms
    uint4 base[2][AHEAD ? Q : 1];
    if constexpr (AHEAD) {
        const uint32_t gn = g + stride < count ? g + stride : g;
        const uint4 *a1 = reinterpret_cast<const uint4 *>(trlwe + (size_t)in1[gn] * 2 * N) + t;
        const uint4 *a0 = reinterpret_cast<const uint4 *>(trlwe + (size_t)in0[gn] * 2 * N) + t;
        // the next CMux's second component goes to LDS (this one's was consumed before its transforms).  After a
        // wavefront's last CMux this loads its own words once more: loads return in order, and the result's stores
        // wait for `base`, requested after it, so no wavefront leaves with such a load in flight.
        if constexpr (STAGE) {
#pragma unroll
            for (int q = 0; q < Q; q++) {
                load_to_lds16(a1 + N / 4 + q * L, &s_stage[wave][q * L]);
                load_to_lds16(a0 + N / 4 + q * L, &s_stage[wave][(Q + q) * L]);
            }
        }
#pragma unroll
        for (int o = 0; o < 2; o++) {
            const uint4 *b0 = reinterpret_cast<const uint4 *>(d0 + o * N) + t;
#pragma unroll
            for (int q = 0; q < Q; q++) base[o][q] = b0[q * L];
        }
#pragma unroll
        for (int q = 0; q < Q; q++) { pu[q] = a1[q * L]; pv[q] = a0[q * L]; }
    }
    {
        double2 *const xch2[2] = {lc.xch, lc.xch};
        inverse_n<PL, 2, true>(lc, xch2, sr, si);
    }
#pragma unroll
    for (int o = 0; o < 2; o++) {
        uint4 *ao = reinterpret_cast<uint4 *>(dst + o * N) + t;
#pragma unroll
        for (int q = 0; q < Q; q++) {
            if (TRACK) {
#pragma unroll
                for (int m = 2 * q; m < 2 * q + 2; m++) {
                    worst = fmaxf(worst, (float)fabs(sr[o][m] - rint(sr[o][m])));
                    worst = fmaxf(worst, (float)fabs(si[o][m] - rint(si[o][m])));
                }
            }
            uint4 v = AHEAD ? base[o][AHEAD ? q : 0] : (reinterpret_cast<const uint4 *>(d0 + o * N) + t)[q * L];
            v.x += (uint32_t)__double2loint(sr[o][2 * q] + 6755399441055744.0);
            v.y += (uint32_t)__double2loint(si[o][2 * q] + 6755399441055744.0);
            v.z += (uint32_t)__double2loint(sr[o][2 * q + 1] + 6755399441055744.0);
            v.w += (uint32_t)__double2loint(si[o][2 * q + 1] + 6755399441055744.0);
            ao[q * L] = v;
        }
    }
    wave_lds_fence();                                                     // the exchange buffer is reused by the next CMux
    }
    if (TRACK && round_err) atomicMax(round_err, __float_as_uint(worst));
}

// ------------------------------------------------------------------------------------------
// Key switch.  Block = KS_GROUP gates x KS_COLS output words; every thread owns one output
// word of all the gates, so each key row that is loaded serves KS_GROUP gates.
// ------------------------------------------------------------------------------------------
constexpr int KS_COLS = 128;

__global__ __launch_bounds__(KS_COLS) void k_key_switch(CtSpace cs, const uint32_t *__restrict__ ks,
                                                        uint32_t ks_stride, const uint16_t *__restrict__ ksd,
                                                        const uint32_t *__restrict__ ext_b,
                                                        const uint32_t *__restrict__ out_ids, uint32_t N, uint32_t t,
                                                        uint32_t bb, uint32_t n, uint32_t gates)
{
    const uint32_t grp = blockIdx.x;
    const uint32_t col = blockIdx.y * KS_COLS + threadIdx.x;
    const uint32_t colc = col <= n ? col : n;
    const uint32_t nrows = (1u << bb) - 1;
    uint32_t acc[KS_GROUP];
#pragma unroll
    for (int g = 0; g < KS_GROUP; g++) acc[g] = 0;

    const uint32_t *dg = (const uint32_t *)(ksd + (size_t)grp * N * KS_GROUP);
    for (uint32_t i = 0; i < N; i++) {
        uint32_t yw[KS_GROUP / 2];
#pragma unroll
        for (int q = 0; q < KS_GROUP / 2; q++) yw[q] = dg[(size_t)i * (KS_GROUP / 2) + q];
        for (uint32_t j = 0; j < t; j++) {
            const uint32_t sh = (t - 1 - j) * bb;
            const uint32_t *rows = ks + ((size_t)(i * t + j) * nrows) * ks_stride + colc;
            for (uint32_t v = 1; v <= nrows; v++) {
                const uint32_t r = rows[(size_t)(v - 1) * ks_stride];
#pragma unroll
                for (int g = 0; g < KS_GROUP; g++) {
                    const uint32_t y = (yw[g >> 1] >> (16 * (g & 1))) & 0xffffu;
                    const uint32_t d = (y >> sh) & nrows;
                    acc[g] -= (d == v) ? r : 0u;
                }
            }
        }
    }
    if (col > n) return;
#pragma unroll
    for (int g = 0; g < KS_GROUP; g++) {
        const uint32_t gi = grp * KS_GROUP + g;
        if (gi < gates) {
            uint32_t v = acc[g];
            if (col == n) v += ext_b[gi];
            ct_ptr(cs, out_ids[gi])[col] = v;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Key switch as an int8 matrix product on the MFMA units (base 4, 8 digits).
//   out[g][c] = (0, b'')[c] - sum_{i,j} KS[i][j][d_gij][c]
// is sum_k A[g][k] * KS[k][c] with A the one-hot encoding of the digits, k = (i, j, v).  A is
// 0/1 and every KS word is split into four signed bytes, so four i32 += i8*i8 products
// (|sum| <= 2^20) recombined with shifts give the exact result modulo 2^32.
// One v_mfma_i32_32x32x32_i8 consumes the 32 k of one i (8 digits x 4 values; the v = 0
// column of A is always 0).  A wavefront owns 64 gates x 32 output words; a block of four
// wavefronts shares the key bytes through LDS; blockIdx.z splits the i range and partial
// sums are subtracted atomically from the slot that the blind rotation initialised.
// ------------------------------------------------------------------------------------------
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
constexpr int KSM_WAVES = 4, KSM_TILES = 2;   // measured: 1 tile (4 or 6 waves per SIMD), 3 and 4 tiles are slower

__device__ __forceinline__ int onehot_byte(uint32_t d) { return (int)((1u << (d << 3)) & 0xFFFFFF00u); }

// The four wavefronts of a workgroup work on the same 32 output words, so the 4 KiB of key bytes of a step (four byte
// planes x 64 lanes x 16 bytes) are fetched once per workgroup, wavefront w bringing plane w straight into LDS
// (global_load_lds), and every wavefront reads them from there.  (Each wavefront loading them for itself through the
// vector L1 kept that cache's pending-request stall at 60 % of the kernel's time: 0.375 against 0.278 ms per 4096 gates.)
// Two stages: a step's bytes are requested during the step before; requesting two steps ahead through four stages is
// no faster (0.284 ms).  Every wavefront of a workgroup meets every barrier: one with no gates of its own still brings
// its plane.  i_per_block must be even.
__global__ __launch_bounds__(64 * KSM_WAVES, 3) void k_key_switch_mfma(CtSpace cs, const int8_t *__restrict__ ksb,
                                                                     uint32_t cols_p, const uint16_t *__restrict__ ksd,
                                                                     const uint32_t *__restrict__ out_ids, uint32_t N,
                                                                     uint32_t n, uint32_t gates, uint32_t i_per_block)
{
    __shared__ uint4 s_b0[4 * 64], s_b1[4 * 64];                           // [plane][lane], one array per stage
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5, c32 = lane & 31;
    const uint32_t tile_first = blockIdx.x * KSM_WAVES * KSM_TILES;              // live: the workgroup exists for it
    const uint32_t tile0 = tile_first + wave * KSM_TILES;                        // in units of 32 gates
    const uint32_t col = blockIdx.y * 32 + c32;
    const uint32_t i0 = blockIdx.z * i_per_block, i1 = min(N, i0 + i_per_block);

    v16i acc[KSM_TILES][4];
#pragma unroll
    for (int t = 0; t < KSM_TILES; t++)
#pragma unroll
        for (int p = 0; p < 4; p++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[t][p][r] = 0;

    const uint16_t *yp[KSM_TILES];
    bool tile_live[KSM_TILES];
#pragma unroll
    for (int t = 0; t < KSM_TILES; t++) {
        tile_live[t] = (tile0 + t) * 32 < gates;
        yp[t] = ksd + ((size_t)(tile_live[t] ? tile0 + t : tile_first) * N) * KS_GROUP + c32;
    }
    // this wavefront's plane of a step: 1 KiB, lane (half, c32) takes the 16 bytes of column c32, half `half`
    const uint4 *mine = reinterpret_cast<const uint4 *>(ksb + ((size_t)wave * cols_p + col) * 32 + 16 * half);
    const size_t step_u4 = (size_t)4 * cols_p * 2;                          // one i further, in 16-byte units
    const uint32_t ysh = 8 * (1 - half);

    uint32_t y_next[KSM_TILES];
    load_to_lds16(mine + (size_t)i0 * step_u4, s_b0 + wave * 64);
#pragma unroll
    for (int t = 0; t < KSM_TILES; t++) y_next[t] = yp[t][(size_t)i0 * KS_GROUP];

    auto step = [&](uint32_t i, const uint4 *cur, uint4 *other) {
        // this step's bytes have landed (every wavefront waits for its own plane, then all meet), and nobody still
        // reads the other stage (its readers waited for their values before their products, a step ago)
        __builtin_amdgcn_s_waitcnt(0x0F70);                                 // vmcnt(0)
        __builtin_amdgcn_s_barrier();
        uint32_t yv[KSM_TILES];
#pragma unroll
        for (int t = 0; t < KSM_TILES; t++) yv[t] = y_next[t];
        const uint32_t in = min(i + 1, i1 - 1);                             // past the end: the last step again, unused
        load_to_lds16(mine + (size_t)in * step_u4, other + wave * 64);
#pragma unroll
        for (int t = 0; t < KSM_TILES; t++) y_next[t] = yp[t][(size_t)in * KS_GROUP];
        __builtin_amdgcn_sched_barrier(0);                                  // the requests stay ahead of the products
        v4i b[4];
#pragma unroll
        for (int p = 0; p < 4; p++) {
            const uint4 w = cur[p * 64 + lane];
            b[p] = v4i{(int)w.x, (int)w.y, (int)w.z, (int)w.w};
        }
#pragma unroll
        for (int t = 0; t < KSM_TILES; t++) {
            const uint32_t y = (yv[t] >> ysh) & 0xffu;                                    // this half's four digits
            v4i a;
            a.x = onehot_byte((y >> 6) & 3);
            a.y = onehot_byte((y >> 4) & 3);
            a.z = onehot_byte((y >> 2) & 3);
            a.w = onehot_byte(y & 3);
#pragma unroll
            for (int p = 0; p < 4; p++) acc[t][p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b[p], acc[t][p], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);                                  // the next step's wait stays behind the products
    };
    for (uint32_t i = i0; i < i1; i += 2) {
        step(i, s_b0, s_b1);
        step(i + 1, s_b1, s_b0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                                     // no load into LDS is in flight at the end

    if (col > n) return;
#pragma unroll
    for (int t = 0; t < KSM_TILES; t++) {
        if (!tile_live[t]) continue;
#pragma unroll
        for (int r = 0; r < 16; r++) {
            const uint32_t row = 8 * (r / 4) + 4 * half + (r % 4);
            const uint32_t g = (tile0 + t) * 32 + row;
            if (g >= gates) continue;
            const uint32_t v = (uint32_t)acc[t][0][r] + ((uint32_t)acc[t][1][r] << 8) + ((uint32_t)acc[t][2][r] << 16) +
                               ((uint32_t)acc[t][3][r] << 24);
            atomicAdd(ct_ptr(cs, out_ids[g]) + col, 0u - v);
        }
    }
}

// ------------------------------------------------------------------------------------------
// Pool plumbing
// ------------------------------------------------------------------------------------------
__global__ void k_scatter(CtSpace cs, const uint32_t *__restrict__ src, const uint32_t *__restrict__ ids, uint32_t n)
{
    uint32_t *dst = ct_ptr(cs, ids[blockIdx.x]);
    const uint32_t *s = src + (size_t)blockIdx.x * (n + 1);
    for (uint32_t i = threadIdx.x; i <= n; i += blockDim.x) dst[i] = s[i];
}
__global__ void k_gather(CtSpace cs, uint32_t *__restrict__ dst, const uint32_t *__restrict__ ids, uint32_t n)
{
    const uint32_t *s = ct_ptr(cs, ids[blockIdx.x]);
    uint32_t *d = dst + (size_t)blockIdx.x * (n + 1);
    for (uint32_t i = threadIdx.x; i <= n; i += blockDim.x) d[i] = s[i];
}
// dst <- src, or its complement (word-wise negation) when the source id carries WIRE_NEG
__global__ void k_copy_ct(CtSpace cs, const uint32_t *__restrict__ src_ids, const uint32_t *__restrict__ dst_ids,
                          uint32_t n)
{
    const uint32_t ref = src_ids[blockIdx.x];
    const bool neg = (ref & WIRE_NEG) != 0;
    const uint32_t *s = ct_ptr(cs, ref & ~WIRE_NEG);
    uint32_t *d = ct_ptr(cs, dst_ids[blockIdx.x]);
    for (uint32_t i = threadIdx.x; i <= n; i += blockDim.x) d[i] = neg ? 0u - s[i] : s[i];
}

// ------------------------------------------------------------------------------------------
// Host launchers
// ------------------------------------------------------------------------------------------
using Plan256 = Plan<1, 7>;
using Plan512 = Plan<2, 4>;
using Plan1024 = Plan<3, 3>;

// N = 2048 has transforms, key spectra and the leveled CMux; the blind rotation is built for N <= 1024
bool plan_supported(uint32_t N) { return N == 256 || N == 512 || N == 1024 || N == 2048; }

template <class PL> static size_t tw_doubles() { return 2 * (size_t)TwTable<PL>::COUNT; }

size_t twiddle_doubles(uint32_t N)
{
    switch (N) {
    case 256: return tw_doubles<Plan256>();
    case 512: return tw_doubles<Plan512>();
    case 1024: return tw_doubles<Plan1024>();
    case 2048: return tw_doubles<Plan2048>();
    }
    return 0;
}

void fill_twiddles(uint32_t N, double *out)
{
    switch (N) {
    case 256: make_twiddles<Plan256>(out); break;
    case 512: make_twiddles<Plan512>(out); break;
    case 1024: make_twiddles<Plan1024>(out); break;
    case 2048: make_twiddles<Plan2048>(out); break;
    }
}

size_t bk_hat_elems(const she_params &P) { return (size_t)P.n * 2 * P.l * 2 * (P.N / 2); }

template <class PL>
static hipError_t bk_transform_t(const she_params &P, const uint32_t *d_bk_int, const DeviceKeys &K, hipStream_t st)
{
    const uint32_t polys = P.n * 2 * P.l * 2;
    const uint32_t per_block = BR_WAVES * PL::GPW;
    hipLaunchKernelGGL((k_bk_transform<PL>), dim3((polys + per_block - 1) / per_block), dim3(64 * BR_WAVES), 0, st,
                       d_bk_int, K.twiddles, K.bk_hat, polys, (const uint32_t *)nullptr, 1u);
    return hipGetLastError();
}

template <class PL>
static hipError_t trgsw_transform_t(const she_params &P, const DeviceKeys &K, const uint32_t *d_int, double2 *trgsw_hat,
                                    const uint32_t *d_ids, size_t samples, hipStream_t st)
{
    const uint32_t pps = 2 * P.l * 2, polys = (uint32_t)(samples * pps);
    const uint32_t per_block = BR_WAVES * PL::GPW;
    hipLaunchKernelGGL((k_bk_transform<PL>), dim3((polys + per_block - 1) / per_block), dim3(64 * BR_WAVES), 0, st,
                       d_int, K.twiddles, trgsw_hat, polys, d_ids, pps);
    return hipGetLastError();
}

template <class PL>
static hipError_t cmux_t(const she_params &P, const DeviceKeys &K, const double2 *trgsw_hat, uint32_t *trlwe,
                         const uint32_t *d_sel, const uint32_t *d_in1, const uint32_t *d_in0, const uint32_t *d_out,
                         size_t count, unsigned *d_round_err, hipStream_t st)
{
    // persistent: at most the workgroups per compute unit that fit (two; one at N = 2048), each wavefront loops over its share
    const size_t wgs = (count + BR_WAVES - 1) / BR_WAVES;
    const size_t per_cu = 2;
    const dim3 grid((unsigned)std::min<size_t>(wgs, per_cu * std::max<uint32_t>(K.cus, 1))), block(64 * BR_WAVES);
    if (d_round_err)
        hipLaunchKernelGGL((k_cmux<PL, true, 0>), grid, block, 0, st, trgsw_hat, trlwe, d_sel, d_in1, d_in0, d_out,
                           (uint32_t)count, P.l, P.bg_bit, K.twiddles, d_round_err);
    else if (P.l == 3 && PL::P <= 8)
        hipLaunchKernelGGL((k_cmux<PL, false, 3>), grid, block, 0, st, trgsw_hat, trlwe, d_sel, d_in1, d_in0, d_out,
                           (uint32_t)count, P.l, P.bg_bit, K.twiddles, d_round_err);
    else
        hipLaunchKernelGGL((k_cmux<PL, false, 0>), grid, block, 0, st, trgsw_hat, trlwe, d_sel, d_in1, d_in0, d_out,
                           (uint32_t)count, P.l, P.bg_bit, K.twiddles, d_round_err);
    return hipGetLastError();
}

hipError_t launch_trgsw_transform(const she_params &P, const DeviceKeys &K, const uint32_t *d_int, double2 *trgsw_hat,
                                  const uint32_t *d_ids, size_t samples, hipStream_t st)
{
    if (!samples) return hipSuccess;
    switch (P.N) {
    case 256: return trgsw_transform_t<Plan256>(P, K, d_int, trgsw_hat, d_ids, samples, st);
    case 512: return trgsw_transform_t<Plan512>(P, K, d_int, trgsw_hat, d_ids, samples, st);
    case 1024: return trgsw_transform_t<Plan1024>(P, K, d_int, trgsw_hat, d_ids, samples, st);
    case 2048: return trgsw_transform_t<Plan2048>(P, K, d_int, trgsw_hat, d_ids, samples, st);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_cmux(const she_params &P, const DeviceKeys &K, const double2 *trgsw_hat, uint32_t *trlwe,
                       const uint32_t *d_sel, const uint32_t *d_in1, const uint32_t *d_in0, const uint32_t *d_out,
                       size_t count, unsigned *d_round_err, hipStream_t st)
{
    if (!count) return hipSuccess;
    switch (P.N) {
    case 256: return cmux_t<Plan256>(P, K, trgsw_hat, trlwe, d_sel, d_in1, d_in0, d_out, count, d_round_err, st);
    case 512: return cmux_t<Plan512>(P, K, trgsw_hat, trlwe, d_sel, d_in1, d_in0, d_out, count, d_round_err, st);
    case 1024: return cmux_t<Plan1024>(P, K, trgsw_hat, trlwe, d_sel, d_in1, d_in0, d_out, count, d_round_err, st);
    case 2048: return cmux_t<Plan2048>(P, K, trgsw_hat, trlwe, d_sel, d_in1, d_in0, d_out, count, d_round_err, st);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_bk_transform(const she_params &P, const uint32_t *d_bk_int, const DeviceKeys &K, hipStream_t st)
{
    switch (P.N) {
    case 256: return bk_transform_t<Plan256>(P, d_bk_int, K, st);
    case 512: return bk_transform_t<Plan512>(P, d_bk_int, K, st);
    case 1024: return bk_transform_t<Plan1024>(P, d_bk_int, K, st);
    case 2048: return bk_transform_t<Plan2048>(P, d_bk_int, K, st);
    }
    return hipErrorInvalidValue;
}

static uint32_t ilog2(uint32_t v) { uint32_t r = 0; while ((1u << r) < v) r++; return r; }

hipError_t launch_lincomb(const she_params &P, const CtSpace &cs, const uint8_t *d_type, const uint32_t *d_in0,
                          const uint32_t *d_in1, const uint32_t *d_in2, size_t gates, const LevelWork &W, hipStream_t st)
{
    if (!gates) return hipSuccess;
    hipLaunchKernelGGL(k_lincomb, dim3((unsigned)gates), dim3(128), 0, st, cs, d_type, d_in0, d_in1, d_in2, P.n,
                       ilog2(2 * P.N), W.bar, W.bar_stride);
    return hipGetLastError();
}

template <class PL>
static hipError_t blind_rotate_t(const she_params &P, const DeviceKeys &K, size_t gates, const LevelWork &W,
                                 unsigned *d_round_err, const CtSpace &cs, const uint32_t *d_out, hipStream_t st,
                                 uint32_t *raw_ext, bool split)
{
    const uint32_t ks_bits = P.ks_t * P.ks_basebit;
    if (split) {
        // One gate (two wavefronts) or two gates per workgroup.  Measured at n=630, N=1024 on 256 compute units, in ms
        // for 256 / 512 / 768 / 1024 / 1280 / 1536 gates: one per workgroup 3.4 / 5.1 / 5.3 / 6.2 / 9.2 / 12.1, two per
        // workgroup 4.2 / 4.2 / 6.2 / 6.3 / 10.1 / 9.8 (the unsplit kernel: 6.5 up to 1024 gates, 10.4 to 11.1 beyond).
        // What counts is the wavefronts on the fullest compute unit; two workgroups of one gate share a SIMD pair badly.
        const size_t per_cu = (gates + K.cus - 1) / std::max<uint32_t>(K.cus, 1);
        const bool two = per_cu == 2 || per_cu == 6;
        const dim3 grid((unsigned)(two ? (gates + 1) / 2 : gates)), block(two ? 256 : 128);
#define SHE_LAUNCH_SPLIT(TRACK, GB, LR)                                                                               \
    hipLaunchKernelGGL((k_blind_rotate_split<PL, TRACK, GB, LR>), grid, block, 0, st, W.bar, W.bar_stride, P.n, P.l,  \
                       P.bg_bit, K.bk_hat, K.twiddles, ks_bits, W.ext_b, W.ksd, (uint32_t)gates, d_round_err, cs,     \
                       d_out, raw_ext)
        const bool triple = P.l == 3;
        if (triple) {
            if (d_round_err) { if (two) SHE_LAUNCH_SPLIT(true, 2, 3); else SHE_LAUNCH_SPLIT(true, 1, 3); }
            else { if (two) SHE_LAUNCH_SPLIT(false, 2, 3); else SHE_LAUNCH_SPLIT(false, 1, 3); }
        } else {
            if (d_round_err) { if (two) SHE_LAUNCH_SPLIT(true, 2, 0); else SHE_LAUNCH_SPLIT(true, 1, 0); }
            else { if (two) SHE_LAUNCH_SPLIT(false, 2, 0); else SHE_LAUNCH_SPLIT(false, 1, 0); }
        }
#undef SHE_LAUNCH_SPLIT
        return hipGetLastError();
    }
    const uint32_t per_block = BR_WAVES * PL::GPW;
    const dim3 grid((unsigned)((gates + per_block - 1) / per_block)), block(64 * BR_WAVES);
    if (d_round_err)
        hipLaunchKernelGGL((k_blind_rotate<PL, true, 0>), grid, block, 0, st, W.bar, W.bar_stride, P.n, P.l, P.bg_bit,
                           K.bk_hat, K.twiddles, ks_bits, W.ext_b, W.ksd, (uint32_t)gates, d_round_err, cs, d_out, raw_ext);
    else if (P.l == 3)
        hipLaunchKernelGGL((k_blind_rotate<PL, false, 3>), grid, block, 0, st, W.bar, W.bar_stride, P.n, P.l, P.bg_bit,
                           K.bk_hat, K.twiddles, ks_bits, W.ext_b, W.ksd, (uint32_t)gates, d_round_err, cs, d_out, raw_ext);
    else
        hipLaunchKernelGGL((k_blind_rotate<PL, false, 0>), grid, block, 0, st, W.bar, W.bar_stride, P.n, P.l, P.bg_bit,
                           K.bk_hat, K.twiddles, ks_bits, W.ext_b, W.ksd, (uint32_t)gates, d_round_err, cs, d_out, raw_ext);
    return hipGetLastError();
}

hipError_t launch_blind_rotate(const she_params &P, const DeviceKeys &K, const CtSpace &cs, const uint32_t *d_out,
                               size_t gates, const LevelWork &W, unsigned *d_round_err, hipStream_t st, bool raw, bool split)
{
    if (!gates) return hipSuccess;
    if (!K.ks_bytes) d_out = nullptr;      // the generic key switch writes the slot itself
    uint32_t *raw_ext = raw ? W.raw_ext : nullptr;
    switch (P.N) {
    case 256: return blind_rotate_t<Plan256>(P, K, gates, W, d_round_err, cs, d_out, st, raw_ext, split);
    case 512: return blind_rotate_t<Plan512>(P, K, gates, W, d_round_err, cs, d_out, st, raw_ext, split);
    case 1024: return blind_rotate_t<Plan1024>(P, K, gates, W, d_round_err, cs, d_out, st, raw_ext, split);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_mux_combine(const she_params &P, const DeviceKeys &K, const CtSpace &cs, const uint32_t *d_out,
                              size_t muxes, const LevelWork &W, hipStream_t st)
{
    if (!muxes) return hipSuccess;
    hipLaunchKernelGGL(k_mux_combine, dim3((unsigned)muxes), dim3(256), 0, st, W.raw_ext, P.N, P.n,
                       P.ks_t * P.ks_basebit, W.ext_b, W.ksd, cs, K.ks_bytes ? d_out : nullptr);
    return hipGetLastError();
}

hipError_t launch_key_switch(const she_params &P, const DeviceKeys &K, const CtSpace &cs, const uint32_t *d_out,
                             size_t gates, const LevelWork &W, hipStream_t st)
{
    if (!gates) return hipSuccess;
    if (K.ks_bytes) {
        const unsigned per_block = 32 * KSM_TILES * KSM_WAVES;                 // gates per workgroup
        const unsigned gate_blocks = (unsigned)((gates + per_block - 1) / per_block);
        const unsigned col_tiles = K.ks_cols / 32;
        // split the i range until about a thousand blocks are in flight
        unsigned split = 1;
        while (split < 32 && gate_blocks * col_tiles * split < 1024 && P.N / (split * 2) >= 8) split *= 2;
        const dim3 grid(gate_blocks, col_tiles, split);
        hipLaunchKernelGGL(k_key_switch_mfma, grid, dim3(64 * KSM_WAVES), 0, st, cs, K.ks_bytes, K.ks_cols, W.ksd, d_out,
                           P.N, P.n, (uint32_t)gates, P.N / split);              // N / split: a power of two >= 8
        return hipGetLastError();
    }
    const dim3 grid((unsigned)((gates + KS_GROUP - 1) / KS_GROUP), (P.n + 1 + KS_COLS - 1) / KS_COLS);
    hipLaunchKernelGGL(k_key_switch, grid, dim3(KS_COLS), 0, st, cs, K.ks, K.ks_stride, W.ksd, W.ext_b, d_out, P.N,
                       P.ks_t, P.ks_basebit, P.n, (uint32_t)gates);
    return hipGetLastError();
}

hipError_t launch_scatter(const CtSpace &cs, const uint32_t *d_src, const uint32_t *d_ids, size_t count, uint32_t n,
                          hipStream_t st)
{
    if (!count) return hipSuccess;
    hipLaunchKernelGGL(k_scatter, dim3((unsigned)count), dim3(128), 0, st, cs, d_src, d_ids, n);
    return hipGetLastError();
}
hipError_t launch_gather(const CtSpace &cs, uint32_t *d_dst, const uint32_t *d_ids, size_t count, uint32_t n,
                         hipStream_t st)
{
    if (!count) return hipSuccess;
    hipLaunchKernelGGL(k_gather, dim3((unsigned)count), dim3(128), 0, st, cs, d_dst, d_ids, n);
    return hipGetLastError();
}
hipError_t launch_copy_ct(const CtSpace &cs, const uint32_t *d_src_ids, const uint32_t *d_dst_ids, size_t count,
                          uint32_t n, hipStream_t st)
{
    if (!count) return hipSuccess;
    hipLaunchKernelGGL(k_copy_ct, dim3((unsigned)count), dim3(128), 0, st, cs, d_src_ids, d_dst_ids, n);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Scratch of the entry point that allocates nothing (she_eval_gates_device_noalloc): the level's rounded
// samples, extracted bodies and key-switch digits live in this file-scope array instead of allocated
// buffers.  Every GPU that loads the library holds its own 16 MiB copy until the process ends.  In host code
// the array's name is only a stand-in: the device address comes from hipGetSymbolAddress, once per device
// with that device current, and only that pointer is handed to kernels.
// ------------------------------------------------------------------------------------------
constexpr size_t NOALLOC_SCRATCH_BYTES = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];

hipError_t noalloc_scratch(int device, void **ptr, size_t *bytes)
{
    constexpr int MAX_DEVICES = 64;
    static void *address[MAX_DEVICES] = {};
    static std::mutex guard;
    if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(guard);
    if (!address[device]) {
        int current = -1;
        hipError_t rc = hipGetDevice(&current);
        if (rc != hipSuccess) return rc;
        if (current != device) return hipErrorInvalidDevice;
        void *p = nullptr;
        rc = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (rc != hipSuccess) return rc;
        if (!p) return hipErrorInvalidSymbol;
        address[device] = p;
    }
    *ptr = address[device];
    *bytes = NOALLOC_SCRATCH_BYTES;
    return hipSuccess;
}

// ------------------------------------------------------------------------------------------
// FP64 issue-rate probe (diagnostic): independent chains of one instruction form, 2 wavefronts per SIMD
// like the blind rotation.  form 0: fma with scalar multiplier and addend (the best case), 1: fma with
// three vector-register operands (the form of the pointwise products), 2: add of two vector registers
// (the butterflies).  form 3: the add stream of form 2 with the blind rotation's memory instructions
// beside it, per 64 additions 6 LDS reads and 3 LDS writes of 16 bytes per lane in the exchange buffer's
// layout and 2 global loads of 16 bytes per lane that stream `src` the way the key rows are streamed
// (the kernel has 6.5, 3.3 and 2.5 per 64 FP64 instructions); every loaded value is consumed by one of
// the 64 additions.  out receives one value per thread so that the chains stay alive.
// ------------------------------------------------------------------------------------------
template <int FORM> __global__ __launch_bounds__(256) void k_fp64_probe(double *out, int iters, double mul, double add,
                                                                        const double2 *__restrict__ src, uint32_t src_rows)
{
    double a[8], b = mul + threadIdx.x * 1e-12, c = add + threadIdx.x * 1e-15;
#pragma unroll
    for (int k = 0; k < 8; k++) a[k] = threadIdx.x * 1e-3 + k;
    if (FORM == 3) {
        __shared__ double2 s_buf[4][8 * 65];
        const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        double2 *buf = s_buf[wave];
        for (int e = lane; e < 8 * 65; e += 64) buf[e] = make_double2(0.0, 0.0);
        wave_lds_fence();
        const int rd = (lane & 7) * 65 + (lane >> 3);                      // the transposing read of an exchange
        uint32_t row = (blockIdx.x * 4 + wave) % src_rows;                  // rows of 64 x 16 bytes
        // global loads run four iterations (256 additions) ahead, about as far as the kernel requests its key rows
        double2 g[4][2];
#pragma unroll
        for (int j = 0; j < 4; j++) { g[j][0] = src[(size_t)row * 64 + lane]; g[j][1] = g[j][0]; }
        for (int it = 0; it < iters; it += 4) {
#pragma unroll
            for (int j = 0; j < 4; j++) {
                // 3 stores, 6 loads, 64 additions; loaded values replace c in 16 of the additions
                buf[0 * 65 + lane] = make_double2(a[0], a[1]);
                buf[3 * 65 + lane] = make_double2(a[2], a[3]);
                buf[6 * 65 + lane] = make_double2(a[4], a[5]);
                wave_lds_fence();
                double2 v[6];
#pragma unroll
                for (int q = 0; q < 6; q++) v[q] = buf[rd + q * 8];
#pragma unroll
                for (int rep = 0; rep < 6; rep++)
#pragma unroll
                    for (int k = 0; k < 8; k++) a[k] = a[k] + c;
                wave_lds_fence();
#pragma unroll
                for (int q = 0; q < 6; q++) { a[q] = a[q] + v[q].x; a[q + 2] = a[q + 2] + v[q].y; }
                a[0] = a[0] + g[j][0].x; a[1] = a[1] + g[j][0].y; a[2] = a[2] + g[j][1].x; a[3] = a[3] + g[j][1].y;
                row = row + 2 < src_rows ? row + 2 : 0;
                g[j][0] = src[(size_t)row * 64 + lane];
                g[j][1] = src[(size_t)(row + 1) * 64 + lane];
            }
        }
    } else {
        for (int it = 0; it < iters; it++) {
#pragma unroll
            for (int rep = 0; rep < 8; rep++)
#pragma unroll
                for (int k = 0; k < 8; k++) {
                    if (FORM == 0) a[k] = __builtin_fma(a[k], mul, add);
                    if (FORM == 1) a[k] = __builtin_fma(a[k], b, c);
                    if (FORM == 2) a[k] = a[k] + c;
                }
        }
    }
    double sum = 0;
#pragma unroll
    for (int k = 0; k < 8; k++) sum += a[k];
    out[blockIdx.x * blockDim.x + threadIdx.x] = sum;
}

// LDS throughput probe: every lane moves 16 bytes per operation, eight operations per iteration, in the exchange
// buffer's layout; ROW = slots per row.  PATTERN 0: loads of consecutive slots, 1: stores of consecutive slots,
// 2: loads at a*ROW + b + 8m for lane 8a + b, 3: loads at b*ROW + 8a + m.
template <int PATTERN, int ROW> __global__ __launch_bounds__(256) void k_lds_probe(uint32_t *out, int iters)
{
    __shared__ uint4 buf[4][8 * ROW];
    const int wave = threadIdx.x >> 6, t = threadIdx.x & 63, a = t >> 3, b8 = t & 7;
    uint4 acc = make_uint4(t, 1, 2, 3);
    uint4 *b = buf[wave];
    for (int k = t; k < 8 * ROW; k += 64) b[k] = acc;
    wave_lds_fence();
    for (int i = 0; i < iters; i++) {
#pragma unroll
        for (int m = 0; m < 8; m++) {
            if (PATTERN == 1) { acc.x += i; b[m * ROW + t] = acc; continue; }
            const uint4 v = PATTERN == 0 ? b[m * ROW + t] : PATTERN == 2 ? b[a * ROW + b8 + 8 * m] : b[b8 * ROW + 8 * a + m];
            acc.x += v.x; acc.y ^= v.y; acc.z += v.z; acc.w ^= v.w;
        }
        wave_lds_fence();
    }
    out[blockIdx.x * 256 + threadIdx.x] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

hipError_t launch_lds_probe(int form, uint32_t *d_out, uint32_t blocks, int iters, hipStream_t st)
{
    constexpr int ROW0 = Plan1024::xrow(0), ROW1 = Plan1024::xrow(1);
    switch (form) {
    case 0: hipLaunchKernelGGL((k_lds_probe<0, ROW1>), dim3(blocks), dim3(256), 0, st, d_out, iters); break;
    case 1: hipLaunchKernelGGL((k_lds_probe<1, ROW1>), dim3(blocks), dim3(256), 0, st, d_out, iters); break;
    case 2: hipLaunchKernelGGL((k_lds_probe<2, ROW0>), dim3(blocks), dim3(256), 0, st, d_out, iters); break;
    case 3: hipLaunchKernelGGL((k_lds_probe<2, 65>), dim3(blocks), dim3(256), 0, st, d_out, iters); break;
    case 4: hipLaunchKernelGGL((k_lds_probe<3, ROW1>), dim3(blocks), dim3(256), 0, st, d_out, iters); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_fp64_probe(int form, double *d_out, uint32_t blocks, int iters, const double2 *src, uint32_t src_rows,
                             hipStream_t st)
{
#define SHE_LAUNCH_PROBE(F) hipLaunchKernelGGL(k_fp64_probe<F>, dim3(blocks), dim3(256), 0, st, d_out, iters, 1.0000001, 1e-9, src, src_rows)
    switch (form) {
    case 0: SHE_LAUNCH_PROBE(0); break;
    case 1: SHE_LAUNCH_PROBE(1); break;
    case 2: SHE_LAUNCH_PROBE(2); break;
    case 3: if (!src || src_rows < 4) return hipErrorInvalidValue; SHE_LAUNCH_PROBE(3); break;
    default: return hipErrorInvalidValue;
    }
#undef SHE_LAUNCH_PROBE
    return hipGetLastError();
}

}  // namespace she
