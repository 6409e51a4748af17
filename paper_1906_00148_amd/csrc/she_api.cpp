// C ABI of the library (declared in include/she.h): context, pool, level scheduler.
#include <algorithm>
#include <cstring>
#include <memory>
#include <new>

#include "she_ctx.h"
#include "../../include/she_diag.h"

using namespace she;

namespace she {
thread_local std::string g_keygen_error;

int fail(she_ctx *c, int code, const std::string &msg)
{
    try {
        if (c) c->err = msg; else g_keygen_error = msg;
    } catch (...) {          // no memory for the text: the code still goes back
    }
    return code;
}

// what an exception that reached the C boundary becomes
int fail_exception(she_ctx *c)
{
    try {
        throw;
    } catch (const std::bad_alloc &) {
        return fail(c, SHE_ENOMEM, "host allocation failed");
    } catch (const std::exception &e) {
        return fail(c, SHE_EDEVICE, std::string("unexpected failure: ") + e.what());
    } catch (...) {
        return fail(c, SHE_EDEVICE, "unexpected failure");
    }
}
}  // namespace she

namespace she {
int ensure_stage(she_ctx *c, size_t words)
{
    if (words <= c->d_stage_words) return SHE_OK;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (c->d_stage) hipFree(c->d_stage);
    c->d_stage = nullptr; c->d_stage_words = 0;
    HIP_TRY(c, hipMalloc((void **)&c->d_stage, words * sizeof(uint32_t)));
    c->d_stage_words = words;
    return SHE_OK;
}
}  // namespace she

namespace {

CtSpace space(const she_ctx *c) { return CtSpace{c->pool, c->temp, c->cap, c->stride}; }

int ensure_temp(she_ctx *c, size_t slots)
{
    if (slots <= c->temp_slots) return SHE_OK;
    if (c->temp) { HIP_TRY(c, hipStreamSynchronize(c->stream)); HIP_TRY(c, hipFree(c->temp)); c->temp = nullptr; c->temp_slots = 0; }
    slots = std::max<size_t>(slots + slots / 8, 1024);
    HIP_TRY(c, hipMalloc((void **)&c->temp, slots * c->stride * sizeof(uint32_t)));
    c->temp_slots = slots;
    // trivial ciphertexts of 0 and 1: zero mask, body -1/8 and +1/8
    std::vector<uint32_t> consts(2 * (size_t)c->stride, 0u);
    consts[c->P.n] = 0u - (1u << 29);
    consts[c->stride + c->P.n] = 1u << 29;
    HIP_TRY(c, hipMemcpyAsync(c->temp, consts.data(), consts.size() * sizeof(uint32_t), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return SHE_OK;
}

int ensure_work(she_ctx *c, size_t gates)
{
    if (gates <= c->work.gates) return SHE_OK;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (c->work.bar) { hipFree(c->work.bar); hipFree(c->work.ext_b); hipFree(c->work.ksd); c->work = LevelWork{}; }
    const size_t groups = (gates + KS_GROUP - 1) / KS_GROUP;
    c->work.bar_stride = round_up(c->P.n + 1, 2);
    HIP_TRY(c, hipMalloc((void **)&c->work.bar, gates * c->work.bar_stride * sizeof(uint16_t)));
    HIP_TRY(c, hipMalloc((void **)&c->work.ext_b, gates * sizeof(uint32_t)));
    HIP_TRY(c, hipMalloc((void **)&c->work.ksd, groups * c->P.N * KS_GROUP * sizeof(uint16_t)));
    HIP_TRY(c, hipMemset(c->work.ksd, 0, groups * c->P.N * KS_GROUP * sizeof(uint16_t)));
    c->work.gates = gates;
    return SHE_OK;
}

int ensure_gate_arrays(she_ctx *c, size_t gates)
{
    if (gates <= c->d_gate_cap) return SHE_OK;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (c->d_type) { hipFree(c->d_type); hipFree(c->d_in0); hipFree(c->d_in1); hipFree(c->d_in2); hipFree(c->d_out); }
    c->d_type = nullptr; c->d_in0 = c->d_in1 = c->d_in2 = c->d_out = nullptr; c->d_gate_cap = 0;
    gates += gates / 4;
    HIP_TRY(c, hipMalloc((void **)&c->d_type, gates));
    HIP_TRY(c, hipMalloc((void **)&c->d_in0, gates * sizeof(uint32_t)));
    HIP_TRY(c, hipMalloc((void **)&c->d_in1, gates * sizeof(uint32_t)));
    HIP_TRY(c, hipMalloc((void **)&c->d_in2, gates * sizeof(uint32_t)));
    HIP_TRY(c, hipMalloc((void **)&c->d_out, gates * sizeof(uint32_t)));
    c->d_gate_cap = gates;
    return SHE_OK;
}

int ensure_raw(she_ctx *c, size_t jobs)
{
    if (jobs <= c->work.raw_jobs) return SHE_OK;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (c->work.raw_ext) hipFree(c->work.raw_ext);
    c->work.raw_ext = nullptr; c->work.raw_jobs = 0;
    HIP_TRY(c, hipMalloc((void **)&c->work.raw_ext, jobs * (size_t)(c->P.N + 1) * sizeof(uint32_t)));
    c->work.raw_jobs = jobs;
    return SHE_OK;
}

int ensure_mux_arrays(she_ctx *c, size_t muxes)
{
    if (muxes <= c->d_mux_cap) return SHE_OK;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (c->d_mtype) { hipFree(c->d_mtype); hipFree(c->d_min0); hipFree(c->d_min1); hipFree(c->d_mout); }
    c->d_mtype = nullptr; c->d_min0 = c->d_min1 = c->d_mout = nullptr; c->d_mux_cap = 0;
    muxes += muxes / 4;
    HIP_TRY(c, hipMalloc((void **)&c->d_mtype, 2 * muxes));
    HIP_TRY(c, hipMalloc((void **)&c->d_min0, 2 * muxes * sizeof(uint32_t)));
    HIP_TRY(c, hipMalloc((void **)&c->d_min1, 2 * muxes * sizeof(uint32_t)));
    HIP_TRY(c, hipMalloc((void **)&c->d_mout, muxes * sizeof(uint32_t)));
    c->d_mux_cap = muxes;
    return SHE_OK;
}


// Enqueues one level (device arrays), cut into chunks of at most MAX_LEVEL_CHUNK gates.
// `W` is the level's scratch (the context's own buffers, or the caller-free static buffer); `timed` records HIP events
// around the kernels (creating an event allocates, so the entry point that must not allocate passes false).
int enqueue_level_on(she_ctx *c, const LevelWork &W, bool timed, const uint8_t *d_type, const uint32_t *d_in0,
                     const uint32_t *d_in1, const uint32_t *d_out, size_t gates, const uint32_t *d_in2 = nullptr)
{
    if (c->P.N > 1024) return fail(c, SHE_EINVAL, "gate bootstrapping is built for N <= 1024; N = 2048 serves the leveled calls");
    const CtSpace cs = space(c);
    LevelTimer *timer = timed ? &c->timer : nullptr;
    if (timed) c->timer_levels++;
    for (size_t off = 0; off < gates; off += MAX_LEVEL_CHUNK) {
        const size_t cnt = std::min<size_t>(MAX_LEVEL_CHUNK, gates - off);
        if (timer) HIP_TRY(c, timer->mark(c->stream));
        HIP_TRY(c, launch_lincomb(c->P, cs, d_type + off, d_in0 + off, d_in1 + off, d_in2 ? d_in2 + off : nullptr, cnt, W,
                                  c->stream));
        if (timer) HIP_TRY(c, timer->mark(c->stream));
        HIP_TRY(c, launch_blind_rotate(c->P, c->dk, cs, d_out + off, cnt, W, c->track_round ? c->d_round_err : nullptr, c->stream,
                                       false, cnt <= c->split_below));
        if (timer) HIP_TRY(c, timer->mark(c->stream));
        HIP_TRY(c, launch_key_switch(c->P, c->dk, cs, d_out + off, cnt, W, c->stream));
        if (timer) HIP_TRY(c, timer->mark(c->stream));
    }
    return SHE_OK;
}

int enqueue_level(she_ctx *c, const uint8_t *d_type, const uint32_t *d_in0, const uint32_t *d_in1,
                  const uint32_t *d_out, size_t gates, const uint32_t *d_in2 = nullptr)
{
    return enqueue_level_on(c, c->work, c->timing, d_type, d_in0, d_in1, d_out, gates, d_in2);
}

// Enqueues one level of native MUX entries: jobs 2m and 2m+1 are the two rotations of entry m
// (device arrays of 2*muxes jobs), d_out has one id per entry.
int enqueue_mux_level(she_ctx *c, const uint8_t *d_jtype, const uint32_t *d_jin0, const uint32_t *d_jin1,
                      const uint32_t *d_out, size_t muxes)
{
    if (c->P.N > 1024) return fail(c, SHE_EINVAL, "gate bootstrapping is built for N <= 1024; N = 2048 serves the leveled calls");
    const CtSpace cs = space(c);
    LevelTimer *timer = c->timing ? &c->timer : nullptr;
    const size_t step = MAX_LEVEL_CHUNK / 2;
    for (size_t off = 0; off < muxes; off += step) {
        const size_t cnt = std::min<size_t>(step, muxes - off);
        if (timer) HIP_TRY(c, timer->mark(c->stream));
        HIP_TRY(c, launch_lincomb(c->P, cs, d_jtype + 2 * off, d_jin0 + 2 * off, d_jin1 + 2 * off, nullptr, 2 * cnt, c->work,
                                  c->stream));
        if (timer) HIP_TRY(c, timer->mark(c->stream));
        HIP_TRY(c, launch_blind_rotate(c->P, c->dk, cs, nullptr, 2 * cnt, c->work,
                                       c->track_round ? c->d_round_err : nullptr, c->stream, true, 2 * cnt <= c->split_below));
        if (timer) HIP_TRY(c, timer->mark(c->stream));
        HIP_TRY(c, launch_mux_combine(c->P, c->dk, cs, d_out + off, cnt, c->work, c->stream));
        HIP_TRY(c, launch_key_switch(c->P, c->dk, cs, d_out + off, cnt, c->work, c->stream));
        if (timer) HIP_TRY(c, timer->mark(c->stream));
    }
    return SHE_OK;
}

// Folds the recorded events into last_ms; the stream must have finished.
int finish_timing(she_ctx *c)
{
    LevelTimer &timer = c->timer;
    const size_t levels = c->timer_levels;
    c->timer_levels = 0;
    double ms[3] = {0, 0, 0};
    for (size_t q = 0; q + 3 < timer.ev.size(); q += 4)
        for (int f = 0; f < 3; f++) {
            float t = 0;
            HIP_TRY(c, hipEventElapsedTime(&t, timer.ev[q + f], timer.ev[q + f + 1]));
            ms[f] += t;
        }
    timer.clear();
    c->last_ms[0] = ms[0]; c->last_ms[1] = ms[1]; c->last_ms[2] = ms[2]; c->last_ms[3] = (double)levels;
    return SHE_OK;
}

bool params_supported(const she_params &P, std::string &why)
{
    if (P.k != 1) { why = "k must be 1"; return false; }
    if (!plan_supported(P.N)) { why = "N must be 256, 512, 1024 or 2048"; return false; }
    if (P.n < 1 || P.n > 4096) { why = "n must be in [1, 4096]"; return false; }
    if (P.l < 1 || P.l > 8 || P.bg_bit < 1 || P.l * P.bg_bit > 31) { why = "need 1 <= l <= 8 and l*bg_bit <= 31"; return false; }
    // the FP64 transforms stay exact after rounding only while the products are small enough:
    // typical magnitude ~ sqrt(2 l N) * Bg/2 * 2^31 must leave a wide margin below 2^53.  At the bound (N = 1024,
    // l = 2, Bg = 2^10) sums of products with every digit at full magnitude land within 0.07 of an integer.
    if ((uint64_t)2 * P.l * P.N * ((uint64_t)1 << (2 * P.bg_bit)) > ((uint64_t)1 << 32)) {
        why = "need 2*l*N*Bg^2 <= 2^32 (exactness of the FP64 polynomial products)"; return false;
    }
    // the kernels round by adding 1.5*2^52 and keeping the low word, which is right for |v| < 2^51: the largest sum that
    // any digits and key words can produce is 2*l*N * Bg/2 * 2^31, so l*N*Bg must stay at or below 2^20
    if ((uint64_t)P.l * P.N * ((uint64_t)1 << P.bg_bit) > ((uint64_t)1 << 20)) {
        why = "need l*N*Bg <= 2^20 (the sums of products must stay below 2^51 for the rounding step)"; return false;
    }
    if (P.ks_t < 1 || P.ks_basebit < 1 || P.ks_basebit > 4 || P.ks_t * P.ks_basebit > 16) {
        why = "need ks_basebit <= 4 and ks_t*ks_basebit <= 16"; return false;
    }
    if (!(P.lwe_std >= 0) || !(P.bk_std >= 0)) { why = "noise deviations must be >= 0"; return false; }
    return true;
}

// Runs a finished netlist: levelize, bind outputs, upload, per level one batch of gates and one of
// MUX entries, copies, sync.
int run_netlist(she_ctx *c, Netlist &nl, const std::vector<uint32_t> &out_wires, const uint32_t *out_ids,
                uint64_t *gates_out)
{
    if (nl.overflow) return fail(c, SHE_ERANGE, "netlist too large for 31-bit wire ids");
    std::vector<size_t> mux_start;
    const std::vector<size_t> bounds = nl.levelize(&mux_start);
    nl.bind_outputs(out_wires, out_ids);
    const size_t G = nl.type.size(), levels = bounds.size() - 1;
    if (gates_out) *gates_out = G;
    // temporaries share slots by lifetime: the buffer holds the widest set of live wires, not one slot per entry
    const size_t temp_slots = nl.compact_temporaries(bounds);
    if (!temp_slots) return fail(c, SHE_EDEVICE, "internal error: a temporary lost its slot while it was live");
    int rc = ensure_temp(c, temp_slots);
    if (rc) return rc;
    // MUX entries become two rotation jobs each, kept in level order in their own arrays
    std::vector<uint8_t> jt;
    std::vector<uint32_t> j0, j1, mo;
    std::vector<size_t> mux_first(levels + 1, 0);          // index of each level's first entry in mo
    size_t widest = 0;
    for (size_t lv = 0; lv < levels; lv++) {
        mux_first[lv] = mo.size();
        for (size_t g = mux_start[lv]; g < bounds[lv + 1]; g++) {
            const uint32_t m = nl.type[g] - MUX_BASE;
            jt.push_back((uint8_t)(m >> 4)); j0.push_back(nl.in0[g]); j1.push_back(nl.in1[g]);
            jt.push_back((uint8_t)(m & 15)); j0.push_back(nl.in0[g]); j1.push_back(nl.in2[g]);
            mo.push_back(nl.out[g]);
        }
        widest = std::max(widest, std::max(mux_start[lv] - bounds[lv], 2 * (bounds[lv + 1] - mux_start[lv])));
    }
    mux_first[levels] = mo.size();
    c->level_gates.resize(levels);
    c->level_muxes.resize(levels);
    for (size_t lv = 0; lv < levels; lv++) {
        c->level_gates[lv] = mux_start[lv] - bounds[lv];
        c->level_muxes[lv] = bounds[lv + 1] - mux_start[lv];
    }
    if ((rc = ensure_work(c, std::min<size_t>(widest, MAX_LEVEL_CHUNK)))) return rc;
    if ((rc = ensure_gate_arrays(c, std::max(G, nl.copy_src.size())))) return rc;
    if (!mo.empty()) {
        if ((rc = ensure_mux_arrays(c, mo.size()))) return rc;
        if ((rc = ensure_raw(c, std::min<size_t>(widest, MAX_LEVEL_CHUNK)))) return rc;
    }
    c->timer.clear();
    c->timer_levels = 0;
    if (G) {
        HIP_TRY(c, hipMemcpyAsync(c->d_type, nl.type.data(), G, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->d_in0, nl.in0.data(), G * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->d_in1, nl.in1.data(), G * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->d_in2, nl.in2.data(), G * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->d_out, nl.out.data(), G * 4, hipMemcpyHostToDevice, c->stream));
        if (!mo.empty()) {
            HIP_TRY(c, hipMemcpyAsync(c->d_mtype, jt.data(), jt.size(), hipMemcpyHostToDevice, c->stream));
            HIP_TRY(c, hipMemcpyAsync(c->d_min0, j0.data(), j0.size() * 4, hipMemcpyHostToDevice, c->stream));
            HIP_TRY(c, hipMemcpyAsync(c->d_min1, j1.data(), j1.size() * 4, hipMemcpyHostToDevice, c->stream));
            HIP_TRY(c, hipMemcpyAsync(c->d_mout, mo.data(), mo.size() * 4, hipMemcpyHostToDevice, c->stream));
        }
        for (size_t lv = 0; lv < levels; lv++) {
            const size_t a = bounds[lv], m = mux_start[lv];
            if (m > a && (rc = enqueue_level(c, c->d_type + a, c->d_in0 + a, c->d_in1 + a, c->d_out + a, m - a, c->d_in2 + a)))
                return rc;
            const size_t f = mux_first[lv], cnt = mux_first[lv + 1] - f;
            if (cnt) {
                if (m > a) c->timer_levels--;              // gates and MUX entries of one level count once
                c->timer_levels++;
                if ((rc = enqueue_mux_level(c, c->d_mtype + 2 * f, c->d_min0 + 2 * f, c->d_min1 + 2 * f, c->d_mout + f, cnt))) return rc;
            }
        }
    }
    if (!nl.copy_src.empty()) {
        // the gate arrays are free again once the levels are enqueued in stream order
        const size_t n_copy = nl.copy_src.size();
        HIP_TRY(c, hipMemcpyAsync(c->d_in0, nl.copy_src.data(), n_copy * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->d_in1, nl.copy_dst.data(), n_copy * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, launch_copy_ct(space(c), c->d_in0, c->d_in1, n_copy, c->P.n, c->stream));
    }
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return finish_timing(c);
}

// ids must be inside the pool; marks them in `seen` (if given) and reports duplicates
int check_ids(she_ctx *c, const uint32_t *ids, size_t count, const char *what)
{
    for (size_t k = 0; k < count; k++)
        if (ids[k] >= c->cap) return fail(c, SHE_ERANGE, std::string(what) + ": id outside the pool");
    return SHE_OK;
}

int check_disjoint(she_ctx *c, const uint32_t *ins, size_t n_in, const uint32_t *ins2, size_t n_in2,
                   const uint32_t *outs, size_t n_out)
{
    std::vector<uint8_t> mark(c->cap, 0);
    for (size_t k = 0; k < n_in; k++) mark[ins[k]] = 1;
    for (size_t k = 0; k < n_in2; k++) mark[ins2[k]] = 1;
    for (size_t k = 0; k < n_out; k++) {
        if (mark[outs[k]] == 1) return fail(c, SHE_EINVAL, "an output id is also an input id");
        if (mark[outs[k]] == 2) return fail(c, SHE_EINVAL, "an output id appears twice");
        mark[outs[k]] = 2;
    }
    return SHE_OK;
}

// Runs one layer operator, or records it when a deferred circuit is open.  `build(nl, ids)` appends the operator's
// entries to nl, reading the wires ids[0..n_in), and returns its n_out output wires.
template <class BUILD>
int run_operator(she_ctx *c, const uint32_t *x_ids, size_t n_in, const uint32_t *out_ids, size_t n_out, uint64_t *gates_out,
                 BUILD build)
{
    if (!c->deferred) {
        Netlist nl(c->cap, c->fold, c->native_mux, c->cells3, c->columns);
        const std::vector<uint32_t> wires = build(nl, x_ids);
        return run_netlist(c, nl, wires, out_ids, gates_out);
    }
    Deferred &d = *c->deferred;
    // the scheduler is free to run this operator's entries before those of earlier operators that do not feed it: its
    // outputs must not land in a slot that the circuit reads as it was, nor in one that is already written
    for (size_t k = 0; k < n_out; k++) {
        if (d.read[out_ids[k]]) return fail(c, SHE_EINVAL, "deferred circuit: an output id is read by an earlier operator");
        if (d.produced[out_ids[k]] != Deferred::NONE) return fail(c, SHE_EINVAL, "deferred circuit: an output id is written twice");
    }
    try {
        std::vector<uint32_t> ids(n_in);
        for (size_t k = 0; k < n_in; k++) {
            const uint32_t w = d.produced[x_ids[k]];
            ids[k] = w == Deferred::NONE ? x_ids[k] : w;             // an earlier operator's result: its wire, not its slot
        }
        const size_t before = d.nl->type.size();
        const std::vector<uint32_t> wires = build(*d.nl, ids.data());
        if (d.nl->overflow) { c->deferred.reset(); return fail(c, SHE_ERANGE, "deferred circuit too large for 31-bit wire ids (dropped)"); }
        for (size_t k = 0; k < n_in; k++)
            if (d.produced[x_ids[k]] == Deferred::NONE) d.read[x_ids[k]] = 1;
        for (size_t k = 0; k < n_out; k++) {
            d.produced[out_ids[k]] = wires[k];
            d.out_wires.push_back(wires[k]);
            d.out_ids.push_back(out_ids[k]);
        }
        if (gates_out) *gates_out = d.nl->type.size() - before;
        return SHE_OK;
    } catch (...) {
        c->deferred.reset();                                           // the recorded netlist may be half extended
        throw;
    }
}

}  // namespace

extern "C" {

int she_defer_begin(she_ctx *c)
try {
    if (!c) return SHE_EINVAL;
    SHE_NOT_WHILE_DEFERRED(c);
    std::unique_ptr<Deferred> d(new Deferred);
    d->nl.reset(new Netlist(c->cap, c->fold, c->native_mux, c->cells3, c->columns));
    d->produced.assign(c->cap, Deferred::NONE);
    d->read.assign(c->cap, 0);
    c->deferred = std::move(d);
    return SHE_OK;
} SHE_NOTHROW(c)

int she_defer_run(she_ctx *c, uint64_t *entries_out)
try {
    if (!c) return SHE_EINVAL;
    if (entries_out) *entries_out = 0;
    if (!c->deferred) return fail(c, SHE_EINVAL, "no deferred circuit is open");
    std::unique_ptr<Deferred> d = std::move(c->deferred);              // closed whatever happens below
    if (d->out_ids.empty()) return SHE_OK;
    return run_netlist(c, *d->nl, d->out_wires, d->out_ids.data(), entries_out);
} SHE_NOTHROW(c)

int she_keygen(const she_params *params, uint64_t seed, uint32_t pool_capacity, she_ctx **out)
try {
    if (!params || !out) return fail(nullptr, SHE_EINVAL, "null argument");
    *out = nullptr;
    std::string why;
    if (!params_supported(*params, why)) return fail(nullptr, SHE_EINVAL, "unsupported parameters: " + why);
    if (pool_capacity == 0 || pool_capacity > 0x7FFFFFF0u) return fail(nullptr, SHE_EINVAL, "bad pool capacity");
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return fail(nullptr, SHE_EDEVICE, "no HIP device");

    // she_free as the deleter: an exception on the way out releases the device buffers too
    std::unique_ptr<she_ctx, void (*)(she_ctx *)> c(new (std::nothrow) she_ctx, she_free);
    if (!c) return fail(nullptr, SHE_ENOMEM, "host allocation");
    c->P = *params;
    c->cap = pool_capacity;
    c->stride = round_up(params->n + 1, 32);
    auto bail = [&](int code) { g_keygen_error = c->err; she_free(c.release()); return code; };
    if (hipGetDevice(&c->device) != hipSuccess) return bail(fail(c.get(), SHE_EDEVICE, "hipGetDevice"));
    {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device) != hipSuccess || cus < 1)
            return bail(fail(c.get(), SHE_EDEVICE, "hipDeviceGetAttribute(multiprocessor count)"));
        c->dk.cus = (uint32_t)cus;
        c->split_below = 6 * (size_t)cus;
    }

    try {
        generate_keys(c->P, seed, c->hk);
    } catch (const std::bad_alloc &) {
        return bail(fail(c.get(), SHE_ENOMEM, "host allocation for keys"));
    }

    auto body = [&]() -> int {
        she_ctx *cc = c.get();
        const she_params &P = cc->P;
        // twiddles
        std::vector<double> tw(twiddle_doubles(P.N));
        fill_twiddles(P.N, tw.data());
        HIP_TRY(cc, hipMalloc((void **)&cc->dk.twiddles, std::max<size_t>(tw.size(), 2) * sizeof(double)));
        HIP_TRY(cc, hipMemcpy(cc->dk.twiddles, tw.data(), tw.size() * sizeof(double), hipMemcpyHostToDevice));
        // bootstrapping key: upload integers, transform on the device, drop the integers
        uint32_t *d_bk_int = nullptr;
        HIP_TRY(cc, hipMalloc((void **)&d_bk_int, cc->hk.bk.size() * sizeof(uint32_t)));
        hipError_t e = hipMemcpy(d_bk_int, cc->hk.bk.data(), cc->hk.bk.size() * sizeof(uint32_t), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMalloc((void **)&cc->dk.bk_hat, bk_hat_elems(P) * sizeof(double2));
        if (e == hipSuccess) e = launch_bk_transform(P, d_bk_int, cc->dk, nullptr);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        hipFree(d_bk_int);
        HIP_TRY(cc, e);
        // key-switching key: signed byte planes for the MFMA kernel (base 4, 8 digits), else padded rows
        if (P.ks_basebit == 2 && P.ks_t == 8) {
            cc->dk.ks_cols = round_up(P.n + 1, 32);
            std::vector<int8_t> packed;
            pack_ks_bytes(P, cc->hk.ks, cc->dk.ks_cols, packed);
            HIP_TRY(cc, hipMalloc((void **)&cc->dk.ks_bytes, packed.size()));
            HIP_TRY(cc, hipMemcpy(cc->dk.ks_bytes, packed.data(), packed.size(), hipMemcpyHostToDevice));
        } else {
            const uint32_t rows = P.N * P.ks_t * ((1u << P.ks_basebit) - 1);
            cc->dk.ks_stride = cc->stride;
            HIP_TRY(cc, hipMalloc((void **)&cc->dk.ks, (size_t)rows * cc->dk.ks_stride * sizeof(uint32_t)));
            HIP_TRY(cc, hipMemset(cc->dk.ks, 0, (size_t)rows * cc->dk.ks_stride * sizeof(uint32_t)));
            HIP_TRY(cc, hipMemcpy2D(cc->dk.ks, cc->dk.ks_stride * sizeof(uint32_t), cc->hk.ks.data(), (P.n + 1) * sizeof(uint32_t),
                                    (P.n + 1) * sizeof(uint32_t), rows, hipMemcpyHostToDevice));
        }
        // pool and internal slots
        HIP_TRY(cc, hipMalloc((void **)&cc->pool, (size_t)cc->cap * cc->stride * sizeof(uint32_t)));
        HIP_TRY(cc, hipMemset(cc->pool, 0, (size_t)cc->cap * cc->stride * sizeof(uint32_t)));
        HIP_TRY(cc, hipMalloc((void **)&cc->d_round_err, sizeof(unsigned)));
        HIP_TRY(cc, hipMemset(cc->d_round_err, 0, sizeof(unsigned)));
        int rc = ensure_temp(cc, 2);
        if (rc) return rc;
        // address of this device's copy of the static scratch buffer (the entry point that allocates nothing)
        HIP_TRY(cc, noalloc_scratch(cc->device, &cc->na_scratch, &cc->na_bytes));
        return SHE_OK;
    };
    int rc = body();
    if (rc) return bail(rc);
    *out = c.release();
    return SHE_OK;
} SHE_NOTHROW(nullptr)

void she_free(she_ctx *c)
{
    if (!c) return;
    if (c->stream) hipStreamSynchronize(c->stream); else hipDeviceSynchronize();
    hipFree(c->dk.bk_hat); hipFree(c->dk.ks); hipFree(c->dk.ks_bytes); hipFree(c->dk.twiddles);
    if (c->pool_owned) hipFree(c->pool);
    hipFree(c->temp);
    hipFree(c->work.bar); hipFree(c->work.ext_b); hipFree(c->work.ksd);
    hipFree(c->d_type); hipFree(c->d_in0); hipFree(c->d_in1); hipFree(c->d_in2); hipFree(c->d_out);
    hipFree(c->d_stage); hipFree(c->d_round_err); hipFree(c->work.raw_ext);
    hipFree(c->d_mtype); hipFree(c->d_min0); hipFree(c->d_min1); hipFree(c->d_mout);
    free_leveled(c);
    delete c;
}

int she_encrypt_bits(she_ctx *c, const uint8_t *bits, size_t nbits, uint64_t enc_seed, const uint32_t *dst_ids)
try {
    if (!c) return SHE_EINVAL;
    SHE_NOT_WHILE_DEFERRED(c);
    if (nbits == 0) return SHE_OK;
    if (!bits || !dst_ids) return fail(c, SHE_EINVAL, "null argument");
    for (size_t k = 0; k < nbits; k++)
        if (bits[k] > 1) return fail(c, SHE_EINVAL, "bits must be 0 or 1");
    int rc = check_ids(c, dst_ids, nbits, "she_encrypt_bits");
    if (rc) return rc;
    const size_t w = c->P.n + 1;
    std::vector<uint32_t> host;
    try { host.resize(nbits * w); } catch (const std::bad_alloc &) { return fail(c, SHE_ENOMEM, "host staging"); }
    fresh_samples(c->P, c->hk.lwe_key, bits, nbits, enc_seed, host.data());
    if ((rc = ensure_stage(c, nbits * w + nbits))) return rc;
    uint32_t *d_ids = c->d_stage + nbits * w;
    HIP_TRY(c, hipMemcpyAsync(c->d_stage, host.data(), nbits * w * 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(d_ids, dst_ids, nbits * 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, launch_scatter(space(c), c->d_stage, d_ids, nbits, c->P.n, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return SHE_OK;
} SHE_NOTHROW(c)

static int fetch(she_ctx *c, const uint32_t *ids, size_t count, std::vector<uint32_t> &host)
{
    const size_t w = c->P.n + 1;
    try { host.resize(count * w); } catch (const std::bad_alloc &) { return fail(c, SHE_ENOMEM, "host staging"); }
    int rc = ensure_stage(c, count * w + count);
    if (rc) return rc;
    uint32_t *d_ids = c->d_stage + count * w;
    HIP_TRY(c, hipMemcpyAsync(d_ids, ids, count * 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, launch_gather(space(c), c->d_stage, d_ids, count, c->P.n, c->stream));
    HIP_TRY(c, hipMemcpyAsync(host.data(), c->d_stage, count * w * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return SHE_OK;
}

int she_decrypt(she_ctx *c, const uint32_t *ids, size_t count, uint8_t *bits_out)
try {
    if (!c) return SHE_EINVAL;
    SHE_NOT_WHILE_DEFERRED(c);
    if (count == 0) return SHE_OK;
    if (!ids || !bits_out) return fail(c, SHE_EINVAL, "null argument");
    int rc = check_ids(c, ids, count, "she_decrypt");
    if (rc) return rc;
    std::vector<uint32_t> host;
    if ((rc = fetch(c, ids, count, host))) return rc;
    phases_to_bits(c->P, c->hk.lwe_key, host.data(), count, bits_out);
    return SHE_OK;
} SHE_NOTHROW(c)

int she_eval_gates(she_ctx *c, const uint8_t *type, const uint32_t *in0, const uint32_t *in1, const uint32_t *out,
                   size_t ngates)
try {
    if (!c) return SHE_EINVAL;
    SHE_NOT_WHILE_DEFERRED(c);
    if (ngates == 0) return SHE_OK;
    if (!type || !in0 || !in1 || !out) return fail(c, SHE_EINVAL, "null argument");
    for (size_t g = 0; g < ngates; g++)
        if (type[g] >= SHE_NUM_GATES) return fail(c, SHE_EINVAL, "unknown gate code");
    int rc;
    if ((rc = check_ids(c, in0, ngates, "she_eval_gates in0"))) return rc;
    if ((rc = check_ids(c, in1, ngates, "she_eval_gates in1"))) return rc;
    if ((rc = check_ids(c, out, ngates, "she_eval_gates out"))) return rc;
    if ((rc = check_disjoint(c, in0, ngates, in1, ngates, out, ngates))) return rc;
    if ((rc = ensure_work(c, std::min<size_t>(ngates, MAX_LEVEL_CHUNK)))) return rc;
    if ((rc = ensure_gate_arrays(c, ngates))) return rc;
    HIP_TRY(c, hipMemcpyAsync(c->d_type, type, ngates, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->d_in0, in0, ngates * 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->d_in1, in1, ngates * 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->d_out, out, ngates * 4, hipMemcpyHostToDevice, c->stream));
    c->timer.clear();
    c->timer_levels = 0;
    if ((rc = enqueue_level(c, c->d_type, c->d_in0, c->d_in1, c->d_out, ngates))) return rc;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return finish_timing(c);
} SHE_NOTHROW(c)

int she_eval_gates3(she_ctx *c, const uint8_t *type, const uint32_t *in0, const uint32_t *in1, const uint32_t *in2,
                    const uint32_t *out, size_t ngates)
try {
    if (!c) return SHE_EINVAL;
    SHE_NOT_WHILE_DEFERRED(c);
    if (ngates == 0) return SHE_OK;
    if (!type || !in0 || !in1 || !in2 || !out) return fail(c, SHE_EINVAL, "null argument");
    for (size_t g = 0; g < ngates; g++)
        if (type[g] < SHE_MAJ3 || type[g] >= SHE_XOR3 + 8) return fail(c, SHE_EINVAL, "unknown three-input gate code");
    int rc;
    if ((rc = check_ids(c, in0, ngates, "she_eval_gates3 in0"))) return rc;
    if ((rc = check_ids(c, in1, ngates, "she_eval_gates3 in1"))) return rc;
    if ((rc = check_ids(c, in2, ngates, "she_eval_gates3 in2"))) return rc;
    if ((rc = check_ids(c, out, ngates, "she_eval_gates3 out"))) return rc;
    if ((rc = check_disjoint(c, in0, ngates, in1, ngates, out, ngates))) return rc;
    if ((rc = check_disjoint(c, in2, ngates, nullptr, 0, out, ngates))) return rc;
    if ((rc = ensure_work(c, std::min<size_t>(ngates, MAX_LEVEL_CHUNK)))) return rc;
    if ((rc = ensure_gate_arrays(c, ngates))) return rc;
    HIP_TRY(c, hipMemcpyAsync(c->d_type, type, ngates, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->d_in0, in0, ngates * 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->d_in1, in1, ngates * 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->d_in2, in2, ngates * 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->d_out, out, ngates * 4, hipMemcpyHostToDevice, c->stream));
    c->timer.clear();
    c->timer_levels = 0;
    if ((rc = enqueue_level(c, c->d_type, c->d_in0, c->d_in1, c->d_out, ngates, c->d_in2))) return rc;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return finish_timing(c);
} SHE_NOTHROW(c)

int she_eval_gates_device(she_ctx *c, const uint8_t *d_type, const uint32_t *d_in0, const uint32_t *d_in1,
                          const uint32_t *d_out, size_t ngates)
try {
    if (!c) return SHE_EINVAL;
    SHE_NOT_WHILE_DEFERRED(c);
    if (ngates == 0) return SHE_OK;
    if (!d_type || !d_in0 || !d_in1 || !d_out) return fail(c, SHE_EINVAL, "null argument");
    int rc = ensure_work(c, std::min<size_t>(ngates, MAX_LEVEL_CHUNK));
    if (rc) return rc;
    return enqueue_level(c, d_type, d_in0, d_in1, d_out, ngates);
} SHE_NOTHROW(c)

int she_eval_gates_device_noalloc(she_ctx *c, const uint8_t *d_type, const uint32_t *d_in0, const uint32_t *d_in1,
                                  const uint32_t *d_out, size_t ngates)
try {
    if (!c) return SHE_EINVAL;
    SHE_NOT_WHILE_DEFERRED(c);
    if (ngates == 0) return SHE_OK;
    if (!d_type || !d_in0 || !d_in1 || !d_out) return fail(c, SHE_EINVAL, "null argument");
    if (!c->na_scratch) return fail(c, SHE_EDEVICE, "the static scratch buffer has no address on this device");
    // carve the level's three arrays out of the static buffer, each on a 256-byte boundary
    auto up256 = [](size_t v) { return (v + 255) & ~(size_t)255; };
    const uint32_t bar_stride = round_up(c->P.n + 1, 2);
    const size_t groups = (ngates + KS_GROUP - 1) / KS_GROUP;
    const size_t bar_bytes = up256(ngates * bar_stride * sizeof(uint16_t)), ext_bytes = up256(ngates * sizeof(uint32_t));
    const size_t ksd_bytes = up256(groups * c->P.N * KS_GROUP * sizeof(uint16_t));
    if (ngates > MAX_LEVEL_CHUNK || bar_bytes + ext_bytes + ksd_bytes > c->na_bytes) {
        const size_t per_group = KS_GROUP * (bar_stride * sizeof(uint16_t) + sizeof(uint32_t)) + c->P.N * KS_GROUP * sizeof(uint16_t);
        const size_t most = std::min<size_t>(MAX_LEVEL_CHUNK, (c->na_bytes - 3 * 256) / per_group * KS_GROUP);
        return fail(c, SHE_ERANGE, "she_eval_gates_device_noalloc: " + std::to_string(ngates) + " gates need more than the " +
                                       std::to_string(c->na_bytes) + " bytes of static scratch; at most " +
                                       std::to_string(most) + " gates per call at these parameters");
    }
    LevelWork W;
    unsigned char *base = static_cast<unsigned char *>(c->na_scratch);
    W.bar = reinterpret_cast<uint16_t *>(base);
    W.ext_b = reinterpret_cast<uint32_t *>(base + bar_bytes);
    W.ksd = reinterpret_cast<uint16_t *>(base + bar_bytes + ext_bytes);
    W.bar_stride = bar_stride;
    W.gates = ngates;
    // nothing in the scratch has to start at zero: every word a live gate reads is written earlier in the same call,
    // and what the key switch computes from stale digits of gates past the end is discarded
    return enqueue_level_on(c, W, false, d_type, d_in0, d_in1, d_out, ngates);
} SHE_NOTHROW(c)

int she_eval_mux(she_ctx *c, const uint32_t *sel, const uint32_t *in1, const uint32_t *in0, const uint32_t *out,
                 size_t nmux)
try {
    if (!c) return SHE_EINVAL;
    SHE_NOT_WHILE_DEFERRED(c);
    if (nmux == 0) return SHE_OK;
    if (!sel || !in1 || !in0 || !out) return fail(c, SHE_EINVAL, "null argument");
    int rc;
    if ((rc = check_ids(c, sel, nmux, "she_eval_mux sel"))) return rc;
    if ((rc = check_ids(c, in1, nmux, "she_eval_mux in1"))) return rc;
    if ((rc = check_ids(c, in0, nmux, "she_eval_mux in0"))) return rc;
    if ((rc = check_ids(c, out, nmux, "she_eval_mux out"))) return rc;
    if ((rc = check_disjoint(c, sel, nmux, in1, nmux, out, nmux))) return rc;
    if ((rc = check_disjoint(c, in0, nmux, nullptr, 0, out, nmux))) return rc;
    try {
        std::vector<uint8_t> jt(2 * nmux);
        std::vector<uint32_t> j0(2 * nmux), j1(2 * nmux);
        for (size_t m = 0; m < nmux; m++) {
            jt[2 * m] = SHE_AND;       j0[2 * m] = sel[m];     j1[2 * m] = in1[m];        // sel and in1
            jt[2 * m + 1] = SHE_ANDNY; j0[2 * m + 1] = sel[m]; j1[2 * m + 1] = in0[m];    // (not sel) and in0
        }
        if ((rc = ensure_work(c, std::min<size_t>(2 * nmux, MAX_LEVEL_CHUNK)))) return rc;
        if ((rc = ensure_raw(c, std::min<size_t>(2 * nmux, MAX_LEVEL_CHUNK)))) return rc;
        if ((rc = ensure_mux_arrays(c, nmux))) return rc;
        HIP_TRY(c, hipMemcpyAsync(c->d_mtype, jt.data(), jt.size(), hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->d_min0, j0.data(), j0.size() * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->d_min1, j1.data(), j1.size() * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->d_mout, out, nmux * 4, hipMemcpyHostToDevice, c->stream));
        c->timer.clear();
        c->timer_levels = 1;
        if ((rc = enqueue_mux_level(c, c->d_mtype, c->d_min0, c->d_min1, c->d_mout, nmux))) return rc;
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        return finish_timing(c);
    } catch (const std::bad_alloc &) {
        return fail(c, SHE_ENOMEM, "host staging");
    }
} SHE_NOTHROW(c)

// ---- netlist construction shared by the operators and the planning calls ----
// bias: one plaintext constant per unit, or null.  With the adder trees a constant that is not 0 modulo 2^acc_bits is
// one more acc_bits-wide addition of trivial wires to the positive tree's sum, before the subtraction; with column
// compression it joins the negative terms' constants in plain arithmetic.
static std::vector<uint32_t> wires_shift_acc(Netlist &nl, const uint32_t *x_ids, uint32_t units, uint32_t terms,
                                             uint32_t in_bits, const int8_t *w_sign, const int8_t *w_exp,
                                             uint32_t acc_bits, const int32_t *bias = nullptr)
{
    std::vector<uint32_t> wires;
    wires.reserve((size_t)units * acc_bits);
    for (uint32_t u = 0; nl.columns && u < units; u++) {
        std::vector<SignedTerm> signed_terms(terms);
        for (uint32_t t = 0; t < terms; t++) {
            const size_t k = (size_t)u * terms + t;
            const uint32_t drop = (uint32_t)(-(int)w_exp[k]);            // x >> drop: the low wires fall away
            signed_terms[t].bits.assign(x_ids + k * in_bits + std::min(drop, in_bits), x_ids + (k + 1) * in_bits);
            signed_terms[t].sign = w_sign[k] > 0 ? 1 : -1;
        }
        const std::vector<uint32_t> total = nl_columns(nl, signed_terms, acc_bits, bias ? (int64_t)bias[u] : 0);
        wires.insert(wires.end(), total.begin(), total.end());
    }
    for (uint32_t u = 0; !nl.columns && u < units; u++) {
        std::vector<std::vector<uint32_t>> pos, neg;
        for (uint32_t t = 0; t < terms; t++) {
            const size_t k = (size_t)u * terms + t;
            const uint32_t drop = (uint32_t)(-(int)w_exp[k]);
            // x >> drop: the low `drop` wires fall away, trivial zeros refill the top
            std::vector<uint32_t> term(x_ids + k * in_bits + drop, x_ids + (k + 1) * in_bits);
            term.resize(in_bits, nl.zero());
            (w_sign[k] > 0 ? pos : neg).push_back(std::move(term));
        }
        const bool has_neg = !neg.empty();
        std::vector<uint32_t> total = nl_tree(nl, std::move(pos), in_bits, acc_bits);
        if (bias && ((uint64_t)(int64_t)bias[u] & (((uint64_t)1 << acc_bits) - 1)))
            total = nl_add(nl, total, nl_constant(nl, bias[u], acc_bits), acc_bits);
        if (has_neg) total = nl_sub(nl, total, nl_tree(nl, std::move(neg), in_bits, acc_bits));
        wires.insert(wires.end(), total.begin(), total.end());
    }
    return wires;
}

static std::vector<uint32_t> wires_relu(Netlist &nl, const uint32_t *x_ids, uint32_t count, uint32_t bits)
{
    std::vector<uint32_t> wires;
    wires.reserve((size_t)count * bits);
    for (uint32_t v = 0; v < count; v++) {
        const uint32_t *x = x_ids + (size_t)v * bits;
        for (uint32_t i = 0; i + 1 < bits; i++) wires.push_back(nl.gate(SHE_ANDNY, x[bits - 1], x[i]));
        wires.push_back(nl.zero());
    }
    return wires;
}

static std::vector<uint32_t> wires_maxpool(Netlist &nl, const uint32_t *x_ids, uint32_t H, uint32_t W, uint32_t C,
                                           uint32_t bits)
{
    std::vector<uint32_t> wires;
    wires.reserve((size_t)(H / 2) * (W / 2) * C * bits);
    auto pixel = [&](uint32_t h, uint32_t w, uint32_t ch) {
        const uint32_t *p = x_ids + (((size_t)h * W + w) * C + ch) * bits;
        return std::vector<uint32_t>(p, p + bits);
    };
    for (uint32_t h = 0; h < H / 2; h++)
        for (uint32_t w = 0; w < W / 2; w++)
            for (uint32_t ch = 0; ch < C; ch++) {
                const auto top = nl_max(nl, pixel(2 * h, 2 * w, ch), pixel(2 * h, 2 * w + 1, ch));
                const auto bot = nl_max(nl, pixel(2 * h + 1, 2 * w, ch), pixel(2 * h + 1, 2 * w + 1, ch));
                const auto best = nl_max(nl, top, bot);
                wires.insert(wires.end(), best.begin(), best.end());
            }
    return wires;
}

// ReLU of every pooled value: max(., 0) is monotone, so this equals pooling the ReLUs of the window
static std::vector<uint32_t> wires_relu_maxpool(Netlist &nl, const uint32_t *x_ids, uint32_t H, uint32_t W, uint32_t C,
                                                uint32_t bits)
{
    std::vector<uint32_t> wires = wires_maxpool(nl, x_ids, H, W, C, bits);
    for (size_t v = 0; v + bits <= wires.size(); v += bits) {
        const uint32_t sign = wires[v + bits - 1];
        for (uint32_t i = 0; i + 1 < bits; i++) wires[v + i] = nl.gate(SHE_ANDNY, sign, wires[v + i]);
        wires[v + bits - 1] = nl.zero();
    }
    return wires;
}

static bool weights_ok(const int8_t *w_sign, const int8_t *w_exp, size_t count, uint32_t in_bits, const char **why)
{
    for (size_t k = 0; k < count; k++) {
        if (w_sign[k] != 1 && w_sign[k] != -1) { *why = "w_sign must be +1 or -1"; return false; }
        if (w_exp[k] > 0 || -(int)w_exp[k] >= (int)in_bits) { *why = "w_exp must be in [-(in_bits-1), 0]"; return false; }
    }
    return true;
}

int she_shift_acc(she_ctx *c, const uint32_t *x_ids, uint32_t units, uint32_t terms, uint32_t in_bits,
                  const int8_t *w_sign, const int8_t *w_exp, uint32_t acc_bits, const uint32_t *out_ids,
                  uint64_t *gates_out)
{
    return she_shift_acc_bias(c, x_ids, units, terms, in_bits, w_sign, w_exp, nullptr, acc_bits, out_ids, gates_out);
}

int she_shift_acc_bias(she_ctx *c, const uint32_t *x_ids, uint32_t units, uint32_t terms, uint32_t in_bits,
                       const int8_t *w_sign, const int8_t *w_exp, const int32_t *bias, uint32_t acc_bits,
                       const uint32_t *out_ids, uint64_t *gates_out)
try {
    if (!c) return SHE_EINVAL;
    if (gates_out) *gates_out = 0;
    if (units == 0) return SHE_OK;
    if (!out_ids || (terms && (!x_ids || !w_sign || !w_exp))) return fail(c, SHE_EINVAL, "null argument");
    if (in_bits < 1 || in_bits > acc_bits || acc_bits > 32) return fail(c, SHE_EINVAL, "need 1 <= in_bits <= acc_bits <= 32");
    const size_t n_in = (size_t)units * terms * in_bits, n_out = (size_t)units * acc_bits;
    int rc;
    if ((rc = check_ids(c, x_ids, n_in, "she_shift_acc x_ids"))) return rc;
    if ((rc = check_ids(c, out_ids, n_out, "she_shift_acc out_ids"))) return rc;
    if ((rc = check_disjoint(c, x_ids, n_in, nullptr, 0, out_ids, n_out))) return rc;
    const char *why = "";
    if (!weights_ok(w_sign, w_exp, (size_t)units * terms, in_bits, &why)) return fail(c, SHE_EINVAL, why);
    if (c->columns && !(c->fold && c->cells3))
        return fail(c, SHE_EINVAL, "SHE_OPT_COLUMN_ADDER needs SHE_OPT_FOLD_CONSTANTS and SHE_OPT_GATE3_CELLS");
    try {
        return run_operator(c, x_ids, n_in, out_ids, n_out, gates_out, [&](Netlist &nl, const uint32_t *ids) {
            return wires_shift_acc(nl, ids, units, terms, in_bits, w_sign, w_exp, acc_bits, bias);
        });
    } catch (const std::bad_alloc &) {
        return fail(c, SHE_ENOMEM, "host allocation for the netlist");
    }
} SHE_NOTHROW(c)

int she_relu(she_ctx *c, const uint32_t *x_ids, uint32_t count, uint32_t bits, const uint32_t *out_ids,
             uint64_t *gates_out)
try {
    if (!c) return SHE_EINVAL;
    if (gates_out) *gates_out = 0;
    if (count == 0) return SHE_OK;
    if (!x_ids || !out_ids) return fail(c, SHE_EINVAL, "null argument");
    if (bits < 2 || bits > 64) return fail(c, SHE_EINVAL, "need 2 <= bits <= 64");
    const size_t total = (size_t)count * bits;
    int rc;
    if ((rc = check_ids(c, x_ids, total, "she_relu x_ids"))) return rc;
    if ((rc = check_ids(c, out_ids, total, "she_relu out_ids"))) return rc;
    if ((rc = check_disjoint(c, x_ids, total, nullptr, 0, out_ids, total))) return rc;
    try {
        return run_operator(c, x_ids, total, out_ids, total, gates_out,
                            [&](Netlist &nl, const uint32_t *ids) { return wires_relu(nl, ids, count, bits); });
    } catch (const std::bad_alloc &) {
        return fail(c, SHE_ENOMEM, "host allocation for the netlist");
    }
} SHE_NOTHROW(c)

int she_maxpool(she_ctx *c, const uint32_t *x_ids, uint32_t H, uint32_t W, uint32_t C, uint32_t bits,
                const uint32_t *out_ids, uint64_t *gates_out)
try {
    if (!c) return SHE_EINVAL;
    if (gates_out) *gates_out = 0;
    const uint32_t Ho = H / 2, Wo = W / 2;
    if (Ho == 0 || Wo == 0 || C == 0) return SHE_OK;
    if (!x_ids || !out_ids) return fail(c, SHE_EINVAL, "null argument");
    if (bits < 2 || bits > 64) return fail(c, SHE_EINVAL, "need 2 <= bits <= 64");
    const size_t n_in = (size_t)H * W * C * bits, n_out = (size_t)Ho * Wo * C * bits;
    int rc;
    if ((rc = check_ids(c, x_ids, n_in, "she_maxpool x_ids"))) return rc;
    if ((rc = check_ids(c, out_ids, n_out, "she_maxpool out_ids"))) return rc;
    if ((rc = check_disjoint(c, x_ids, n_in, nullptr, 0, out_ids, n_out))) return rc;
    try {
        return run_operator(c, x_ids, n_in, out_ids, n_out, gates_out,
                            [&](Netlist &nl, const uint32_t *ids) { return wires_maxpool(nl, ids, H, W, C, bits); });
    } catch (const std::bad_alloc &) {
        return fail(c, SHE_ENOMEM, "host allocation for the netlist");
    }
} SHE_NOTHROW(c)

int she_relu_maxpool(she_ctx *c, const uint32_t *x_ids, uint32_t H, uint32_t W, uint32_t C, uint32_t bits,
                     const uint32_t *out_ids, uint64_t *gates_out)
try {
    if (!c) return SHE_EINVAL;
    if (gates_out) *gates_out = 0;
    const uint32_t Ho = H / 2, Wo = W / 2;
    if (Ho == 0 || Wo == 0 || C == 0) return SHE_OK;
    if (!x_ids || !out_ids) return fail(c, SHE_EINVAL, "null argument");
    if (bits < 2 || bits > 64) return fail(c, SHE_EINVAL, "need 2 <= bits <= 64");
    const size_t n_in = (size_t)H * W * C * bits, n_out = (size_t)Ho * Wo * C * bits;
    int rc;
    if ((rc = check_ids(c, x_ids, n_in, "she_relu_maxpool x_ids"))) return rc;
    if ((rc = check_ids(c, out_ids, n_out, "she_relu_maxpool out_ids"))) return rc;
    if ((rc = check_disjoint(c, x_ids, n_in, nullptr, 0, out_ids, n_out))) return rc;
    try {
        return run_operator(c, x_ids, n_in, out_ids, n_out, gates_out,
                            [&](Netlist &nl, const uint32_t *ids) { return wires_relu_maxpool(nl, ids, H, W, C, bits); });
    } catch (const std::bad_alloc &) {
        return fail(c, SHE_ENOMEM, "host allocation for the netlist");
    }
} SHE_NOTHROW(c)

int she_set_option(she_ctx *c, int option, int value)
{
    if (!c) return SHE_EINVAL;
    SHE_NOT_WHILE_DEFERRED(c);
    if (option == SHE_OPT_FOLD_CONSTANTS) { c->fold = value != 0; return SHE_OK; }
    if (option == SHE_OPT_NATIVE_MUX) { c->native_mux = value != 0; return SHE_OK; }
    if (option == SHE_OPT_GATE3_CELLS) { c->cells3 = value != 0; return SHE_OK; }
    if (option == SHE_OPT_COLUMN_ADDER) { c->columns = value != 0; return SHE_OK; }
    if (option == SHE_OPT_SPLIT_BELOW) {
        if (value < 0) return fail(c, SHE_EINVAL, "SHE_OPT_SPLIT_BELOW takes a gate count >= 0");
        c->split_below = (size_t)value;
        return SHE_OK;
    }
    return fail(c, SHE_EINVAL, "unknown option");
}

int she_get_option(she_ctx *c, int option, int *value)
{
    if (!c) return SHE_EINVAL;
    if (!value) return fail(c, SHE_EINVAL, "null argument");
    if (option == SHE_OPT_FOLD_CONSTANTS) { *value = c->fold; return SHE_OK; }
    if (option == SHE_OPT_NATIVE_MUX) { *value = c->native_mux; return SHE_OK; }
    if (option == SHE_OPT_GATE3_CELLS) { *value = c->cells3; return SHE_OK; }
    if (option == SHE_OPT_COLUMN_ADDER) { *value = c->columns; return SHE_OK; }
    if (option == SHE_OPT_SPLIT_BELOW) { *value = (int)std::min<size_t>(c->split_below, 0x7FFFFFFF); return SHE_OK; }
    return fail(c, SHE_EINVAL, "unknown option");
}

static int plan_finish(Netlist &nl, uint64_t *gates, uint32_t *levels, uint64_t *rotations);

// ---- a caller's own circuit ----
// Appends the entries of a circuit given as reference arrays to `nl`; wires[g] receives the wire of entry g
// (under folding possibly a constant, an earlier wire or a complement).  Returns "" or what is wrong.
static std::string circuit_to_netlist(Netlist &nl, const uint8_t *type, const uint32_t *in0, const uint32_t *in1,
                                      const uint32_t *in2, size_t ngates, std::vector<uint32_t> &wires, bool *range_error)
{
    wires.assign(ngates, 0);
    *range_error = false;
    std::string why;
    auto wire_of = [&](uint32_t ref, size_t g, uint32_t &w) {
        const bool neg = (ref & SHE_WIRE_NOT) != 0;
        const uint32_t r = ref & ~SHE_WIRE_NOT;
        if (neg && !nl.fold) { why = "SHE_WIRE_NOT needs SHE_OPT_FOLD_CONSTANTS"; return false; }
        if (r == SHE_WIRE_ZERO) w = nl.zero();
        else if (r == SHE_WIRE_ONE) w = nl.one();
        else if (r & SHE_WIRE_GATE) {
            const uint32_t h = r & ~SHE_WIRE_GATE;
            if (h >= g) { why = "an entry refers to itself or to a later entry"; return false; }
            w = wires[h];
        } else {
            if (r >= nl.cap) { why = "id outside the pool"; *range_error = true; return false; }
            w = r;
        }
        if (neg) w ^= WIRE_NEG;
        return true;
    };
    for (size_t g = 0; g < ngates; g++) {
        const uint8_t t = type[g];
        uint32_t a = 0, b = 0, c = 0;
        if (!wire_of(in0[g], g, a) || !wire_of(in1[g], g, b)) return why;
        if (t < SHE_NUM_GATES) {
            wires[g] = nl.gate(t, a, b);
        } else if (t == SHE_CIRCUIT_MUX || (t >= SHE_MAJ3 && t < SHE_XOR3 + 8)) {
            if (!in2) return "three-input entries need in2";
            if (!wire_of(in2[g], g, c)) return why;
            if (t == SHE_CIRCUIT_MUX) {
                wires[g] = nl.mux(a, b, c);
            } else if (!nl.fold) {
                wires[g] = nl.gate3(t, a, b, c);                     // the code carries its complement mask as it is
            } else {
                const int base = t >= SHE_XOR3 ? SHE_XOR3 : SHE_MAJ3, mask = t - base;
                wires[g] = nl.gate3(base, a ^ ((mask & 1) ? WIRE_NEG : 0u), b ^ ((mask & 2) ? WIRE_NEG : 0u),
                                    c ^ ((mask & 4) ? WIRE_NEG : 0u));
            }
        } else {
            return "unknown gate code";
        }
        if (nl.overflow) return "circuit too large for 31-bit wire ids";
    }
    return "";
}

int she_eval_circuit(she_ctx *c, const uint8_t *type, const uint32_t *in0, const uint32_t *in1, const uint32_t *in2,
                     size_t ngates, const uint32_t *out_refs, const uint32_t *out_ids, size_t nout, uint64_t *entries_out)
try {
    if (!c) return SHE_EINVAL;
    SHE_NOT_WHILE_DEFERRED(c);
    if (entries_out) *entries_out = 0;
    if (nout == 0) return SHE_OK;                                      // nothing asked for: nothing to evaluate
    if ((ngates && (!type || !in0 || !in1)) || !out_refs || !out_ids) return fail(c, SHE_EINVAL, "null argument");
    if (ngates >= SHE_WIRE_GATE - 2) return fail(c, SHE_EINVAL, "too many entries for one call");
    int rc;
    if ((rc = check_ids(c, out_ids, nout, "she_eval_circuit out_ids"))) return rc;
    try {
        Netlist nl(c->cap, c->fold, c->native_mux, c->cells3, c->columns);
        std::vector<uint32_t> wires;
        bool range_error = false;
        const std::string why = circuit_to_netlist(nl, type, in0, in1, in2, ngates, wires, &range_error);
        if (!why.empty()) return fail(c, range_error ? SHE_ERANGE : SHE_EINVAL, "she_eval_circuit: " + why);
        // pool ids the circuit reads (operands and outputs that name an input directly)
        std::vector<uint32_t> reads;
        auto note = [&](uint32_t ref) {
            const uint32_t r = ref & ~SHE_WIRE_NOT;
            if (!(r & SHE_WIRE_GATE) && r != SHE_WIRE_ZERO && r != SHE_WIRE_ONE) reads.push_back(r);
        };
        for (size_t g = 0; g < ngates; g++) {
            note(in0[g]); note(in1[g]);
            if (type[g] >= SHE_NUM_GATES) note(in2[g]);
        }
        std::vector<uint32_t> out_wires(nout);
        for (size_t k = 0; k < nout; k++) {
            const bool neg = (out_refs[k] & SHE_WIRE_NOT) != 0;
            const uint32_t r = out_refs[k] & ~SHE_WIRE_NOT;
            uint32_t w;
            if (neg && !nl.fold) return fail(c, SHE_EINVAL, "she_eval_circuit: SHE_WIRE_NOT needs SHE_OPT_FOLD_CONSTANTS");
            if (r == SHE_WIRE_ZERO) w = nl.zero();
            else if (r == SHE_WIRE_ONE) w = nl.one();
            else if (r & SHE_WIRE_GATE) {
                if ((r & ~SHE_WIRE_GATE) >= ngates) return fail(c, SHE_EINVAL, "she_eval_circuit: output refers to a missing entry");
                w = wires[r & ~SHE_WIRE_GATE];
            } else {
                if (r >= c->cap) return fail(c, SHE_ERANGE, "she_eval_circuit: id outside the pool");
                w = r;
                reads.push_back(r);
            }
            out_wires[k] = neg ? (w ^ WIRE_NEG) : w;
        }
        if ((rc = check_disjoint(c, reads.data(), reads.size(), nullptr, 0, out_ids, nout))) return rc;
        return run_netlist(c, nl, out_wires, out_ids, entries_out);
    } catch (const std::bad_alloc &) {
        return fail(c, SHE_ENOMEM, "host allocation for the netlist");
    }
} SHE_NOTHROW(c)

int she_plan_circuit(uint32_t capacity, const uint8_t *type, const uint32_t *in0, const uint32_t *in1, const uint32_t *in2,
                     size_t ngates, int options, uint64_t *gates, uint32_t *levels, uint64_t *rotations)
try {
    if (ngates && (!type || !in0 || !in1)) return SHE_EINVAL;
    if (capacity == 0 || capacity > 0x3FFFFFF0u || ngates >= SHE_WIRE_GATE - 2) return SHE_EINVAL;
    try {
        Netlist nl(capacity, (options & SHE_OPT_FOLD_CONSTANTS) != 0, (options & SHE_OPT_NATIVE_MUX) != 0,
                   (options & SHE_OPT_GATE3_CELLS) != 0, (options & SHE_OPT_COLUMN_ADDER) != 0);
        std::vector<uint32_t> wires;
        bool range_error = false;
        const std::string why = circuit_to_netlist(nl, type, in0, in1, in2, ngates, wires, &range_error);
        if (!why.empty()) return range_error ? SHE_ERANGE : SHE_EINVAL;
        return plan_finish(nl, gates, levels, rotations);
    } catch (const std::bad_alloc &) {
        return SHE_ENOMEM;
    }
} SHE_NOTHROW(nullptr)

// ---- planning: the operators' netlists without a GPU (inputs are wires 0, 1, 2, ... in argument order) ----
static int plan_finish(Netlist &nl, uint64_t *gates, uint32_t *levels, uint64_t *rotations)
{
    if (nl.overflow) return SHE_ERANGE;
    if (gates) *gates = nl.type.size();
    if (rotations) *rotations = nl.rotations();
    if (levels) *levels = (uint32_t)(nl.levelize().size() - 1);
    return SHE_OK;
}

int she_plan_shift_acc(uint32_t units, uint32_t terms, uint32_t in_bits, const int8_t *w_sign, const int8_t *w_exp,
                       uint32_t acc_bits, int options, uint64_t *gates, uint32_t *levels, uint64_t *rotations)
{
    return she_plan_shift_acc_bias(units, terms, in_bits, w_sign, w_exp, nullptr, acc_bits, options, gates, levels, rotations);
}

// Smallest two's-complement width that holds bias + every sum of the unit, for each unit; the widest of them.
int she_plan_accumulator_bits(uint32_t units, uint32_t terms, uint32_t in_bits, const int8_t *w_sign, const int8_t *w_exp,
                              const int32_t *bias, uint32_t *bits_out)
try {
    if (!bits_out || in_bits < 1 || in_bits > 32 || (terms && units && (!w_sign || !w_exp))) return SHE_EINVAL;
    const char *why = "";
    if (!weights_ok(w_sign, w_exp, (size_t)units * terms, in_bits, &why)) return SHE_EINVAL;
    const int64_t top = ((int64_t)1 << in_bits) - 1;                 // largest input
    uint32_t bits = in_bits;
    for (uint32_t u = 0; u < units; u++) {
        // extreme sums: every positive-weight input at its maximum and the others at zero, and the other way round
        int64_t hi = bias ? bias[u] : 0, lo = hi;
        for (uint32_t t = 0; t < terms; t++) {
            const size_t k = (size_t)u * terms + t;
            const int64_t most = top >> -(int)w_exp[k];
            if (w_sign[k] > 0) hi += most; else lo -= most;
        }
        uint32_t b = 1;
        while (b < 63 && !(lo >= -((int64_t)1 << (b - 1)) && hi <= ((int64_t)1 << (b - 1)) - 1)) b++;
        bits = std::max(bits, b);
    }
    *bits_out = bits;
    return SHE_OK;
} SHE_NOTHROW(nullptr)

int she_plan_shift_acc_bias(uint32_t units, uint32_t terms, uint32_t in_bits, const int8_t *w_sign, const int8_t *w_exp,
                            const int32_t *bias, uint32_t acc_bits, int options, uint64_t *gates, uint32_t *levels,
                            uint64_t *rotations)
try {
    if (in_bits < 1 || in_bits > acc_bits || acc_bits > 32) return SHE_EINVAL;
    const size_t n_in = (size_t)units * terms * in_bits;
    if (n_in > 0x40000000u || (terms && units && (!w_sign || !w_exp))) return SHE_EINVAL;
    const char *why = "";
    if (!weights_ok(w_sign, w_exp, (size_t)units * terms, in_bits, &why)) return SHE_EINVAL;
    if ((options & SHE_OPT_COLUMN_ADDER) && !((options & SHE_OPT_FOLD_CONSTANTS) && (options & SHE_OPT_GATE3_CELLS))) return SHE_EINVAL;
    try {
        std::vector<uint32_t> ids(n_in);
        for (size_t k = 0; k < n_in; k++) ids[k] = (uint32_t)k;
        Netlist nl((uint32_t)std::max<size_t>(n_in, 1), (options & SHE_OPT_FOLD_CONSTANTS) != 0, (options & SHE_OPT_NATIVE_MUX) != 0,
                   (options & SHE_OPT_GATE3_CELLS) != 0, (options & SHE_OPT_COLUMN_ADDER) != 0);
        wires_shift_acc(nl, ids.data(), units, terms, in_bits, w_sign, w_exp, acc_bits, bias);
        return plan_finish(nl, gates, levels, rotations);
    } catch (const std::bad_alloc &) {
        return SHE_ENOMEM;
    }
} SHE_NOTHROW(nullptr)

int she_plan_relu(uint32_t count, uint32_t bits, int options, uint64_t *gates, uint32_t *levels, uint64_t *rotations)
try {
    if (bits < 2 || bits > 64 || (size_t)count * bits > 0x40000000u) return SHE_EINVAL;
    try {
        std::vector<uint32_t> ids((size_t)count * bits);
        for (size_t k = 0; k < ids.size(); k++) ids[k] = (uint32_t)k;
        Netlist nl((uint32_t)std::max<size_t>(ids.size(), 1), (options & SHE_OPT_FOLD_CONSTANTS) != 0, (options & SHE_OPT_NATIVE_MUX) != 0,
                   (options & SHE_OPT_GATE3_CELLS) != 0, (options & SHE_OPT_COLUMN_ADDER) != 0);
        wires_relu(nl, ids.data(), count, bits);
        return plan_finish(nl, gates, levels, rotations);
    } catch (const std::bad_alloc &) {
        return SHE_ENOMEM;
    }
} SHE_NOTHROW(nullptr)

int she_plan_relu_maxpool(uint32_t H, uint32_t W, uint32_t C, uint32_t bits, int options, uint64_t *gates, uint32_t *levels,
                          uint64_t *rotations)
try {
    const size_t n_in = (size_t)H * W * C * bits;
    if (bits < 2 || bits > 64 || n_in > 0x40000000u) return SHE_EINVAL;
    try {
        std::vector<uint32_t> ids(n_in);
        for (size_t k = 0; k < n_in; k++) ids[k] = (uint32_t)k;
        Netlist nl((uint32_t)std::max<size_t>(n_in, 1), (options & SHE_OPT_FOLD_CONSTANTS) != 0, (options & SHE_OPT_NATIVE_MUX) != 0,
                   (options & SHE_OPT_GATE3_CELLS) != 0, (options & SHE_OPT_COLUMN_ADDER) != 0);
        wires_relu_maxpool(nl, ids.data(), H, W, C, bits);
        return plan_finish(nl, gates, levels, rotations);
    } catch (const std::bad_alloc &) {
        return SHE_ENOMEM;
    }
} SHE_NOTHROW(nullptr)

int she_plan_maxpool(uint32_t H, uint32_t W, uint32_t C, uint32_t bits, int options, uint64_t *gates, uint32_t *levels,
                     uint64_t *rotations)
try {
    const size_t n_in = (size_t)H * W * C * bits;
    if (bits < 2 || bits > 64 || n_in > 0x40000000u) return SHE_EINVAL;
    try {
        std::vector<uint32_t> ids(n_in);
        for (size_t k = 0; k < n_in; k++) ids[k] = (uint32_t)k;
        Netlist nl((uint32_t)std::max<size_t>(n_in, 1), (options & SHE_OPT_FOLD_CONSTANTS) != 0, (options & SHE_OPT_NATIVE_MUX) != 0,
                   (options & SHE_OPT_GATE3_CELLS) != 0, (options & SHE_OPT_COLUMN_ADDER) != 0);
        wires_maxpool(nl, ids.data(), H, W, C, bits);
        return plan_finish(nl, gates, levels, rotations);
    } catch (const std::bad_alloc &) {
        return SHE_ENOMEM;
    }
} SHE_NOTHROW(nullptr)

int she_read_ct(she_ctx *c, uint32_t id, uint32_t *dst)
try {
    if (!c) return SHE_EINVAL;
    SHE_NOT_WHILE_DEFERRED(c);
    if (!dst) return fail(c, SHE_EINVAL, "null argument");
    if (id >= c->cap) return fail(c, SHE_ERANGE, "she_read_ct: id outside the pool");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    HIP_TRY(c, hipMemcpy(dst, c->pool + (size_t)id * c->stride, (c->P.n + 1) * 4, hipMemcpyDeviceToHost));
    return SHE_OK;
} SHE_NOTHROW(c)

int she_write_ct(she_ctx *c, uint32_t id, const uint32_t *src)
try {
    if (!c) return SHE_EINVAL;
    SHE_NOT_WHILE_DEFERRED(c);
    if (!src) return fail(c, SHE_EINVAL, "null argument");
    if (id >= c->cap) return fail(c, SHE_ERANGE, "she_write_ct: id outside the pool");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    HIP_TRY(c, hipMemcpy(c->pool + (size_t)id * c->stride, src, (c->P.n + 1) * 4, hipMemcpyHostToDevice));
    return SHE_OK;
} SHE_NOTHROW(c)

int she_export_keys(she_ctx *c, uint8_t *lwe_key, uint8_t *ring_key, uint32_t *bk, uint32_t *ks)
try {
    if (!c) return SHE_EINVAL;
    if (lwe_key) std::memcpy(lwe_key, c->hk.lwe_key.data(), c->hk.lwe_key.size());
    if (ring_key) std::memcpy(ring_key, c->hk.ring_key.data(), c->hk.ring_key.size());
    if (bk) std::memcpy(bk, c->hk.bk.data(), c->hk.bk.size() * 4);
    if (ks) std::memcpy(ks, c->hk.ks.data(), c->hk.ks.size() * 4);
    return SHE_OK;
} SHE_NOTHROW(c)

int she_set_stream(she_ctx *c, void *hip_stream)
{
    if (!c) return SHE_EINVAL;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->stream = (hipStream_t)hip_stream;
    return SHE_OK;
}

size_t she_pool_bytes(const she_ctx *c) { return c ? (size_t)c->cap * c->stride * sizeof(uint32_t) : 0; }

int she_bind_pool(she_ctx *c, void *dev_ptr, size_t bytes)
{
    if (!c) return SHE_EINVAL;
    SHE_NOT_WHILE_DEFERRED(c);
    if (!dev_ptr || bytes < she_pool_bytes(c) || ((uintptr_t)dev_ptr & 255)) return fail(c, SHE_EINVAL, "bad pool memory");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (c->pool_owned) hipFree(c->pool);
    c->pool = (uint32_t *)dev_ptr;
    c->pool_owned = false;
    return SHE_OK;
}

int she_set_round_tracking(she_ctx *c, int on)
{
    if (!c) return SHE_EINVAL;
    c->track_round = on != 0;
    return SHE_OK;
}

int she_get_round_error(she_ctx *c, double *max_abs_frac, int reset)
try {
    if (!c) return SHE_EINVAL;
    if (!max_abs_frac) return fail(c, SHE_EINVAL, "null argument");
    unsigned raw = 0;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    HIP_TRY(c, hipMemcpy(&raw, c->d_round_err, sizeof(raw), hipMemcpyDeviceToHost));
    float f;
    std::memcpy(&f, &raw, sizeof(f));
    *max_abs_frac = f;
    if (reset) HIP_TRY(c, hipMemset(c->d_round_err, 0, sizeof(unsigned)));
    return SHE_OK;
} SHE_NOTHROW(c)

int she_probe_fp64_rate(she_ctx *c, int form, double *ns_per_instruction, double *tflops_as_fma)
try {
    if (!c) return SHE_EINVAL;
    if (form < 0 || form > 3 || (!ns_per_instruction && !tflops_as_fma)) return fail(c, SHE_EINVAL, "form must be 0, 1, 2 or 3");
    // form 3 streams the spectral bootstrapping key in rows of 64 x 16 bytes
    const uint32_t src_rows = (uint32_t)std::min<size_t>(bk_hat_elems(c->P) / 64, 1u << 30);
    const uint32_t blocks = 2 * c->dk.cus;                    // 8 wavefronts per compute unit = 2 per SIMD
    const int iters = 30000;                                  // 64 instructions each: ~8 ms
    double *d_out = nullptr;
    HIP_TRY(c, hipMalloc((void **)&d_out, (size_t)blocks * 256 * sizeof(double)));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t rc = hipEventCreate(&e0);
    if (rc == hipSuccess) rc = hipEventCreate(&e1);
    if (rc == hipSuccess) rc = launch_fp64_probe(form, d_out, blocks, 200, c->dk.bk_hat, src_rows, c->stream);           // warm-up
    if (rc == hipSuccess) rc = hipEventRecord(e0, c->stream);
    if (rc == hipSuccess) rc = launch_fp64_probe(form, d_out, blocks, iters, c->dk.bk_hat, src_rows, c->stream);
    if (rc == hipSuccess) rc = hipEventRecord(e1, c->stream);
    if (rc == hipSuccess) rc = hipEventSynchronize(e1);
    float ms = 0.f;
    if (rc == hipSuccess) rc = hipEventElapsedTime(&ms, e0, e1);
    if (e0) hipEventDestroy(e0);
    if (e1) hipEventDestroy(e1);
    hipFree(d_out);
    if (rc != hipSuccess) return fail(c, SHE_EDEVICE, std::string("FP64 probe: ") + hipGetErrorString(rc));
    const double inst_per_simd = 2.0 * 64.0 * iters;          // 2 wavefronts per SIMD
    const double ns = (double)ms * 1e6 / inst_per_simd;
    if (ns_per_instruction) *ns_per_instruction = ns;
    if (tflops_as_fma) *tflops_as_fma = 128.0 * 4.0 * c->dk.cus / ns / 1e3;   // 64 lanes x 2 flop, 4 SIMDs per compute unit
    return SHE_OK;
} SHE_NOTHROW(c)

int she_probe_lds_rate(she_ctx *c, int form, double *bytes_per_ns_per_cu)
try {
    if (!c) return SHE_EINVAL;
    if (form < 0 || form > 4 || !bytes_per_ns_per_cu) return fail(c, SHE_EINVAL, "form must be 0..4");
    const uint32_t blocks = 2 * c->dk.cus;                    // 8 wavefronts per compute unit
    const int iters = 20000;                                  // 8 KiB per wavefront and iteration: a few ms
    uint32_t *d_out = nullptr;
    HIP_TRY(c, hipMalloc((void **)&d_out, (size_t)blocks * 256 * sizeof(uint32_t)));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t rc = hipEventCreate(&e0);
    if (rc == hipSuccess) rc = hipEventCreate(&e1);
    if (rc == hipSuccess) rc = launch_lds_probe(form, d_out, blocks, 200, c->stream);           // warm-up
    if (rc == hipSuccess) rc = hipEventRecord(e0, c->stream);
    if (rc == hipSuccess) rc = launch_lds_probe(form, d_out, blocks, iters, c->stream);
    if (rc == hipSuccess) rc = hipEventRecord(e1, c->stream);
    if (rc == hipSuccess) rc = hipEventSynchronize(e1);
    float ms = 0.f;
    if (rc == hipSuccess) rc = hipEventElapsedTime(&ms, e0, e1);
    if (e0) hipEventDestroy(e0);
    if (e1) hipEventDestroy(e1);
    hipFree(d_out);
    if (rc != hipSuccess) return fail(c, SHE_EDEVICE, std::string("LDS probe: ") + hipGetErrorString(rc));
    *bytes_per_ns_per_cu = 8.0 * 1024.0 * iters * 8.0 / ((double)ms * 1e6);   // 8 operations x 1 KiB x 8 wavefronts
    return SHE_OK;
} SHE_NOTHROW(c)

int she_set_timing(she_ctx *c, int on)
try {
    if (!c) return SHE_EINVAL;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->timer.clear();
    c->timer_levels = 0;
    c->timing = on != 0;
    return SHE_OK;
} SHE_NOTHROW(c)

int she_last_timing(she_ctx *c, double ms[4])
try {
    if (!c || !ms) return SHE_EINVAL;
    if (!c->timer.ev.empty()) {          // events of she_eval_gates_device calls still pending
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        int rc = finish_timing(c);
        if (rc) return rc;
    }
    for (int i = 0; i < 4; i++) ms[i] = c->last_ms[i];
    return SHE_OK;
} SHE_NOTHROW(c)

int she_last_level_sizes(const she_ctx *c, uint64_t *gates, uint64_t *muxes, size_t capacity, size_t *levels_out)
{
    if (!c || (capacity && (!gates || !muxes))) return SHE_EINVAL;
    const size_t levels = c->level_gates.size();
    if (levels_out) *levels_out = levels;
    for (size_t v = 0; v < levels && v < capacity; v++) { gates[v] = c->level_gates[v]; muxes[v] = c->level_muxes[v]; }
    return SHE_OK;
}

const char *she_last_error(const she_ctx *c) { return c ? c->err.c_str() : g_keygen_error.c_str(); }

}  // extern "C"
