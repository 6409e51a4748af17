// Netlists of SHE's layer operators and the level scheduler (host code).
// (SHE, arXiv 1906.00148: Section 3.1 builds ReLU and max-pooling units from 2-input gates,
// Section 3.2 turns multiplications by power-of-two weights into shifts that only re-wire
// encrypted bits, Section 3.3 sums the shifted terms with a mixed-bitwidth adder tree.)
#include <algorithm>

#include "she_internal.h"

namespace she {

namespace {

// truth table of a gate code: bit (2a + b) = gate(a, b)
constexpr uint8_t kTruth[SHE_NUM_GATES] = {
    /* NAND  */ 0x7, /* AND   */ 0x8, /* OR    */ 0xE, /* XOR   */ 0x6, /* XNOR  */ 0x9,
    /* NOR   */ 0x1, /* ANDNY */ 0x2, /* ANDYN */ 0x4, /* ORNY  */ 0xB, /* ORYN  */ 0xD};

int code_of_truth(uint8_t table)
{
    for (int c = 0; c < SHE_NUM_GATES; c++)
        if (kTruth[c] == table) return c;
    return -1;      // constant or single-operand function: never reached for two free operands
}

struct Operand {     // a wire reference taken apart
    bool is_const;
    uint32_t value;  // constant value, or the plain wire id
    uint32_t flip;   // 1 if the reference is complemented
};

}  // namespace

static uint32_t emit_entry(Netlist &nl, int c, uint32_t x, uint32_t y, uint32_t z)
{
    if (nl.next_temp >= WIRE_NEG - 1) { nl.overflow = true; return nl.zero(); }
    const uint32_t w = nl.next_temp++;
    nl.type.push_back((uint8_t)c);
    nl.in0.push_back(x);
    nl.in1.push_back(y);
    nl.in2.push_back(z);
    nl.out.push_back(w);
    return w;
}

uint64_t Netlist::rotations() const
{
    uint64_t r = 0;
    for (uint8_t t : type) r += is_mux_type(t) ? 2 : 1;
    return r;
}

uint32_t Netlist::gate(int code, uint32_t a, uint32_t b)
{
    auto emit = [&](int c, uint32_t x, uint32_t y) { return emit_entry(*this, c, x, y, 0); };
    if (!fold) return emit(code, a, b);

    auto take = [&](uint32_t ref) {
        const uint32_t w = ref & ~WIRE_NEG, f = ref >> 31;
        if (w == zero()) return Operand{true, f, 0};
        if (w == one()) return Operand{true, 1u - f, 0};
        return Operand{false, w, f};
    };
    const Operand A = take(a), B = take(b);
    const uint8_t tt = kTruth[code];
    // the gate as a function of the plain wires' values x (under a) and y (under b)
    auto eval = [&](uint32_t x, uint32_t y) -> uint32_t {
        const uint32_t va = A.is_const ? A.value : x ^ A.flip;
        const uint32_t vb = B.is_const ? B.value : y ^ B.flip;
        return (tt >> (2 * va + vb)) & 1u;
    };
    if (A.is_const || B.is_const || A.value == B.value) {
        // zero or one free variable: constant, that wire, or its complement
        const bool none = A.is_const && B.is_const;
        const uint32_t at0 = eval(0, 0), at1 = none ? at0 : eval(1, 1);
        if (at0 == at1) return at0 ? one() : zero();
        const uint32_t wire = A.is_const ? B.value : A.value;
        return at0 == 0 ? wire : (wire | WIRE_NEG);
    }
    uint8_t table = 0;
    for (uint32_t x = 0; x < 2; x++)
        for (uint32_t y = 0; y < 2; y++) table |= (uint8_t)(eval(x, y) << (2 * x + y));
    return emit(code_of_truth(table), A.value, B.value);
}

// s ? u : v.  Three 2-input gates, or (native_mux) one entry whose two blind rotations bootstrap
// code1(s, u) and code0(s, v): AND and ANDNY for plain operands, ANDYN / NOR when u / v is complemented.
uint32_t Netlist::mux(uint32_t s, uint32_t u, uint32_t v)
{
    if (!native_mux) {
        const uint32_t taken = gate(SHE_AND, s, u);
        const uint32_t other = gate(SHE_ANDNY, s, v);
        return gate(SHE_OR, taken, other);
    }
    if (!fold) return emit_entry(*this, MUX_BASE + 16 * SHE_AND + SHE_ANDNY, s, u, v);

    auto is_const = [&](uint32_t ref) { const uint32_t w = ref & ~WIRE_NEG; return w == zero() || w == one(); };
    auto const_value = [&](uint32_t ref) { return ((ref & ~WIRE_NEG) == one() ? 1u : 0u) ^ (ref >> 31); };
    if (is_const(s)) return const_value(s) ? u : v;
    if (s & WIRE_NEG) { std::swap(u, v); s &= ~WIRE_NEG; }            // not s ? u : v  ==  s ? v : u
    // a branch that repeats the selector is a constant on that branch
    if (!is_const(u) && (u & ~WIRE_NEG) == s) u = (u & WIRE_NEG) ? zero() : one();
    if (!is_const(v) && (v & ~WIRE_NEG) == s) v = (v & WIRE_NEG) ? one() : zero();
    const bool cu = is_const(u), cv = is_const(v);
    if (cu && cv) {
        const uint32_t a = const_value(u), b = const_value(v);
        if (a == b) return a ? one() : zero();
        return a ? s : (s | WIRE_NEG);
    }
    if (cu) return gate(const_value(u) ? SHE_OR : SHE_ANDNY, s, v);     // s ? 1 : v = s or v;   s ? 0 : v = not s and v
    if (cv) return gate(const_value(v) ? SHE_ORNY : SHE_AND, s, u);     // s ? u : 1 = not s or u; s ? u : 0 = s and u
    if ((u & ~WIRE_NEG) == (v & ~WIRE_NEG)) {
        if (u == v) return u;
        return gate((u & WIRE_NEG) ? SHE_XOR : SHE_XNOR, s, u & ~WIRE_NEG);   // s ? u : not u
    }
    const int code1 = (u & WIRE_NEG) ? SHE_ANDYN : SHE_AND;             // s and (not) u
    const int code0 = (v & WIRE_NEG) ? SHE_NOR : SHE_ANDNY;             // (not s) and (not) v
    return emit_entry(*this, MUX_BASE + 16 * code1 + code0, s, u & ~WIRE_NEG, v & ~WIRE_NEG);
}

// Majority or parity of three wire references with ONE bootstrap (the pre-bootstrap sample is +-a +- b +- c, or
// -2 times it for the parity).  With folding, the cell is first written as a truth table over the distinct plain
// wires under its operands: no wire left -> a constant; one -> that wire or its complement; two -> a 2-input gate
// (or a single wire when the pair cancels, e.g. majority(a, not a, c) = c); three -> a three-input entry whose
// complement mask carries the operands' flips (for the parity only their number matters: mask 0 or 1).
uint32_t Netlist::gate3(int base, uint32_t a, uint32_t b, uint32_t c)
{
    if (!fold) return emit_entry(*this, base, a, b, c);
    const uint32_t refs[3] = {a, b, c};
    uint32_t wires[3] = {0, 0, 0};
    int var_of[3], flips[3], consts[3], n_vars = 0;
    for (int k = 0; k < 3; k++) {
        const uint32_t w = refs[k] & ~WIRE_NEG, f = refs[k] >> 31;
        flips[k] = (int)f;
        consts[k] = -1;
        var_of[k] = -1;
        if (w == zero()) { consts[k] = (int)f; continue; }
        if (w == one()) { consts[k] = 1 - (int)f; continue; }
        for (int v = 0; v < n_vars; v++)
            if (wires[v] == w) var_of[k] = v;
        if (var_of[k] < 0) { wires[n_vars] = w; var_of[k] = n_vars++; }
    }
    // bit `assign` of tt = value of the cell when variable v takes bit v of `assign`
    uint32_t tt = 0;
    for (uint32_t assign = 0; assign < (1u << n_vars); assign++) {
        int ones = 0;
        for (int k = 0; k < 3; k++) ones += consts[k] >= 0 ? consts[k] : (int)((assign >> var_of[k]) & 1u) ^ flips[k];
        const uint32_t val = base == SHE_MAJ3 ? (ones >= 2) : (ones & 1);
        tt |= val << assign;
    }
    auto wire_or_not = [&](uint32_t w, uint32_t at0, uint32_t at1) {
        if (at0 == at1) return at0 ? one() : zero();
        return at0 ? (w | WIRE_NEG) : w;
    };
    if (n_vars == 0) return (tt & 1u) ? one() : zero();
    if (n_vars == 1) return wire_or_not(wires[0], tt & 1u, (tt >> 1) & 1u);
    if (n_vars == 2) {
        const bool needs0 = ((tt ^ (tt >> 1)) & 0x5u) != 0, needs1 = ((tt ^ (tt >> 2)) & 0x3u) != 0;
        if (!needs1) return wire_or_not(wires[0], tt & 1u, (tt >> 1) & 1u);
        if (!needs0) return wire_or_not(wires[1], tt & 1u, (tt >> 2) & 1u);
        // kTruth counts its first operand as the high bit of the index
        uint8_t table = 0;
        for (uint32_t x = 0; x < 2; x++)
            for (uint32_t y = 0; y < 2; y++) table |= (uint8_t)(((tt >> (x + 2 * y)) & 1u) << (2 * x + y));
        return emit_entry(*this, code_of_truth(table), wires[0], wires[1], 0);
    }
    int mask = flips[0] | (flips[1] << 1) | (flips[2] << 2);
    if (base == SHE_XOR3) mask = (flips[0] + flips[1] + flips[2]) & 1;
    return emit_entry(*this, base + mask, wires[0], wires[1], wires[2]);
}

void Netlist::bind_outputs(const std::vector<uint32_t> &wires, const uint32_t *dst)
{
    const uint32_t first_temp = cap + 2, unbound = 0xFFFFFFFFu;
    std::vector<uint32_t> rename(next_temp - first_temp, unbound);     // temporary wire -> caller id
    for (size_t k = 0; k < wires.size(); k++) {
        const uint32_t w = wires[k];
        if (!(w & WIRE_NEG) && w >= first_temp && rename[w - first_temp] == unbound) {
            rename[w - first_temp] = dst[k];
        } else {                     // input, constant, complemented wire, or a wire already bound
            copy_src.push_back(w);
            copy_dst.push_back(dst[k]);
        }
    }
    auto fix = [&](uint32_t &ref) {
        const uint32_t w = ref & ~WIRE_NEG;
        if (w >= first_temp && rename[w - first_temp] != unbound) ref = rename[w - first_temp] | (ref & WIRE_NEG);
    };
    for (size_t g = 0; g < type.size(); g++) {
        fix(in0[g]); fix(in1[g]); fix(out[g]);
        if (has_third_operand(type[g])) fix(in2[g]);
    }
    for (auto &w : copy_src) fix(w);
}

// Must run before bind_outputs (every gate output is still a temporary wire).
std::vector<size_t> Netlist::levelize(std::vector<size_t> *mux_start)
{
    // depth of a wire = 0 for inputs and constants, else 1 + deepest operand; entries were
    // appended in topological order, so one pass suffices
    const uint32_t first_temp = cap + 2;
    std::vector<uint32_t> depth(next_temp - first_temp, 0);
    std::vector<uint32_t> lev(type.size());
    uint32_t deepest = 0;
    auto depth_of = [&](uint32_t w) { return w >= first_temp ? depth[w - first_temp] : 0u; };
    for (size_t g = 0; g < type.size(); g++) {
        uint32_t d = std::max(depth_of(in0[g]), depth_of(in1[g]));
        if (has_third_operand(type[g])) d = std::max(d, depth_of(in2[g]));
        lev[g] = d + 1;
        depth[out[g] - first_temp] = d + 1;
        deepest = std::max(deepest, d + 1);
    }
    // bucket = 2*level + (1 for a MUX entry): gates of a level come before its MUX entries
    std::vector<size_t> start(2 * (size_t)deepest + 3, 0);
    auto bucket = [&](size_t g) { return 2 * (size_t)lev[g] + (is_mux_type(type[g]) ? 1 : 0); };
    for (size_t g = 0; g < type.size(); g++) start[bucket(g) + 1]++;
    for (size_t i = 1; i < start.size(); i++) start[i] += start[i - 1];
    std::vector<size_t> cursor(start.begin(), start.end() - 1);
    std::vector<uint8_t> t2(type.size());
    std::vector<uint32_t> a2(type.size()), b2(type.size()), c2(type.size()), o2(type.size());
    for (size_t g = 0; g < type.size(); g++) {
        const size_t pos = cursor[bucket(g)]++;
        t2[pos] = type[g]; a2[pos] = in0[g]; b2[pos] = in1[g]; c2[pos] = in2[g]; o2[pos] = out[g];
    }
    type.swap(t2); in0.swap(a2); in1.swap(b2); in2.swap(c2); out.swap(o2);
    // level lv (1-based) occupies [start[2 lv], start[2 lv + 2]), its MUX entries start at start[2 lv + 1]
    std::vector<size_t> bounds;
    if (mux_start) mux_start->clear();
    for (uint32_t lv = 1; lv <= deepest; lv++) {
        bounds.push_back(start[2 * lv]);
        if (mux_start) mux_start->push_back(start[2 * lv + 1]);
    }
    bounds.push_back(type.size());
    return bounds;
}

// Gives every wire that is still a temporary (after levelize and bind_outputs) a slot of the internal buffer that
// is free while the wire is live: a slot is handed out when the wire's entry runs and taken back once the level of the
// wire's last reader has run (entries of one level run side by side, so a slot freed by level v serves level v + 1 at
// the earliest; a wire that a final copy reads is never freed).  The walk checks itself: every operand must still own
// its slot when it is read.  Returns the number of slots used (the two constants included), 0 if the check failed.
size_t Netlist::compact_temporaries(const std::vector<size_t> &bounds)
{
    const uint32_t first_temp = cap + 2, none = 0xFFFFFFFFu;
    const size_t wires = next_temp - first_temp, levels = bounds.size() - 1;
    auto temp_index = [&](uint32_t ref, size_t &idx) {
        const uint32_t w = ref & ~WIRE_NEG;
        if (w < first_temp) return false;
        idx = w - first_temp;
        return true;
    };
    // last level that reads each wire (levels are 1-based; 0 = never read; levels + 1 = read by a final copy)
    std::vector<uint32_t> last(wires, 0);
    size_t idx = 0;
    for (size_t lv = 0; lv < levels; lv++)
        for (size_t g = bounds[lv]; g < bounds[lv + 1]; g++) {
            if (temp_index(in0[g], idx)) last[idx] = (uint32_t)lv + 1;
            if (temp_index(in1[g], idx)) last[idx] = (uint32_t)lv + 1;
            if (has_third_operand(type[g]) && temp_index(in2[g], idx)) last[idx] = (uint32_t)lv + 1;
        }
    for (uint32_t w : copy_src)
        if (temp_index(w, idx)) last[idx] = (uint32_t)levels + 1;
    std::vector<uint32_t> slot(wires, none), owner, free_slots;
    std::vector<std::vector<uint32_t>> expiring(levels + 2);      // wires whose last reader is in that level
    bool ok = true;
    auto rename = [&](uint32_t &ref) {
        size_t i = 0;
        if (!temp_index(ref, i)) return;
        if (slot[i] == none || owner[slot[i]] != i) { ok = false; return; }
        ref = (first_temp + slot[i]) | (ref & WIRE_NEG);
    };
    for (size_t lv = 0; lv < levels; lv++) {
        // what the level before the previous one read last is free now; so is what nobody reads at all
        if (lv >= 1)
            for (uint32_t i : expiring[lv]) free_slots.push_back(slot[i]);
        for (size_t g = bounds[lv]; g < bounds[lv + 1]; g++) {
            rename(in0[g]); rename(in1[g]);
            if (has_third_operand(type[g])) rename(in2[g]);
        }
        for (size_t g = bounds[lv]; g < bounds[lv + 1]; g++) {
            size_t i = 0;
            if (!temp_index(out[g], i)) continue;                  // bound to a caller's pool slot
            uint32_t s;
            if (free_slots.empty()) { s = (uint32_t)owner.size(); owner.push_back(none); }
            else { s = free_slots.back(); free_slots.pop_back(); }
            slot[i] = s;
            owner[s] = (uint32_t)i;
            out[g] = first_temp + s;
            // a wire read last in level v frees its slot for level v + 1; an unread wire lives for its own level only
            const uint32_t until = std::max<uint32_t>(last[i], (uint32_t)lv + 1);
            if (until <= levels) expiring[until].push_back((uint32_t)i);
        }
    }
    for (uint32_t &w : copy_src) rename(w);
    if (!ok) return 0;
    next_temp = first_temp + (uint32_t)owner.size();
    return owner.size() + 2;
}

// a + b for equally wide unsigned vectors; one more bit than the operands unless that
// would exceed cap_bits (then the last carry is not formed and the sum wraps).
std::vector<uint32_t> nl_add(Netlist &nl, const std::vector<uint32_t> &a, const std::vector<uint32_t> &b, uint32_t cap_bits)
{
    const size_t w = a.size();
    std::vector<uint32_t> sum;
    sum.push_back(nl.gate(SHE_XOR, a[0], b[0]));
    if (w == 1 && cap_bits == 1) return sum;
    uint32_t carry = nl.gate(SHE_AND, a[0], b[0]);
    if (nl.cells3) {
        // full-adder cell: sum = parity(a_i, b_i, carry), next carry = majority of the same three
        for (size_t i = 1; i < w; i++) {
            sum.push_back(nl.gate3(SHE_XOR3, a[i], b[i], carry));
            if (i + 1 == w && w >= cap_bits) return sum;
            carry = nl.gate3(SHE_MAJ3, a[i], b[i], carry);
        }
        sum.push_back(carry);
        return sum;
    }
    for (size_t i = 1; i < w; i++) {
        const uint32_t half = nl.gate(SHE_XOR, a[i], b[i]);
        sum.push_back(nl.gate(SHE_XOR, half, carry));
        if (i + 1 == w && w >= cap_bits) return sum;
        const uint32_t gen = nl.gate(SHE_AND, a[i], b[i]);
        const uint32_t prop = nl.gate(SHE_AND, half, carry);
        carry = nl.gate(SHE_OR, gen, prop);
    }
    sum.push_back(carry);
    return sum;
}

// p - q modulo 2^w = p + not(q) + 1; the complement sits in the gate types, the chain starts at trivial 1
std::vector<uint32_t> nl_sub(Netlist &nl, const std::vector<uint32_t> &p, const std::vector<uint32_t> &q)
{
    const size_t w = p.size();
    std::vector<uint32_t> diff;
    uint32_t carry = nl.one();
    if (nl.cells3) {
        // the same cell on (p_i, not q_i, carry); without folding the complement sits in the entry's mask
        for (size_t i = 0; i < w; i++) {
            diff.push_back(nl.fold ? nl.gate3(SHE_XOR3, p[i], q[i] ^ WIRE_NEG, carry)
                                   : emit_entry(nl, SHE_XOR3 + 1, p[i], q[i], carry));
            if (i + 1 == w) break;
            carry = nl.fold ? nl.gate3(SHE_MAJ3, p[i], q[i] ^ WIRE_NEG, carry) : emit_entry(nl, SHE_MAJ3 + 2, p[i], q[i], carry);
        }
        return diff;
    }
    for (size_t i = 0; i < w; i++) {
        const uint32_t half = nl.gate(SHE_XNOR, p[i], q[i]);
        diff.push_back(nl.gate(SHE_XOR, half, carry));
        if (i + 1 == w) break;
        const uint32_t gen = nl.gate(SHE_ANDYN, p[i], q[i]);
        const uint32_t prop = nl.gate(SHE_AND, half, carry);
        carry = nl.gate(SHE_OR, gen, prop);
    }
    return diff;
}

// Mixed-bitwidth accumulator: tree level j adds neighbours with min(in_bits+j, acc_bits)-bit adders,
// an unpaired last vector moves up zero-extended; the result is zero-extended to acc_bits.
// Section 3.3 wants an accumulator whose adders are only as wide as the bits that reach them.  Here every bit sits in
// the column of its weight.  A negative term contributes the complements of its w wires and the constant 1 - 2^w
// (-t = not(t) - 2^w + 1 on w bits); the constants are summed in plain arithmetic and enter as trivial-one wires.
// A stage turns each run of three wires of a column, from the front, into a parity wire in that column and a
// majority wire in the next one (none beyond the top column); what is left of the column follows unchanged.  In the
// new column the carries from below come first, then the parities, then the leftovers; a wire that folding proves
// zero is dropped.  Once no column holds more than two wires a ripple adder of cells finishes the sum.
// `bias` is the unit's plaintext constant: it joins the constants of the negative terms.
std::vector<uint32_t> nl_columns(Netlist &nl, const std::vector<SignedTerm> &terms, uint32_t acc_bits, int64_t bias)
{
    std::vector<std::vector<uint32_t>> cols(acc_bits);
    uint64_t constant = (uint64_t)bias;                      // mod 2^acc_bits at the end (acc_bits <= 32)
    for (const SignedTerm &term : terms) {
        for (size_t b = 0; b < term.bits.size() && b < acc_bits; b++)
            cols[b].push_back(term.sign > 0 ? term.bits[b] : term.bits[b] ^ WIRE_NEG);
        if (term.sign < 0) constant += 1 - ((uint64_t)1 << term.bits.size());      // wraps mod 2^64: fine
    }
    for (uint32_t j = 0; j < acc_bits; j++)
        if ((constant >> j) & 1u) cols[j].push_back(nl.one());
    auto widest = [&]() { size_t w = 0; for (const auto &c : cols) w = std::max(w, c.size()); return w; };
    while (widest() > 2) {
        std::vector<std::vector<uint32_t>> next(acc_bits);
        for (uint32_t j = 0; j < acc_bits; j++) {
            const std::vector<uint32_t> &bits = cols[j];
            size_t k = 0;
            for (; bits.size() - k >= 3; k += 3) {
                const uint32_t s = nl.gate3(SHE_XOR3, bits[k], bits[k + 1], bits[k + 2]);
                if (s != nl.zero()) next[j].push_back(s);
                if (j + 1 < acc_bits) {
                    const uint32_t m = nl.gate3(SHE_MAJ3, bits[k], bits[k + 1], bits[k + 2]);
                    if (m != nl.zero()) next[j + 1].push_back(m);
                }
            }
            next[j].insert(next[j].end(), bits.begin() + k, bits.end());
        }
        cols.swap(next);
    }
    std::vector<uint32_t> out;
    out.reserve(acc_bits);
    bool have_carry = false;
    uint32_t carry = 0;
    for (uint32_t j = 0; j < acc_bits; j++) {
        std::vector<uint32_t> ops = cols[j];
        if (have_carry) ops.push_back(carry);
        const bool last = j + 1 == acc_bits;
        have_carry = false;
        if (ops.empty()) {
            out.push_back(nl.zero());
        } else if (ops.size() == 1) {
            out.push_back(ops[0]);
        } else if (ops.size() == 2) {
            out.push_back(nl.gate(SHE_XOR, ops[0], ops[1]));
            if (!last) { carry = nl.gate(SHE_AND, ops[0], ops[1]); have_carry = true; }
        } else {
            out.push_back(nl.gate3(SHE_XOR3, ops[0], ops[1], ops[2]));
            if (!last) { carry = nl.gate3(SHE_MAJ3, ops[0], ops[1], ops[2]); have_carry = true; }
        }
        if (have_carry && carry == nl.zero()) have_carry = false;
    }
    return out;
}

// two's complement of a plaintext integer as trivial wires, least significant bit first: no gate
std::vector<uint32_t> nl_constant(Netlist &nl, int64_t value, uint32_t bits)
{
    std::vector<uint32_t> wires(bits);
    for (uint32_t i = 0; i < bits; i++) wires[i] = (((uint64_t)value >> i) & 1u) ? nl.one() : nl.zero();
    return wires;
}

std::vector<uint32_t> nl_tree(Netlist &nl, std::vector<std::vector<uint32_t>> terms, uint32_t in_bits, uint32_t acc_bits)
{
    uint32_t width = in_bits;
    while (terms.size() > 1) {
        const uint32_t next_width = std::min(width + 1, acc_bits);
        std::vector<std::vector<uint32_t>> next;
        for (size_t m = 0; m + 1 < terms.size(); m += 2) next.push_back(nl_add(nl, terms[m], terms[m + 1], acc_bits));
        if (terms.size() & 1) {
            std::vector<uint32_t> last = terms.back();
            last.resize(next_width, nl.zero());
            next.push_back(std::move(last));
        }
        terms.swap(next);
        width = next_width;
    }
    std::vector<uint32_t> total = terms.empty() ? std::vector<uint32_t>() : terms[0];
    total.resize(acc_bits, nl.zero());
    return total;
}

// max of two two's-complement vectors: equality bits, a ripple "x > y so far" from the least
// significant bit up, the sign position decided the other way round, then one MUX per bit
std::vector<uint32_t> nl_max(Netlist &nl, const std::vector<uint32_t> &x, const std::vector<uint32_t> &y)
{
    const size_t w = x.size();
    if (nl.cells3) {
        // "x > y so far" from one majority gate per bit: majority(x_i, not y_i, gt) is 1 where x has the 1, 0 where y
        // has it, and gt where the bits agree; at the sign position the operands swap roles
        uint32_t above = nl.zero();
        for (size_t i = 0; i < w; i++) {
            const uint32_t hi = i + 1 < w ? x[i] : y[i], lo = i + 1 < w ? y[i] : x[i];
            above = nl.fold ? nl.gate3(SHE_MAJ3, hi, lo ^ WIRE_NEG, above) : emit_entry(nl, SHE_MAJ3 + 2, hi, lo, above);
        }
        std::vector<uint32_t> best(w);
        for (size_t i = 0; i < w; i++) best[i] = nl.mux(above, x[i], y[i]);
        return best;
    }
    std::vector<uint32_t> eq(w);
    for (size_t i = 0; i < w; i++) eq[i] = nl.gate(SHE_XNOR, x[i], y[i]);
    uint32_t gt = nl.zero();
    for (size_t i = 0; i + 1 < w; i++) gt = nl.mux(eq[i], gt, x[i]);
    gt = nl.mux(eq[w - 1], gt, y[w - 1]);
    std::vector<uint32_t> z(w);
    for (size_t i = 0; i < w; i++) z[i] = nl.mux(gt, x[i], y[i]);
    return z;
}

}  // namespace she
