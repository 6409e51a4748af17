// The context behind the C ABI and the helpers its source files share (internal).
#pragma once
#include <memory>
#include <string>
#include <vector>

#include "she_internal.h"

namespace she {
struct LevelTimer {           // events around the three kernel families of every chunk
    std::vector<hipEvent_t> ev;
    ~LevelTimer() { clear(); }
    void clear() { for (auto e : ev) hipEventDestroy(e); ev.clear(); }
    hipError_t mark(hipStream_t st)
    {
        hipEvent_t e;
        hipError_t rc = hipEventCreate(&e);
        if (rc != hipSuccess) return rc;
        ev.push_back(e);
        return hipEventRecord(e, st);
    }
};

struct LeveledPools {         // leveled mode: TRGSW selectors (spectral form) and TRLWE samples
    double2 *trgsw_hat = nullptr;   // [trgsw_cap][2l][2][P][L]
    uint32_t *trlwe = nullptr;      // [trlwe_cap][2][N]
    uint32_t trgsw_cap = 0, trlwe_cap = 0;
    uint32_t *d_ids = nullptr;      // device staging of the id arrays of one call (4 x ids_cap)
    size_t ids_cap = 0;
};
// Layer operators recorded between she_defer_begin and she_defer_run: one netlist for all of them, so that the
// scheduler can overlap the tail of one operator with the head of the next.
struct Deferred {
    static constexpr uint32_t NONE = 0xFFFFFFFFu;
    std::unique_ptr<Netlist> nl;
    std::vector<uint32_t> produced;     // [cap] wire reference of a pool id that a recorded operator writes, else NONE
    std::vector<uint8_t> read;          // [cap] 1: a recorded operator reads the slot as it was before the circuit
    std::vector<uint32_t> out_wires, out_ids;
};
}  // namespace she

struct she_ctx {
    she_params P{};
    int device = 0;
    hipStream_t stream = nullptr;
    she::HostKeys hk;
    she::DeviceKeys dk;
    uint32_t cap = 0, stride = 0;
    uint32_t *pool = nullptr;
    bool pool_owned = true;
    uint32_t *temp = nullptr;            // internal slots: 0 = trivial 0, 1 = trivial 1, then temporaries
    size_t temp_slots = 0;
    she::LevelWork work;
    // device staging for host-array calls (grown on demand)
    uint8_t *d_type = nullptr;
    uint32_t *d_in0 = nullptr, *d_in1 = nullptr, *d_in2 = nullptr, *d_out = nullptr;
    size_t d_gate_cap = 0;
    uint32_t *d_stage = nullptr;         // ciphertext staging [slots][n+1] and id lists
    size_t d_stage_words = 0;
    unsigned *d_round_err = nullptr;
    bool track_round = false;
    bool fold = false;                   // SHE_OPT_FOLD_CONSTANTS
    bool native_mux = false;             // SHE_OPT_NATIVE_MUX
    bool cells3 = false;                 // SHE_OPT_GATE3_CELLS
    bool columns = false;                // SHE_OPT_COLUMN_ADDER
    size_t split_below = 0;              // SHE_OPT_SPLIT_BELOW (set at creation: 6 x compute units)
    uint8_t *d_mtype = nullptr;          // device staging of MUX rotations: 2 jobs per MUX entry
    uint32_t *d_min0 = nullptr, *d_min1 = nullptr, *d_mout = nullptr;
    size_t d_mux_cap = 0;
    bool timing = true;                  // record HIP events around every kernel
    she::LevelTimer timer;               // events not yet folded into last_ms
    size_t timer_levels = 0;
    std::vector<uint64_t> level_gates, level_muxes;   // schedule of the last circuit (she_last_level_sizes)
    double last_ms[4] = {0, 0, 0, 0};
    she::LeveledPools lev;
    std::unique_ptr<she::Deferred> deferred;   // non-null between she_defer_begin and she_defer_run
    void *na_scratch = nullptr;          // this device's copy of the static scratch buffer (never freed)
    size_t na_bytes = 0;
    std::string err;
};

namespace she {
extern thread_local std::string g_keygen_error;        // message of a failed she_keygen (no context yet)
int fail(she_ctx *c, int code, const std::string &msg); // records the message, returns the code; never throws
int fail_exception(she_ctx *c);                         // inside a catch block: maps the exception in flight to a code
// Nothing may be thrown across the C boundary: every extern "C" function that can allocate on the host or start a
// thread is a function-try-block that ends with this handler.
#define SHE_NOTHROW(ctx) catch (...) { return she::fail_exception(ctx); }
int ensure_stage(she_ctx *c, size_t words);             // grows she_ctx::d_stage
void free_leveled(she_ctx *c);                          // releases the leveled-mode pools
}  // namespace she

// calls that read or write the pool are refused while operators are being recorded
#define SHE_NOT_WHILE_DEFERRED(ctx)                                                               \
    do {                                                                                          \
        if ((ctx)->deferred)                                                                      \
            return she::fail(ctx, SHE_EINVAL, "a deferred circuit is pending: call she_defer_run first"); \
    } while (0)

#define HIP_TRY(ctx, expr)                                                                        \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess)                                                                     \
            return she::fail(ctx, e_ == hipErrorOutOfMemory ? SHE_ENOMEM : SHE_EDEVICE,           \
                             std::string(#expr) + ": " + hipGetErrorString(e_));                  \
    } while (0)
