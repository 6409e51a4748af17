// Leveled mode of the C ABI (declared in include/she.h): TRGSW selectors, TRLWE data, batched CMux.
#include <algorithm>
#include <new>

#include "she_ctx.h"

using namespace she;

namespace {

constexpr size_t kTrgswChunk = 512;     // selectors generated, uploaded and transformed per round trip

size_t trgsw_hat_elems(const she_params &P) { return (size_t)2 * P.l * 2 * (P.N / 2); }   // double2 per selector

int need_pools(she_ctx *c)
{
    if (!c->lev.trlwe) return fail(c, SHE_EINVAL, "she_leveled_init has not been called");
    return SHE_OK;
}

int check_range(she_ctx *c, const uint32_t *ids, size_t count, uint32_t cap, const char *what)
{
    for (size_t k = 0; k < count; k++)
        if (ids[k] >= cap) return fail(c, SHE_ERANGE, std::string(what) + ": id outside the pool");
    return SHE_OK;
}

int ensure_ids(she_ctx *c, size_t count)
{
    if (count <= c->lev.ids_cap) return SHE_OK;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (c->lev.d_ids) hipFree(c->lev.d_ids);
    c->lev.d_ids = nullptr; c->lev.ids_cap = 0;
    count += count / 4;
    HIP_TRY(c, hipMalloc((void **)&c->lev.d_ids, 4 * count * sizeof(uint32_t)));
    c->lev.ids_cap = count;
    return SHE_OK;
}

}  // namespace

namespace she {
void free_leveled(she_ctx *c)
{
    hipFree(c->lev.trgsw_hat); hipFree(c->lev.trlwe); hipFree(c->lev.d_ids);
    c->lev = LeveledPools{};
}
}  // namespace she

extern "C" {

int she_leveled_init(she_ctx *c, uint32_t trgsw_capacity, uint32_t trlwe_capacity)
try {
    if (!c) return SHE_EINVAL;
    if (!trgsw_capacity || !trlwe_capacity) return fail(c, SHE_EINVAL, "capacities must be positive");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    free_leveled(c);
    HIP_TRY(c, hipMalloc((void **)&c->lev.trgsw_hat, (size_t)trgsw_capacity * trgsw_hat_elems(c->P) * sizeof(double2)));
    c->lev.trgsw_cap = trgsw_capacity;
    HIP_TRY(c, hipMalloc((void **)&c->lev.trlwe, (size_t)trlwe_capacity * 2 * c->P.N * sizeof(uint32_t)));
    c->lev.trlwe_cap = trlwe_capacity;
    HIP_TRY(c, hipMemsetAsync(c->lev.trgsw_hat, 0, (size_t)trgsw_capacity * trgsw_hat_elems(c->P) * sizeof(double2), c->stream));
    HIP_TRY(c, hipMemsetAsync(c->lev.trlwe, 0, (size_t)trlwe_capacity * 2 * c->P.N * sizeof(uint32_t), c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return SHE_OK;
} SHE_NOTHROW(c)

int she_trgsw_encrypt_bits(she_ctx *c, const uint8_t *bits, size_t count, uint64_t seed, const uint32_t *dst_ids)
try {
    if (!c) return SHE_EINVAL;
    int rc;
    if ((rc = need_pools(c))) return rc;
    if (count == 0) return SHE_OK;
    if (!bits || !dst_ids) return fail(c, SHE_EINVAL, "null argument");
    for (size_t k = 0; k < count; k++)
        if (bits[k] > 1) return fail(c, SHE_EINVAL, "bits must be 0 or 1");
    if ((rc = check_range(c, dst_ids, count, c->lev.trgsw_cap, "she_trgsw_encrypt_bits"))) return rc;
    const size_t words = (size_t)2 * c->P.l * 2 * c->P.N;           // Torus32 words per selector
    std::vector<uint32_t> host;
    try { host.resize(count * words); } catch (const std::bad_alloc &) { return fail(c, SHE_ENOMEM, "host staging"); }
    fresh_trgsw(c->P, c->hk.ring_key, bits, count, seed, host.data());
    const size_t step = std::min(count, kTrgswChunk);
    if ((rc = ensure_stage(c, step * words + step))) return rc;
    for (size_t off = 0; off < count; off += step) {
        const size_t cnt = std::min(step, count - off);
        uint32_t *d_ids = c->d_stage + step * words;
        HIP_TRY(c, hipMemcpyAsync(c->d_stage, host.data() + off * words, cnt * words * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(d_ids, dst_ids + off, cnt * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, launch_trgsw_transform(c->P, c->dk, c->d_stage, c->lev.trgsw_hat, d_ids, cnt, c->stream));
        HIP_TRY(c, hipStreamSynchronize(c->stream));
    }
    return SHE_OK;
} SHE_NOTHROW(c)

// Device order of a TRLWE component (the order the CMux kernel's lanes read it in): lane t of a transform works on
// the coefficients t + 64 m and t + 64 m + N/2 (m < N/128), and the 16-byte word (q, t) holds those of m = 2q and
// m = 2q + 1, so that one load per lane fetches four of them and a wavefront's load is one contiguous KiB.
static inline size_t device_pos(uint32_t N, uint32_t j)
{
    const uint32_t M = N / 2, h = j / M, r = j % M, t = r % 64, m = r / 64;
    return ((size_t)(m >> 1) * 64 + t) * 4 + (m & 1) * 2 + h;
}

static int upload_trlwe(she_ctx *c, const uint32_t *host, size_t count, const uint32_t *dst_ids)
{
    const uint32_t N = c->P.N;
    const size_t words = (size_t)2 * N;
    std::vector<uint32_t> dev(count * words);
    for (size_t k = 0; k < count; k++)
        for (uint32_t comp = 0; comp < 2; comp++)
            for (uint32_t j = 0; j < N; j++)
                dev[k * words + comp * N + device_pos(N, j)] = host[k * words + comp * N + j];
    for (size_t k = 0; k < count; k++)
        HIP_TRY(c, hipMemcpyAsync(c->lev.trlwe + dst_ids[k] * words, dev.data() + k * words, words * 4, hipMemcpyHostToDevice,
                                  c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return SHE_OK;
}

int she_trlwe_encrypt(she_ctx *c, const uint32_t *mu, size_t count, uint64_t seed, const uint32_t *dst_ids)
try {
    if (!c) return SHE_EINVAL;
    int rc;
    if ((rc = need_pools(c))) return rc;
    if (count == 0) return SHE_OK;
    if (!mu || !dst_ids) return fail(c, SHE_EINVAL, "null argument");
    if ((rc = check_range(c, dst_ids, count, c->lev.trlwe_cap, "she_trlwe_encrypt"))) return rc;
    std::vector<uint32_t> host;
    try { host.resize(count * 2 * c->P.N); } catch (const std::bad_alloc &) { return fail(c, SHE_ENOMEM, "host staging"); }
    fresh_trlwe(c->P, c->hk.ring_key, mu, count, seed, host.data());
    return upload_trlwe(c, host.data(), count, dst_ids);
} SHE_NOTHROW(c)

int she_trlwe_write(she_ctx *c, const uint32_t *samples, size_t count, const uint32_t *dst_ids)
try {
    if (!c) return SHE_EINVAL;
    int rc;
    if ((rc = need_pools(c))) return rc;
    if (count == 0) return SHE_OK;
    if (!samples || !dst_ids) return fail(c, SHE_EINVAL, "null argument");
    if ((rc = check_range(c, dst_ids, count, c->lev.trlwe_cap, "she_trlwe_write"))) return rc;
    return upload_trlwe(c, samples, count, dst_ids);
} SHE_NOTHROW(c)

int she_trlwe_read(she_ctx *c, const uint32_t *ids, size_t count, uint32_t *samples)
try {
    if (!c) return SHE_EINVAL;
    int rc;
    if ((rc = need_pools(c))) return rc;
    if (count == 0) return SHE_OK;
    if (!samples || !ids) return fail(c, SHE_EINVAL, "null argument");
    if ((rc = check_range(c, ids, count, c->lev.trlwe_cap, "she_trlwe_read"))) return rc;
    const uint32_t N = c->P.N;
    const size_t words = (size_t)2 * N;
    std::vector<uint32_t> dev(count * words);
    for (size_t k = 0; k < count; k++)
        HIP_TRY(c, hipMemcpyAsync(dev.data() + k * words, c->lev.trlwe + ids[k] * words, words * 4, hipMemcpyDeviceToHost,
                                  c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    for (size_t k = 0; k < count; k++)
        for (uint32_t comp = 0; comp < 2; comp++)
            for (uint32_t j = 0; j < N; j++)
                samples[k * words + comp * N + j] = dev[k * words + comp * N + device_pos(N, j)];
    return SHE_OK;
} SHE_NOTHROW(c)

int she_trlwe_phase(she_ctx *c, const uint32_t *ids, size_t count, uint32_t *phases)
try {
    if (!c) return SHE_EINVAL;
    if (count == 0) return SHE_OK;
    if (!phases) return fail(c, SHE_EINVAL, "null argument");
    std::vector<uint32_t> host;
    try { host.resize(count * 2 * c->P.N); } catch (const std::bad_alloc &) { return fail(c, SHE_ENOMEM, "host staging"); }
    int rc = she_trlwe_read(c, ids, count, host.data());
    if (rc) return rc;
    trlwe_phases(c->P, c->hk.ring_key, host.data(), count, phases);
    return SHE_OK;
} SHE_NOTHROW(c)

int she_eval_cmux(she_ctx *c, const uint32_t *sel, const uint32_t *in1, const uint32_t *in0, const uint32_t *out,
                  size_t count)
try {
    if (!c) return SHE_EINVAL;
    int rc;
    if ((rc = need_pools(c))) return rc;
    if (count == 0) return SHE_OK;
    if (!sel || !in1 || !in0 || !out) return fail(c, SHE_EINVAL, "null argument");
    if (count > 0xFFFFFFFFu) return fail(c, SHE_EINVAL, "too many CMux entries for one call");
    if ((rc = check_range(c, sel, count, c->lev.trgsw_cap, "she_eval_cmux sel"))) return rc;
    if ((rc = check_range(c, in1, count, c->lev.trlwe_cap, "she_eval_cmux in1"))) return rc;
    if ((rc = check_range(c, in0, count, c->lev.trlwe_cap, "she_eval_cmux in0"))) return rc;
    if ((rc = check_range(c, out, count, c->lev.trlwe_cap, "she_eval_cmux out"))) return rc;
    try {
        // a level's entries run concurrently: nothing may be written that another entry reads or writes
        std::vector<uint8_t> mark(c->lev.trlwe_cap, 0);
        for (size_t k = 0; k < count; k++) mark[in1[k]] = mark[in0[k]] = 1;
        for (size_t k = 0; k < count; k++) {
            if (mark[out[k]] == 1) return fail(c, SHE_EINVAL, "an output id is also an input id");
            if (mark[out[k]] == 2) return fail(c, SHE_EINVAL, "an output id appears twice");
            mark[out[k]] = 2;
        }
    } catch (const std::bad_alloc &) {
        return fail(c, SHE_ENOMEM, "host staging");
    }
    // The entries are independent, so their order is the library's to choose: grouped by selector (a counting sort),
    // the wavefronts that run at the same time read the same few selectors' spectra (96 KiB each at N = 1024, l = 3) and
    // find them in the L2 caches.  Measured on 16384 entries over 256 selectors in random order: 233 -> 162 us.
    std::vector<uint32_t> staged;
    try {
        staged.resize(4 * count);
        std::vector<uint32_t> first(c->lev.trgsw_cap + 1, 0);
        for (size_t k = 0; k < count; k++) first[sel[k] + 1]++;
        for (size_t v = 0; v < c->lev.trgsw_cap; v++) first[v + 1] += first[v];
        for (size_t k = 0; k < count; k++) {
            const size_t pos = first[sel[k]]++;
            staged[pos] = sel[k];
            staged[count + pos] = in1[k];
            staged[2 * count + pos] = in0[k];
            staged[3 * count + pos] = out[k];
        }
    } catch (const std::bad_alloc &) {
        return fail(c, SHE_ENOMEM, "host staging");
    }
    if ((rc = ensure_ids(c, count))) return rc;
    uint32_t *d = c->lev.d_ids;
    const size_t cap = c->lev.ids_cap;
    for (int a = 0; a < 4; a++)
        HIP_TRY(c, hipMemcpyAsync(d + a * cap, staged.data() + a * count, count * 4, hipMemcpyHostToDevice, c->stream));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (c->timing) {
        HIP_TRY(c, hipEventCreate(&e0));
        HIP_TRY(c, hipEventCreate(&e1));
        HIP_TRY(c, hipEventRecord(e0, c->stream));
    }
    HIP_TRY(c, launch_cmux(c->P, c->dk, c->lev.trgsw_hat, c->lev.trlwe, d, d + cap, d + 2 * cap, d + 3 * cap, count,
                           c->track_round ? c->d_round_err : nullptr, c->stream));
    if (c->timing) HIP_TRY(c, hipEventRecord(e1, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (c->timing) {
        float ms = 0.f;
        hipEventElapsedTime(&ms, e0, e1);
        hipEventDestroy(e0); hipEventDestroy(e1);
        c->last_ms[0] = 0; c->last_ms[1] = ms; c->last_ms[2] = 0; c->last_ms[3] = 1;   // the CMux kernel, one level
    }
    return SHE_OK;
} SHE_NOTHROW(c)

}  // extern "C"
