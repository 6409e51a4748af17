#!/usr/bin/env python3
"""Benchmark of the bootstrapped-gate hot path on one MI355X.

A step = one pass of the whole path (linear combination + modulus switch, blind rotation,
sample extraction, key switch) over one circuit level of 4096 independent gates at
n=630, N=1024 (the workload the metric is quoted on), with keys, input ciphertexts and the
gate arrays already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--no-conv-layer]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GATES_PER_LEVEL = 4096
# Algorithmic FP64 work of the blind rotation per gate at n=630, N=1024, l=3 (FFT route):
# per CMux 6 forward + 2 inverse 512-point complex transforms (5*512*9 butterfly flops plus
# the 6*512 twist each = 26.1 KFLOP) and 12*512 complex multiply-adds (8 flops each = 49.2 KFLOP),
# i.e. 0.258 MFLOP per CMux, times 630 CMux.
FLOP_PER_CMUX = 8 * (5 * 512 * 9 + 6 * 512) + 12 * 512 * 8
FLOP_PER_GATE = 630 * FLOP_PER_CMUX
FP64_VECTOR_PEAK_TFLOPS = 78.6      # 256 CUs x 4 SIMDs x 16 lanes x 2 flop/FMA x 2.4 GHz
# FP64 vector instructions one wavefront executes per CMux in k_blind_rotate at N=1024, l=3, counted in the kernel's
# ISA: 6 forward rows x 323 + 518 (inverse transforms, rounding); beside them 443 LDS, 97 global-load and about 535
# integer vector instructions
FP64_INSTR_PER_CMUX = 2456
# HBM-side bytes per blind-rotation launch.  NOT measured by this program: the figure comes from two separate
# rocprofv3 --pmc runs of this same command (FETCH_SIZE 948,610 KiB scaled by 2.00, WRITE_SIZE 110,478 KiB scaled by
# 1.00; scales from a 256 MiB device copy in the same runs) whose summary is the file named below.  Algorithmic bytes
# are ~85 MB: the excess is the key spectra streamed once per XCD L2 and per resident batch (8 x 2 x 61.9 MB), served
# by the Infinity Cache.
MEASURED_TRAFFIC_BYTES = 2.06e9
TRAFFIC_SOURCE = ("profiles/k_blind_rotate_level4096_n630_N1024_counters.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                  "passes over `bench.py --calibrate-copy`, scaled by a 256 MiB device copy; carried over, not measured "
                  "in this run")


def cpu_baseline(sample_gates: int, single_thread_gates: int = 8):
    """The oracle, as it stands, on this machine's host cores, on the first gates of the same workload: once spread
    over the host threads, once on a single thread (a smaller sample, so that both legs stay within ~30 s)."""
    import numpy as np

    import synth_inputs as S
    from oracle import tfhe as O

    threads = max(1, min(os.cpu_count() or 1, 16))
    bits, codes = S.cfg2_real_level(GATES_PER_LEVEL)
    K = O.keygen(O.REAL, S.KEY_SEED)

    def leg(g, thr):
        fresh = O.encrypt_bits(K, bits[: 2 * g], S.data_seed(2))
        pool = np.zeros((3 * g, K.params.n + 1), np.uint32)
        pool[: 2 * g] = fresh
        ids = np.arange(2 * g, dtype=np.uint32)
        t0 = time.perf_counter()
        O.eval_gates(K, pool, codes[:g], ids[0::2], ids[1::2], np.arange(2 * g, 3 * g, dtype=np.uint32), threads=thr)
        dt = time.perf_counter() - t0
        return {"value": g / dt, "unit": "gates/s", "cores": min(thr, g), "kind": "oracle",
                "sample": f"first {g} gates of the 4096-gate level, schoolbook negacyclic products, "
                          f"{min(thr, g)} OpenMP thread(s), {dt:.1f} s wall"}

    return leg(sample_gates, threads), leg(single_thread_gates, 1)


def conv_layer(ctx_factory, fold: bool, native_mux: bool = False, cells3: bool = False, fused_pool: bool = False,
               narrow: bool = False, columns: bool = False):
    """Config 5: 28x28x1 8-bit image, 3x3 conv to 8 channels (log-quantized weights, 16-bit
    accumulators), ReLU, 2x2 max pool; returns latency and gate counts.  fold: let the operators
    skip gates fixed by constant operands (SHE_OPT_FOLD_CONSTANTS); cells3: full-adder cells of
    two three-input gates (SHE_OPT_GATE3_CELLS); narrow: the accumulators, the ReLU and the pooling
    get the width that the layer's plaintext weights can fill (the same integers come out)."""
    import numpy as np

    import synth_inputs as S
    from paper_1906_00148_amd.layers import accumulator_bits

    img, sign, exp = S.cfg5_conv_layer()
    H, W = img.shape
    oc, k = sign.shape[0], sign.shape[1]
    oh, ow = H - k + 1, W - k + 1
    n_in = H * W * 8
    AB = min(16, accumulator_bits(sign.reshape(oc, -1), exp.reshape(oc, -1), 8)) if narrow else 16
    conv_ids = n_in + np.arange(oh * ow * oc * AB, dtype=np.uint32)
    relu_ids = conv_ids[-1] + 1 + np.arange(oh * ow * oc * AB, dtype=np.uint32)
    pool_ids = relu_ids[-1] + 1 + np.arange((oh // 2) * (ow // 2) * oc * AB, dtype=np.uint32)
    ctx = ctx_factory(int(pool_ids[-1]) + 1)
    ctx.set_option(1, int(fold))
    ctx.set_option(2, int(native_mux))
    ctx.set_option(4, int(cells3))
    ctx.set_option(8, int(columns))      # SHE_OPT_COLUMN_ADDER: the sums by column compression
    bits = ((img[..., None] >> np.arange(8)) & 1).astype(np.uint8)
    in_ids = np.arange(n_in, dtype=np.uint32).reshape(H, W, 8)
    ctx.encrypt_bits(bits.ravel(), S.data_seed(5), in_ids.ravel())
    # receptive fields: unit (y, x, c) reads the k*k pixels under it
    x_ids = np.zeros((oh, ow, oc, k * k, 8), np.uint32)
    for dy in range(k):
        for dx in range(k):
            x_ids[:, :, :, dy * k + dx, :] = in_ids[dy:dy + oh, dx:dx + ow, None, :]
    w_sign = np.broadcast_to(sign.reshape(1, 1, oc, k * k), (oh, ow, oc, k * k)).reshape(-1, k * k)
    w_exp = np.broadcast_to(exp.reshape(1, 1, oc, k * k), (oh, ow, oc, k * k)).reshape(-1, k * k)
    t0 = time.perf_counter()
    g1 = ctx.shift_acc(x_ids.reshape(-1, k * k, 8), w_sign, w_exp, AB, conv_ids.reshape(-1, AB))
    t1 = time.perf_counter()
    schedules = [ctx.last_level_sizes()]
    if fused_pool:                       # ReLU and pooling as one operator (she_relu_maxpool)
        g2, t2 = 0, t1
        g3 = ctx.relu_maxpool(conv_ids.reshape(oh, ow, oc, AB), pool_ids.reshape(oh // 2, ow // 2, oc, AB))
    else:
        g2 = ctx.relu(conv_ids.reshape(-1, AB), relu_ids.reshape(-1, AB))
        t2 = time.perf_counter()
        schedules.append(ctx.last_level_sizes())
        g3 = ctx.maxpool(relu_ids.reshape(oh, ow, oc, AB), pool_ids.reshape(oh // 2, ow // 2, oc, AB))
    t3 = time.perf_counter()
    schedules.append(ctx.last_level_sizes())
    # all 13x13x8 outputs against plain integer arithmetic (16-bit accumulators: the narrow widths hold the same values)
    dec = ctx.decrypt(pool_ids.reshape(-1, AB)).astype(np.int64)
    got = (dec << np.arange(AB)).sum(axis=1)
    got = np.where(got >= (1 << (AB - 1)), got - (1 << AB), got).reshape(oh // 2, ow // 2, oc)
    conv = np.zeros((oh, ow, oc), np.int64)
    for dy in range(k):
        for dx in range(k):
            conv += (img[dy:dy + oh, dx:dx + ow, None] >> -exp[None, None, :, dy, dx].astype(np.int64)) * sign[None, None, :, dy, dx]
    conv = ((conv + 32768) % 65536) - 32768
    act = np.maximum(conv, 0)[: oh // 2 * 2, : ow // 2 * 2]
    want = np.maximum(np.maximum(act[0::2, 0::2], act[0::2, 1::2]), np.maximum(act[1::2, 0::2], act[1::2, 1::2]))
    assert np.array_equal(got, want), "conv layer decrypts wrongly"
    ctx.close()
    total = g1 + g2 + g3
    return {"workload": "28x28x1 -> conv3x3x8 (shift-accumulate) -> ReLU -> maxpool2x2, n=630 N=1024",
            "constant_folding": bool(fold), "native_mux": bool(native_mux), "cells3": bool(cells3), "relu_and_pool_fused": bool(fused_pool),
            "accumulator_bits": int(AB), "column_adder": bool(columns),
            "latency_s": t3 - t0, "gates": int(total), "gates_per_s": total / (t3 - t0),
            "conv_s": t1 - t0, "relu_s": t2 - t1, "pool_s": t3 - t2,
            "conv_gates": int(g1), "relu_gates": int(g2), "pool_gates": int(g3), "schedule": level_histogram(schedules)}


def neuron_576(ctx_factory, lean: bool):
    """Config 3: one neuron of 576 shifted 8-bit terms into a 16-bit accumulator (latency-bound: ~500 gates per
    level); the literal adder tree, or with folding, three-input cells and column compression (lean)."""
    import numpy as np

    import synth_inputs as S

    x, sign, exp = S.cfg3_neuron()
    ctx = ctx_factory(8192)
    if lean:
        for opt in (1, 4, 8):
            ctx.set_option(opt, 1)
    bits = ((x.reshape(-1)[:, None] >> np.arange(8)) & 1).astype(np.uint8)
    ids = np.arange(bits.size, dtype=np.uint32)
    ctx.encrypt_bits(bits.ravel(), S.data_seed(3), ids)
    out = np.arange(6000, 6016, dtype=np.uint32).reshape(1, 16)
    best = None
    for _ in range(3):
        t0 = time.perf_counter()
        g = ctx.shift_acc(ids.reshape(1, 576, 8), sign, exp, 16, out)
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    schedule = level_histogram([ctx.last_level_sizes()])
    got = int((ctx.decrypt(out).astype(np.int64) << np.arange(16)).sum())
    want = int(((x >> -exp.astype(np.int64)) * sign).sum()) % 65536
    assert got == want, "the neuron decrypts wrongly"
    ctx.close()
    return {"workload": "one neuron: 576 terms x 8 bits, weights sign * 2^e, 16-bit accumulator, n=630 N=1024"
                        + (", folding + three-input cells + column compression" if lean else ", literal adder tree"),
            "latency_s": best, "gates": int(g), "gates_per_s": g / best, "schedule": schedule}


def relu_pool_map(ctx_factory):
    """Config 4: ReLU then 2x2 max pooling over a 32x32x16 map of 16-bit values (1.62 M gates as stated netlists)."""
    import numpy as np

    import synth_inputs as S

    v = S.cfg4_feature_map()
    H, W, Cn = v.shape
    bits = (((v % 65536)[..., None] >> np.arange(16)) & 1).astype(np.uint8)
    n_in = bits.size
    in_ids = np.arange(n_in, dtype=np.uint32).reshape(H, W, Cn, 16)
    relu_ids = (n_in + np.arange(n_in, dtype=np.uint32)).reshape(H, W, Cn, 16)
    pool_ids = (2 * n_in + np.arange(n_in // 4, dtype=np.uint32)).reshape(H // 2, W // 2, Cn, 16)
    ctx = ctx_factory(int(pool_ids.max()) + 1)
    ctx.encrypt_bits(bits.ravel(), S.data_seed(4), in_ids.ravel())
    t0 = time.perf_counter()
    g1 = ctx.relu(in_ids.reshape(-1, 16), relu_ids.reshape(-1, 16))
    t1 = time.perf_counter()
    schedules = [ctx.last_level_sizes()]
    g2 = ctx.maxpool(relu_ids, pool_ids)
    t2 = time.perf_counter()
    schedules.append(ctx.last_level_sizes())
    dec = ctx.decrypt(pool_ids.reshape(-1, 16)).astype(np.int64)
    got = (dec << np.arange(16)).sum(axis=1).reshape(H // 2, W // 2, Cn)
    act = np.maximum(v, 0)
    want = np.maximum(np.maximum(act[0::2, 0::2], act[0::2, 1::2]), np.maximum(act[1::2, 0::2], act[1::2, 1::2]))
    assert np.array_equal(got, want), "ReLU + pooling decrypts wrongly"
    ctx.close()
    return {"workload": "32x32x16 map of 16-bit values -> ReLU -> maxpool2x2, n=630 N=1024, stated netlists",
            "latency_s": t2 - t0, "gates": int(g1 + g2), "gates_per_s": (g1 + g2) / (t2 - t0),
            "relu_s": t1 - t0, "pool_s": t2 - t1, "relu_gates": int(g1), "pool_gates": int(g2),
            "schedule": level_histogram(schedules)}


def level_histogram(schedules):
    """Entries per level of the circuits a call ran (she_last_level_sizes; a native MUX entry is two blind rotations):
    how many levels fall into each size class, and the blind rotations they hold."""
    import numpy as np

    rot = np.concatenate([g.astype(np.int64) + 2 * m.astype(np.int64) for g, m in schedules]) if schedules else np.zeros(0, np.int64)
    edges = [1, 257, 1025, 2049, 4097, 16385]
    names = ["1-256", "257-1024", "1025-2048", "2049-4096", "4097-16384", ">16384"]
    hist = {}
    for i, name in enumerate(names):
        lo, hi = edges[i], edges[i + 1] if i + 1 < len(edges) else None
        pick = (rot >= lo) & ((rot < hi) if hi else True)
        hist[name] = {"levels": int(pick.sum()), "rotations": int(rot[pick].sum())}
    return {"levels": int((rot > 0).sum()), "rotations": int(rot.sum()), "rotations_per_level_classes": hist}


def network(ctx_factory, deferred: bool = False, batch: int = 1):
    """deferred: the five operator calls are recorded (she_defer_begin) and run as ONE circuit, so that the scheduler
    overlaps one operator's last levels with the next one's first.
    batch > 1 (deferred only): that many images (the same network; image b is the seeded image with its rows rolled by b)
    recorded into ONE circuit, so every level holds the entries of all of them: the way a serving loop fills the
    chip where one image's small levels cannot.
    A second, deeper workload: conv - ReLU - pool - conv - ReLU - pool - dense on a 14x14 8-bit image (the MNIST
    network's layer sequence, shrunk), chained on the device without decrypting in between; folding, native MUX, three-input cells and the column adder on."""
    import numpy as np

    import synth_inputs as S
    from paper_1906_00148_amd.layers import Chain

    img, w1, w2, w3 = S.cfg6_network()

    def conv_plain(x, sign, exp):
        k = sign.shape[1]
        oh, ow = x.shape[0] - k + 1, x.shape[1] - k + 1
        out = np.zeros((oh, ow, sign.shape[0]), np.int64)
        for dy in range(k):
            for dx in range(k):
                for ci in range(x.shape[2]):
                    out += (x[dy:dy + oh, dx:dx + ow, ci, None] >> -exp[None, None, :, dy, dx, ci].astype(np.int64)) \
                        * sign[None, None, :, dy, dx, ci]
        return ((out + 32768) % 65536) - 32768

    def pool_plain(x):
        x = np.maximum(x, 0)[: x.shape[0] // 2 * 2, : x.shape[1] // 2 * 2]
        return np.maximum(np.maximum(x[0::2, 0::2], x[0::2, 1::2]), np.maximum(x[1::2, 0::2], x[1::2, 1::2]))

    assert batch == 1 or deferred
    imgs = [np.roll(img, b, axis=0) for b in range(batch)]

    def plain(im):
        feat = pool_plain(conv_plain(pool_plain(conv_plain(im[..., None], *w1)), *w2)).reshape(-1)
        want = ((feat[None, :] >> -w3[1].astype(np.int64)) * w3[0]).sum(axis=1)
        return ((want + 32768) % 65536) - 32768

    ctx = ctx_factory(32768 * batch)
    ctx.set_option(1, 1)
    ctx.set_option(2, 1)
    ctx.set_option(4, 1)
    ctx.set_option(8, 1)
    bits = np.stack([((im[..., None, None] >> np.arange(8)) & 1).astype(np.uint8) for im in imgs])
    x_ids = np.arange(bits.size, dtype=np.uint32).reshape(bits.shape)
    ctx.encrypt_bits(bits.ravel(), S.data_seed(6), x_ids.ravel())
    net = Chain(ctx, x_ids.size)
    t0 = time.perf_counter()
    if deferred:
        ctx.defer_begin()
    schedules = []

    def ran(x):                          # the schedule of the operator that just ran (nothing runs while recording)
        if not deferred:
            schedules.append(ctx.last_level_sizes())
        return x

    scores = []
    for b in range(batch):
        a1 = ran(net.relu_maxpool(ran(net.conv(x_ids[b], w1[0], w1[1], 16))))
        a2 = ran(net.relu_maxpool(ran(net.conv(Chain.unsigned_view(a1), w2[0], w2[1], 16))))
        scores.append(ran(net.dense(Chain.unsigned_view(a2), w3[0], w3[1], 16)))
    if deferred:
        ctx.defer_run()
        schedules.append(ctx.last_level_sizes())
    dt = time.perf_counter() - t0
    for b in range(batch):
        dec = ctx.decrypt(scores[b]).astype(np.int64)
        got = (dec << np.arange(16)).sum(axis=1)
        got = np.where(got >= 32768, got - 65536, got)
        assert np.array_equal(got, plain(imgs[b])), "network decrypts wrongly"
    ctx.close()
    return {"workload": "14x14x1 -> conv3x3x4 -> ReLU -> pool -> conv3x3x4 -> ReLU -> pool -> dense 10, n=630 N=1024, "
                        "constant folding, native MUX, three-input cells and column-compression accumulators on"
                        + (", the five operators run as one deferred circuit" if deferred else "")
                        + (f", {batch} images in that one circuit" if batch > 1 else ""),
            "images": batch, "latency_s": dt, "images_per_s": batch / dt, "entries": int(net.gates),
            "entries_per_s": net.gates / dt, "schedule": level_histogram(schedules)}


def cmux_level(ctx_factory, count: int = 4096, reps: int = 5):
    """Leveled mode: one level of `count` independent CMuxes (TRGSW selector x TRLWE data) at the context's ring degree
    (1024, or Section 4's N-bar = 2048); the kernel's time from the library's HIP events, and a check that every
    output carries the selected branch's message."""
    import numpy as np

    ctx = ctx_factory(16)
    N = ctx.params.N
    nsel, ndat = 64, 256
    ctx.leveled_init(nsel, ndat + count)
    rng = np.random.default_rng(2024)
    sel_bits = rng.integers(0, 2, nsel).astype(np.uint8)
    ctx.trgsw_encrypt_bits(sel_bits, 1, np.arange(nsel, dtype=np.uint32))
    mu = np.where(rng.integers(0, 2, (ndat, N)) == 1, 1 << 29, (1 << 32) - (1 << 29)).astype(np.uint32)
    ctx.trlwe_encrypt(mu, 2, np.arange(ndat, dtype=np.uint32))
    s, i1, i0 = rng.integers(0, nsel, count), rng.integers(0, ndat, count), rng.integers(0, ndat, count)
    out = (ndat + np.arange(count)).astype(np.uint32)
    ms = []
    for _ in range(reps):
        ctx.eval_cmux(s, i1, i0, out)
        ms.append(ctx.last_timing()["blind_rotate_ms"])
    picks = np.unique(np.linspace(0, count - 1, 64).astype(np.int64))         # spread over every round of the grid
    phases = ctx.trlwe_phase(out[picks]).astype(np.int32)
    for k, m in enumerate(picks):
        want = mu[i1[m]] if sel_bits[s[m]] else mu[i0[m]]
        assert np.array_equal(phases[k] > 0, want.astype(np.int32) > 0), "CMux selected the wrong branch"
    ctx.close()
    best = float(np.median(ms))
    # per CMux 8 transforms of N/2 complex points (5 (N/2) log2(N/2) + 6 (N/2) flops) and 12 (N/2) complex multiply-adds:
    # 0.258 MFLOP at N = 1024 (one step of the blind rotation), 0.557 MFLOP at N = 2048
    flop = (8 * (5 * (N // 2) * int(np.log2(N // 2)) + 6 * (N // 2)) + 12 * (N // 2) * 8) * count
    # bytes that must move: two TRLWE operands in, one out (8 KiB each) per CMux, every distinct selector (96 KiB) once
    moved = count * 3 * 2 * N * 4 + nsel * 2 * 3 * 2 * (N // 2) * 16
    return {"workload": f"one level of {count} CMuxes over {nsel} distinct selectors, N={N} l=3 Bgbit=7 "
                        "(leveled mode: no bootstrap)",
            "kernel_ms": best, "cmux_per_s": count / (best * 1e-3), "achieved_tflops": flop / (best * 1e-3) / 1e12,
            "algorithmic_bytes": moved, "achieved_gb_per_s": moved / (best * 1e-3) / 1e9}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-gates", type=int, default=32)
    ap.add_argument("--no-conv-layer", action="store_true", help="skip config 5 (one conv layer, ~2.5M gates, ~15 s)")
    ap.add_argument("--leveled-only", action="store_true",
                    help="run only the leveled-mode CMux level and print its entry (for profiling k_cmux)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy (reference kernel for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only; gates of a level would be sharded across GPUs "
              "with replicated keys, which is not built. Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_1906_00148_amd as she
    import synth_inputs as S

    assert torch.cuda.is_available(), "bench.py needs a GPU (there is no CPU path)"
    torch.cuda.set_device(0)
    if args.leveled_only:
        print(json.dumps({"cmux_level": cmux_level(lambda cap: she.Context(she.REAL, S.KEY_SEED, cap), reps=args.steps),
                          "cmux_level_section4_2048": cmux_level(lambda cap: she.Context(she.SECTION4_LEVELED, S.KEY_SEED, cap),
                                                                 reps=args.steps)}))
        return
    G = GATES_PER_LEVEL
    bits, codes = S.cfg2_real_level(G)
    ctx = she.Context(she.REAL, S.KEY_SEED, 3 * G)
    in_ids = np.arange(2 * G, dtype=np.uint32)
    ctx.encrypt_bits(bits, S.data_seed(2), in_ids)
    d_type = torch.from_numpy(codes.copy()).cuda()
    d_in0 = torch.from_numpy(in_ids[0::2].astype(np.int32)).cuda()
    d_in1 = torch.from_numpy(in_ids[1::2].astype(np.int32)).cuda()
    d_out = torch.arange(2 * G, 3 * G, dtype=torch.int32, device="cuda")

    def step():
        ctx.eval_gates_device(d_type.data_ptr(), d_in0.data_ptr(), d_in1.data_ptr(), d_out.data_ptr(), G)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.last_timing()                       # drop the warm-up's events
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    tim = ctx.last_timing()                 # HIP events on the kernels' stream, summed over the timed steps
    # correctness of what was timed: every output decrypts to the plain gate
    dec = ctx.decrypt(np.arange(2 * G, 3 * G, dtype=np.uint32))
    table = {0: lambda a, b: 1 - (a & b), 1: lambda a, b: a & b, 2: lambda a, b: a | b, 3: lambda a, b: a ^ b,
             4: lambda a, b: 1 - (a ^ b)}
    want = np.array([table[int(c)](int(bits[2 * g]), int(bits[2 * g + 1])) for g, c in enumerate(codes)], np.uint8)
    assert np.array_equal(dec, want), "timed level decrypts wrongly"

    ms_per_step = dt / args.steps * 1e3
    br_ms = tim["blind_rotate_ms"] / args.steps
    achieved = FLOP_PER_GATE * G / (br_ms * 1e-3) / 1e12
    out = {
        "metric": "bootstrapped TFHE gates/sec at n=630,N=1024 on 1 MI355X; conv-layer latency",
        "value": G * args.steps / dt, "unit": "gates/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": "one level of 4096 independent bootstrapped gates (NAND/AND/OR/XOR/XNOR uniform) on "
                               "fresh encryptions of uniform bits, n=630 N=1024 k=1 Bgbit=7 l=3 ks t=8 base 4",
                   "gates_per_step": G, "seed": S.KEY_SEED},
        "kernels_ms_per_step": {"lincomb": tim["lincomb_ms"] / args.steps, "blind_rotate": br_ms,
                                "key_switch": tim["key_switch_ms"] / args.steps},
        "roofline": {"bound": "alu", "kernel": "k_blind_rotate", "achieved": achieved,
                     "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / FP64_VECTOR_PEAK_TFLOPS,
                     "traffic": MEASURED_TRAFFIC_BYTES, "traffic_source": TRAFFIC_SOURCE},
        "paper_context": {"value": 77, "unit": "gates/s", "note": "implied by the paper's projected fully-homomorphic "
                          "latency / gate count (about 13 ms per gate), Xeon E7-4850, different parameter set"},
    }
    # exactness of what was timed: the same level once more with the kernel recording the largest distance from an
    # integer of everything it rounds (outside the timed region; the tracking kernel is slower)
    ctx.set_round_tracking(True)
    ctx.get_round_error(reset=True)
    step()
    torch.cuda.synchronize()
    worst = ctx.get_round_error()
    ctx.set_round_tracking(False)
    ctx.last_timing()
    assert 0.0 < worst < 0.2, f"FP64 products are not safely exact: largest distance from an integer {worst}"
    out["max_distance_from_integer_before_rounding"] = worst
    # DIAGNOSTICS, not rooflines: what the FP64 pipes of this box issue at (2 wavefronts per SIMD, sustained; the
    # published peak assumes one FMA per lane and cycle at 2.4 GHz = 1.67 ns per wave64 instruction and SIMD), and a
    # probe that issues plain additions with the kernel's own LDS and key-load pattern beside them.  The second ratio
    # compares the kernel with something shaped like itself: it says where the time goes, not how far a roofline is.
    probe = {name: ctx.probe_fp64_rate(form) for form, name in ((0, "fma_scalar_operands"), (1, "fma_three_registers"),
                                                               (2, "add_two_registers"),
                                                               (3, "add_with_the_kernels_lds_and_key_loads"))}
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    br_ns = br_ms * 1e6 / (G * 630 * FP64_INSTR_PER_CMUX / (4.0 * cus))
    # the LDS pipe of a compute unit, 16 bytes per lane and operation, 8 wavefronts (she_probe_lds_rate): the rows of
    # the exchange buffers were chosen from these figures; an exchange is 8 stores and 8 loads per lane
    lds = {name: ctx.probe_lds_rate(form) for form, name in (
        (0, "loads_consecutive"), (1, "stores_consecutive"), (2, "read_back_after_first_pass_row_72"),
        (3, "read_back_after_first_pass_row_65"), (4, "read_back_after_second_pass_row_65"))}
    out["diagnostics"] = {
        "note": "issue-rate probes; not part of the roofline, whose fraction is against the published 78.6 TFLOP/s",
        "measured_fp64_issue": probe,
        "lds_bytes_per_ns_per_compute_unit": lds,
        "blind_rotate_over_measured_fma_rate": achieved / probe["fma_scalar_operands"]["tflops_as_fma"],
        "blind_rotate_ns_per_fp64_instruction_per_simd": br_ns,
        "probe_with_kernel_memory_pattern_over_blind_rotate": probe["add_with_the_kernels_lds_and_key_loads"][
            "ns_per_instruction_per_simd"] / br_ns,
    }
    ctx.close()
    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        out["calibration_copy_bytes"] = int(src.numel() * 4)
        del src, dst
    if not args.no_conv_layer:
        out["conv_layer"] = conv_layer(lambda cap: she.Context(she.REAL, S.KEY_SEED, cap), fold=False)
        out["conv_layer_lean"] = conv_layer(lambda cap: she.Context(she.REAL, S.KEY_SEED, cap), fold=True, native_mux=True,
                                            cells3=True, fused_pool=True)
        out["conv_layer_lean_narrow"] = conv_layer(lambda cap: she.Context(she.REAL, S.KEY_SEED, cap), fold=True,
                                                   native_mux=True, cells3=True, fused_pool=True, narrow=True)
        out["conv_layer_lean_columns"] = conv_layer(lambda cap: she.Context(she.REAL, S.KEY_SEED, cap), fold=True,
                                                    native_mux=True, cells3=True, fused_pool=True, narrow=True, columns=True)
        out["neuron_576"] = neuron_576(lambda cap: she.Context(she.REAL, S.KEY_SEED, cap), lean=False)
        out["neuron_576_lean"] = neuron_576(lambda cap: she.Context(she.REAL, S.KEY_SEED, cap), lean=True)
        out["relu_pool_map"] = relu_pool_map(lambda cap: she.Context(she.REAL, S.KEY_SEED, cap))
        out["network"] = network(lambda cap: she.Context(she.REAL, S.KEY_SEED, cap))
        out["network_deferred"] = network(lambda cap: she.Context(she.REAL, S.KEY_SEED, cap), deferred=True)
        out["network_deferred_batch8"] = network(lambda cap: she.Context(she.REAL, S.KEY_SEED, cap), deferred=True, batch=8)
        out["cmux_level"] = cmux_level(lambda cap: she.Context(she.REAL, S.KEY_SEED, cap))
        out["cmux_level_16k"] = cmux_level(lambda cap: she.Context(she.REAL, S.KEY_SEED, cap), count=16384)
        # the ring degree of the paper's leveled setting (Section 4: n = 500, N-bar = 2048)
        out["cmux_level_section4_2048"] = cmux_level(lambda cap: she.Context(she.SECTION4_LEVELED, S.KEY_SEED, cap))
    if not args.no_cpu_baseline:
        out["cpu_baseline"], out["cpu_baseline_single_thread"] = cpu_baseline(args.cpu_sample_gates)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
