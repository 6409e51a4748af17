"""The entry point that allocates nothing (she_eval_gates_device_noalloc, for callers that cannot call hipMalloc)
against the entry point it is a variant of (she_eval_gates_device), through the C ABI: the same level evaluated by
both must give the same ciphertext words, on two calls in a row, the second with a smaller input (the static
scratch buffer then still holds the first call's contents).  Integer work: the bar is bit-exact.
"""
import numpy as np
import pytest

import synth_inputs as S

pytestmark = pytest.mark.gpu


def _both_ways(ctx, sizes, names, seed, n_words):
    """For each level size in turn: the level through eval_gates_device and through the no-allocation entry point,
    into different output slots; returns the pairs of result arrays."""
    import torch
    G0 = max(sizes)
    in_ids = np.arange(2 * G0, dtype=np.uint32)
    pairs = []
    for call, G in enumerate(sizes):
        bits, codes = S.gate_level(G, names, seed + call)
        print(f"no-alloc parity: call {call}, {G} gates, n+1 = {n_words}", flush=True)
        ctx.encrypt_bits(bits, 77 + call, in_ids[: 2 * G])
        out_a = np.arange(2 * G0, 2 * G0 + G, dtype=np.uint32)
        out_b = np.arange(3 * G0, 3 * G0 + G, dtype=np.uint32)
        d_type = torch.from_numpy(codes.copy()).cuda()
        d_in0 = torch.from_numpy(in_ids[0:2 * G:2].astype(np.int32)).cuda()
        d_in1 = torch.from_numpy(in_ids[1:2 * G:2].astype(np.int32)).cuda()
        d_out_a = torch.from_numpy(out_a.astype(np.int32)).cuda()
        d_out_b = torch.from_numpy(out_b.astype(np.int32)).cuda()
        ctx.eval_gates_device(d_type.data_ptr(), d_in0.data_ptr(), d_in1.data_ptr(), d_out_a.data_ptr(), G)
        torch.cuda.synchronize()
        ctx.eval_gates_device_noalloc(d_type.data_ptr(), d_in0.data_ptr(), d_in1.data_ptr(), d_out_b.data_ptr(), G)
        torch.cuda.synchronize()
        want, got = ctx.read_cts(out_a), ctx.read_cts(out_b)
        assert want.shape == (G, n_words) and want.any()
        # what the level decrypts to is checked too, so that "both wrong in the same way" cannot pass
        from oracle import circuits as OC
        plain = np.array([OC.plain_gate(int(c), int(bits[2 * g]), int(bits[2 * g + 1])) for g, c in enumerate(codes)], np.uint8)
        assert np.array_equal(ctx.decrypt(out_b), plain)
        pairs.append((want, got))
    return pairs


def test_no_alloc_entry_point_matches_eval_gates_device_toy():
    import paper_1906_00148_amd as pkg
    with pkg.Context(pkg.TOY, S.KEY_SEED, 4 * 300) as ctx:
        # 300 gates (one wavefront per gate would not be chosen: below the split threshold), then a ragged 77
        for want, got in _both_ways(ctx, (300, 77), tuple(S.GATE_CODE), 4100, pkg.TOY.n + 1):
            assert np.array_equal(got, want)


def test_no_alloc_entry_point_matches_eval_gates_device_real_and_rejects_oversize():
    import torch

    import paper_1906_00148_amd as pkg
    with pkg.Context(pkg.REAL, S.KEY_SEED, 4 * 96) as ctx:
        for want, got in _both_ways(ctx, (96, 40), S.GATE_NAMES_5, 4200, pkg.REAL.n + 1):
            assert np.array_equal(got, want)
        # a second context on the same GPU uses the same static buffer
        with pkg.Context(pkg.REAL, S.KEY_SEED + 1, 4 * 33) as other:
            for want, got in _both_ways(other, (33,), S.GATE_NAMES_5, 4300, pkg.REAL.n + 1):
                assert np.array_equal(got, want)
        # beyond the static buffer: refused on the host, nothing is launched (16 MiB hold 5056 gates at n=630, N=1024)
        G = 5057
        d = torch.zeros(G, dtype=torch.int32, device="cuda")
        t = torch.zeros(G, dtype=torch.uint8, device="cuda")
        with pytest.raises(pkg.SheError) as err:
            ctx.eval_gates_device_noalloc(t.data_ptr(), d.data_ptr(), d.data_ptr(), d.data_ptr(), G)
        assert err.value.code == -4 and "5056" in str(err.value)
