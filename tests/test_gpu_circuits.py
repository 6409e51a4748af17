"""GPU tests of the layer operators at the benchmark configurations' real parameters: results
are decrypted and compared with plain integer arithmetic (the operators' definitions), which
holds at any size; gate counts are compared with the oracle's netlists."""
import numpy as np
import pytest

import synth_inputs as S
from oracle import circuits as OC

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_1906_00148_amd as pkg
    c = pkg.Context(pkg.REAL, S.KEY_SEED, 300000)
    yield c
    c.close()


def encrypt_values(ctx, values, bits, seed, first_id=0):
    b = OC.to_bits(np.asarray(values), bits)
    ids = np.arange(first_id, first_id + b.size, dtype=np.uint32).reshape(b.shape)
    ctx.encrypt_bits(b.ravel(), seed, ids.ravel())
    return ids


def test_cfg3_neuron_576_terms(ctx):
    x, sign, exp = S.cfg3_neuron()
    ids = encrypt_values(ctx, x, 8, S.data_seed(3))
    out = np.arange(200000, 200016, dtype=np.uint32).reshape(1, 16)
    gates = ctx.shift_acc(ids, sign, exp, 16, out)
    t = ctx.last_timing()
    print(f"\ncfg3: {gates} gates in {t['levels']} levels, blind rotate {t['blind_rotate_ms']:.1f} ms, "
          f"key switch {t['key_switch_ms']:.1f} ms")
    nl, _ = OC.build_shift_acc(1, 576, 8, sign, exp, 16)
    assert gates == len(nl.gtype)
    assert t["levels"] == int(nl.levels().max())
    got = OC.from_bits(ctx.decrypt(out), True)
    assert np.array_equal(got, OC.plain_shift_acc(x, sign, exp, 16))


def test_cfg4_relu_maxpool_reduced_and_corner_values(ctx):
    fm = S.cfg4_feature_map(8, 8, 4)
    fm[0, 0, 0], fm[0, 1, 0], fm[1, 0, 0], fm[1, 1, 0] = -32768, 32767, 0, -1
    fm[2, 2, 1] = fm[2, 3, 1] = fm[3, 2, 1] = fm[3, 3, 1] = 77          # equal operands
    ids = encrypt_values(ctx, fm, 16, S.data_seed(4))
    relu_ids = np.arange(100000, 100000 + ids.size, dtype=np.uint32).reshape(ids.shape)
    g1 = ctx.relu(ids.reshape(-1, 16), relu_ids.reshape(-1, 16))
    assert g1 == 8 * 8 * 4 * 15
    assert np.array_equal(OC.from_bits(ctx.decrypt(relu_ids), True), OC.plain_relu(fm))
    pool_ids = np.arange(150000, 150000 + 4 * 4 * 4 * 16, dtype=np.uint32).reshape(4, 4, 4, 16)
    g2 = ctx.maxpool(relu_ids, pool_ids)
    assert g2 == 4 * 4 * 4 * 3 * 112
    assert np.array_equal(OC.from_bits(ctx.decrypt(pool_ids), True), OC.plain_maxpool2x2(OC.plain_relu(fm)))
    # pooling signed values directly (negative maxima)
    pool2 = pool_ids + 5000
    ctx.maxpool(ids, pool2)
    assert np.array_equal(OC.from_bits(ctx.decrypt(pool2), True), OC.plain_maxpool2x2(fm))
