"""ctypes binding with the same names as the C ABI (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))

GATES = {"NAND": 0, "AND": 1, "OR": 2, "XOR": 3, "XNOR": 4, "NOR": 5, "ANDNY": 6, "ANDYN": 7, "ORNY": 8, "ORYN": 9}


class SheError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"she error {code}: {text}")
        self.code = code


class _CParams(C.Structure):
    _fields_ = [
        ("n", C.c_uint32), ("N", C.c_uint32), ("k", C.c_uint32), ("bg_bit", C.c_uint32), ("l", C.c_uint32),
        ("ks_t", C.c_uint32), ("ks_basebit", C.c_uint32), ("lwe_std", C.c_double), ("bk_std", C.c_double),
    ]


@dataclass(frozen=True)
class Params:
    n: int
    N: int
    k: int = 1
    bg_bit: int = 7
    l: int = 3
    ks_t: int = 8
    ks_basebit: int = 2
    lwe_std: float = 2.0 ** -15
    bk_std: float = 2.0 ** -25


TOY = Params(n=128, N=256)
REAL = Params(n=630, N=1024)
SECTION4_LEVELED = Params(n=500, N=2048)   # Section 4's leveled setting (TLWE n = 500, N-bar = 2048): CMux levels only

_lib = None


def lib_path() -> str:
    """Path of the built library (next to this file)."""
    return os.path.join(_HERE, "libshe_hip.so")


def load_library() -> C.CDLL:
    """Loads the built HIP library; builds it first only if no built library exists.
    There is no fallback: a missing or unloadable library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        from . import build as _build
        _build.build()
    # PyTorch ships its own HIP runtime under the same soname; load it first so that this
    # process holds one runtime only (two runtimes do not share the device).
    import torch  # noqa: F401
    L = C.CDLL(path)
    u8p, u32p, i8p, i32p = C.POINTER(C.c_uint8), C.POINTER(C.c_uint32), C.POINTER(C.c_int8), C.POINTER(C.c_int32)
    ctx, u64p = C.c_void_p, C.POINTER(C.c_uint64)
    sigs = {
        "she_keygen": (C.c_int, [C.POINTER(_CParams), C.c_uint64, C.c_uint32, C.POINTER(C.c_void_p)]),
        "she_free": (None, [ctx]),
        "she_encrypt_bits": (C.c_int, [ctx, u8p, C.c_size_t, C.c_uint64, u32p]),
        "she_decrypt": (C.c_int, [ctx, u32p, C.c_size_t, u8p]),
        "she_eval_gates": (C.c_int, [ctx, u8p, u32p, u32p, u32p, C.c_size_t]),
        "she_shift_acc": (C.c_int, [ctx, u32p, C.c_uint32, C.c_uint32, C.c_uint32, i8p, i8p, C.c_uint32, u32p, u64p]),
        "she_shift_acc_bias": (C.c_int, [ctx, u32p, C.c_uint32, C.c_uint32, C.c_uint32, i8p, i8p, i32p, C.c_uint32, u32p, u64p]),
        "she_plan_shift_acc_bias": (C.c_int, [C.c_uint32, C.c_uint32, C.c_uint32, i8p, i8p, i32p, C.c_uint32, C.c_int, u64p,
                                              C.POINTER(C.c_uint32), u64p]),
        "she_plan_accumulator_bits": (C.c_int, [C.c_uint32, C.c_uint32, C.c_uint32, i8p, i8p, i32p, C.POINTER(C.c_uint32)]),
        "she_relu": (C.c_int, [ctx, u32p, C.c_uint32, C.c_uint32, u32p, u64p]),
        "she_maxpool": (C.c_int, [ctx, u32p, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, u32p, u64p]),
        "she_relu_maxpool": (C.c_int, [ctx, u32p, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, u32p, u64p]),
        "she_plan_relu_maxpool": (C.c_int, [C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_int, u64p,
                                            C.POINTER(C.c_uint32), u64p]),
        "she_defer_begin": (C.c_int, [ctx]),
        "she_defer_run": (C.c_int, [ctx, u64p]),
        "she_set_option": (C.c_int, [ctx, C.c_int, C.c_int]),
        "she_get_option": (C.c_int, [ctx, C.c_int, C.POINTER(C.c_int)]),
        "she_plan_shift_acc": (C.c_int, [C.c_uint32, C.c_uint32, C.c_uint32, i8p, i8p, C.c_uint32, C.c_int, u64p,
                                         C.POINTER(C.c_uint32), u64p]),
        "she_plan_relu": (C.c_int, [C.c_uint32, C.c_uint32, C.c_int, u64p, C.POINTER(C.c_uint32), u64p]),
        "she_plan_maxpool": (C.c_int, [C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_int, u64p,
                                       C.POINTER(C.c_uint32), u64p]),
        "she_eval_mux": (C.c_int, [ctx, u32p, u32p, u32p, u32p, C.c_size_t]),
        "she_eval_circuit": (C.c_int, [ctx, u8p, u32p, u32p, u32p, C.c_size_t, u32p, u32p, C.c_size_t, u64p]),
        "she_plan_circuit": (C.c_int, [C.c_uint32, u8p, u32p, u32p, u32p, C.c_size_t, C.c_int, u64p,
                                       C.POINTER(C.c_uint32), u64p]),
        "she_eval_gates3": (C.c_int, [ctx, u8p, u32p, u32p, u32p, u32p, C.c_size_t]),
        "she_leveled_init": (C.c_int, [ctx, C.c_uint32, C.c_uint32]),
        "she_trgsw_encrypt_bits": (C.c_int, [ctx, u8p, C.c_size_t, C.c_uint64, u32p]),
        "she_trlwe_encrypt": (C.c_int, [ctx, u32p, C.c_size_t, C.c_uint64, u32p]),
        "she_trlwe_write": (C.c_int, [ctx, u32p, C.c_size_t, u32p]),
        "she_trlwe_read": (C.c_int, [ctx, u32p, C.c_size_t, u32p]),
        "she_trlwe_phase": (C.c_int, [ctx, u32p, C.c_size_t, u32p]),
        "she_eval_cmux": (C.c_int, [ctx, u32p, u32p, u32p, u32p, C.c_size_t]),
        "she_read_ct": (C.c_int, [ctx, C.c_uint32, u32p]),
        "she_write_ct": (C.c_int, [ctx, C.c_uint32, u32p]),
        "she_export_keys": (C.c_int, [ctx, u8p, u8p, u32p, u32p]),
        "she_set_stream": (C.c_int, [ctx, C.c_void_p]),
        "she_bind_pool": (C.c_int, [ctx, C.c_void_p, C.c_size_t]),
        "she_pool_bytes": (C.c_size_t, [ctx]),
        "she_eval_gates_device": (C.c_int, [ctx, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t]),
        "she_eval_gates_device_noalloc": (C.c_int, [ctx, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t]),
        "she_set_round_tracking": (C.c_int, [ctx, C.c_int]),
        "she_get_round_error": (C.c_int, [ctx, C.POINTER(C.c_double), C.c_int]),
        "she_probe_fp64_rate": (C.c_int, [ctx, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
        "she_probe_lds_rate": (C.c_int, [ctx, C.c_int, C.POINTER(C.c_double)]),
        "she_set_timing": (C.c_int, [ctx, C.c_int]),
        "she_last_timing": (C.c_int, [ctx, C.POINTER(C.c_double)]),
        "she_last_level_sizes": (C.c_int, [ctx, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.c_size_t,
                                            C.POINTER(C.c_size_t)]),
        "she_last_error": (C.c_char_p, [ctx]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


def _u8(a):
    return np.ascontiguousarray(a, dtype=np.uint8)


def _u32(a):
    return np.ascontiguousarray(a, dtype=np.uint32)


def _i8(a):
    return np.ascontiguousarray(a, dtype=np.int8)


def _p(a, ty):
    return a.ctypes.data_as(C.POINTER(ty))


OPT_FOLD_CONSTANTS = 1
OPT_NATIVE_MUX = 2
OPT_SPLIT_BELOW = 3
OPT_GATE3_CELLS = 4
OPT_COLUMN_ADDER = 8
MAJ3, XOR3 = 176, 184        # three-input gate codes; + mask (bit i complements input i)


def _options(fold: bool, native_mux: bool, cells3: bool = False, columns: bool = False) -> int:
    return ((OPT_FOLD_CONSTANTS if fold else 0) | (OPT_NATIVE_MUX if native_mux else 0) | (OPT_GATE3_CELLS if cells3 else 0)
            | (OPT_COLUMN_ADDER if columns else 0))


def _plan(rc, gates, levels):
    if rc:
        raise SheError(rc, "planning call rejected its arguments")
    return gates.value, levels.value


def _bias(bias, units):
    """int32 array [units] and its pointer, or (None, NULL)"""
    if bias is None:
        return None, None
    b = np.ascontiguousarray(bias, dtype=np.int32).reshape(units)
    return b, _p(b, C.c_int32)


def plan_shift_acc(units: int, terms: int, in_bits: int, w_sign, w_exp, acc_bits: int, fold: bool = False,
                   cells3: bool = False, columns: bool = False, bias=None):
    """(gates, levels) of she_shift_acc(_bias) for these weights; runs on the host, no GPU needed."""
    w_sign, w_exp = _i8(w_sign).reshape(units, terms), _i8(w_exp).reshape(units, terms)
    g, lv = C.c_uint64(0), C.c_uint32(0)
    keep, bp = _bias(bias, units)
    return _plan(load_library().she_plan_shift_acc_bias(units, terms, in_bits, _p(w_sign, C.c_int8), _p(w_exp, C.c_int8),
                                                        bp, acc_bits, _options(fold, False, cells3, columns), C.byref(g),
                                                        C.byref(lv), None), g, lv)


def plan_accumulator_bits(w_sign, w_exp, in_bits: int, bias=None) -> int:
    """she_plan_accumulator_bits for weights [units][terms] (leading axes are flattened into units)."""
    w_sign, w_exp = _i8(w_sign), _i8(w_exp)
    terms = w_sign.shape[-1]
    units = int(np.prod(w_sign.shape[:-1]))
    w_sign, w_exp = w_sign.reshape(units, terms), w_exp.reshape(units, terms)
    keep, bp = _bias(bias, units)
    bits = C.c_uint32(0)
    rc = load_library().she_plan_accumulator_bits(w_sign.shape[0], terms, in_bits, _p(w_sign, C.c_int8), _p(w_exp, C.c_int8),
                                                  bp, C.byref(bits))
    if rc:
        raise SheError(rc, "she_plan_accumulator_bits rejected its arguments")
    return int(bits.value)


def plan_relu(count: int, bits: int, fold: bool = False):
    g, lv = C.c_uint64(0), C.c_uint32(0)
    return _plan(load_library().she_plan_relu(count, bits, _options(fold, False), C.byref(g), C.byref(lv), None), g, lv)


def plan_maxpool(H: int, W: int, Cn: int, bits: int, fold: bool = False, native_mux: bool = False,
                 with_rotations: bool = False, cells3: bool = False):
    """(entries, levels) or, with_rotations, (entries, levels, blind rotations)."""
    g, lv, rot = C.c_uint64(0), C.c_uint32(0), C.c_uint64(0)
    rc = load_library().she_plan_maxpool(H, W, Cn, bits, _options(fold, native_mux, cells3), C.byref(g), C.byref(lv),
                                         C.byref(rot))
    out = _plan(rc, g, lv)
    return out + (rot.value,) if with_rotations else out


def plan_relu_maxpool(H: int, W: int, Cn: int, bits: int, fold: bool = False, native_mux: bool = False,
                      cells3: bool = False):
    """(entries, levels, blind rotations) of she_relu_maxpool."""
    g, lv, rot = C.c_uint64(0), C.c_uint32(0), C.c_uint64(0)
    rc = load_library().she_plan_relu_maxpool(H, W, Cn, bits, _options(fold, native_mux, cells3), C.byref(g), C.byref(lv),
                                              C.byref(rot))
    return _plan(rc, g, lv) + (rot.value,)


# operand references of eval_circuit / plan_circuit (include/she.h)
WIRE_GATE = 0x40000000
WIRE_NOT = 0x80000000
WIRE_ZERO = 0x3FFFFFFE
WIRE_ONE = 0x3FFFFFFF
CIRCUIT_MUX = 255


def plan_circuit(capacity: int, types, in0, in1, in2, fold: bool = False, native_mux: bool = False):
    """(entries, levels, blind rotations) of she_eval_circuit for this circuit; runs on the host, no GPU needed."""
    types, in0, in1, in2 = _u8(types).ravel(), _u32(in0).ravel(), _u32(in1).ravel(), _u32(in2).ravel()
    assert types.size == in0.size == in1.size == in2.size
    g, lv, rot = C.c_uint64(0), C.c_uint32(0), C.c_uint64(0)
    rc = load_library().she_plan_circuit(capacity, _p(types, C.c_uint8), _p(in0, C.c_uint32), _p(in1, C.c_uint32),
                                         _p(in2, C.c_uint32), types.size, _options(fold, native_mux), C.byref(g),
                                         C.byref(lv), C.byref(rot))
    return _plan(rc, g, lv) + (rot.value,)


class Context:
    """Owns one she_ctx.  Method names mirror the C calls (she_ prefix dropped)."""

    def __init__(self, params: Params, seed: int, pool_capacity: int, use_torch_pool: bool = True):
        self._L = load_library()
        self.params = params
        self.capacity = int(pool_capacity)
        cp = _CParams(params.n, params.N, params.k, params.bg_bit, params.l, params.ks_t, params.ks_basebit,
                      params.lwe_std, params.bk_std)
        h = C.c_void_p()
        rc = self._L.she_keygen(C.byref(cp), seed, self.capacity, C.byref(h))
        if rc:
            raise SheError(rc, (self._L.she_last_error(None) or b"").decode())
        self._h = h
        self._pool_tensor = None
        if use_torch_pool:
            import torch
            nbytes = self._L.she_pool_bytes(self._h)
            self._pool_tensor = torch.zeros(nbytes // 4, dtype=torch.int32, device="cuda")
            self._check(self._L.she_bind_pool(self._h, C.c_void_p(self._pool_tensor.data_ptr()), nbytes))
            self.set_stream(torch.cuda.current_stream().cuda_stream)

    # ---- plumbing
    def _check(self, rc: int):
        if rc:
            raise SheError(rc, (self._L.she_last_error(self._h) or b"").decode())

    def close(self):
        if getattr(self, "_h", None):
            self._L.she_free(self._h)
            self._h = None
            self._pool_tensor = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def defer_begin(self):
        self._check(self._L.she_defer_begin(self._h))

    def defer_run(self) -> int:
        """Evaluates the operators recorded since defer_begin as one circuit; returns the entries evaluated."""
        n = C.c_uint64(0)
        self._check(self._L.she_defer_run(self._h, C.byref(n)))
        return n.value

    def set_option(self, option: int, value: int):
        self._check(self._L.she_set_option(self._h, option, value))

    def get_option(self, option: int) -> int:
        v = C.c_int(0)
        self._check(self._L.she_get_option(self._h, option, C.byref(v)))
        return int(v.value)

    def set_stream(self, hip_stream: int):
        self._check(self._L.she_set_stream(self._h, C.c_void_p(hip_stream)))

    # ---- the paper's problem statement
    def encrypt_bits(self, bits, enc_seed: int, dst_ids):
        bits, dst_ids = _u8(bits).ravel(), _u32(dst_ids).ravel()
        assert bits.size == dst_ids.size
        self._check(self._L.she_encrypt_bits(self._h, _p(bits, C.c_uint8), bits.size, enc_seed, _p(dst_ids, C.c_uint32)))

    def decrypt(self, ids) -> np.ndarray:
        ids = _u32(ids)
        out = np.zeros(ids.size, np.uint8)
        self._check(self._L.she_decrypt(self._h, _p(ids.ravel(), C.c_uint32), ids.size, _p(out, C.c_uint8)))
        return out.reshape(ids.shape)

    def eval_gates(self, gtype, in0, in1, out):
        gtype, in0, in1, out = _u8(gtype).ravel(), _u32(in0).ravel(), _u32(in1).ravel(), _u32(out).ravel()
        assert gtype.size == in0.size == in1.size == out.size
        self._check(self._L.she_eval_gates(self._h, _p(gtype, C.c_uint8), _p(in0, C.c_uint32), _p(in1, C.c_uint32),
                                           _p(out, C.c_uint32), gtype.size))

    def eval_mux(self, sel, in1, in0, out):
        sel, in1, in0, out = (_u32(v).ravel() for v in (sel, in1, in0, out))
        assert sel.size == in1.size == in0.size == out.size
        self._check(self._L.she_eval_mux(self._h, _p(sel, C.c_uint32), _p(in1, C.c_uint32), _p(in0, C.c_uint32),
                                         _p(out, C.c_uint32), sel.size))

    def eval_gates3(self, gtype, in0, in1, in2, out):
        gtype = _u8(gtype).ravel()
        in0, in1, in2, out = (_u32(v).ravel() for v in (in0, in1, in2, out))
        assert gtype.size == in0.size == in1.size == in2.size == out.size
        self._check(self._L.she_eval_gates3(self._h, _p(gtype, C.c_uint8), _p(in0, C.c_uint32), _p(in1, C.c_uint32),
                                            _p(in2, C.c_uint32), _p(out, C.c_uint32), gtype.size))

    def shift_acc(self, x_ids, w_sign, w_exp, acc_bits: int, out_ids, bias=None) -> int:
        """she_shift_acc, or she_shift_acc_bias when a constant per unit is given"""
        x_ids = _u32(x_ids)
        units, terms, in_bits = x_ids.shape
        w_sign, w_exp, out_ids = _i8(w_sign), _i8(w_exp), _u32(out_ids)
        assert w_sign.shape == (units, terms) == w_exp.shape and out_ids.shape == (units, acc_bits)
        gates = C.c_uint64(0)
        if bias is None:
            self._check(self._L.she_shift_acc(self._h, _p(x_ids, C.c_uint32), units, terms, in_bits, _p(w_sign, C.c_int8),
                                              _p(w_exp, C.c_int8), acc_bits, _p(out_ids, C.c_uint32), C.byref(gates)))
        else:
            keep, bp = _bias(bias, units)
            self._check(self._L.she_shift_acc_bias(self._h, _p(x_ids, C.c_uint32), units, terms, in_bits,
                                                   _p(w_sign, C.c_int8), _p(w_exp, C.c_int8), bp, acc_bits,
                                                   _p(out_ids, C.c_uint32), C.byref(gates)))
        return gates.value

    def relu(self, x_ids, out_ids) -> int:
        x_ids, out_ids = _u32(x_ids), _u32(out_ids)
        bits = x_ids.shape[-1]
        count = x_ids.size // bits
        assert out_ids.shape == x_ids.shape
        gates = C.c_uint64(0)
        self._check(self._L.she_relu(self._h, _p(x_ids, C.c_uint32), count, bits, _p(out_ids, C.c_uint32), C.byref(gates)))
        return gates.value

    def maxpool(self, x_ids, out_ids) -> int:
        x_ids, out_ids = _u32(x_ids), _u32(out_ids)
        H, W, Cn, bits = x_ids.shape
        assert out_ids.shape == (H // 2, W // 2, Cn, bits)
        gates = C.c_uint64(0)
        self._check(self._L.she_maxpool(self._h, _p(x_ids, C.c_uint32), H, W, Cn, bits, _p(out_ids, C.c_uint32),
                                        C.byref(gates)))
        return gates.value

    def eval_circuit(self, types, in0, in1, in2, out_refs, out_ids) -> int:
        """A whole circuit in one call (references as in include/she.h); returns the entries evaluated."""
        types, in0, in1, in2 = _u8(types).ravel(), _u32(in0).ravel(), _u32(in1).ravel(), _u32(in2).ravel()
        out_refs, out_ids = _u32(out_refs).ravel(), _u32(out_ids).ravel()
        assert types.size == in0.size == in1.size == in2.size and out_refs.size == out_ids.size
        n = C.c_uint64(0)
        self._check(self._L.she_eval_circuit(self._h, _p(types, C.c_uint8), _p(in0, C.c_uint32), _p(in1, C.c_uint32),
                                             _p(in2, C.c_uint32), types.size, _p(out_refs, C.c_uint32),
                                             _p(out_ids, C.c_uint32), out_ids.size, C.byref(n)))
        return n.value

    def relu_maxpool(self, x_ids, out_ids) -> int:
        x_ids, out_ids = _u32(x_ids), _u32(out_ids)
        H, W, Cn, bits = x_ids.shape
        assert out_ids.shape == (H // 2, W // 2, Cn, bits)
        gates = C.c_uint64(0)
        self._check(self._L.she_relu_maxpool(self._h, _p(x_ids, C.c_uint32), H, W, Cn, bits, _p(out_ids, C.c_uint32),
                                             C.byref(gates)))
        return gates.value

    # ---- leveled mode
    def leveled_init(self, trgsw_capacity: int, trlwe_capacity: int):
        self._check(self._L.she_leveled_init(self._h, trgsw_capacity, trlwe_capacity))

    def trgsw_encrypt_bits(self, bits, seed: int, dst_ids):
        bits, dst_ids = _u8(bits).ravel(), _u32(dst_ids).ravel()
        assert bits.size == dst_ids.size
        self._check(self._L.she_trgsw_encrypt_bits(self._h, _p(bits, C.c_uint8), bits.size, seed, _p(dst_ids, C.c_uint32)))

    def trlwe_encrypt(self, mu, seed: int, dst_ids):
        mu, dst_ids = _u32(mu).reshape(-1, self.params.N), _u32(dst_ids).ravel()
        assert mu.shape[0] == dst_ids.size
        self._check(self._L.she_trlwe_encrypt(self._h, _p(mu, C.c_uint32), dst_ids.size, seed, _p(dst_ids, C.c_uint32)))

    def trlwe_write(self, samples, dst_ids):
        samples, dst_ids = _u32(samples).reshape(-1, 2, self.params.N), _u32(dst_ids).ravel()
        assert samples.shape[0] == dst_ids.size
        self._check(self._L.she_trlwe_write(self._h, _p(samples, C.c_uint32), dst_ids.size, _p(dst_ids, C.c_uint32)))

    def trlwe_read(self, ids) -> np.ndarray:
        ids = _u32(ids).ravel()
        out = np.zeros((ids.size, 2, self.params.N), np.uint32)
        self._check(self._L.she_trlwe_read(self._h, _p(ids, C.c_uint32), ids.size, _p(out, C.c_uint32)))
        return out

    def trlwe_phase(self, ids) -> np.ndarray:
        ids = _u32(ids).ravel()
        out = np.zeros((ids.size, self.params.N), np.uint32)
        self._check(self._L.she_trlwe_phase(self._h, _p(ids, C.c_uint32), ids.size, _p(out, C.c_uint32)))
        return out

    def eval_cmux(self, sel, in1, in0, out):
        sel, in1, in0, out = (_u32(v).ravel() for v in (sel, in1, in0, out))
        assert sel.size == in1.size == in0.size == out.size
        self._check(self._L.she_eval_cmux(self._h, _p(sel, C.c_uint32), _p(in1, C.c_uint32), _p(in0, C.c_uint32),
                                          _p(out, C.c_uint32), sel.size))

    # ---- diagnostics
    def read_ct(self, idx: int) -> np.ndarray:
        out = np.zeros(self.params.n + 1, np.uint32)
        self._check(self._L.she_read_ct(self._h, idx, _p(out, C.c_uint32)))
        return out

    def write_ct(self, idx: int, ct):
        ct = _u32(ct)
        assert ct.size == self.params.n + 1
        self._check(self._L.she_write_ct(self._h, idx, _p(ct, C.c_uint32)))

    def read_cts(self, ids) -> np.ndarray:
        return np.stack([self.read_ct(int(i)) for i in np.asarray(ids).ravel()])

    def export_keys(self):
        P = self.params
        lwe, ring = np.zeros(P.n, np.uint8), np.zeros(P.N, np.uint8)
        bk = np.zeros((P.n, 2, P.l, 2, P.N), np.uint32)
        ks = np.zeros((P.N, P.ks_t, (1 << P.ks_basebit) - 1, P.n + 1), np.uint32)
        self._check(self._L.she_export_keys(self._h, _p(lwe, C.c_uint8), _p(ring, C.c_uint8), _p(bk, C.c_uint32),
                                            _p(ks, C.c_uint32)))
        return lwe, ring, bk, ks

    def eval_gates_device(self, d_type, d_in0, d_in1, d_out, ngates: int):
        """Device pointers (ints); enqueues without validation or synchronisation."""
        self._check(self._L.she_eval_gates_device(self._h, C.c_void_p(d_type), C.c_void_p(d_in0), C.c_void_p(d_in1),
                                                  C.c_void_p(d_out), ngates))

    def eval_gates_device_noalloc(self, d_type, d_in0, d_in1, d_out, ngates: int):
        """eval_gates_device with the level's scratch in the library's static device buffer: allocates nothing."""
        self._check(self._L.she_eval_gates_device_noalloc(self._h, C.c_void_p(d_type), C.c_void_p(d_in0),
                                                          C.c_void_p(d_in1), C.c_void_p(d_out), ngates))

    def set_round_tracking(self, on: bool):
        self._check(self._L.she_set_round_tracking(self._h, int(on)))

    def get_round_error(self, reset: bool = True) -> float:
        v = C.c_double(0)
        self._check(self._L.she_get_round_error(self._h, C.byref(v), int(reset)))
        return v.value

    def probe_fp64_rate(self, form: int) -> dict:
        ns, tf = C.c_double(0), C.c_double(0)
        self._check(self._L.she_probe_fp64_rate(self._h, form, C.byref(ns), C.byref(tf)))
        return {"ns_per_instruction_per_simd": ns.value, "tflops_as_fma": tf.value}

    def probe_lds_rate(self, form: int) -> float:
        """bytes per nanosecond and compute unit (see include/she_diag.h)"""
        v = C.c_double(0)
        self._check(self._L.she_probe_lds_rate(self._h, form, C.byref(v)))
        return v.value

    def set_timing(self, on: bool):
        self._check(self._L.she_set_timing(self._h, int(on)))

    def last_timing(self) -> dict:
        ms = (C.c_double * 4)()
        self._check(self._L.she_last_timing(self._h, ms))
        return {"lincomb_ms": ms[0], "blind_rotate_ms": ms[1], "key_switch_ms": ms[2], "levels": int(ms[3])}

    def last_level_sizes(self):
        """(gates, muxes): entries per level of the last circuit, in the order the levels ran."""
        n = C.c_size_t(0)
        self._check(self._L.she_last_level_sizes(self._h, None, None, 0, C.byref(n)))
        gates, muxes = np.zeros(n.value, np.uint64), np.zeros(n.value, np.uint64)
        if n.value:
            self._check(self._L.she_last_level_sizes(self._h, gates.ctypes.data_as(C.POINTER(C.c_uint64)),
                                                     muxes.ctypes.data_as(C.POINTER(C.c_uint64)), n.value, None))
        return gates, muxes
