"""MI355X-native batched bootstrapped TFHE gates and SHE layer operators (arXiv 1906.00148).

Thin ctypes binding over the C ABI in include/she.h.  Every step of the path runs in the HIP
library; this package only marshals arguments.  PyTorch is used for the pool's device memory
and for the stream the kernels run on.
"""
from .binding import (CIRCUIT_MUX, GATES, OPT_COLUMN_ADDER, MAJ3, WIRE_GATE, WIRE_NOT, WIRE_ONE, WIRE_ZERO, plan_circuit, OPT_GATE3_CELLS, OPT_FOLD_CONSTANTS, OPT_NATIVE_MUX, OPT_SPLIT_BELOW, REAL, SECTION4_LEVELED, TOY, XOR3,  # noqa: F401
                      Context, Params, SheError, lib_path, load_library, plan_maxpool, plan_relu, plan_relu_maxpool, plan_shift_acc,
                      plan_accumulator_bits)
