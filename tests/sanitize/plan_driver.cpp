// Runs the library's host-only calls (netlist builders, folding rules, level scheduling, accumulator sizing, argument
// checks) once; the whole library is built for this with the host sanitizers (-fsanitize=address,undefined on the
// host side only) by tests/test_sanitizers.py.  No GPU call is made.  Prints one line per planning call so that the
// test can compare the figures with those of the ordinary build.
#include <cstdint>
#include <cstdio>
#include <vector>

#include "she.h"

int main()
{
    int bad = 0;
    uint64_t gates = 0, rot = 0;
    uint32_t levels = 0;
    // one unit of 9 terms and one of 5 with every option combination that exists, with and without constants
    const int8_t sign[18] = {1, -1, 1, 1, -1, 1, -1, -1, 1, 1, 1, -1, 1, 1, -1, -1, 1, 1};
    const int8_t exp[18] = {0, -1, -7, -2, 0, -3, 0, -6, -1, -4, 0, 0, -2, -5, -1, 0, -3, -2};
    const int32_t bias[2] = {1000, -77};
    const int modes[5] = {0, 1, 4, 5, 13};
    for (int m = 0; m < 5; m++)
        for (int withb = 0; withb < 2; withb++) {
            int rc = she_plan_shift_acc_bias(2, 9, 8, sign, exp, withb ? bias : nullptr, 16, modes[m], &gates, &levels, &rot);
            std::printf("shift_acc mode %d bias %d: rc %d gates %llu levels %u rotations %llu\n", modes[m], withb, rc,
                        (unsigned long long)gates, levels, (unsigned long long)rot);
            bad += rc != SHE_OK;
        }
    // 576 terms: the single-neuron benchmark's shape
    std::vector<int8_t> s576(576), e576(576);
    for (int t = 0; t < 576; t++) { s576[t] = (t * 7) % 3 ? 1 : -1; e576[t] = (int8_t)(-(t % 8)); }
    for (int m : {0, 5, 13}) {
        bad += she_plan_shift_acc(1, 576, 8, s576.data(), e576.data(), 16, m, &gates, &levels, &rot) != SHE_OK;
        std::printf("neuron mode %d: gates %llu levels %u\n", m, (unsigned long long)gates, levels);
    }
    uint32_t bits = 0;
    bad += she_plan_accumulator_bits(2, 9, 8, sign, exp, bias, &bits) != SHE_OK;
    std::printf("accumulator bits %u\n", bits);
    for (int m : {0, 1, 2, 3, 7}) {
        bad += she_plan_relu(33, 16, m, &gates, &levels, &rot) != SHE_OK;
        std::printf("relu mode %d: gates %llu levels %u\n", m, (unsigned long long)gates, levels);
        bad += she_plan_maxpool(5, 4, 3, 9, m, &gates, &levels, &rot) != SHE_OK;
        std::printf("maxpool mode %d: gates %llu levels %u rotations %llu\n", m, (unsigned long long)gates, levels,
                    (unsigned long long)rot);
        bad += she_plan_relu_maxpool(6, 6, 2, 12, m, &gates, &levels, &rot) != SHE_OK;
        std::printf("relu_maxpool mode %d: gates %llu levels %u\n", m, (unsigned long long)gates, levels);
    }
    // a small circuit with every kind of entry and reference
    const uint8_t ty[6] = {SHE_XOR, SHE_MAJ3 + 2, SHE_CIRCUIT_MUX, SHE_AND, SHE_XOR3, SHE_ORNY};
    const uint32_t a[6] = {0, 1, SHE_WIRE_GATE | 0, SHE_WIRE_ONE, SHE_WIRE_GATE | 2, SHE_WIRE_GATE | 4 | SHE_WIRE_NOT};
    const uint32_t b[6] = {1, 2, SHE_WIRE_GATE | 1, SHE_WIRE_GATE | 2, 3, SHE_WIRE_GATE | 4};
    const uint32_t c[6] = {0, SHE_WIRE_GATE | 0, 3, 0, SHE_WIRE_ZERO, 0};
    for (int m : {1, 3}) {
        bad += she_plan_circuit(8, ty, a, b, c, 6, m, &gates, &levels, &rot) != SHE_OK;
        std::printf("circuit mode %d: gates %llu levels %u rotations %llu\n", m, (unsigned long long)gates, levels,
                    (unsigned long long)rot);
    }
    // argument checks: each must refuse without touching memory it should not
    bad += she_plan_circuit(8, ty, a, b, c, 6, 0, &gates, &levels, &rot) != SHE_EINVAL;          // complement without folding
    const uint32_t fwd[1] = {SHE_WIRE_GATE | 0};
    bad += she_plan_circuit(8, ty, fwd, b, c, 1, 1, &gates, &levels, &rot) != SHE_EINVAL;         // refers to itself
    const uint32_t far[1] = {8};
    bad += she_plan_circuit(8, ty, far, b, c, 1, 1, &gates, &levels, &rot) != SHE_ERANGE;         // id outside the pool
    const int8_t badexp[1] = {-8};
    bad += she_plan_shift_acc(1, 1, 8, sign, badexp, 16, 0, &gates, &levels, &rot) != SHE_EINVAL;
    bad += she_plan_shift_acc(1, 1, 8, sign, exp, 7, 0, &gates, &levels, &rot) != SHE_EINVAL;     // accumulator narrower than the inputs
    bad += she_plan_shift_acc(1, 2, 8, sign, exp, 16, 8, &gates, &levels, &rot) != SHE_EINVAL;    // columns without folding and cells
    bad += she_plan_relu(1, 1, 0, &gates, &levels, &rot) != SHE_EINVAL;
    bad += she_plan_accumulator_bits(1, 1, 8, sign, exp, nullptr, nullptr) != SHE_EINVAL;
    // no context: every computing call refuses a null handle
    bad += she_eval_gates(nullptr, ty, a, b, c, 1) != SHE_EINVAL;
    bad += she_decrypt(nullptr, a, 1, nullptr) != SHE_EINVAL;
    she_free(nullptr);
    std::printf("host calls under sanitizers: failures %d\n", bad);
    return bad ? 1 : 0;
}
