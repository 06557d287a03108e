"""The pins have teeth: a mistake planted in a copy of the oracle (on the CPU) fails its pin.

Each case edits one expression of ``oracle/wagma_oracle.c`` in a temporary copy, compiles it
with the oracle's own flags and runs one pin from ``test_oracle_pins`` against it.
"""
import ctypes
import os
import subprocess

import pytest

from oracle import wagma_oracle as orc
import test_oracle_pins as pins
import test_oracle_lag_pins as lag_pins

SRC = os.path.join(os.path.dirname(os.path.abspath(orc.__file__)), "wagma_oracle.c")

MUTATIONS = [
    ("late divisor S instead of S+1",
     "/ (float)(S + 1);", "/ (float)(S);", pins.test_stale_rule_hand_value),
    ("sign of the learning rate",
     "fmaf(-lr, m_new, w[at])", "fmaf(lr, m_new, w[at])", pins.test_local_update_hand_value),
    ("cumulative mask in Algorithm 1",
     "        for (int p = 0; p < P; ++p) {\n            int partner = p ^ (1 << bit);",
     "        static int mask; if (phase == 0) mask = 1; mask <<= bit;\n"
     "        for (int p = 0; p < P; ++p) {\n            int partner = p ^ mask;",
     pins.test_alg1_printed_example_p8_s4),
    ("momentum line not fused",
     "float m_new = fmaf(mu, m[at], g[at]);", "float m_new = mu * m[at] + g[at];",
     pins.test_update_lines_are_fused),
    ("global iteration on t mod tau",
     "((t + 1) % tau) == 0", "(t % tau) == 0", pins.test_global_iteration_predicate),
    ("left-to-right sum",
     "float right = tree_sum_f32(c + count / 2, count / 2);",
     "float right = 0; for (int i = count / 2; i < count; ++i) left += c[i];",
     pins.test_sum_is_a_pairwise_tree_in_member_order),
    ("late member contributes W' instead of its send buffer",
     "contrib[e] = mask_bit(stale_mask, p) ? pub[(int64_t)p * ld + j] : w_prime[p];", "contrib[e] = w_prime[p];",
     pins.test_stale_rule_hand_value),
    ("reciprocal multiply for 1/(S+1)",
     "w[(int64_t)p * ld + j] = (w_sum + w_prime[p]) / (float)(S + 1);",
     "w[(int64_t)p * ld + j] = (w_sum + w_prime[p]) * (1.0f / (float)(S + 1));",
     pins.test_stale_divisor_is_a_true_division),
    ("member digits in reverse phase order",
     "p |= 1 << bits[r];\n            table", "p |= 1 << bits[log2_S - 1 - r];\n            table",
     pins.test_alg1_phase_bits_wrap_order),
    ("send buffer gets W instead of W'",
     "        for (int i = 0; i < P; ++i)\n            pub[(int64_t)i * ld + j] = w_prime[i];",
     "        for (int i = 0; i < P; ++i)\n            pub[(int64_t)i * ld + j] = w[(int64_t)i * ld + j];",
     pins.test_stale_rule_hand_value),
    ("global average ignores half of the replicas",
     "float avg = tree_sum_f32(w_prime, P) * (1.0f / (float)P);",
     "float avg = 2.0f * tree_sum_f32(w_prime, P / 2 ? P / 2 : 1) * (1.0f / (float)P);",
     pins.test_snapshot_script_p4_s2_f32),
    ("late divisor S instead of S+1 in the function with the third state",
     "w[at] = (w_sum + w_prime[p]) / (float)(S + 1);", "w[at] = (w_sum + w_prime[p]) / (float)(S);",
     lag_pins.test_no_busy_process_is_algorithm_2_as_printed),
    ("send buffer gets W instead of W' in the function with the third state",
     "            if (global || !mask_bit(busy_mask, i))\n                pub[(int64_t)i * ld + j] = w_prime[i];",
     "            if (global || !mask_bit(busy_mask, i))\n                pub[(int64_t)i * ld + j] = w[(int64_t)i * ld + j];",
     lag_pins.test_no_busy_process_is_algorithm_2_as_printed),
    ("global sum over half the replicas in the function with the third state",
     "float sum = tree_sum_f32(w_prime, P);", "float sum = 2.0f * tree_sum_f32(w_prime, P / 2 ? P / 2 : 1);",
     lag_pins.test_no_busy_process_is_algorithm_2_as_printed),
    ("a process that is still computing contributes W' instead of its send buffer",
     "contrib[e] = (mask_bit(stale_mask, p) || mask_bit(busy_mask, p))\n"
     "                                     ? pub[(int64_t)p * ld + j] /* send buffer */",
     "contrib[e] = mask_bit(stale_mask, p)\n"
     "                                     ? pub[(int64_t)p * ld + j] /* send buffer */",
     lag_pins.test_busy_member_hand_value),
    ("a process that is still computing receives the average",
     "continue; /* the sum waits in its receive buffer, unread */", ";",
     lag_pins.test_busy_member_hand_value),
    ("a process that is still computing takes its local step",
     "continue; /* still computing: nothing of this process changes */", ";",
     lag_pins.test_snapshot_with_a_step_spanning_two_iterations),
    ("a global iteration leaves out the processes of the busy mask",
     "if (!global && mask_bit(busy_mask, i))\n                continue; /* still",
     "if (mask_bit(busy_mask, i))\n                continue; /* still",
     lag_pins.test_busy_wins_over_late_and_a_global_iteration_waits_for_everybody),
    ("late if finished before the next activation, not before the next read",
     "finish[first] > next_activated + tolerance_ms", "finish[first] > next_activated",
     lag_pins.test_lag_states_hand_timeline_with_tolerance),
    ("a process in time begins its next step when it finishes, not when the allreduce is done",
     "finish[p] = taken + next_ms[p];", "finish[p] += next_ms[p];",
     lag_pins.test_lag_states_hand_timeline_with_tolerance),
    ("a late process does not activate the next allreduce",
     "            if (finish[first] < next_activated)\n                next_activated = finish[first];",
     "",
     lambda: lag_pins.test_lag_states_against_an_event_queue(8, 5, 6, 30)),
]


@pytest.mark.parametrize("name,old,new,pin", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(name, old, new, pin, tmp_path, monkeypatch):
    text = open(SRC).read()
    assert text.count(old) >= 1, "the oracle no longer contains the expression this case edits"
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new, 1))
    lib = tmp_path / "mutant.so"
    subprocess.run(["gcc", *orc.CFLAGS, "-o", str(lib), str(src), "-lm"], check=True)
    monkeypatch.setattr(orc, "_lib", orc.bind(ctypes.CDLL(str(lib))))
    with pytest.raises(AssertionError):
        pin()
    monkeypatch.undo()
    pin()     # and the real oracle passes it
