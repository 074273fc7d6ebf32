"""Do the pins hold the oracle in place?  Each case plants one plausible mistake in the oracle's
source (a dropped term, a wrong sign or index, a swapped operand), on the CPU, and demands that
at least one pin test fails.  A mistake the pins cannot see would mean the oracle could be wrong
there without anyone noticing."""
import contextlib
import inspect
import types

import pytest

import oracle.adamw
import oracle.brute
import oracle.policy
import oracle.proto
from tests import test_oracle_adamw as TA
from tests import test_oracle_policy as TP
from tests import test_oracle_proto as TR


def _functions(ns_or_module):
    """name -> function for module-level functions and methods of classes defined there."""
    items = ns_or_module if isinstance(ns_or_module, dict) else vars(ns_or_module)
    out = {}
    for name, obj in items.items():
        if isinstance(obj, types.FunctionType):
            out[name] = obj
        elif isinstance(obj, type):
            for mname, m in vars(obj).items():
                if isinstance(m, types.FunctionType):
                    out[name + "." + mname] = m
    return out


@contextlib.contextmanager
def planted(module, old, new):
    src = inspect.getsource(module)
    assert src.count(old) == 1, "mutation site must be unique: %r" % old
    ns = {"__name__": module.__name__, "__package__": module.__package__, "__file__": module.__file__}
    exec(compile(src.replace(old, new), module.__file__, "exec"), ns)
    live = {k: f for k, f in _functions(module).items() if f.__module__ == module.__name__}
    mutated = _functions(ns)
    saved = {}
    try:
        for k, f in live.items():
            c0, c1 = f.__code__, mutated[k].__code__ if k in mutated else None
            if c1 is not None and (c0.co_code, c0.co_consts, c0.co_names, c0.co_varnames) != \
                    (c1.co_code, c1.co_consts, c1.co_names, c1.co_varnames):
                saved[k] = f.__code__
                f.__code__ = mutated[k].__code__
        assert saved, "the mutation changed no code"
        yield
    finally:
        for k, code in saved.items():
            live[k].__code__ = code


POLICY_PINS = [TP.test_walkthrough_example_printed_by_the_paper, TP.test_advancement_matches_its_definition,
               TP.test_boundary_extension_matches_its_definition, TP.test_eq1_heavy_attrition_64_replicas,
               TP.test_promotion_needs_a_spare_of_the_same_role,
               TP.test_spare_stays_masked_when_the_minor_fails_without_a_minor_spare,
               TP.test_lost_spare_changes_nothing_but_the_epoch, TP.test_no_survivor,
               TP.test_adaptive_strawman_shrinks_the_batch, TR.test_tiny_schedule_quotas_and_ids]
PROTO_PINS = [TR.test_tiny_schedule_quotas_and_ids,
              lambda: TR.test_iteration_gradient_is_the_mean_over_committed_ids(__import__("numpy").float64, 1e-15),
              lambda: TR.test_each_committed_microbatch_enters_exactly_once(0),
              lambda: TR.test_each_committed_microbatch_enters_exactly_once(2),
              TR.test_promoted_spare_contributes_its_own_microbatches_after_rewind,
              TR.test_spare_is_masked_out_of_the_sum,
              TR.test_constant_gradient_closed_form_and_constant_divisor,
              TR.test_adaptive_policy_commits_fewer_than_B,
              TR.test_restore_after_partial_microbatch_equals_never_started,
              TR.test_failure_run_equals_clean_replay_bit_for_bit, TR.test_bf16_inputs_widen_exactly,
              TR.test_first_microbatch_overwrites_like_zero_then_add, TR.test_protocol_violations_are_errors,
              TR.test_rewind_drops_completed_microbatches_from_the_audit,
              TR.test_inplace_reduction_leaves_the_sum_in_every_survivor,
              TR.test_reduction_under_an_older_epoch_cannot_be_committed]
ADAMW_PINS = [TA.test_against_torch_adamw_fp64, TA.test_first_step_closed_form_without_decay,
              TA.test_zero_gradient_is_pure_decay, TA.test_decay_is_decoupled_from_the_moments]


def caught(pins):
    for pin in pins:
        try:
            pin()
        except KeyboardInterrupt:
            raise
        except BaseException:                       # pytest's own failure signals included
            return True
    return False


P, R, A, Bm = oracle.policy, oracle.proto, oracle.adamw, oracle.brute
CASES = [
    # --- policy (Alg. 6, 7, Record) ---
    (P, "while C_cur + W_cur * G_ext < B:", "while C_cur + W_cur * G_ext <= B:", POLICY_PINS),
    (P, "n_bdry = W_cur * G_ext - (B - C_cur)", "n_bdry = W_cur * G_ext - (B + C_cur)", POLICY_PINS),
    (P, "while W_cur * G < B:", "while W_cur * G <= B:", POLICY_PINS),
    (P, "n_maj = B // G_cur", "n_maj = B // G_cur - 1", POLICY_PINS),
    (P, "R_cur = B - n_maj * G_cur", "R_cur = B - n_maj", POLICY_PINS),
    (P, "n_mi = 1 if (n_min == 1 and spare >= 2) else 0", "n_mi = 1 if (n_min == 1 and spare >= 1) else 0", POLICY_PINS),
    (P, "n_ms = spare - n_mi", "n_ms = spare", POLICY_PINS),
    (P, "self.eps += 1", "self.eps += 0", POLICY_PINS),
    (P, "want = MAJOR_SPARE if role == MAJOR else MINOR_SPARE", "want = MINOR_SPARE if role == MAJOR else MAJOR_SPARE",
     POLICY_PINS),
    (P, "self.target[r] += G_ext - 1", "self.target[r] += G_ext", POLICY_PINS),
    (P, "self.loop_bound += G_ext", "self.loop_bound += G_ext - 1", POLICY_PINS),
    (P, "planned = sum(self.target[r] for r in con)", "planned = sum(self.target[r] for r in self.alive())", POLICY_PINS),
    (P, "[MAJOR] * lay[\"n_maj\"] + [MINOR] * lay[\"n_min\"] +", "[MINOR] * lay[\"n_min\"] + [MAJOR] * lay[\"n_maj\"] +",
     POLICY_PINS),
    (P, "return [r for r in range(self.W_init) if self.role[r] in (MAJOR, MINOR)]",
     "return [r for r in range(self.W_init) if self.role[r] != DEAD]", POLICY_PINS + PROTO_PINS),
    (P, "self.restore_mode = RESTORE_NONBLOCKING", "self.restore_mode = RESTORE_BLOCKING", POLICY_PINS),
    (P, "return self.role[r] != DEAD and self.contributed[r] < self.target[r]",
     "return self.role[r] != DEAD and self.contributed[r] <= self.target[r]", PROTO_PINS),
    # --- protocol simulator (Alg. 1, 2, 5) ---
    (R, "self.acc[r][lo:hi] = self.dtype.type(0) + gb", "self.acc[r][lo:hi] = self.acc[r][lo:hi] + gb", PROTO_PINS),
    (R, "self.acc[r][lo:hi] = self.acc[r][lo:hi] + gb", "self.acc[r][lo:hi] = self.acc[r][lo:hi] - gb", PROTO_PINS),
    (R, "members = [r for r in w.contributors() if self.cnt[r][b] > 0]",
     "members = [r for r in w.alive() if self.cnt[r][b] > 0]", PROTO_PINS),
    (R, "self.grad_out[lo:hi] = total / self.dtype.type(divisor)",
     "self.grad_out[lo:hi] = total / self.dtype.type(len(members) * w.G_init)", PROTO_PINS),
    (R, "total = self.acc[r][lo:hi].copy() if first else total + self.acc[r][lo:hi]",
     "total = self.acc[r][lo:hi].copy() if first else total", PROTO_PINS),
    (R, "and (not stale_only or self.snap_eps[q][b] < w.eps)]", "and (not stale_only or self.snap_eps[q][b] <= w.eps - 2)]",
     PROTO_PINS),
    (R, "self.cnt[q][b] = self.snap_cnt[q][b]", "self.cnt[q][b] = self.cnt[q][b]", PROTO_PINS),
    (R, "self.acc[q][lo:hi] = self.snap[q][lo:hi]", "self.snap[q][lo:hi] = self.acc[q][lo:hi]", PROTO_PINS),
    (R, "del self.ids[q][done:]", "del self.ids[q][done + 1:]", PROTO_PINS),
    (R, "for r in w.alive():\n                    self.acc[r][lo:hi] = total",
     "for r in members:\n                    self.acc[r][lo:hi] = total", PROTO_PINS),
    (R, "if self.red_eps[b] != w.eps or self.red_dirty[b] or self.red_total[b] != want:",
     "if self.red_eps[b] != w.eps or self.red_dirty[b]:", PROTO_PINS),
    (R, "if self.red_eps[b] != w.eps or self.red_dirty[b] or self.red_total[b] != want:",
     "if self.red_dirty[b] or self.red_total[b] != want:", PROTO_PINS),
    (R, "self.snap_cnt[q][b] = self.cnt[q][b]", "self.snap_cnt[q][b] = 0", PROTO_PINS),
    # --- brute-force definition ---
    (Bm, "out[i] = math.fsum(float(c[i]) for c in cols) / B", "out[i] = math.fsum(float(c[i]) for c in cols) / len(cols) * 1.0001",
     PROTO_PINS),
    # --- AdamW ---
    (A, "p = p - lr * weight_decay * p", "p = p + lr * weight_decay * p", ADAMW_PINS),
    (A, "m = beta1 * m + (1.0 - beta1) * g", "m = beta1 * m + (1.0 - beta2) * g", ADAMW_PINS),
    (A, "v = beta2 * v + (1.0 - beta2) * (g * g)", "v = beta2 * v + (1.0 - beta2) * g", ADAMW_PINS),
    (A, "m_hat = m / (1.0 - beta1 ** t)", "m_hat = m", ADAMW_PINS),
    (A, "v_hat = v / (1.0 - beta2 ** t)", "v_hat = v / (1.0 - beta2 ** (t + 1))", ADAMW_PINS),
    (A, "p = p - lr * m_hat / (np.sqrt(v_hat) + eps)", "p = p - lr * m_hat / np.sqrt(v_hat + eps)", ADAMW_PINS),
    (A, "p = p - lr * m_hat / (np.sqrt(v_hat) + eps)", "p = p + lr * m_hat / (np.sqrt(v_hat) + eps)", ADAMW_PINS),
]


@pytest.mark.filterwarnings("ignore::RuntimeWarning")          # a planted mistake may take sqrt of a negative
@pytest.mark.parametrize("case", range(len(CASES)))
def test_planted_mistake_is_caught(case):
    module, old, new, pins = CASES[case]
    assert not caught(pins), "pins must pass on the unmodified oracle"
    with planted(module, old, new):
        assert caught(pins), "no pin notices: %s -> %s" % (old, new)
    assert not caught(pins), "oracle restored"
