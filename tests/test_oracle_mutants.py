"""Every planted mistake in a copy of the oracle must fail at least one pin.

The mistakes are planted on the CPU, in temporary copies of the oracle's C and
Python sources; the real oracle is untouched."""
import os
import types

import pytest

from oracle import slowmo_oracle as O

import oracle_pins as P

C_SRC = open(os.path.join(os.path.dirname(O.__file__), "slowmo_oracle.c")).read()
PY_SRC = open(O.__file__).read()

# (name, old, new, occurrence)   occurrence: which match of `old` to replace
C_MUTANTS = [
    ("sgd_h_sign", "REAL hn = mu * h[j] + grad;", "REAL hn = mu * h[j] - grad;", 0),
    ("sgd_dir_uses_old_h", "REAL dir = mu * hn + grad;", "REAL dir = mu * h[j] + grad;", 0),
    ("sgd_dir_drops_grad", "REAL dir = mu * hn + grad;", "REAL dir = mu * hn;", 0),
    ("sgd_h_drops_mu", "REAL hn = mu * h[j] + grad;", "REAL hn = h[j] + grad;", 0),
    ("sgd_no_weight_decay", "(REAL)g[j] + wd * x[j]", "(REAL)g[j]", 0),
    ("sgd_decoupled_decay_sign", "(REAL)g[j] + wd * x[j]", "(REAL)g[j] - wd * x[j]", 0),
    ("sgd_step_sign", "x[j] = x[j] - lr * dir;", "x[j] = x[j] + lr * dir;", 0),
    ("sgd_step_drops_lr", "x[j] = x[j] - lr * dir;", "x[j] = x[j] - dir;", 0),
    ("adam_h_no_one_minus_b1", "(one - b1) * grad", "grad", 0),
    ("adam_v_not_squared", "(one - b2) * gsq", "(one - b2) * grad", 0),
    ("adam_v_uses_b1", "b2 * v[j]", "b1 * v[j]", 0),
    ("adam_exponent_plus_one", "R_POW(b1, (REAL)l)", "R_POW(b1, (REAL)(l + 1))", 0),
    ("adam_exponent2_plus_one", "R_POW(b2, (REAL)l)", "R_POW(b2, (REAL)(l + 1))", 0),
    ("adam_eps_inside_root", "(R_SQRT(vhat) + eps)", "R_SQRT(vhat + eps)", 0),
    ("adam_no_bias_correction_h", "REAL hhat = hn / c1;", "REAL hhat = hn;", 0),
    ("adam_bias_swapped", "REAL vhat = vn / c2;", "REAL vhat = vn / c1;", 0),
    ("adam_no_root", "R_SQRT(vhat)", "vhat", 0),
    ("adam_step_sign", "x[j] = x[j] - lr * dir;", "x[j] = x[j] + lr * dir;", 1),
    ("adam_v_not_stored", "v[j] = vn;", "v[j] = v[j];", 0),
    ("outer_no_division_by_m", "REAL xbar = s / (REAL)m;", "REAL xbar = s;", 0),
    ("outer_drops_last_worker", "for (int i = 1; i < m; ++i)", "for (int i = 1; i < m - 1; ++i)", 0),
    ("outer_diff_sign", "REAL diff = x0[j] - xbar;", "REAL diff = xbar - x0[j];", 0),
    ("outer_u_no_inverse_lr", "beta * u[j] + diff / lr", "beta * u[j] + diff", 0),
    ("outer_u_times_lr", "beta * u[j] + diff / lr", "beta * u[j] + diff * lr", 0),
    ("outer_u_drops_beta", "beta * u[j] + diff / lr", "u[j] + diff / lr", 0),
    ("outer_x_drops_alpha", "(alpha * lr) * un", "lr * un", 0),
    ("outer_x_drops_lr", "(alpha * lr) * un", "alpha * un", 0),
    ("outer_x_sign", "x0[j] - (alpha * lr) * un", "x0[j] + (alpha * lr) * un", 0),
    ("outer_u_not_stored", "u[j] = un;", "u[j] = u[j];", 0),
    ("outer_broadcasts_mean", "xw[(int64_t)i * d + j] = xn;", "xw[(int64_t)i * d + j] = xbar;", 0),
    ("outer_no_broadcast", "xw[(int64_t)i * d + j] = xn;", ";", 0),
    ("average_no_division", "REAL mean = s / (REAL)m;", "REAL mean = s;", 0),
    ("average_drops_last_worker", "for (int i = 1; i < m; ++i)", "for (int i = 1; i < m - 1; ++i)", 1),
    ("average_not_written_back", "bw[(int64_t)i * d + j] = mean;", ";", 0),
    ("average_writes_sum", "bw[(int64_t)i * d + j] = mean;", "bw[(int64_t)i * d + j] = s;", 0),
    ("mix_uses_receiver_share", "if (j != i) v = v + share[j] * old[j];", "if (j != i) v = v + share[i] * old[j];", 0),
    ("mix_in_place_hazard", "if (j != i) v = v + share[j] * old[j];", "if (j != i) v = v + share[j] * xw[(int64_t)j * d + e];", 0),
    ("mix_weights_not_mixed", "if (j != i) w[i] = w[i] + share[j] * wold[j];", ";", 0),
    ("mix_counts_self_loops", "if (i != j && in_peer[i] == j) ++outdeg;", "if (in_peer[i] == j) ++outdeg;", 0),
    ("mix_drops_own_share", "REAL v = share[i] * old[i];", "REAL v = old[i];", 0),
    ("outer_transposed_replicas", "s = s + xw[(int64_t)i * d + j];", "s = s + xw[(int64_t)j * m + i];", 0),
]

PY_MUTANTS = [
    ("policy_never_reset", 'if self.policy == "reset":', "if False:", 0),
    ("policy_always_reset", 'if self.policy == "reset":', "if True:", 0),
    ("reset_keeps_v", "                self.v[...] = 0\n", "                pass\n", 0),
    ("reset_keeps_step_count", "                self.v[...] = 0\n            self.l = 0\n",
     "                self.v[...] = 0\n", 0),
    ("policy_only_first_iteration", "if self.k == 0:", "if self.k == 0 and self.t == 0:", 0),
    ("policy_every_step", "if self.k == 0:", "if True:", 0),
    ("sgd_all_workers_use_grad0", "_ptr(self.h[i][a:b]), _ptr(g[i][a:b]), b - a,",
     "_ptr(self.h[i][a:b]), _ptr(g[0][a:b]), b - a,", 0),
    ("sgd_workers_share_h", "_ptr(self.x[i][a:b]), _ptr(self.h[i][a:b]), _ptr(g[i][a:b]), b - a,",
     "_ptr(self.x[i][a:b]), _ptr(self.h[0][a:b]), _ptr(g[i][a:b]), b - a,", 0),
    ("adam_all_workers_use_grad0", "_ptr(g[i][a:b]), b - a, lr_j, self.beta1,",
     "_ptr(g[0][a:b]), b - a, lr_j, self.beta1,", 0),
    ("outer_alpha_beta_swapped", "lr, self.alpha, self.beta)", "lr, self.beta, self.alpha)", 0),
    ("average_skips_v", "            if self.v is not None:\n                self.lib.oracle_average_buffers(_ptr(self.v), self.m, self.d)\n", "", 0),
    ("average_skips_h", "            self.lib.oracle_average_buffers(_ptr(self.h), self.m, self.d)\n", "            pass\n", 0),
    ("average_resets_step_count", '        elif self.policy == "average":\n', '        elif self.policy == "average":\n            self.l = 0\n', 0),
    ("noaverage_shares_x0", "_ptr(self.x0[i][a:b]), _ptr(self.u[i][a:b]),", "_ptr(self.x0[0][a:b]), _ptr(self.u[i][a:b]),", 0),
    ("noaverage_shares_u", "_ptr(self.x0[i][a:b]), _ptr(self.u[i][a:b]),", "_ptr(self.x0[i][a:b]), _ptr(self.u[0][a:b]),", 0),
    ("noaverage_only_worker0", "            for i in range(self.m):\n                for a, b, lr_j, _ in self._groups(lr):", "            for i in range(1):\n                for a, b, lr_j, _ in self._groups(lr):", 0),
    ("expgraph_sends_forward", "return ((np.arange(m) - hop) % m)", "return ((np.arange(m) + hop) % m)", 0),
    ("expgraph_hop_linear", "hop = 1 << (step % n_hops)", "hop = 1 + (step % n_hops)", 0),
    ("groups_ignore_lr_scale", "np.float32(lr) * np.float32(s)", "np.float32(lr)", 0),
    ("groups_ignore_tensor_wd", "lr_j, self.momentum, wd_j)", "lr_j, self.momentum, self.weight_decay)", 0),
    ("groups_outer_uses_global_lr", "_ptr(self.u[a:b]), lr_j, self.alpha, self.beta)", "_ptr(self.u[a:b]), lr, self.alpha, self.beta)", 0),
    ("groups_outer_not_copied_back", "                self.x[:, a:b] = xs\n", "", 0),
    ("schedule_milestone_one_step_late", "passed = sum(1 for ms in milestones if step >= ms)",
     "passed = sum(1 for ms in milestones if step > ms)", 0),
    ("schedule_factor_applied_once", "return base_lr * factor ** passed",
     "return base_lr * factor ** min(passed, 1)", 0),
    ("schedule_warmup_starts_at_zero", "return start_lr + (base_lr - start_lr) * step / warmup_steps",
     "return base_lr * step / warmup_steps", 0),
    ("schedule_warmup_ends_one_step_early", "return start_lr + (base_lr - start_lr) * step / warmup_steps",
     "return start_lr + (base_lr - start_lr) * (step + 1) / warmup_steps", 0),
    ("schedule_inverse_not_root", "return peak_lr * (warmup_steps / step) ** 0.5 if step > 0 else peak_lr",
     "return peak_lr * (warmup_steps / step) if step > 0 else peak_lr", 0),
    ("schedule_inverse_sqrt_of_step_only", "return peak_lr * (warmup_steps / step) ** 0.5 if step > 0 else peak_lr",
     "return peak_lr * (1.0 / step) ** 0.5 if step > 0 else peak_lr", 0),
    ("schedule_inverse_warmup_ignores_init", "return init_lr + (peak_lr - init_lr) * step / warmup_steps",
     "return peak_lr * step / warmup_steps", 0),
    ("pushsum_weights_not_reset_at_exact_average",
     "            self.w[...] = 1     # all mass is shared equally again after the exact average\n",
     "            pass\n", 0),
    ("pushsum_weights_reset_without_the_average",
     "        if self.exact_average:\n            self.w[...] = 1", "        if True:\n            self.w[...] = 1", 0),
    ("expgraph_period_log2_m", "np.floor(np.log2(m - 1))", "np.floor(np.log2(m))", 0),
    ("expgraph_one_hop_too_many", "int(np.floor(np.log2(m - 1))) + 1", "int(np.floor(np.log2(m - 1))) + 2", 0),
    ("outer_averages_debiased_points",
     "        if self.exact_average and self.bounds is None:\n",
     "        if self.exact_average and self.bounds is None and not np.all(self.w == 1):\n"
     "            self.x[...] = self.debiased()\n"
     "        if self.exact_average and self.bounds is None:\n", 0),
    ("default_policy_swapped", 'policy = "reset" if base == "sgd_nesterov" else "maintain"',
     'policy = "maintain" if base == "sgd_nesterov" else "reset"', 0),
]


def _replace_nth(src, old, new, n):
    pos = -1
    for _ in range(n + 1):
        pos = src.find(old, pos + 1)
        assert pos >= 0, f"mutation target not found: {old!r}"
    return src[:pos] + new + src[pos + len(old):]


def _killed(make):
    """Names of the pins that fail for this (mutated) oracle."""
    killed = []
    for pin in P.ALL_PINS:
        try:
            pin(make)
        except AssertionError:
            killed.append(pin.__name__)
    return killed


@pytest.mark.parametrize("name,old,new,nth", C_MUTANTS, ids=[m[0] for m in C_MUTANTS])
def test_c_mutant_is_caught(tmp_path, name, old, new, nth):
    src = tmp_path / "mutant.c"
    src.write_text(_replace_nth(C_SRC, old, new, nth))
    lib_path = str(tmp_path / "libmutant_f64.so")
    O.build(force=True, src=str(src), out={"f64": lib_path})
    lib = O.load("f64", path=lib_path)
    killed = _killed(lambda x, **kw: O.SlowMoOracle(x, prec="f64", lib=lib, **kw))
    assert killed, f"no pin notices the planted mistake '{name}'"


@pytest.mark.parametrize("name,old,new,nth", PY_MUTANTS, ids=[m[0] for m in PY_MUTANTS])
def test_python_mutant_is_caught(name, old, new, nth):
    mod = types.ModuleType("oracle_mutant")
    mod.__file__ = O.__file__
    exec(compile(_replace_nth(PY_SRC, old, new, nth), O.__file__, "exec"), mod.__dict__)
    killed = _killed(lambda x, **kw: mod.SlowMoOracle(x, prec="f64", **kw))
    assert killed, f"no pin notices the planted mistake '{name}'"


def test_unmutated_oracle_passes_every_pin():
    assert _killed(lambda x, **kw: O.SlowMoOracle(x, prec="f64", **kw)) == []
