"""Are the oracle's pins sharp?  Each case plants one plausible mistake in the oracle (on the CPU, by
monkeypatching one of its functions) and checks that at least one of the pin tests then fails.
With no mistake planted every pin passes (the other test files)."""
import numpy as np
import pytest

import oracle
import oracle.formatting as fmt
import oracle.optim as opt
import oracle.plan as pln

import test_oracle_format as tf
import test_oracle_lars as tl
import test_oracle_optim as to
import test_oracle_plan as tp

f64 = np.float64


def _fails(tests):
    """True if at least one of the (callable, args) pins raises."""
    for fn, args in tests:
        try:
            fn(*args)
        except (AssertionError, ValueError, IndexError, ZeroDivisionError, FloatingPointError):
            return True
    return False


ADAM_PINS = [(to.test_adam_constant_gradient_closed_form, ()), (to.test_adam_matches_torch_float64, (0.0,)),
             (to.test_adam_matches_torch_float64, (0.01,)), (to.test_adam_zero_gradient_leaves_state_alone, ())]
MOM_PINS = [(to.test_momentum_constant_gradient_closed_form, ()), (to.test_momentum_mu_zero_is_plain_sgd_with_l2, ()),
            (to.test_momentum_matches_torch_float64, ())]
LAMB_PINS = [(to.test_lamb_update_norm_equals_lr_times_weight_norm, ()),
             (to.test_lamb_first_step_without_decay_is_a_scaled_sign_step, ()),
             (to.test_lamb_decay_only_closed_form, ()), (to.test_lamb_single_element_by_hand, ()),
             (to.test_lamb_without_adaptation_is_adamw, (0.01,)), (to.test_lamb_zero_norm_means_ratio_one, ()),
             (to.test_lamb_no_decay_flag_drops_only_the_decay_term, ()),
             (to.test_sharded_lamb_equals_unsharded, ("ragged",)),
             (to.test_lamb_partials_mask_padding_by_position_not_by_value, ())]
LARS_PINS = [(tl.test_first_step_moves_by_lr_times_trust_times_weight_norm, ()), (tl.test_single_element_by_hand, ()),
             (tl.test_without_adaptation_is_momentum_sgd, (5e-5,)), (tl.test_flags_and_zero_norms, ()),
             (tl.test_decay_enters_the_denominator, ()), (tl.test_sharded_equals_unsharded, ([0, 1, 5, 6, 7, 64, 1001, 3], 6)),
             (tl.test_partials_mask_padding_by_position, ())]
PLAN_PINS = [(tp.test_paper_shape_examples, row) for row in tp._golden_rows()] + \
            [(tp.test_invariants_random_lists, (a,)) for a in (1, 8)] + [(tp.test_brute_force_element_ownership, ())]
FORMAT_PINS = [(tf.test_round_trip_random_bit_patterns, (8,)), (tf.test_single_replica_no_align_is_plain_concatenation, ()),
               (tf.test_against_the_layout_equation_element_by_element, ()),
               (tf.test_padding_is_positive_zero_bits_and_sits_at_the_tail, ()),
               (tf.test_format_reads_only_its_own_piece, ()), (tf.test_unshard_ignores_pad_contents, ()),
               (tf.test_bf16_rounding_hand_worked_cases, ()), (tf.test_bf16_rounding_matches_torch_on_random_patterns, ()),
               (tf.test_bf16_format_variants_round_trip, ())]


# ---- mutants of the optimizer arithmetic --------------------------------------------------------

def _adam_mutant(kind):
    def step(w, g, m, v, hp, t):
        lr, b1, b2, eps = f64(hp["lr"]), f64(hp["beta1"]), f64(hp["beta2"]), f64(hp["eps"])
        wd = f64(hp.get("weight_decay", 0.0))
        w, g, m, v = opt._up(w, g, m, v)
        if wd != 0.0 and kind != "no_decay":
            g = g + wd * w
        m = b1 * m + (1.0 - b1) * g
        v = (b1 if kind == "beta_swap" else b2) * v + (1.0 - b2) * g * g
        bc1 = 1.0 if kind == "no_bias_correction" else 1.0 - b1 ** t
        bc2 = 1.0 - b2 ** (t - 1 if kind == "t_off_by_one" and t > 1 else t)
        m_hat, v_hat = m / bc1, v / bc2
        if kind == "eps_inside_sqrt":
            upd = m_hat / np.sqrt(v_hat + eps)
        else:
            upd = m_hat / (np.sqrt(v_hat) + eps)
        w = w + lr * upd if kind == "sign" else w - lr * upd
        return w.astype(np.float32), m.astype(np.float32), v.astype(np.float32)
    return step


@pytest.mark.parametrize("kind", ["sign", "beta_swap", "no_bias_correction", "t_off_by_one", "no_decay"])
def test_adam_mutants_are_caught(monkeypatch, kind):
    mutant = _adam_mutant(kind)
    monkeypatch.setattr(opt, "adam_step", mutant)
    monkeypatch.setattr(to, "adam_step", mutant)
    assert _fails(ADAM_PINS)


def test_adam_eps_placement_is_pinned_by_a_large_eps():
    # eps inside the square root only shows when eps is not negligible; the torch pin uses eps = 1e-8, so check here.
    hp = dict(to.ADAM, eps=1e-3)
    w = np.array([0.5], np.float32); g = np.array([0.25], np.float32); z = np.zeros(1, np.float32)
    w1, _, _ = oracle.adam_step(w, g, z, z, hp, 1)
    assert abs(float(w1[0]) - (0.5 - 1e-3 * 0.25 / (0.25 + 1e-3))) < 1e-7
    wrong, _, _ = _adam_mutant("eps_inside_sqrt")(w, g, z, z, hp, 1)
    assert abs(float(wrong[0]) - float(w1[0])) > 1e-6


def _momentum_mutant(kind):
    def step(w, g, m, hp):
        lr, mu, wd = f64(hp["lr"]), f64(hp["mu"]), f64(hp.get("weight_decay", 0.0))
        w, g, m = opt._up(w, g, m)
        gp = g if kind == "no_decay" else g + wd * w
        m = mu * m + ((1.0 - mu) * gp if kind == "dampening" else gp)
        w = w - lr * (gp + mu * m if kind == "nesterov" else m)
        return w.astype(np.float32), m.astype(np.float32)
    return step


@pytest.mark.parametrize("kind", ["no_decay", "dampening", "nesterov"])
def test_momentum_mutants_are_caught(monkeypatch, kind):
    mutant = _momentum_mutant(kind)
    monkeypatch.setattr(opt, "momentum_step", mutant)
    monkeypatch.setattr(to, "momentum_step", mutant)
    assert _fails(MOM_PINS)


def _lamb_direction_mutant(kind):
    def direction(w, g, m, v, hp, t, decay):
        b1, b2, eps = f64(hp["beta1"]), f64(hp["beta2"]), f64(hp["eps"])
        wd = f64(hp.get("weight_decay", 0.0)) if (decay or kind == "ignore_no_decay") else f64(0.0)
        m = b1 * m + (1.0 - b1) * g
        v = b2 * v + (1.0 - b2) * g * g
        m_hat = m / (1.0 - b1 ** t)
        v_hat = v if kind == "no_v_correction" else v / (1.0 - b2 ** t)
        u = m_hat / (np.sqrt(v_hat) + eps)
        if kind == "decay_on_gradient":
            u = u + wd * g
        elif kind != "drop_decay":
            u = u + wd * w
        return m, v, u
    return direction


@pytest.mark.parametrize("kind", ["drop_decay", "decay_on_gradient", "no_v_correction", "ignore_no_decay"])
def test_lamb_direction_mutants_are_caught(monkeypatch, kind):
    monkeypatch.setattr(opt, "_lamb_direction", _lamb_direction_mutant(kind))
    assert _fails(LAMB_PINS)


@pytest.mark.parametrize("kind", ["inverted", "squared", "always_one", "zero_norm_gives_zero"])
def test_lamb_trust_ratio_mutants_are_caught(monkeypatch, kind):
    def ratio(sum_w2, sum_u2, adapt):
        if not adapt:
            return 1.0
        wn, un = np.sqrt(f64(sum_w2)), np.sqrt(f64(sum_u2))
        if not (wn > 0.0 and un > 0.0):
            return 0.0 if kind == "zero_norm_gives_zero" else 1.0
        return {"inverted": float(un / wn), "squared": float(sum_w2 / sum_u2), "always_one": 1.0,
                "zero_norm_gives_zero": float(wn / un)}[kind]
    monkeypatch.setattr(opt, "_trust_ratio", ratio)
    assert _fails(LAMB_PINS)


def test_lamb_partials_that_forget_the_mask_are_caught(monkeypatch):
    real = opt.lamb_shard_partials

    def unmasked(plan, r, w, g, m, v, hp, t, flags=None):
        m_out, v_out, u_out, partial = real(plan, r, w, g, m, v, hp, t, flags)
        w64 = np.asarray(w, np.float64)
        for i in range(plan.V):
            seg = slice(plan.off[i], plan.off[i] + plan.L[i])
            partial[i, 0] = np.sum(w64[seg] ** 2); partial[i, 1] = np.sum(u_out[seg] ** 2)
        return m_out, v_out, u_out, partial
    monkeypatch.setattr(to, "lamb_shard_partials", unmasked)
    assert _fails(LAMB_PINS)


@pytest.mark.parametrize("kind", ["no_decay_in_denominator", "inverted", "lr_outside_momentum_wrongly", "ignore_flags"])
def test_lars_mutants_are_caught(monkeypatch, kind):
    def local_lr(sum_w2, sum_g2, wd, hp, adapt):
        if not adapt and kind != "ignore_flags":
            return 1.0
        wn, gn = np.sqrt(f64(sum_w2)), np.sqrt(f64(sum_g2))
        if not (wn > 0.0 and gn > 0.0):
            return 1.0
        tc = f64(hp["trust_coeff"])
        if kind == "inverted":
            return float(tc * gn / (wn + wd * gn))
        return float(tc * wn / (gn + (0.0 if kind == "no_decay_in_denominator" else wd * wn)))

    def apply(w, g, m, llr, wd, hp):
        lr, mu = f64(hp["lr"]), f64(hp["mu"])
        if kind == "lr_outside_momentum_wrongly":
            m = mu * m + llr * (g + wd * w)
            return w - lr * lr * m, m
        m = mu * m + lr * llr * (g + wd * w)
        return w - m, m
    monkeypatch.setattr(opt, "_lars_local_lr", local_lr)
    monkeypatch.setattr(opt, "_lars_apply", apply)
    assert _fails(LARS_PINS)


# ---- mutants of the layout ----------------------------------------------------------------------

@pytest.mark.parametrize("kind", ["floor_instead_of_ceil", "no_align_round_up", "offsets_not_cumulative", "pad_up_front"])
def test_plan_mutants_are_caught(monkeypatch, kind):
    def make_plan(numel, N, align=8):
        if N < 1 or align < 1 or (align & (align - 1)):
            raise ValueError
        L, off, pos = [], [], 0
        for n in numel:
            n = int(n)
            if n < 0:
                raise ValueError
            per = n // N if kind == "floor_instead_of_ceil" else -(-n // N)
            length = per if kind == "no_align_round_up" else -(-per // align) * align
            if kind == "pad_up_front":
                length += align
            L.append(length); off.append(0 if kind == "offsets_not_cumulative" else pos); pos += length
        return pln.Plan(tuple(int(n) for n in numel), int(N), int(align), tuple(L), tuple(off), pos, tuple(L))
    monkeypatch.setattr(tp, "make_plan", make_plan)
    assert _fails(PLAN_PINS)


@pytest.mark.parametrize("kind", ["wrong_replica_offset", "pad_with_ones", "reads_past_piece", "unshard_wrong_row"])
def test_format_mutants_are_caught(monkeypatch, kind):
    def shard_format(plan, r, flats, dst=None):
        src_is_bf16 = len(flats) > 0 and flats[0].dtype == np.uint16
        if dst is None:
            dst = "bf16" if src_is_bf16 else "f32"
        out = np.zeros(plan.S, dtype=np.uint16 if dst == "bf16" else np.uint32)
        if kind == "pad_with_ones":
            out[:] = 0x3F80 if dst == "bf16" else 0x3F800000
        for i, flat in enumerate(flats):
            start = (r + 1) * plan.L[i] if kind == "wrong_replica_offset" else r * plan.L[i]
            real = max(0, min(plan.L[i], plan.numel[i] - start))
            if kind == "reads_past_piece":
                real = max(0, min(plan.L[i] + 1, plan.numel[i] - start, plan.S - plan.off[i]))
            if real > 0:
                out[plan.off[i]:plan.off[i] + real] = fmt._convert(flat[start:start + real], dst).view(out.dtype)
        return out if dst == "bf16" else out.view(np.float32)

    def unshard_format(plan, gathered, dst=None):
        src_is_bf16 = gathered.dtype == np.uint16
        if dst is None:
            dst = "bf16" if src_is_bf16 else "f32"
        flats = []
        for i in range(plan.V):
            flat = np.zeros(plan.numel[i], dtype=np.uint16 if dst == "bf16" else np.float32)
            for r in range(plan.N):
                start, real = r * plan.L[i], plan.real_count(i, r)
                row = (r + 1) % plan.N if kind == "unshard_wrong_row" else r
                if real > 0:
                    flat[start:start + real] = fmt._convert(gathered[row, plan.off[i]:plan.off[i] + real], dst)
            flats.append(flat)
        return flats
    if kind == "unshard_wrong_row":
        monkeypatch.setattr(tf, "unshard_format", unshard_format)
    else:
        monkeypatch.setattr(tf, "shard_format", shard_format)
    assert _fails(FORMAT_PINS)


@pytest.mark.parametrize("kind", ["truncate", "round_half_up", "round_half_away"])
def test_bf16_rounding_mutants_are_caught(monkeypatch, kind):
    def to_bf16(x):
        bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
        if kind == "truncate":
            r = bits >> 16
        else:
            r = (bits + 0x8000) >> 16            # ties always up in magnitude
        return (r & 0xFFFF).astype(np.uint16)
    monkeypatch.setattr(tf, "f32_to_bf16_bits", to_bf16)
    monkeypatch.setattr(fmt, "f32_to_bf16_bits", to_bf16)
    assert _fails(FORMAT_PINS)


# ---- mutants of the replica-array arithmetic -----------------------------------------------------

import oracle.topology as topo  # noqa: E402
import test_oracle_topology as tt  # noqa: E402
from fractions import Fraction  # noqa: E402

TOPO_PINS = [(tt.test_papers_subgroup_example, (row,)) for row in tt._golden("rowgroup")] + \
            [(tt.test_papers_pod_example, row) for row in tt._golden("groups")] + \
            [(tt.test_partial_sharding_equals_the_full_all_reduce_piece, rc) for rc in ((2, 4), (4, 6))] + \
            [(tt.test_two_phase_shard_id_by_simulation, rc) for rc in ((2, 3), (3, 5))] + \
            [(tt.test_degenerate_arrays, ())] + \
            [(tt.test_memory_model_hand_worked, row) for row in tt._golden("memory")] + \
            [(tt.test_memory_model_properties, ())] + \
            [(tt.test_concat_partition_tiles_the_concatenation, (13, 4)), (tt.test_combined_all_reduce_ignores_tensor_boundaries, ())]


@pytest.mark.parametrize("kind", ["column_major_ids", "groups_are_columns", "shard_id_is_row"])
def test_partial_sharding_mutants_are_caught(monkeypatch, kind):
    def partial_sharding(rows, cols, replica):
        topo._check_array(rows, cols, replica)
        if kind == "column_major_ids":
            col, row = divmod(replica, rows)
            return row, col, [j * rows + row for j in range(cols)], [col * rows + i for i in range(rows)]
        row, col = divmod(replica, cols)
        sg, rg = [row * cols + j for j in range(cols)], [i * cols + col for i in range(rows)]
        if kind == "groups_are_columns":
            return col, row, rg, sg
        return row, row, sg, rg                                  # shard_id_is_row
    monkeypatch.setattr(tt, "partial_sharding", partial_sharding)
    assert _fails(TOPO_PINS)


@pytest.mark.parametrize("kind", ["row_major", "column_phase_first"])
def test_two_phase_mutants_are_caught(monkeypatch, kind):
    def two_phase(rows, cols, replica):
        topo._check_array(rows, cols, replica)
        i, j = divmod(replica, cols)
        return i * cols + j if kind == "row_major" else i + j * cols
    monkeypatch.setattr(tt, "two_phase_shard_id", two_phase)
    assert _fails(TOPO_PINS)


@pytest.mark.parametrize("kind", ["no_floor_of_full_state", "activations_not_counted", "weights_sharded_too", "sum_not_max"])
def test_memory_model_mutants_are_caught(monkeypatch, kind):
    def peak_memory(W, V, P, N):
        if N < 1:
            raise ValueError
        W, V, P = Fraction(W), Fraction(V), Fraction(P)
        a, b = W + V / N + P, W + V
        if kind == "no_floor_of_full_state":
            return W + V + P, a
        if kind == "activations_not_counted":
            return W + V + P, max(W + V / N, b)
        if kind == "weights_sharded_too":
            return W + V + P, max(W / N + V / N + P, b)
        return W + V + P, a + b
    monkeypatch.setattr(tt, "peak_memory", peak_memory)
    assert _fails(TOPO_PINS)


@pytest.mark.parametrize("kind", ["floor_pieces", "respects_nothing_but_overlaps"])
def test_concat_partition_mutants_are_caught(monkeypatch, kind):
    def concat_partition(total, parts, part):
        piece = total // parts if kind == "floor_pieces" else -(-total // parts)
        start = part * piece if kind == "floor_pieces" else max(0, min(part * piece, total) - 1)
        return start, min(piece, total - start)
    monkeypatch.setattr(tt, "concat_partition", concat_partition)
    assert _fails(TOPO_PINS)


# ---- mutants of Adafactor ------------------------------------------------------------------------

import oracle.adafactor as ada  # noqa: E402
import test_oracle_adafactor as ta  # noqa: E402

ADAFACTOR_PINS = [(ta.test_schedule_values, ()), (ta.test_two_by_two_matrix_by_hand, ()),
                  (ta.test_vector_by_hand_with_clipping_on_the_second_step, ()),
                  (ta.test_rank_one_gradient_first_step_is_a_sign_step, (1.0, 1.0)),
                  (ta.test_rank_one_gradient_first_step_is_a_sign_step, (0.5, 0.5)),
                  (ta.test_factored_estimate_keeps_the_row_and_column_sums, ()),
                  (ta.test_update_size_and_invariances, ()), (ta.test_against_torch_adafactor_float64, (5,)),
                  (ta.test_sharded_equals_unsharded, ([(9, 6), (5, 1), (4, 16)], 4, 8))]


@pytest.mark.parametrize("kind", ["constant_beta2", "rho_uncapped", "rho_not_decaying", "beta2_exponent_sign"])
def test_adafactor_schedule_mutants_are_caught(monkeypatch, kind):
    def schedule(t, hp):
        e = ada._hp(hp, "decay_exponent")
        beta2 = f64(0.999) if kind == "constant_beta2" else f64(1.0) - f64(t) ** (e if kind == "beta2_exponent_sign" else -e)
        rho = f64(1.0) / np.sqrt(f64(t)) if kind == "rho_uncapped" else min(ada._hp(hp, "max_rho"), f64(1.0) / np.sqrt(f64(t)))
        if kind == "rho_not_decaying":
            rho = ada._hp(hp, "max_rho")
        return beta2, rho
    monkeypatch.setattr(ada, "adafactor_schedule", schedule)
    monkeypatch.setattr(ta, "adafactor_schedule", schedule)
    assert _fails(ADAFACTOR_PINS)


@pytest.mark.parametrize("kind", ["no_division_by_sum", "mean_instead_of_sum", "eps1_dropped", "rows_and_columns_swapped",
                                  "eps1_added_once_per_row"])
def test_adafactor_second_moment_mutants_are_caught(monkeypatch, kind):
    def second_moment(G, R, C, beta2, eps1):
        G = np.asarray(G, f64)
        term = G * G + (0.0 if kind == "eps1_dropped" else eps1)
        if G.shape[1] == 1:
            R = beta2 * R + (1.0 - beta2) * term[:, 0]
            return R, C, R[:, None]
        if kind == "rows_and_columns_swapped" and G.shape[0] == G.shape[1]:
            R = beta2 * R + (1.0 - beta2) * term.sum(axis=0)
            C = beta2 * C + (1.0 - beta2) * term.sum(axis=1)
        else:
            rs = (G * G).sum(axis=1) + eps1 if kind == "eps1_added_once_per_row" else term.sum(axis=1)
            R = beta2 * R + (1.0 - beta2) * rs
            C = beta2 * C + (1.0 - beta2) * term.sum(axis=0)
        if kind == "no_division_by_sum":
            return R, C, np.outer(R, C)
        if kind == "mean_instead_of_sum":
            return R, C, np.outer(R, C) / R.mean()
        return R, C, np.outer(R, C) / R.sum()
    monkeypatch.setattr(ada, "adafactor_second_moment", second_moment)
    monkeypatch.setattr(ta, "adafactor_second_moment", second_moment)
    pins = ADAFACTOR_PINS
    if kind == "eps1_added_once_per_row":            # only visible where eps1 matters: make it large
        pins = [(_eps1_counts_every_element, ())]
    assert _fails(pins)


def _eps1_counts_every_element():
    # with eps1 far above g^2 the row term is cols * eps1 and the column term rows * eps1
    G = np.zeros((3, 5))
    R, C, _ = ada.adafactor_second_moment(G, np.zeros(3), np.zeros(5), 0.0, 2.0)
    assert R.tolist() == [10.0] * 3 and C.tolist() == [6.0] * 5


def test_eps1_counts_every_element():
    _eps1_counts_every_element()


@pytest.mark.parametrize("kind", ["no_eps2_floor", "clip_with_min", "rms_is_a_norm", "sign", "no_clipping",
                                  "step_not_relative", "rms_of_new_weights"])
def test_adafactor_step_mutants_are_caught(monkeypatch, kind):
    def step(shapes, ws, gs, Rs, Cs, hp, t):
        beta2, rho = ada.adafactor_schedule(t, hp)
        eps1, eps2, d = ada._hp(hp, "eps1"), ada._hp(hp, "eps2"), ada._hp(hp, "clip_threshold")
        out_w, out_R, out_C = [], [], []
        for (rows, cols), w, g, R, C in zip(shapes, ws, gs, Rs, Cs):
            n = rows * cols
            if n == 0:
                out_w.append(np.asarray(w, np.float32).copy()); out_R.append(np.asarray(R, np.float32).copy())
                out_C.append(np.asarray(C, np.float32).copy())
                continue
            X, G = ada._up(w).reshape(rows, cols), ada._up(g).reshape(rows, cols)
            R, C, Vhat = ada.adafactor_second_moment(G, ada._up(R), ada._up(C), beta2, eps1)
            U = G / np.sqrt(Vhat)
            rms_u = np.sqrt(np.sum(U * U)) if kind == "rms_is_a_norm" else np.sqrt(np.sum(U * U) / n)
            if kind == "clip_with_min":
                U_hat = U / min(f64(1.0), rms_u / d)
            elif kind == "no_clipping":
                U_hat = U
            else:
                U_hat = U / max(f64(1.0), rms_u / d)
            rms_x = np.sqrt(np.sum(X * X) / n)
            alpha = (rms_x if kind == "no_eps2_floor" else max(eps2, rms_x)) * rho
            if kind == "step_not_relative":
                alpha = rho
            X_new = X + alpha * U_hat if kind == "sign" else X - alpha * U_hat
            if kind == "rms_of_new_weights":
                X_new = X - max(eps2, np.sqrt(np.sum(X_new * X_new) / n)) * rho * U_hat
            out_w.append(X_new.reshape(-1).astype(np.float32)); out_R.append(R.astype(np.float32)); out_C.append(C.astype(np.float32))
        return out_w, out_R, out_C
    monkeypatch.setattr(ta, "adafactor_unsharded_step", step)
    assert _fails(ADAFACTOR_PINS)


@pytest.mark.parametrize("kind", ["forgets_the_row_mask", "sum_R_without_decay"])
def test_adafactor_sharding_mutants_are_caught(monkeypatch, kind):
    if kind == "forgets_the_row_mask":
        def piece(plan, r, i, x64):
            Lr, cols = plan.Lr[i], plan.cols[i]
            return x64[plan.off[i]:plan.off[i] + Lr * cols].reshape(Lr, cols), np.ones(Lr, bool)
        monkeypatch.setattr(ada, "_piece", piece)
    else:
        orig = ada.adafactor_shard_partials

        def partials(plan, r, w, g, R_rows, hp):
            a, b, table = orig(plan, r, w, g, R_rows, hp)
            table[:, 1] = 0.0                         # the old row state's sum is left out of the all-reduce
            return a, b, table
        monkeypatch.setattr(ta, "adafactor_shard_partials", partials)
    assert _fails([(ta.test_sharded_equals_unsharded, ([(9, 6), (5, 1), (4, 16)], 4, 8)),
                   (ta.test_sharded_equals_unsharded, ([(10, 3), (0, 5), (7, 1), (3, 0), (1, 8)], 3, 1))])
