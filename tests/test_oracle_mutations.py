"""The pins must be able to fail: plant plausible mistakes in the oracle (on the CPU) and check a pin trips.

Each mutation swaps one oracle function for a subtly wrong variant (a transposed operand, a wrong
rounding mode, a dropped term, the wrong scale index) and re-runs one pinned test, which must fail.
"""
import numpy as np
import pytest

from oracle import svdq_oracle as O
import tests.test_oracle_layer as TL
import tests.test_oracle_quantizer as TQ
import tests.test_oracle_gptq as TG


def _must_fail(fn):
    with pytest.raises(AssertionError):
        fn()


def test_wrong_rounding_mode_is_caught(monkeypatch):
    real = np.rint
    monkeypatch.setattr(O.np, "rint", lambda a: np.sign(a) * np.floor(np.abs(a) + 0.5))   # half away from zero
    _must_fail(TQ.test_round_half_to_even_ties_from_golden_file)
    monkeypatch.setattr(O.np, "rint", real)
    TQ.test_round_half_to_even_ties_from_golden_file()


def test_unrounded_scale_is_caught(monkeypatch):
    def bad(v):
        v = np.ascontiguousarray(v, dtype=np.float32)
        vg = v.reshape(v.shape[:-1] + (v.shape[-1] // 64, 64))
        s = np.max(np.abs(vg), axis=-1) / np.float32(7)          # scale never rounded to 16 bit
        q = np.clip(np.rint(vg / np.where(s > 0, s, 1)[..., None]), -7, 7).astype(np.int8)
        return q.reshape(v.shape), s.astype(np.float16)
    monkeypatch.setattr(O, "quantize_groups", bad)
    _must_fail(TQ.test_bruteforce_against_exact_rationals)


def test_column_scaling_instead_of_row_scaling_is_caught(monkeypatch):
    monkeypatch.setattr(O, "smooth_weight", lambda W, lam: np.asarray(W, np.float64) * np.asarray(lam, np.float64)[: W.shape[1]][None, :])
    _must_fail(TL.test_smoothing_leaves_the_product_unchanged_and_moves_outliers)


def test_sigma_split_mistake_is_caught(monkeypatch):
    def bad(W_hat, r):
        U, S, Vt = np.linalg.svd(W_hat, full_matrices=False)
        return U[:, :r] * np.sqrt(S[:r]), np.sqrt(S[:r])[:, None] * Vt[:r], S      # Sigma split between factors
    monkeypatch.setattr(O, "lowrank_svd", bad)
    _must_fail(TL.test_lowrank_matches_eckart_young_and_known_factors)


def test_dropped_lowrank_term_and_wrong_scale_index_are_caught(monkeypatch):
    real_forward = O.forward
    monkeypatch.setattr(O, "forward", lambda xb, P, **kw: real_forward(xb, P, **{**kw, "lowrank": False}))
    _must_fail(TL.test_forward_equals_plain_definition_of_eq5)
    monkeypatch.setattr(O, "forward", real_forward)

    def bad_quantize_residual(R):            # groups taken along N instead of K
        q, s = O.quantize_groups(np.asarray(R, np.float64).astype(np.float32))
        return q, np.ascontiguousarray(np.repeat(s, 64, axis=1)[: R.shape[0] // 64, :])
    monkeypatch.setattr(O, "quantize_residual", bad_quantize_residual)
    _must_fail(TL.test_prepare_residual_identity_and_ranges)


def test_transposed_group_sum_is_caught(monkeypatch):
    real = O.group_sums
    monkeypatch.setattr(O, "group_sums", lambda qx, qw: real(qx, np.ascontiguousarray(qw[::-1])))
    _must_fail(TL.test_group_sums_against_integer_loops_and_extremes)


def test_adapter_applied_to_the_smoothed_input_is_caught(monkeypatch):
    real = O.append_lora

    def bad(prep, down, up, scale=1.0, rank_multiple=16):      # treats the adapter like L1 instead of like L1s
        return real(prep, np.asarray(down, np.float32) * prep["rinv"][:, None], up, scale, rank_multiple)
    monkeypatch.setattr(O, "append_lora", bad)
    _must_fail(TL.test_lora_appended_to_the_lowrank_branch_adds_x_down_up_and_nothing_else)


def test_fp4_mistakes_are_caught(monkeypatch):
    from oracle import svdq_fp4_oracle as F
    import tests.test_oracle_fp4 as TF
    real_round, real_scale = F.round_e2m1, F.block_scale_byte

    def away(y):                                  # ties away from zero instead of to even
        y = np.asarray(y, np.float32)
        a = np.minimum(np.abs(y), 6).astype(np.float64)
        idx = np.argmin(np.abs(a[..., None] - F.E2M1.astype(np.float64))[..., ::-1], axis=-1)
        return ((7 - idx) + 8 * (y < 0)).astype(np.uint8)
    monkeypatch.setattr(F, "round_e2m1", away)
    _must_fail(TF.test_e2m1_ties_from_golden_file)
    monkeypatch.setattr(F, "round_e2m1", real_round)
    # scale from floor(log2(max)) - 2, the other common convention: blocks with max in (6 s, 8 s) would clip
    monkeypatch.setattr(F, "block_scale_byte", lambda a: np.where(np.asarray(a) > 0, np.clip(np.frexp(np.asarray(a, np.float64))[1] - 3 + 127, 0, 254), 0).astype(np.uint8))
    _must_fail(TF.test_block_scale_is_the_smallest_power_of_two_that_keeps_the_block_in_range)
    _must_fail(TF.test_quantizer_invariants)
    monkeypatch.setattr(F, "block_scale_byte", real_scale)
    # the weight side quantized from the smoothed weight instead of the residual (low-rank term dropped from R)
    monkeypatch.setattr(F.O, "residual", lambda W, lam, a, b: np.asarray(W, np.float64) * np.asarray(lam, np.float64)[:, None])
    _must_fail(TF.test_forward_equals_the_dense_definition_of_eq5)


def test_refinement_that_ignores_the_quantized_residual_is_caught(monkeypatch):
    real = O.lowrank_svd
    state = {"first": None}

    def bad(A, r):                      # every iterate decomposes W^ again instead of W^ - Q(R)
        if state["first"] is None:
            state["first"] = np.array(A, copy=True)
        return real(state["first"], r)
    monkeypatch.setattr(O, "lowrank_svd", bad)
    _must_fail(lambda: TL.test_iterative_update_of_the_lowrank_branch("int4"))


def test_w8a8_mistakes_are_caught(monkeypatch):
    from oracle import svdq_w8a8_oracle as W8
    import tests.test_oracle_w8a8 as TW
    real = W8.quantize_rows

    def per_tensor(v):                       # one scale for the whole tensor instead of one per row
        v = np.ascontiguousarray(v, np.float32)
        q, s = real(v.reshape(1, -1))
        return q.reshape(v.shape), np.full(v.shape[:-1], s[0], np.float16)
    monkeypatch.setattr(W8, "quantize_rows", per_tensor)
    _must_fail(TW.test_quantizer_against_exact_rationals_and_invariants)
    monkeypatch.setattr(W8, "quantize_rows", real)
    # weights quantized per input channel (rows of R) instead of per output channel
    monkeypatch.setattr(W8, "quantize_residual", lambda R: (lambda q, s: (q, np.resize(s, R.shape[1])))(*real(np.asarray(R, np.float64).astype(np.float32))))
    _must_fail(TW.test_forward_equals_the_dense_definition_and_integer_sums_are_exact)


def test_gptq_mistakes_are_caught(monkeypatch):
    real = O.gptq_feedback
    for bad in (lambda U, k, e: -real(U, k, e),                                  # error pushed the wrong way
                lambda U, k, e: np.outer(U[k + 1:, k], e),                       # the factor's other triangle: no feedback at all
                lambda U, k, e: np.outer(U[k, k + 1:] / U[k, k], e)):            # divided by the diagonal twice
        monkeypatch.setattr(O, "gptq_feedback", bad)
        _must_fail(TG.test_remaining_rows_are_the_least_squares_optimum_given_the_fixed_ones)
    for bad in (lambda U, k, e: -real(U, k, e), lambda U, k, e: np.outer(U[k + 1:, k], e)):
        monkeypatch.setattr(O, "gptq_feedback", bad)
        _must_fail(TG.test_objective_drops_below_round_to_nearest_and_so_does_the_layer_error)
    monkeypatch.setattr(O, "gptq_feedback", real)
    # the Hessian of the unsmoothed activations
    real_h = O.gptq_hessian
    monkeypatch.setattr(O, "gptq_hessian", lambda x, rinv: real_h(x, np.ones_like(rinv)))
    _must_fail(TG.test_objective_drops_below_round_to_nearest_and_so_does_the_layer_error)
    monkeypatch.setattr(O, "gptq_hessian", real_h)
    TG.test_remaining_rows_are_the_least_squares_optimum_given_the_fixed_ones()
