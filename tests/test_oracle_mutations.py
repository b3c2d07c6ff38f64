"""Plant plausible mistakes in a COPY of the oracle (CPU only) and check that the
pins notice each one.  The copy is compiled into a temp dir; oracle/ is untouched."""
import ctypes
import os
import subprocess
import numpy as np
import pytest

import oracle
import test_oracle_conv as tc
import test_oracle_pool as tp
import test_oracle_upsample as tu
import test_oracle_pool_sub as ts
import test_oracle_block as tb
import test_oracle_idiss as ti
import test_oracle_knn as tk

SRC = open(os.path.join(os.path.dirname(oracle.__file__), "oracle.c")).read()

FWD_PINS = [lambda: tc.test_fwd_bruteforce_dense_weight_tensor(0, 2, 11, 3, 3, 2),
            tc.test_fwd_grid_reduces_to_2d_correlation,
            lambda: tc.test_fwd_named_image_operators("prewitt_x", (1, 0, 0), 0.0),
            lambda: tc.test_fwd_named_image_operators("blur", (0, 0, 0), 1.0 / 9.0),
            tc.test_fwd_theta_zero_is_bias_weighted_neighbour_sum]
BWD_PINS = [tc.test_bwd_bruteforce_dense, tc.test_bwd_finite_differences_full_jacobian,
            tc.test_bwd_adjoint_identities_cfg0, tc.test_bwd_grad_feat_at_matches_full]
POOL_PINS = [tp.test_pool_fwd_bruteforce_with_ties, tp.test_pool_fwd_invariants,
             tp.test_pool_fwd_k1_identity_and_constant_feature, tp.test_pool_bwd_bruteforce_and_mass,
             tp.test_pool_bwd_is_adjoint_of_selection]

UP_PINS = [tu.test_upsample_fwd_bruteforce_with_ties, tu.test_upsample_fwd_is_zero_fill_then_pool,
           tu.test_upsample_grid_is_zero_insertion_then_3x3_max, tu.test_upsample_bwd_bruteforce_mass_and_composition]

SUB_PINS = [ts.test_pool_sub_fwd_bruteforce_with_ties, ts.test_pool_sub_fwd_grid_is_3x3_maxpool_stride2,
            ts.test_pool_sub_bwd_bruteforce_mass_and_repeats, ts.test_pool_sub_bwd_is_directional_derivative]

BLOCK_PINS = [tb.test_block_fwd_bruteforce_dense, tb.test_block_identity_1x1_is_plain_flexconv,
              tb.test_block_bwd_finite_differences_full_jacobian]

def _idiss_quantisation_pin():
    for N, Ns, log2_top in ((40, 10, 27), (97, 31, 26), (64, 16, 28), (300, 75, 27)):
        ti.test_quantisation_against_integer_arithmetic_on_dyadic_weights(N, Ns, log2_top)


IDISS_PINS = [ti.test_phi_bruteforce_and_grid_closed_form, ti.test_sample_matches_exact_integer_reference,
              _idiss_quantisation_pin,
              ti.test_sample_uniform_density_is_one_point_per_block, ti.test_make_distinct_bruteforce_and_properties]

KNN_PINS = [tk.test_knn_matches_float32_numpy_ranking_with_ties, tk.test_knn_agrees_with_a_kd_tree_on_generic_points,
            tk.test_knn_k_equals_n_and_duplicates]

POS_PINS = [tc.test_bwd_pos_finite_differences, tc.test_bwd_pos_bruteforce_translation_and_self_edges]

# (name, text to replace, replacement, occurrence index or None for all, pins that must catch it)
MUTATIONS = [
    ("fwd_sign_dx", "(double)pos[IDX3(b, 0, n, 3, N)] - (double)pos[IDX3(b, 0, l, 3, N)]",
     "(double)pos[IDX3(b, 0, l, 3, N)] - (double)pos[IDX3(b, 0, n, 3, N)]", 0, FWD_PINS),
    ("fwd_drop_bias", " + (double)tb[o];\n                            acc[o] += w * f;",
     ";\n                            acc[o] += w * f;", 0, FWD_PINS),
    ("fwd_drop_z", "+ (double)tz[o] * dz + (double)tb[o];\n                            acc[o]",
     "+ (double)tb[o];\n                            acc[o]", 0, FWD_PINS),
    ("fwd_feat_of_centre", "const double f = (double)feat[IDX3(b, c, n, Din, N)];\n                        const float *tx = theta + IDX3(0, c, 0, Din, Dout);\n                        const float *ty = theta + IDX3(1, c, 0, Din, Dout);\n                        const float *tz = theta + IDX3(2, c, 0, Din, Dout);\n                        const float *tb = bias + (int64_t)c * Dout;\n                        for (int o = 0; o < Dout; ++o) {\n                            const double w",
     "const double f = (double)feat[IDX3(b, c, l, Din, N)];\n                        const float *tx = theta + IDX3(0, c, 0, Din, Dout);\n                        const float *ty = theta + IDX3(1, c, 0, Din, Dout);\n                        const float *tz = theta + IDX3(2, c, 0, Din, Dout);\n                        const float *tb = bias + (int64_t)c * Dout;\n                        for (int o = 0; o < Dout; ++o) {\n                            const double w", 0, FWD_PINS),
    ("nbr_layout_transposed", "nbr[IDX3(b, k, l, K, N)]", "nbr[((int64_t)b * N + l) * K + k]", None, FWD_PINS),
    ("bwd_gfeat_to_centre", "grad_feat[IDX3(b, c, n, Din, N)] += s;", "grad_feat[IDX3(b, c, l, Din, N)] += s;", 0, BWD_PINS),
    ("bwd_gtheta_xy_swapped", "gtx[o] += dx * fg;", "gtx[o] += dy * fg;", 0, BWD_PINS),
    ("bwd_gbias_uses_position", "gbb[o] += fg;", "gbb[o] += dz * fg;", 0, BWD_PINS),
    ("bwd_at_wrong_g_column", "s += w * (double)grad_out[IDX3(b, o, l, Dout, N)];",
     "s += w * (double)grad_out[IDX3(b, o, n, Dout, N)];", 0, BWD_PINS),
    ("pool_tie_by_slot", "if (v > bv || (v == bv && n < best))", "if (v > bv)", 0, POOL_PINS),
    ("pool_min_instead_of_max", "if (v > bv || (v == bv && n < best))", "if (v < bv || (v == bv && n < best))", 0, POOL_PINS),
    ("upsample_copy_to_own_index", "dense[IDX3(b, c, m, C, Nf)] = feat_small[IDX3(b, c, j, C, Ns)];",
     "dense[IDX3(b, c, j, C, Nf)] = feat_small[IDX3(b, c, j, C, Ns)];", 0, UP_PINS),
    ("upsample_tie_by_slot", "if (v > bv || (v == bv && n < best))", "if (v > bv)", 1, UP_PINS),
    ("upsample_bwd_reads_own_index", "grad_small[IDX3(b, c, j, C, Ns)] = dense[IDX3(b, c, m, C, Nf)];",
     "grad_small[IDX3(b, c, j, C, Ns)] = dense[IDX3(b, c, j, C, Nf)];", 0, UP_PINS),
    ("bwd_pos_centre_sign", "grad_pos[IDX3(b, d, l, 3, N)] -= s;", "grad_pos[IDX3(b, d, l, 3, N)] += s;", 0, POS_PINS),
    ("bwd_pos_feature_of_centre", "s += (double)theta[IDX3(d, c, o, Din, Dout)] * f * (double)grad_out[IDX3(b, o, l, Dout, N)];",
     "s += (double)theta[IDX3(d, c, o, Din, Dout)] * (double)feat[IDX3(b, c, l, Din, N)] * (double)grad_out[IDX3(b, o, l, Dout, N)];", 0, POS_PINS),
    ("bwd_pos_gradient_of_neighbour", "s += (double)theta[IDX3(d, c, o, Din, Dout)] * f * (double)grad_out[IDX3(b, o, l, Dout, N)];",
     "s += (double)theta[IDX3(d, c, o, Din, Dout)] * f * (double)grad_out[IDX3(b, o, n, Dout, N)];", 0, POS_PINS),
    ("pool_sub_reads_row_j", "out[IDX3(b, c, j, C, Ns)] = pooled[IDX3(b, c, l, C, N)];",
     "out[IDX3(b, c, j, C, Ns)] = pooled[IDX3(b, c, j, C, N)];", 0, SUB_PINS),
    ("pool_sub_tie_by_slot", "if (v > bv || (v == bv && n < best))", "if (v > bv)", 2, SUB_PINS),
    ("pool_sub_bwd_to_kept_centre", "grad_feat[IDX3(b, c, m, C, N)] += gpooled[IDX3(b, c, l, C, N)];",
     "grad_feat[IDX3(b, c, l, C, N)] += gpooled[IDX3(b, c, l, C, N)];", 0, SUB_PINS),
    ("block_1x1_transposed", "s += (double)W[(int64_t)c * Din0 + c0] * (double)feat[IDX3(b, c0, n, Din0, N)];\n                mid",
     "s += (double)W[(int64_t)c0 * Dmid + c] * (double)feat[IDX3(b, c0, n, Din0, N)];\n                mid", 0, BLOCK_PINS),
    ("block_grad_w_uses_centre_gradient", "gmid[IDX3(b, c, n, Dmid, N)] += s;", "gmid[IDX3(b, c, l, Dmid, N)] += s;", 0, BLOCK_PINS),
    ("block_grad_feat_untransposed", "for (int c = 0; c < Dmid; ++c) s += (double)W[(int64_t)c * Din0 + c0] * gmid[IDX3(b, c, n, Dmid, N)];",
     "for (int c = 0; c < Dmid; ++c) s += (double)W[(int64_t)c * Din0 + c0] * gmid[IDX3(b, c0 % Dmid, n, Dmid, N)];", 0, BLOCK_PINS),
    ("idiss_phi_squared_distance", "s += sqrt(d2);", "s += d2;", 0, IDISS_PINS),
    ("idiss_threshold_inclusive", "while (C[l] <= t) ++l;", "while (C[l] < t) ++l;", 0, IDISS_PINS),
    ("idiss_weights_rounded_up", "(uint32_t)(ph[l] * scale)", "(uint32_t)(ph[l] * scale + 0.999f)", 0, IDISS_PINS),
    ("idiss_scale_by_sum_not_max", "if (ph[l] > mx) mx = ph[l];", "mx += ph[l];", 0, IDISS_PINS),
    ("idiss_remainder_dropped", "const uint64_t len = width + ((uint64_t)j < rem ? 1u : 0u);", "const uint64_t len = width;", 0, IDISS_PINS),
    ("knn_ties_to_later_index", "while (at > 0 && d2 < bd[at - 1])", "while (at > 0 && d2 <= bd[at - 1])", 0, KNN_PINS),
    ("knn_drops_z", "const float d2 = xy + zz;", "const float d2 = xy;", 0, KNN_PINS),
    ("distinct_keeps_equal_entries", "if (s[j] <= s[j - 1]) s[j] = s[j - 1] + 1;", "if (s[j] < s[j - 1]) s[j] = s[j - 1] + 1;", 0, IDISS_PINS),
    ("distinct_tail_not_packed", "if (s[j] > N - Ns + j) s[j] = N - Ns + j;", "if (s[j] > N - 1) s[j] = N - 1;", 0, IDISS_PINS),
    ("pool_bwd_to_centre", "grad_feat[IDX3(b, c, m, C, N)] += (double)grad_out", "grad_feat[IDX3(b, c, l, C, N)] += (double)grad_out", 0, POOL_PINS),
]


def _replace(text, old, new, which):
    assert old in text, old
    if which is None:
        return text.replace(old, new)
    parts = text.split(old)
    assert which < len(parts) - 1
    return old.join(parts[:which + 1]) + new + old.join(parts[which + 1:])


@pytest.mark.parametrize("name,old,new,which,pins", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, monkeypatch, name, old, new, which, pins):
    src = tmp_path / "mut.c"
    lib = tmp_path / "libmut.so"
    src.write_text(_replace(SRC, old, new, which))
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", "-std=c11", "-o", str(lib), str(src), "-lm"], check=True)
    mut = ctypes.CDLL(str(lib))
    mut.oracle_count_bad_neighbors.restype = ctypes.c_int64
    oracle._load()
    monkeypatch.setattr(oracle, "_lib", mut)
    caught = 0
    for pin in pins:
        try:
            pin()
        except (AssertionError, RuntimeError):
            caught += 1
    assert caught >= 1, f"mutation {name} slipped through every pin"
