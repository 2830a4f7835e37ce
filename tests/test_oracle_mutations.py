"""Checks of the pins themselves: plant one plausible mistake at a time in a COPY of the oracle's
source (CPU only), and require that at least one pin fails.  A mistake that every pin accepts
would mean that the oracle is not pinned where the mistake sits."""
import os

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)), "mae_oracle.c")


class _Golden:
    def __call__(self, name):
        from conftest import read_golden
        return read_golden(name)


# (label, text in the source, replacement, pins that must notice)
MUTATIONS = [
    ("hash shift", "(z ^ (z >> 30))", "(z ^ (z >> 31))", ["test_hash_known_answers"]),
    ("hash stream field", "(stream & 0xFFu) << 24", "(stream & 0xFFu) << 23",
     ["test_hash_known_answers"]),
    ("batch key offset", "(batch_index + 1)", "(batch_index)", ["test_hash_known_answers"]),
    ("exp degree", "for (int k = 13; k >= 1; --k) {", "for (int k = 3; k >= 1; --k) {",
     ["test_exp_polynomial_matches_libm"]),
    ("scale law on the side, not the area", "double T = area * s;", "double T = area * s * s;",
     ["test_rrc_proposal_statistics_match_eq2"]),
    ("ratio transposed", "double cw = rint(sqrt(T * r));\n  double ch = rint(sqrt(T / r));",
     "double cw = rint(sqrt(T / r));\n  double ch = rint(sqrt(T * r));",
     ["test_rrc_fixed_ratio_orientation"]),
    ("ratio uniform instead of log-uniform", "double r = mae_oracle_exp_poly(x);",
     "double r = 0.75 + (4.0 / 3.0 - 0.75) * u_ratio;",
     ["test_rrc_proposal_statistics_match_eq2", "test_rrc_proposal_recomputed_with_libm"]),
    ("offset range off by one", "(uint64_t)(H - ch + 1)", "(uint64_t)(H - ch)",
     ["test_rrc_offsets_are_uniform_over_positions_that_fit"]),
    ("fallback not centred", "box[1] = (int32_t)((W - cw) / 2);", "box[1] = 0;",
     ["test_rrc_fallback_is_centred_square"]),
    ("fallback ratio side", "ch = (int64_t)rint((double)W / (double)ratio_lo);",
     "ch = (int64_t)rint((double)W * (double)ratio_lo);", ["test_rrc_fallback_is_centred_square"]),
    ("flip threshold", "return u < flip_p ? 1 : 0;", "return u > flip_p ? 1 : 0;",
     ["test_flip_probability_extremes_and_rate"]),
    ("pixel centres dropped", "(2 * (int64_t)o + 1) * (int64_t)crop_len - (int64_t)out_size",
     "(2 * (int64_t)o) * (int64_t)crop_len",
     ["test_resize_taps_printed_example", "test_resize_against_library_bilinear"]),
    ("second tap not clamped", "*i1 = (*i0 + 1 < crop_len) ? *i0 + 1 : crop_len - 1;",
     "*i1 = *i0 + 1;", ["test_resize_clamps_to_crop_box_not_image",
                        "test_resize_identity_constant_and_single_pixel"]),
    ("weights swapped", "double rt = a00 + fx * (a01 - a00);",
     "double rt = a01 + fx * (a00 - a01);", ["test_resize_taps_printed_example"]),
    ("rows and columns swapped in the blend", "out[((int64_t)oy * S + ox) * 3 + c] = rt + fy * (rb - rt);",
     "out[((int64_t)oy * S + ox) * 3 + c] = rt + fx * (rb - rt);",
     ["test_resize_reproduces_affine_ramps"]),
    ("crop offset ignored", "double a00 = img[((int64_t)(top + y0) * W + (left + x0)) * 3 + c];",
     "double a00 = img[((int64_t)(top + y0) * W + (x0)) * 3 + c];",
     ["test_resize_identity_constant_and_single_pixel", "test_resize_reproduces_affine_ramps"]),
    ("flip ignored", "int32_t sx = flip ? (S - 1 - ox) : ox;", "int32_t sx = ox;",
     ["test_flip_twice_is_identity_and_mirrors_columns"]),
    ("normalise order", "return (v / 255.0 - mean) / std;", "return (v / 255.0) / std - mean;",
     ["test_normalise_end_points"]),
    ("patch order transposed", "int64_t l = (int64_t)(y / p) * G + (x / p);",
     "int64_t l = (int64_t)(x / p) * G + (y / p);", ["test_patchify_layout"]),
    ("channel not fastest", "int64_t e = ((int64_t)(y % p) * p + (x % p)) * 3 + c;",
     "int64_t e = (int64_t)c * p * p + (int64_t)(y % p) * p + (x % p);", ["test_patchify_layout"]),
    ("ties broken the other way", "(key[j] == key[l] && j < l)", "(key[j] == key[l] && j > l)",
     ["test_masking_invariants_and_library_argsort"]),
    ("descending noise", "if (key[j] < key[l] ||", "if (key[j] > key[l] ||",
     ["test_masking_worked_example"]),
    ("mask polarity", "mask[l] = (rank >= K) ? 1 : 0;", "mask[l] = (rank >= K) ? 0 : 1;",
     ["test_masking_worked_example"]),
    ("num_keep rounds", "return (int32_t)floor((double)L * (1.0 - mask_ratio));",
     "return (int32_t)rint((double)L * (1.0 - mask_ratio));", ["test_num_keep_values"]),
    ("gather uses rank as index", "(float)patches[(int64_t)keep[r] * D + e];",
     "(float)patches[(int64_t)r * D + e];", ["test_prep_gather_and_slicing"]),
    ("unreadable sample still masked", "if (mask) mask[n * L + l] = 0;",
     "if (mask) mask[n * L + l] = (l >= K) ? 1 : 0;", ["test_prep_unreadable_samples_take_no_part"]),
    ("unreadable sample keeps a shuffled order", "if (ids_restore) ids_restore[n * L + l] = l;",
     "if (ids_restore) ids_restore[n * L + l] = L - 1 - l;",
     ["test_prep_unreadable_samples_take_no_part"]),
    ("biased variance", "double var = ss / (double)(D - 1);", "double var = ss / (double)D;",
     ["test_loss_normalised_target_statistics"]),
    ("eps outside the root", "double sd = sqrt(var + eps);", "double sd = sqrt(var) + eps;",
     ["test_loss_normalised_target_statistics"]),
    ("gradient factor", "mask[row] ? (float)(grad_scale * 2.0 * diff / ((double)D * M)) : 0.0f;\n    }\n    row_losses",
     "mask[row] ? (float)(grad_scale * diff / ((double)D * M)) : 0.0f;\n    }\n    row_losses",
     ["test_loss_euler_identity_and_finite_differences"]),
    ("pixel loss normalises anyway", "double diff = (double)pred[row * D + e] - (double)target[row * D + e];",
     "double diff = (double)pred[row * D + e] - 0.5 * (double)target[row * D + e];",
     ["test_pixel_loss_against_library_and_closed_form"]),
    ("pixel loss divisor", "if (mask[row]) total += row_loss / (double)D;",
     "if (mask[row]) total += row_loss;", ["test_pixel_loss_against_library_and_closed_form"]),
    ("scheme 5 not a palindrome", "{224, 192, 224},  /* 5: palindrome   ",
     "{224, 192, 160},  /* 5: palindrome   ", ["test_progressive_schemes_match_the_printed_tables"]),
    ("scheme 4 ratios", "{0.75, 0.80, 0.85}, {0.75, 0.75, 0.75}, {0.75, 0.75, 0.85},",
     "{0.75, 0.80, 0.80}, {0.75, 0.75, 0.75}, {0.75, 0.75, 0.85},",
     ["test_progressive_schemes_match_the_printed_tables"]),
    ("resize to bytes truncates", "(uint8_t)((2 * num + den * den) / (2 * den * den));",
     "(uint8_t)((2 * num) / (2 * den * den));",
     ["test_three_aug_worked_examples", "test_resize_u8_is_the_exactly_rounded_bilinear_value"]),
    ("resize to bytes, weights of the rows swapped",
     "(den - ry) * ((den - rx) * a00 + rx * a01) + ry * ((den - rx) * a10 + rx * a11);",
     "ry * ((den - rx) * a00 + rx * a01) + (den - ry) * ((den - rx) * a10 + rx * a11);",
     ["test_resize_u8_is_the_exactly_rounded_bilinear_value"]),
    ("luma weights swapped", "(299 * r + 587 * g + 114 * b + 500) / 1000",
     "(587 * r + 299 * g + 114 * b + 500) / 1000", ["test_three_aug_worked_examples"]),
    ("luma truncated", "(299 * r + 587 * g + 114 * b + 500) / 1000",
     "(299 * r + 587 * g + 114 * b) / 1000", ["test_gray_and_solarise_over_their_whole_domain"]),
    ("solarise threshold off by one", "return v >= 128 ? 255 - v : v;",
     "return v > 128 ? 255 - v : v;", ["test_three_aug_worked_examples"]),
    ("blur radius", "(int32_t)ceil(3.0 * sigma);", "(int32_t)ceil(2.0 * sigma);",
     ["test_blur_matches_the_library_gaussian_filter"]),
    ("blur taps not scaled to one", "for (int32_t k = 0; k <= 2 * radius; ++k) w[k] /= sum;",
     "for (int32_t k = 0; k <= 2 * radius; ++k) w[k] /= 1.0;",
     ["test_blur_matches_the_library_gaussian_filter"]),
    ("blur variance", "exp(-(double)(k * k) / (2.0 * sigma * sigma));",
     "exp(-(double)(k * k) / (sigma * sigma));", ["test_blur_matches_the_library_gaussian_filter"]),
    ("blur border wraps", "(double)u8[((int64_t)clampi(y + k, 0, S - 1) * S + x) * 3 + c];",
     "(double)u8[((int64_t)((y + k + S) % S) * S + x) * 3 + c];",
     ["test_blur_matches_the_library_gaussian_filter"]),
    ("blur along one axis only", "acc += w[k + radius] * tmp[((int64_t)y * S + clampi(x + k, 0, S - 1)) * 3 + c];",
     "acc += (k == 0 ? 1.0 : 0.0) * tmp[((int64_t)y * S + clampi(x + k, 0, S - 1)) * 3 + c];",
     ["test_blur_matches_the_library_gaussian_filter"]),
    ("operation drawn from the blur stream",
     "floor(3.0 * draw_unit(seed, batch_index, sample, 6u, 0u));",
     "floor(3.0 * draw_unit(seed, batch_index, sample, 7u, 0u));",
     ["test_aug_draws_are_uniform_and_independent"]),
    ("blur width range", "*sigma = 0.1 + 1.9 * draw_unit", "*sigma = 0.1 + 2.9 * draw_unit",
     ["test_aug_draws_are_uniform_and_independent"]),
    ("jitter factors one-sided", "bcs[j] = 1.0 + jitter * (2.0 * draw_unit(seed, batch_index, sample, 8u + j, 0u) - 1.0);",
     "bcs[j] = 1.0 + jitter * (draw_unit(seed, batch_index, sample, 8u + j, 0u));",
     ["test_aug_draws_are_uniform_and_independent"]),
    ("brightness not clamped", "img[i] = clampd(img[i] * bcs[0]);", "img[i] = img[i] * bcs[0];",
     ["test_three_aug_worked_examples"]),
    ("contrast mean taken before brightness",
     "for (int64_t i = 0; i < n; ++i) mean += luma(img + i * 3);\n  mean /= (double)n;",
     "for (int64_t i = 0; i < n; ++i) mean += luma(img + i * 3);\n  mean /= (double)n * bcs[0];",
     ["test_color_jitter_special_cases"]),
    ("contrast blends with the wrong factor", "(1.0 - bcs[1]) * mean", "(1.0 - bcs[0]) * mean",
     ["test_three_aug_worked_examples"]),
    ("saturation blends with the image mean", "double g = luma(img + i * 3);\n    for",
     "double g = mean;\n    for", ["test_color_jitter_special_cases"]),
    ("luma weight of green", "0.299 * px[0] + 0.587 * px[1]", "0.299 * px[0] + 0.578 * px[1]",
     ["test_three_aug_worked_examples"]),
    ("jitter applied in plain 3 Aug", "if (a->aug_mode == 2) mae_oracle_color_jitter",
     "if (a->aug_mode >= 1) mae_oracle_color_jitter",
     ["test_prep_batch_with_finetune_augmentation_is_the_composition_of_its_steps"]),
    ("augmentation before the flip is undone", "mae_oracle_resize_u8(img, H, W, box, S, flip, u8);",
     "mae_oracle_resize_u8(img, H, W, box, S, 0, u8);",
     ["test_prep_batch_with_finetune_augmentation_is_the_composition_of_its_steps"]),
    ("zig-zag order", "0,  1,  8,  16, 9,  2,  3,  10,", "0,  1,  8,  16, 2,  9,  3,  10,",
     ["test_jpeg_decoder_against_the_imaging_library"]),
    ("sign extension of coefficients", "? v - (1 << s) + 1 : v;", "? v - (1 << s) : v;",
     ["test_jpeg_decoder_against_the_imaging_library"]),
    ("predictor kept across restarts", "pred[0] = pred[1] = pred[2] = 0;\n    }", "}",
     ["test_jpeg_decoder_does_not_depend_on_how_the_stream_is_organised"]),
    ("quantiser indexed in natural order",
     "coef[ZIGZAG[k]] = extend(receive(&r, size), size) * (int32_t)h.q[h.tq[c]][k];",
     "coef[ZIGZAG[k]] = extend(receive(&r, size), size) * (int32_t)h.q[h.tq[c]][ZIGZAG[k]];",
     ["test_jpeg_decoder_against_the_imaging_library"]),
    ("zero run of sixteen", "k += 16;\n              continue;", "k += 15;\n              continue;",
     ["test_jpeg_decoder_does_not_depend_on_how_the_stream_is_organised"]),
    ("canonical code of the next length", "code += t->counts[len - 1];\n    index",
     "code += t->counts[len - 1] + 1;\n    index", ["test_jpeg_decoder_against_the_imaging_library"]),
    ("codes not doubled between lengths", "      lengths[i++] = (uint8_t)len;\n    }\n    code <<= 1;",
     "      lengths[i++] = (uint8_t)len;\n    }\n    code += 0;",
     ["test_huffman_codes_are_the_canonical_ones"]),
    ("inverse transform transposed", "acc += (int64_t)idct_basis(y, v) * clamp16(coef[v * 8 + u]);",
     "acc += (int64_t)idct_basis(y, v) * clamp16(coef[u * 8 + v]);",
     ["test_idct_matches_the_library_transform"]),
    ("DC term not scaled by 1/sqrt 2", "double c = (u == 0) ? sqrt(0.5) :", "double c = (u == 0) ? 1.0 :",
     ["test_idct_matches_the_library_transform"]),
    ("level shift", "floor_shift(acc + (1 << 16), 17) + 128;", "floor_shift(acc + (1 << 16), 17) + 127;",
     ["test_idct_matches_the_library_transform"]),
    ("chroma planes swapped", "int64_t b = cb - 128, r = cr - 128;", "int64_t b = cr - 128, r = cb - 128;",
     ["test_colour_conversion_matches_the_jfif_matrix"]),
    ("green coefficient", "22554 * b + 46802 * r", "22554 * b + 46208 * r",
     ["test_colour_conversion_matches_the_jfif_matrix"]),
    ("chroma not repeated vertically", "plane[1][(size_t)(y * h.vs[1] / vmax) * pw[1]",
     "plane[1][(size_t)(y * h.vs[1]) * pw[1] / vmax",
     ["test_jpeg_decoder_against_the_imaging_library"]),
    ("stuffed byte kept", "r->pos += 2;\n        } else {\n          r->hit_marker = 1;",
     "r->pos += 1;\n        } else {\n          r->hit_marker = 1;",
     ["test_jpeg_decoder_against_the_imaging_library",
      "test_jpeg_decoder_does_not_depend_on_how_the_stream_is_organised"]),
    ("block order inside an MCU", "int32_t x0 = (mx * h.hs[c] + bh) * 8, y0 = (my * h.vs[c] + bv) * 8;",
     "int32_t x0 = (mx * h.hs[c] + bv) * 8, y0 = (my * h.vs[c] + bh) * 8;",
     ["test_jpeg_decoder_against_the_imaging_library"]),
    ("embedding weight transposed", "acc += (double)v[d] * (double)weight[(int64_t)e * D + d];",
     "acc += (double)v[d] * (double)weight[((int64_t)d * E + e) % ((int64_t)E * D)];",
     ["test_patch_embed_closed_forms_and_library_matmul"]),
    ("positional embedding by rank", "if (pos) acc += (double)pos[(int64_t)l * E + e];",
     "if (pos) acc += (double)pos[(row % K) * (int64_t)E + e];",
     ["test_patch_embed_closed_forms_and_library_matmul"]),
    ("bias dropped", "if (bias) acc += (double)bias[e];", "if (bias) acc += 0.0;",
     ["test_patch_embed_closed_forms_and_library_matmul"]),
    ("stage boundary", "if (epoch < end) return s + 1;", "if (epoch <= end) return s + 1;",
     ["test_progressive_schemes_match_the_printed_tables"]),
    ("loss over all rows", "if (mask[row]) total += row_losses[row];",
     "total += row_losses[row];", ["test_loss_constant_offset_closed_form"]),
    ("per-row mean dropped", "row_losses[row] = row_loss / (double)D;",
     "row_losses[row] = row_loss;", ["test_loss_constant_offset_closed_form"]),
    ("gradient on visible rows",
     "mask[row] ? (float)(grad_scale * 2.0 * diff / ((double)D * M)) : 0.0f;\n    }\n    row_losses",
     "(float)(grad_scale * 2.0 * diff / ((double)D * M));\n    }\n    row_losses",
     ["test_loss_against_library_autograd"]),
]


@pytest.mark.parametrize("label,old,new,watchers", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(label, old, new, watchers, tmp_path, monkeypatch):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for '{label}' not unique in the oracle source"
    mutated = tmp_path / "mutated_oracle.c"
    mutated.write_text(text.replace(old, new))
    so = oracle.compile_source(str(mutated), str(tmp_path / "libmutated.so"))
    monkeypatch.setattr(oracle, "_lib", oracle.load_library(so))
    caught = []
    for name in watchers:
        fn = getattr(pins, name)
        kwargs = {"golden": _Golden()} if "golden" in fn.__code__.co_varnames[:fn.__code__.co_argcount] else {}
        params = [m.args for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        calls = [kwargs]
        if params:
            names = [n.strip() for n in params[0][0].split(",")]
            calls = [dict(kwargs, **dict(zip(names, v if isinstance(v, tuple) else (v,))))
                     for v in params[0][1]]
        for kw in calls:
            try:
                fn(**kw)
            except (AssertionError, ValueError):  # a wrong value, or the oracle giving up
                caught.append(name)
                break
    assert caught, f"no pin noticed the planted mistake '{label}'"
