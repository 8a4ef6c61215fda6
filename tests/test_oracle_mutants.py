"""Are the pins sharp?  Plant one plausible mistake at a time in a copy of the
oracle's source (CPU only), rebuild it, and require that at least one pin fails.
"""
import os
import subprocess

import pytest

from oracle import CFLAGS, SOURCE, Oracle
from pins import ALL_PINS

# (name, text in nms_oracle.c, replacement, how many occurrences must be replaced)
MUTANTS = [
    ("denominator_is_victim_area", "float a = box_area(bj);", "float a = box_area(bi);", 1),
    ("intersection_over_union", "return (w * h) / a;", "return (w * h) / ((a + box_area(bi)) - (w * h));", 1),
    ("equality_survives", "(q < theta) ? 1 : 0", "(q <= theta) ? 1 : 0", 2),
    ("no_plus_one_on_width", "float w = (far_x - near_x) + 1.0f;", "float w = (far_x - near_x);", 1),
    ("no_plus_one_on_height", "float h = (far_y - near_y) + 1.0f;", "float h = (far_y - near_y);", 1),
    ("no_plus_one_in_area", "float w = (b[2] - b[0]) + 1.0f;", "float w = (b[2] - b[0]);", 1),
    ("tie_to_higher_index", "scores[j] == scores[i] && j < i", "scores[j] == scores[i] && j > i", 1),
    ("ties_ignored", "if (scores[j] == scores[i] && j < i) return 1;", "", 1),
    ("rank_reversed", "if (scores[j] > scores[i]) return 1;", "if (scores[j] < scores[i]) return 1;", 1),
    ("width_not_floored", "if (!(w > 0.0f)) w = 0.0f;\n\n    float far_y", "\n    float far_y", 1),
    ("height_not_floored", "if (!(h > 0.0f)) h = 0.0f;\n\n    float a = box_area(bj);", "\n    float a = box_area(bj);", 1),
    ("far_edge_is_max", "float far_x = bi[2] < bj[2] ? bi[2] : bj[2];", "float far_x = bi[2] > bj[2] ? bi[2] : bj[2];", 1),
    ("near_edge_is_min", "float near_y = bi[1] > bj[1] ? bi[1] : bj[1];", "float near_y = bi[1] < bj[1] ? bi[1] : bj[1];", 1),
    ("y_uses_x_edges", "float far_y = bi[3] < bj[3] ? bi[3] : bj[3];", "float far_y = bi[2] < bj[2] ? bi[2] : bj[2];", 1),
    ("operands_transposed_keep", "float q = overlap(boxes + 4 * (size_t)i, boxes + 4 * (size_t)j);\n                b = ",
     "float q = overlap(boxes + 4 * (size_t)j, boxes + 4 * (size_t)i);\n                b = ", 1),
    ("operands_transposed_map", "float q = overlap(boxes + 4 * (size_t)i, boxes + 4 * (size_t)j);\n                B[",
     "float q = overlap(boxes + 4 * (size_t)j, boxes + 4 * (size_t)i);\n                B[", 1),
    ("reduce_is_or", "v = (uint8_t)(v & B[(size_t)i * n + j]);", "v = (uint8_t)(v | B[(size_t)i * n + j]);", 1),
    ("keep_stops_at_diagonal", "for (int j = 0; j < n; ++j) {\n            uint8_t b = 1;", "for (int j = 0; j < i; ++j) {\n            uint8_t b = 1;", 1),
    ("area_is_square_of_width", "return w * h;", "return w * w;", 1),
    ("greedy_counts_dead_boxes", "if (keep[j]) {", "if (1) {", 1),
    ("ranked_bits_upper_triangle", "for (int c = 0; c < r; ++c) {\n            float q = overlap(boxes + 4 * (size_t)order[r], boxes + 4 * (size_t)order[c]);\n            E[",
     "for (int c = 0; c <= r; ++c) {\n            float q = overlap(boxes + 4 * (size_t)order[r], boxes + 4 * (size_t)order[c]);\n            E[", 1),
    ("ranked_words_wrong_bit", "(uint64_t)1 << (c & 63)", "(uint64_t)1 << (c & 31)", 1),
    ("ranked_area_missing", "out[5 * (size_t)r + 4] = box_area(b);", "out[5 * (size_t)r + 4] = b[2] - b[0];", 1),
    ("square_form_drops_partition", "for (int part = 0; part < k; ++part) {", "for (int part = 0; part < k - 1; ++part) {", 1),
    ("square_form_nonstrict", "if (s_i < s_j) {", "if (s_i <= s_j) {", 1),
    ("square_form_ignores_empty_slots_term", "b = (uint8_t)(below && z_j != 0.0f);", "b = (uint8_t)below;", 1),
    ("square_form_far_corner", "box[4 * t + 3] = d[1] + d[2];", "box[4 * t + 3] = d[1] + d[3];", 1),
    # operation order and precision of the measure (caught only on inputs where float32 operations round)
    ("width_plus_one_before_subtraction", "float w = (far_x - near_x) + 1.0f;", "float w = (far_x + 1.0f) - near_x;", 1),
    ("height_plus_one_before_subtraction", "float h = (far_y - near_y) + 1.0f;", "float h = (far_y + 1.0f) - near_y;", 1),
    ("width_one_taken_from_near_edge", "float w = (far_x - near_x) + 1.0f;", "float w = far_x - (near_x - 1.0f);", 1),
    ("area_width_plus_one_before_subtraction", "float w = (b[2] - b[0]) + 1.0f;", "float w = (b[2] + 1.0f) - b[0];", 1),
    ("area_height_plus_one_before_subtraction", "float h = (b[3] - b[1]) + 1.0f;", "float h = (b[3] + 1.0f) - b[1];", 1),
    ("quotient_in_double", "return (w * h) / a;", "return (float)(((double)w * (double)h) / (double)a);", 1),
    ("measure_all_in_double",
     "    float a = box_area(bj);\n    return (w * h) / a;",
     "    double dw = ((double)far_x - (double)near_x) + 1.0; if (!(dw > 0.0)) dw = 0.0;\n"
     "    double dh = ((double)far_y - (double)near_y) + 1.0; if (!(dh > 0.0)) dh = 0.0;\n"
     "    double da = (((double)bj[2] - (double)bj[0]) + 1.0) * (((double)bj[3] - (double)bj[1]) + 1.0);\n"
     "    return (float)((dw * dh) / da);", 1),
    ("area_in_double_extents", "return w * h;\n}\n\n/* Overlap of victim",
     "return (float)((((double)b[2] - (double)b[0]) + 1.0) * (((double)b[3] - (double)b[1]) + 1.0));\n}\n\n/* Overlap of victim", 1),
    ("division_by_reciprocal", "return (w * h) / a;", "return (w * h) * (1.0f / a);", 1),
    ("quotient_rounded_down", "return (w * h) / a;",
     "float q = (w * h) / a; if ((double)q * (double)a > (double)(w * h)) { uint32_t u; memcpy(&u, &q, 4); u -= 1; memcpy(&q, &u, 4); } return q;", 1),
    # the selectable variants
    ("ex_extent_offset_before_subtraction",
     "static float extent(float lo, float hi, float offset) { return (hi - lo) + offset; }",
     "static float extent(float lo, float hi, float offset) { return (hi + offset) - lo; }", 1),
    ("ex_union_subtracts_first", "q = inter / ((area_i + area_j) - inter);", "q = inter / (area_i + (area_j - inter));", 1),
    ("ex_iou_in_double", "q = inter / ((area_i + area_j) - inter);",
     "q = (float)((double)inter / (((double)area_i + (double)area_j) - (double)inter));", 1),
    ("ex_union_forgets_intersection", "q = inter / ((area_i + area_j) - inter);", "q = inter / (area_i + area_j);", 1),
    ("ex_iou_divides_by_victim", "q = inter / ((area_i + area_j) - inter);", "q = inter / area_i;", 1),
    ("ex_measure_switch_inverted", "if (measure == 0) {", "if (measure != 0) {", 1),
    ("ex_strict_switch_inverted", "return strict ? (q > theta) : !(q < theta);", "return strict ? !(q < theta) : (q > theta);", 1),
    ("ex_strict_ignored", "return strict ? (q > theta) : !(q < theta);", "return !(q < theta);", 1),
    ("ex_ties_ignored_switch_dead", "if (ties ? !(scores[j] > scores[i]) : !outranks(scores, j, i)) return 0;",
     "if (!outranks(scores, j, i)) return 0;", 1),
    ("ex_ties_lets_equal_scores_through", "if (ties ? !(scores[j] > scores[i])", "if (ties ? !(scores[j] >= scores[i])", 1),
    ("ex_classes_ignored", "if (classes && classes[j] != classes[i]) return 0;", "", 1),
    ("ex_classes_inverted", "classes[j] != classes[i]", "classes[j] == classes[i]", 1),
    ("ex_offset_always_one", "static float extent(float lo, float hi, float offset) { return (hi - lo) + offset; }",
     "static float extent(float lo, float hi, float offset) { return (hi - lo) + 1.0f; }", 1),
    ("ex_offset_missing_in_area", "float area_j = extent(bj[0], bj[2], offset) * extent(bj[1], bj[3], offset);",
     "float area_j = (bj[2] - bj[0]) * (bj[3] - bj[1]);", 1),
    ("ex_width_not_floored", "float w = extent(left, right, offset);\n    if (!(w > 0.0f)) w = 0.0f;", "float w = extent(left, right, offset);", 1),
    ("ex_height_not_floored", "float h = extent(top, bottom, offset);\n    if (!(h > 0.0f)) h = 0.0f;", "float h = extent(top, bottom, offset);", 1),
    ("ex_greedy_counts_dead_boxes", "if (keep[j] && eliminates_ex(", "if (eliminates_ex(", 1),
    ("ex_greedy_switch_dead", "if (!greedy) {", "if (1) {", 1),
    ("ex_right_edge_is_max", "float right = bi[2] < bj[2] ? bi[2] : bj[2];", "float right = bi[2] > bj[2] ? bi[2] : bj[2];", 1),
    ("ex_top_edge_is_min", "float top = bi[1] > bj[1] ? bi[1] : bj[1];", "float top = bi[1] < bj[1] ? bi[1] : bj[1];", 1),
    ("ex_operands_transposed", "const float *bi = boxes + 4 * (size_t)i;\n    const float *bj = boxes + 4 * (size_t)j;",
     "const float *bi = boxes + 4 * (size_t)j;\n    const float *bj = boxes + 4 * (size_t)i;", 1),
]


@pytest.mark.parametrize("name,old,new,count", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, name, old, new, count):
    text = open(SOURCE).read()
    assert text.count(old) == count, f"mutation site for {name} not found exactly {count} time(s)"
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    lib = tmp_path / f"libmutant_{name}.so"
    subprocess.run(["gcc", *CFLAGS, str(src), "-o", str(lib)], check=True)
    mutant = Oracle(str(lib))
    def fails(pin):
        try:
            pin(mutant)
        except AssertionError:
            return True
        return False

    # one failing pin is enough
    assert any(fails(pin) for _, pin in ALL_PINS), f"no pin notices the planted mistake '{name}'"
