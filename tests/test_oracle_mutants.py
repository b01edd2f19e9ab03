"""The pins must be able to fail: plant one plausible mistake at a time in a
copy of the oracle's C source (CPU only), rebuild it, and require that the pin
suite rejects it."""
import os
import subprocess
import sys

import pytest

from oracle import build as obuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (name, text in oracle/cdsgd_oracle.c, replacement)
MUTANTS = [
    ("strict_threshold", "if (a >= t) {", "if (a > t) {"),
    ("strict_negative", "} else if (a <= -t) {", "} else if (a < -t) {"),
    ("residual_wrong_sign", "residual[e] = a + t;", "residual[e] = a - t;"),
    ("residual_dropped_on_send", "residual[e] = a - t;", "residual[e] = 0.0f;"),
    ("compare_gradient_not_sum", "float a = residual[e] + grad[e];\n        if (a >= t) {",
     "float a = residual[e] + grad[e];\n        if (grad[e] >= t) {"),
    ("codes_swapped", "if (code == ORACLE_CODE_POS) return t;", "if (code == ORACLE_CODE_POS) return -t;"),
    ("code3_decodes_nonzero", "if (code == ORACLE_CODE_NEG) return -t;", "if (code >= ORACLE_CODE_NEG) return -t;"),
    ("big_endian_fields", "<< (2 * (e % 16));", "<< (2 * (15 - e % 16));"),
    ("unpack_wrong_shift", "(word[e / 16] >> (2 * (e % 16))) & 3u);\n}", "(word[e / 16] >> (e % 16)) & 3u);\n}"),
    ("stale_pad_bits", "for (size_t w = 0; w < nw; ++w) word[w] = 0u;", "(void)nw;"),
    ("sum_reverse_order", "for (int j = 0; j < num_workers; ++j) {\n            uint8_t c",
     "for (int j = num_workers - 1; j >= 0; --j) {\n            uint8_t c"),
    ("sum_skips_a_worker", "for (int j = 0; j < num_workers; ++j) s = s + grad[j][e];",
     "for (int j = 1; j < num_workers; ++j) s = s + grad[j][e];"),
    ("no_average", "float scale = lr_global / (float)num_workers;", "float scale = lr_global;"),
    ("update_sign", "fmaf(-scale, agg[e], w)", "fmaf(scale, agg[e], w)"),
    ("local_two_roundings", "fmaf(-lr_local, grad_local[e], w)", "(w - lr_local * grad_local[e])"),
    ("local_sees_new_global", "float w = w_global[e];\n        if (w_local && grad_local) w_local[e] = fmaf(-lr_local, grad_local[e], w);\n        if (agg) w_global[e] = fmaf(-scale, agg[e], w);",
     "float w = w_global[e];\n        if (agg) { w = fmaf(-scale, agg[e], w); w_global[e] = w; }\n        if (w_local && grad_local) w_local[e] = fmaf(-lr_local, grad_local[e], w);"),
    ("local_uses_aggregate_rate", "fmaf(-lr_local, grad_local[e], w)", "fmaf(-scale, grad_local[e], w)"),
    ("mode_inverted", "int compressed = (count % k) != 0;", "int compressed = (count % k) == 0;"),
    ("count_starts_at_one", "int compressed = (count % k) != 0;", "int compressed = ((count + 1) % k) != 0;"),
    ("residual_flushed_on_correction", "oracle_full_sum(grad, num_workers, agg, n);",
     "oracle_full_sum(grad, num_workers, agg, n); for (int j = 0; j < num_workers; ++j) memset(residual[j], 0, n * sizeof(float));"),
    ("shared_residual", "oracle_quantize(grad[j], residual[j], code_scratch, n, t);",
     "oracle_quantize(grad[j], residual[0], code_scratch, n, t);"),
    ("warmup_copy_one_pass_late", "if (i == n - 1) memcpy(w_local, w_global, n_elems * sizeof(float));",
     "if (i == n) memcpy(w_local, w_global, n_elems * sizeof(float));"),
    ("warmup_copy_before_update", "    oracle_update(w_global, NULL, NULL, agg, n_elems, lr_local, lr_global, num_workers);\n    if (i == n - 1) memcpy",
     "    if (i == n - 1) memcpy(w_local, w_global, n_elems * sizeof(float));\n    oracle_update(w_global, NULL, NULL, agg, n_elems, lr_local, lr_global, num_workers);\n    if (0) memcpy"),
    ("warmup_local_update_every_pass", "if (i == n) {\n        if (n == 0)", "if (i <= n) {\n        if (n == 0)"),
    ("warmup_local_uses_global_rate", "w_local[e] = fmaf(-lr_local, grad[self][e], w_local[e]);",
     "w_local[e] = fmaf(-lr_global, grad[self][e], w_local[e]);"),
    # the two rejected hand-over readings: the local buffer as the caller left it (n == 0), and the
    # first formal local update made in place on what the warm-up left in the local buffer
    ("warmup_n0_base_is_callers_buffer",
     "if (n == 0) memcpy(w_local, w_global, n_elems * sizeof(float)); /* the copy no earlier pass could make */", ""),
    ("first_formal_local_update_in_place",
     "    return oracle_step(w_global, w_local, residual, grad, word, agg, code_scratch, n_elems, num_workers, self,\n"
     "                       iter - warmup_n - 1,",
     "    if (iter == warmup_n + 1) {\n"
     "        float *keep = w_local;\n"
     "        for (size_t e = 0; e < n_elems; ++e) keep[e] = fmaf(-lr_local, grad[self][e], keep[e]);\n"
     "        oracle_full_sum(grad, num_workers, agg, n_elems);\n"
     "        oracle_update(w_global, NULL, NULL, agg, n_elems, lr_local, lr_global, num_workers);\n"
     "        return 2;\n"
     "    }\n"
     "    return oracle_step(w_global, w_local, residual, grad, word, agg, code_scratch, n_elems, num_workers, self,\n"
     "                       iter - warmup_n - 1,"),
    ("warmup_one_pass_short", "if (iter <= warmup_n) {", "if (iter < warmup_n) {"),
    ("formal_count_not_reset", "iter - warmup_n - 1, k, t,", "iter, k, t,"),
    ("cost_correction_case_swapped", "double phi_cd = (i % k != 0) ? delta + psi : phi;",
     "double phi_cd = (i % k == 0) ? delta + psi : phi;"),
    ("cost_local_is_sum", "double t_loc = tau > phi ? tau : phi;", "double t_loc = tau + phi;"),
    ("cost_bit_forgets_delta", "double t_bit = tau + delta + psi;", "double t_bit = tau + psi;"),
    ("cost_cd_is_min", "double t_cd = tau > phi_cd ? tau : phi_cd;", "double t_cd = tau < phi_cd ? tau : phi_cd;"),
    ("sparse_bitmap_msb_first", "seg[i / 32] |= 1u << (i % 32);", "seg[i / 32] |= 1u << (31 - i % 32);"),
    ("sparse_segment_stride_256", "uint32_t *seg = sparse + 264 * s;", "uint32_t *seg = sparse + 256 * s;"),
    ("sparse_count_misses_bitmap", "seg_words[s] = 8u + count;", "seg_words[s] = count;"),
    ("sparse_zero_words_travel", "if (w < nw && word[w] != 0u) {", "if (w < nw) {"),
    ("sparse_decode_counts_own_bit", "for (size_t b = 0; b < i; ++b) before", "for (size_t b = 0; b <= i; ++b) before"),
    ("sparse_decode_ignores_bitmap", "if ((seg[i / 32] >> (i % 32)) & 1u) {", "if (1) {"),
    ("local_uses_wrong_worker", "oracle_update(w_global, w_local, grad[self],", "oracle_update(w_global, w_local, grad[num_workers - 1 - self],"),
]


def test_mutant_list_matches_source():
    src = open(obuild.SRC).read()
    for name, old, _ in MUTANTS:
        assert src.count(old) == 1, "mutant %s: anchor text not found exactly once" % name


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_reject_mutant(tmp_path, name, old, new):
    src = open(obuild.SRC).read()
    assert src.count(old) == 1
    csrc = tmp_path / "mutant.c"
    csrc.write_text(src.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.run(["gcc", *[f for f in obuild.CFLAGS if not f.startswith("-W")], str(csrc), "-o", str(lib), "-lm"],
                   check=True)
    env = dict(os.environ, CDSGD_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        "-k", "not bruteforce or 0.125"],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 1, "pins did not catch mutant %s:\n%s" % (name, r.stdout[-1500:])
    assert "failed" in r.stdout
