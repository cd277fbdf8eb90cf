"""Plants one mistake at a time in a COPY of the oracle's source (CPU only) and checks the pins notice.

This is what makes the pins trustworthy: a dropped abs, a wrong divisor, the
wrong rounding mode, an unfused multiply-add, a wrong scale or partial index,
a transposed operand -- each must fail at least one pin.  The real oracle is
untouched; mutants are compiled into a temporary directory.
"""
import os

import pytest

import oracle_pins
from oracle import equarx_oracle as o

MUTANTS = {
    # name: (text in the oracle's source, replacement)
    "no_abs": ("float m = fabsf(v[j]);", "float m = v[j];"),
    "divisor_128": ("scale = a / 127.0f;", "scale = a / 128.0f;"),
    "inv_from_scale": ("inv = 127.0f / a;", "inv = 1.0f / scale;"),
    "inv_128": ("inv = 127.0f / a;", "inv = 128.0f / a;"),
    "round_half_away": ("r = nearbyintf(r);", "r = roundf(r);"),
    "truncate": ("r = nearbyintf(r);", "r = truncf(r);"),
    "divide_instead_of_multiply": ("float r = v[j] * inv;", "float r = (scale > 0.0f) ? v[j] / scale : 0.0f;"),
    "no_tiny_threshold": ("if (a < 127.0f * FLT_MIN) {", "if (a == 0.0f) {"),
    "unfused_add": ("t[j] = fmaf((float)codes_in[at + j], scales_in[b], widen_bf16(local[at + j]));",
                    "t[j] = (float)codes_in[at + j] * scales_in[b] + widen_bf16(local[at + j]);"),
    "hop_subtracts": ("t[j] = fmaf((float)codes_in[at + j], scales_in[b], widen_bf16(local[at + j]));",
                      "t[j] = fmaf((float)codes_in[at + j], scales_in[b], -widen_bf16(local[at + j]));"),
    "hop_wrong_scale": ("t[j] = fmaf((float)codes_in[at + j], scales_in[b], widen_bf16(local[at + j]));",
                        "t[j] = fmaf((float)codes_in[at + j], scales_in[0], widen_bf16(local[at + j]));"),
    "hop_quantizes_local": ("t[j] = fmaf((float)codes_in[at + j], scales_in[b], widen_bf16(local[at + j]));",
                            "t[j] = fmaf((float)codes_in[at + j], scales_in[b], nearbyintf(widen_bf16(local[at + j]) * 64.0f) / 64.0f);"),
    "dequant_wrong_block": ("float d = (float)codes[j] * scales[j / B];", "float d = (float)codes[j] * scales[0];"),
    "dequant_f32_wrong_block": ("out[j] = (float)codes[j] * scales[j / B];", "out[j] = (float)codes[j] * scales[(j + 1) / B];"),
    "bf16_round_half_up": ("if (drop > 0x8000u || (drop == 0x8000u && (keep & 1u))) {", "if (drop >= 0x8000u) {"),
    "bf16_truncate": ("if (drop > 0x8000u || (drop == 0x8000u && (keep & 1u))) {", "if (0) {"),
    "chain_reuses_first_partial": ("equarx_oracle_hop(c_prev, s_prev, partials[i], n, B, c_next, s_next);",
                                   "equarx_oracle_hop(c_prev, s_prev, partials[0], n, B, c_next, s_next);"),
    "chain_skips_last": ("for (int32_t i = 1; i < P; ++i) {\n        equarx_oracle_hop(",
                         "for (int32_t i = 1; i < P - 1; ++i) {\n        equarx_oracle_hop("),
    "chain_no_swap": ("int8_t *tc = c_prev; c_prev = c_next; c_next = tc;", "int8_t *tc = c_prev; (void)tc;"),
    "chain_out_not_requantized": ("equarx_oracle_dequantize_bf16(c_prev, s_prev, n, B, out);",
                                  "equarx_oracle_dequantize_bf16(c_next, s_next, n, B, out);"),
    "f32_sum_in_f64": ("for (int32_t i = 1; i < P; ++i) acc = acc + widen_bf16(partials[i][j]);",
                       "double a2 = acc; for (int32_t i = 1; i < P; ++i) a2 += widen_bf16(partials[i][j]); acc = (float)a2;"),
    "stages_rs_off_uses_fma_path": ("t[j] = t[j] + widen_bf16(partials[i][at + j]);\n            }\n        }\n        if (quantize_ag)",
                                    "t[j] = t[j] - widen_bf16(partials[i][at + j]);\n            }\n        }\n        if (quantize_ag)"),
    "stages_always_quantizes_ag": ("        if (quantize_ag) {\n            quantize_block(t, len, c, &s);", "        if (1) {\n            quantize_block(t, len, c, &s);"),
    "stages_ignores_rs_knob": ("            if (quantize_rs) {", "            if (1) {"),
    "semi_wrong_half": ("    int32_t h = P / 2;", "    int32_t h = (P - 1) / 2;"),
    "semi_cw_first": ("for (int64_t j = 0; j < len; ++j) own[j] = widen_bf16(partials[0][at + j]);",
                      "for (int64_t j = 0; j < len; ++j) own[j] = widen_bf16(partials[0][at + j]);\n        if (h >= 1 && h + 1 <= P - 1) { for (int64_t j = 0; j < len; ++j) t[j] = widen_bf16(partials[h][at + j]); for (int32_t i = h - 1; i >= 1; --i) { quantize_block(t, len, c, &s); for (int64_t j = 0; j < len; ++j) t[j] = fmaf((float)c[j], s, widen_bf16(partials[i][at + j])); } quantize_block(t, len, c, &s); for (int64_t j = 0; j < len; ++j) own[j] = fmaf((float)c[j], s, own[j]); h = 0; }"),
    "semi_ccw_walks_backwards": ("for (int32_t i = h + 2; i <= P - 1; ++i) {", "for (int32_t i = P - 1; i >= h + 2; --i) {"),
    "semi_owner_quantized": ("for (int64_t j = 0; j < len; ++j) own[j] = widen_bf16(partials[0][at + j]);",
                             "for (int64_t j = 0; j < len; ++j) own[j] = nearbyintf(widen_bf16(partials[0][at + j]) * 32.0f) / 32.0f;"),
    "flat_unfused": ("acc[j] = fmaf((float)codes[r][at + j], scales[r][b], acc[j]);", "acc[j] = (float)codes[r][at + j] * scales[r][b] + acc[j];"),
    "flat_wrong_scale_block": ("acc[j] = fmaf((float)codes[r][at + j], scales[r][b], acc[j]);", "acc[j] = fmaf((float)codes[r][at + j], scales[r][0], acc[j]);"),
    "flat_skips_last_remote": ("for (int32_t r = 0; r < R; ++r) {", "for (int32_t r = 0; r + 1 < R || (R == 1 && r < 1); ++r) {"),
    "exact_sum_drops_last": ("for (int32_t i = 0; i < P; ++i) acc += (double)widen_bf16(partials[i][j]);",
                             "for (int32_t i = 0; i + 1 < P; ++i) acc += (double)widen_bf16(partials[i][j]);"),
}


def _failing_pins(lib, first_only=False):
    failed = []
    for pin in oracle_pins.ALL_PINS:
        try:
            pin(lib)
        except AssertionError:
            failed.append(pin.__name__)
            if first_only:
                break
    return failed


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_mutant(oracle, tmp_path, name):
    old, new = MUTANTS[name]
    with open(os.path.join(os.path.dirname(o.__file__), "equarx_oracle.c")) as f:
        src = f.read()
    assert src.count(old) == 1, f"mutation site for {name} not found exactly once"
    mutated = tmp_path / "mutant.c"
    mutated.write_text(src.replace(old, new))
    lib_path = o.build(force=True, src=str(mutated), lib=str(tmp_path / "libmutant.so"))
    lib = o.load(lib_path)
    failed = _failing_pins(lib, first_only=True)
    assert failed, f"no pin noticed the planted mistake {name!r}"


def test_unmutated_copy_passes(oracle, tmp_path):
    """The harness itself: an unchanged copy of the source passes every pin."""
    src = os.path.join(os.path.dirname(o.__file__), "equarx_oracle.c")
    lib = o.load(o.build(force=True, src=src, lib=str(tmp_path / "libcopy.so")))
    assert _failing_pins(lib) == []


# ----------------------------------------------------------------------------------------------------------
# The ring layout (shard split, per-shard rotation, pass-through of the semi-loop flag and the stage knobs) is
# composed in the oracle's Python front end, so its mistakes are planted there: a mutated copy of the module is
# imported from a temporary file and its reduce_ring / ring_order / shard_bounds stand in for the real ones.

PY_MUTANTS = {
    "ring_semi_owner_is_next_device": ("order = [(k + j) % P for j in range(P)]", "order = [(k + 1 + j) % P for j in range(P)]"),
    "ring_semi_walks_backwards": ("order = [(k + j) % P for j in range(P)]", "order = [(k - j) % P for j in range(P)]"),
    "ring_semi_not_rotated": ("order = [(k + j) % P for j in range(P)]", "order = list(range(P))"),
    "ring_semi_drops_ag_knob": ("reduce_semi_loop([arrs[d][lo:hi] for d in order], B, quantize_ag, lib=lib)",
                                "reduce_semi_loop([arrs[d][lo:hi] for d in order], B, True, lib=lib)"),
    "ring_drops_rs_knob": ("B, quantize_rs, quantize_ag, lib=lib)", "B, True, quantize_ag, lib=lib)"),
    "ring_drops_ag_knob": ("B, quantize_rs, quantize_ag, lib=lib)", "B, quantize_rs, True, lib=lib)"),
    "ring_swaps_knobs": ("B, quantize_rs, quantize_ag, lib=lib)", "B, quantize_ag, quantize_rs, lib=lib)"),
    "ring_ignores_semi_flag": ("        if semi:\n            order", "        if False:\n            order"),
    "ring_starts_at_own_device": ("return [(shard + 1 + i) % P for i in range(P)]", "return [(shard + i) % P for i in range(P)]"),
    "ring_walks_backwards": ("return [(shard + 1 + i) % P for i in range(P)]", "return [(shard - 1 - i) % P for i in range(P)]"),
    "strided_stages_drops_rs_knob": ("from_block_major(reduce_stages(moved, chunks, quantize_rs, quantize_ag, lib=lib), chunks)",
                                     "from_block_major(reduce_stages(moved, chunks, True, quantize_ag, lib=lib), chunks)"),
    "strided_stages_swaps_knobs": ("from_block_major(reduce_stages(moved, chunks, quantize_rs, quantize_ag, lib=lib), chunks)",
                                   "from_block_major(reduce_stages(moved, chunks, quantize_ag, quantize_rs, lib=lib), chunks)"),
    "strided_stages_not_moved_back": ("from_block_major(reduce_stages(moved, chunks, quantize_rs, quantize_ag, lib=lib), chunks)",
                                      "reduce_stages(moved, chunks, quantize_rs, quantize_ag, lib=lib)"),
    "strided_semi_is_the_full_loop": ("from_block_major(reduce_semi_loop(moved, chunks, quantize_ag, lib=lib), chunks)",
                                      "from_block_major(reduce_stages(moved, chunks, True, quantize_ag, lib=lib), chunks)"),
    "strided_semi_contiguous_blocks": ("from_block_major(reduce_semi_loop(moved, chunks, quantize_ag, lib=lib), chunks)",
                                       "reduce_semi_loop([_arr(p, np.uint16) for p in partials], chunks, quantize_ag, lib=lib)"),
    "ring_strided_shards_of_two_minishards": ("enumerate(shard_bounds(n, CHUNK * chunks, P))",
                                              "enumerate(shard_bounds(n, 2 * CHUNK * chunks, P))"),
    "ring_strided_no_rotation": ("shard = [arrs[d][lo:hi] for d in ring_order(P, k)]", "shard = [arrs[d][lo:hi] for d in range(P)]"),
    "ring_strided_owner_off_by_one": ("around = [arrs[(k + step) % P][lo:hi] for step in range(P)]",
                                      "around = [arrs[(k + 1 + step) % P][lo:hi] for step in range(P)]"),
    "ring_strided_walks_backwards": ("around = [arrs[(k + step) % P][lo:hi] for step in range(P)]",
                                     "around = [arrs[(k - step) % P][lo:hi] for step in range(P)]"),
    "ring_strided_semi_flag_ignored": ("        if not semi:\n            shard =", "        if True:\n            shard ="),
    "ring_strided_drops_rs_knob": ("reduce_stages_strided(shard, chunks, quantize_rs, quantize_ag, lib=lib)",
                                   "reduce_stages_strided(shard, chunks, True, quantize_ag, lib=lib)"),
    "ring_strided_contiguous_blocks": ("reduce_stages_strided(shard, chunks, quantize_rs, quantize_ag, lib=lib)",
                                       "reduce_stages(shard, chunks, quantize_rs, quantize_ag, lib=lib)"),
    "shards_not_on_block_boundaries": ("per = (nb + P - 1) // P\n    return [(min(n, k * per * B), min(n, (k + 1) * per * B)) for k in range(P)]",
                                       "per = (n + P - 1) // P\n    return [(min(n, k * per), min(n, (k + 1) * per)) for k in range(P)]"),
}


FRONT_END = ("reduce_ring", "ring_order", "shard_bounds", "reduce_stages_strided", "reduce_semi_loop_strided",
             "reduce_ring_strided")


def _mutated_front_end(tmp_path, old, new):
    import importlib.util

    with open(o.__file__) as f:
        src = f.read()
    assert src.count(old) == 1, "mutation site not found exactly once"
    path = tmp_path / "equarx_oracle_mutant.py"
    path.write_text(src.replace(old, new))
    spec = importlib.util.spec_from_file_location("equarx_oracle_mutant", str(path))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod._lib = o._L()           # the C library is the real, unmutated one
    return mod


@pytest.mark.parametrize("name", sorted(PY_MUTANTS))
def test_pins_catch_front_end_mutant(oracle, tmp_path, monkeypatch, name):
    mod = _mutated_front_end(tmp_path, *PY_MUTANTS[name])
    for attr in FRONT_END:
        monkeypatch.setattr(o, attr, getattr(mod, attr))
    failed = _failing_pins(None, first_only=True)
    assert failed, f"no pin noticed the planted mistake {name!r}"


def test_unmutated_front_end_copy_passes(oracle, tmp_path, monkeypatch):
    mod = _mutated_front_end(tmp_path, "import ctypes\n", "import ctypes  \n")
    for attr in FRONT_END:
        monkeypatch.setattr(o, attr, getattr(mod, attr))
    assert [p for p in ("pin_ring_order", "pin_ring_variants", "pin_strided_variants", "pin_ring_strided")
            if p in _failing_pins(None)] == []
