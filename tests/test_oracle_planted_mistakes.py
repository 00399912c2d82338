"""The oracle's pins fail when a plausible mistake is planted in the oracle (CPU only).

Each case edits one expression of oracle/litevar_oracle.c in a temporary copy, compiles the
copy, points the oracle's Python front-end at it and runs one named pin from the pin tests,
which must fail.  The unedited source, run through the same machinery, must pass every one
of those pins.  Nothing here touches the HIP library.
"""
import ctypes as C
import os
import subprocess

import pytest

import oracle
import oracle.oracle as front
import test_oracle_calibrate_band_pins as band_cal_pins
import test_oracle_calibrate_pins as cal_pins
import test_oracle_pins as pins
import test_oracle_qkv8_pins as q8_pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "litevar_oracle.c")

# name, (text in the source, replacement) pairs, the pin that must catch it
MISTAKES = [
    ("centre map without the half-cell shift",
     [("((2 * (int64_t)qy + 1) * sj) / (2 * sk)", "((int64_t)qy * sj) / sk"),
      ("((2 * (int64_t)qx + 1) * sj) / (2 * sk)", "((int64_t)qx * sj) / sk")],
     pins.test_golden_worked_example),
    ("same-scale tokens hidden (strict causal clause)",
     [("if (kj > qk) return 0;                 /* block-causal across scales */\n  if (kj < n_sink) return 1;",
       "if (kj >= qk && !(kj == qk && ky == qy && kx == qx)) return 0;\n  if (kj < n_sink) return 1;")],
     pins.test_golden_worked_example),
    ("diamond instead of square window",
     [("return dy <= r && dx <= r;", "return dy + dx <= r;")],
     pins.test_golden_worked_example),
    ("window centred on the key's row only (column clause dropped)",
     [("return dy <= r && dx <= r;", "return dy <= r;")],
     pins.test_golden_worked_example),
    ("softmax scale dropped",
     [("z[t] = sm_scale * s;", "z[t] = s;")],
     pins.test_full_window_reduces_to_dense_sdpa),
    ("rows and columns of a token swapped",
     [("*y_out = (int32_t)(local / scales[k]);", "*y_out = (int32_t)(local % scales[k]);"),
      ("*x_out = (int32_t)(local % scales[k]);", "*x_out = (int32_t)(local / scales[k]);")],
     pins.test_token_coords_row_major),
    ("weights not normalised",
     [("isnan(z[t]) ? 0.0 : z[t] / denom;", "isnan(z[t]) ? 0.0 : z[t];")],
     pins.test_softmax_rows_sum_to_one_and_respect_mask),
    ("softmax taken before masking (masked keys stay in the denominator)",
     [("c[t].k, c[t].y, c[t].x)) { z[t] = NAN; continue; }",
       "c[t].k, c[t].y, c[t].x)) { z[t] = NAN; double s0 = 0.0; for (int32_t d = 0; d < D; ++d) s0 += qrow[d] * Kd[t * D + d]; extra += exp(sm_scale * s0); continue; }"),
      ("double m = -INFINITY;", "double m = -INFINITY, extra = 0.0;"),
      ("double denom = 0.0;", "double denom = extra * 0.0; int use_extra = 1;"),
      ("for (int32_t d = 0; d < D; ++d) out[d] = 0.0;",
       "if (use_extra) denom += extra * exp(-m); for (int32_t d = 0; d < D; ++d) out[d] = 0.0;")],
     pins.test_softmax_rows_sum_to_one_and_respect_mask),
    ("K read transposed with V",
     [("s += qrow[d] * Kd[t * D + d];", "s += qrow[d] * Vd[t * D + d];")],
     pins.test_bruteforce_tiny_config),
    ("unconditional row copied onto the conditional one",
     [("double* src = o + (((int64_t)b * H + h) * Lq + a) * D;",
       "double* dst = o + (((int64_t)b * H + h) * Lq + a) * D;"),
      ("double* dst = o + (((int64_t)(b + half) * H + h) * Lq + a) * D;",
       "double* src = o + (((int64_t)(b + half) * H + h) * Lq + a) * D;")],
     pins.test_cfg_share_copies_cond_to_uncond),
    ("sharing table indexed by scale only",
     [("if (!share[(int64_t)h * K + kq]) continue;", "if (!share[kq]) continue;")],
     pins.test_cfg_share_copies_cond_to_uncond),
    ("leading dense parts ignored",
     [("if (kj < n_sink) return 1;", "if (kj < 0) return 1;")],
     pins.test_golden_worked_example),
    ("calibration ratio taken against the whole row instead of the part",
     [("if (found < 0 && (all == 0.0 || in / all >= r0)) found = r;",
       "if (found < 0 && (all == 0.0 || in / (all + 1.0) >= r0)) found = r;")],
     cal_pins.test_split_mass_between_centre_and_ring),
    ("quantiser scale as printed (no integer range)",
     [("const float s = ((mx - mn) * 0.5f) / qmax;", "const float s = fmaxf(fabsf(mx), fabsf(mn));")],
     q8_pins.test_hand_derived_rows),
    ("quantiser without the zero point",
     [("const float z = (mx + mn) * 0.5f;", "const float z = 0.0f * (mx + mn);")],
     q8_pins.test_hand_derived_rows),
    ("quantiser rounds half away from zero",
     [("t = nearbyintf(t);", "t = roundf(t);")],
     q8_pins.test_hand_derived_rows),
    ("quantiser truncates",
     [("t = nearbyintf(t);", "t = truncf(t);")],
     q8_pins.test_code_range_extremes_and_round_trip_bound),
    ("dequantisation forgets the zero point",
     [("out[r * D + d] = scale[r] * (double)codes[r * D + d] + zero[r];",
       "out[r * D + d] = scale[r] * (double)codes[r * D + d];")],
     q8_pins.test_constant_value_rows_are_exact),
    ("quantised attention leaves V unquantised",
     [("if (!rc) rc = lvo_dequantize_rows(codes, sc, zp, nk, D, vd);",
       "if (!rc) for (int64_t i = 0; i < nk * D; ++i) vd[i] = load_elem(v, dtype, i);")],
     q8_pins.test_quantised_attention_is_attention_of_the_dequantised_tensors_and_close_to_plain),
    ("calibration window one key too wide",
     [("for (int32_t i = 0; i < K * K; ++i) rad[i] = r;", "for (int32_t i = 0; i < K * K; ++i) rad[i] = r + 1;")],
     lambda: cal_pins.test_mass_at_a_known_distance_from_the_centre(1)),
    ("band calibration sums a part over its last key scale only",
     [("                for (int32_t j = first; j <= last; ++j)\n                  for (int32_t ky = 0; ky < scales[j]; ++ky)",
       "                for (int32_t j = last; j <= last; ++j)\n                  for (int32_t ky = 0; ky < scales[j]; ++ky)")],
     band_cal_pins.test_hand_placed_mass_in_the_merged_part),
    ("band calibration stops one radius late",
     [("          if (found < 0 && (all == 0.0 || in / all >= r0)) found = (int32_t)r;",
       "          if (found < 0 && (all == 0.0 || in / all >= r0)) found = (int32_t)r + 1;")],
     band_cal_pins.test_hand_placed_mass_in_the_last_part),
]


def _compile(text, path):
    c = path + ".c"
    with open(c, "w") as f:
        f.write(text)
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-w", "-o", path, c, "-lm"])
    lib = C.CDLL(path)
    lib.lvo_seq_len.restype = C.c_int64
    lib.lvo_scale_offset.restype = C.c_int64
    return lib


@pytest.fixture
def swap_oracle_library():
    """points the oracle's front-end at another build of the C file for one test"""
    front._L()                      # the real library is built and loaded first
    saved = front._lib

    def use(lib):
        front._lib = lib
    yield use
    front._lib = saved


def test_unedited_source_passes_the_named_pins(tmp_path, swap_oracle_library):
    swap_oracle_library(_compile(open(SRC).read(), str(tmp_path / "clean.so")))
    for _, _, pin in MISTAKES:
        pin()


@pytest.mark.parametrize("case", range(len(MISTAKES)), ids=[m[0] for m in MISTAKES])
def test_planted_mistake_fails_its_pin(case, tmp_path, swap_oracle_library):
    name, edits, pin = MISTAKES[case]
    text = open(SRC).read()
    for old, new in edits:
        assert text.count(old) == 1, f"{name}: source text to edit not found exactly once: {old!r}"
        text = text.replace(old, new)
    swap_oracle_library(_compile(text, str(tmp_path / f"planted{case}.so")))
    with pytest.raises((AssertionError, ValueError)):
        pin()
