"""The pins must notice a plausible mistake anywhere in the oracle.

(Planted mistakes are chosen so that the broken build still stays inside the arrays it is
given: the broken libraries run inside the test process.)

Each case below plants one mistake in a copy of oracle/mpo_ref.c (a dropped
term, a wrong sign or index, swapped operands, a rounding shortcut), builds it
into a scratch library on the CPU, and checks that at least one pin from
test_oracle_split.py / test_oracle_steps.py fails on it, while all of them
pass on the untouched source built the same way.
"""
import subprocess

import pytest

from oracle import build as obuild
from oracle import ref as oref

import test_oracle_rounding as tr
import test_oracle_split as ts
import test_oracle_steps as tp

SRC = open(obuild.SRC).read()

PINS = [
    ts.pins_golden_patterns,
    lambda r: ts.pins_split_value_definition(r, "bf16"),
    lambda r: ts.pins_split_value_definition(r, "fp16"),
    tp.pins_torch_optim,
    tp.pins_fp32_master_equivalence,
    tp.pins_fp32_master_sgd,
    tp.pins_exact_rational_adam,
    tp.pins_exact_rational_sgd,
    tp.pins_adam_first_step_closed_form,
    tp.pins_adam_constant_gradient,
    tp.pins_sgd_geometric_series,
    tp.pins_decay_only_steps,
    tp.pins_loss_scale_power_of_two,
    tp.pins_residual_carries_small_updates,
    tp.pins_mixed_formats,
    lambda r: ts.pins_partial_bits_value_definition(r, "bf16"),
    lambda r: ts.pins_partial_bits_value_definition(r, "fp16"),
    ts.pins_partial_bits_is_truncation,
    ts.pins_packed_storage,
    tp.pins_partial_bits_master_equivalence,
    tp.pins_partial_bits_torch_optim,
    tp.pins_grad_clip,
    tr.pins_philox,
    tr.pins_value_is_mode_independent,
    tr.pins_nearest_matches_library_cast,
    tr.pins_stochastic_statistics,
    tr.pins_stochastic_stream,
    tr.pins_trajectory_is_mode_independent,
    tr.pins_first_index,
    tr.pins_nearest_keeps_nan,
]

# (name, text in mpo_ref.c, what it is replaced with, occurrences expected)
MUTANTS = [
    ("update sign", "float w1 = w - upd;", "float w1 = w + upd;", 2),
    ("second moment not squared", "float o2gg = o2g * g;", "float o2gg = o2g;", 1),
    ("epsilon dropped", "float d = rootc + EPS;", "float d = rootc;", 1),
    ("epsilon inside the root", "float root = sqrtf(v1);", "float root = sqrtf(v1 + EPS);", 1),
    ("no first bias correction", "cfg->lr / (1.0 - pow(cfg->beta1, t))", "cfg->lr", 1),
    ("no second bias correction", "(float)sqrt(1.0 - pow(cfg->beta2, t))", "1.0f", 1),
    ("step count off by one", "pow(cfg->beta2, t)", "pow(cfg->beta2, t + 1.0)", 1),
    ("beta1 correction uses beta2", "pow(cfg->beta1, t)", "pow(cfg->beta2, t)", 1),
    ("decay kinds swapped", "if (cfg->decoupled_wd) {", "if (!cfg->decoupled_wd) {", 1),
    ("decoupled decay ignores lr", "1.0 - cfg->lr * cfg->weight_decay", "1.0 - cfg->weight_decay", 1),
    ("loss scale ignored", "g = g * IS;", "g = g * 1.0f;", 2),
    ("loss scale multiplied", "(float)(1.0 / cfg->loss_scale)", "(float)(cfg->loss_scale)", 2),
    ("moment coefficients swapped", "float b1m = B1 * m[i];", "float b1m = O1 * m[i];", 1),
    ("first moment not stored", "m[i] = m1;", "m[i] = m[i];", 1),
    ("m and v swapped on store", "v[i] = v1;", "v[i] = m1;", 1),
    ("momentum with dampening", "b = mub + g;", "b = mub + (1.0f - MU) * g;", 1),
    ("momentum buffer not stored", "buf[i] = b;", "", 1),
    ("sgd decay dropped", "float wdw = WD * w;\n            g = g + wdw;\n        }\n        float b = g;",
     "float wdw = WD * w;\n            g = g + 0.0f * wdw;\n        }\n        float b = g;", 1),
    ("fused multiply-add in m", "float m1 = b1m + o1g;", "float m1 = fmaf(O1, g, b1m);", 1),
    ("double-precision quotient", "float upd = SS * q;",
     "float upd = (float)((double)SS * ((double)m1 / (double)d));", 1),
    ("bf16 hi rounded to nearest", "*hi = (uint16_t)(b >> 16);", "*hi = (uint16_t)((b + 0x8000u) >> 16);", 1),
    ("bf16 merge halves swapped", "((uint32_t)hi << 16) | (uint32_t)res", "((uint32_t)res << 16) | (uint32_t)hi", 1),
    ("bf16 residual one bit short", "*res = (uint16_t)(b & 0xFFFFu);", "*res = (uint16_t)(b & 0x7FFFu);", 1),
    ("fp16 split bias", "(uint32_t)(e + 15) << 10", "(uint32_t)(e + 16) << 10", 1),
    ("fp16 merge bias", "((E + 112u) << 23)", "((E + 111u) << 23)", 1),
    ("fp16 residual mask", "*res = (uint16_t)(M & 0x1FFFu);", "*res = (uint16_t)(M & 0x0FFFu);", 1),
    ("fp16 subnormal shift", "int shift = -14 - e;", "int shift = -15 - e;", 1),
    ("fp16 subnormal scale", "ldexpf((float)((k << 13) | r), -37)", "ldexpf((float)((k << 13) | r), -36)", 1),
    ("fp16 no saturation", "if (e > 15) {", "if (e > 16) {", 1),
    ("fp16 sign lost in subnormal merge", "return s ? -mag : mag;", "return mag;", 1),
    ("partial bits: kept bits left-aligned on load", "uint16_t full = (uint16_t)(kept << (L->full - L->kept));",
     "uint16_t full = (uint16_t)(kept << (16 - L->kept));", 1),
    ("partial bits: trailing bits kept instead of leading", "uint16_t kept = (uint16_t)(res_full >> (L->full - L->kept));",
     "uint16_t kept = (uint16_t)(res_full & ((1u << L->kept) - 1u));", 1),
    ("partial bits: rounds up", "uint16_t kept = (uint16_t)(res_full >> (L->full - L->kept));",
     "uint16_t kept = (uint16_t)((res_full + (L->kept < L->full ? (1u << (L->full - L->kept - 1)) : 0u)) >> (L->full - L->kept));", 1),
    ("partial bits: fp16 uses the bf16 width", "L.full = fmt == MPO_REF_FP16 ? 13 : 16;", "L.full = 16;", 1),
    ("packed: pieces in the wrong order", "    if (S & 8) { left -= 8; plane_put(plane, i, 8, (r >> left) & 0xFFu); plane += round16(n); }",
     "    if (S & 8) { plane_put(plane, i, 8, r & 0xFFu); plane += round16(n); }", 1),
    ("packed: planes not aligned", "static uint64_t round16(uint64_t x) { return (x + 15u) / 16u * 16u; }",
     "static uint64_t round16(uint64_t x) { return x; }", 1),
    ("packed: high nibble first", "    return (plane[bit / 8] >> (bit % 8)) & ((1u << w) - 1u);",
     "    return (plane[bit / 8] >> ((8 - w) - bit % 8)) & ((1u << w) - 1u);", 1),
    ("packed: put clobbers the neighbours", "    plane[bit / 8] = (uint8_t)((plane[bit / 8] & ~mask) | ((x << (bit % 8)) & mask));",
     "    plane[bit / 8] = (uint8_t)((x << (bit % 8)) & mask);", 1),
    ("packed: pieces read in another order than written",
     "    if (S & 4) { r = (r << 4) | plane_get(plane, i, 4); plane += round16((n + 1) / 2); }\n    if (S & 2) { r = (r << 2) | plane_get(plane, i, 2); plane += round16((n + 3) / 4); }",
     "    if (S & 2) { r = (r << 2) | plane_get(plane, i, 2); }\n    if (S & 4) { r = (r << 4) | plane_get(plane, i, 4); }", 1),
    ("packed: the 1-bit plane starts inside the 2-bit plane", " plane += round16((n + 3) / 4); }", " }", 2),
    ("packed: 1-bit piece not the last bit", "    if (S & 1) { left -= 1; plane_put(plane, i, 1, (r >> left) & 0x1u); }",
     "    if (S & 1) { plane_put(plane, i, 1, (r >> (S - 1)) & 0x1u); }", 1),
    ("packed: stochastic flag not among the stored bits", "    if (packed && round == MPO_REF_STOCHASTIC) L.kept = res_bits - 1;\n", "", 1),
    ("clip: lower bound missing", "            if (g < -CLIP) g = -CLIP;\n", "", 2),
    ("clip: applied to the scaled gradient", "        g = g * IS;\n        if (has_clip) {                    /* Sec. 4.1: element-wise clipping inside the step */\n            if (g > CLIP) g = CLIP;\n            if (g < -CLIP) g = -CLIP;\n        }\n",
     "        if (has_clip) {\n            if (g > CLIP) g = CLIP;\n            if (g < -CLIP) g = -CLIP;\n        }\n        g = g * IS;\n", 2),
    ("rounding: value not un-rounded", "*hi_trunc = (uint16_t)(hi[i] - was_rounded_up);", "*hi_trunc = hi[i];", 1),
    ("rounding: probability inverted", "draw(L, i) < res_full;", "draw(L, i) >= res_full;", 1),
    ("rounding: flag in the wrong bit", "kept = (uint16_t)(kept | (up << L->kept));", "kept = (uint16_t)(kept | (up << 15));", 1),
    ("rounding: step not in the counter", "(uint32_t)(block >> 32), L->step32, L->tensor_id", "(uint32_t)(block >> 32), 0u, L->tensor_id", 1),
    ("rounding: tensor not in the counter", "(uint32_t)(block >> 32), L->step32, L->tensor_id", "(uint32_t)(block >> 32), L->step32, 0u", 1),
    ("rounding: one draw per block of four", "return out[i % 4] >> (32 - L->full);", "return out[0] >> (32 - L->full);", 1),
    ("rounding: low bits of the draw", "return out[i % 4] >> (32 - L->full);", "return out[i % 4] & ((1u << L->full) - 1u);", 1),
    ("rounding: nearest at a quarter", "up = !is_nan16(hi_trunc, L->fmt) && ((res_full >> (L->full - 1)) & 1);",
     "up = !is_nan16(hi_trunc, L->fmt) && ((res_full >> (L->full - 2)) != 0);", 1),
    ("rounding: nearest rounds a NaN pattern up", "up = !is_nan16(hi_trunc, L->fmt) && ((res_full >> (L->full - 1)) & 1);",
     "up = (res_full >> (L->full - 1)) & 1;", 1),
    ("rounding: nearest un-rounds a NaN pattern", "was_rounded_up = !is_nan16(hi[i], L->fmt) && ((full >> (L->full - 1)) & 1);",
     "was_rounded_up = (full >> (L->full - 1)) & 1;", 1),
    ("rounding: infinity counted as a NaN", "(uint16_t)(h & 0x7FFFu) > (fmt == MPO_REF_FP16 ? 0x7C00u : 0x7F80u)",
     "(uint16_t)(h & 0x7FFFu) >= (fmt == MPO_REF_FP16 ? 0x7C00u : 0x7F80u)", 1),
    ("rounding: position of the slice ignored", "    i += L->first;\n", "", 1),
    ("rounding: position of the slice counted in blocks", "    i += L->first;\n", "    i += 4 * L->first;\n", 1),
    ("rounding: stochastic may overflow", "(uint16_t)(hi_trunc & 0x7FFFu) < max_finite_hi(L->fmt) && draw(L, i) < res_full;",
     "draw(L, i) < res_full;", 1),
    ("rounding: philox multiplier", "(uint64_t)0xCD9E8D57u * c2", "(uint64_t)0xCD9E8D57u * c0", 1),
    ("rounding: philox key schedule", "k1 += 0xBB67AE85u;", "k1 += 0x9E3779B9u;", 1),
    ("rounding: philox nine rounds", "for (int round = 0; round < 10; ++round) {", "for (int round = 0; round < 9; ++round) {", 1),
]


def _build(tmp_path, name, text):
    c = tmp_path / (name + ".c")
    c.write_text(text)
    so = tmp_path / (name + ".so")
    flags = [f for f in obuild.CFLAGS if f != "-Werror"] + ["-w"]
    subprocess.check_call(["gcc", *flags, "-I", obuild.HERE, "-o", str(so), str(c), "-lm"])
    return oref.Oracle(str(so))


def _failing_pins(lib, first_only=False):
    failed = []
    for i, pin in enumerate(PINS):
        if first_only and failed:
            break
        try:
            pin(lib)
        except (AssertionError, ValueError, OverflowError, ZeroDivisionError, TypeError):   # NaN/inf reaching exact arithmetic counts
            failed.append(i)
    return failed


def test_untouched_source_passes_every_pin(tmp_path):
    assert _failing_pins(_build(tmp_path, "clean", SRC)) == []


@pytest.mark.parametrize("name,old,new,count", MUTANTS, ids=[m[0].replace(" ", "_") for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new, count):
    assert SRC.count(old) == count, "mutation site moved: %r" % old
    lib = _build(tmp_path, "mutant", SRC.replace(old, new))
    assert _failing_pins(lib, first_only=True), "no pin noticed: " + name
