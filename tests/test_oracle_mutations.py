"""Are the pins sharp?  Each case plants one plausible mistake in a copy of the
oracle's C source (on the CPU), compiles it, and checks that the pin battery of
test_oracle_pins.py fails for it.  The unmodified source must pass the battery."""
import os
import subprocess

import pytest

from oracle import pier_oracle as O
import test_oracle_pins as pins

SRC = open(os.path.join(os.path.dirname(O.__file__), "pier_oracle.c")).read()

# (name, text in the oracle, mistaken replacement)
MUTATIONS = [
    ("drop weight decay", "+ wd * (*p);", ";"),
    ("decay with the wrong sign", "+ wd * (*p);", "- wd * (*p);"),
    ("ascent instead of descent", "*p = *p - lr * u;", "*p = *p + lr * u;"),
    ("eps inside the root", "mh / (sqrtf(vh) + eps)", "mh / sqrtf(vh + eps)"),
    ("no bias correction of m", "float mh = mn / bc1;", "float mh = mn;"),
    ("no bias correction of v", "float vh = vn / bc2;", "float vh = vn;"),
    ("bias correction one step late", "pow((double)beta1, (double)step)", "pow((double)beta1, (double)(step - 1) + 1e-9)"),
    ("betas swapped in the moments", "float mn = beta1 * (*m) + om1 * g;", "float mn = beta2 * (*m) + om2 * g;"),
    ("first moment of g squared", "om1 * g;", "om1 * g * g;"),
    ("second moment of g, not g^2", "(om2 * g) * g;", "(om2 * g);"),
    ("moments not stored", "*m = mn;", ""),
    ("decay uses updated theta", "float u = mh / (sqrtf(vh) + eps) + wd * (*p);\n    *p = *p - lr * u;",
     "*p = *p - lr * (mh / (sqrtf(vh) + eps));\n    *p = *p - lr * wd * (*p) * 40.0f;"),
    ("bf16 shifted wrong", "(uint32_t)g[i] << 16", "(uint32_t)g[i] << 15"),
    ("grad_scale ignored", "if (grad_scale != 1.0f) g = g * grad_scale;", ""),
    ("clip: norm without the root", "(sqrt(sumsq) + 1e-6)", "(sumsq + 1e-6)"),
    ("clip: epsilon dropped", "(sqrt(sumsq) + 1e-6)", "(sqrt(sumsq))"),
    ("clip: always scales", "return coef < 1.0 ? (float)coef : 1.0f;", "return (float)coef;"),
    ("clip: sum of values, not squares", "acc = acc + (double)g[i] * (double)g[i];", "acc = acc + (double)g[i];"),
    ("clip: accumulator restarts per tensor", "double pier_oracle_sumsq(const float* g, int64_t n, double acc)\n{",
     "double pier_oracle_sumsq(const float* g, int64_t n, double acc)\n{ acc = 0;"),
    ("clip: bf16 shifted wrong", "uint32_t bits = (uint32_t)g[i] << 16;\n        float gf;\n        memcpy(&gf, &bits, sizeof gf);\n        acc",
     "uint32_t bits = (uint32_t)g[i] << 15;\n        float gf;\n        memcpy(&gf, &bits, sizeof gf);\n        acc"),
    ("bf16: truncation instead of rounding", "out[i] = (uint16_t)((b + 0x7FFFu + lsb) >> 16);", "out[i] = (uint16_t)(b >> 16);"),
    ("bf16: ties away from zero", "out[i] = (uint16_t)((b + 0x7FFFu + lsb) >> 16);", "out[i] = (uint16_t)((b + 0x8000u) >> 16);"),
    ("bf16: NaN not quieted", "if ((b & 0x7FFFFFFFu) > 0x7F800000u) { out[i] = 0x7FC0; continue; }", ""),
    ("inner lr: cosine over T instead of T - W", "double progress = ((double)t - W) / ((double)T - W);", "double progress = ((double)t - W) / ((double)T);"),
    ("inner lr: warmup from lr_min", "return (float)(hi * (double)t / W);", "return (float)(lo + (hi - lo) * (double)t / W);"),
    ("inner lr: full cosine period", "cos(pi * progress)", "cos(2.0 * pi * progress)"),
    ("inner lr: decays to zero", "(float)(lo + cosine_share(progress) * (hi - lo))", "(float)(cosine_share(progress) * hi)"),
    ("sum instead of mean", "float d = s * invG;", "float d = s;"),
    ("anchor minus model", "s = s + (theta[g][i] - a[i]);", "s = s + (a[i] - theta[g][i]);"),
    ("first group only", "for (int g = 0; g < G; ++g) s = s + (theta[g][i] - a[i]);",
     "for (int g = 0; g < 1; ++g) s = s + (theta[g][i] - a[i]) * (float)G;"),
    ("momentum without mu", "float Mn = mu * M[i] + d;", "float Mn = M[i] + d;"),
    ("heavy ball, no Nesterov term", "lr * (mu * Mn + d)", "lr * Mn"),
    ("look-ahead uses the old momentum",
     "M[i] = Mn;\n        float x = a[i] + lr * (mu * Mn + d);",
     "float Mold = M[i]; M[i] = Mn;\n        float x = a[i] + lr * (mu * Mold + d);"),
    ("lr on the gradient only", "a[i] + lr * (mu * Mn + d)", "a[i] + (mu * Mn + lr * d)"),
    ("momentum not stored", "M[i] = Mn;", ""),
    ("groups not re-synchronised", "for (int g = 0; g < G; ++g) theta[g][i] = x;", "theta[0][i] = x;"),
    ("anchor not advanced", "a[i] = x;", ""),
    ("warmup applies the step", "if (phase == 1) pier_sync", "if (phase == 1 || phase == 0) pier_sync"),
    ("warmup keeps the old anchor", "a[i] = model[i];", ""),
    ("warmup anchor is the fp32 mean of the copies (3 theta / 3 is not theta)",
     "else lazy_start_sync(theta[0], a, M, n, mu);",
     "else { lazy_start_sync(theta[0], a, M, n, mu);"
     " for (int64_t i = 0; i < n; ++i) { float s2 = 0.0f; for (int g = 0; g < G; ++g) s2 = s2 + theta[g][i];"
     " a[i] = s2 * (1.0f / (float)G); } }"),
    ("warmup difference averaged over the copies",
     "float delta = model[i] - a[i];\n        M[i] = mu * M[i] + delta;",
     "float delta = ((model[i] - a[i]) + (model[i] - a[i]) + (model[i] - a[i])) * (1.0f / 3.0f);\n        M[i] = mu * M[i] + delta;"),
    ("warmup difference with the wrong sign", "float delta = model[i] - a[i];", "float delta = a[i] - model[i];"),
    ("warmup momentum without mu", "M[i] = mu * M[i] + delta;", "M[i] = M[i] + delta;"),
    ("warmup momentum overwritten, not accumulated", "M[i] = mu * M[i] + delta;", "M[i] = delta;"),
    ("warmup writes the model", "a[i] = model[i];", "a[i] = model[i]; ((float*)model)[i] = a[i] + delta;"),
    ("mu bands swapped", "return 0.99f;", "return 0.95f;"),
    ("mu boundary at 15% closed on the wrong side", "if (reached(t, T, k15pct)) return 0.95f;", "if (passed(t, T, k15pct)) return 0.95f;"),
    ("mu: 15% typed as 3/25", "k15pct = {3, 20}", "k15pct = {3, 25}"),
    ("lr plateau values swapped", "if (reached(t, T, k80pct)) return 0.9f;\n    if (reached(t, T, k20pct)) return 1.1f;",
     "if (reached(t, T, k80pct)) return 1.1f;\n    if (reached(t, T, k20pct)) return 0.9f;"),
    ("lr ramp from 0.1 T as fraction of T", "(double)above / (double)T", "(double)above / (double)(10 * T)"),
    ("lr ramp measured from 0", "int64_t above = 10 * t - T;", "int64_t above = 10 * t;"),
    ("lazy start ends one step early", "return passed(t, T, k10pct) ? 1 : 0;", "return reached(t, T, k10pct) ? 1 : 0;"),
    ("warmup mu taken from the decay schedule", "if (*phase == 0) { *mu = 0.9f; *lr = 0.0f; }",
     "if (*phase == 0) { *mu = pier_oracle_mu(t, T); *lr = 0.0f; }"),
    ("v bias-corrected with beta1's factor", "float vh = vn / bc2;", "float vh = vn / bc1;"),
    ("om1 from beta2", "float om1 = 1.0f - beta1;", "float om1 = 1.0f - beta2;"),
    ("om2 from beta1", "float om2 = 1.0f - beta2;", "float om2 = 1.0f - beta1;"),
    ("bias correction one step early", "pow((double)beta2, (double)step)", "pow((double)beta2, (double)(step + 1))"),
    ("decay not scaled by lr", "float u = mh / (sqrtf(vh) + eps) + wd * (*p);\n    *p = *p - lr * u;",
     "float u = mh / (sqrtf(vh) + eps);\n    *p = *p - lr * u - wd * (*p);"),
    ("clip coefficient inverted", "double coef = (double)max_norm / (sqrt(sumsq) + 1e-6);",
     "double coef = (sqrt(sumsq) + 1e-6) / (double)max_norm;"),
    ("clip: squares formed in float", "acc = acc + (double)g[i] * (double)g[i];", "acc = acc + (double)(g[i] * g[i]);"),
    ("clip: accumulated in float", "acc = acc + (double)g[i] * (double)g[i];", "acc = (double)((float)acc + g[i] * g[i]);"),
    ("outer: rate on the momentum term only", "a[i] + lr * (mu * Mn + d)", "a[i] + (lr * mu * Mn + d)"),
    ("outer: mean over G-1", "float invG = 1.0f / (float)G;", "float invG = 1.0f / (float)(G > 1 ? G - 1 : 1);"),
    ("outer: mu squared in the look-ahead", "lr * (mu * Mn + d)", "lr * (mu * mu * Mn + d)"),
    ("outer: anchor moved by the plain difference", "float x = a[i] + lr * (mu * Mn + d);", "float x = a[i] + d;"),
    ("lr: 80% breakpoint at 85%", "k80pct = {4, 5}", "k80pct = {17, 20}"),
    ("lr: plateau 1.0 instead of 1.1", "if (reached(t, T, k20pct)) return 1.1f;", "if (reached(t, T, k20pct)) return 1.0f;"),
    ("lr: final value 1.0 instead of 0.9", "if (reached(t, T, k80pct)) return 0.9f;", "if (reached(t, T, k80pct)) return 1.0f;"),
    ("mu 0.999 instead of 0.99", "return 0.99f;", "return 0.999f;"),
    ("mu: 20% typed as 1/4", "k20pct = {1, 5}", "k20pct = {1, 4}"),
    ("mu: 10% typed as 1/8", "k10pct = {1, 10}", "k10pct = {1, 8}"),
    ("inner lr: warmup one iteration late", "return (float)(hi * (double)t / W);", "return (float)(hi * (double)(t - 1) / W);"),
    ("inner lr: lr_min reached half way", "double progress = ((double)t - W) / ((double)T - W);",
     "double progress = 2.0 * ((double)t - W) / ((double)T - W); if (progress > 1.0) progress = 1.0;"),
    ("bf16: rounds the magnitude up always", "out[i] = (uint16_t)((b + 0x7FFFu + lsb) >> 16);", "out[i] = (uint16_t)((b + 0xFFFFu) >> 16);"),
    ("bf16 gradient: low half used", "uint32_t bits = (uint32_t)g[i] << 16;\n        float gf;\n        memcpy(&gf, &bits, sizeof gf);\n        adamw_one",
     "uint32_t bits = (uint32_t)g[i];\n        float gf;\n        memcpy(&gf, &bits, sizeof gf);\n        adamw_one"),
    ("lazy start: momentum from the old model only", "float delta = model[i] - a[i];", "float delta = -a[i];"),
    ("warmup scalars: rate not zero", "if (*phase == 0) { *mu = 0.9f; *lr = 0.0f; }",
     "if (*phase == 0) { *mu = 0.9f; *lr = pier_oracle_outer_lr(t, T) + 0.5f; }"),
]


def battery():
    calls = [
        (pins.test_adamw_first_step_closed_form_hand_case, ()),
        (pins.test_adamw_constant_gradient_closed_form, (10,)),
        (pins.test_adamw_matches_torch_library, (pins.HP,)),
        (pins.test_adamw_bf16_gradients_widen_exactly, ()),
        (pins.test_adamw_grad_scale_is_a_gradient_multiplier, ()),
        (pins.test_bf16_rounding_matches_the_library_and_the_definition, ()),
        (pins.test_inner_lr_schedule_endpoints_and_library_cosine, ()),
        (pins.test_clip_hand_case_and_closed_form, ()),
        (pins.test_clip_matches_torch_clip_grad_norm, ()),
        (pins.test_outer_single_group_unit_rate_returns_the_model, ()),
        (pins.test_outer_unit_rate_no_momentum_is_the_replica_mean, ()),
        (pins.test_lazy_start_sync_returns_the_model_bit_for_bit, (1,)),
        (pins.test_lazy_start_sync_returns_the_model_bit_for_bit, (3,)),
        (pins.test_lazy_start_sync_returns_the_model_bit_for_bit, (8,)),
        (pins.test_outer_nesterov_two_rounds_by_hand, ()),
        (pins.test_outer_matches_torch_sgd_nesterov, ()),
        (pins.test_warmup_accumulates_without_touching_the_model, (3,)),
        (pins.test_rounds_against_torch_optimizers, ()),
    ]
    calls += [(pins.test_schedules_match_the_printed_constants, (row,)) for row in pins._golden_rows()]
    return calls


def run_battery(oracle):
    """Names of the pins that fail with ``oracle`` in place of the real one."""
    saved = pins.O
    pins.O = oracle
    failed = []
    try:
        for fn, args in battery():
            try:
                fn(*args)
            except AssertionError:
                failed.append(fn.__name__)
    finally:
        pins.O = saved
    return failed


def compile_variant(tmp_path, name, text):
    c = tmp_path / "variant.c"
    so = tmp_path / ("variant_%d.so" % abs(hash(name)))
    c.write_text(text)
    flags = [f for f in O.CFLAGS if f not in ("-Wall", "-Wextra")]
    subprocess.check_call(["gcc", *flags, "-w", "-o", str(so), str(c), "-lm"])
    return O.Oracle(str(so))


def test_unmodified_source_passes_the_battery(tmp_path):
    assert run_battery(compile_variant(tmp_path, "identity", SRC)) == []


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    assert SRC.count(old) >= 1, "mutation target not found in the oracle source: " + name
    broken = compile_variant(tmp_path, name, SRC.replace(old, new, 1))
    assert run_battery(broken), "no pin notices: " + name
