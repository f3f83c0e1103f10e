"""Plant one mistake at a time in a COPY of the oracle's C source (CPU only) and
check that the pins notice: a pin suite that a wrong oracle passes pins nothing."""
import os
import subprocess

import pytest

import oracle.shadow as osh
import pins

SRC = open(osh._SRC).read()

# (name, text to replace, replacement) -- each a plausible slip
MUTANTS = [
    ("fold_skips_worker0", "float acc = widen_bf16(g[0][i]);\n        for (uint32_t w = 1;", "float acc = 0.0f;\n        for (uint32_t w = 1;"),
    ("fold_f32_reverse_order", "float acc = g[0][i];\n        for (uint32_t w = 1; w < W; ++w) acc = acc + g[w][i];",
     "float acc = g[W - 1][i];\n        for (uint32_t w = 1; w < W; ++w) acc = acc + g[W - 1 - w][i];"),
    ("fold_no_mean", "if (mean) acc = acc * invW;\n        r[i] = acc;\n    }\n}\n\nvoid oracle_fold_bf16(", "r[i] = acc;\n    }\n}\n\nvoid oracle_fold_bf16("),
    ("widen_shift", "(uint32_t)h << 16", "(uint32_t)h << 15"),
    ("clip_no_sqrt", "long double norm = sqrtl(*sumsq);\n    long double c = (long double)max_norm / (norm + (long double)1e-6);\n    if (c > 1.0L) c = 1.0L;\n    return (float)c;",
     "long double norm = (*sumsq);\n    long double c = (long double)max_norm / (norm + (long double)1e-6);\n    if (c > 1.0L) c = 1.0L;\n    return (float)c;"),
    ("clip_no_guard", "(norm + (long double)1e-6);\n    if (c > 1.0L) c = 1.0L;\n    return (double)c;", "(norm);\n    if (c > 1.0L) c = 1.0L;\n    return (double)c;"),
    ("clip_no_min", "if (c > 1.0L) c = 1.0L;\n    return (float)c;", "return (float)c;"),
    ("sumsq_not_squared", "s += (long double)r[i] * (long double)r[i];\n    *acc = s;\n}\n\nvoid oracle_sumsq_accumulate_f64", "s += fabsl((long double)r[i]);\n    *acc = s;\n}\n\nvoid oracle_sumsq_accumulate_f64"),
    ("adam_v_not_squared", "(omb2 * g) * g", "(omb2 * g)"),
    ("adam_swapped_betas", "float mi = beta1 * m[i] + omb1 * g;", "float mi = beta2 * m[i] + omb1 * g;"),
    ("adam_plus_sign", "pi = pi - step_size * (mi / denom);", "pi = pi + step_size * (mi / denom);"),
    ("adam_eps_inside_sqrt", "float denom = sqrtf(vi) * isq + eps;", "float denom = sqrtf(vi + eps) * isq;"),
    ("adam_no_bias_correction2", "out[4] = (float)(1.0 / sqrt(bc2));", "out[4] = 1.0f;"),
    ("adam_no_bias_correction1", "out[3] = (float)((double)lr / bc1);", "out[3] = lr;"),
    ("adam_t_off_by_one", "double bc1 = 1.0 - pow((double)beta1, (double)t);\n    double bc2", "double bc1 = 1.0 - pow((double)beta1, (double)t + 1.0);\n    double bc2"),
    ("decay_after_step", "if (wd_flag) pi = pi * decay;\n        float mi", "float mi"),
    ("decay_ignores_mask", "if (wd_flag) pi = pi * decay;", "pi = pi * decay;"),
    ("decay_coupled_l2", "if (wd_flag) pi = pi * decay;\n        float mi = beta1 * m[i] + omb1 * g;", "if (wd_flag) g = g + wd * pi;\n        float mi = beta1 * m[i] + omb1 * g;"),
    ("clip_not_applied", "if (clip) g = g * c;", ""),
    ("f64_no_decay", "if (wd_flag) pi = pi * (1.0 - lr * wd);", ""),
    ("f64_mhat_uses_bc2", "double mhat = mi / bc1;", "double mhat = mi / bc2;"),
    ("f64_clip_not_applied", "double g = clip ? r[i] * c : r[i];", "double g = r[i];"),
    ("adam_decay_decoupled_instead", "if (wd_flag) g = g + wd * pi;\n        float mi = beta1 * m[i] + omb1 * g;", "if (wd_flag) pi = pi * (1.0f - lr * wd);\n        float mi = beta1 * m[i] + omb1 * g;"),
    ("adam_penalty_sign", "if (wd_flag) g = g + wd * pi;\n        float mi", "if (wd_flag) g = g - wd * pi;\n        float mi"),
    ("adam_f64_penalty_dropped", "if (wd_flag) g = g + wd * pi;\n        double mi", "double mi"),
    ("sgd_momentum_on_gradient", "float bi = mu * b[i] + g;", "float bi = b[i] + mu * g;"),
    ("sgd_dampening", "float bi = mu * b[i] + g;", "float bi = mu * b[i] + (1.0f - mu) * g;"),
    ("sgd_step_uses_gradient", "pi = pi - lr * bi;\n        p[i] = pi;\n        b[i] = bi;\n    }\n}\n\nvoid oracle_sgd_f64", "pi = pi - lr * g;\n        p[i] = pi;\n        b[i] = bi;\n    }\n}\n\nvoid oracle_sgd_f64"),
    ("sgd_penalty_ignores_mask", "if (wd_flag) g = g + wd * pi;\n        float bi", "g = g + wd * pi;\n        float bi"),
    ("sgd_clip_after_penalty", "if (clip) g = g * c;\n        float pi = p[i];\n        if (wd_flag) g = g + wd * pi;\n        float bi", "float pi = p[i];\n        if (wd_flag) g = g + wd * pi;\n        if (clip) g = g * c;\n        float bi"),
    ("scalars_decay_wrong", "out[0] = (float)(1.0 - (double)lr * (double)wd);", "out[0] = (float)(1.0 - (double)wd);"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new):
    assert SRC.count(old) >= 1, f"mutation anchor for {name} not found in the oracle source"
    src = tmp_path / "mutant.c"
    src.write_text(SRC.replace(old, new, 1))
    so = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", *[f for f in osh.CFLAGS if f != "-Wall"], "-w", "-o", str(so), str(src), "-lm"])
    caught = []
    with osh._bind_alternate(str(so)):
        for pin in pins.ALL_PINS:
            try:
                pin()
            except AssertionError:
                caught.append(pin.__name__)
    assert caught, f"no pin noticed the planted mistake '{name}'"
    # the real oracle is bound again afterwards
    pins.pin_fold_order_and_precision()
