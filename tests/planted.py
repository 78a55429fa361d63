"""Plausible mistakes, each a textual replacement in a COPY of the CPU oracle's source, and the means to build
such a copy and to point the oracle's ctypes front end at it.  Used to show that the checks have teeth: the pins
(CPU) and the GPU parity comparisons must notice every one.  The mistake is always planted in the oracle, on the
CPU; the GPU library is never altered."""
import contextlib
import os
import subprocess

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "adagc_oracle.c")

MISTAKES = [
    ("epsilon inside the square root", "(sqrt(vhat) + hp->eps)", "sqrt(vhat + hp->eps)"),
    ("weight decay dropped from AdamW", "th - hp->lr * hp->weight_decay * th - ", "th - "),
    ("EMA fed the unclipped norm", "double clipped_norm = active ? threshold : norm;", "double clipped_norm = norm;"),
    ("clip on >= instead of >", "int active = (norm > threshold);", "int active = (norm >= threshold);"),
    ("second bias correction uses beta1", "double bias2 = 1.0 - pow(hp->beta2", "double bias2 = 1.0 - pow(hp->beta1"),
    ("Lion interpolation uses beta2", "double c = hp->beta1 * mprev + (1.0 - hp->beta1)",
     "double c = hp->beta2 * mprev + (1.0 - hp->beta2)"),
    ("Lion momentum built from the interpolation", "double mj = hp->beta2 * mprev + (1.0 - hp->beta2) * ghat;",
     "double mj = hp->beta2 * mprev + (1.0 - hp->beta2) * c;"),
    ("second moment without the square", "(1.0 - hp->beta2) * ghat * ghat", "(1.0 - hp->beta2) * ghat"),
    ("warm-up one step short", "int warmup = (step - 1) < hp->t_start;", "int warmup = step < hp->t_start;"),
    ("running maximum instead of minimum", "return clipped_norm < gamma_prev ? clipped_norm : gamma_prev;",
     "return clipped_norm > gamma_prev ? clipped_norm : gamma_prev;"),
    ("bf16 ties always round up", "(dropped == 0x8000u && (kept & 1u))", "(dropped == 0x8000u)"),
    ("coefficient applied after the moments", "double mj = hp->beta1 * (double)m[j] + (1.0 - hp->beta1) * ghat;",
     "double mj = hp->beta1 * (double)m[j] + (1.0 - hp->beta1) * grad_at(g, j, grad_dtype);"),
    ("global norm without the root", "double global_norm = sqrt(s);", "double global_norm = s;"),
    ("EMA weights swapped", "*gamma_new = beta * gamma_prev + (1.0 - beta) * clipped_norm;",
     "*gamma_new = (1.0 - beta) * gamma_prev + beta * clipped_norm;"),
    ("first bias correction dropped", "double mhat = mj / bias1;", "double mhat = mj;"),
    ("second bias correction dropped", "double vhat = vj / bias2;", "double vhat = vj;"),
    ("bias corrections one step late", "double bias1 = 1.0 - pow(hp->beta1, (double)t);",
     "double bias1 = 1.0 - pow(hp->beta1, (double)(t + 1));"),
    ("coefficient inverted", "double coef = active ? threshold / norm : 1.0;", "double coef = active ? norm / threshold : 1.0;"),
    ("warm-up minimum fed the unclipped norm", "gamma_new = oracle_warmup_gamma(gamma_prev, h * norm, step == 1);",
     "gamma_new = oracle_warmup_gamma(gamma_prev, norm, step == 1);"),
    ("first step keeps the initial gamma", "    if (first_step)\n        return clipped_norm;\n", ""),
    ("warm-up applies no global coefficient", "                h = h_global;\n                clipped = clipped_global;\n                gamma_new",
     "                h = 1.0;\n                clipped = 0;\n                gamma_new"),
    ("Lion: sign(0) taken as +1", "double sgn = (c > 0.0) ? 1.0 : ((c < 0.0) ? -1.0 : 0.0);",
     "double sgn = (c >= 0.0) ? 1.0 : -1.0;"),
    ("Lion: update from the new momentum", "double sgn = (c > 0.0) ? 1.0 : ((c < 0.0) ? -1.0 : 0.0);",
     "double cm = hp->beta2 * mprev + (1.0 - hp->beta2) * ghat; double sgn = (cm > 0.0) ? 1.0 : ((cm < 0.0) ? -1.0 : 0.0);"),
    ("GlobalGC coefficient not capped at 1", "return active ? lambda_abs / global_norm : 1.0;",
     "return lambda_abs / global_norm;"),
    ("updates read bf16 bits as integers", "return (double)oracle_bf16_to_float(((const uint16_t *)g)[j]);",
     "return (double)(((const uint16_t *)g)[j]);"),
    ("weight decay dropped from Lion", "th = th - hp->lr * (update_coef * sgn + hp->weight_decay * th);", "th = th - hp->lr * update_coef * sgn;"),
    ("ZClip: clip on >= instead of >", "int active = (z > z_thres);", "int active = (z >= z_thres);"),
    ("ZClip: threshold without the reciprocal adjustment", "double xi = z_thres * z_thres / z;", "double xi = z_thres;"),
    ("ZClip: z-score from the variance, not the deviation", "double sigma = sqrt(var_prev);", "double sigma = var_prev;"),
    ("ZClip: statistics fed the unclipped norm", "double clipped_norm = active ? tau : norm;\n    double mu = alpha",
     "double clipped_norm = norm;\n    double mu = alpha"),
    ("ZClip: variance around the old mean", "double dev = clipped_norm - mu;\n    *h = coef;", "double dev = clipped_norm - mu_prev;\n    *h = coef;"),
    ("ZClip: variance without the square", "*var_new = alpha * var_prev + (1.0 - alpha) * dev * dev;\n    *clipped = active;",
     "*var_new = alpha * var_prev + (1.0 - alpha) * dev;\n    *clipped = active;"),
    ("ZClip: EMA weights swapped", "double mu = alpha * mu_prev + (1.0 - alpha) * clipped_norm;\n    double dev = clipped_norm - mu;\n    *h = coef;",
     "double mu = (1.0 - alpha) * mu_prev + alpha * clipped_norm;\n    double dev = clipped_norm - mu;\n    *h = coef;"),
    ("ZClip: coefficient inverted", "double coef = active ? tau / norm : 1.0;", "double coef = active ? norm / tau : 1.0;"),
    ("ZClip: first step averages instead of setting", "    if (first_step) {\n        *mu_new = clipped_norm;\n        *var_new = 0.0;\n        return;\n    }\n", ""),
    ("ZClip: statistics gathered from the raw norm during the first steps", "oracle_zclip_gather(h_global * global_norm,", "oracle_zclip_gather(global_norm,"),
    ("ZClip: z-score rule already during the first steps", "} else if (mode == 3 && !warmup) {", "} else if (mode == 3) {"),
    ("AGC: ratio inverted", "double ratio = lambda_rel * theta_norm / delta_norm;", "double ratio = lambda_rel * delta_norm / theta_norm;"),
    ("AGC: relative threshold dropped", "double ratio = lambda_rel * theta_norm / delta_norm;", "double ratio = theta_norm / delta_norm;"),
    ("Clippy: learning rate left out", "/ (lr * delta_inf);", "/ delta_inf;"),
    ("Clippy: absolute term dropped", "(lambda_rel * theta_inf + lambda_abs)", "(lambda_rel * theta_inf)"),
    ("update clipping: coefficient not capped at 1", "    int active = (ratio < 1.0);            /* false for NaN */", "    int active = 1;"),
    ("update clipping: coefficient applied to the gradient", "adamw_update_scaled(theta, m, v, g, grad_dtype, numel, 1.0, update_coef, hp, t, theta_bf16);",
     "adamw_update_scaled(theta, m, v, g, grad_dtype, numel, update_coef, 1.0, hp, t, theta_bf16);"),
    ("update clipping: weight decay scaled too", "th - hp->lr * hp->weight_decay * th - update_coef * (", "th - update_coef * (hp->lr * hp->weight_decay * th) - update_coef * ("),
    ("update clipping: direction from the old moments", "double mj = hp->beta1 * (double)m[j] + (1.0 - hp->beta1) * gj;", "double mj = (double)m[j];"),
    ("update clipping: direction without bias correction", "delta = (mj / bias1) / (sqrt(vj / bias2) + hp->eps);", "delta = mj / (sqrt(vj) + hp->eps);"),
    ("Clippy given the l2 norms", "c = oracle_clippy_coef(thinf, dinf,", "c = oracle_clippy_coef(th2, d2,"),
    ("AGC given the l-infinity norms", "c = oracle_agc_coef(th2, d2,", "c = oracle_agc_coef(thinf, dinf,"),
    ("update clipping: Lion coefficient on the decay instead of the sign", "th = th - hp->lr * (update_coef * sgn + hp->weight_decay * th);",
     "th = th - hp->lr * (sgn + update_coef * hp->weight_decay * th);"),
    ("update clipping: squared norms compared", "    *theta_l2 = sqrt(s_theta);\n    *delta_l2 = sqrt(s_delta);", "    *theta_l2 = s_theta;\n    *delta_l2 = s_delta;"),
]


def source():
    with open(SRC) as f:
        return f.read()


def mutated_source(k):
    what, old, new = MISTAKES[k]
    original = source()
    assert original.count(old) >= 1, "pattern of '%s' no longer occurs in the oracle" % what
    return original.replace(old, new)


def build(tmp_path, tag, text):
    c = os.path.join(str(tmp_path), "oracle_%s.c" % tag)
    so = os.path.join(str(tmp_path), "liboracle_%s.so" % tag)
    with open(c, "w") as f:
        f.write(text)
    subprocess.run(["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-w",
                    "-o", so, c, "-lm"], check=True)
    return so


@contextlib.contextmanager
def wrong_oracle(tmp_path, k):
    """Inside the block, the oracle package computes with mistake k planted."""
    so = build(tmp_path, "m%02d" % k, mutated_source(k))
    saved = oracle._lib
    os.environ["ADAGC_ORACLE_LIB"] = so
    oracle._lib = None
    try:
        oracle.lib()
        yield MISTAKES[k][0]
    finally:
        os.environ.pop("ADAGC_ORACLE_LIB", None)
        oracle._lib = saved
