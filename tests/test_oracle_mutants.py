"""Mutation check of the oracle's pins (CPU only).

Each entry plants one plausible mistake in a copy of the oracle's source (a
dropped term, a wrong sign, a transposed index, eps inside the root, ...),
builds it, and runs the pin tests against that build.  Every mutant must be
caught by at least one pin; if one survives, the pins are too weak."""
import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor


from oracle import build as obuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_TESTS = ["tests/test_oracle_half.py", "tests/test_oracle_norm_clip.py", "tests/test_oracle_adam.py",
             "tests/test_oracle_whole_clip.py", "tests/test_oracle_bf16.py", "tests/test_oracle_lamb.py",
             "tests/test_oracle_compare.py"]

MUTANTS = [
    ("norm: sum of |x| instead of squares", "s += x * x;", "s += std::fabs(x);"),
    ("norm: square root dropped", "norms[b] = std::sqrt(s);", "norms[b] = s;"),
    ("norm: segment begin ignored", "for (uint64_t i = seg_begin[k]; i < seg_begin[k] + seg_len[k]; ++i) {\n        const double x",
     "for (uint64_t i = 0; i < seg_len[k]; ++i) {\n        const double x"),
    ("norm: last element of each segment dropped", "i < seg_begin[k] + seg_len[k]; ++i) {\n        const double x",
     "i + 1 < seg_begin[k] + seg_len[k]; ++i) {\n        const double x"),
    ("norm: sum not reset between buckets", "    double s = 0.0;\n    for (uint64_t k = bucket_seg_off[b]", "    static double s = 0.0;\n    for (uint64_t k = bucket_seg_off[b]"),
    ("coef: inverted ratio", "coef = c / n;", "coef = n / c;"),
    ("coef: clips when below threshold", "} else if (n >= c) {", "} else if (n <= c) {"),
    ("coef: torch-style fudge term", "coef = c / n;", "coef = c / (n + 1e-6);"),
    ("coef: squared norm compared", "} else if (n >= c) {", "} else if (n * n >= c) {"),
    ("alg1: threshold divided by B instead of sqrt(B)", "return c / std::sqrt(static_cast<double>(n_buckets));",
     "return c / static_cast<double>(n_buckets);"),
    ("scale: unclipped buckets rewritten through fp32 multiply by wrong bucket", "store_scaled_grad(g, gdt, i, coefs[b]);",
     "store_scaled_grad(g, gdt, i, coefs[0]);"),
    ("scale: fp16 product truncated instead of rounded", "g[i] = float_to_half_bits(prod);",
     "g[i] = float_to_half_bits(prod) & 0xfffe;"),
    ("half: subnormal exponent off by one", "std::ldexp(static_cast<double>(frac), -24)", "std::ldexp(static_cast<double>(frac), -25)"),
    ("half: ties away from zero", "const double r = std::nearbyint(q);", "const double r = std::floor(q + 0.5);"),
    ("adam: beta1 and 1-beta1 swapped", "m = h.beta1 * m + (1.0 - h.beta1) * g;", "m = (1.0 - h.beta1) * m + h.beta1 * g;"),
    ("adam: second moment uses g not g^2", "v = h.beta2 * v + (1.0 - h.beta2) * g * g;", "v = h.beta2 * v + (1.0 - h.beta2) * g;"),
    ("adam: no bias correction on m", "const double mhat = m / bc1;", "const double mhat = m;"),
    ("adam: no bias correction on v", "const double vhat = v / bc2;", "const double vhat = v;"),
    ("adam: eps inside the root", "std::sqrt(vhat) + h.eps", "std::sqrt(vhat + h.eps)"),
    ("adam: eps before bias correction", "p = p - h.lr * (mhat / (std::sqrt(vhat) + h.eps) + h.wd * p);",
     "p = p - h.lr * (mhat / ((std::sqrt(v) + h.eps) / std::sqrt(bc2)) + h.wd * p);"),
    ("adam: ascent instead of descent", "p = p - h.lr * (mhat", "p = p + h.lr * (mhat"),
    ("adam: weight decay dropped", " + h.wd * p);", ");"),
    ("adam: weight decay not scaled by lr", "p = p - h.lr * (mhat / (std::sqrt(vhat) + h.eps) + h.wd * p);",
     "p = p - h.lr * (mhat / (std::sqrt(vhat) + h.eps)) - h.wd * p;"),
    ("adam: coupled (L2) weight decay", "  m = h.beta1 * m + (1.0 - h.beta1) * g;", "  g += h.wd * p;\n  m = h.beta1 * m + (1.0 - h.beta1) * g;"),
    ("adam: bias correction uses step-1", "const double bc1 = 1.0 - std::pow(beta1, static_cast<double>(step));\n  const double bc2 = 1.0 - std::pow(beta2, static_cast<double>(step));\n  for (uint32_t t",
     "const double bc1 = 1.0 - std::pow(beta1, static_cast<double>(step + 1));\n  const double bc2 = 1.0 - std::pow(beta2, static_cast<double>(step + 1));\n  for (uint32_t t"),
    ("adam: beta1 used for second-moment correction", "const double bc2 = 1.0 - std::pow(beta2, static_cast<double>(step));\n  for (uint32_t t",
     "const double bc2 = 1.0 - std::pow(beta1, static_cast<double>(step));\n  for (uint32_t t"),
    ("fused: Adam sees unscaled gradient", "const double ghat = coef * load_grad(grads[t], gdt, i);", "const double ghat = load_grad(grads[t], gdt, i);"),
    ("fused: Adam sees storage-rounded gradient", "adam_element(ghat, p[t][i], m[t][i], v[t][i], h, bc1, bc2);\n          if (write_back",
     "adam_element(gdt == GRAD_F16 ? half_bits_to_double(float_to_half_bits((float)ghat)) : (double)(float)ghat, p[t][i], m[t][i], v[t][i], h, bc1, bc2);\n          if (write_back"),
    ("fused: write-back always on", "if (write_back && coefs[b] != 1.0f)", "if (coefs[b] != 1.0f)"),
    ("fused: skip flag ignored", "if (!(skip_on_nonfinite && (status & ORC_STATUS_NONFINITE))) {", "if (true) {"),
    ("whole: sum of squares restarts at every bucket", "total += s;", "total = s;"),
    ("whole: square root dropped", "const double whole = std::sqrt(total);", "const double whole = total;"),
    ("whole: Adam sees the unscaled gradient", "const double ghat = static_cast<double>(coef) * load_grad(grads[t], gdt, i);",
     "const double ghat = load_grad(grads[t], gdt, i);"),
    ("whole: per-bucket norms not rooted", "if (norms_out) norms_out[b] = std::sqrt(s);", "if (norms_out) norms_out[b] = s;"),
    ("bf16: subnormal exponent off by one", "std::ldexp(static_cast<double>(frac), -133)", "std::ldexp(static_cast<double>(frac), -134)"),
    ("bf16: exponent bias of binary16", "std::ldexp(static_cast<double>(128 + frac), expo - 134)", "std::ldexp(static_cast<double>(128 + frac), expo - 22)"),
    ("bf16: truncation instead of rounding", "const double r = std::nearbyint(std::ldexp(a, -ulp_exp));", "const double r = std::floor(std::ldexp(a, -ulp_exp));"),
    ("bf16: ties away from zero", "const double r = std::nearbyint(std::ldexp(a, -ulp_exp));", "const double r = std::floor(std::ldexp(a, -ulp_exp) + 0.5);"),
    ("bf16: scaled gradient stored through binary16 rounding", "g[i] = float_to_bf16_bits(prod);", "g[i] = float_to_bf16_bits((float)half_bits_to_double(float_to_half_bits(prod)));"),
    ("mask: inverted", "if (decay != nullptr && decay[t] == 0) h.wd = 0.0;", "if (decay != nullptr && decay[t] != 0) h.wd = 0.0;"),
    ("mask: ignored", "if (decay != nullptr && decay[t] == 0) h.wd = 0.0;", ""),
    ("mask: indexed by the wrong tensor", "if (decay != nullptr && decay[t] == 0) h.wd = 0.0;", "if (decay != nullptr && decay[t ? t - 1 : 0] == 0) h.wd = 0.0;"),
    ("lamb: inverted trust ratio", "? p_norm / u_norm : 1.0;", "? u_norm / p_norm : 1.0;"),
    ("lamb: squared norms in the ratio", "const double p_norm = std::sqrt(sum_pp), u_norm = std::sqrt(sum_uu);", "const double p_norm = sum_pp, u_norm = sum_uu;"),
    ("lamb: decay term left out of the update norm", "sum_uu += u[i] * u[i];", "sum_uu += (u[i] - h.wd * p[i]) * (u[i] - h.wd * p[i]);"),
    ("lamb: decay term left out of the update", "u[i] = mhat / (std::sqrt(vhat) + h.eps) + h.wd * p[i];", "u[i] = mhat / (std::sqrt(vhat) + h.eps);"),
    ("lamb: no guard for zero norms", "(p_norm > 0.0 && u_norm > 0.0) ? p_norm / u_norm : 1.0;", "p_norm / u_norm;"),
    ("lamb: trust ratio not applied", "p[i] = p[i] - h.lr * trust * u[i];", "p[i] = p[i] - h.lr * u[i];"),
    ("lamb: no bias correction", "    const double mhat = m[i] / bc1;", "    const double mhat = m[i];"),
    ("lamb: eps inside the root", "u[i] = mhat / (std::sqrt(vhat) + h.eps)", "u[i] = mhat / (std::sqrt(vhat + h.eps))"),
    ("lamb: max norm instead of Euclidean", "sum_pp += p[i] * p[i];", "sum_pp = std::fmax(sum_pp, p[i] * p[i]);"),
    ("clip+lamb: LAMB sees the unscaled gradient", "ghat[t][i] = static_cast<double>(coefs[b]) * load_grad(grads[t], gdt, i);", "ghat[t][i] = load_grad(grads[t], gdt, i);"),
    ("clip+lamb: one coefficient for all buckets", "ghat[t][i] = static_cast<double>(coefs[b]) * load_grad(grads[t], gdt, i);", "ghat[t][i] = static_cast<double>(coefs[0]) * load_grad(grads[t], gdt, i);"),
    ("clip+lamb: write-back always on", "if (write_back && coefs[b] != 1.0f) store_scaled_grad(grads[t], gdt, i, coefs[b]);\n      }\n    }\n  const Adam h_all", "if (coefs[b] != 1.0f) store_scaled_grad(grads[t], gdt, i, coefs[b]);\n      }\n    }\n  const Adam h_all"),
    ("fused: wrong tensor for state", "adam_element(ghat, p[t][i], m[t][i], v[t][i], h, bc1, bc2);", "adam_element(ghat, p[t][i], v[t][i], m[t][i], h, bc1, bc2);"),
    # the acceptance rule that every GPU parity assertion goes through
    ("compare: absolute clause joined by 'or'", "ok = (rel <= rel_tol) || (aw < small && err <= abs_tol);",
     "ok = (rel <= rel_tol) || (aw < small || err <= abs_tol);"),
    ("compare: 'small' bound ignored", "ok = (rel <= rel_tol) || (aw < small && err <= abs_tol);",
     "ok = (rel <= rel_tol) || (err <= abs_tol);"),
    ("compare: absolute clause also at |oracle| == small", "ok = (rel <= rel_tol) || (aw < small && err <= abs_tol);",
     "ok = (rel <= rel_tol) || (aw <= small && err <= abs_tol);"),
    ("compare: strict relative bound", "ok = (rel <= rel_tol) || (aw < small && err <= abs_tol);",
     "ok = (rel < rel_tol) || (aw < small && err <= abs_tol);"),
    ("compare: strict absolute bound", "ok = (rel <= rel_tol) || (aw < small && err <= abs_tol);",
     "ok = (rel <= rel_tol) || (aw < small && err < abs_tol);"),
    ("compare: relative error against the GPU value", "const double rel = aw > 0.0 ? err / aw :", "const double rel = aw > 0.0 ? err / std::fabs(g) :"),
    ("compare: signs ignored", "const double err = std::fabs(g - w), aw = std::fabs(w);", "const double err = std::fabs(std::fabs(g) - std::fabs(w)), aw = std::fabs(w);"),
    ("compare: one NaN is enough", "ok = std::isnan(w) && std::isnan(g);", "ok = std::isnan(w) || std::isnan(g);"),
    ("compare: infinities always pass", "ok = (w == g);", "ok = true;"),
    ("compare: failures counted once", "      ++bad;\n      if (worst < 0)", "      bad = 1;\n      if (worst < 0)"),
    ("compare: worst element is the first failure", "if (!ok && err > worst_err) {", "if (!ok && worst_err < 0) {"),
    ("compare: max_rel_all leaves out values below 'small'", "if (aw > tiny && rel > max_rel_all) max_rel_all = rel;",
     "if (aw >= small && rel > max_rel_all) max_rel_all = rel;"),
    ("compare: 'tiny' bound ignored", "if (aw > tiny && rel > max_rel_all) max_rel_all = rel;", "if (rel > max_rel_all) max_rel_all = rel;"),
    ("compare: zero oracle value has zero relative error", "(err == 0.0 ? 0.0 : INFINITY)", "0.0"),
]


LBS_PIN_TESTS = ["tests/test_oracle_lbs.py"]

LBS_MUTANTS = [
    ("rng: increment not multiplied by the draw number", "seed + (k + 1) * 0x9E3779B97F4A7C15ull", "seed + (k + 1) + 0x9E3779B97F4A7C15ull"),
    ("rng: draw numbers start at 0 instead of 1", "seed + (k + 1) * 0x9E3779B97F4A7C15ull", "seed + k * 0x9E3779B97F4A7C15ull"),
    ("rng: wrong shift in the first mixing step", "(z ^ (z >> 30))", "(z ^ (z >> 31))"),
    ("sampling: lower half of the draw used", "const uint64_t u = orc_lbs_splitmix64(seed, k0 + j) >> 32;\n      out[j] = orc_lbs_length_of(cum, max_len, static_cast<uint32_t>((u * total) >> 32));",
     "const uint64_t u = orc_lbs_splitmix64(seed, k0 + j) & 0xffffffffull;\n      out[j] = orc_lbs_length_of(cum, max_len, static_cast<uint32_t>((u * total) >> 32));"),
    ("sampling: inverse histogram off by one", "if (cum[l] > index) return l;", "if (cum[l] >= index) return l;"),
    ("sampling: GPUs of a trial share their draws", "const uint64_t k0 = (trial * n_gpus + gpu) * static_cast<uint64_t>(local_batch);",
     "const uint64_t k0 = (trial * n_gpus + gpu);"),
    ("sampling: trials share their draws", "const uint64_t k0 = (trial * n_gpus + gpu) * static_cast<uint64_t>(local_batch);",
     "const uint64_t k0 = (gpu) * static_cast<uint64_t>(local_batch);"),
    ("strata: lower bound of the previous stratum's start", "const uint32_t lo = cum[s == 0 ? 0 : stratum_end[s - 1]];   // entries before", "const uint32_t lo = cum[s <= 1 ? 0 : stratum_end[s - 2]];   // entries before"),
    ("strata: offset inside the stratum dropped", "lo + static_cast<uint32_t>((u * size) >> 32)", "static_cast<uint32_t>((u * size) >> 32)"),
    ("strata: quota ignored", "for (uint32_t q = 0; q < quota[s]; ++q, ++j) {", "for (uint32_t q = 0; q < local_batch / n_strata; ++q, ++j) {"),
    ("scatter: no sort", "std::sort(lengths, lengths + static_cast<size_t>(n_group) * local_batch);", ""),
    ("scatter: snake reverses the even rows", "(snake && (r % 2 == 1))", "(snake && (r % 2 == 0))"),
    ("scatter: snake never reverses", "(snake && (r % 2 == 1))", "(false)"),
    ("scatter: contiguous blocks instead of rows", "tokens[g] += lengths[static_cast<size_t>(r) * n_group + c];", "tokens[g] += lengths[static_cast<size_t>(c) * local_batch + r];"),
    ("local: raster and snake swapped", "method == LBS_LOCAL_SNAKE,\n", "method == LBS_LOCAL_RASTER,\n"),
    ("local: every node reads the first node's sequences", "const size_t first = static_cast<size_t>(node) * gpus_per_node * local_batch;", "const size_t first = 0;"),
    ("global: drawn from the stratified dataset", "const bool stratified = method == LBS_STRATIFIED || method == LBS_LOCAL_RASTER || method == LBS_LOCAL_SNAKE;",
     "const bool stratified = method != LBS_NONE;"),
    ("global: snake order", "orc_lbs_presort_scatter(gathered.data(), n_gpus, local_batch, 0, tokens.data());", "orc_lbs_presort_scatter(gathered.data(), n_gpus, local_batch, 1, tokens.data());"),
    ("result: last GPU left out of min/max", "for (uint32_t g = 1; g < n_gpus; ++g) lo =", "for (uint32_t g = 1; g + 1 < n_gpus; ++g) lo ="),
    ("result: sums not accumulated", "sums[0] += lo;", "sums[0] = lo;"),
]


def _run_mutant(args, src_path=None, env_name="BCA_ORACLE_LIB", pin_tests=None):
    idx, (name, old, new) = args
    pin_tests = pin_tests or PIN_TESTS
    src = open(src_path or obuild.SRC).read()
    if src.count(old) < 1:
        return name, "pattern not found in oracle source"
    with tempfile.TemporaryDirectory() as td:
        msrc, mlib = os.path.join(td, "m.cpp"), os.path.join(td, f"libm{idx}.so")
        open(msrc, "w").write(src.replace(old, new, 1))
        try:
            subprocess.run(["g++", "-O1", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-o", mlib, msrc],
                           check=True, capture_output=True)
        except subprocess.CalledProcessError as e:
            return name, "mutant does not compile: " + e.stderr.decode()[-300:]
        env = dict(os.environ, **{env_name: mlib})
        r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *pin_tests],
                           cwd=ROOT, env=env, capture_output=True)
        if r.returncode == 0:
            return name, "SURVIVED: no pin test failed"
        if r.returncode != 1:
            return name, f"pytest exit {r.returncode}: " + r.stdout.decode()[-300:]
    return name, None


def test_every_planted_mistake_is_caught_by_a_pin():
    with ThreadPoolExecutor(max_workers=6) as ex:
        results = list(ex.map(_run_mutant, enumerate(MUTANTS)))
    problems = [f"{n}: {why}" for n, why in results if why]
    assert not problems, "\n".join(problems)


def test_every_planted_mistake_in_the_load_balancing_oracle_is_caught_by_a_pin():
    run = lambda a: _run_mutant(a, obuild.LBS_SRC, "LBS_ORACLE_LIB", LBS_PIN_TESTS)
    with ThreadPoolExecutor(max_workers=6) as ex:
        results = list(ex.map(run, enumerate(LBS_MUTANTS)))
    problems = [f"{n}: {why}" for n, why in results if why]
    assert not problems, "\n".join(problems)
