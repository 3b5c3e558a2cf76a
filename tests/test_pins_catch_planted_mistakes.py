"""Do the oracle's pins notice a mistake?  Copies of oracle/ddef_oracle.cpp are made with one
plausible mistake planted in each (a wrong sign, index, order, constant, boundary or a dropped
term), compiled, and the pin files (tests/test_oracle_*.py) are run against each copy in a child
process.  Every copy must make at least one pin fail; the untouched copy must pass them all.
Everything here happens on the CPU and in the oracle: nothing is planted in the GPU path.
"""
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCE = os.path.join(ROOT, "oracle", "ddef_oracle.cpp")
PIN_FILES = sorted(f for f in os.listdir(os.path.join(ROOT, "tests")) if re.fullmatch(r"test_oracle_\w+\.py", f))

# name: (text as it stands, text with the mistake, which occurrence of the text)
MISTAKES = {
    # S1, error-feedback accumulate (Algorithm 1, worker side)
    "accumulate subtracts the gradient": ("p[j] = o->e[i][j] + scaled;", "p[j] = o->e[i][j] - scaled;", 0),
    "stepsize dropped from the accumulate": ("float scaled = lr * o->g[i][j];", "float scaled = o->g[i][j];", 0),
    # S2, Top-k under the total order
    "ties go to the higher index": ("return a < b;", "return a > b;", 0),
    "smallest magnitudes selected": ("if (ka != kb) return ka > kb;", "if (ka != kb) return ka < kb;", 0),
    "sign not cleared in the key": ("return bits_of(f) & 0x7fffffffu; }", "return bits_of(f); }", 0),
    "k rounded down": ("double kd = std::ceil(delta * (double)d);", "double kd = std::floor(delta * (double)d);", 0),
    "threshold count off by one": ("if (magnitude_key(p[order[m]]) == T) ++r;",
                                   "if (magnitude_key(p[order[m]]) >= T && m > 0) ++r;", 0),
    "threshold is the largest sent magnitude": ("T = std::min(T, magnitude_key(p[order[m]]));", "T = std::max(T == 0xffffffffu ? 0u : T, magnitude_key(p[order[m]]));", 0),
    # S3, message and residual
    "message not in ascending order": ("    std::sort(order.begin(), order.begin() + k);\n", "", 0),
    "sent entries stay in the error buffer": ("for (uint64_t j = 0; j < d; ++j) o->e[i][j] = p[j] - dense[j];",
                                              "for (uint64_t j = 0; j < d; ++j) o->e[i][j] = p[j];", 0),
    "message carries the gradient, not p": ("o->msg_val[i][m] = p[j];\n        dense[j] = p[j];",
                                            "o->msg_val[i][m] = lr * o->g[i][j];\n        dense[j] = p[j];", 0),
    # S4, aggregation in worker order
    "workers summed in reverse order": ("    for (uint32_t i = 0; i < o->n; ++i)\n        for (size_t m = 0; m < o->msg_idx[i].size(); ++m)",
                                        "    for (uint32_t i = o->n; i-- > 0;)\n        for (size_t m = 0; m < o->msg_idx[i].size(); ++m)", 0),
    "update overwritten instead of summed": ("o->U[o->msg_idx[i][m]] = o->U[o->msg_idx[i][m]] + o->msg_val[i][m];",
                                             "o->U[o->msg_idx[i][m]] = o->msg_val[i][m];", 0),
    # S5, delayed apply and the ring
    "update added to the model": ("xn[j] = x[j] - avg;", "xn[j] = x[j] + avg;", 0),
    "no average over the workers": ("float avg = o->U[j] / nf;\n        xn[j]", "float avg = o->U[j];\n        xn[j]", 0),
    "gradient taken one snapshot too late": ("o->slot(o->t - o->tau);", "o->slot(o->t - o->tau + (o->tau > 0 ? 1 : 0));", 0),
    "one empty iteration too many": ("o->step_is_noop = o->t < o->tau;", "o->step_is_noop = o->t <= o->tau;", 0),
    "step index not advanced": ("        xn[j] = x[j] - avg;\n    }\n    o->t += 1;", "        xn[j] = x[j] - avg;\n    }\n    o->t += 2;", 0),
    # S0, the gradient and its noise
    "gradient ignores the optimum": ("float diff = xs[j] - optimum;", "float diff = xs[j];", 0),
    "noise not scaled": ("float xi = o->noise_scale * noise_z(o->seed, o->t,", "float xi = noise_z(o->seed, o->t,", 0),
    "noise keyed by the next iteration": ("noise_z(o->seed, o->t, i, (uint32_t)j, o->noise_kind)",
                                          "noise_z(o->seed, o->t + 1, i, (uint32_t)j, o->noise_kind)", 0),
    "same noise for every worker": ("uint32_t ctr[4] = {j >> 2, worker, (uint32_t)t, (uint32_t)(t >> 32)};",
                                    "uint32_t ctr[4] = {j >> 2, 0u, (uint32_t)t, (uint32_t)(t >> 32)};", 0),
    "Philox multipliers swapped": ("uint64_t p0 = (uint64_t)0xD2511F53u * c0;\n        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;",
                                   "uint64_t p0 = (uint64_t)0xCD9E8D57u * c0;\n        uint64_t p1 = (uint64_t)0xD2511F53u * c2;", 0),
    "Philox with nine rounds": ("for (int round = 0; round < 10; ++round)", "for (int round = 0; round < 9; ++round)", 0),
    "Philox key schedule": ("k1 += 0xBB67AE85u;", "k1 += 0x9E3779B9u;", 0),
    "uniform may be zero": ("uint32_t a = (w >> 8) + 1u;", "uint32_t a = (w >> 8) | 1u;", 0),
    "logarithm's last coefficient": ("g = std::fmaf(g, f, -0x1.fffffep-2f);", "g = std::fmaf(g, f, 0x1.fffffep-2f);", 0),
    "sine and cosine exchanged": ("return (j & 1u) ? radius * s01 : radius * c01;", "return (j & 1u) ? radius * c01 : radius * s01;", 0),
    "quadrant rotation": ("case 1: *cos_out = -s; *sin_out = c;  break;", "case 1: *cos_out = s; *sin_out = c;  break;", 0),
    "Student-t with two degrees of freedom": ("float ratio = (3.0f * r2) / chi2_3;", "float ratio = (2.0f * r2) / chi2_3;", 0),
    "Student-t reuses the radius word": ("float chi2_2 = neg2ln_uniform(word[2]);", "float chi2_2 = neg2ln_uniform(word[0]);", 0),
    "second Gaussian pair uses the first pair's words": ("uint32_t pair = (j >> 1) & 1u;", "uint32_t pair = 0u;", 0),
    "angle without the half step": ("float phi = (float)(2 * r + 1) * 0x1.921fb6p-23f;", "float phi = (float)(2 * r) * 0x1.921fb6p-23f;", 0),
    "angle without the eighth turn": ("uint32_t b = ((w >> 8) + 0x200000u) & 0xffffffu;", "uint32_t b = (w >> 8) & 0xffffffu;", 0),
    "sine series coefficient": ("sp = std::fmaf(sp, p2, 1.0f / 120.0f);", "sp = std::fmaf(sp, p2, 1.0f / 24.0f);", 0),
    "logarithm without the fold's exponent": ("if (mant > 0x3504f3u) { m = m * 0.5f; e += 1; }", "if (mant > 0x3504f3u) { m = m * 0.5f; }", 0),
    "ln u, not twice": ("    return 2.0f * v;\n}", "    return v;\n}", 0),
    "Student-t words in reverse": ("uint32_t at = 3u * (j & 3u) + m;", "uint32_t at = 3u * (j & 3u) + (2u - m);", 0),
    "Student-t blocks overlap between quads": ("uint32_t ctr[4] = {3u * (j >> 2) + (at >> 2), worker,", "uint32_t ctr[4] = {2u * (j >> 2) + (at >> 2), worker,", 0),
    "a thread's range of coordinates ends one early": ("grad_worker(o, i, j0, std::min(o->d, j0 + per));", "grad_worker(o, i, j0, std::min(o->d, j0 + per) - 1);", 0),
    "error buffers survive a new problem": ("    for (auto& e : o->e) std::fill(e.begin(), e.end(), 0.0f);\n    o->seed = seed;", "    o->seed = seed;", 0),
    # Algorithm 1 as printed (message queue)
    "queue applies one iteration late": ("if (u >= q->tau)\n        for (uint32_t i = 0; i < q->n; ++i) {\n            const std::vector<uint32_t>& idx = q->sent_idx[u - q->tau][i];\n            const std::vector<float>& val = q->sent_val[u - q->tau][i];",
                                         "if (u >= q->tau + 1)\n        for (uint32_t i = 0; i < q->n; ++i) {\n            const std::vector<uint32_t>& idx = q->sent_idx[u - q->tau - 1][i];\n            const std::vector<float>& val = q->sent_val[u - q->tau - 1][i];", 0),
    "queue keys may repeat": ("const uint64_t key = std::max(u + q->tau, q->next_key_floor);", "const uint64_t key = u + q->tau;", 0),
    "batch queue run keyed by the sending step": ("noise_z(seed, u + tau, i, (uint32_t)j, noise_kind)", "noise_z(seed, u, i, (uint32_t)j, noise_kind)", 0),
    "queue accumulate subtracts the gradient": ("p[j] = q->e[i][j] + scaled;", "p[j] = q->e[i][j] - scaled;", 0),
    "queue keeps sent entries in the error buffer": ("for (uint64_t j = 0; j < d; ++j) q->e[i][j] = p[j] - dense[j];",
                                                     "for (uint64_t j = 0; j < d; ++j) q->e[i][j] = p[j];", 0),
    "queue adds the update": ("q->x[j] = q->x[j] - avg;", "q->x[j] = q->x[j] + avg;", 0),
    "queue gradient at the optimum's sign": ("float diff = q->x[j] - optimum;", "float diff = optimum - q->x[j];", 0),
    # Random-k and the composed compressor
    "hash finaliser shift": ("h ^= h >> 13;", "h ^= h >> 15;", 0),
    "walk stops one early": ("while (y >= key.d) y = feistel_forward(key, y);", "while (y > key.d) y = feistel_forward(key, y);\n    if (y == key.d) y = 0;", 0),
    "same subset in every iteration": ("uint32_t ctr[4] = {0xffffffffu, worker, (uint32_t)t, (uint32_t)(t >> 32)};",
                                       "uint32_t ctr[4] = {0xffffffffu, worker, 0u, 0u};", 0),
    "quantiser step over eight levels": ("const float step = largest / 7.0f;", "const float step = largest / 8.0f;", 0),
    "quantiser truncates": ("float nearest = std::nearbyint(ratio);", "float nearest = std::trunc(ratio);", 0),
    "nibbles exchanged": ("<< ((m & 1) * 4));", "<< (((m + 1) & 1) * 4));", 0),
    "composed keeps k of d": ("const uint64_t k = k_from_delta(delta, k1);", "const uint64_t k = k_from_delta(delta, d) < k1 ? k_from_delta(delta, d) : k1;", 0),
    "composed residual not quantised": ("for (uint64_t m = 0; m < k; ++m) dense[o->msg_idx[i][m]] = o->msg_val[i][m];",
                                        "for (uint64_t m = 0; m < k; ++m) dense[o->msg_idx[i][m]] = chosen[m];", 0),
    "composed sends positions, not coordinates": ("o->msg_idx[i][m] = subset[pos[m]];", "o->msg_idx[i][m] = pos[m];", 0),
    "quantiser's largest value keeps its sign": ("largest = std::max(largest, std::fabs(v[m]));", "largest = std::max(largest, v[m]);", 0),
    "quantiser blocks of 128": ("constexpr uint64_t kQuantBlock = 256;", "constexpr uint64_t kQuantBlock = 128;", 0),
    "random subset not sorted": ("    std::sort(idx_out, idx_out + k);\n", "", 0),
    "Feistel halves not exchanged": ("        left = right;\n        right = new_right;", "        right = right;\n        left = new_right;", 0),
    "Feistel on too few bits": ("while (((uint64_t)1 << (2 * key.w)) < d) ++key.w;", "while (((uint64_t)1 << (2 * key.w)) < d / 2) ++key.w;", 0),
    # non-IID variant and the objective
    "shift of the optima not scaled": ("optimum = o->xstar[j] + o->zeta * noise_z(o->seed, kHeterogeneityKey, i, (uint32_t)j, 1);\n        float diff",
                                       "optimum = o->xstar[j] + noise_z(o->seed, kHeterogeneityKey, i, (uint32_t)j, 1);\n        float diff", 0),
    "objective without the half": ("return 0.5 * total;", "return total;", 0),
    "objective uses another shift than the gradient": ("optimum = o->xstar[j] + o->zeta * noise_z(o->seed, kHeterogeneityKey, i, (uint32_t)j, 1);\n            double diff",
                                                       "optimum = o->xstar[j] + o->zeta * noise_z(o->seed, kHeterogeneityKey - 1, i, (uint32_t)j, 1);\n            double diff", 0),
    "objective not averaged over the workers": ("total += (double)o->lambda[j] * (squares / (double)o->n);", "total += (double)o->lambda[j] * squares;", 0),
    # DeCo (Algorithm 3) and the timing model (Theorem 3)
    "non-IID scan minimises phi": ("double obj = oracle_phi_prime(delta, (double)tau);", "double obj = phi_value(delta, (double)tau);", 0),
    "scan without the bandwidth cap": ("double delta = std::min(std::min((tau * t_comp - b) * a / v_g, t_comp * a / v_g), 1.0);\n        if (!(delta > 0.0)) continue;\n        double phi",
                                       "double delta = std::min((tau * t_comp - b) * a / v_g, 1.0);\n        if (!(delta > 0.0)) continue;\n        double phi", 0),
    "recurrence forgets the latency of the last message": ("return (TM[E] + b) / (double)E;", "return TM[E] / (double)E;", 0),
    "recurrence waits for a message one iteration older": ("if (k >= tau && k - tau >= 1) tc_old = TM[k - tau] + b;", "if (k >= tau + 1 && k - tau >= 2) tc_old = TM[k - tau - 1] + b;", 0),
    "phi with full contraction per step": ("return (1.0 - delta) / (delta * std::pow(1.0 - 0.5 * delta, tau));",
                                           "return (1.0 - delta) / (delta * std::pow(1.0 - delta, tau));", 0),
    "phi prime with one delta": ("return (1.0 - delta) / (delta * delta * std::pow(1.0 - 0.5 * delta, tau));",
                                 "return (1.0 - delta) / (delta * std::pow(1.0 - 0.5 * delta, tau));", 0),
    "scan starts one short": ("long hi = (long)std::ceil((b + v_g / a) / t_comp);\n    long lo = (long)std::ceil(b / t_comp);\n    double best = std::numeric_limits<double>::infinity();\n    int found = -1;\n    for (long tau = hi; tau >= lo; --tau) {\n        double delta = std::min(std::min((tau * t_comp - b) * a / v_g, t_comp * a / v_g), 1.0);\n        if (!(delta > 0.0)) continue;\n        double phi",
                              "long hi = (long)std::ceil((b + v_g / a) / t_comp) - 1;\n    long lo = (long)std::ceil(b / t_comp);\n    double best = std::numeric_limits<double>::infinity();\n    int found = -1;\n    for (long tau = hi; tau >= lo; --tau) {\n        double delta = std::min(std::min((tau * t_comp - b) * a / v_g, t_comp * a / v_g), 1.0);\n        if (!(delta > 0.0)) continue;\n        double phi", 0),
    "delta star without the latency": ("double first = std::max(0.0, (tau * t_comp - b) * a / v_g);", "double first = std::max(0.0, (tau * t_comp) * a / v_g);", 0),
    "recurrence without the pipeline wait": ("TS[k + 1] = t_comp + std::max(tc_old, TS[k]);", "TS[k + 1] = t_comp + TS[k];", 0),
    "closed form without the bandwidth term": ("return std::max(std::max((t_comp + b + xfer) / (tau + 1.0), xfer), t_comp);",
                                               "return std::max((t_comp + b + xfer) / (tau + 1.0), t_comp);", 0),
}


def plant(source, was, becomes, nth):
    at = -1
    for _ in range(nth + 1):
        at = source.find(was, at + 1)
        assert at >= 0, f"the oracle no longer contains: {was!r}"
    return source[:at] + becomes + source[at + len(was):]


def pins_against(workdir, name, source):
    """(exit status of the pin run, the end of its output) for one copy of the oracle."""
    stem = re.sub(r"\W+", "_", name)
    cpp, so = os.path.join(workdir, stem + ".cpp"), os.path.join(workdir, stem + ".so")
    with open(cpp, "w") as f:
        f.write(source)
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
                           "-pthread", cpp, "-o", so])
    env = dict(os.environ, DDEF_ORACLE_LIB=so)
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                          *[os.path.join("tests", f) for f in PIN_FILES]],
                         cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    return run.returncode, run.stdout[-3000:]


@pytest.fixture(scope="module")
def verdicts(tmp_path_factory):
    workdir = str(tmp_path_factory.mktemp("planted"))
    with open(SOURCE) as f:
        source = f.read()
    copies = {"untouched": source}
    for name, (was, becomes, nth) in MISTAKES.items():
        copies[name] = plant(source, was, becomes, nth)
    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as pool:
        jobs = {name: pool.submit(pins_against, workdir, name, text) for name, text in copies.items()}
        return {name: job.result() for name, job in jobs.items()}


def test_the_untouched_oracle_passes_every_pin(verdicts):
    status, tail = verdicts["untouched"]
    assert status == 0, tail


@pytest.mark.parametrize("name", list(MISTAKES))
def test_a_planted_mistake_fails_a_pin(verdicts, name):
    status, tail = verdicts[name]
    # 1: some pin failed.  Anything else (0: all passed; 2 and up, or a signal: the run itself broke)
    # means this mistake went unnoticed or the copy is not a fair one.
    assert status == 1, f"{name}: pin run ended with status {status}\n{tail}"
    assert re.search(r"^FAILED tests/test_oracle_\w+\.py::", tail, re.M), tail
