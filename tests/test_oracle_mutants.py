"""Do the oracle's pins notice a plausible mistake?

Each case plants ONE mistake in a copy of the oracle's C source (a dropped
term, a wrong sign, a transposed operand, a wrong index, an unstable order),
builds the copy and runs the pin tests against it in a child process.  The pins
are worth something only if at least one of them fails for every such copy.
The mistakes live in the CPU oracle alone; nothing here touches a GPU, and every
planted index stays inside its array.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "moe_oracle.c")

ROUTE = ["tests/test_oracle_route_pins.py"]
LAYER = ["tests/test_oracle_layer_pins.py"]
STAGE = ["tests/test_oracle_stage_pins.py"]
FP8ACT = ["tests/test_oracle_fp8act_pins.py"]

# (name, text in the source, replacement, how many times the text occurs, pins to run)
MUTANTS = [
    # ---- route
    ("gate_w_transposed", "(double)gate_w[(size_t)e * H + h]", "(double)gate_w[(size_t)h * E + e]", 1, ROUTE),
    ("x_row_ignored", "(double)x[(size_t)t * H + h] * (double)gate_w", "(double)x[h] * (double)gate_w", 1, ROUTE),
    ("logit_bias_dropped", "if (logit_bias) acc += (double)logit_bias[e];", "", 1, ROUTE),
    ("logit_bias_sign", "acc += (double)logit_bias[e]", "acc -= (double)logit_bias[e]", 1, ROUTE),
    ("softmax_no_max_shift_sign", "s[e] = exp(z[e] - zmax)", "s[e] = exp(zmax - z[e])", 1, ROUTE),
    ("softmax_over_picks_only_missing", "for (int j = 0; j < k; ++j) den += s[ids[(size_t)t * k + j]];",
     "den = 1.0;", 1, ROUTE),
    ("sigmoid_sign", "s[e] = 1.0 / (1.0 + exp(-z[e]))", "s[e] = 1.0 / (1.0 + exp(z[e]))", 1, ROUTE),
    ("select_bias_dropped", "key[e] = s[e] + (select_bias ? (double)select_bias[e] : 0.0);", "key[e] = s[e];", 1, ROUTE),
    ("weights_from_biased_key", "w[(size_t)t * k + j] = (float)(s[ids[(size_t)t * k + j]] / den",
     "w[(size_t)t * k + j] = (float)(key[ids[(size_t)t * k + j]] / den", 1, ROUTE),
    ("routed_scale_dropped", "/ den * routed_scale)", "/ den)", 1, ROUTE),
    ("topk_ties_to_highest", "if (eligible[e] && !taken[e] && (best < 0 || key[e] > key[best])) best = e;",
     "if (eligible[e] && !taken[e] && (best < 0 || key[e] >= key[best])) best = e;", 1, ROUTE),
    ("topk_picks_smallest", "if (eligible[e] && !taken[e] && (best < 0 || key[e] > key[best])) best = e;",
     "if (eligible[e] && !taken[e] && (best < 0 || key[e] < key[best])) best = e;", 1, ROUTE),
    ("group_score_one_key", "for (int r = 0; r < group_score_n && r < gs; ++r) {", "for (int r = 0; r < 1; ++r) {", 1, ROUTE),
    ("group_ties_to_highest", "if (!gkept[g] && (best < 0 || gscore[g] > gscore[best])) best = g;",
     "if (!gkept[g] && (best < 0 || gscore[g] >= gscore[best])) best = g;", 1, ROUTE),
    ("group_limit_ignored", "for (int e = g * gs; e < (g + 1) * gs; ++e) eligible[e] = 0;", "", 1, ROUTE),
    ("group_score_from_score_not_key", "sum += key[best];", "sum += s[best];", 1, ROUTE),
    ("margin_skips_unpicked", "if (eligible[e] && !taken[e] && prev - key[e] < mgn) mgn = prev - key[e];", "", 1, ROUTE),
    # ---- dispatch
    ("dispatch_unstable", "int pos = offsets[e] + fill[e]++;", "int pos = offsets[e + 1] - 1 - fill[e]++;", 2, LAYER + STAGE),
    ("dispatch_wrong_token_row", "x + (size_t)(a / k) * H, sizeof(float) * H", "x + (size_t)(a % T) * H, sizeof(float) * H", 1, LAYER),
    ("dispatch_range_shifted", "if (ids[a] >= e_lo && ids[a] < e_hi) counts[ids[a] - e_lo]++;",
     "if (ids[a] > e_lo && ids[a] < e_hi) counts[ids[a] - e_lo]++;", 2, LAYER + STAGE),
    ("dispatch_inv_not_marked", "inv[a] = -1;", "inv[a] = 0;", 2, LAYER + STAGE),
    ("shard_wrong_columns", "x[(size_t)(a / k) * H + (size_t)tp_rank * Hs + c]", "x[(size_t)(a / k) * H + c]", 1, STAGE),
    # ---- expert MLP
    ("silu_sign", "hmid[i] = g / (1.0 + exp(-g)) * u;", "hmid[i] = g / (1.0 + exp(g)) * u;", 1, LAYER),
    ("gate_and_up_swapped", "hmid[i] = g / (1.0 + exp(-g)) * u;", "hmid[i] = u / (1.0 + exp(-u)) * g;", 1, LAYER),
    ("no_activation", "hmid[i] = g / (1.0 + exp(-g)) * u;", "hmid[i] = g * u;", 1, LAYER),
    ("w_down_transposed", "double wd = (double)Wd[(size_t)h * I + i];", "double wd = (double)Wd[(size_t)i * H + h];", 1, LAYER),
    ("w_gate_transposed", "double wg = (double)Wg[(size_t)i * H + h];", "double wg = (double)Wg[(size_t)h * I + i];", 1, LAYER),
    ("expert_weights_not_advanced", "const float *Wu = w_up + (size_t)e * I * H;\n        const float *Wd = w_down + (size_t)e * H * I;\n#pragma omp parallel for schedule(dynamic, 1)\n        for (int r = offsets[e]; r < offsets[e + 1]; ++r) {\n            const float *xr",
     "const float *Wu = w_up;\n        const float *Wd = w_down + (size_t)e * H * I;\n#pragma omp parallel for schedule(dynamic, 1)\n        for (int r = offsets[e]; r < offsets[e + 1]; ++r) {\n            const float *xr", 1, LAYER),
    ("gate_scale_index_transposed", "if (s_gate) wg *= (double)s_gate[((size_t)e * bI + i / 128) * bH + h / 128];",
     "if (s_gate) wg *= (double)s_gate[((size_t)e * bH + h / 128) * bI + i / 128];", 1, LAYER),
    ("down_scale_dropped", "if (s_down) wd *= (double)s_down[((size_t)e * bH + h / 128) * bI + i / 128];", "", 1, LAYER),
    # ---- combine
    ("combine_weight_dropped", "if (pos >= 0) acc += (double)w[(size_t)t * k + j] * ys[(size_t)pos * H + h];",
     "if (pos >= 0) acc += ys[(size_t)pos * H + h];", 1, LAYER),
    ("combine_weight_of_wrong_pick", "if (pos >= 0) acc += (double)w[(size_t)t * k + j] * ys[(size_t)pos * H + h];",
     "if (pos >= 0) acc += (double)w[(size_t)t * k + (k - 1 - j)] * ys[(size_t)pos * H + h];", 1, LAYER),
    ("combine_shared_dropped", "if (shared_ys) acc += shared_ys[(size_t)t * H + h];", "", 1, LAYER),
    ("stage_never_accumulates", "if (accumulate) acc += (double)out_block[(size_t)t * Hb + c];", "", 1, STAGE),
    ("stage_always_accumulates", "if (accumulate) acc += (double)out_block[(size_t)t * Hb + c];",
     "acc += (double)out_block[(size_t)t * Hb + c];", 1, STAGE),
    # ---- storage formats and the activation quantiser
    ("e4m3_bias_off_by_one", "else v = ldexp(1.0 + (double)m / 8.0, ex - 7);", "else v = ldexp(1.0 + (double)m / 8.0, ex - 8);", 1, LAYER),
    ("e4m3_subnormal_exponent", "else if (ex == 0) v = ldexp((double)m / 8.0, -6);", "else if (ex == 0) v = ldexp((double)m / 8.0, -7);", 1, LAYER),
    ("bf16_lower_half", "uint32_t u = (uint32_t)bits[i] << 16;", "uint32_t u = (uint32_t)bits[i];", 1, LAYER),
    ("quant_code_value_bias", ": ldexp(1.0 + (double)m / 8.0, ex - 7);", ": ldexp(1.0 + (double)m / 8.0, ex - 8);", 1, FP8ACT),
    ("quant_scale_of_max_not_amax", "amax = fmaxf(amax, fabsf(xb[j]));", "amax = fmaxf(amax, xb[j]);", 1, FP8ACT),
    ("quant_ties_away", "if (d < bd || (d == bd && (c & 1) == 0 && (best & 1) == 1)) { bd = d; best = c; }",
     "if (d <= bd) { bd = d; best = c; }", 1, FP8ACT),
    ("quant_range_240", "float scale = amax > 0.0f ? amax / 448.0f : 1.0f;", "float scale = amax > 0.0f ? amax / 240.0f : 1.0f;", 1, FP8ACT),
    ("quant_hmid_skipped", "hq[i] = e4m3_value(ch[i]) * (double)sh[i / 128];", "hq[i] = (double)hb[i];", 1, FP8ACT),
    ("quant_hmid_without_up", "hb[i] = (float)(g / (1.0 + exp(-g)) * u);", "hb[i] = (float)(g / (1.0 + exp(-g)));", 1, FP8ACT),
    ("quant_hmid_cut_to_upper_half", "hb[i] = (float)(g / (1.0 + exp(-g)) * u);",
     "{ float f_ = (float)(g / (1.0 + exp(-g)) * u); uint32_t b_; memcpy(&b_, &f_, 4); b_ &= 0xFFFF0000u; memcpy(&hb[i], &b_, 4); }", 1, FP8ACT),
    ("quant_act_scale_dropped", "xq[h] = e4m3_value(cx[h]) * (double)sx[h / 128];", "xq[h] = e4m3_value(cx[h]);", 1, FP8ACT),
    ("quant_weight_scale_index_transposed", "(double)Wg[(size_t)i * H + h] * (double)s_gate[((size_t)e * bI + i / 128) * bH + h / 128]",
     "(double)Wg[(size_t)i * H + h] * (double)s_gate[((size_t)e * bH + h / 128) * bI + i / 128]", 1, FP8ACT),
    ("quant_hidden_scale_of_block_0", "hq[i] = e4m3_value(ch[i]) * (double)sh[i / 128];", "hq[i] = e4m3_value(ch[i]) * (double)sh[0];", 1, FP8ACT),
]


def _run_pins(lib, files):
    env = dict(os.environ, MOE_ORACLE_LIB=lib, OMP_NUM_THREADS="1")
    p = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    return p.returncode, p.stdout[-1500:]


def _build(src_text, path_c, path_so):
    with open(path_c, "w") as f:
        f.write(src_text)
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", path_so, path_c, "-lm"])


def test_unchanged_copy_passes(tmp_path):
    """The harness itself: a verbatim copy of the source passes every pin."""
    so = str(tmp_path / "copy.so")
    _build(open(SRC).read(), str(tmp_path / "copy.c"), so)
    rc, out = _run_pins(so, ROUTE + LAYER + STAGE + FP8ACT)
    assert rc == 0, out


def test_every_planted_mistake_fails_a_pin(tmp_path):
    src = open(SRC).read()
    for name, old, new, count, files in MUTANTS:
        assert src.count(old) == count, "%s: the text to replace occurs %d times" % (name, src.count(old))

    def job(m):
        name, old, new, _, files = m
        so = str(tmp_path / (name + ".so"))
        _build(src.replace(old, new), str(tmp_path / (name + ".c")), so)
        return (name,) + _run_pins(so, files)

    with ThreadPoolExecutor(max_workers=6) as pool:
        results = list(pool.map(job, MUTANTS))
    # pytest exits with 1 when a test failed; anything else (a crash, a usage
    # error) is a broken harness, not a caught mistake
    broken = [(n, rc, out) for n, rc, out in results if rc not in (0, 1)]
    assert not broken, broken
    survivors = [n for n, rc, _ in results if rc == 0]
    assert not survivors, "no pin notices: %s" % survivors
