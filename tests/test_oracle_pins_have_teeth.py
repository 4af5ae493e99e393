"""Do the oracle's pins notice a mistake?  Each case below plants ONE plausible error in a copy of the
oracle's C source (a dropped term, a wrong sign or index, swapped operands or constants), builds it, and
runs the pin tests of the part it touches against that build: they must fail.  An unchanged copy must
pass.  Everything here runs on the CPU; the product library is not involved."""
import concurrent.futures
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "difr_oracle.c")

NOISE = ["test_oracle_noise.py"]
GUMBEL = ["test_oracle_gumbel.py"]
IPT = ["test_oracle_ipt.py"]
LIK = ["test_oracle_likelihood.py"]
FILT = ["test_oracle_ipt_filtered.py"]
ADM = ["test_oracle_admissible.py"]
LM = ["test_oracle_lmhead.py"]
RANK = ["test_oracle_rank.py"]
ALL = sorted(set(NOISE + GUMBEL + IPT + LIK + FILT + ADM + LM + RANK))

# (name, text in the source, what it becomes, which occurrence (0-based), pin files that must notice)
MUTATIONS = [
    ("philox_multipliers_swapped", "M0 = 0xD2511F53u, M1 = 0xCD9E8D57u", "M0 = 0xCD9E8D57u, M1 = 0xD2511F53u", 0, NOISE),
    ("philox_nine_rounds", "round < 10; ++round", "round < 9; ++round", 0, NOISE),
    ("philox_wrong_key_word", "(uint32_t)(p1 >> 32) ^ c1 ^ k0;", "(uint32_t)(p1 >> 32) ^ c1 ^ k1;", 0, NOISE),
    ("philox_no_key_schedule", "k0 += W0;", "k0 += 0;", 0, NOISE),
    ("counter_words_transposed", "{ (uint32_t)(v >> 2), pos, seq, stream }", "{ (uint32_t)(v >> 2), seq, pos, stream }", 0, NOISE),
    ("counter_block_index", "{ (uint32_t)(v >> 2), pos,", "{ (uint32_t)(v >> 3), pos,", 0, NOISE),
    ("output_word_order", "return out[v & 3u];", "return out[3u - (v & 3u)];", 0, NOISE),
    ("seed_halves_swapped", "{ (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32) }",
     "{ (uint32_t)(seed >> 32), (uint32_t)(seed & 0xFFFFFFFFu) }", 0, NOISE),
    ("uniform_cell_edge", "(2.0 * (double)k + 1.0) * 0x1p-24", "(2.0 * (double)k) * 0x1p-24", 0, NOISE),
    ("uniform_24_bits", "uint32_t k = r >> 9;", "uint32_t k = r >> 8;", 0, NOISE),
    ("gumbel_sign", "    return -log(t);", "    return log(t);", 0, NOISE),
    ("gumbel_upper_branch", "t = -log1p(-(1.0 - u));", "t = -log1p(-u);", 0, NOISE),
    ("bf16_decode_shift", "uint32_t w = (uint32_t)h << 16;", "uint32_t w = (uint32_t)h << 15;", 0, GUMBEL),
    ("temperature_multiplied", "double y = x[v] / T + g;", "double y = x[v] * T + g;", 0, GUMBEL),
    ("noise_dropped", "double y = x[v] / T + g;", "double y = x[v] / T;", 0, GUMBEL),
    ("margin_sign", "*margin = best - yt;", "*margin = yt - best;", 0, GUMBEL),
    ("argmax_keeps_first", "if (best_v < 0 || y > best) {", "if (best_v < 0) {", 0, GUMBEL),
    ("gumbel_uses_ipt_stream", "ORACLE_STREAM_GUMBEL, (uint64_t)v);\n        double u", "ORACLE_STREAM_IPT, (uint64_t)v);\n        double u", 0, GUMBEL),
    ("ipt_uses_gumbel_stream", "oracle_noise_word(seed, seq, pos, ORACLE_STREAM_IPT, 0);", "oracle_noise_word(seed, seq, pos, ORACLE_STREAM_GUMBEL, 0);", 0, IPT),
    ("softmax_temperature", "Z += exp(x[v] / T - m);", "Z += exp(x[v] * T - m);", 0, IPT),
    ("prefix_includes_claim", "        c += e;\n        if (first < 0 && c / Z > u) first = v;",
     "        if (first < 0 && c / Z > u) first = v;\n        c += e;", 0, IPT),
    ("interval_starts_after_claim", "        double e = exp(x[v] / T - m);\n        if (valid && v == claimed) {\n            a = c / Z;",
     "        double e = exp(x[v] / T - m);\n        if (valid && v == claimed) {\n            a = (c + e) / Z;", 0, IPT),
    ("distance_term_dropped", "if (a - u > d) d = a - u;", "", 0, IPT),
    ("distance_sign", "if (u - b > d) d = u - b;", "if (b - u > d) d = b - u;", 0, IPT),
    ("match_ignores_upper_end", "if (a <= u && u < b) f |= ORACLE_FLAG_MATCH;", "if (a <= u) f |= ORACLE_FLAG_MATCH;", 0, IPT),
    ("log_mass_sign", "mass = 0.5 * (erf(zb) + erf(-za));", "mass = 0.5 * (erf(zb) - erf(-za));", 0, IPT),
    ("log_mass_sigma", "double zb = (b - u) / (sigma * M_SQRT2);", "double zb = (b - u) / (sigma * 2.0);", 0, IPT),
    ("admissible_strict", "if (m <= delta) ++c;", "if (m < delta) ++c;", 0, ADM),
    ("admissible_sign", "double m = max_score - y[v];", "double m = y[v] - max_score;", 0, ADM),
    ("active_set_keeps_claim", "if (v == claimed) continue;", "", 0, LIK),
    ("active_set_ascending", "if (p->key > q->key) return -1;\n    if (p->key < q->key) return 1;",
     "if (p->key > q->key) return 1;\n    if (p->key < q->key) return -1;", 0, LIK),
    ("rank_ties_to_higher_index", "return p->idx < q->idx ? -1 : (p->idx > q->idx ? 1 : 0);",
     "return p->idx > q->idx ? -1 : (p->idx < q->idx ? 1 : 0);", 0, FILT),
    ("A_without_temperature", "A[j] = x[claimed] - x[i] + T * (g[claimed] - g[i]);", "A[j] = x[claimed] - x[i] + (g[claimed] - g[i]);", 0, LIK),
    ("A_sign", "A[j] = x[claimed] - x[i] + T * (g[claimed] - g[i]);", "A[j] = x[i] - x[claimed] + T * (g[i] - g[claimed]);", 0, LIK),
    ("B_sign", "B[j] = tau - x[i];", "B[j] = x[i] - tau;", 0, LIK),
    ("indicator_dropped", "if (x[claimed] + xj > tau) {", "if (1) {", 0, LIK),
    ("max_becomes_min", "normal_cdf(fmax(xj + A[i], B[i]) / sigma)", "normal_cdf(fmin(xj + A[i], B[i]) / sigma)", 0, LIK),
    ("normal_cdf_tail", "return 0.5 * erfc(-z / M_SQRT2);", "return 0.5 * erfc(z / M_SQRT2);", 0, LIK),
    ("noise_not_scaled", "const double xj = sigma * z[j];", "const double xj = z[j];", 0, LIK),
    ("top_p_before_renormalising", "cum += exp((order[r].key - order[0].key) / T) / Z;", "cum += exp((order[r].key - order[0].key) / T);", 0, LIK),
    ("tau_is_first_dropped", "tau = a[kept - 1].key;", "tau = a[kept < V ? kept : kept - 1].key;", 0, LIK),
    ("filtered_not_renormalised", "if (in_K[v]) Z += exp((x[v] - top) / T);", "Z += exp((x[v] - top) / T);", 0, FILT),
    ("filtered_keeps_everything", "double e = in_K[v] ? exp((x[v] - top) / T) : 0.0;", "double e = exp((x[v] - top) / T);", 0, FILT),
    ("filtered_top_p_ignored", "    if (top_p < 1.0) {\n        double Z = 0.0;", "    if (0) {\n        double Z = 0.0;", 0, FILT),
    ("lmhead_k_reversed", "acc += decode_bf16(h[k]) * decode_bf16(w[k]);", "acc += decode_bf16(h[k]) * decode_bf16(w[d - 1 - k]);", 0, LM),
    ("lmhead_row_stride", "const uint16_t *w = W + (size_t)v * (size_t)ldw;", "const uint16_t *w = W + (size_t)(V - 1 - v) * (size_t)ldw;", 0, LM),
    ("rank_counts_ties", "if (x[v] > x[claimed]) ++r;", "if (x[v] >= x[claimed]) ++r;", 0, RANK),
    ("class_rank_cutoff", "(int64_t)ranks[n] < R) {", "(int64_t)ranks[n] <= R) {", 0, RANK),
    ("class_bits", "bits[n] = log2((double)R);", "bits[n] = log2((double)V);", 0, RANK),
    ("pool_sum_not_mean", "double mean = sum / (double)(hi - lo);", "double mean = sum;", 0, GUMBEL + IPT),
    ("flag_direction", "seq_flag[s] = (mean <= tau) ? 0 : 1;", "seq_flag[s] = (mean <= tau) ? 1 : 0;", 0, GUMBEL + IPT),
]


def _build(tmp, name, source):
    c = os.path.join(tmp, name + ".c")
    so = os.path.join(tmp, name + ".so")
    with open(c, "w") as f:
        f.write(source)
    subprocess.run(["gcc", "-O2", "-std=gnu11", "-fopenmp", "-fPIC", "-shared", "-w", "-o", so, c, "-lm"], check=True)
    return so


def _pins(lib, files):
    env = dict(os.environ, DIFR_ORACLE_LIB=lib, OMP_NUM_THREADS="2")
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + [os.path.join(HERE, f) for f in files]
    return subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)


def _mutate(src, old, new, which):
    parts = src.split(old)
    assert len(parts) > which + 1, "the oracle no longer contains: " + old
    mutated = old.join(parts[:which + 1]) + new + old.join(parts[which + 1:])
    assert mutated != src
    return mutated


@pytest.fixture(scope="module")
def outcomes(tmp_path_factory):
    """Build and check every variant once, a few at a time (each is a compiler run and a short pytest run)."""
    tmp = str(tmp_path_factory.mktemp("oracle_variants"))
    src = open(SRC).read()
    jobs = {"unchanged": (src, ALL)}
    for name, old, new, which, files in MUTATIONS:
        jobs[name] = (_mutate(src, old, new, which), files)

    def run(item):
        name, (source, files) = item
        return name, _pins(_build(tmp, name, source), files)

    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as pool:
        return dict(pool.map(run, jobs.items()))


def test_unchanged_copy_passes_every_pin(outcomes):
    r = outcomes["unchanged"]
    assert r.returncode == 0, r.stdout[-3000:]


@pytest.mark.parametrize("name", [m[0] for m in MUTATIONS])
def test_planted_mistake_is_noticed(outcomes, name):
    r = outcomes[name]
    assert r.returncode == 1, "no pin noticed '%s':\n%s" % (name, r.stdout[-1500:])
