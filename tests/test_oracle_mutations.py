"""The pins are only worth something if they catch mistakes.  Each case below plants one plausible slip in a
copy of the oracle's C source (on the CPU, in a temporary build) and demands that the pin suite fails."""
import os
import subprocess
import sys
import tempfile

import pytest

import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "jo_attention.c")

MUTATIONS = {
    "scale dropped": ("return p->scale * s;", "return s;"),
    "kv head by modulo": ("int kv = h / (p->Hq / p->Hkv);\n    const uint16_t *qr", "int kv = h % p->Hkv;\n    const uint16_t *qr"),
    "slot off by one": ("int slot = j % p->page;", "int slot = (j + 1) % p->page;"),
    "last token dropped": ("int L = p->lens[b];\n    int kv", "int L = p->lens[b] - 1;\n    int kv"),
    "weights not normalised": ("w[j] /= z;", "w[j] /= 1.0;"),
    "scores from V": ("const uint16_t *kr = token_row(p, p->k, b, kv, j);", "const uint16_t *kr = token_row(p, p->v, b, kv, j);"),
    "values from K": ("const uint16_t *vr = token_row(p, p->v, b, kv, j);", "const uint16_t *vr = token_row(p, p->k, b, kv, j);"),
    "no max subtraction": ("w[j] = exp(w[j] - m);", "w[j] = exp(w[j]);"),
    "pages of a request read in reverse": ("p->bt[(int64_t)b * p->maxp + j / p->page]", "p->bt[(int64_t)b * p->maxp + (p->lens[b] - 1) / p->page - j / p->page]"),
    "query row of another head": ("((int64_t)b * p->Hq + h) * p->D", "((int64_t)b * p->Hq + (h ^ 1)) * p->D"),
    "merge ignores the maxima": ("double e = exp(m[i] - M);", "double e = 1.0;"),
    "partial sum counts tokens": ("l += e;", "l += 1.0;"),
    "bf16 widened with a shifted exponent": ("uint32_t u = (uint32_t)bits << 16;", "uint32_t u = ((uint32_t)bits << 16) + 0x00800000u;"),
}


def run_pins(jo):
    """All pins that need no pytest machinery; raises AssertionError (or a numeric error) on the first failure."""
    pins.test_single_key_returns_v_exactly(jo)
    for L in (2, 16, 17, 31, 32, 33, 100):
        pins.test_identical_keys_give_mean_of_v(jo, L)
    for L in (17, 31, 32, 33):
        pins.test_zero_query_is_uniform_over_exactly_L_tokens(jo, L)
    pins.test_page_permutation_invariance_bitwise(jo)
    pins.test_weights_sum_to_one_and_reproduce_output(jo)
    pins.test_convex_hull_and_constant_v(jo)
    for D in (64, 128):
        pins.test_two_keys_logistic_weight_and_default_scale(jo, D)
    pins.test_shift_invariance_of_keys(jo)
    pins.test_dominant_key_no_overflow(jo)
    pins.test_gqa_structure(jo)
    pins.test_split_and_merge_equals_whole(jo)
    pins.test_matches_torch_sdpa_float64(jo)
    pins.test_matches_numpy_brute_force(jo)
    pins.test_poisoned_slots_never_influence(jo)
    pins.test_empty_request_gives_zero_row_and_rows_subset(jo)


def test_unmutated_oracle_passes(jo):
    run_pins(jo)


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_pins_catch_planted_mistake(name):
    # each mutant runs in a process of its own: a planted indexing slip may read anywhere
    old, new = MUTATIONS[name]
    src = open(SRC).read()
    assert src.count(old) >= 1, f"mutation site for '{name}' not found"
    here = os.path.dirname(os.path.abspath(__file__))
    with tempfile.TemporaryDirectory() as tmp:
        c = os.path.join(tmp, "mutant.c")
        so = os.path.join(tmp, "mutant.so")
        open(c, "w").write(src.replace(old, new, 1))
        subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", so, c, "-lm"])
        code = ("import sys; sys.path[:0] = [%r, %r]\n"
                "from oracle import jo\n"
                "import test_oracle_mutations as t\n"
                "jo._lib = jo.load_library(%r)\n"
                "try:\n"
                "    t.run_pins(jo)\n"
                "except (AssertionError, ValueError, FloatingPointError) as e:\n"
                "    print('caught:', type(e).__name__); sys.exit(3)\n"
                "sys.exit(0)\n") % (os.path.dirname(here), here, so)
        r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
        assert r.returncode == 3, f"mutant '{name}' was not caught by an assertion (exit {r.returncode}): {r.stdout[-300:]} {r.stderr[-300:]}"


# ---- the prefill oracle: the same exercise with its own pins ----
import test_oracle_prefill_pins as ppins

PREFILL_MUTATIONS = {
    "prefill: own position not visible": ("int last = c + t; /* attends to positions 0 .. last */", "int last = c + t - 1;"),
    "prefill: sees one token of the future": ("int last = c + t; /* attends to positions 0 .. last */", "int last = c + t + 1 < L ? c + t + 1 : L - 1;"),
    "prefill: context length ignored": ("int n = q_lens[b], c = L - n, kv = h / G;", "int n = q_lens[b], c = 0, kv = h / G;"),
    "prefill: query row ignores the offset": ("int64_t row = (int64_t)q_offsets[b] + t;", "int64_t row = (int64_t)t;"),
    "prefill: kv head by modulo": ("int n = q_lens[b], c = L - n, kv = h / G;", "int n = q_lens[b], c = L - n, kv = h % Hkv;"),
    "prefill: weights not normalised": ("double wj = w[j] / z;", "double wj = w[j];"),
    "prefill: scale dropped": ("w[j] = p.scale * s;", "w[j] = s;"),
}


def run_prefill_pins(jo):
    ppins.test_single_new_token_is_decode_attention(jo)
    ppins.test_matches_torch_sdpa_with_causal_mask_float64(jo)
    ppins.test_first_token_of_a_full_prefill_returns_v0_and_future_tokens_do_not_matter(jo)
    ppins.test_chunked_prefill_equals_one_shot(jo)
    ppins.test_malformed_arguments_are_rejected(jo)


def test_unmutated_prefill_oracle_passes(jo):
    run_prefill_pins(jo)


@pytest.mark.parametrize("name", sorted(PREFILL_MUTATIONS))
def test_prefill_pins_catch_planted_mistake(name):
    old, new = PREFILL_MUTATIONS[name]
    src = open(SRC).read()
    assert src.count(old) >= 1, f"mutation site for '{name}' not found"
    here = os.path.dirname(os.path.abspath(__file__))
    with tempfile.TemporaryDirectory() as tmp:
        c = os.path.join(tmp, "mutant.c")
        so = os.path.join(tmp, "mutant.so")
        open(c, "w").write(src.replace(old, new, 1))
        subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", so, c, "-lm"])
        code = ("import sys; sys.path[:0] = [%r, %r]\n"
                "from oracle import jo\n"
                "import test_oracle_mutations as t\n"
                "jo._lib = jo.load_library(%r)\n"
                "try:\n"
                "    t.run_prefill_pins(jo)\n"
                "except (AssertionError, ValueError, FloatingPointError) as e:\n"
                "    print('caught:', type(e).__name__); sys.exit(3)\n"
                "sys.exit(0)\n") % (os.path.dirname(here), here, so)
        r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
        assert r.returncode == 3, f"mutant '{name}' was not caught by an assertion (exit {r.returncode}): {r.stdout[-300:]} {r.stderr[-300:]}"
