"""Do the pins of the CPU oracle discriminate?  Each case plants ONE plausible mistake in a private copy of the oracle's
C source (a wrong sign, bound, constant, index, a dropped term), builds it on the CPU, and requires that a named pin of
test_oracle_pins.py fails on it.  The unmodified copy must pass the same pins.  Nothing here touches the GPU, the HIP
library or the repository's own oracle build."""
import importlib.util
import os
import re
import shutil
import sys

import pytest

import test_oracle_pins as pins
from paper_2604_03950_amd import workloads as wl

ORACLE_DIR = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle")

# (what is planted, regular expression in dma_oracle.c, replacement, the pin that must notice)
MUTATIONS = [
    ("causal mask also hides the diagonal",
     r"if \(\(causal && j > i\) \|\| j >= S\) \{\n                acc = -INFINITY;",
     "if ((causal && j >= i && i > 0) || j >= S) {\n                acc = -INFINITY;", "skeleton"),
    ("window one tile too wide", r"dist < \(int64_t\)band", "dist <= (int64_t)band", "mixed"),
    ("rescale factor inverted", r"exp2\(m - mnew\)", "exp2(mnew - m)", "skeleton"),
    ("running sum not rescaled", r"l = alpha \* l \+ psum;", "l = l + psum;", "skeleton"),
    ("accumulator not rescaled", r"for \(int d = 0; d < D; \+\+d\) O\[d\] \*= alpha;", ";", "skeleton"),
    ("e_max of E2M1 off by one", r"fmt == ORACLE_FMT_E2M1 \? 2 :", "fmt == ORACLE_FMT_E2M1 ? 3 :", "e8m0"),
    ("e_max of E4M3 off by one", r"ORACLE_FMT_E5M2 \? 15 : 8;", "ORACLE_FMT_E5M2 ? 15 : 7;", "e8m0"),
    ("softmax factor 1/D instead of 1/sqrt(D)", r"const double c = 1\.4426950408889634074 / sqrt\(\(double\)D\);",
     "const double c = 1.4426950408889634074 / (double)D;", "skeleton"),
    ("query pre-scale with ln 2 instead of log2 e", r"return \(float\)\(1\.4426950408889634074 / sqrt\(\(double\)D\)\);",
     "return (float)(0.6931471805599453 / sqrt((double)D));", "prescale"),
    ("dot product pairs the wrong elements", r"acc \+= qq\[d\] \* kr\[d\];", "acc += qq[d] * kr[D - 1 - d];", "skeleton"),
    ("query formats swapped between the phases", r"use_hi \? q_hi : q_lo", "use_hi ? q_lo : q_hi", "all_high"),
    ("key formats swapped between the phases", r"use_hi \? kseen_hi : kseen_lo", "use_hi ? kseen_lo : kseen_hi", "all_high"),
    ("P never rounded to 16 bit", r"p_round \? oracle_round_to_bf16\(p\) : p", "p", "mixed"),
    ("bf16 rounding keeps 7 bits", r"int quantum = \(ex - 1\) - 7;       /\* spacing", "int quantum = (ex - 1) - 6;       /* spacing", "bf16"),
    ("E2M1 mantissa carry lost", r"if \(m == 2\) \{ e \+= 1; m = 0; \}", "if (m == 2) { m = 1; }", "e2m1_grid"),
    ("E2M1 ties round half up", r"mag = \(int\)nearbyint\(2\.0 \* a\);", "mag = (int)floor(2.0 * a + 0.5);", "e2m1_paper"),
    ("E8M0 lower clamp wrong", r"if \(biased < 0\) biased = 0;", "if (biased < 0) biased = 1;", "e8m0"),
    ("row sum from the rounded P", r"psum \+= pt\[t\];", "psum += oracle_round_to_bf16(pt[t]);", "skeleton"),
    ("key tiles visited in descending order", r"for \(int64_t jt = 0; jt < n_tiles; \+\+jt\) \{\n        const int64_t dist",
     "for (int64_t jt = n_tiles - 1; jt >= 0; --jt) {\n        const int64_t dist", "mixed"),
    ("sink window one tile too wide", r"jt < \(int64_t\)sink", "jt <= (int64_t)sink", "mixed"),
    ("e_max of E5M2 off by one", r"ORACLE_FMT_E5M2 \? 15 : 8;", "ORACLE_FMT_E5M2 ? 14 : 8;", "e5m2"),
    ("window without the causal mask looks back only", r"\(it >= jt\) \? it - jt : jt - it", "it - jt", "noncausal"),
    ("per-token scale divides by 448 instead of 448 * 6", r"amax / 2688\.0f, b = 2688\.0f / amax", "amax / 448.0f, b = 448.0f / amax", "token"),
    ("MX-format P V in blocks of 16 keys", r"for \(int t0 = 0; t0 < tile; t0 \+= 32\) \{\n                const int n = \(tile - t0 < 32\) \? tile - t0 : 32;",
     "for (int t0 = 0; t0 < tile; t0 += 16) {\n                const int n = (tile - t0 < 16) ? tile - t0 : 16;", "pv_mx"),
    ("FP4 nibbles packed the other way round", r"if \(d & 1\) codes\[d >> 1\] = \(uint8_t\)\(codes\[d >> 1\] \| \(cd << 4\)\);\n                else       codes\[d >> 1\] = cd;",
     "if (d & 1) codes[d >> 1] = (uint8_t)(codes[d >> 1] | cd);\n                else       codes[d >> 1] = (uint8_t)(cd << 4);", "packing"),
    ("E2M1 clamps at 4 instead of 6", r"fmt == ORACLE_FMT_E2M1 \? 6\.0 :", "fmt == ORACLE_FMT_E2M1 ? 4.0 :", "saturating"),
    ("E4M3 saturates at 480 (code 0x7F)", r"if \(mag > 0x7E\) mag = 0x7E;", "if (mag > 0x7F) mag = 0x7F;", "e4m3_fixed"),
    ("E4M3 subnormals truncated", r"mag = \(int\)nearbyint\(ldexp\(a, 9\)\);", "mag = (int)floor(ldexp(a, 9));", "e4m3_fixed"),
    ("E4M3 mantissa carry lost", r"if \(m == 8\) \{ e \+= 1; m = 0; \}", "if (m == 8) { m = 7; }", "e4m3_brute"),
    ("shared scale from blocks of 16", r"float v = oracle_bf16_to_f32\(x\[blk \* 32 \+ t\]\);\n            if \(is_query\) \{\n                volatile float prod = v \* c;     /\* one binary32 multiply, rounded once \*/",
     "float v = oracle_bf16_to_f32(x[blk * 32 + t % 16]);\n            if (is_query) {\n                volatile float prod = v * c;     /* one binary32 multiply, rounded once */", "tiny_quant"),
    ("noise allowance of the open decisions four times larger", r"ldexp\(fabs\(s\) \+ fabs\(m\) \+ 1\.0, -22\)",
     "ldexp(fabs(s) + fabs(m) + 1.0, -20)", "open"),
    ("a decision taken the other way lands on the same neighbour", r"return \(rounded == lower\) \? lower \+ ldexp\(1\.0, quantum\) : lower;",
     "return rounded;", "other_way"),
    ("sign of an underflowed element dropped", r"int neg = signbit\(xs\[t\]\) \? 1 : 0;", "int neg = (xs[t] < 0.0f && fabsf(xs[t]) > 0x1p-20f) ? 1 : 0;", "edge_blocks"),
]


def run_pin(which, oracle, tiny):
    if which == "skeleton":
        pins.test_online_softmax_skeleton_against_sdpa(oracle, tiny)
    elif which == "mixed":
        for band in (1, 2):
            pins.test_mixed_tiles_match_per_element_rewrite(oracle, tiny, band, True)
    elif which == "all_high":
        pins.test_all_high_equals_softmax_of_dequantized(oracle, tiny)
    elif which == "e8m0":
        pins.test_e8m0_hand_built_blocks(oracle)
    elif which == "prescale":
        pins.test_query_prescale_single_rounding(oracle)
    elif which == "bf16":
        pins.test_round_to_bf16_against_torch_and_ties(oracle)
    elif which == "e2m1_grid":
        pins.test_e2m1_grid_roundtrip_and_ties(oracle)
    elif which == "e2m1_paper":
        pins.test_e2m1_paper_examples(oracle)
    elif which == "packing":
        pins.test_packing_nibbles(oracle)
    elif which == "saturating":
        pins.test_saturating_block(oracle)
    elif which == "e4m3_fixed":
        pins.test_e4m3_codes_roundtrip_and_fixed_points(oracle)
    elif which == "e4m3_brute":
        pins.test_e4m3_bruteforce_all_bf16(oracle)
    elif which == "tiny_quant":
        pins.test_quantizer_matches_bruteforce_on_tiny_workload(oracle)
    elif which == "edge_blocks":
        pins.test_edge_blocks(oracle)
    elif which == "e5m2":
        pins.test_e5m2_shared_scale_and_blocks(oracle)
    elif which == "noncausal":
        pins.test_noncausal_mixed_tiles_match_per_element_rewrite(oracle, tiny, 1, 0, True)
    elif which == "token":
        pins.test_token_scale_fixed_points(oracle)
    elif which == "open":
        pins.test_open_decisions_cover_a_binary32_implementation_and_little_more(oracle)
    elif which == "other_way":
        pins.test_row_with_decisions_taken_the_other_way_matches_per_element_rewrite(oracle, tiny)
    elif which == "pv_mx":
        pins.test_mx_pv_matches_per_element_rewrite(oracle, tiny, 1, True, 256)
    else:
        raise KeyError(which)


def private_oracle(tmp_path, name, pattern=None, replacement=None):
    """A copy of the oracle package under tmp_path (its C source optionally changed), imported under its own name."""
    dst = os.path.join(str(tmp_path), name)
    shutil.copytree(ORACLE_DIR, dst, ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    if pattern is not None:
        path = os.path.join(dst, "dma_oracle.c")
        src = open(path).read()
        changed, n = re.subn(pattern, lambda m: replacement, src, count=1)
        assert n == 1, "the text this case changes is no longer in the oracle: update the case"
        open(path, "w").write(changed)
    spec = importlib.util.spec_from_file_location(name, os.path.join(dst, "__init__.py"), submodule_search_locations=[dst])
    mod = importlib.util.module_from_spec(spec)
    sys.modules[name] = mod
    try:
        spec.loader.exec_module(mod)
        mod.build(force=True)
    finally:
        sys.modules.pop(name, None)
    return mod


@pytest.fixture(scope="module")
def tiny():
    w = wl.CONFIGS["tiny"]
    return (w,) + wl.generate(w)


def test_unmodified_copy_passes_the_pins_used_here(tmp_path, tiny):
    oracle = private_oracle(tmp_path, "oracle_copy")
    for which in ("skeleton", "mixed", "all_high", "e8m0", "prescale", "bf16", "e2m1_grid", "e2m1_paper", "e5m2", "noncausal",
                  "token", "pv_mx", "packing", "saturating", "e4m3_fixed", "e4m3_brute", "tiny_quant", "edge_blocks", "other_way"):
        run_pin(which, oracle, tiny)


@pytest.mark.parametrize("case", range(len(MUTATIONS)), ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, tiny, case):
    what, pattern, replacement, which = MUTATIONS[case]
    oracle = private_oracle(tmp_path, f"oracle_mut_{case}", pattern, replacement)
    with pytest.raises(AssertionError):
        run_pin(which, oracle, tiny)
