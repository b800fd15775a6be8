"""The pins have teeth: plant one plausible mistake at a time in a COPY of the
oracle's source (on the CPU), rebuild it, and check that the pin suite fails.
A mistake that no pin catches would mean the oracle is not really pinned there."""
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "nf4_oracle.c")

MUTATIONS = [
    ("nibble order swapped",
     "(i & 1) == 0 ? (unsigned)(q >> 4) : (unsigned)(q & 0x0Fu)",
     "(i & 1) == 0 ? (unsigned)(q & 0x0Fu) : (unsigned)(q >> 4)"),
    ("scale indexed by a 512-element tile", "float scale = absmax[i / blocksize];", "float scale = absmax[i / 512];"),
    ("one level off by 1e-4 relative", "-0.39491748809814453f,", "-0.39495698f,"),
    ("two levels transposed", "0.16093020141124725f,\n    0.24611230194568634f,", "0.24611230194568634f,\n    0.16093020141124725f,"),
    ("fp16 ties round up instead of to even",
     "if (dropped > 0x1000u || (dropped == 0x1000u && (h & 1u))) h += 1;", "if (dropped >= 0x1000u) h += 1;"),
    ("fp16 subnormals flushed", "if (shift > 24) return sign;", "if (shift > 0) return sign;"),
    ("bf16 truncates", "if (dropped > 0x8000u || (dropped == 0x8000u && (kept & 1u))) kept += 1;", ";"),
    ("double-quant offset dropped", "return prod + offset;", "return prod;"),
    ("double-quant multiply-add fused", "float prod = code2[absmax_q8[b]] * scale2[b / 256];\n    return prod + offset;",
     "return fmaf(code2[absmax_q8[b]], scale2[b / 256], offset);"),
    ("double-quant groups of 128", "scale2[b / 256]", "scale2[b / 128]"),
    ("quantiser ties go to the upper level", "if (d < best_d) { best_d = d; best = k; }", "if (d <= best_d) { best_d = d; best = k; }"),
    ("quantiser zero block gets code 0", "unsigned best = 7;", "unsigned best = 0;"),
    ("quantiser absmax is the signed max", "float m = fabsf(src[i]);", "float m = src[i];"),
    ("second-level code truncated instead of rounded", "float r = rintf(scaled / s);", "float r = truncf(scaled / s);"),
    ("second-level offset is the median-free zero", "float off = nb > 0 ? (float)(sum / (double)nb) : 0.0f;", "float off = 0.0f;"),
    ("gemv reads activations backwards", "f16_bits_to_double(x[(int64_t)b * K + k])", "f16_bits_to_double(x[(int64_t)b * K + (K - 1 - k)])"),
    ("gemm weight not rounded to fp16", "double w16 = f16_bits_to_double(nf4o_f32_to_f16(w));", "double w16 = (double)w;"),
    ("gemv weight rounded to fp16 first", "acc += f16_bits_to_double(x[(int64_t)b * K + k]) * (double)w;",
     "acc += f16_bits_to_double(x[(int64_t)b * K + k]) * f16_bits_to_double(nf4o_f32_to_f16(w));"),
    ("codebook form ignores its table", "float level = table[code_of(packed, i)];\n        float scale = absmax[i / blocksize];",
     "float level = NF4_LEVEL[code_of(packed, i)];\n        float scale = absmax[i / blocksize];"),
    ("codebook double-quant form uses groups of 256", "float prod = code2[absmax_q8[b]] * scale2[b / group];",
     "float prod = code2[absmax_q8[b]] * scale2[b / 256];"),
    ("codebook quantiser ties go to the upper code", "float d = fabsf(xn - table[k]);\n        if (d < best_d) { best_d = d; best = k; }",
     "float d = fabsf(xn - table[k]);\n        if (d <= best_d) { best_d = d; best = k; }"),
    ("codebook quantiser zero code fixed at 7", "unsigned zero_code = nearest_code(table, 0.0f);", "unsigned zero_code = 7;"),
    ("group encoder strides by 256", "int64_t lo = g * group;", "int64_t lo = g * 256;"),
    ("codebook gemv ignores its table", "float w = table[code_of(packed, i)] * scale;", "float w = NF4_LEVEL[code_of(packed, i)] * scale;"),
    ("codebook gemv uses groups of 256", "float prod = code2[absmax_q8[blk]] * scale2[blk / group];",
     "float prod = code2[absmax_q8[blk]] * scale2[blk / 256];"),
    ("codebook gemv always rounds its weights", "double wd = round_weights_to_fp16 ? f16_bits_to_double(nf4o_f32_to_f16(w)) : (double)w;",
     "double wd = f16_bits_to_double(nf4o_f32_to_f16(w));"),
    ("codebook gemv indexes blocks by the column alone", "int64_t blk = i / blocksize;", "int64_t blk = k / blocksize;"),
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation target not found: {old!r}"
    mutated = tmp_path / "nf4_oracle_mutated.c"
    mutated.write_text(text.replace(old, new, 1))
    lib = tmp_path / "libnf4_oracle_mutated.so"
    subprocess.run(["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fPIC", "-shared", "-o", str(lib), str(mutated),
                    "-lm"], check=True)
    env = dict(os.environ, NF4_ORACLE_LIB=str(lib))
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                         cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode != 0, f"no pin noticed: {name}"
    assert re.search(r"\d+ failed", res.stdout), res.stdout[-2000:]
