"""The pins must notice a plausible mistake anywhere in the oracle: each case plants one (a dropped
term, a wrong sign or index, a transposed operand, an off-by-one in the mask) in a COPY of the C
source, builds it, and runs the pin tests against that build in a subprocess; they have to fail."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "pevlm_oracle.c")

MUTATIONS = [
    ("rope_sign", "o[i] = x0 * c - x1 * sn;", "o[i] = x0 * c + x1 * sn;"),
    ("rope_pairing", "x1 = widen(x, dtype, in0 + i + half);", "x1 = widen(x, dtype, in0 + ((i + 1) % half) + half);"),
    ("rope_freq_exponent", "pow(rope_base, -2.0 * (double)i / (double)D)", "pow(rope_base, -1.0 * (double)i / (double)D)"),
    ("rope_rebased_positions", "pos[t] = (int32_t)(t - lay->cu_seqlens[s]) + (pos_offset ? pos_offset[s] : 0);",
     "pos[t] = (int32_t)((t - lay->cu_seqlens[s]) % 7) + (pos_offset ? pos_offset[s] : 0);"),
    ("mask_not_causal", "if (j > i) return 0;                    /* causal */", "if (j > i + 1) return 0;"),
    ("mask_previous_blocks", "return ((i - S) / B) == ((j - S) / B);  /* context row, context key: same block only */",
     "return ((i - S) / B) >= ((j - S) / B);"),
    ("mask_sink_hidden", "if (j < S) return 1;                    /* context row, sink key */", "if (j < S) return j + 1 < S;"),
    ("scale_dropped", "dot / sqrt((double)D)", "dot"),
    ("kv_head_transposed", "int32_t g = kv_head_of_q ? kv_head_of_q[h] : h / (Hq / Hkv);", "int32_t g = kv_head_of_q ? kv_head_of_q[h] : h % Hkv;"),
    ("softmax_not_normalised", "for (int32_t d = 0; d < D; ++d) o[d] /= l;", "for (int32_t d = 0; d < D; ++d) o[d] /= (l + 1e-3);"),
    ("value_index", "int64_t v0 = (j * Hkv + g) * (int64_t)D;", "int64_t v0 = (j * Hkv + (Hkv - 1 - g)) * (int64_t)D;"),
    ("lse_dropped_log", "lse[r * Hq + h] = m + log(l);", "lse[r * Hq + h] = m;"),
    ("window_keeps_oldest_instead_of_newest", "if ((j - S) / B < first_kept) vis[base + j] = 0;",
     "if ((j - S) / B >= lay->window_blocks[s]) vis[base + j] = 0;"),
    ("window_off_by_one_block", "int64_t first_kept = n_blocks - lay->window_blocks[s];",
     "int64_t first_kept = n_blocks - lay->window_blocks[s] - 1;"),
    ("window_applied_to_context_rows", "lay->window_blocks[s] >= 0 && t - base >= S + C) {", "lay->window_blocks[s] >= 0 && t - base >= S) {"),
    ("mrope_section_boundary", "int axis = i < section[0] ? 0 :", "int axis = i <= section[0] ? 0 :"),
    ("mrope_axes_swapped", "(i < section[0] + section[1] ? 1 : 2);", "(i < section[0] + section[1] ? 2 : 1);"),
    ("mrope_sign", "o[i] = lo * ca - hi * sa;", "o[i] = lo * ca + hi * sa;"),
    ("position_offset_dropped", "pos[t] = (int32_t)(t - lay->cu_seqlens[s]) + (pos_offset ? pos_offset[s] : 0);",
     "pos[t] = (int32_t)(t - lay->cu_seqlens[s]);"),
    ("position_offset_of_sequence_0_for_all", "pos[t] = (int32_t)(t - lay->cu_seqlens[s]) + (pos_offset ? pos_offset[s] : 0);",
     "pos[t] = (int32_t)(t - lay->cu_seqlens[s]) + (pos_offset ? pos_offset[0] : 0);"),
    ("custom_scale_doubled", "softmax_scale > 0.0 ? dot * softmax_scale :", "softmax_scale > 0.0 ? dot * softmax_scale * 2.0 :"),
    ("custom_scale_ignored", "softmax_scale > 0.0 ? dot * softmax_scale :", "softmax_scale > 1e300 ? dot * softmax_scale :"),
    ("mrope_frequency_restarts_per_section", "double angle = p_axis * pow(rope_base, -(2.0 * i) / D);",
     "double angle = p_axis * pow(rope_base, -(2.0 * (i - (axis == 0 ? 0 : axis == 1 ? section[0] : section[0] + section[1]))) / D);"),
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation anchor for {name} not found exactly once"
    mutated = tmp_path / "oracle_mut.c"
    mutated.write_text(src.replace(old, new))
    lib = tmp_path / "liboracle_mut.so"
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-o", str(lib), str(mutated), "-lm"])
    env = dict(os.environ, PEVLM_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], env=env, cwd=ROOT, capture_output=True, text=True)
    assert r.returncode != 0, f"no pin noticed the planted mistake '{name}'"
    assert "failed" in r.stdout
