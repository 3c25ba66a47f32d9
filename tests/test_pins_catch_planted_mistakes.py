"""Do the pins bite?  Each case plants ONE plausible mistake (a dropped term, a wrong sign or index, a transposed
operand, the other branch's parameter) in a temporary COPY of the oracle's sources, builds that copy with the
oracle's own compiler flags and runs the pin tests against it in a child process: at least one pin must fail.
The unchanged copy must pass.  Everything happens on the CPU; the oracle in the tree is never touched.
"""
import concurrent.futures
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle")
SOURCES = ["mixaq_oracle.c", "uniform_block.c", "downsample.c"]
BLOCK, ARITH, DOWN = "mixaq_oracle.c", "arith.h", "downsample.c"

# (name, file, text as it stands (must occur exactly once), text with the mistake)
MISTAKES = [
    ("zero point correction of a linear layer dropped", BLOCK,
     "acc[t * N + n] = s - z_a * cs;", "acc[t * N + n] = s;"),
    ("query and key swapped in the score product", BLOCK,
     "s += cqkv[i * 3 * C + hh * hd + k] * cqkv[j * 3 * C + C + hh * hd + k];",
     "s += cqkv[j * 3 * C + hh * hd + k] * cqkv[i * 3 * C + C + hh * hd + k];"),
    ("shift rolled the other way", BLOCK,
     "int pr = (wr * ws + tr + d->shift) % Hp;", "int pr = (wr * ws + tr - d->shift + Hp) % Hp;"),
    ("mask: neighbours in one direction suffice", BLOCK,
     "return !(dr < d->window && dc < d->window);", "return !(dr < d->window || dc < d->window);"),
    ("relative position bias transposed", BLOCK,
     "sh->rel_pos_bias[((size_t)hh * T + i) * T + j]", "sh->rel_pos_bias[((size_t)hh * T + j) * T + i]"),
    ("mask added with the wrong sign", BLOCK,
     "bias = bias + MASK_VALUE;", "bias = bias - MASK_VALUE;"),
    ("logits not scaled by 1/sqrt(head dim)", BLOCK,
     "(float)(1.0 / sqrt((double)hd))", "1.0f"),
    ("first residual dropped", BLOCK,
     "hres[t * C + n] = f + xin[t * C + n];", "hres[t * C + n] = f;"),
    ("second residual dropped", BLOCK,
     "float out = f + hres[t * C + n];", "float out = f;"),
    ("second LayerNorm takes the first one's parameters", BLOCK,
     "orc_layernorm(hres + (size_t)t * C, C, br->ln2_gamma, br->ln2_beta, d->ln_eps, ln);",
     "orc_layernorm(hres + (size_t)t * C, C, br->ln1_gamma, br->ln1_beta, d->ln_eps, ln);"),
    ("branches exchanged", BLOCK,
     "process_slot(d, sh, &br[hi ? 0 : 1],", "process_slot(d, sh, &br[hi ? 1 : 0],"),
    ("bit widths of the branches exchanged", BLOCK,
     "hi ? d->act_bits_high : d->act_bits_low, x, b,", "hi ? d->act_bits_low : d->act_bits_high, x, b,"),
    ("selection keeps the lowest scores", BLOCK,
     "int ahead = reverse ? (sv < sw) : (sv > sw);", "int ahead = reverse ? (sv > sw) : (sv < sw);"),
    ("ties go to the higher index", BLOCK,
     "(nv != nw ? nw : v < w)", "(nv != nw ? nw : v > w)"),
    ("keys used in place of values", BLOCK,
     "o += (pc[j] - zp) * cqkv[j * 3 * C + 2 * C + hh * hd + k];", "o += (pc[j] - zp) * cqkv[j * 3 * C + C + hh * hd + k];"),
    ("zero point of the probabilities not removed", BLOCK,
     "o += (pc[j] - zp) * cqkv", "o += pc[j] * cqkv"),
    ("softmax without the row maximum", BLOCK,
     "prob[j] = orc_exp2_pinned(lg[j] - mx);", "prob[j] = orc_exp2_pinned(lg[j]);"),
    ("softmax not normalised", BLOCK,
     "prob[j] = prob[j] * rden;", "prob[j] = prob[j];"),
    ("score is the sum of magnitudes", BLOCK,
     "acc += (double)u[ch] * (double)u[ch];", "acc += fabs((double)u[ch]);"),
    ("scoring LayerNorm skipped", BLOCK,
     "if (d->score_mode == 1) orc_layernorm(px,", "if (0) orc_layernorm(px,"),
    ("score counts the padded area too (reads past the map edge clamped)", BLOCK,
     "if (!orc_token_source(&g, w, t, &r, &c)) continue;",
     "if (!orc_token_source(&g, w, t, &r, &c)) { r = r < d->H ? r : d->H - 1; c = c < d->W ? c : d->W - 1; }"),
    ("score taken on the shifted grid", BLOCK,
     "orc_desc g = *d; g.shift = 0;", "orc_desc g = *d;"),
    ("padded tokens enter as the LayerNorm of zeros", BLOCK,
     "for (int c = 0; c < C; ++c) ln[c] = 0.0f;", "for (int c = 0; c < C; ++c) ln[c] = br->ln1_beta[c];"),
    ("pruned windows not forwarded", BLOCK,
     "memcpy(y + off, x + off, sizeof(float) * d->C);", "(void)off;"),
    ("keep count rounded down", BLOCK,
     "double k = floor(keep_ratio * (double)nW + 0.5);", "double k = floor(keep_ratio * (double)nW);"),
    ("key and value quantizers exchanged", BLOCK,
     "n < C ? &br->a_q : (n < 2 * C ? &br->a_k : &br->a_v);", "n < C ? &br->a_q : (n < 2 * C ? &br->a_v : &br->a_k);"),
    ("projection bias dropped", BLOCK,
     "br->a_proj_in.scale * sh->s_proj[n], br->b_proj[n]);", "br->a_proj_in.scale * sh->s_proj[n], 0.0f);"),
    ("FC1 dequantized with the FC2 input step", BLOCK,
     "br->a_fc1_in.scale * sh->s_fc1[n], br->b_fc1[n]);", "br->a_fc2_in.scale * sh->s_fc1[n], br->b_fc1[n]);"),
    ("attention output scaled by the probability step only", BLOCK,
     "m_o = br->a_p.scale * br->a_v.scale,", "m_o = br->a_p.scale,"),
    ("scatter writes the window in gather order of another token", BLOCK,
     "if (src_ok[t]) y[(((size_t)b * d->H + src_r[t]) * d->W + src_c[t]) * C + n] = out;",
     "if (src_ok[t]) y[(((size_t)b * d->H + src_r[T - 1 - t]) * d->W + src_c[T - 1 - t]) * C + n] = out;"),
    ("quantizer rounds ties away from zero", ARITH,
     "if (fr > 0.5 || (fr == 0.5 && fmod(n, 2.0) != 0.0)) n += 1.0;", "if (fr >= 0.5) n += 1.0;"),
    ("quantizer clamps to a symmetric range", ARITH,
     "const double lo = -(double)(1 << (bits - 1)),", "const double lo = -(double)((1 << (bits - 1)) - 1),"),
    ("LayerNorm with the sample variance", ARITH,
     "float var = (float)(v / (double)C);", "float var = (float)(v / (double)(C - 1));"),
    ("LayerNorm without eps", ARITH,
     "float rstd = 1.0f / sqrtf(var + eps);", "float rstd = 1.0f / sqrtf(var);"),
    ("GELU without its remainder (a ReLU)", ARITH,
     "return fmaxf(x, 0.0f) - h;", "return fmaxf(x, 0.0f);"),
    ("exponential: one polynomial coefficient off by an ulp-scale slip", ARITH,
     "p = fmaf(p, r, 0x1.ebf906p-3f);", "p = fmaf(p, r, 0x1.ebf806p-3f);"),
    ("patch merging: neighbours (1,0) and (0,1) exchanged", DOWN,
     "{{0, 0}, {1, 0}, {0, 1}, {1, 1}}", "{{0, 0}, {0, 1}, {1, 0}, {1, 1}}"),
    ("patch embedding: patch flattened column first", DOWN,
     "v[(di * P + dj) * C + ch] =", "v[(dj * P + di) * C + ch] ="),
    ("layers between stages: zero point correction dropped", DOWN,
     "acc -= (int64_t)z * colsum[n];", ""),
    ("patch merging: LayerNorm skipped", DOWN,
     "if (d->kind == 1) { orc_layernorm(v, K, p->ln_gamma, p->ln_beta, d->ln_eps, u); src = u; }", ""),
    ("patch embedding: LayerNorm after the linear layer skipped", DOWN,
     "if (d->kind == 0) orc_layernorm(f, N, p->ln_gamma, p->ln_beta, d->ln_eps, out + tok * N);\n                else memcpy",
     "memcpy"),
]


def build_copy(dst, mistake=None):
    """Copies the oracle's sources to dst, plants the mistake, builds with the oracle's flags; returns the library."""
    os.makedirs(dst, exist_ok=True)
    for name in SOURCES + ["arith.h"]:
        shutil.copy(os.path.join(ORACLE, name), os.path.join(dst, name))
    if mistake is not None:
        _, fname, old, new = mistake
        path = os.path.join(dst, fname)
        text = open(path).read()
        assert text.count(old) == 1, f"the text to replace must occur exactly once in {fname}: {old!r}"
        open(path, "w").write(text.replace(old, new))
    lib = os.path.join(dst, "liboracle.so")
    cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared", "-w", "-o", lib] + \
          [os.path.join(dst, s) for s in SOURCES] + ["-lm"]
    subprocess.run(cmd, check=True)
    return lib


def run_pins(lib):
    env = dict(os.environ, ORACLE_LIBRARY_UNDER_TEST=lib, OMP_NUM_THREADS="2")
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", os.path.join(ROOT, "tests", "test_oracle_pins.py")]
    r = subprocess.run(cmd, env=env, cwd=ROOT, capture_output=True, text=True, timeout=600)
    return r.returncode, r.stdout[-1500:]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    rc, out = run_pins(build_copy(str(tmp_path / "unchanged")))
    assert rc == 0, "the unchanged copy must pass its pins:\n" + out

    def trial(i):
        lib = build_copy(str(tmp_path / f"m{i}"), MISTAKES[i])
        return run_pins(lib)
    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(trial, range(len(MISTAKES))))
    survivors = [MISTAKES[i][0] for i, (rc, _) in enumerate(results) if rc == 0]
    broken = [(MISTAKES[i][0], out) for i, (rc, out) in enumerate(results) if rc not in (0, 1)]
    assert not broken, f"pin runs that did not end in a test verdict: {broken}"
    assert not survivors, f"mistakes no pin noticed: {survivors}"


@pytest.mark.parametrize("fname", sorted({m[1] for m in MISTAKES}))
def test_the_mistakes_still_apply_to_the_sources(fname):
    text = open(os.path.join(ORACLE, fname)).read()
    for name, f, old, _ in MISTAKES:
        if f == fname:
            assert text.count(old) == 1, name
