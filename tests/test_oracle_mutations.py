"""Mutation check of the oracle's CPU pins.

Each entry below is ONE plausible mistake (a dropped term, a wrong sign or index, a transposed
operand, a swapped matrix) planted into a scratch copy of oracle/moe_oracle.c.  The pins of
tests/test_oracle_pins.py are then run against that copy and must fail: a mistake that the pins
let through would make every parity claim of the GPU tests rest on the kernels agreeing with a
wrong reference.  Nothing here touches the GPU or the working tree.
"""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MUTATIONS = [
    # router (Sec. 2: softmax over all experts, top-k, optional renormalisation over the selected k)
    ("router: gate matrix read transposed",
     "const uint16_t* wr = wg + (size_t)h * E;\n                for (int e = 0; e < E; ++e) acc[e] += xv * (double)bf16_to_f32(wr[e]);",
     "for (int e = 0; e < E; ++e) acc[e] += xv * (double)bf16_to_f32(wg[(size_t)e * H + h]);"),
    ("router: bias dropped", "acc[e] = bias ? (double)bias[e] : 0.0;", "acc[e] = 0.0;"),
    ("router: softmax not normalised over all experts",
     "for (int e = 0; e < E; ++e) p[e] = (float)((double)p[e] / Z);", "for (int e = 0; e < E; ++e) p[e] = (float)((double)p[e]);"),
    ("router: ties go to the higher expert id",
     "if (!taken[e] && (best < 0 || lg[e] > lg[best])) best = e;", "if (!taken[e] && (best < 0 || lg[e] >= lg[best])) best = e;"),
    ("router: renormalisation skipped", "if (renormalize) v = (float)((double)v / wsum);", "if (0) v = (float)((double)v / wsum);"),
    ("router: renormalisation always on", "if (renormalize) v = (float)((double)v / wsum);", "if (1) v = (float)((double)v / wsum);"),
    ("router: routed_scale dropped", "w[(size_t)n * k + j] = v * routed_scale;", "w[(size_t)n * k + j] = v;"),
    ("router: logits off by 1e-3 relative", "lg[e] = (float)acc[e];", "lg[e] = (float)(acc[e] * (1.0 + 1e-3));"),
    # permutation (canonical order: expert id, then token id)
    ("permute: tokens descending inside an expert",
     "for (int t = 0; t < T; ++t)\n        for (int j = 0; j < k; ++j) {\n            const int e = idx[(size_t)t * k + j];\n            const int32_t r",
     "for (int t = T - 1; t >= 0; --t)\n        for (int j = 0; j < k; ++j) {\n            const int e = idx[(size_t)t * k + j];\n            const int32_t r"),
    ("permute: perm loses the rank", "perm[r] = t * k + j;", "perm[r] = t * k;"),
    ("permute: inv_perm written at the mirrored rank", "inv_perm[(size_t)t * k + j] = r;", "inv_perm[(size_t)t * k + (k - 1 - j)] = r;"),
    ("permute: offsets[0] is not zero", "offsets[e + 1] = (int32_t)cursor[e + 1]; }", "offsets[e + 1] = (int32_t)cursor[e + 1]; } offsets[0] = (int32_t)cursor[1];"),
    # SwiGLU expert
    ("expert: SiLU applied to the up projection", "a[f] = (gf / (1.0f + expf(-gf))) * uf;", "a[f] = (uf / (1.0f + expf(-uf))) * gf;"),
    ("expert: sign inside the sigmoid", "a[f] = (gf / (1.0f + expf(-gf))) * uf;", "a[f] = (gf / (1.0f + expf(gf))) * uf;"),
    ("expert: W1 and W3 swapped",
     "g[f] += xv * (double)bf16_to_f32(r1[f]);\n            u[f] += xv * (double)bf16_to_f32(r3[f]);",
     "g[f] += xv * (double)bf16_to_f32(r3[f]);\n            u[f] += xv * (double)bf16_to_f32(r1[f]);"),
    ("expert: W2 read transposed",
     "const uint16_t* r2 = w2 + (size_t)f * H;\n        for (int h = 0; h < H; ++h) y64[h] += av * (double)bf16_to_f32(r2[h]);",
     "for (int h = 0; h < H; ++h) y64[h] += av * (double)bf16_to_f32(w2[(size_t)h * F + f]);"),
    ("expert_rows: every row through expert 0", "const int e = eid[n];", "const int e = 0; (void)eid;"),
    # layer and combine (weighted sum of the k experts' outputs plus the shared experts)
    ("layer: weight of rank 0 for every rank", "const float wj = w[(size_t)n * k + j];\n                expert_row(", "const float wj = w[(size_t)n * k];\n                expert_row("),
    ("layer: shared experts dropped", "for (int s = 0; s < num_shared; ++s) {\n                expert_row(xr, w1[E + s]", "for (int s = 0; s < 0; ++s) {\n                expert_row(xr, w1[E + s]"),
    ("layer: shared expert scaled by a routing weight", "for (int h = 0; h < H; ++h) o[h] += y[h];", "for (int h = 0; h < H; ++h) o[h] += w[(size_t)n * k + k - 1] * y[h];"),
    ("layer: every shared expert uses the first one's weights",
     "expert_row(xr, w1[E + s], w3[E + s], w2[E + s], H, F, g, g + F, g + 2 * F, a, y);\n                for (int h = 0; h < H; ++h) o[h] += y[h];",
     "expert_row(xr, w1[E], w3[E], w2[E], H, F, g, g + F, g + 2 * F, a, y);\n                for (int h = 0; h < H; ++h) o[h] += y[h];"),
    ("combine: shared output dropped",
     "if (y_shared)\n            for (int h = 0; h < H; ++h) o[h] += y_at(y_shared, y_is_f32, (size_t)t * H + h);",
     "if (0)\n            for (int h = 0; h < H; ++h) o[h] += y_at(y_shared, y_is_f32, (size_t)t * H + h);"),
    ("combine: weight of rank 0 for every rank",
     "const float wj = w[(size_t)t * k + j];\n            for (int h = 0; h < H; ++h) o[h] += wj * y_at(",
     "const float wj = w[(size_t)t * k];\n            for (int h = 0; h < H; ++h) o[h] += wj * y_at("),
    ("combine: fp32 input read one element off", "return y_is_f32 ? ((const float*)y)[i]", "return y_is_f32 ? ((const float*)y)[i ^ 1]"),
    ("combine: bf16 input read one element off", ": bf16_to_f32(((const uint16_t*)y)[i]);", ": bf16_to_f32(((const uint16_t*)y)[i ^ 1]);"),
]


def _scratch_copy(dst: str, source_text: str) -> None:
    for d in ("oracle", "workloads"):
        shutil.copytree(os.path.join(ROOT, d), os.path.join(dst, d),
                        ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    os.makedirs(os.path.join(dst, "tests"))
    for f in ("conftest.py", "test_oracle_pins.py"):
        shutil.copy(os.path.join(ROOT, "tests", f), os.path.join(dst, "tests", f))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(dst, "tests", "golden"))
    with open(os.path.join(dst, "oracle", "moe_oracle.c"), "w") as f:
        f.write(source_text)


def _run_pins(dst: str):
    env = dict(os.environ, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-m", "not gpu",
                        "-p", "no:cacheprovider", "--no-header"], cwd=dst, capture_output=True, text=True, env=env)
    return r.returncode, r.stdout + r.stderr


def test_pins_pass_on_an_unchanged_copy(tmp_path):
    """Control: the scratch-copy harness itself runs the pins green."""
    src = open(os.path.join(ROOT, "oracle", "moe_oracle.c")).read()
    _scratch_copy(str(tmp_path / "repo"), src)
    rc, out = _run_pins(str(tmp_path / "repo"))
    assert rc == 0, out[-2000:]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    src = open(os.path.join(ROOT, "oracle", "moe_oracle.c")).read()
    missing = [name for name, old, _ in MUTATIONS if src.count(old) != 1]
    assert not missing, "mutation patterns no longer match the oracle's source: %s" % missing

    def one(i):
        name, old, new = MUTATIONS[i]
        dst = str(tmp_path / ("m%02d" % i))
        _scratch_copy(dst, src.replace(old, new))
        rc, out = _run_pins(dst)
        failed_in_a_test = rc != 0 and "FAILED tests/test_oracle_pins.py::" in out and "rror while" not in out
        return name, failed_in_a_test, out[-600:]

    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(one, range(len(MUTATIONS))))
    survivors = [(n, o) for n, ok, o in results if not ok]
    assert not survivors, "pins let these mistakes through (or the copy did not build): %s" % survivors
