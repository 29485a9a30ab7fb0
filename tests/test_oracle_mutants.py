"""Do the pins bite?  Each case plants ONE plausible mistake (a dropped term, a wrong sign or index, a
scale in the wrong place) in a COPY of the C oracle, on the CPU, and runs the pin tests of that
function against the copy: at least one pin has to fail.  The untouched copy has to pass, so a
kill is the mutation's doing and not the harness's.  Nothing here touches the GPU or the HIP path."""
import os
import shutil
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)

# (name, text in oracle/ape_oracle.c, replacement, pin file)
MUTANTS = [
    # main equation, weights form (Section 4.4)
    ("scaling factor dropped from the context partition sum",
     "const double ctx_log = (M > 0) ? S * L_C : -INFINITY;", "const double ctx_log = (M > 0) ? L_C : -INFINITY;", "test_oracle_pins.py"),
    ("temperature multiplies instead of divides",
     "sC[t] = dot_fd(qv, k_ctx + t * kv_stride + (long)hk * d, d) * inv_sqrt_d / T;",
     "sC[t] = dot_fd(qv, k_ctx + t * kv_stride + (long)hk * d, d) * inv_sqrt_d * T;", "test_oracle_pins.py"),
    ("temperature also on the prefix scores",
     "sP[j] = dot_fd(qv, k_prefix + j * kv_stride + (long)hk * d, d) * inv_sqrt_d;",
     "sP[j] = dot_fd(qv, k_prefix + j * kv_stride + (long)hk * d, d) * inv_sqrt_d / T;", "test_oracle_pins.py"),
    ("causal limit of the own tokens off by one",
     "const long n_self = (long)self_len - q_len + r + 1;      /* causal */", "const long n_self = (long)self_len - q_len + r;", "test_oracle_pins.py"),
    ("context weights lose the S - 1 exponent",
     "const double w = exp(sC[t] - L_C) * exp(ctx_log - g) / D;", "const double w = exp(sC[t] - g) / D;", "test_oracle_pins.py"),
    ("denominator takes the unscaled context sum",
     "if (M > 0) D += exp(ctx_log - g);", "if (M > 0) D += exp(L_C - g);", "test_oracle_pins.py"),
    # block form (Appendix C)
    ("block form: scaling factor dropped", "A[b] = S * L;", "A[b] = L;", "test_oracle_pins.py"),
    ("block form: temperature dropped",
     "x[t - t0] = dot_fd(qv, k_ctx + t * kv_stride + (long)hk * d, d) * inv_sqrt_d / T;",
     "x[t - t0] = dot_fd(qv, k_ctx + t * kv_stride + (long)hk * d, d) * inv_sqrt_d;", "test_oracle_pins.py"),
    # encode (Section 2.2 / 4.1)
    ("encode: context of a row found with the wrong comparison",
     "while (i + 1 < n_chunks && cu_chunk_lens[i + 1] <= r) ++i;", "while (i + 1 < n_chunks && cu_chunk_lens[i + 1] < r) ++i;", "test_oracle_pins.py"),
    ("encode: a row does not see itself",
     "const long n_own = r - c0 + 1;               /* causal inside the context */", "const long n_own = r - c0;", "test_oracle_pins.py"),
    # tree (Appendix C.2 per node, C.5)
    ("tree: a node's scaling factor dropped", "return tq->node_scale[n] * L;", "return L;", "test_oracle_tree_pins.py"),
    ("tree: children weighted against the scaled LogSumExp",
     "const double w = exp(A[i] - L);\n            for (int c = 0; c < d; ++c) vh[c] += w * V[(long)i * d + c];",
     "const double w = exp(A[i] - tq->node_scale[n] * L);\n            for (int c = 0; c < d; ++c) vh[c] += w * V[(long)i * d + c];", "test_oracle_tree_pins.py"),
    ("tree: temperature dropped from the context scores",
     "tq.kv_stride = kv_stride; tq.score_scale = inv_sqrt_d / T;", "tq.kv_stride = kv_stride; tq.score_scale = inv_sqrt_d;", "test_oracle_tree_pins.py"),
    ("tree: root and prefix+self block swapped in the final weights",
     "o[c] = w_root * v_root[c] + w_other * v_other[c];", "o[c] = w_other * v_root[c] + w_root * v_other[c];", "test_oracle_tree_pins.py"),
    # rotary embedding
    ("rope: rotation turns the other way", "yr[c + half] = x2 * cs + x1 * sn;", "yr[c + half] = x2 * cs - x1 * sn;", "test_oracle_rope_pins.py"),
    ("rope: frequency exponent without the factor two",
     "const double a = pos * pow(base, -2.0 * (double)c / (double)d);", "const double a = pos * pow(base, -1.0 * (double)c / (double)d);", "test_oracle_rope_pins.py"),
    ("rope: positions do not restart in every context",
     "const double pos = (double)(position_offset + (t - cu_chunk_lens[i]));", "const double pos = (double)(position_offset + t);", "test_oracle_rope_pins.py"),
]
# the layer around the attention (numpy): (name, text in oracle/layer_oracle.py, replacement)
LAYER_MUTANTS = [
    ("layer: epsilon outside the root", "x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)", "x / (np.sqrt(np.mean(x * x, axis=-1, keepdims=True)) + eps)"),
    ("layer: first residual dropped", "x1 = x[sel] + a @ f(w[\"wo\"]).T", "x1 = a @ f(w[\"wo\"]).T"),
    ("layer: second residual dropped", "y = x1 + (silu(g) * u) @ f(w[\"wd\"]).T", "y = (silu(g) * u) @ f(w[\"wd\"]).T"),
    ("layer: activation on the wrong branch", "(silu(g) * u)", "(g * silu(u))"),
    ("layer: the MLP reads the un-normalised stream", "g, u = h2 @ f(w[\"wg\"]).T, h2 @ f(w[\"wu\"]).T", "g, u = x1 @ f(w[\"wg\"]).T, x1 @ f(w[\"wu\"]).T"),
    ("layer: keys are not rotated", "    k = rope_f64(k, chunk_lens, lp, rope_base)\n", ""),
    ("layer: positions start at zero instead of behind the prefix", "q = rope_f64(q, chunk_lens, lp, rope_base)", "q = rope_f64(q, chunk_lens, 0, rope_base)"),
]
# every query head reads its KV head: planted in all four functions at once
GQA = ("wrong map from query heads to KV heads", "const int hk = h / G;", "const int hk = h % n_kv_heads;", "test_oracle_pins.py")


def _copy_tree(tmp_path, old=None, new=None, every=False, target="ape_oracle.c"):
    root = tmp_path / "copy"
    (root / "oracle").mkdir(parents=True)
    (root / "tests").mkdir()
    for name in os.listdir(os.path.join(ROOT, "oracle")):
        if name.endswith((".py", ".c")):
            shutil.copy(os.path.join(ROOT, "oracle", name), root / "oracle" / name)
    for name in ("conftest.py", "test_oracle_pins.py", "test_oracle_tree_pins.py", "test_oracle_rope_pins.py", "test_oracle_layer_pins.py"):
        shutil.copy(os.path.join(HERE, name), root / "tests" / name)
    shutil.copytree(os.path.join(HERE, "golden"), root / "tests" / "golden")
    if old is not None:
        path = root / "oracle" / target
        src = path.read_text()
        assert src.count(old) >= 1 if every else src.count(old) == 1, "mutation site not found exactly once: %r" % old
        path.write_text(src.replace(old, new))
    return root


def _run_pins(root, pin_file):
    env = dict(os.environ)
    env["PYTHONPATH"] = ROOT + os.pathsep + env.get("PYTHONPATH", "")     # the input generator; `oracle` resolves to the copy (conftest puts it first)
    env["OMP_NUM_THREADS"] = "4"
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", os.path.join(str(root), "tests", pin_file)],
                          cwd=str(root), env=env, capture_output=True, text=True, timeout=900)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_the_untouched_copy_passes_every_pin(tmp_path):
    root = _copy_tree(tmp_path)
    for pin_file in ("test_oracle_pins.py", "test_oracle_tree_pins.py", "test_oracle_rope_pins.py", "test_oracle_layer_pins.py"):
        run = _run_pins(root, pin_file)
        assert run.returncode == 0, (pin_file, run.stdout[-3000:], run.stderr[-2000:])
        assert str(root) in run.stdout or "passed" in run.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
@pytest.mark.parametrize("name, old, new, pin_file", MUTANTS + [GQA], ids=[m[0] for m in MUTANTS + [GQA]])
def test_a_planted_mistake_fails_a_pin(tmp_path, name, old, new, pin_file):
    root = _copy_tree(tmp_path, old, new, every=(old == GQA[1]))
    run = _run_pins(root, pin_file)
    assert run.returncode == 1, "the pins did not notice: %s\n%s\n%s" % (name, run.stdout[-3000:], run.stderr[-2000:])
    assert "failed" in run.stdout and "error" not in run.stdout.splitlines()[-1], run.stdout[-2000:]      # a pin failed; nothing broke on the way


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
@pytest.mark.parametrize("name, old, new", LAYER_MUTANTS, ids=[m[0] for m in LAYER_MUTANTS])
def test_a_planted_mistake_in_the_layer_fails_a_pin(tmp_path, name, old, new):
    root = _copy_tree(tmp_path, old, new, target="layer_oracle.py")
    run = _run_pins(root, "test_oracle_layer_pins.py")
    assert run.returncode == 1, "the pins did not notice: %s\n%s\n%s" % (name, run.stdout[-3000:], run.stderr[-2000:])
    assert "failed" in run.stdout and "error" not in run.stdout.splitlines()[-1], run.stdout[-2000:]
