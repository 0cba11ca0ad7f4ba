"""Do the pins pin?  Each case plants one plausible mistake in a copy of the C oracle's source
(a dropped term, a wrong sign or index, a transposed operand, a wrong layout), builds it, and
re-runs the oracle's pin file against it in a child pytest: at least one pin has to fail.
CPU only; every mistake keeps all memory accesses in bounds."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ATTN = os.path.join(ROOT, "oracle", "oracle_attn.c")
COMMIT = os.path.join(ROOT, "oracle", "oracle_commit.c")

# (name, file, text to find, replacement, how many times the text must occur)
ATTN_MUTATIONS = [
    ("scale 1/D instead of 1/sqrt(D)", ATTN, "1.0 / sqrt((double)D)", "1.0 / (double)D", 3),
    ("block-causal comparison strict", ATTN,
     "(d + k) / p->block_size <= (d + j) / p->block_size",
     "(d + k) / p->block_size < (d + j) / p->block_size", 1),
    ("block-causal mask ignores the cached part of the block", ATTN,
     "(d + k) / p->block_size <= (d + j) / p->block_size",
     "k / p->block_size <= j / p->block_size", 1),
    ("explicit positions: comparison strict", ATTN,
     "(pos[k] - s) / p->block_size <= (pos[j] - s) / p->block_size",
     "(pos[k] - s) / p->block_size < (pos[j] - s) / p->block_size", 1),
    ("explicit positions: block index counted from position 0 instead of the block origin", ATTN,
     "(pos[k] - s) / p->block_size <= (pos[j] - s) / p->block_size",
     "pos[k] / p->block_size <= pos[j] / p->block_size", 1),
    ("explicit positions of the first request used for every request", ATTN,
     "q_pos ? q_pos + cu_q[i] : NULL", "q_pos ? q_pos : NULL", 1),
    ("chunk keys gathered in reverse order", ATTN,
     "  for (int k = 0; k < c; ++k) {\n    int64_t t = cu_q[i] + k;",
     "  for (int k = 0; k < c; ++k) {\n    int64_t t = cu_q[i] + (c - 1 - k);", 1),
    ("GQA head map h mod Hkv instead of h div G", ATTN, "const int g = h / G,", "const int g = h % Hkv,", 1),
    ("cached keys read from the next slot of the page", ATTN,
     "    int slot = n % P;\n    for (int d = 0; d < D; ++d) {\n      K[",
     "    int slot = (n + 1) % P;\n    for (int d = 0; d < D; ++d) {\n      K[", 1),
    ("grouped K layout with slot and d-group swapped", ATTN,
     "((int64_t)(d / 8) * p->page_size + slot) * 8 + d % 8",
     "((int64_t)slot * (p->head_dim / 8) + d / 8) * 8 + d % 8", 1),
    ("grouped V layout slot-major instead of d-major", ATTN,
     "return base + (int64_t)d * p->page_size + slot;",
     "return base + (int64_t)slot * p->head_dim + d;", 1),
    ("output not normalised", ATTN, "out[(t * Hq + h) * D + d] = o[d] / l;",
     "out[(t * Hq + h) * D + d] = o[d];", 1),
    ("query-key product with reversed d", ATTN, "acc += q[d] * K[(int64_t)n * D + d];",
     "acc += q[d] * K[(int64_t)n * D + (D - 1 - d)];", 1),
    ("value accumulated without its weight", ATTN, "o[d] += e * V[(int64_t)n * D + d];",
     "o[d] += V[(int64_t)n * D + d];", 1),
    ("masked keys given weight one", ATTN,
     "double e = (s[n - lo] == -INFINITY) ? 0.0 : exp(s[n - lo] - mx);",
     "double e = (s[n - lo] == -INFINITY) ? 1.0 : exp(s[n - lo] - mx);", 1),
    ("merge weights with the wrong sign", ATTN, "double w = exp(m[s] - M);", "double w = exp(M - m[s]);", 1),
    ("merge denominator ignores the weights", ATTN, "z += w * l[s];", "z += l[s];", 1),
    ("append writes K of the mirrored kv head", ATTN,
     "k_pool[k_offset(p, page, g, slot, d)] = k_new[(t * Hkv + g) * D + d];",
     "k_pool[k_offset(p, page, g, slot, d)] = k_new[(t * Hkv + (Hkv - 1 - g)) * D + d];", 1),
    ("append puts V into the K slot order", ATTN,
     "v_pool[v_offset(p, page, g, slot, d)] = v_new[(t * Hkv + g) * D + d];",
     "v_pool[v_offset(p, page, g, (slot + 1) % P, d)] = v_new[(t * Hkv + g) * D + d];", 1),
    ("cached length inside the block taken as zero", ATTN,
     "n_keys = L + c, dblk = L - block_start[i];", "n_keys = L + c, dblk = 0 * block_start[i];", 1),
]
COMMIT_MUTATIONS = [
    ("commit on confidence >= threshold", COMMIT, "conf_out[t] > threshold ? 1 : 0", "conf_out[t] >= threshold ? 1 : 0", 1),
    ("argmax keeps the last maximum", COMMIT, "if (x > mx) { mx = x; arg = v; }", "if (x >= mx) { mx = x; arg = v; }", 1),
    ("confidence without the exponential of the maximum removed", COMMIT,
     "if (x != -INFINITY) z += exp(x - mx);", "if (x != -INFINITY) z += exp(x - mx) + 1e-3;", 1),
    ("NaN logits enter the sum", COMMIT, "return isnan(x) ? -INFINITY : x;", "return x;", 1),
    ("a fully masked row reports a confidence", COMMIT, "conf_out[t] = 0.0;", "conf_out[t] = 1.0;", 1),
    ("progress rule picks the least confident token", COMMIT,
     "if (best < 0 || conf_out[t] > conf_out[best]) best = t;",
     "if (best < 0 || conf_out[t] < conf_out[best]) best = t;", 1),
    ("progress rule does not look at the last token of a request", COMMIT,
     "for (int t = cu_q[i]; t < cu_q[i + 1]; ++t) {", "for (int t = cu_q[i]; t < cu_q[i + 1] - 1; ++t) {", 1),
]


def run_pins_against(tmp_path, file, find, repl, count, pin_file):
    srcs = {ATTN: open(ATTN).read(), COMMIT: open(COMMIT).read()}
    assert srcs[file].count(find) == count, f"mutation site not found exactly {count} time(s)"
    srcs[file] = srcs[file].replace(find, repl)
    paths = []
    for orig, text in srcs.items():
        q = tmp_path / os.path.basename(orig)
        q.write_text(text)
        paths.append(str(q))
    lib = str(tmp_path / "liboracle_mutant.so")
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-w", *paths, "-o", lib, "-lm"],
                   check=True)
    env = dict(os.environ, ORACLE_MUTANT_LIB=lib, OMP_NUM_THREADS="4")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", pin_file), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True)
    return r


@pytest.mark.parametrize("name,file,find,repl,count", ATTN_MUTATIONS, ids=[m[0] for m in ATTN_MUTATIONS])
def test_attention_pins_catch(tmp_path, name, file, find, repl, count):
    r = run_pins_against(tmp_path, file, find, repl, count, "test_oracle_pins.py")
    assert r.returncode == 1, f"no pin noticed: {name}\n{r.stdout[-2000:]}"
    assert " failed" in r.stdout


@pytest.mark.parametrize("name,file,find,repl,count", COMMIT_MUTATIONS, ids=[m[0] for m in COMMIT_MUTATIONS])
def test_commit_pins_catch(tmp_path, name, file, find, repl, count):
    r = run_pins_against(tmp_path, file, find, repl, count, "test_commit_oracle_pins.py")
    assert r.returncode == 1, f"no pin noticed: {name}\n{r.stdout[-2000:]}"
    assert " failed" in r.stdout


def test_unmutated_copy_passes(tmp_path):
    r = run_pins_against(tmp_path, ATTN, "1.0 / sqrt((double)D)", "1.0 / sqrt((double)D)", 3, "test_oracle_pins.py")
    assert r.returncode == 0, r.stdout[-2000:]


# ---------------------------------------------------------------- the two Python oracles

REORG = os.path.join(ROOT, "oracle", "oracle_reorg.py")
SELECTOR = os.path.join(ROOT, "oracle", "oracle_selector.py")

REORG_MUTATIONS = [
    ("chunk takes decoded positions", "if not decoded[i, b]:", "if decoded[i, b]:"),
    ("cached length ignores the decoded positions of the block", "L = int(block_start[i]) + n_dec", "L = int(block_start[i])"),
    ("KV slot = sequence position", "kv_slot.append(L + taken)", "kv_slot.append(int(block_start[i]) + b)"),
    ("position relative to the block", "q_pos.append(int(block_start[i]) + b)", "q_pos.append(b)"),
    ("one position too many", "if taken >= want:", "if taken > want:"),
    ("cu_q inclusive instead of exclusive", "cu_q = [0]", "cu_q = [int(chunk[0])] if chunk else [0]"),
]
SELECTOR_MUTATIONS = [
    ("second hinge at the first boundary", "np.maximum(0.0, x - b1)], axis=1)", "np.maximum(0.0, x - b0)], axis=1)"),
    ("keeps the worst pair of boundaries", "if best is None or sse < best[\"sse\"]:", "if best is None or sse > best[\"sse\"]:"),
    ("intercept dropped", "np.stack([np.ones_like(x), x,", "np.stack([np.zeros_like(x), x,"),
    ("middle regime's intercept without the hinge shift", "beta0=np.array([alpha, alpha - g0 * b0,", "beta0=np.array([alpha, alpha,"),
    ("last regime's slope without the second hinge", "beta1=np.array([beta, beta + g0, beta + g0 + g1])", "beta1=np.array([beta, beta + g0, beta + g0])"),
    ("regime chosen with <= at the first boundary only", "k = 0 if x < model[\"x_break\"][0] else (1 if x < model[\"x_break\"][1] else 2)",
     "k = 0 if x < model[\"x_break\"][1] else (1 if x < model[\"x_break\"][1] else 2)"),
    ("objective without the batch size in the latency", "latency_eval(model, float(batch) * chunk_sizes[i])", "latency_eval(model, float(chunk_sizes[i]))"),
    ("objective = token utilisation only", "n_commit[i] * batch / latency_eval(", "n_commit[i] / chunk_sizes[i] + 0 * latency_eval("),
    ("argmin instead of argmax", "int(np.argmax(rates))", "int(np.argmin(rates))"),
]


def load_mutant(path, find, repl, name):
    import importlib.util
    import types
    src = open(path).read()
    assert src.count(find) == 1, "mutation site not found exactly once"
    mod = types.ModuleType(name)
    exec(compile(src.replace(find, repl), path, "exec"), mod.__dict__)
    return mod


def pins_that_fail(test_module, shim, prefix="test_"):
    failed = []
    for fname in dir(test_module):
        fn = getattr(test_module, fname)
        if not fname.startswith(prefix) or not callable(fn):
            continue
        try:
            fn(shim)
        except AssertionError:
            failed.append(fname)
        except Exception:       # a mutant may also make numpy raise
            failed.append(fname)
    return failed


@pytest.mark.parametrize("name,find,repl", REORG_MUTATIONS, ids=[m[0] for m in REORG_MUTATIONS])
def test_reorg_pins_catch(name, find, repl):
    import types
    from tests import test_reorg_oracle_pins as pins
    mut = load_mutant(REORG, find, repl, "oracle_reorg_mutant")
    assert pins_that_fail(pins, types.SimpleNamespace(reorganise=mut.reorganise)), f"no pin noticed: {name}"


@pytest.mark.parametrize("name,find,repl", SELECTOR_MUTATIONS, ids=[m[0] for m in SELECTOR_MUTATIONS])
def test_selector_pins_catch(name, find, repl):
    import types
    from tests import test_selector as pins
    mut = load_mutant(SELECTOR, find, repl, "oracle_selector_mutant")
    assert pins_that_fail(pins, types.SimpleNamespace(selector=mut), prefix="test_oracle_"), f"no pin noticed: {name}"


def test_unmutated_python_oracles_pass():
    import types
    from tests import test_reorg_oracle_pins, test_selector
    a = load_mutant(REORG, "cu_q = [0]", "cu_q = [0]", "oracle_reorg_copy")
    b = load_mutant(SELECTOR, "int(np.argmax(rates))", "int(np.argmax(rates))", "oracle_selector_copy")
    assert pins_that_fail(test_reorg_oracle_pins, types.SimpleNamespace(reorganise=a.reorganise)) == []
    assert pins_that_fail(test_selector, types.SimpleNamespace(selector=b), prefix="test_oracle_") == []
