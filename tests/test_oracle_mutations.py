"""Are the oracle's pins sharp?  (CPU only.)

Each case plants one plausible mistake in a COPY of the oracle's C source (a wrong sign, a
swapped operand, an off-by-one index or comparison, a dropped factor), builds it, and runs the
pin tests of the function concerned against the mutated build: at least one pin has to fail.
The real oracle is untouched; nothing here runs on the GPU.
"""
import importlib.util
import os
import subprocess

import pytest

import test_oracle_attention as pins_attention
import test_oracle_greedy as pins_greedy
import test_oracle_kd as pins_kd
import test_oracle_paged as pins_paged
import test_oracle_sampler as pins_sampler
import test_oracle_tree as pins_tree

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "respec_oracle.c")

# (name, text in the source, replacement, module whose pins must catch it)
MUTATIONS = [
    ("attention: causal limit one key short", "L - 1 : L - R + i; /* inclusive */", "L - 1 : L - R + i - 1; /* inclusive */",
     pins_attention),
    ("attention: scale dropped", "score[j] = sm_scale * dot;", "score[j] = dot;", pins_attention),
    ("attention: KV head of a query head", "const int32_t hk = h / G;", "const int32_t hk = h % Hkv;", pins_attention),
    ("attention: weights not normalised by the row sum", "const double a = score[j] / denom;",
     "const double a = score[j];", pins_attention),
    ("attention: V read from the K cache's head", "const int64_t voff = ((kv0 + j) * Hkv + hk) * D;",
     "const int64_t voff = ((kv0 + j) * Hkv + (Hkv - 1 - hk)) * D;", pins_attention),
    ("softmax: temperature multiplies", "p[x] = load_elem(logits, row * ld + x, dtype) / T;",
     "p[x] = load_elem(logits, row * ld + x, dtype) * T;", pins_sampler),
    ("Eq. 1: ratio inverted", "rho = p[x] / q[x];", "rho = q[x] / p[x];", pins_sampler),
    ("Eq. 1: accept on equality", "if (u < thr) { /* Eq. 1: accepted", "if (u <= thr) { /* Eq. 1: accepted", pins_sampler),
    ("Eq. 2: residual sign", "const double w = p[y] - q[y];", "const double w = q[y] - p[y];", pins_sampler),
    ("Eq. 2: residual not clipped at zero", "q[y] = w > 0.0 ? w : 0.0;", "q[y] = w > 0.0 ? w : -w;", pins_sampler),
    ("inverse CDF: non-strict crossing", "if (c > t) {\n            const double lo = fabs(t - before)",
     "if (c >= t) {\n            const double lo = fabs(t - before)", pins_sampler),
    ("bonus token from the wrong row", "softmax_row(target_logits, row0 + k, ld_t, V, T, dtype, p);\n        final_token",
     "softmax_row(target_logits, row0 + (k > 0 ? k - 1 : 0), ld_t, V, T, dtype, p);\n        final_token", pins_sampler),
    ("greedy: last maximum instead of the first", "if (z > zbest) {", "if (z >= zbest) {", pins_greedy),
    ("greedy: bonus row", "out_tokens[n] = argmax_row(target_logits, row0 + n, ld_t, V, dtype);",
     "out_tokens[n] = argmax_row(target_logits, row0 + (n > 0 ? n - 1 : 0), ld_t, V, dtype);", pins_greedy),
    ("KD: gradient sign", "grad[(int64_t)r * V + x] = w * (q[x] - p[x]);", "grad[(int64_t)r * V + x] = w * (p[x] - q[x]);",
     pins_kd),
    ("KD: direction of the divergence", "kl += p[x] * (log(p[x]) - log(q[x]));", "kl += q[x] * (log(q[x]) - log(p[x]));",
     pins_kd),
    ("KD: weight dropped from the loss", "row_loss[r] = w * kl;", "row_loss[r] = kl;", pins_kd),
    ("tree: running distribution not renormalised after a rejected sibling",
     "                for (int32_t y = 0; y < V; ++y)\n                    p[y] /= Z;",
     "                for (int32_t y = 0; y < V; ++y)\n                    p[y] /= 1.0;", pins_tree),
    ("tree: mask bit of a new token", "!((tree_mask[q0 + i] >> (j - first_new)) & 1u)",
     "!((tree_mask[q0 + i] >> (j - first_new + 1)) & 1u)", pins_tree),
    ("paged: slot of a token inside its page", "(size_t)pg * page_size + (size_t)(j % page_size)) * tok_bytes;",
     "(size_t)pg * page_size + (size_t)((j + 1) % page_size)) * tok_bytes;", pins_paged),
    ("commit: position an accepted token moves to", "const int64_t from = first_new + r, to = first_new + 1 + j;",
     "const int64_t from = first_new + r, to = first_new + j;", pins_paged),
    ("commit: new length", "kv_len[b] = (int32_t)(first_new + 1 + n);", "kv_len[b] = (int32_t)(first_new + n);", pins_paged),
]


def _mutated_oracle(tmp_path, old, new):
    text = open(SRC).read()
    # the chain sampler comes first in the file: where a line also occurs in the tree sampler,
    # the first occurrence (the chain function's) is the one mutated
    assert text.count(old) >= 1, f"mutation site gone: {old!r}"
    src = tmp_path / "mutated.c"
    src.write_text(text.replace(old, new, 1))
    lib = tmp_path / "libmutated.so"
    subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", str(lib), str(src), "-lm"],
                   check=True, stderr=subprocess.DEVNULL)
    spec = importlib.util.spec_from_file_location("oracle_mutated", os.path.join(ROOT, "oracle", "__init__.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod._SRC, mod._LIB = str(src), str(lib)      # this copy of the wrapper loads the mutated build
    return mod


def _pins(module):
    return [getattr(module, n) for n in sorted(dir(module)) if n.startswith("test_")]


def _call(fn, oracle):
    """Calls one pin with the given oracle; parametrised pins run over all their parameter sets."""
    marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
    names = fn.__code__.co_varnames[:fn.__code__.co_argcount]
    if not marks:
        fn(**({"oracle": oracle} if "oracle" in names else {}))
        return
    import itertools
    axes = []
    for m in marks:
        keys = [k.strip() for k in m.args[0].split(",")]
        axes.append([(keys, v if len(keys) > 1 else (v,)) for v in m.args[1]])
    for combo in itertools.product(*axes):
        kw = {"oracle": oracle} if "oracle" in names else {}
        for keys, vals in combo:
            kw.update(dict(zip(keys, vals)))
        fn(**kw)


@pytest.mark.parametrize("name,old,new,module", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_a_pin(tmp_path, name, old, new, module):
    mutated = _mutated_oracle(tmp_path, old, new)
    caught = []
    for fn in _pins(module):
        try:
            _call(fn, mutated)
        except Exception as e:  # an assertion, or the mutated build reporting an error
            caught.append(f"{fn.__name__}: {type(e).__name__}")
    assert caught, f"no pin of {module.__name__} noticed: {name}"
    print(f"{name}: caught by {len(caught)} pin(s), e.g. {caught[0]}")


def test_the_unmutated_copy_passes_the_same_pins(tmp_path):
    """The harness itself: a copy without a mutation passes every pin it is given."""
    same = _mutated_oracle(tmp_path, "#define BOUNDARY_EPS 1e-6", "#define BOUNDARY_EPS 1e-6 ")
    for module in (pins_greedy, pins_kd):
        for fn in _pins(module):
            _call(fn, same)
