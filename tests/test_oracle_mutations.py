"""Are the oracle's pins strong enough?  Each case plants one plausible mistake in a COPY of oracle/pod_oracle.c
(a wrong window edge, the wrong layer's key or query, a wrong head mapping, a dropped demotion ...), builds it
and runs the pin tests against it in a child process: they must fail.  CPU only; the GPU path is not involved."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "pod_oracle.c")

# (name, text in the source, replacement); every text must occur exactly `count` times
MUTATIONS = [
    ("window edge one too wide", "return (j < S) || (j > i - W);", "return (j < S) || (j >= i - W);", 1),
    ("sink edge one too wide", "return (j < S) || (j > i - W);", "return (j <= S) || (j > i - W);", 1),
    ("distant logit from the layer's own key", "a[j] = scale * dot_bf16(qsi, k_shared + off, d);", "a[j] = scale * dot_bf16(qsi, k + off, d);", 1),
    ("distant logit from the layer's own query", "a[j] = scale * dot_bf16(qsi, k_shared + off, d);", "a[j] = scale * dot_bf16(qi, k_shared + off, d);", 1),
    ("proximal logit from the lowest layer's key", "a[j] = scale * dot_bf16(qi, k + off, d);         /* Eq. 3, line 1 */", "a[j] = scale * dot_bf16(qi, k_shared + off, d);", 1),
    ("value from the wrong kv head", "const uint16_t *vj = v + ((size_t)j * Hkv + kv) * d;  /* values: always this layer */", "const uint16_t *vj = v + ((size_t)j * Hkv + (kv + 1) % Hkv) * d;", 1),
    ("ring demotes one token early", "if (s->n_recent == c->W) {", "if (s->n_recent == c->W - 1) {", 1),
    ("demoted key dropped at the lowest layer", "copy_lowest_heads(c, layer, s->distK + (size_t)s->n_dist * re, s->recK, 1);", "(void)0;", 1),
    ("decode: distant logit with the layer's own query", "a[m] = scale * dot_bf16(qs, sa->distK + (size_t)t * re + (size_t)kv * d, d);", "a[m] = scale * dot_bf16(qi, sa->distK + (size_t)t * re + (size_t)kv * d, d);", 1),
    ("decode: recent tokens left out", "for (long t = 0; t < s->n_recent; ++t, ++m) {\n            a[m] = scale * dot_bf16(qi, s->recK", "for (long t = 1; t < s->n_recent; ++t, ++m) {\n            a[m] = scale * dot_bf16(qi, s->recK", 1),
    ("several tokens: the last one is not stored", "for (int t = 0; t < cnt; ++t) {", "for (int t = 0; t + 1 < cnt; ++t) {", 1),
    ("chunk: proximal test at the chunk's first position", "if (is_proximal(j, i, c->S, c->W)) {\n                key = j < p0", "if (is_proximal(j, p0, c->S, c->W)) {\n                key = j < p0", 1),
    ("chunk: value of a stored position from the chunk rows", "const uint16_t *vj = j < p0 ? stored_value(c, s, j, kv) : v + ((size_t)(j - p0) * Hkv + kv) * d;", "const uint16_t *vj = j < p0 - 1 ? stored_value(c, s, j, kv) : v + ((size_t)(j < p0 ? 0 : j - p0) * Hkv + kv) * d;", 1),
    ("gate: the lowest layer skips too", "const int skip = nD > 0 && layer != lowest_layer && g >= tau;", "const int skip = nD > 0 && g >= tau;", 1),
]


def _build(text, out):
    src = out[:-3] + ".c"
    with open(src, "w") as f:
        f.write(text)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", src, "-o", out, "-lm"], check=True)


def _pins_pass(lib):
    env = dict(os.environ, POD_ORACLE_LIB=lib)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")], cwd=ROOT, env=env, capture_output=True, text=True)
    return r.returncode == 0, r.stdout[-600:]


def test_an_unchanged_copy_passes_the_pins(tmp_path):
    lib = str(tmp_path / "same.so")
    _build(open(SRC).read(), lib)
    ok, tail = _pins_pass(lib)
    assert ok, tail


@pytest.mark.parametrize("name,old,new,count", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_the_pins(tmp_path, name, old, new, count):
    text = open(SRC).read()
    assert text.count(old) == count, f"the oracle's source no longer holds the line this case changes: {old!r}"
    lib = str(tmp_path / "mutant.so")
    _build(text.replace(old, new), lib)
    ok, tail = _pins_pass(lib)
    assert not ok, f"the pins did not notice: {name}"


# ---- the token-selection oracle (oracle/pod_select.py): the same question for its pins ----
SELECT_SRC = os.path.join(ROOT, "oracle", "pod_select.py")
SELECT_PINS = os.path.join(ROOT, "tests", "test_oracle_select_pins.py")

SELECT_MUTATIONS = [
    ("a query sees one key too few", "logits = scale * (kf[:pos + 1, h, :] @ qf[i, hq, :])", "logits = scale * (kf[:pos, h, :] @ qf[i, hq, :])", 1),
    ("the window starts one position late", "pos = n - obs + i ", "pos = n - obs + i + 1 if i + 1 < obs else n - 1 ", 1),
    ("votes of a query head go to the wrong kv head", "h = hq // rep", "h = hq % Hkv", 1),
    ("the distant range starts one token early", "votes[h] += w[S:n - W]", "votes[h] += np.concatenate([w[S - 1:S], w[S:n - W - 1]]) if S else w[S:n - W]", 1),
    ("weights not normalised", "w /= w.sum()", "w /= w.max()", 1),
    ("pooling window off centre", "lo, hi = max(0, t - r), min(m, t + r + 1)", "lo, hi = max(0, t - r + 1), min(m, t + r + 2)", 1),
    ("mean over the positions that exist", "out[h, t] = acc / votes.dtype.type(width)", "out[h, t] = acc / votes.dtype.type(hi - lo)", 1),
    ("of equal votes the later token wins", "key=lambda t: (-pooled[h, t], t)", "key=lambda t: (-pooled[h, t], -t)", 1),
    ("selection left in vote order", "sel[h] = sorted(order[:keep])", "sel[h] = order[:keep]", 1),
    ("selected index taken as a position", "[S + int(t) for t in sel_of_head[h]]", "[int(t) for t in sel_of_head[h]]", 1),
    ("recent window one token short", "list(range(n - W, n))", "list(range(n - W + 1, n)) + [n - 1]", 1),
]

_DRIVER = """
import importlib.util, sys
sys.path.insert(0, {root!r})
import oracle
spec = importlib.util.spec_from_file_location("oracle.pod_select", {mutant!r})
mod = importlib.util.module_from_spec(spec)
sys.modules["oracle.pod_select"] = mod
spec.loader.exec_module(mod)
oracle.pod_select = mod
import pytest
sys.exit(pytest.main(["-x", "-q", "-p", "no:cacheprovider", {pins!r}]))
"""


def _select_pins_pass(path):
    r = subprocess.run([sys.executable, "-c", _DRIVER.format(root=ROOT, mutant=path, pins=SELECT_PINS)], cwd=ROOT,
                       capture_output=True, text=True)
    return r.returncode == 0, r.stdout[-600:]


def test_an_unchanged_copy_of_the_selection_oracle_passes_its_pins(tmp_path):
    path = str(tmp_path / "same_select.py")
    open(path, "w").write(open(SELECT_SRC).read())
    ok, tail = _select_pins_pass(path)
    assert ok, tail


@pytest.mark.parametrize("name,old,new,count", SELECT_MUTATIONS, ids=[m[0] for m in SELECT_MUTATIONS])
def test_a_planted_mistake_fails_the_selection_pins(tmp_path, name, old, new, count):
    text = open(SELECT_SRC).read()
    assert text.count(old) == count, f"the oracle's source no longer holds the line this case changes: {old!r}"
    path = str(tmp_path / "mutant_select.py")
    open(path, "w").write(text.replace(old, new))
    ok, tail = _select_pins_pass(path)
    assert not ok, f"the pins did not notice: {name}"
