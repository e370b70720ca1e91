"""Do the oracle's pins bite? Each case plants one plausible mistake in a copy of the oracle's source (a wrong sign or
index, a dropped term, a swapped operand, an off-by-one) and runs the pin tests of the stage against that copy: at
least one of them has to fail. The oracle module itself is never modified; nothing here touches the GPU path."""
import importlib
import itertools
import os
import sys
import types

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = open(os.path.join(ROOT, "oracle", "audiokv_oracle.py")).read()

# (name, text in the oracle, the planted mistake, pin modules that must catch it)
MUTANTS = [
    ("score: causal mask off by one", "cols[None, :] <= last_visible[:, None]", "cols[None, :] < last_visible[:, None]",
     ["test_oracle_score"]),
    ("score: window row i placed one position early", "last_visible = (L - W) + np.arange(W)",
     "last_visible = (L - W - 1) + np.arange(W)", ["test_oracle_score"]),
    ("score: softmax normalised over the whole window instead of per row", "p = e / e.sum(axis=1, keepdims=True)",
     "p = e / e.sum()", ["test_oracle_score"]),
    ("score: query heads interleaved over KV heads instead of grouped", "qh = q_win[h * G + g]",
     "qh = q_win[g * H_kv + h]", ["test_oracle_score"]),
    ("score: scale 1/d instead of 1/sqrt(d)", "scale = 1.0 / math.sqrt(d)\n    raw = np.zeros", "scale = 1.0 / d\n    raw = np.zeros",
     ["test_oracle_score"]),
    ("score: only the first query head of a group is summed", "        for g in range(G):\n            qh = q_win", "        for g in range(1):\n            qh = q_win",
     ["test_oracle_score"]),
    ("score: mean over the window rows instead of the sum", "raw[h] += p.sum(axis=0)", "raw[h] += p.mean(axis=0)",
     ["test_oracle_score"]),
    ("pool: max pooling padded with zeros", 'pad_val = 0.0 if mode == "avg" else -np.inf', "pad_val = 0.0", ["test_oracle_score"]),
    ("pool: window shifted by one tap", "pad = [(0, 0)] * (x.ndim - 1) + [(half, half)]",
     "pad = [(0, 0)] * (x.ndim - 1) + [(half + 1, half - 1)]", ["test_oracle_score"]),
    ("pool: divisor counts only the taps inside the sequence", "return acc / kernel",
     "return acc / np.minimum(kernel, np.minimum(np.arange(L) + half + 1, L - np.arange(L) + half))", ["test_oracle_score"]),
    ("n_keep: truncation instead of round-half-up", "return int(math.floor(float(ratio) * float(L) + 0.5))",
     "return int(math.floor(float(ratio) * float(L)))", ["test_oracle_allocate"]),
    ("allocate: floor r taken of n_keep instead of n_keep - window", "r = int(math.floor(float(floor_frac) * float(nk - window)))",
     "r = int(math.floor(float(floor_frac) * float(nk)))", ["test_oracle_allocate"]),
    ("allocate: leftover units to the smallest fractional parts", "order = sorted(free, key=lambda h: (-frac[h], h))",
     "order = sorted(free, key=lambda h: (frac[h], h))", ["test_oracle_allocate"]),
    ("allocate: remainder ties to the higher head", "order = sorted(free, key=lambda h: (-frac[h], h))",
     "order = sorted(free, key=lambda h: (-frac[h], -h))", ["test_oracle_allocate"]),
    ("allocate: no cap at L", "over = [h for h in free if x[h] > float(cap)]", "over = []", ["test_oracle_allocate"]),
    ("allocate: capped heads' share is not re-spread", "T = float(B_score - int(capped.sum()) * cap)", "T = float(B_score)",
     ["test_oracle_allocate"]),
    ("allocate: group weights averaged over the wrong axis", "S = S.reshape(-1, group)", "S = S.reshape(group, -1).T",
     ["test_oracle_allocate"]),
    ("allocate: what is shared out forgets the uniform floor", "B_score = n * (nk - f)", "B_score = n * (nk - window)",
     ["test_oracle_allocate"]),
    ("irdft: sign of the exponent", "tw = _twiddle_table(L)\n    n = np.arange(L, dtype=np.int64)\n    g = np.full",
     "tw = np.conj(_twiddle_table(L))\n    n = np.arange(L, dtype=np.int64)\n    g = np.full", ["test_oracle_smooth"]),
    ("rdft: sign of the exponent", "tw = np.conj(_twiddle_table(L))", "tw = _twiddle_table(L)", ["test_oracle_smooth"]),
    ("irdft: positive-frequency bins not doubled", "g = np.full(nb, 2.0)", "g = np.full(nb, 1.0)", ["test_oracle_smooth"]),
    ("irdft: Nyquist bin doubled", "if L % 2 == 0 and nb == L // 2 + 1:\n        g[-1] = 1.0", "if False:\n        g[-1] = 1.0",
     ["test_oracle_smooth"]),
    ("irdft: 1/L forgotten", "return out / float(L)", "return out", ["test_oracle_smooth"]),
    ("cutoff: fraction of L/2 + 1 bins", "return int(math.floor(float(cutoff_frac) * float(L // 2)))",
     "return int(math.floor(float(cutoff_frac) * float(L // 2 + 1)))", ["test_oracle_smooth"]),
    ("mask: bin k* itself dropped", "w = np.where(i <= k_star, 1.0, 0.0)", "w = np.where(i < k_star, 1.0, 0.0)",
     ["test_oracle_smooth"]),
    ("smooth: alpha and 1 - alpha swapped", "return (1.0 - float(alpha)) * s + float(alpha) * s_tilde",
     "return float(alpha) * s + (1.0 - float(alpha)) * s_tilde", ["test_oracle_smooth"]),
    ("energy cutoff: strict inequality", "return int(np.argmax(E >= target))", "return int(np.argmax(E > target))",
     ["test_oracle_smooth"]),
    ("energy cutoff: amplitudes summed instead of energies", "m2 = np.abs(np.asarray(F, dtype=np.complex128)) ** 2",
     "m2 = np.abs(np.asarray(F, dtype=np.complex128))", ["test_oracle_smooth"]),
    ("taper: band divided by T instead of T + 1", "np.cos(np.pi * (i - k_star) / float(T + 1))",
     "np.cos(np.pi * (i - k_star) / float(T))", ["test_oracle_smooth"]),
    ("select: ties to the higher index", "cand.sort(key=lambda j: (-float(s_hat[j]), j))",
     "cand.sort(key=lambda j: (-float(s_hat[j]), -j))", ["test_oracle_select_compact"]),
    ("select: lowest scores kept", "cand.sort(key=lambda j: (-float(s_hat[j]), j))",
     "cand.sort(key=lambda j: (float(s_hat[j]), j))", ["test_oracle_select_compact"]),
    ("select: window positions compete with the prefix", "cand = list(range(n_cand))\n", "cand = list(range(L))\n",
     ["test_oracle_select_compact"]),
    ("select: output not in ascending order", "kept = sorted(cand[:want]) + list(range(n_cand, L))",
     "kept = cand[:want] + list(range(n_cand, L))", ["test_oracle_select_compact"]),
    ("select: forced window dropped", "kept = sorted(cand[:want]) + list(range(n_cand, L))", "kept = sorted(cand[:want])",
     ["test_oracle_select_compact"]),
    ("compact: V rows taken from the wrong head", "vo = [v[h][np.asarray(ix, dtype=np.int64)] for h, ix in enumerate(indices)]",
     "vo = [v[h - 1][np.asarray(ix, dtype=np.int64)] for h, ix in enumerate(indices)]", ["test_oracle_select_compact"]),
    ("decode: values of the wrong KV head", "V = np.asarray(v_rows[j // G], dtype=np.float64)",
     "V = np.asarray(v_rows[j % H_kv], dtype=np.float64)", ["test_oracle_decode"]),
    ("decode: query head j reads KV head j % H_kv", "K = np.asarray(k_rows[j // G], dtype=np.float64)",
     "K = np.asarray(k_rows[j % H_kv], dtype=np.float64)", ["test_oracle_decode"]),
    ("decode: weights not normalised", "out[j] = (e / e.sum()) @ V", "out[j] = e @ V", ["test_oracle_decode"]),
    ("decode: scale 1/d", "scale = 1.0 / math.sqrt(d)\n    out = np.empty", "scale = 1.0 / d\n    out = np.empty",
     ["test_oracle_decode"]),
]


def _mutated_module(old, new):
    assert SRC.count(old) == 1, f"the oracle's source no longer contains exactly one {old!r}"
    mod = types.ModuleType("audiokv_oracle_mutant")
    mod.__dict__["__name__"] = "audiokv_oracle_mutant"
    exec(compile(SRC.replace(old, new), "audiokv_oracle_mutant.py", "exec"), mod.__dict__)
    return mod


def _calls(fn):
    """Argument sets of a (possibly parametrised) test function that takes no fixtures."""
    marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
    if not marks:
        return [{}]
    axes = []
    for m in marks:
        names = [n.strip() for n in m.args[0].split(",")] if isinstance(m.args[0], str) else list(m.args[0])
        rows = []
        for v in m.args[1]:
            v = getattr(v, "values", v)
            rows.append(dict(zip(names, v if len(names) > 1 else [v])))
        axes.append(rows)
    return [dict(kv for d in combo for kv in d.items()) for combo in itertools.product(*axes)]


def _first_failure(pin_module, oracle_module):
    here = os.path.dirname(os.path.abspath(__file__))
    if here not in sys.path:
        sys.path.insert(0, here)
    pins = importlib.import_module(pin_module)
    saved = pins.O
    pins.O = oracle_module
    try:
        for name in sorted(dir(pins)):
            fn = getattr(pins, name)
            if not name.startswith("test_") or not callable(fn):
                continue
            for kwargs in _calls(fn):
                try:
                    fn(**kwargs)
                except pytest.skip.Exception:   # a pin that declares a case out of its scope
                    continue
                except Exception as e:          # an assertion, or the planted mistake tripping an internal check
                    return f"{name}{kwargs or ''}: {type(e).__name__}"
    finally:
        pins.O = saved
    return None


@pytest.mark.parametrize("name,old,new,pin_modules", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, old, new, pin_modules):
    mutant = _mutated_module(old, new)
    caught = [f for f in (_first_failure(pm, mutant) for pm in pin_modules) if f]
    assert caught, f"no pin notices: {name}"


def test_the_unmodified_copy_passes_every_pin():
    """The harness itself: the same copy without a planted mistake goes through all pin modules clean."""
    clean = types.ModuleType("audiokv_oracle_copy")
    exec(compile(SRC, "audiokv_oracle_copy.py", "exec"), clean.__dict__)
    for pm in sorted({p for m in MUTANTS for p in m[3]}):
        assert _first_failure(pm, clean) is None, pm
