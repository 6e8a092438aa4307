"""The oracle's pins have teeth: a mistake planted in the oracle makes at least one pin fail.

Each case rewrites one expression of `oracle/moga_oracle.py` or `oracle/stga_oracle.py` (a dropped
term, a wrong sign, a transposed operand, a wrong index), loads the rewritten source as a module,
substitutes its functions for the real ones and runs the pin tests of `test_oracle_forward.py`,
`test_oracle_backward.py` (or `test_oracle_stga.py`) until one of them fails.  A planted mistake
that no pin notices fails this test, which means a pin is missing.  Everything here runs on the
CPU.
"""
import inspect
import os
import types

import pytest

from oracle import moga_oracle as orc
from oracle import stga_oracle as sto
from tests import test_oracle_backward as pins_bwd
from tests import test_oracle_forward as pins_fwd
from tests import test_oracle_stga as pins_stga

ORACLE_DIR = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle")
ORACLE_SOURCE = os.path.join(ORACLE_DIR, "moga_oracle.py")
STGA_SOURCE = os.path.join(ORACLE_DIR, "stga_oracle.py")

# (what is planted, text in the oracle, replacement).  The text must occur exactly `count` times.
MUTATIONS = [
    ("Eq. 2: sign of the logits", "r = _f64(X) @ _f64(W).T", "r = -(_f64(X) @ _f64(W).T)", 1),
    ("Eq. 4: argmin instead of argmax",
     "group = np.argmax(r32, axis=1).astype(np.int32)", "group = np.argmin(r32, axis=1).astype(np.int32)", 1),
    ("Eq. 3: probabilities not normalised", "probs = e / denom", "probs = e", 1),
    ("Eq. 5: gate inverted", "gate = 1.0 / denom[:, 0]", "gate = denom[:, 0]", 1),
    ("Eq. 1: scale dropped in the forward", "    S = (q @ K.T) * scale\n    m = S.max", "    S = (q @ K.T)\n    m = S.max", 1),
    ("Eq. 1: softmax not normalised", "out = (P / l) @ V", "out = P @ V", 1),
    ("log-sum-exp without the row maximum", "lse = m[:, 0] + np.log(l[:, 0])", "lse = np.log(l[:, 0])", 1),
    ("offsets are not a prefix sum", "cu[g + 1] = cu[g] + counts[g]", "cu[g + 1] = counts[g]", 1),
    ("order inside a group reversed", "perm[cu[g]:cu[g + 1]] = members", "perm[cu[g]:cu[g + 1]] = members[::-1]", 1),
    ("inverse permutation is the permutation", "inv_perm[perm] = np.arange(N, dtype=np.int32)",
     "inv_perm[:] = perm", 1),
    ("max_seqlen is the minimum", "np.int32(counts.max() if", "np.int32(counts.min() if", 1),
    ("Alg. 1 step 4 gathers instead of scattering", "    O[perm] = A\n", "    O[:] = A[perm]\n", 1),
    ("Eq. 5: gate not applied to the output", "O = O * _f64(gate)[:, None, None]", "O = O * 1.0", 1),
    ("attention sees the keys of every group",
     "softmax_attention(Qh[s:e, h], Kh[s:e, h], Vh[s:e, h], scale)",
     "softmax_attention(Qh[s:e, h], Kh[:, h], Vh[:, h], scale)", 1),
    ("dense definition: mask is not an equality", "mask = g[:, None] == g[None, :]", "mask = g[:, None] >= g[None, :]", 1),
    ("dense definition: gate dropped", "O[:, h] = gate[:, None] * (P @ V[:, h])", "O[:, h] = (P @ V[:, h])", 1),
    ("dV uses P instead of P^T", "dV = P.T @ dA", "dV = P @ dA", 1),
    ("dS without the row-sum term", "dS = P * (dP - (dP * P).sum(axis=1, keepdims=True))", "dS = P * dP", 1),
    ("dq without the scale", "dq = scale * (dS @ K)", "dq = dS @ K", 1),
    ("dK with dS not transposed", "dK = scale * (dS.T @ q)", "dK = scale * (dS @ q)", 1),
    ("softmax Jacobian with the wrong sign", "(onehot - probs)", "(onehot + probs)", 1),
    ("dr without the gate factor", "dr = (d_gate * gate)[:, None]", "dr = (d_gate)[:, None]", 1),
    ("d_gate from the sorted-order output", "d_gate = (dO * A_tok).sum(axis=(1, 2))", "d_gate = (dO * A).sum(axis=(1, 2))", 1),
    ("upstream gradient not multiplied by the gate", "dA = (dO * gate[:, None, None])[perm]", "dA = (dO * 1.0)[perm]", 1),
    ("gradients gathered instead of scattered back", "dQ[perm], dK[perm], dV[perm] = dQh, dKh, dVh",
     "dQ[:], dK[:], dV[:] = dQh[perm], dKh[perm], dVh[perm]", 1),
    ("Eq. 8 summed over all tokens", "P[i] = gate[sel].sum() / N", "P[i] = gate.sum() / N", 1),
    ("Eq. 6 without the factor M", "return alpha * M * float((F * P).sum()), F, P", "return alpha * float((F * P).sum()), F, P", 1),
    ("balancing-loss gradient without 1/N", "return alpha * M * F[group] / N", "return alpha * M * F[group]", 1),
]


# Section 3.2 (static groups), same form.
STGA_MUTATIONS = [
    ("tokens column-major inside a frame", "(i // Ww) % Hh, i % Ww", "i % Hh, (i // Hh) % Ww", 1),
    ("temporal runs continue across a shot boundary", "if new_shot or in_run == tg:", "if t == 0 or in_run == tg:", 1),
    ("temporal runs one frame too long", "if new_shot or in_run == tg:", "if new_shot or in_run == tg + 1:", 1),
    ("window height and width swapped", "(y // wh) * nwx + (x // ww)", "(y // ww) * nwx + (x // wh)", 2),
    ("group ids of different runs collide", "run[t] * (nwy * nwx) + win", "run[t] * nwx + win", 1),
    ("first frames of the previous shot added instead of its last", "[-a_prev:]", "[:a_prev]", 1),
    ("last frames of the next shot added instead of its first", "[:a_next]", "[-a_next:]", 1),
    ("added frames not restricted to the group's window", "np.nonzero((t == f) & (win == w))[0]", "np.nonzero(t == f)[0]", 1),
    ("added frames also become queries", "        kv_index.extend(kv)\n", "        kv_index.extend(kv)\n        q_index[len(q_index) - len(own):] = kv\n", 1),
    ("pair count uses n_q squared", "(cu_q[1:] - cu_q[:-1]) * (cu_k[1:] - cu_k[:-1])", "(cu_q[1:] - cu_q[:-1]) * (cu_q[1:] - cu_q[:-1])", 1),
    ("keys and values swapped in the backward", "_mo.softmax_attention_bwd(Q[qi, h], K[ki, h], V[ki, h], dA[qi, h], scale)",
     "_mo.softmax_attention_bwd(Q[qi, h], V[ki, h], K[ki, h], dA[qi, h], scale)", 1),
    ("a key shared by several groups keeps only the last contribution", "np.add.at(dK[:, h], ki, dk)", "dK[ki, h] = dk", 1),
    ("mean of three divides by two", "O = (moga[\"O\"] + O_s + O_f) / 3.0", "O = (moga[\"O\"] + O_s + O_f) / 2.0", 1),
    ("branches receive the whole upstream gradient", "dO3 = _f64(dO) / 3.0", "dO3 = _f64(dO)", 1),
    ("per-frame branch missing from dK", "\"dK\": b[\"dK\"] + dKs + dKf", "\"dK\": b[\"dK\"] + dKs", 1),
]


def load_mutated(old, new, count, source=ORACLE_SOURCE):
    src = open(source).read()
    assert src.count(old) == count, f"{old!r} occurs {src.count(old)} times in the oracle, expected {count}"
    mod = types.ModuleType("oracle.mutated")
    mod.__package__ = "oracle"          # the static-branch oracle imports its sibling relatively
    exec(compile(src.replace(old, new), source + " (mutated)", "exec"), mod.__dict__)
    return mod


def pin_calls(modules=None):
    """Every pin test as a zero-argument callable (parametrised tests once per parameter set)."""
    calls = []
    for module in (modules or (pins_fwd, pins_bwd)):
        for name, fn in sorted(vars(module).items()):
            if not name.startswith("test_") or not inspect.isfunction(fn):
                continue
            marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
            if not marks:
                calls.append((name, fn, ()))
                continue
            names = [n.strip() for n in marks[0].args[0].split(",")]
            for values in marks[0].args[1]:
                values = values if isinstance(values, (tuple, list)) and len(names) > 1 else (values,)
                calls.append((f"{name}{list(values)}", fn, tuple(values)))
    return calls


def first_failing_pin(modules=None):
    for name, fn, args in pin_calls(modules):
        try:
            fn(*args)
        except Exception:          # an assertion, or the arithmetic breaking down
            return name
    return None


def test_the_unchanged_oracle_passes_every_pin():
    assert first_failing_pin() is None


@pytest.mark.parametrize("what,old,new,count", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(what, old, new, count, monkeypatch):
    mutated = load_mutated(old, new, count)
    for name in orc.__all__:
        monkeypatch.setattr(orc, name, getattr(mutated, name))
    caught_by = first_failing_pin()
    assert caught_by is not None, f"no pin notices: {what}"


def test_the_unchanged_static_branch_oracle_passes_every_pin():
    assert first_failing_pin((pins_stga,)) is None


@pytest.mark.parametrize("what,old,new,count", STGA_MUTATIONS, ids=[m[0] for m in STGA_MUTATIONS])
def test_planted_mistake_in_the_static_branches_is_caught(what, old, new, count, monkeypatch):
    mutated = load_mutated(old, new, count, STGA_SOURCE)
    for name in sto.__all__:
        monkeypatch.setattr(sto, name, getattr(mutated, name))
    caught_by = first_failing_pin((pins_stga,))
    assert caught_by is not None, f"no pin notices: {what}"
