"""The pins of the attention oracle catch planted mistakes.

Each case below takes the SOURCE of oracle/attention.py, plants one plausible mistake in the tier that the parity
tests use (a dropped factor, a wrong sign, an off-by-one mask, a transposed operand, a wrong head mapping, ...),
loads the result as a throw-away module and runs the pins of tests/test_oracle_attention.py against it.  At least
one pin has to fail for every mutant, and all pass for the untouched source.  Nothing here touches the GPU path.
"""
import inspect
import types

import pytest

import oracle.attention as real
import test_oracle_attention as pins
import test_oracle_spaco as spaco_pins
import oracle.relay as real_relay
import test_oracle_relay as relay_pins
import oracle.model as real_model
import oracle.selection as real_selection
import test_oracle_selection as selection_pins
import test_oracle_sparse_dq as sparse_dq_pins
import test_oracle_model as model_pins

SOURCE = inspect.getsource(real)

# (name, text in the matmul tier, replacement)
MUTANTS = [
    ("mask excludes the diagonal", "np.arange(L)[None, :] <= (q_start + np.arange(C))[:, None]",
     "np.arange(L)[None, :] < (q_start + np.arange(C))[:, None]"),
    ("mask ignores q_start", "np.arange(L)[None, :] <= (q_start + np.arange(C))[:, None]",
     "np.arange(L)[None, :] <= (np.arange(C))[:, None]"),
    ("forward: scale dropped", "            s = scale * (q[b, h] @ kk.T)\n            s[~vis] = -np.inf",
     "            s = (q[b, h] @ kk.T)\n            s[~vis] = -np.inf"),
    ("forward: LSE without the shift", "lse[b, h] = (top + np.log(z))[:, 0]", "lse[b, h] = (np.log(z))[:, 0]"),
    ("forward: wrong KV head", "            kk = k_cache[b, h // G, :L]\n            vv = v_cache[b, h // G, :L]\n            s = scale * (q[b, h] @ kk.T)\n            s[~vis]",
     "            kk = k_cache[b, h % Hkv, :L]\n            vv = v_cache[b, h % Hkv, :L]\n            s = scale * (q[b, h] @ kk.T)\n            s[~vis]"),
    ("backward: sign of delta", "ds = prob * (dp - delta)", "ds = prob * (dp + delta)"),
    ("backward: delta from dO alone", "delta = (d_o[b, h] * o[b, h]).sum(axis=1, keepdims=True)",
     "delta = (d_o[b, h] * d_o[b, h]).sum(axis=1, keepdims=True)"),
    ("backward: dQ without the scale", "dq[b, h] = scale * (ds @ kk)", "dq[b, h] = (ds @ kk)"),
    ("backward: dK without the scale", "dk[b, g] += scale * (ds.T @ q[b, h])", "dk[b, g] += (ds.T @ q[b, h])"),
    ("backward: dK from dO", "dk[b, g] += scale * (ds.T @ q[b, h])", "dk[b, g] += scale * (ds.T @ d_o[b, h])"),
    ("backward: dV from dS", "dv[b, g] += prob.T @ d_o[b, h]", "dv[b, g] += ds.T @ d_o[b, h]"),
    ("backward: dP from K", "dp = d_o[b, h] @ vv.T", "dp = d_o[b, h] @ kk.T"),
    ("backward: group sum overwritten", "dv[b, g] += prob.T @ d_o[b, h]", "dv[b, g] = prob.T @ d_o[b, h]"),
    ("backward: masked probabilities kept", "prob = np.where(vis, np.exp(s - lse[b, h][:, None]), 0.0)",
     "prob = np.exp(s - lse[b, h][:, None])"),
    ("layer: contributions of a call overwrite gK", "        gK[:, :, :s0 + c] += dk\n        gV[:, :, :s0 + c] += dv\n    return O, LSE, dQ, gK, gV",
     "        gK[:, :, :s0 + c] = dk\n        gV[:, :, :s0 + c] += dv\n    return O, LSE, dQ, gK, gV"),
    ("layer: contributions of a call overwrite gV", "        gV[:, :, :s0 + c] += dv\n    return O, LSE, dQ, gK, gV",
     "        gV[:, :, :s0 + c] = dv\n    return O, LSE, dQ, gK, gV"),
]


def _load(source):
    import sys
    name = "oracle_mutant"
    mod = types.ModuleType(name)
    sys.modules[name] = mod            # (dataclasses look the defining module up while a class is created)
    try:
        exec(compile(source, name, "exec"), mod.__dict__)
    finally:
        del sys.modules[name]
    return mod


def _pin_calls(pins=pins):
    """Every pin of a test module, with its parameter grid expanded by hand from the marks."""
    calls = []
    for name, fn in inspect.getmembers(pins, inspect.isfunction):
        if not name.startswith("test_") or name == "test_argument_checks":
            continue
        grids = [[]]
        for mark in getattr(fn, "pytestmark", []):
            if mark.name != "parametrize":
                continue
            names = [n.strip() for n in mark.args[0].split(",")]
            new = []
            for g in grids:
                for vals in mark.args[1]:
                    vals = vals if isinstance(vals, (tuple, list)) and len(names) > 1 else (vals,)
                    new.append(g + list(zip(names, vals)))
            grids = new
        for g in grids:
            kw = dict(g)
            if kw.get("tier") == "loops":        # the mistakes are planted in the matmul tier
                continue
            calls.append((name, fn, kw))
    return calls


def _failures(module, monkeypatch, pins=pins):
    monkeypatch.setattr(pins, "A", module)
    failed = []
    for name, fn, kw in _pin_calls(pins):
        try:
            fn(**kw)
        except AssertionError:
            failed.append(name)
        except (ValueError, FloatingPointError, IndexError):
            failed.append(name)
    return failed


def test_untouched_source_passes_every_pin(monkeypatch):
    assert len(_pin_calls()) >= 15
    assert _failures(_load(SOURCE), monkeypatch) == []


@pytest.mark.parametrize("what,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(what, old, new, monkeypatch):
    assert SOURCE.count(old) >= 1, f"the oracle no longer contains the text this case edits: {old!r}"
    failed = _failures(_load(SOURCE.replace(old, new)), monkeypatch)
    assert failed, f"no pin noticed: {what}"


# mistakes in the SpaCO schedule (Alg. 2 at one layer), against the pins of tests/test_oracle_spaco.py
SPACO_MUTANTS = [
    ("factor also on the chunk's own rows", "gK[:, :, s0:s0 + c] += dk[:, :, s0:s0 + c]            # own rows: weight 1",
     "gK[:, :, s0:s0 + c] += factor * dk[:, :, s0:s0 + c]"),
    ("factor not applied to earlier chunks", "gK[:, :, t0:t0 + ci] += factor * dk[:, :, t0:t0 + ci]",
     "gK[:, :, t0:t0 + ci] += dk[:, :, t0:t0 + ci]"),
    ("deposits on later selected chunks instead of earlier ones", "            if i < j:                                         # earlier selected chunk",
     "            if i > j:"),
    ("deposits on every earlier chunk, selected or not", "        for i in sel:\n            if i < j:                                         # earlier selected chunk",
     "        for i in range(len(chunks)):\n            if i < j:"),
    ("dQ of selected chunks dropped", "        dQ[:, :, s0:s0 + c] = dq\n        gK[:, :, s0:s0 + c] += dk[:, :, s0:s0 + c]",
     "        gK[:, :, s0:s0 + c] += dk[:, :, s0:s0 + c]"),
]


def test_untouched_source_passes_every_spaco_pin(monkeypatch):
    assert len(_pin_calls(spaco_pins)) >= 10
    assert _failures(_load(SOURCE), monkeypatch, spaco_pins) == []


@pytest.mark.parametrize("what,old,new", SPACO_MUTANTS, ids=[m[0] for m in SPACO_MUTANTS])
def test_planted_mistake_in_the_sparse_schedule_is_caught(what, old, new, monkeypatch):
    assert SOURCE.count(old) == 1, f"the oracle no longer contains the text this case edits: {old!r}"
    failed = _failures(_load(SOURCE.replace(old, new)), monkeypatch, spaco_pins)
    assert failed, f"no pin noticed: {what}"


# mistakes in the cache append / gradient read-out / rotary embedding oracle, against tests/test_oracle_relay.py
RELAY_SOURCE = inspect.getsource(real_relay)
RELAY_MUTANTS = [
    ("rotation turns the wrong way", "return np.concatenate([a * cos - b * sin, b * cos + a * sin], axis=-1)",
     "return np.concatenate([a * cos + b * sin, b * cos - a * sin], axis=-1)"),
    ("frequency exponent -i/D instead of -2i/D", "np.power(float(base), -2.0 * i / D)", "np.power(float(base), -1.0 * i / D)"),
    ("positions start one late", "th = rope_angles(pos0 + np.arange(C), D, base)", "th = rope_angles(pos0 + 1 + np.arange(C), D, base)"),
    ("inverse does not turn back", "np.sin(th) * (-1.0 if inverse else 1.0)", "np.sin(th)"),
    ("pairs (2i, 2i+1) instead of (i, i + D/2)", "a, b = x[..., :D // 2], x[..., D // 2:]\n    return np.concatenate([a * cos - b * sin, b * cos + a * sin], axis=-1)",
     "a, b = x[..., 0::2], x[..., 1::2]\n    return np.stack([a * cos - b * sin, b * cos + a * sin], axis=-1).reshape(x.shape)"),
]


def _relay_failures(module, monkeypatch):
    monkeypatch.setattr(relay_pins, "R", module)
    failed = []
    for name, fn in inspect.getmembers(relay_pins, inspect.isfunction):
        if name.startswith("test_"):
            try:
                fn()
            except AssertionError:
                failed.append(name)
    return failed


def test_untouched_relay_source_passes_its_pins(monkeypatch):
    assert _relay_failures(_load(RELAY_SOURCE), monkeypatch) == []


@pytest.mark.parametrize("what,old,new", RELAY_MUTANTS, ids=[m[0] for m in RELAY_MUTANTS])
def test_planted_mistake_in_the_rotary_embedding_is_caught(what, old, new, monkeypatch):
    assert RELAY_SOURCE.count(old) == 1, f"the oracle no longer contains the text this case edits: {old!r}"
    assert _relay_failures(_load(RELAY_SOURCE.replace(old, new)), monkeypatch), f"no pin noticed: {what}"


# mistakes in the multi-layer schedules (Alg. 1 / Alg. 2 over a decoder), against tests/test_oracle_model.py
MODEL_SOURCE = inspect.getsource(real_model)
MODEL_MUTANTS = [
    ("factor on the key gradient only", "grads += [factor * gk, factor * gv]", "grads += [factor * gk, gv]"),
    ("value gradient not handed over", "                roots += [k, v]\n                grads += [factor * gk, factor * gv]",
     "                roots += [k]\n                grads += [factor * gk]"),
    ("second loop in ascending order", "range(len(ckpt) - 1, -1, -1), 1.0, dq_weights)", "range(len(ckpt)), 1.0, dq_weights)"),
    ("a chunk also sees its own checkpoint", "(torch.cat([c[l][0] for c in ckpt[:i]], 2), torch.cat([c[l][1] for c in ckpt[:i]], 2)) if i",
     "(torch.cat([c[l][0] for c in ckpt[:i + 1]], 2), torch.cat([c[l][1] for c in ckpt[:i + 1]], 2)) if i"),
    ("mask without the diagonal", "vis = torch.arange(L)[None, :] <= (q_start + torch.arange(C))[:, None]",
     "vis = torch.arange(L)[None, :] <= (q_start + torch.arange(C) - 1)[:, None]"),
    ("query heads mapped to the wrong KV head", "    k_rep = k_all.repeat_interleave(G, 1)\n", "    k_rep = k_all.repeat(1, G, 1, 1)\n"),
]


def _model_failures(module, monkeypatch):
    monkeypatch.setattr(model_pins, "om", module)
    failed = []
    for name, fn, kw in _pin_calls(model_pins):
        if "monkeypatch" in inspect.signature(fn).parameters:
            kw = dict(kw, monkeypatch=monkeypatch)
        try:
            fn(**kw)
        except (AssertionError, RuntimeError, ValueError, IndexError):
            failed.append(name)
    return failed


def test_untouched_model_source_passes_its_pins(monkeypatch):
    assert _model_failures(_load(MODEL_SOURCE), monkeypatch) == []


@pytest.mark.parametrize("what,old,new", MODEL_MUTANTS, ids=[m[0] for m in MODEL_MUTANTS])
def test_planted_mistake_in_the_multi_layer_schedule_is_caught(what, old, new, monkeypatch):
    assert MODEL_SOURCE.count(old) == 1, f"the oracle no longer contains the text this case edits: {old!r}"
    assert _model_failures(_load(MODEL_SOURCE.replace(old, new)), monkeypatch), f"no pin noticed: {what}"


# mistakes in the selection of Alg. 2, against tests/test_oracle_selection.py
SELECTION_SOURCE = inspect.getsource(real_selection)
SELECTION_MUTANTS = [
    ("a wrong multiplier in the generator's finaliser", "0xBF58476D1CE4E5B9", "0xBF58476D1CE4E5B7"),
    ("bounded draw without rejection", "            if u < limit:\n                return u % m", "            return u % m"),
    ("draws with replacement", "        r = i + rng.below(k - i)\n", "        r = rng.below(k)\n"),
    ("ascending output", "return np.array(sorted(perm[:t], reverse=True), dtype=np.int32)",
     "return np.array(sorted(perm[:t]), dtype=np.int32)"),
    ("the step does not enter the key", "_finalise((seed & _MASK) ^ _finalise((step + _GOLDEN) & _MASK))",
     "_finalise((seed & _MASK) ^ _finalise(_GOLDEN & _MASK))"),
    ("never selects the last chunk", "        r = i + rng.below(k - i)\n", "        r = i + rng.below(max(k - i - 1, 1))\n"),
]


def _selection_failures(module, monkeypatch):
    monkeypatch.setattr(selection_pins, "S", module)
    failed = []
    for name, fn, kw in _pin_calls(selection_pins):
        try:
            fn(**kw)
        except (AssertionError, ValueError, IndexError):
            failed.append(name)
    return failed


def test_untouched_selection_source_passes_its_pins(monkeypatch):
    assert _selection_failures(_load(SELECTION_SOURCE), monkeypatch) == []


@pytest.mark.parametrize("what,old,new", SELECTION_MUTANTS, ids=[m[0] for m in SELECTION_MUTANTS])
def test_planted_mistake_in_the_selection_is_caught(what, old, new, monkeypatch):
    assert SELECTION_SOURCE.count(old) == 1, f"the oracle no longer contains the text this case edits: {old!r}"
    assert _selection_failures(_load(SELECTION_SOURCE.replace(old, new)), monkeypatch), f"no pin noticed: {what}"


# mistakes in the column-weighted dQ, against tests/test_oracle_sparse_dq.py
SPARSE_DQ_MUTANTS = [
    ("weights squared", "dq[b, h] = scale * ((ds * w[None, :]) @ kk)", "dq[b, h] = scale * ((ds * w[None, :] * w[None, :]) @ kk)"),
    ("weights applied to the rows", "dq[b, h] = scale * ((ds * w[None, :]) @ kk)", "dq[b, h] = scale * ((ds * w[-C:, None]) @ kk)"),
    ("delta restricted to the weighted columns", "            ds = prob * (d_o[b, h] @ vv.T - delta)\n            dq[b, h] = scale * ((ds * w[None, :]) @ kk)",
     "            ds = prob * (d_o[b, h] @ vv.T - ((prob * w[None, :]) * (d_o[b, h] @ vv.T)).sum(axis=1, keepdims=True))\n"
     "            dq[b, h] = scale * ((ds * w[None, :]) @ kk)"),
]


@pytest.mark.parametrize("what,old,new", [("untouched", "", "")] + SPARSE_DQ_MUTANTS,
                         ids=["untouched"] + [m[0] for m in SPARSE_DQ_MUTANTS])
def test_planted_mistake_in_the_weighted_dq_is_caught(what, old, new, monkeypatch):
    assert what == "untouched" or SOURCE.count(old) == 1, f"the oracle no longer contains the text this case edits: {old!r}"
    failed = _failures(_load(SOURCE.replace(old, new) if old else SOURCE), monkeypatch, sparse_dq_pins)
    assert (failed == []) if what == "untouched" else failed, f"{what}: {failed}"
