"""The pins must notice plausible mistakes.  Each mutant is the numpy oracle with one
line changed (a dropped term, a wrong operand, a swapped gate, a transposed matrix);
every one of them has to fail at least one pin.  All of this runs on the CPU."""
import os

import numpy as np
import pytest

import test_oracle_treelstm as pins

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "treelstm_oracle.py")

MUTANTS = {
    "forget gate from the summed h": ("f = _sigmoid(fx + Uf @ h[k])", "f = _sigmoid(fx + Uf @ hs)"),
    "forget bias dropped": ("fx = Wf @ x[j] + bf", "fx = Wf @ x[j]"),
    "output and candidate rows swapped": ("Wi, Wo, Wu, Wf = (W[g * H:(g + 1) * H] for g in range(4))",
                                          "Wi, Wu, Wo, Wf = (W[g * H:(g + 1) * H] for g in range(4))"),
    "cell from o instead of i": ("cj = i * u", "cj = o * u"),
    "tanh on c missing": ("h[j] = o * np.tanh(cj)", "h[j] = o * cj"),
    "U_i transposed": ("i = _sigmoid(Wi @ x[j] + Ui @ hs + bi)", "i = _sigmoid(Wi @ x[j] + Ui.T @ hs + bi)"),
    "U_f transposed": ("f = _sigmoid(fx + Uf @ h[k])", "f = _sigmoid(fx + Uf.T @ h[k])"),
    "candidate through sigmoid": ("u = np.tanh(Wu @ x[j] + Uu @ hs + bu)", "u = _sigmoid(Wu @ x[j] + Uu @ hs + bu)"),
    "child sum misses the last child": ("        for k in ch[j]:\n            hs = hs + h[k]",
                                        "        for k in ch[j][:-1]:\n            hs = hs + h[k]"),
    "forget times h instead of c": ("cj = cj + f * c[k]", "cj = cj + f * h[k]"),
    "recurrent term of o dropped": ("o = _sigmoid(Wo @ x[j] + Uo @ hs + bo)", "o = _sigmoid(Wo @ x[j] + bo)"),
    "forget gate ignored": ("cj = cj + f * c[k]", "cj = cj + c[k]"),
    "sign of the forget sum": ("cj = cj + f * c[k]", "cj = cj - f * c[k]"),
    "input bias dropped": ("i = _sigmoid(Wi @ x[j] + Ui @ hs + bi)", "i = _sigmoid(Wi @ x[j] + Ui @ hs)"),
}


def _mutant(old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, old
    ns = {}
    exec(compile(text.replace(old, new), "mutant_oracle", "exec"), ns)
    return lambda *a: ns["forward"](*a)


def test_unmutated_source_passes_every_pin():
    ns = {}
    exec(compile(open(SRC).read(), "oracle_copy", "exec"), ns)
    for pin in pins.ALL_PINS:
        pin(lambda *a: ns["forward"](*a))


@pytest.mark.parametrize("what", sorted(MUTANTS))
def test_every_mutant_fails_some_pin(what):
    fwd = _mutant(*MUTANTS[what])
    caught = []
    for pin in pins.ALL_PINS:
        try:
            pin(fwd)
        except AssertionError:
            caught.append(pin)
    assert caught, f"no pin notices: {what}"
