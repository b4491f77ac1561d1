"""The oracle against the hand-evaluated cases stored under tests/golden/ (Section 3.2.2 quantisers Q, CQ, SQ at
k = 8; Section 3.1 residual-branch weight scale; the two requantising steps of the backward chain, Q_e(e2 * gamma)
of Section 3.2.1 and the merge of branch and shortcut errors).  Each fixture's header says where its lines come
from."""
import ast
import os

import numpy as np
import pytest

from oracle import fixup
from oracle import ops as oo
from oracle import quant as oq

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "quantiser_hand_cases.txt")
GOLDEN_BWD = os.path.join(os.path.dirname(__file__), "golden", "backward_hand_cases.txt")


def _cases(path=GOLDEN):
    out = []
    with open(path) as f:
        for ln, line in enumerate(f, 1):
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, args, want = (t.strip() for t in line.split(";"))
            out.append(pytest.param(name, ast.literal_eval("(" + args + ",)"), ast.literal_eval(want), id=f"{name}-line{ln}"))
    return out


def test_fixture_is_complete():
    names = {p.values[0] for p in _cases()}
    assert names == {"rne", "q", "cq", "sq_real", "sq_int", "alpha"}
    assert len(_cases()) >= 20


@pytest.mark.parametrize("name,args,want", _cases())
def test_hand_case(name, args, want):
    if name == "rne":
        assert oq.rne_shift(np.array(args[0], dtype=np.int64), args[1]).tolist() == want
    elif name == "q":
        assert oq.q_code(np.array(args[0], dtype=np.float64)).tolist() == want
    elif name == "cq":
        assert oq.cq_code(np.array(args[0], dtype=np.float64)).tolist() == want
    elif name == "sq_real":
        c, E = oq.sq_real(np.array(args[0], dtype=np.float64))
        assert (c.tolist(), E) == want
    elif name == "sq_int":
        c, E = oq.sq_int(np.array(args[0], dtype=np.int64), args[1])
        assert (c.tolist(), E) == want
    elif name == "alpha":
        assert fixup.alpha(*args) == pytest.approx(want, rel=1e-12)
    else:
        raise AssertionError(name)


def test_backward_fixture_is_complete():
    cases = _cases(GOLDEN_BWD)
    assert {p.values[0] for p in cases} == {"gamma", "merge"}
    assert sum(p.values[0] == "gamma" for p in cases) >= 5 and sum(p.values[0] == "merge" for p in cases) >= 6


@pytest.mark.parametrize("name,args,want", _cases(GOLDEN_BWD))
def test_backward_hand_case(name, args, want):
    if name == "gamma":
        e1, E, g = args
        c, E3 = oo.sq_error_gamma(np.array(e1, dtype=np.int8), E, g)
    elif name == "merge":
        a, Ea, b, Eb = args
        c, E3 = oo.merge_errors(np.array(a, dtype=np.int8), Ea, np.array(b, dtype=np.int8), Eb)
    else:
        raise AssertionError(name)
    assert c.dtype == np.int8 and (c.tolist(), E3) == want
