"""Seeded sweep of irregular shapes through the update entry points, each compared with the oracle like the named
workloads: widths that are no multiple of any tile, single-layer and deep networks, one to seven minibatches,
action widths across the padded head sizes, with and without symmetry; the same for the recurrent update (both
cells) and the behaviour-cloning update."""
from dataclasses import replace
import numpy as np
import pytest

from workloads import WORKLOADS
import test_gpu_update as U
import test_gpu_recurrent as R

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rx():
    import paper_2509_10771_amd as m
    m.rslx_device_check()
    return m


def _shapes(seed, count):
    g = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        M = int(g.choice([1, 2, 3, 5, 7]))
        nb = int(g.integers(3, 60))
        depth = int(g.integers(1, 4))
        hidden = tuple(int(g.choice([8, 20, 33, 64, 100, 128, 130, 256])) for _ in range(depth))
        out.append(dict(N=nb * M, T=int(g.integers(1, 10)), D=int(g.integers(1, 70)), A=int(g.integers(1, 33)), hidden=hidden,
                        minibatches=M))
    return out


@pytest.mark.parametrize("i,shape", list(enumerate(_shapes(101, 10))))
def test_ppo_update_irregular_shapes(rx, i, shape):
    sym = i % 3 == 0
    base = WORKLOADS["rough" if sym else "tiny"]
    w = replace(base, N=shape["N"], T=shape["T"], Da=shape["D"], Dc=shape["D"], A=shape["A"], hidden=shape["hidden"],
                minibatches=shape["minibatches"], height_scan=0)
    if sym:
        w = replace(w, symmetry=True)
    case = U.Case(w, 1, sym_on=sym, perturb=0.15)
    U.check_forced_steps(rx, case)


@pytest.mark.parametrize("i,shape", list(enumerate(_shapes(202, 8))))
def test_recurrent_update_irregular_shapes(rx, i, shape):
    H = int(np.random.default_rng(300 + i).choice([4, 12, 36, 64, 100]))
    w = replace(WORKLOADS["recurrent"], N=shape["N"], T=shape["T"], Da=shape["D"], Dc=shape["D"], A=shape["A"],
                hidden=shape["hidden"], minibatches=shape["minibatches"], memory_hidden=H, done_p=0.1,
                memory_cell="lstm" if i % 2 else "gru")
    case = R.RCase(w, 1, perturb=0.1)
    R.check_forced_steps(rx, case, floor=5e-2)


# Observation widths around the staged-input decision of the update: a width that is a whole number of 16-column
# tiles is read in place unless the minibatch is mirrored; any other width is copied into zero-padded rows once per
# call, unless the first layer is too small for the padded contraction to stay inside the parameter buffer, in
# which case the rows are read in place through the slow path.  All four must agree with the oracle.
@pytest.mark.parametrize("D,hidden,sym", [(48, (64, 64), True), (37, (64, 64), False), (37, (64,), False), (235, (128, 64), True),
                                          (16, (8,), True)])
def test_ppo_update_staged_and_in_place_inputs(rx, D, hidden, sym):
    base = WORKLOADS["rough" if sym else "tiny"]
    w = replace(base, N=96, T=5, Da=D, Dc=D, A=4, hidden=hidden, minibatches=3, height_scan=0)
    if sym:
        w = replace(w, symmetry=True)
    case = U.Case(w, 1, sym_on=sym, perturb=0.15)
    U.check_forced_steps(rx, case)
