"""The bf16 storage model used to bound deep-stack parity: without rounding it IS the oracle's layer; with rounding
its distance from the oracle grows with depth and with the spread of the attention scores, as the tolerances assume."""
import numpy as np

from oracle import dsk_oracle as O
from paper_2411_02820_amd import synth
from tests import bf16_storage_model as M
from tests.helpers import oracle_config, weights_fn

SHAPE = synth.ModelShape(4, 256, 8, 2, 64, 512, 10000.0, 1e-5, "bf16")


def _run(rounded, scale=1.0, lens=(37, 5, 70)):
    cfg = oracle_config(SHAPE)
    cu = synth.cu_seqlens(lens)
    pos = synth.packed_positions(lens)
    T = int(cu[-1])
    base = weights_fn(SHAPE, 0)
    h = synth.hidden_states(SHAPE, T).astype(np.float64)
    h_ref = h.copy()
    errs = []
    for l in range(SHAPE.n_layers):
        w = {k: (v if k in ("g1", "g2") else v * scale) for k, v in base(l).items()}
        h_ref, K_ref, V_ref = O.prefix_layer(cfg, w, h_ref, pos, cu)
        h, K, V = M.prefix_layer(cfg, w, h, pos, cu, rounded=rounded)
        errs.append((O.max_rel_err(K, K_ref), O.max_rel_err(V, V_ref), O.max_rel_err(h, h_ref)))
    return errs


def test_without_rounding_it_is_the_oracle_layer():
    for eK, eV, eh in _run(False):
        assert max(eK, eV, eh) <= 1e-12


def test_rounding_costs_a_few_1e3_per_layer_and_adds_up():
    errs = _run(True)
    assert 1e-3 <= errs[0][0] <= 8e-3 and errs[0][2] <= 1e-2        # one layer: the storage error of its operands
    assert errs[-1][2] > errs[0][2]                                  # deeper is worse
    assert max(max(e) for e in errs) <= 2e-2                         # four narrow layers stay inside the spec bar


def test_peaked_softmax_amplifies_the_rounding_of_q_and_k():
    mild, strong = _run(True, 1.0), _run(True, 8.0)
    assert strong[-1][2] > 3 * mild[-1][2]
