"""CPU checks of this build's own readings of the paper, made with the oracle alone.

Reading: squat_prepare stores the update matrix of Lemma 2 on the fp16 grid (relative 2^-12 per entry) so that the
quantize kernels contract in two fp16 passes.  What that costs the METHOD is measured here on the oracle, where
nothing else differs: the iteration of Algorithm 1 `Quant` run with the float64 matrix and with the same matrix
rounded to fp16."""
import numpy as np
import pytest

from oracle import squat_oracle as O
from paper_2503_24358_amd import synth


@pytest.mark.parametrize("planted", [0, 12])
@pytest.mark.parametrize("lam", [1e-3, np.inf])
def test_update_matrix_on_the_fp16_grid_leaves_the_objective_alone(planted, lam):
    qpk, n, r, g, bits, G = 4, 2048, 16, 32, 2, 32
    _, qval = synth.store(synth.queries(11, qpk, n, planted_rank=planted), synth.BF16)
    _, kval = synth.store(synth.keys(12, 1, n, batch=1), synth.BF16)
    k = kval[0, 0]
    Qh, _ = O.subspace(qval, r)
    U = O.update_matrix_lowrank(Qh, lam, g)
    Ug = U.astype(np.float16).astype(np.float64)
    exact = O.quantize_keys(k, U, bits, G, g)
    grid = O.quantize_keys(k, Ug, bits, G, g)
    rtn = O.quantize_keys(k, None, bits, G, g)
    energy = lambda out: float(np.sum(((out["xhat"] - k) @ Qh.T) ** 2))      # noqa: E731
    # a few 1e-4 of the codes move (each by one step, with its cascade) ...
    assert (exact["codes"] != grid["codes"]).mean() <= 2e-3
    # ... and the objective of Eq. (1)'s relaxation, the projected error energy, moves by well under 1 %,
    # while the method's gain over round-to-nearest is a factor of 4 to 12 (it grows with the prompt length)
    assert abs(energy(grid) / energy(exact) - 1.0) <= 5e-3
    assert energy(exact) <= 0.3 * energy(rtn) and energy(grid) <= 0.3 * energy(rtn)
