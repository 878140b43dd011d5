"""The parity bar itself (tests/parity_util.check_layer) must notice single wrong elements: a whole-tensor
relative L2 alone lets one dropped output element of a large result through."""
import numpy as np
import pytest

from parity_util import ELEM_C_BF16, REL_L2_BF16, check_layer, rel_l2


def _fake(T=8, d=4096, E=8, k=2, seed=0, eps=2.7e-3):
    rng = np.random.default_rng(seed)
    out = rng.standard_normal((T, d)) * 0.05
    logits = rng.standard_normal((T, E))
    idx = np.argsort(-logits, axis=1, kind="stable")[:, :k].astype(np.int32)
    w = np.full((T, k), 1.0 / k)
    ref = dict(out=out, idx=idx, w=w, logits=logits)
    # a result with the rounding error the bf16 path shows: independent, normal, eps * rms per element
    noisy = out + eps * 0.05 * rng.standard_normal((T, d))
    gpu = dict(out=noisy.astype(np.float32), idx=idx.copy(), w=w.copy(), logits=logits.copy())
    return gpu, ref


def test_rounding_noise_of_the_expected_size_passes():
    gpu, ref = _fake()
    rep = check_layer(gpu, ref, 2, REL_L2_BF16)
    assert rep["rel_l2"] < 4e-3 and rep["max_elem_err_over_rms"] < 0.6 * ELEM_C_BF16


@pytest.mark.parametrize("what", ["zeroed", "doubled", "neighbour"])
def test_one_wrong_element_fails_although_the_norm_would_pass(what):
    gpu, ref = _fake()
    t = 5
    i = int(np.argmin(np.abs(np.abs(ref["out"][t]) - 0.05)))     # an element of typical size (the row's rms)
    if what == "zeroed":
        gpu["out"][t, i] = 0.0
    elif what == "doubled":
        gpu["out"][t, i] *= 2.0
    else:
        gpu["out"][t, i] = gpu["out"][t, i + 1 if i + 1 < gpu["out"].shape[1] else i - 1]
    if what != "neighbour":
        assert rel_l2(gpu["out"], ref["out"]) < REL_L2_BF16      # the whole-tensor norm does not see it
    with pytest.raises(AssertionError, match="element" if what != "neighbour" else None):
        check_layer(gpu, ref, 2, REL_L2_BF16)


def test_one_wrong_token_row_fails():
    gpu, ref = _fake(T=32)
    gpu["out"][7] *= 1.02                                         # 2 % off on one of 32 rows: 3.5e-3 in the whole norm
    assert rel_l2(gpu["out"], ref["out"]) < REL_L2_BF16
    with pytest.raises(AssertionError, match="token 7"):
        check_layer(gpu, ref, 2, REL_L2_BF16)
