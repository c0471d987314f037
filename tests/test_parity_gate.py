"""The gate the GPU parity tests apply (tests/parity_util.compare_tensor / compare_outputs), tried on the CPU against
planted mistakes: the implementation's output is imitated by the reference plus rounding noise of the size the bfloat16
path shows, and then damaged the way an indexing mistake in a kernel would damage it.  Every damage must be refused, at
the row counts of the LLaMA-7B MLP projection, where a whole-tensor norm alone lets a wrong row pass."""
import types

import numpy as np
import pytest

from paper_2402_04902_amd import inputs

from parity_util import BOUNDS, compare_outputs, compare_tensor

ROWS, COLS = 11008, 512     # the up projection's 11008 rows; fewer columns than 4096 to keep the test short


def _pair(seed=0, noise=2.3e-3):
    rng = np.random.default_rng(seed)
    ref = rng.standard_normal((ROWS, COLS))
    got = ref * (1.0 + noise * rng.standard_normal(ref.shape))
    return got, ref


def test_gate_accepts_rounding_noise():
    got, ref = _pair()
    m = compare_tensor("Y", got, ref, *BOUNDS[inputs.DTYPE_BF16]["Y"])
    assert 1e-3 < m["fro"] < 4e-3


def test_whole_tensor_norm_alone_would_let_a_wrong_row_pass():
    got, ref = _pair()
    got[4711, :] = 0.0
    fro = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    assert fro < 2e-2            # sqrt(1 / 11008) = 9.5e-3 on top of the noise: inside the whole-tensor bound
    with pytest.raises(AssertionError):
        compare_tensor("Y", got, ref, 2e-2, 2e-2)


@pytest.mark.parametrize("damage", ["zero_row", "zero_column", "stale_row", "one_element", "shifted_row", "row_x2"])
def test_gate_refuses_planted_damage(damage):
    got, ref = _pair(seed=1)
    if damage == "zero_row":
        got[ROWS - 1, :] = 0.0
    elif damage == "zero_column":
        got[:, 17] = 0.0
    elif damage == "stale_row":
        got[300, :] = got[299, :]
    elif damage == "one_element":
        got[5000, 100] += 0.2
    elif damage == "shifted_row":
        got[77, :] = np.roll(got[77, :], 1)
    elif damage == "row_x2":
        got[1234, :] *= 2.0
    with pytest.raises(AssertionError):
        compare_tensor("Y", got, ref, 2e-2, 2e-2)


def test_gate_refuses_one_wrong_group_of_dscale():
    """d(scale) is binary32 end to end (observed error 2e-5): one wrong group among 352 256 must not pass."""
    rng = np.random.default_rng(2)
    o, G = 11008, 32
    refs = {"Y": rng.standard_normal((64, 64)), "dX": rng.standard_normal((64, 64)),
            "dA": rng.standard_normal((16, 256)), "dB": rng.standard_normal((o, 16)),
            "dscale": rng.standard_normal((o, G)), "dzero": rng.standard_normal((o, G))}
    gr = types.SimpleNamespace(dX=refs["dX"], dA=refs["dA"], dB=refs["dB"], dscale=refs["dscale"], dzero=refs["dzero"],
                               dWq=rng.standard_normal((64, 64)))
    outs = {k: v * (1.0 + 2e-5 * rng.standard_normal(v.shape)) for k, v in refs.items()}
    compare_outputs(inputs.DTYPE_BF16, 128, outs, refs["Y"], gr)
    bad = dict(outs)
    bad["dscale"] = outs["dscale"].copy()
    bad["dscale"][9000, 5] *= 1.05                       # 5 % off in one group
    with pytest.raises(AssertionError):
        compare_outputs(inputs.DTYPE_BF16, 128, bad, refs["Y"], gr)
    bad = dict(outs)
    bad["dB"] = outs["dB"].copy()
    bad["dB"][10999, :] = 0.0                            # a dropped last row of dB
    with pytest.raises(AssertionError):
        compare_outputs(inputs.DTYPE_BF16, 128, bad, refs["Y"], gr)


def test_gate_handles_identically_zero_dzero():
    rng = np.random.default_rng(3)
    refs = {n: rng.standard_normal((32, 32)) for n in ("Y", "dX", "dA", "dB", "dscale")}
    refs["dzero"] = np.zeros((32, 4))
    gr = types.SimpleNamespace(dX=refs["dX"], dA=refs["dA"], dB=refs["dB"], dscale=refs["dscale"], dzero=refs["dzero"],
                               dWq=rng.standard_normal((32, 32)))
    outs = dict(refs)
    compare_outputs(inputs.DTYPE_F32, 8, outs, refs["Y"], gr)
    bad = dict(refs)
    bad["dzero"] = refs["dzero"].copy()
    bad["dzero"][3, 1] = 0.5
    with pytest.raises(AssertionError):
        compare_outputs(inputs.DTYPE_F32, 8, bad, refs["Y"], gr)
