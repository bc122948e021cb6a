"""GPU parity: the C-ABI path against the CPU oracle, element by element, on seeded inputs."""
import pytest

from tests.parity import run_case

pytestmark = pytest.mark.gpu


def _assert_ok(rep):
    bad = {k: v for k, v in rep.items() if v == "MISMATCH"}
    assert rep["ok"], {"bad": bad, "report": {k: v for k, v in rep.items() if isinstance(v, tuple)}}


def test_config0_tiny_rgcn_fp32():
    _assert_ok(run_case(0, verbose=True, check_naive=True))


def test_config0_per_edge_type_input():
    _assert_ok(run_case(0, verbose=True, use_edge_id=False))


def test_config1_fp32_scaled():
    _assert_ok(run_case(1, scale=0.05, batch=256, verbose=True, check_naive=True))


def test_config2_bf16_scaled():
    _assert_ok(run_case(2, scale=0.05, batch=512, verbose=True, check_naive=True))


def test_config2_bf16_scaled_without_input_grads_of_fixed_features():
    # T0 carries fixed features, T1-T3 learnable embeddings: only those need input gradients in layer 1
    _assert_ok(run_case(2, scale=0.05, batch=512, verbose=True, input_grad=[0, 1, 1, 1]))


def test_config3_many_types_fp32_scaled():
    _assert_ok(run_case(3, scale=0.02, batch=128, verbose=True, check_naive=True))


def test_config2_full_size_headline_workload():
    """The workload bench.py times (full graph, 4096 targets, bf16, hidden 512, input gradients only for the
    learnable embeddings), compared element by element with the oracle."""
    rep = run_case(2, scale=1.0, verbose=True, input_grad=[0, 1, 1, 1])
    _assert_ok(rep)
    assert rep["sizes"][0][2] > 900_000 and rep["sizes"][1][1] == 4096
