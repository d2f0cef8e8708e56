"""BASELINE configs 3 and 4: LeNet-5-shaped (batch 64) and CifarNet-shaped (batch 128)
training steps, every dot-product layer bit-exact against the oracle (see nn_harness)."""
import pytest

import workloads

import nn_harness

pytestmark = pytest.mark.gpu


def _run(net, batch):
    x, params, labels = workloads.network_inputs(net, batch)
    log = nn_harness.training_step(net, batch, x, params, labels)
    assert all(bad == 0 for _, _, bad in log)
    names = [n for n, _, _ in log]
    return names


def test_config3_lenet_step_batch64():
    names = _run(workloads.LENET, 64)
    for needed in ("conv0 fwd", "conv1 fwd", "avgpool fwd", "fc4 fwd", "fc2 bwd_weight", "conv1 bwd_data", "conv0 bwd_weight",
                   "avgpool bwd", "sgd w0", "sgd b4 copy"):
        assert needed in names, needed


def test_config4_cifarnet_step_batch128():
    names = _run(workloads.CIFARNET, 128)
    for needed in ("conv0 fwd", "conv4 fwd", "fc5 fwd", "fc5 bwd_data", "conv4 bwd_weight", "conv1 bwd_data", "conv0 bwd_bias", "sgd w3"):
        assert needed in names, needed
