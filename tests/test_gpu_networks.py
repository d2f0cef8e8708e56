"""Benchmark configs 3 and 4: LeNet-5-shaped (batch 64) and CifarNet-shaped (batch 128)
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


FINAL = ("p8_2", "p12_2", "p10_2")  # Sec. 4, Table 4: posit(8,2) layers, posit(12,2) optimizer, posit(10,2) loss


@pytest.mark.parametrize("net,batch,fmts", [(workloads.LENET, 64, nn_harness.DEFAULT_FORMATS), (workloads.CIFARNET, 128, nn_harness.DEFAULT_FORMATS),
                                            (workloads.LENET, 64, FINAL), (workloads.CIFARNET, 128, FINAL),
                                            (workloads.LENET, 64, ("p8_1", "p16", "p12_1")), (workloads.CIFARNET, 32, ("p8_1", "p12_1", "p16"))])
def test_device_resident_step_matches_layerwise_harness(net, batch, fmts):
    """The all-on-GPU step (library glue kernels for ReLU / pooling, nothing on the host) ends in
    exactly the weights the layer-by-layer, oracle-checked harness ends in, in the default formats
    and in the configuration the paper ends up with (both at the batch sizes the benchmark times)."""
    import numpy as np
    import torch

    from paper_2105_00053_amd import posit_round as pn_round
    from paper_2105_00053_amd import train_step
    from gpu_util import to_np

    x, params, labels = workloads.network_inputs(net, batch)
    state = {}
    fc, fm, fl = fmts
    log = nn_harness.training_step(net, batch, x, params, labels, final_state=state, fmts=fmts)
    assert all(bad == 0 for _, _, bad in log)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    model = train_step.Net(net["layers"], [(dev(w), dev(b)) for w, b in params], compute=fc, master=fm, loss=fl)
    logits = train_step.training_step(model, dev(x), torch.from_numpy(labels).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(to_np(logits, fc), state["logits"])
    changed = 0
    for li in range(len(params)):
        assert np.array_equal(to_np(model.w16[li], fm), state["W16"][li]), "master weights of layer %d" % li
        assert np.array_equal(to_np(model.b16[li], fm), state["B16"][li])
        assert np.array_equal(to_np(model.w8[li], fc), state["W8"][li])
        assert np.array_equal(to_np(model.b8[li], fc), state["B8"][li])
        before = to_np(pn_round(dev(params[li][0]), fm), fm)
        changed += int((before != state["W16"][li]).sum())
    assert changed > 0, "the step must move some master weight"


@pytest.mark.parametrize("net,batch", [(workloads.LENET, 64), (workloads.CIFARNET, 32)])
def test_graph_replay_equals_eager_steps(net, batch):
    """The captured step replayed four times on changing batches, with eager library calls and
    synchronisations between the replays, leaves exactly the weights that four eager steps leave."""
    import numpy as np
    import torch

    import paper_2105_00053_amd as pn
    from paper_2105_00053_amd import train_step
    from gpu_util import to_np

    x, params, labels = workloads.network_inputs(net, batch)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    eager = train_step.Net(net["layers"], [(dev(w), dev(b)) for w, b in params])
    graphed = train_step.Net(net["layers"], [(dev(w), dev(b)) for w, b in params])
    runner = train_step.GraphedStep(graphed, x.shape)
    for li in range(len(params)):  # construction put the weights back
        assert np.array_equal(to_np(graphed.w16[li], "p16"), to_np(eager.w16[li], "p16"))
    rng = np.random.default_rng(11)
    for step in range(4):
        xs = np.roll(x, step, axis=0) * np.float32(1.0 + 0.25 * step)
        ls = torch.from_numpy(np.roll(labels, 3 * step).astype(np.int32)).cuda()
        want_logits = train_step.training_step(eager, dev(xs), ls)
        got_logits = runner.step(dev(xs), ls)
        torch.cuda.synchronize()
        assert np.array_equal(to_np(got_logits, "p8"), to_np(want_logits, "p8")), "logits of step %d" % step
        for li in range(len(params)):
            assert np.array_equal(to_np(graphed.w16[li], "p16"), to_np(eager.w16[li], "p16")), "step %d layer %d" % (step, li)
            assert np.array_equal(to_np(graphed.w8[li], "p8"), to_np(eager.w8[li], "p8"))
            assert np.array_equal(to_np(graphed.b16[li], "p16"), to_np(eager.b16[li], "p16"))
        # unrelated eager work between the replays
        junk = pn.posit_round(torch.from_numpy(rng.standard_normal(5000).astype(np.float32)).cuda(), "p16")
        pn.posit_gemm(pn.posit_convert(junk[:4096].reshape(64, 64), "p16", "p8"), pn.posit_convert(junk[:4096].reshape(64, 64), "p16", "p8"), "p8", "p8")
        torch.cuda.synchronize()
