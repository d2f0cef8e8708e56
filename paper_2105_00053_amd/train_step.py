"""Device-resident training step for small CNNs described as layer lists.

Chains the library's entry points (convolution / linear forward, backward-data,
backward-weight, ReLU, pooling, SGD update) so that a LeNet-5-shaped or
CifarNet-shaped step runs without leaving the GPU.  Pure orchestration: every
number is produced by a kernel of libpositnn_hip.so, the softmax cross-entropy
gradient included (posit_cross_entropy in the posit<16,1> loss format).  The
kernels of a step are issued on one stream (moving the weight-gradient branch
to a second stream was measured and lost: cross-stream waits cost more than
they hide).  GraphedStep captures the whole step once as a HIP graph and
replays it: the LeNet-5-shaped step, about fifty short kernels, is bound by
the host-side launches and runs 1.6x faster replayed; the CifarNet-shaped
step is bound by its kernels and gains nothing.

Formats (mixed precision of Sec. 3.3 / Fig. 3): activations, weight copies and
back-propagated errors posit<8,0>; weight gradients rounded from the quire to
posit<16,1>; master weights and optimizer posit<16,1>.
"""
import torch

from . import binding as pn

ALPHA_MINUS_0P1 = 0xEB33  # posit<16,1> pattern of -(0x14CD), the rounded -0.1


class Net:
    """Weights of a layer list [("conv", cin, cout, k, pad) | ("fc", in, out) | ("relu",) |
    ("avgpool",) | ("maxpool",) | ("flatten",)] as posit<16,1> masters and posit<8,0> copies."""

    def __init__(self, layers, params_f32):
        self.layers = layers
        self.w16, self.b16, self.w8, self.b8 = [], [], [], []
        for w, b in params_f32:
            w16 = pn.posit_round(w.contiguous(), "p16")
            b16 = pn.posit_round(b.contiguous(), "p16")
            self.w16.append(w16)
            self.b16.append(b16)
            self.w8.append(pn.posit_convert(w16, "p16", "p8"))
            self.b8.append(pn.posit_convert(b16, "p16", "p8"))


def loss_gradient(logits_p8, labels):
    """Softmax cross-entropy gradient in the posit<16,1> loss format (Sec. 4: a 16-bit loss next to 8-bit
    layers), then its posit<8,0> copy for the backward pass.  labels: int32 device tensor."""
    if labels.dtype != torch.int32:
        labels = labels.to(torch.int32)
    _, g16 = pn.posit_cross_entropy(logits_p8, labels, "p8", "p16", "p16", want_loss=False)
    return pn.posit_convert(g16, "p16", "p8"), g16


def forward(net, x8, tape=None):
    li = 0
    x = x8
    for layer in net.layers:
        kind = layer[0]
        if kind == "conv":
            _, cin, cout, k, pad = layer
            d = pn.conv_desc(tuple(x.shape), (cout, cin, k, k), (pad, pad), (1, 1))
            y = pn.posit_conv2d_fwd(x, net.w8[li], d, "p8", "p8", bias=net.b8[li])
            if tape is not None:
                tape.append(("conv", li, d, x))
            x = y
            li += 1
        elif kind == "fc":
            y = pn.posit_gemm(x, net.w8[li], "p8", "p8", trans_b=True, bias=net.b8[li])
            if tape is not None:
                tape.append(("fc", li, None, x))
            x = y
            li += 1
        elif kind == "relu":
            x = pn.posit_relu(x, "p8")
            if tape is not None:
                tape.append(("relu", None, None, x))
        elif kind == "avgpool":
            if tape is not None:
                tape.append(("avgpool", None, None, None))
            x = pn.posit_avgpool2d_fwd(x, "p8", "p8")
        elif kind == "maxpool":
            x, idx = pn.posit_maxpool2d_fwd(x, "p8")
            if tape is not None:
                tape.append(("maxpool", None, idx, None))
        elif kind == "flatten":
            if tape is not None:
                tape.append(("flatten", None, None, tuple(x.shape)))
            x = x.reshape(x.shape[0], -1)
    return x


def backward_and_update(net, tape, dy, alpha=ALPHA_MINUS_0P1, grads=None):
    """Back-propagates dy (posit<8,0>) through the tape and applies the SGD update layer by
    layer.  When `grads` is a list, (layer, dw, db) posit<16,1> tensors are appended to it."""
    pending = []
    for kind, li, aux, saved in reversed(tape):
        if kind == "fc":
            dw = pn.posit_gemm(dy, saved, "p8", "p16", trans_a=True)
            ones = torch.full((dy.shape[0], 1), 0x40, dtype=torch.uint8, device=dy.device)
            db = pn.posit_gemm(dy, ones, "p8", "p16", trans_a=True).reshape(-1)
            dx = pn.posit_gemm(dy, net.w8[li], "p8", "p8")
            _update(net, li, dw, db, alpha, grads, pending)
            dy = dx
        elif kind == "conv":
            dw, db = pn.posit_conv2d_bwd_weight(dy, saved, aux, "p8", "p16", with_bias=True)
            dx = pn.posit_conv2d_bwd_data(dy, net.w8[li], aux, "p8", "p8") if li > 0 else None
            _update(net, li, dw, db, alpha, grads, pending)
            dy = dx
        elif kind == "relu":
            dy = pn.posit_relu_bwd(saved, dy, "p8", "p8")
        elif kind == "avgpool":
            dy = pn.posit_avgpool2d_bwd(dy, "p8", "p8")
        elif kind == "maxpool":
            dy = pn.posit_maxpool2d_bwd(dy, aux, "p8")
        elif kind == "flatten":
            dy = dy.reshape(saved)
    _apply_updates(pending, alpha)


def _update(net, li, dw, db, alpha, grads, pending):
    """Queues the SGD update of layer li: all layers are updated by one launch when the backward pass is over
    (nothing reads the weights between a layer's own backward-data and the next forward pass)."""
    if grads is not None:
        grads.append((li, dw.clone(), db.clone()))
    pending.append((dw, net.w16[li], net.w8[li]))
    pending.append((db, net.b16[li], net.b8[li]))


def _apply_updates(pending, alpha):
    if pending:
        pn.posit_axpy_multi(alpha, [g for g, _, _ in pending], [w for _, w, _ in pending], "p16", "p16", fcopy="p8",
                            y_copies=[c for _, _, c in pending])


def training_step(net, x_f32, labels, alpha=ALPHA_MINUS_0P1, grads=None):
    """One full step; returns the logits (posit<8,0>)."""
    x8 = pn.posit_round(x_f32.contiguous(), "p8")
    tape = []
    logits = forward(net, x8, tape)
    dy, _ = loss_gradient(logits, labels)
    backward_and_update(net, tape, dy, alpha, grads)
    return logits


class GraphedStep:
    """training_step captured once as a HIP graph and replayed on fixed input buffers.

    The capture records only kernels (the library clears its flags with a fill kernel, never with a
    memset node).  Two uncaptured warm-up steps run first so that lazy initialisation and the
    allocator's pools are settled; the weights are put back afterwards, so constructing a
    GraphedStep leaves the network as it was."""

    def __init__(self, net, x_shape, alpha=ALPHA_MINUS_0P1):
        dev = net.w16[0].device
        self.net = net
        self.x = torch.zeros(tuple(x_shape), dtype=torch.float32, device=dev)
        self.labels = torch.zeros((x_shape[0],), dtype=torch.int32, device=dev)
        saved = [[t.clone() for t in group] for group in (net.w16, net.b16, net.w8, net.b8)]
        side = torch.cuda.Stream()  # default priority
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(2):
                training_step(net, self.x, self.labels, alpha)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        for group, keep in zip((net.w16, net.b16, net.w8, net.b8), saved):
            for t, k in zip(group, keep):
                t.copy_(k)
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            self.logits = training_step(net, self.x, self.labels, alpha)

    def step(self, x_f32, labels):
        """Copies the batch into the captured buffers, replays the graph, returns the (static) logits tensor."""
        self.x.copy_(x_f32)
        self.labels.copy_(labels)
        self.graph.replay()
        return self.logits
