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

Formats (mixed precision of Sec. 3.3 / Fig. 3) are those of the Net: activations, weight
copies and back-propagated errors in its `compute` format; weight gradients rounded from the
quire straight to its `master` format, which also holds the master weights and runs the
optimizer; the loss in its `loss` format.  Defaults: posit<8,0>, posit<16,1>, posit<16,1>.
Net(..., compute="p8_2", master="p12_2", loss="p10_2") is the configuration the paper ends up
with (Sec. 4, Table 4: posit(8,2) everywhere, optimizer posit(12,2), loss posit(10,2)).
"""
import torch

from . import binding as pn

ALPHA_MINUS_0P1 = 0xEB33  # posit<16,1> pattern of -(0x14CD), the rounded -0.1 (default master format)


class Net:
    """Weights of a layer list [("conv", cin, cout, k, pad) | ("fc", in, out) | ("relu",) |
    ("avgpool",) | ("maxpool",) | ("flatten",)] as masters (format `master`) and compute copies
    (format `compute`).  `alpha` is the pattern of -0.1 in the master format, rounded by the library."""

    def __init__(self, layers, params_f32, compute="p8", master="p16", loss="p16"):
        self.layers = layers
        self.compute, self.master, self.loss = compute, master, loss
        self.w16, self.b16, self.w8, self.b8 = [], [], [], []  # masters and compute copies (names from the default formats)
        for w, b in params_f32:
            w16 = pn.posit_round(w.contiguous(), master)
            b16 = pn.posit_round(b.contiguous(), master)
            self.w16.append(w16)
            self.b16.append(b16)
            self.w8.append(pn.posit_convert(w16, master, compute))
            self.b8.append(pn.posit_convert(b16, master, compute))
        self.one = 1 << (pn.FORMAT_BITS[compute] - 2)  # the pattern of the value one
        lr = pn.posit_round(torch.tensor([-0.1], dtype=torch.float32, device=params_f32[0][0].device), master)
        raw = lr.cpu().contiguous().view(torch.uint8).numpy()  # little-endian bytes of the one pattern
        self.alpha = int.from_bytes(raw.tobytes(), "little")


def loss_gradient(logits, labels, compute="p8", loss="p16"):
    """Softmax cross-entropy gradient in the loss format (Sec. 4: a wider loss next to 8-bit layers), then its
    copy in the compute format for the backward pass.  labels: int32 device tensor."""
    if labels.dtype != torch.int32:
        labels = labels.to(torch.int32)
    _, g = pn.posit_cross_entropy(logits, labels, compute, loss, loss, want_loss=False)
    return pn.posit_convert(g, loss, compute), g


def forward(net, x8, tape=None):
    fc = net.compute
    li = 0
    x = x8
    for layer in net.layers:
        kind = layer[0]
        if kind == "conv":
            _, cin, cout, k, pad = layer
            d = pn.conv_desc(tuple(x.shape), (cout, cin, k, k), (pad, pad), (1, 1))
            y = pn.posit_conv2d_fwd(x, net.w8[li], d, fc, fc, bias=net.b8[li])
            if tape is not None:
                tape.append(("conv", li, d, x))
            x = y
            li += 1
        elif kind == "fc":
            y = pn.posit_gemm(x, net.w8[li], fc, fc, trans_b=True, bias=net.b8[li])
            if tape is not None:
                tape.append(("fc", li, None, x))
            x = y
            li += 1
        elif kind == "relu":
            x = pn.posit_relu(x, fc)
            if tape is not None:
                tape.append(("relu", None, None, x))
        elif kind == "avgpool":
            if tape is not None:
                tape.append(("avgpool", None, None, None))
            x = pn.posit_avgpool2d_fwd(x, fc, fc)
        elif kind == "maxpool":
            x, idx = pn.posit_maxpool2d_fwd(x, fc)
            if tape is not None:
                tape.append(("maxpool", None, idx, None))
        elif kind == "flatten":
            if tape is not None:
                tape.append(("flatten", None, None, tuple(x.shape)))
            x = x.reshape(x.shape[0], -1)
    return x


def backward_and_update(net, tape, dy, alpha=None, grads=None):
    """Back-propagates dy (compute format) through the tape and applies the SGD update (alpha: pattern of
    minus the learning rate in the master format; default the net's -0.1).  When `grads` is a list,
    (layer, dw, db) tensors in the master format are appended to it."""
    fc, fm = net.compute, net.master
    alpha = net.alpha if alpha is None else alpha
    pending = []
    for kind, li, aux, saved in reversed(tape):
        if kind == "fc":
            dw = pn.posit_gemm(dy, saved, fc, fm, trans_a=True)
            ones = torch.full((dy.shape[0], 1), net.one, dtype=dy.dtype, device=dy.device)
            db = pn.posit_gemm(dy, ones, fc, fm, trans_a=True).reshape(-1)
            dx = pn.posit_gemm(dy, net.w8[li], fc, fc)
            _update(net, li, dw, db, alpha, grads, pending)
            dy = dx
        elif kind == "conv":
            dw, db = pn.posit_conv2d_bwd_weight(dy, saved, aux, fc, fm, with_bias=True)
            dx = pn.posit_conv2d_bwd_data(dy, net.w8[li], aux, fc, fc) if li > 0 else None
            _update(net, li, dw, db, alpha, grads, pending)
            dy = dx
        elif kind == "relu":
            dy = pn.posit_relu_bwd(saved, dy, fc, fc)
        elif kind == "avgpool":
            dy = pn.posit_avgpool2d_bwd(dy, fc, fc)
        elif kind == "maxpool":
            dy = pn.posit_maxpool2d_bwd(dy, aux, fc)
        elif kind == "flatten":
            dy = dy.reshape(saved)
    _apply_updates(pending, alpha, fm, fc)


def _update(net, li, dw, db, alpha, grads, pending):
    """Queues the SGD update of layer li: all layers are updated by one launch when the backward pass is over
    (nothing reads the weights between a layer's own backward-data and the next forward pass)."""
    if grads is not None:
        grads.append((li, dw.clone(), db.clone()))
    pending.append((dw, net.w16[li], net.w8[li]))
    pending.append((db, net.b16[li], net.b8[li]))


def _apply_updates(pending, alpha, fm, fc):
    if pending:
        pn.posit_axpy_multi(alpha, [g for g, _, _ in pending], [w for _, w, _ in pending], fm, fm, fcopy=fc,
                            y_copies=[c for _, _, c in pending])


def training_step(net, x_f32, labels, alpha=None, grads=None):
    """One full step; returns the logits (compute format)."""
    x8 = pn.posit_round(x_f32.contiguous(), net.compute)
    tape = []
    logits = forward(net, x8, tape)
    dy, _ = loss_gradient(logits, labels, net.compute, net.loss)
    backward_and_update(net, tape, dy, alpha, grads)
    return logits


class GraphedStep:
    """training_step captured once as a HIP graph and replayed on fixed input buffers.

    The capture records only kernels (the library clears its flags with a fill kernel, never with a
    memset node).  Two uncaptured warm-up steps run first so that lazy initialisation and the
    allocator's pools are settled; the weights are put back afterwards, so constructing a
    GraphedStep leaves the network as it was."""

    def __init__(self, net, x_shape, alpha=None):
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
