"""The five-convolution stack of the network the paper trains, as a sequence of
C-ABI calls: forward through conv1..conv5 with ReLU and 3x3/stride-2 max
pooling after conv1, conv2 and conv5, then back-propagation from a gradient on
the last pooling output down to the first layer's filter gradient.

Second layer: two model-parallel columns (channels 0..47 -> filters 0..127,
channels 48..95 -> filters 128..255) -- the two-column layout of the paper's
model-parallelism paragraph -- run as one grouped call per pass on the shared
NCHW tensors (filters of both columns in one [256, 48, 5, 5] tensor).  Layers three to five run at full width.  The
first layer computes no input gradient (nothing lies below it).

With dtype="bf16" the input, the filters and every activation and gradient
tensor are bfloat16: convolutions accumulate in fp32 and round each output once
(forward and backward-data write bfloat16, backward-filter writes fp32 filter
gradients), the glue layers work on bfloat16 tensors.

This module only owns buffers and the order of calls; all arithmetic happens
in the library.
"""
import numpy as np
import torch

from . import binding as hp
from . import synth

CONV_ORDER = ("conv1", "conv2", "conv3", "conv4", "conv5")


def conv_flops(N, L):
    """Nominal FLOPs of one pass of a layer: 2*N*K*P*Q*C*R*S (padding taps counted)."""
    return 2.0 * N * L["K"] * L["P"] * L["Q"] * L["C"] * L["R"] * L["S"]


def stack_flops(N):
    """Nominal conv FLOPs of one forward+backward step of the stack."""
    Ls = synth.LAYERS
    total = 2 * conv_flops(N, Ls["conv1"])                    # fwd + wgrad
    total += 2 * 3 * conv_flops(N, Ls["conv2"])               # two columns, three passes
    for name in ("conv3", "conv4", "conv5"):
        total += 3 * conv_flops(N, Ls[name])
    return total


class ConvStack:
    def __init__(self, N, seed=synth.SEED_BASE + 64, device="cuda", dtype="f32"):
        self.N = N
        self.bf16 = dtype == "bf16"
        act = dict(dtype=torch.bfloat16 if self.bf16 else torch.float32, device=device)

        def t(a):
            """Seeded host tensor on the device, in the stack's storage type."""
            v = torch.from_numpy(a).to(device)
            return hp.convert_f32_to_bf16(v) if self.bf16 else v

        self.x0 = t(synth.gaussian((N, 3, 224, 224), seed + 0))
        self.w = {
            "conv1": t(synth.gaussian((96, 3, 11, 11), seed + 1, synth.STD_FILTER)),
            # the two columns' filters, column a first
            "conv2": t(np.concatenate([synth.gaussian((128, 48, 5, 5), seed + 2, synth.STD_FILTER),
                                       synth.gaussian((128, 48, 5, 5), seed + 3, synth.STD_FILTER)])),
            "conv3": t(synth.gaussian((384, 256, 3, 3), seed + 4, synth.STD_FILTER)),
            "conv4": t(synth.gaussian((384, 384, 3, 3), seed + 5, synth.STD_FILTER)),
            "conv5": t(synth.gaussian((256, 384, 3, 3), seed + 6, synth.STD_FILTER)),
        }
        self.g5 = t(synth.gaussian((N, 256, 6, 6), seed + 7))
        self.dw = {k: torch.empty(v.shape, dtype=torch.float32, device=device) for k, v in self.w.items()}
        # activations (y3, y4 hold relu(conv): the ReLU is applied where the convolution stores its sums, and its
        # backward where the next layer's backward-data stores; y1, y2, y5 keep the pre-activation: their ReLU is
        # fused into the pooling calls)
        self.y1 = torch.empty((N, 96, 55, 55), **act)
        self.a1 = torch.empty((N, 96, 27, 27), **act)
        self.y2 = torch.empty((N, 256, 27, 27), **act)
        self.a2 = torch.empty((N, 256, 13, 13), **act)
        self.y3 = torch.empty((N, 384, 13, 13), **act)
        self.y4 = torch.empty((N, 384, 13, 13), **act)
        self.y5 = torch.empty((N, 256, 13, 13), **act)
        self.a5 = torch.empty((N, 256, 6, 6), **act)
        # gradients
        self.dy5 = torch.empty_like(self.y5)
        self.dy4 = torch.empty_like(self.y4)
        self.dy3 = torch.empty_like(self.y3)
        self.da2 = torch.empty_like(self.a2)
        self.dy2 = torch.empty_like(self.y2)
        self.da1 = torch.empty_like(self.a1)
        self.dy1 = torch.empty_like(self.y1)
        self.ws = hp.Workspace(device)
        self.timers = None          # optional dict name -> (start, stop) events per conv call

    # -- helpers ------------------------------------------------------------
    def _timed(self, key, fn):
        if self.timers is None:
            return fn()
        s, e = self.timers.setdefault(key, (torch.cuda.Event(enable_timing=True),
                                            torch.cuda.Event(enable_timing=True)))
        s.record()
        out = fn()
        e.record()
        return out

    def forward(self):
        w, ws = self.w, self.ws
        self._timed(("conv1", "fwd"), lambda: hp.conv_fwd(self.x0, w["conv1"], 4, 2, y=self.y1, ws=ws))
        hp.relu_maxpool3x3s2_fwd(self.y1, self.a1)
        self._timed(("conv2", "fwd"), lambda: hp.conv_fwd_grouped(self.a1, w["conv2"], 1, 2, 2, y=self.y2, ws=ws))
        hp.relu_maxpool3x3s2_fwd(self.y2, self.a2)
        self._timed(("conv3", "fwd"),
                    lambda: hp.conv_fwd_bias_relu(self.a2, w["conv3"], None, 1, 1, y=self.y3, ws=ws))
        self._timed(("conv4", "fwd"),
                    lambda: hp.conv_fwd_bias_relu(self.y3, w["conv4"], None, 1, 1, y=self.y4, ws=ws))
        self._timed(("conv5", "fwd"), lambda: hp.conv_fwd(self.y4, w["conv5"], 1, 1, y=self.y5, ws=ws))
        hp.relu_maxpool3x3s2_fwd(self.y5, self.a5)
        return self.a5

    def backward(self):
        w, dw, ws = self.w, self.dw, self.ws
        hp.relu_maxpool3x3s2_bwd(self.y5, self.g5, self.dy5)
        self._timed(("conv5", "wgrad"),
                    lambda: hp.conv_bwd_filter(self.y4, self.dy5, 3, 3, 1, 1, dw=dw["conv5"], ws=ws))
        self._timed(("conv5", "dgrad"),
                    lambda: hp.conv_bwd_data_relu(self.dy5, w["conv5"], self.y4, 1, 1, dx=self.dy4, ws=ws))
        self._timed(("conv4", "wgrad"),
                    lambda: hp.conv_bwd_filter(self.y3, self.dy4, 3, 3, 1, 1, dw=dw["conv4"], ws=ws))
        self._timed(("conv4", "dgrad"),
                    lambda: hp.conv_bwd_data_relu(self.dy4, w["conv4"], self.y3, 1, 1, dx=self.dy3, ws=ws))
        self._timed(("conv3", "wgrad"),
                    lambda: hp.conv_bwd_filter(self.a2, self.dy3, 3, 3, 1, 1, dw=dw["conv3"], ws=ws))
        self._timed(("conv3", "dgrad"),
                    lambda: hp.conv_bwd_data(self.dy3, w["conv3"], 13, 13, 1, 1, dx=self.da2, ws=ws))
        hp.relu_maxpool3x3s2_bwd(self.y2, self.da2, self.dy2)
        self._timed(("conv2", "wgrad"),
                    lambda: hp.conv_bwd_filter_grouped(self.a1, self.dy2, 5, 5, 1, 2, 2, dw=dw["conv2"], ws=ws))
        self._timed(("conv2", "dgrad"),
                    lambda: hp.conv_bwd_data_grouped(self.dy2, w["conv2"], 27, 27, 1, 2, 2, dx=self.da1, ws=ws))
        hp.relu_maxpool3x3s2_bwd(self.y1, self.da1, self.dy1)
        self._timed(("conv1", "wgrad"),
                    lambda: hp.conv_bwd_filter(self.x0, self.dy1, 11, 11, 4, 2, dw=dw["conv1"], ws=ws))
        return dw

    def step(self):
        self.forward()
        return self.backward()

    def capture(self):
        """One step recorded into a HIP graph (torch's capture of the stream the binding launches on).  A step is
        run first so that the workspace has its final size: nothing allocates while the graph is recorded, and the
        library itself issues only kernel launches (no memsets, copies or synchronisation).  Replaying the graph
        runs the step on the buffers this object owns."""
        self.step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.step()
        return graph


FC_LAYERS = (("fc6", 256 * 6 * 6, 4096), ("fc7", 4096, 4096), ("fc8", 4096, 1000))


def fc_flops(N):
    """Nominal FLOPs of the three fully connected layers, forward + backward-data + backward-filter (the first one
    included: its input gradient feeds the convolutional stack)."""
    return sum(3 * 2.0 * N * i * o for _, i, o in FC_LAYERS)


class FullNetwork(ConvStack):
    """The convolutional stack with the three fully connected layers of the network on top (9216 -> 4096 -> 4096 ->
    1000, bias and ReLU after the first two) and the SGD update of every parameter: one whole synchronous training
    step on one GPU's shard, fp32.  The loss is replaced by a seeded gradient on the last layer's output; dropout,
    response normalisation and the soft-max are not part of it."""

    def __init__(self, N, seed=synth.SEED_BASE + 96, device="cuda", lr=0.01, momentum=0.9, weight_decay=5e-4):
        super().__init__(N, seed=seed, device=device, dtype="f32")
        self.lr, self.momentum, self.weight_decay = lr, momentum, weight_decay
        f = dict(dtype=torch.float32, device=device)
        self.fc_w, self.fc_b, self.fc_dw, self.fc_db, self.fc_y, self.fc_dy = {}, {}, {}, {}, {}, {}
        for j, (name, i, o) in enumerate(FC_LAYERS):
            self.fc_w[name] = torch.from_numpy(synth.gaussian((o, i), seed + 20 + 2 * j, synth.STD_FILTER)).to(device)
            self.fc_b[name] = torch.from_numpy(synth.gaussian((o,), seed + 21 + 2 * j, 0.1)).to(device)
            self.fc_dw[name] = torch.empty((o, i), **f)
            self.fc_db[name] = torch.empty((o,), **f)
            self.fc_y[name] = torch.empty((N, o), **f)
            self.fc_dy[name] = torch.empty((N, o), **f)
        self.g8 = torch.from_numpy(synth.gaussian((N, 1000), seed + 30)).to(device)
        # one velocity per parameter tensor
        self.params = ([(self.w[k], self.dw[k]) for k in CONV_ORDER]
                       + [(self.fc_w[n], self.fc_dw[n]) for n, _, _ in FC_LAYERS]
                       + [(self.fc_b[n], self.fc_db[n]) for n, _, _ in FC_LAYERS])
        self.vel = [torch.zeros_like(p) for p, _ in self.params]

    def forward(self):
        a = super().forward().view(self.N, -1)
        ws = self.ws
        for name, _, _ in FC_LAYERS:
            a = hp.fc_fwd(a, self.fc_w[name], self.fc_b[name], relu=name != "fc8", y=self.fc_y[name], ws=ws)
        return a

    def backward(self):
        ws, N = self.ws, self.N
        d = self.g8
        for idx in range(len(FC_LAYERS) - 1, -1, -1):
            name = FC_LAYERS[idx][0]
            if name != "fc8":                   # through the ReLU that follows the layer
                d = hp.relu_bwd(self.fc_y[name], d, self.fc_dy[name])
            inp = self.fc_y[FC_LAYERS[idx - 1][0]] if idx > 0 else self.a5.view(N, -1)
            hp.fc_bwd_filter(inp, d, dw=self.fc_dw[name], ws=ws)
            hp.bias_bwd(d.view(N, -1, 1, 1), db=self.fc_db[name], ws=ws)
            dx = self.fc_dy[FC_LAYERS[idx - 1][0]] if idx > 0 else self.g5.view(N, -1)
            d = hp.fc_bwd_data(d, self.fc_w[name], dx=dx, ws=ws)
        return super().backward()

    def update(self):
        """Mean gradient over this shard's N samples (a data-parallel job would first sum the shards' gradients)."""
        hp.sgd_update_multi([p for p, _ in self.params], [g for _, g in self.params], self.vel, self.lr,
                            self.momentum, self.weight_decay, 1.0 / self.N)

    def step(self):
        self.forward()
        self.backward()
        self.update()
