"""Measured compute times t_c (Sec. 5.1): a harness OUTSIDE the search library.

The paper obtains t_c(l, c) by "processing the layer under that configuration multiple times on the
device and measuring the average execution time", forward and backward.  Under a configuration
(n, h, w, c) every device processes one part of the layer's output: N/n samples, Cout/c channels and an
(Hout/h) x (Wout/w) window, for which it needs the window-expanded part of the input.  This module
times that part's forward + backward pass on the current GPU with PyTorch's own layer kernels (the
layers being parallelised are PyTorch's, not this library's) and returns one int32 nanosecond value
per configuration row, ready for lwp_build_cost_tables_graph(measured_tc=...).  Configurations that
differ only in their device block share one measurement.
"""
from __future__ import annotations

import numpy as np

KIND_CONV, KIND_POOL, KIND_FC = 0, 1, 2


def _ceil_div(a, b):
    return -(-a // b)


def part_shape(layer, cfg):
    """Largest part a device gets under cfg = (n, h, w, c, ...): (samples, out channels, out height, out width)."""
    kind, N, Cin, Hin, Win, Cout, Hout, Wout = (int(x) for x in layer[:8])
    n, h, w, c = (int(x) for x in cfg[:4])
    return _ceil_div(N, n), _ceil_div(Cout, c), _ceil_div(Hout, h), _ceil_div(Wout, w)


def _time_part(layer, shape, reps, warmup):
    import torch
    import torch.nn.functional as F
    kind, N, Cin, Hin, Win, Cout, Hout, Wout, kh, kw, sh, sw, ph, pw = (int(x) for x in layer)
    pn, pc, pH, pW = shape
    dev = torch.device("cuda")
    if kind == KIND_FC:
        x = torch.randn(pn, Cin * Hin * Win, device=dev, requires_grad=True)
        wgt = torch.randn(pc, Cin * Hin * Win, device=dev, requires_grad=True)
        b = torch.randn(pc, device=dev, requires_grad=True)

        def run():
            y = F.linear(x, wgt, b)
            y.backward(torch.ones_like(y))
    else:
        # the input window the part needs; padding is applied by the layer itself only at the tensor's
        # border, so the part is timed unpadded on its halo-expanded input
        in_h = min(Hin + 2 * ph, (pH - 1) * sh + kh)
        in_w = min(Win + 2 * pw, (pW - 1) * sw + kw)
        if kind == KIND_CONV:
            x = torch.randn(pn, Cin, in_h, in_w, device=dev, requires_grad=True)
            wgt = torch.randn(pc, Cin, kh, kw, device=dev, requires_grad=True)
            b = torch.randn(pc, device=dev, requires_grad=True)

            def run():
                y = F.conv2d(x, wgt, b, stride=(sh, sw))
                y.backward(torch.ones_like(y))
        else:
            x = torch.randn(pn, pc, in_h, in_w, device=dev, requires_grad=True)

            def run():
                y = F.max_pool2d(x, (kh, kw), stride=(sh, sw))
                y.backward(torch.ones_like(y))
    for _ in range(warmup):
        run()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(reps):
        run()
    stop.record()
    stop.synchronize()
    return max(1, int(round(start.elapsed_time(stop) * 1e6 / reps)))      # ms -> ns per pass


def measure_tc(layers, configs, C_node, reps=5, warmup=2):
    """int32 [sum(C_node)]: measured forward + backward nanoseconds of each configuration's part.

    layers int32 [L][14], configs int32 [rows][6] (the layers' lists one after another), C_node [L]."""
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("measuring layer times needs the GPU")
    layers = np.asarray(layers, np.int32).reshape(-1, 14)
    configs = np.asarray(configs, np.int32).reshape(-1, 6)
    C_node = np.asarray(C_node, np.int32).reshape(-1)
    out = np.zeros(int(C_node.sum()), np.int32)
    row = 0
    for l, layer in enumerate(layers):
        seen = {}
        for _ in range(int(C_node[l])):
            cfg = configs[row]
            key = tuple(int(x) for x in cfg[:4])
            if key not in seen:
                seen[key] = _time_part(layer, part_shape(layer, cfg), reps, warmup) if min(key) >= 1 else 0
            out[row] = seen[key]
            row += 1
    return out
