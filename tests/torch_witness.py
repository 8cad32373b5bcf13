"""A second witness for whole-network tests: the same network built from an autograd
library's conv2d / max_pool2d / linear in double precision.  Test helper only; it is not
the oracle and shares no code with it or with the GPU path."""
import re

import numpy as np
import torch

A, B = 1.7159, 0.6666


def parse(arch):
    toks = arch.split("-")
    c, h, w = (int(v) for v in toks[0].split("x"))
    layers = []
    for t in toks[1:]:
        m = re.fullmatch(r"(\d+)C(\d+)(?:x(\d+))?(?:S(\d+)(?:x(\d+))?)?", t)
        if m:
            ky = int(m.group(2))
            kx = int(m.group(3) or ky)
            sy = int(m.group(4) or 0)
            sx = int(m.group(5) or sy)
            layers.append(("conv", int(m.group(1)), (ky, kx), (sy, sx)))
            continue
        m = re.fullmatch(r"MP(\d+)(?:x(\d+))?", t)
        if m:
            layers.append(("pool", (int(m.group(1)), int(m.group(2) or m.group(1)))))
            continue
        m = re.fullmatch(r"(\d+)N", t)
        layers.append(("fc", int(m.group(1))))
    return (c, h, w), layers


def loss_and_grads(arch, weights, image, label, tables=None, frontend=None, tanh_outputs=False):
    """Returns (loss, grad in the canonical flat layout, probs).  tables: {conv_index: [mo, mi]}.
    frontend: (filters [n, k, k], src_channel [n]) applied to the raw image first (linear).
    tanh_outputs: scaled-tanh output units and half the squared error against +-1 targets
    (the outputs are then returned in place of the probabilities)."""
    tables = tables or {}
    (c, h, w), layers = parse(arch)
    wt = torch.tensor(np.asarray(weights, dtype=np.float64), requires_grad=True)
    x = torch.tensor(np.asarray(image, dtype=np.float64))
    if frontend is not None:
        filt, src = frontend
        outs = []
        for f in range(filt.shape[0]):
            ch = x[int(src[f])][None, None]
            outs.append(torch.nn.functional.conv2d(ch, torch.tensor(filt[f], dtype=torch.float64)[None, None])[0, 0])
        x = torch.stack(outs)
    x = x.reshape(1, c, h, w)
    off = 0
    conv_idx = 0
    maps = c
    for li, l in enumerate(layers):
        if l[0] == "conv":
            _, mo, (ky, kx), (sy, sx) = l
            table = np.asarray(tables.get(conv_idx, np.ones((mo, maps), dtype=np.uint8)))
            conv_idx += 1
            bias = wt[off:off + mo]
            off += mo
            rows = []
            for j in range(mo):
                cols = []
                for i in range(maps):
                    if table[j, i]:
                        cols.append(wt[off:off + ky * kx].reshape(ky, kx))
                        off += ky * kx
                    else:
                        cols.append(torch.zeros(ky, kx, dtype=torch.float64))
                rows.append(torch.stack(cols))
            dense = torch.stack(rows)
            x = A * torch.tanh(B * torch.nn.functional.conv2d(x, dense, bias, stride=(sy + 1, sx + 1)))
            maps = mo
        elif l[0] == "pool":
            x = torch.nn.functional.max_pool2d(x, l[1])
        else:
            n = l[1]
            v = x.reshape(1, -1)
            n_in = v.shape[1]
            bias = wt[off:off + n]
            off += n
            W = wt[off:off + n * n_in].reshape(n, n_in)
            off += n * n_in
            x = torch.nn.functional.linear(v, W, bias)
            if li + 1 < len(layers):
                x = A * torch.tanh(B * x)
    assert off == wt.numel()
    if tanh_outputs:
        y = A * torch.tanh(B * x[0])
        target = -torch.ones_like(y)
        target[int(label)] = 1.0
        loss = 0.5 * torch.sum((y - target) ** 2)
        loss.backward()
        return loss.item(), wt.grad.numpy().copy(), y.detach().numpy()
    logp = torch.log_softmax(x[0], 0)
    loss = -logp[int(label)]
    loss.backward()
    return loss.item(), wt.grad.numpy().copy(), torch.exp(logp).detach().numpy()
