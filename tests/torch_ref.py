"""Textbook network forward written with torch.nn.functional + autograd, used
by the CPU tests as the library routine the oracle's hand-written layer
backward formulas are pinned against.  Float64, batch of one."""
import torch
import torch.nn.functional as F

from oracle import pb_oracle as O


def leaf_params(net, seed):
    ps = O.init_params(net, seed)
    return [{k: t.clone().requires_grad_(True) for k, t in p.items()} for p in ps]


def forward_loss(net, params, x, label):
    x = torch.as_tensor(x, dtype=torch.float64).reshape(1, net["in_c"], net["in_h"], net["in_w"])
    inputs = []
    for s, stage in enumerate(net["stages"]):
        P = params[s]
        inputs.append(x)
        for op in stage:
            k = op["kind"]
            if k == "gn":
                x = F.group_norm(x, op["groups"], P["gamma"], P["beta"], eps=1e-5)
            elif k == "relu":
                x = F.relu(x)
            elif k == "conv":
                x = F.conv2d(x, P["w"], P.get("b"), stride=op["stride"], padding=op["pad"])
            elif k == "linear":
                x = F.linear(x.reshape(1, -1), P["w"], P.get("b"))
            elif k == "maxpool":
                x = F.max_pool2d(x, op["k"], op["stride"], op["pad"])
            elif k == "gap":
                x = F.adaptive_avg_pool2d(x, 1)
            elif k == "add":
                sk = inputs[op["skip_from"]]
                if op["proj"]:
                    sk = F.conv2d(sk, P["wp"], None, stride=op["stride"])
                x = x + sk
            elif k == "ce":
                return F.cross_entropy(x.reshape(1, -1), torch.tensor([int(label)]), reduction="sum")
    raise AssertionError("no loss op")


def flat(params):
    return torch.cat([t.detach().reshape(-1) for p in params for t in p.values()])


def flat_grads(params):
    return torch.cat([t.grad.reshape(-1) for p in params for t in p.values()])
