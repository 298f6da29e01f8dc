"""Independent fp64 replica of a student block on PyTorch's CPU autograd, used
only to pin the oracle (library conv / batch-norm / pooling routines)."""
import torch
import torch.nn.functional as F

from paper_2301_12443_amd import workloads as W


def run_block(block, x, params, train, eps=1e-5, alphas=None):
    """params[(j, slot)] -> tensor; alphas[j] -> architecture parameters of mix op j (its weights are
    then softmax(alphas[j]) instead of the descriptor's).  Returns (output, {j: (batch mean, biased var)})."""
    vals = [x]
    stats = {}
    for j, op in enumerate(block.ops):
        a = vals[op.inputs[0]]
        if op.type == W.OP_CBA:
            y = F.conv2d(a, params[(j, W.P_WEIGHT)], stride=op.stride, padding=op.pad, groups=op.groups)
            if train:
                stats[j] = (y.mean(dim=(0, 2, 3)).detach(), y.var(dim=(0, 2, 3), unbiased=False).detach())
                y = F.batch_norm(y, None, None, params[(j, W.P_GAMMA)], params[(j, W.P_BETA)],
                                 training=True, eps=eps)
            else:
                y = F.batch_norm(y, params[(j, W.P_RMEAN)], params[(j, W.P_RVAR)],
                                 params[(j, W.P_GAMMA)], params[(j, W.P_BETA)], training=False, eps=eps)
            if op.act == W.ACT_RELU:
                y = F.relu(y)
            elif op.act == W.ACT_RELU6:
                y = F.hardtanh(y, 0.0, 6.0)
            vals.append(y)
        elif op.type == W.OP_POOL:
            vals.append(F.max_pool2d(a, op.k, op.stride, op.pad))
        elif op.type == W.OP_ADD:
            y = a + vals[op.inputs[1]]
            vals.append(F.relu(y) if op.act == W.ACT_RELU else y)
        elif op.type == W.OP_MIX:
            p = torch.softmax(alphas[j], dim=0) if alphas is not None and j in alphas else op.p
            vals.append(sum(p[k] * vals[i] for k, i in enumerate(op.inputs)))
    return vals[-1], stats


def block_params(wl, net, b, requires_grad):
    out = {}
    for (j, slot), shape in W.param_shapes(wl, net, b).items():
        t = torch.from_numpy(W.make_param(wl, net, b, j, slot, shape)).double()
        if requires_grad and slot in (W.P_WEIGHT, W.P_GAMMA, W.P_BETA):
            t.requires_grad_()
        out[(j, slot)] = t
    return out
