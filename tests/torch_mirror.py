"""Independent statement of the networks with torch.nn.functional (fp64, autograd), used to pin
the CPU reference.  Consumes the same flat parameter vector (op order; conv weights
[Cout][kh][kw][Cin]) and NHWC pixels."""
import torch
import torch.nn.functional as F


class _Params:
    def __init__(self, flat):
        self.flat = flat
        self.pos = 0

    def take(self, *shape):
        n = 1
        for s in shape:
            n *= s
        v = self.flat[self.pos:self.pos + n].reshape(*shape)
        self.pos += n
        return v


def _conv(p, x, cout, k, stride, pad):
    w = p.take(cout, k, k, x.shape[1]).permute(0, 3, 1, 2)
    return F.conv2d(x, w, None, stride, pad)


def _bn(p, x, relu, res=None):
    c = x.shape[1]
    g, b = p.take(c), p.take(c)
    y = F.batch_norm(x, None, None, g, b, training=True, eps=1e-5)
    if res is not None:
        y = y + res
    return F.relu(y) if relu else y


def _basic(p, x, cout, stride):
    cin = x.shape[1]
    y = _bn(p, _conv(p, x, cout, 3, stride, 1), True)
    y = _conv(p, y, cout, 3, 1, 1)
    sc = x
    if stride != 1 or cin != cout:
        sc = _bn(p, _conv(p, x, cout, 1, stride, 0), False)
    return _bn(p, y, True, sc)


def _bottleneck(p, x, width, stride):
    cin, cout = x.shape[1], 4 * width
    y = _bn(p, _conv(p, x, width, 1, 1, 0), True)
    y = _bn(p, _conv(p, y, width, 3, stride, 1), True)
    y = _conv(p, y, cout, 1, 1, 0)
    sc = x
    if stride != 1 or cin != cout:
        sc = _bn(p, _conv(p, x, cout, 1, stride, 0), False)
    return _bn(p, y, True, sc)


def _wide(p, x, cout, stride):
    cin = x.shape[1]
    o = _bn(p, x, True)
    y = _bn(p, _conv(p, o, cout, 3, stride, 1), True)
    # parameter order: conv1, bn2, [shortcut conv], conv2
    sc = x
    if stride != 1 or cin != cout:
        sc = _conv(p, o, cout, 1, stride, 0)
    return _conv(p, y, cout, 3, 1, 1) + sc


def _head(p, x, classes):
    f = x.mean(dim=(2, 3))
    w = p.take(classes, f.shape[1])
    b = p.take(classes)
    return f @ w.t() + b


def logits(arch, flat, x_nhwc, classes, mean=None, std=None):
    p = _Params(flat)
    x = x_nhwc.permute(0, 3, 1, 2)
    if mean is not None:
        m = torch.tensor(mean, dtype=x.dtype).view(1, 3, 1, 1)
        s = torch.tensor(std, dtype=x.dtype).view(1, 3, 1, 1)
        x = (x - m) / s
    if arch == 0:      # tiny CNN
        x = _conv(p, x, 16, 3, 1, 1); x = F.relu(x + p.take(16).view(1, -1, 1, 1))
        x = _conv(p, x, 32, 3, 2, 1); x = F.relu(x + p.take(32).view(1, -1, 1, 1))
    elif arch == 1:    # CIFAR ResNet-18
        x = _bn(p, _conv(p, x, 64, 3, 1, 1), True)
        for g, w in enumerate([64, 128, 256, 512]):
            for b in range(2):
                x = _basic(p, x, w, 2 if (b == 0 and g > 0) else 1)
    elif arch in (2, 5):    # WRN-34-10, WRN-28-10
        x = _conv(p, x, 16, 3, 1, 1)
        for g, w in enumerate([160, 320, 640]):
            for b in range(5 if arch == 2 else 4):
                x = _wide(p, x, w, 2 if (b == 0 and g > 0) else 1)
        x = _bn(p, x, True)
    elif arch == 4:    # pre-activation ResNet-18
        x = _conv(p, x, 64, 3, 1, 1)
        for g, w in enumerate([64, 128, 256, 512]):
            for b in range(2):
                x = _wide(p, x, w, 2 if (b == 0 and g > 0) else 1)
        x = _bn(p, x, True)
    elif arch == 3:    # ResNet-50
        x = _bn(p, _conv(p, x, 64, 7, 2, 3), True)
        x = F.max_pool2d(x, 3, 2, 1)
        for g, (w, n) in enumerate(zip([64, 128, 256, 512], [3, 4, 6, 3])):
            for b in range(n):
                x = _bottleneck(p, x, w, 2 if (b == 0 and g > 0) else 1)
    elif arch == 100:  # small net with every op kind
        x = _bn(p, _conv(p, x, 8, 3, 1, 1), True)
        x = F.max_pool2d(x, 3, 2, 1)
        x = _basic(p, x, 8, 1)
        x = _basic(p, x, 16, 2)
        x = _bottleneck(p, x, 8, 2)
        x = _wide(p, x, 16, 1)
        x = _wide(p, x, 16, 1)
        x = _bn(p, x, True)
    elif arch == 101:
        pass
    else:
        raise ValueError(arch)
    out = _head(p, x, classes)
    assert p.pos == flat.numel(), (p.pos, flat.numel())
    return out


def loss_and_grads(arch, flat64, x64_nhwc, y, classes, reduction="sum", mean=None, std=None):
    flat = torch.tensor(flat64, dtype=torch.float64, requires_grad=True)
    x = torch.tensor(x64_nhwc, dtype=torch.float64, requires_grad=True)
    z = logits(arch, flat, x, classes, mean, std)
    loss = F.cross_entropy(z, torch.tensor(y, dtype=torch.long), reduction=reduction)
    loss.backward()
    return loss.item(), z.detach().numpy(), x.grad.numpy(), flat.grad.numpy()


def objective_and_grads(arch, flat64, x64, xadv64, y, classes, lam, phi, mean=None, std=None):
    """F = lam * mean CE(net(x), y) + mean phi, phi = CE(net(xadv), y) (0) or KL(softmax net(x) || softmax net(xadv)) (1),
    each network evaluation its own train-mode forward.  Returns F, dF/dtheta, and d(sum_n phi_n)/dxadv with the
    clean evaluation held constant."""
    flat = torch.tensor(flat64, dtype=torch.float64, requires_grad=True)
    x = torch.tensor(x64, dtype=torch.float64)
    xadv = torch.tensor(xadv64, dtype=torch.float64, requires_grad=True)
    yt = torch.tensor(y, dtype=torch.long)
    z_adv = logits(arch, flat, xadv, classes, mean, std)
    if phi == 0:
        phi_n = F.cross_entropy(z_adv, yt, reduction="none")
        total = phi_n.mean()
        if lam != 0:
            total = total + lam * F.cross_entropy(logits(arch, flat, x, classes, mean, std), yt, reduction="mean")
        gx = torch.autograd.grad(phi_n.sum(), xadv, retain_graph=True)[0]
    else:
        z = logits(arch, flat, x, classes, mean, std)
        lp, lq = F.log_softmax(z, dim=1), F.log_softmax(z_adv, dim=1)
        phi_n = (lp.exp() * (lp - lq)).sum(dim=1)
        total = phi_n.mean() + lam * F.cross_entropy(z, yt, reduction="mean")
        lpc = lp.detach()
        gx = torch.autograd.grad((lpc.exp() * (lpc - lq)).sum(), xadv, retain_graph=True)[0]
    gt = torch.autograd.grad(total, flat)[0]
    return total.item(), gt.numpy(), gx.numpy()
