"""Independent reference for pinning the CPU oracle: the same module written with torch's own CPU
operators and differentiated by torch.autograd in float64.  Used only by the `not gpu` oracle pins;
it shares nothing with oracle/ or with the HIP path."""
import torch
import torch.nn.functional as F

STEM, BASIC_POSTACT, BASIC_PREACT, HEAD_POSTACT, HEAD_PREACT, BOTTLENECK_POSTACT = 0, 1, 2, 3, 4, 5
STEM_POOL, INVERTED_RESIDUAL = 6, 7


def _bn(x, g, b, eps):
    return F.batch_norm(x, None, None, g, b, training=True, momentum=0.0, eps=eps)


def split_params(spec, shapes, flat):
    """flat -> list of leaf tensors (float64, requires_grad) in flat order."""
    out, off = [], 0
    for _, shape, _ in shapes:
        n = 1
        for s in shape:
            n *= s
        out.append(torch.tensor(flat[off:off + n], dtype=torch.float64).reshape(shape).requires_grad_(True))
        off += n
    return out


def forward(spec, params, x, labels=None):
    """Returns the module output (top module: (loss, logits))."""
    it = iter(params)
    z = x
    eps = spec.bn_eps
    for L in spec.layers:
        proj = L.kind in (BASIC_POSTACT, BASIC_PREACT, BOTTLENECK_POSTACT) and (L.stride != 1 or L.c_in != L.c_out)
        if L.kind == STEM:
            w, g, b = next(it), next(it), next(it)
            z = F.relu(_bn(F.conv2d(z, w, stride=L.stride, padding=1), g, b, eps))
        elif L.kind == BASIC_POSTACT:
            w1, g1, b1, w2, g2, b2 = (next(it) for _ in range(6))
            a = F.relu(_bn(F.conv2d(z, w1, stride=L.stride, padding=1), g1, b1, eps))
            r = _bn(F.conv2d(a, w2, stride=1, padding=1), g2, b2, eps)
            if proj:
                wp, gp, bp = next(it), next(it), next(it)
                sc = _bn(F.conv2d(z, wp, stride=L.stride), gp, bp, eps)
            else:
                sc = z
            z = F.relu(r + sc)
        elif L.kind == BOTTLENECK_POSTACT:
            w1, g1, b1, w2, g2, b2, w3, g3, b3 = (next(it) for _ in range(9))
            a = F.relu(_bn(F.conv2d(z, w1), g1, b1, eps))
            a = F.relu(_bn(F.conv2d(a, w2, stride=L.stride, padding=1), g2, b2, eps))
            r = _bn(F.conv2d(a, w3), g3, b3, eps)
            if proj:
                wp, gp, bp = next(it), next(it), next(it)
                sc = _bn(F.conv2d(z, wp, stride=L.stride), gp, bp, eps)
            else:
                sc = z
            z = F.relu(r + sc)
        elif L.kind == STEM_POOL:
            w, g, b = next(it), next(it), next(it)
            z = F.max_pool2d(F.relu(_bn(F.conv2d(z, w, stride=2, padding=3), g, b, eps)), 3, stride=2, padding=1)
        elif L.kind == INVERTED_RESIDUAL:
            w1, g1, b1, w2, g2, b2, w3, g3, b3 = (next(it) for _ in range(9))
            a = F.relu6(_bn(F.conv2d(z, w1), g1, b1, eps))
            a = F.relu6(_bn(F.conv2d(a, w2, stride=L.stride, padding=1, groups=a.shape[1]), g2, b2, eps))
            r = _bn(F.conv2d(a, w3), g3, b3, eps)
            z = r + z if (L.stride == 1 and L.c_in == L.c_out) else r
        elif L.kind == BASIC_PREACT:
            g1, b1, w1, g2, b2, w2 = (next(it) for _ in range(6))
            o1 = F.relu(_bn(z, g1, b1, eps))
            c1 = F.conv2d(o1, w1, stride=L.stride, padding=1)
            o2 = F.relu(_bn(c1, g2, b2, eps))
            c2 = F.conv2d(o2, w2, stride=1, padding=1)
            sc = F.conv2d(o1, next(it), stride=L.stride) if proj else z
            z = c2 + sc
        else:
            if L.kind == HEAD_PREACT:
                g, b = next(it), next(it)
                z = F.relu(_bn(z, g, b, eps))
            W, bias = next(it), next(it)
            logits = F.linear(z.mean(dim=(2, 3)), W, bias)
            loss = F.cross_entropy(logits, torch.as_tensor(labels, dtype=torch.long))
            return loss, logits
    return z
