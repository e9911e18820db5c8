"""Independent fp64 evaluation of an op list with PyTorch CPU library routines (conv2d, batch_norm,
max_pool2d, autograd).  Used only to pin the oracle; shares nothing with it but the op-list format."""
import numpy as np
import torch
import torch.nn.functional as F

CONV, DENSE, RELU, MAXPOOL, BN, ADD, GAP = range(7)


def split_params(ops, in_shape, vec):
    """Views of the flat vector as torch leaf tensors, per op, in the documented layout."""
    shapes = {0: tuple(in_shape)}
    off = 0
    leaves = {}
    vec = torch.as_tensor(np.asarray(vec, dtype=np.float64))
    for i, (typ, in0, in1, out, k, stride, pad, cout, bias) in enumerate(ops.tolist()):
        h, w, c = shapes[in0]
        if typ == CONV:
            n = k * k * c * cout
            leaves[i, "w"] = vec[off:off + n].clone().reshape(k, k, c, cout).requires_grad_(True); off += n
            if bias:
                leaves[i, "b"] = vec[off:off + cout].clone().requires_grad_(True); off += cout
            shapes[out] = ((h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1, cout)
        elif typ == DENSE:
            n = h * w * c * cout
            leaves[i, "w"] = vec[off:off + n].clone().reshape(h * w * c, cout).requires_grad_(True); off += n
            if bias:
                leaves[i, "b"] = vec[off:off + cout].clone().requires_grad_(True); off += cout
            shapes[out] = (1, 1, cout)
        elif typ == BN:
            leaves[i, "w"] = vec[off:off + c].clone().requires_grad_(True); off += c
            leaves[i, "b"] = vec[off:off + c].clone().requires_grad_(True); off += c
            shapes[out] = (h, w, c)
        elif typ == MAXPOOL:
            shapes[out] = (h // 2, w // 2, c)
        elif typ == GAP:
            shapes[out] = (1, 1, c)
        else:
            shapes[out] = (h, w, c)
    return leaves, shapes, off


def loss_grad(ops, in_shape, vec, x, y=None, target=None):
    """-> (loss, grad[m_train], logits) with the same conventions as the oracle (channels-last data)."""
    leaves, shapes, m_train = split_params(ops, in_shape, vec)
    B = x.shape[0]
    t = {0: torch.as_tensor(np.asarray(x, dtype=np.float64)).reshape(B, *in_shape).permute(0, 3, 1, 2)}
    for i, (typ, in0, in1, out, k, stride, pad, cout, bias) in enumerate(ops.tolist()):
        a = t[in0]
        if typ == CONV:
            w = leaves[i, "w"].permute(3, 2, 0, 1)           # HWIO -> OIHW
            t[out] = F.conv2d(a, w, leaves.get((i, "b")), stride=stride, padding=pad)
        elif typ == DENSE:
            flat = a.permute(0, 2, 3, 1).reshape(B, -1)      # flatten in H, W, C order
            z = flat @ leaves[i, "w"]
            if bias:
                z = z + leaves[i, "b"]
            t[out] = z.reshape(B, cout, 1, 1)
        elif typ == RELU:
            t[out] = F.relu(a)
        elif typ == MAXPOOL:
            t[out] = F.max_pool2d(a, 2)
        elif typ == BN:
            t[out] = F.batch_norm(a, None, None, leaves[i, "w"], leaves[i, "b"], training=True, eps=1e-5)
        elif typ == ADD:
            t[out] = a + t[in1]
        elif typ == GAP:
            t[out] = a.mean(dim=(2, 3), keepdim=True)
    logits = t[len(ops)].reshape(B, -1)
    if target is not None:
        loss = 0.5 * ((logits - torch.as_tensor(np.asarray(target, dtype=np.float64))) ** 2).sum() / B
    else:
        loss = F.cross_entropy(logits, torch.as_tensor(np.asarray(y, dtype=np.int64)))
    loss.backward()
    grad = np.zeros(m_train)
    off = 0
    for i in range(len(ops)):
        for nm in ("w", "b"):
            if (i, nm) in leaves:
                g = leaves[i, nm].grad
                n = leaves[i, nm].numel()
                grad[off:off + n] = (g if g is not None else torch.zeros(n)).reshape(-1).numpy()
                off += n
    return float(loss.detach()), grad, logits.detach().numpy()
